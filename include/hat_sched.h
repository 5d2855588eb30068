/* hat_sched -- the cloud's state monitor and chunk-size rule of HAT (arXiv 2503.18989),
 * host-side companion of hat_mid: it consumes the (tokens, delay) pair that
 * hat_mid_last_step_stats reports after every step.
 *
 * Plain host code (no GPU work, no allocation other than the handle itself).  One caller
 * thread per handle.  Units are the caller's: delays in any one time unit, bandwidths in
 * bytes per that unit, sizes in bytes.
 *
 * What the paper fixes: the moving averages of Sec. 3.2 (Eq. 1, Eq. 2), the balance equation
 * of Sec. 3.3 (Eq. 3), the floor formula of Sec. 3.5.  The paper does not say how the predictive
 * function g(.) is stored or updated at a point; this library keeps a table over fixed knots:
 *   - g(x): linear interpolation between the knots observed so far; beyond the first / last
 *     observed knot the nearest linear piece continues; one observed knot gives a constant;
 *     none gives 0;
 *   - an observation (mu_hat, eta_hat) updates the knot nearest to mu_hat (ties: the lower
 *     one) with g <- alpha g + (1 - alpha) eta_hat -- eta_hat was measured for mu_hat tokens,
 *     so that is where Eq. 2 is applied; a knot without history takes eta_hat itself, and the
 *     first observation likewise initialises mu;
 *   - the chunk size is the smallest integer X in [x_min, x_max] whose upload time
 *     X * A / beta_up is at least (g(mu) + g(mu + X)) / P (Eq. 3 holds with equality between
 *     X - 1 and X); x_max if no size in the range does. */
#ifndef HAT_SCHED_H
#define HAT_SCHED_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hat_sched hat_sched_t; /* opaque */

/* knots: host array of n_knots token counts, strictly ascending, >= 1 entry (copied).
 * alpha in [0, 1] (the paper's experiments use 0.8).  Returns 0 and sets *out, or -1
 * (invalid argument; *out = NULL). */
int32_t hat_sched_create(const int32_t* knots, int32_t n_knots, double alpha, hat_sched_t** out);
void hat_sched_destroy(hat_sched_t* s);

/* One round of state collection (Sec. 3.2): mu <- alpha mu + (1 - alpha) mu_hat (Eq. 1) and the
 * update of g at mu_hat by eta_hat (Eq. 2).  Returns 0, or -1 if s is NULL or a value is not
 * finite / negative. */
int32_t hat_sched_observe(hat_sched_t* s, double mu_hat, double eta_hat);

/* The averaged batched token size mu (0 before the first observation). */
double hat_sched_mu(const hat_sched_t* s);

/* g(tokens): the predicted in-cloud computation delay of a batch of that many tokens. */
double hat_sched_predict(const hat_sched_t* s, double tokens);

/* Chunk size for a device (Sec. 3.3, Eq. 3): bytes_per_token = A (size of one token's hidden
 * state), beta_up = its upload bandwidth, pipeline_len = P.  Returns the size, or -1 on an
 * invalid argument (NULL, non-positive A, beta_up or P, x_min < 1, x_max < x_min). */
int32_t hat_sched_chunk_size(const hat_sched_t* s, double bytes_per_token, double beta_up, int32_t pipeline_len,
                             int32_t x_min, int32_t x_max);

/* Number of inference steps a device may spend on parallel drafting during verification
 * (Sec. 3.5): floor((draft_len A / beta_up + g(mu) + draft_len A / beta_down) / gamma), gamma =
 * the device's drafting delay per step, clamped at 0 (far from the observed knots the linear
 * continuation of g can dip below zero).  Returns the count, or -1 on an invalid argument. */
int32_t hat_sched_parallel_draft_steps(const hat_sched_t* s, double draft_len, double bytes_per_token,
                                       double beta_up, double beta_down, double gamma);

#ifdef __cplusplus
}
#endif
#endif /* HAT_SCHED_H */
