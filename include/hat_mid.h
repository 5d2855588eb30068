/*
 * hat_mid.h -- C ABI of the cloud-side middle-submodel forward of HAT
 * (arXiv 2503.18989) for AMD MI355X (gfx950).
 *
 * The problem (paper Sec. 2.4 "Our Proposed Framework", Sec. 3.1 "System
 * Overview", Fig. 3): the cloud holds the decoder layers between the device's
 * first m layers and the device's head, plus one KV cache per device (Sec. 2.1).
 * At every inference step it receives hidden states from many devices -- prompt
 * chunks of devices in the prefill phase (Sec. 2.1 batched inference, Sec. 3.3
 * prompt chunking) and draft sequences to verify from devices in the decode
 * phase (Sec. 3.4) -- processes them as one batch and returns the deep hidden
 * states.  Devices join and leave between steps (Sec. 2.1 continuous batching).
 *
 * The layer is LLaMA-style: pre-RMSNorm, rotary embedding (rotate-half pairing:
 * element i pairs with i + head_dim/2, angle pos * theta^(-2i/head_dim)),
 * multi-head attention with as many KV heads as query heads, softmax scale
 * 1/sqrt(head_dim), SwiGLU feed-forward, no biases, residual after each
 * sub-block.  A row at absolute position p attends to keys 0..p of its own
 * device only.
 *
 * Arithmetic: weights hold bf16 values, the KV cache bf16 or fp16 values
 * (hat_kv_dtype_t); matrix products take fp16 operands (activations are produced
 * in fp16, saturating; bf16 weights and bf16 cache rows are widened to fp16, exact
 * for magnitudes in [2^-17, 65504]) and accumulate in fp32; softmax, normalisation, rotary embedding, SiLU and the
 * residual stream are fp32.  Supported activation range: every intermediate that
 * feeds a matrix product (norm outputs, q/k/v, attention outputs, the SwiGLU
 * product) is converted to fp16 with saturation, so a magnitude above 65504 is
 * clamped to +-65504 (never infinity, no error raised); results are exact to the
 * stated tolerance only while those intermediates stay below that bound, which
 * holds by orders of magnitude for unit-scale hidden states and trained LLaMA
 * weights.  The fp32 residual stream itself is not clamped.
 *
 * Conventions
 *  - "device pointer" = address in GPU memory (HBM) of the current HIP device;
 *    "host pointer" = ordinary process memory.  Every struct is read during the
 *    call only.
 *  - The library allocates no GPU memory: KV pool and workspace are supplied by
 *    the caller (sizes from hat_mid_kv_bytes / hat_mid_workspace_bytes, 256-byte
 *    aligned) and stay owned by the caller, who must keep them alive until
 *    hat_mid_destroy.  hat_mid_create copies the weights into the workspace in a
 *    tiled layout; the caller's weight arrays may be freed once the stream work
 *    of hat_mid_create has completed.
 *  - All GPU work is enqueued on the HIP stream passed to the call
 *    (a hipStream_t cast to void*; NULL = the default stream).  Calls return
 *    once the work is enqueued; outputs are valid after the stream is synced.
 *  - Consecutive calls on one handle must be stream-ordered (same stream, or
 *    synchronised by the caller): they share the workspace.
 *  - One caller thread per handle.  No exceptions cross the ABI: every call
 *    returns a hat_status_t (or a size / pointer), and hat_mid_last_error gives
 *    the text of the last failure on the handle.
 *  - hat_mid_forward validates every segment and the page demand of the whole
 *    step before it changes anything: on a validation error (HAT_EINVAL,
 *    HAT_ENOMEM, HAT_EPOS, HAT_EDUP, HAT_EDEVICE) no KV row, page or length
 *    moves.  If a HIP runtime call fails while the step is being enqueued
 *    (HAT_EHIP), lengths and page lists are put back as they were before the
 *    call, but kernels already enqueued may still run: cache rows at or beyond
 *    the start positions of that step's segments are then unspecified, and the
 *    caller should regard the stream as failed.
 */
#ifndef HAT_MID_H
#define HAT_MID_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hat_mid hat_mid_t; /* opaque handle */

typedef enum {
  HAT_OK = 0,
  HAT_EINVAL = -1,  /* malformed argument (n <= 0, verify segment longer than 8, bad tree, beyond max_pos ...) */
  HAT_ENOMEM = -2,  /* KV pool exhausted for this step */
  HAT_EPOS = -3,    /* start_pos beyond the device's cache length (would leave a gap) */
  HAT_EDUP = -4,    /* the same device twice in one step */
  HAT_EDEVICE = -5, /* device id outside [0, max_devices) */
  HAT_EHIP = -6     /* a HIP runtime call or a host allocation failed */
} hat_status_t;

typedef enum { HAT_SEG_CHUNK = 0, HAT_SEG_VERIFY = 1 } hat_seg_kind_t;
typedef enum { HAT_BF16 = 0, HAT_F32 = 1 } hat_dtype_t;
/* Element type of the KV cache (two bytes either way).  HAT_KV_BF16 is the format the workload
 * definitions name.  HAT_KV_F16 keeps 11 instead of 8 significand bits: the rounding of cache rows is
 * the largest error of the whole path (it is amplified from layer to layer), and a 38-layer stack of
 * 13B-shaped random-init layers exceeds the 2e-2 parity bar with a bf16 cache (2.2e-2 measured) while
 * an fp16 cache stays near 4e-3; fp16 elements are also matrix-core operands as they are, so the
 * attention kernels skip the widening.  Cache values (keys, values of unit-scale activations) are far
 * inside the fp16 range; anything beyond +-65504 saturates. */
typedef enum { HAT_KV_BF16 = 0, HAT_KV_F16 = 1 } hat_kv_dtype_t;

#define HAT_PAGE_SIZE 16  /* tokens per KV page */
#define HAT_MAX_VERIFY 8  /* longest verify segment */

typedef struct {
  int32_t n_layers;        /* decoder layers in the middle submodel */
  int32_t d_model;         /* = n_heads * head_dim; multiple of 64 */
  int32_t n_heads;
  int32_t head_dim;        /* 64 or 128 */
  int32_t d_ffn;           /* SwiGLU inner width (any positive value) */
  float rms_eps;           /* added to the mean of squares, inside the root */
  float rope_theta;
  int32_t page_size;       /* must be HAT_PAGE_SIZE */
  int32_t n_pages;         /* pool capacity; one page id addresses all layers */
  int32_t max_devices;     /* device ids are 0 .. max_devices-1 */
  int32_t max_step_tokens; /* upper bound on the rows of one step */
  int32_t max_pos;         /* upper bound on any device's cache length */
  int32_t io_dtype;        /* hat_dtype_t of hidden_in / hidden_out */
  int32_t kv_dtype;        /* hat_kv_dtype_t of the cache elements */
} hat_mid_config_t;

/* One layer's weights: device pointers to bf16 arrays, linear weights row-major
 * [out_features, in_features], norm gains [d_model]. */
typedef struct {
  const void *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
} hat_mid_layer_weights_t;

/* One device's rows in a step: n rows of hidden states at consecutive absolute
 * positions start_pos .. start_pos+n-1.  kind does not change the mathematics
 * (both are causal over prefix + own rows); it routes the attention work: a
 * VERIFY segment (Sec. 3.4: the draft sequence verified in one step) has
 * n <= HAT_MAX_VERIFY rows and takes the bandwidth-bound path, a CHUNK segment
 * (Sec. 3.3) takes the matrix-core path.
 * start_pos must satisfy 0 <= start_pos <= cache length of the device.
 * start_pos < length first rolls the cache back to start_pos: that is how the
 * rows of rejected draft tokens disappear (Sec. 3.4: the next round starts after
 * the last accepted token).  A device not seen before starts with length 0.
 *
 * Tree verification (Sec. 2.2, last paragraph: candidates combined into a tree whose
 * every branch may be the accepted path; Sec. 4.1 uses trees of 8 for the
 * tree-verifying comparison system): a VERIFY segment with tree_mask != NULL holds
 * the n nodes of a forest in parents-first order.  tree_mask[i] has bit j set when
 * node j is node i itself or one of its ancestors (bit i always, no bit above i, and
 * the ancestors must be one path).  Node i is evaluated exactly as if its path had
 * been submitted alone as a chain: its position is start_pos + depth(i) and it
 * attends to the cache rows below start_pos, to its ancestors and to itself.  Its
 * K/V row is stored at cache row start_pos + i, so the cache length becomes
 * start_pos + n as for any segment; hat_mid_kv_compact then keeps the accepted path.
 * tree_mask == NULL means consecutive rows (the chain mask (2 << i) - 1). */
typedef struct {
  int32_t device_id;
  int32_t kind;           /* hat_seg_kind_t */
  int32_t n;
  int32_t start_pos;
  const void* hidden_in;  /* device pointer, [n, d_model] row-major, io_dtype */
  void* hidden_out;       /* device pointer, [n, d_model] row-major, io_dtype; may equal hidden_in */
  const uint8_t* tree_mask; /* HOST pointer to n bytes, or NULL; only with HAT_SEG_VERIFY */
} hat_mid_segment_t;

/* Bytes of KV pool / workspace the configuration needs (0 if cfg is invalid). */
size_t hat_mid_kv_bytes(const hat_mid_config_t* cfg);
size_t hat_mid_workspace_bytes(const hat_mid_config_t* cfg);

/* Builds a handle.  layers: host array of cfg->n_layers entries (device
 * pointers inside).  kv_pool, workspace: device pointers, caller-owned.
 * Enqueues the weight re-tiling on hip_stream.  *out is NULL on failure and the
 * status says why (HAT_EINVAL for a bad config, HAT_EHIP for a runtime error). */
hat_status_t hat_mid_create(const hat_mid_config_t* cfg, const hat_mid_layer_weights_t* layers,
                            void* kv_pool, void* workspace, void* hip_stream, hat_mid_t** out);

/* One inference step over a ragged batch (Sec. 3.1: hidden states of devices in
 * different phases processed in one batch per step).  segs: host array.  For
 * every segment the n output rows are written to hidden_out.  KV rows of the new
 * tokens are appended to each device's cache; pages follow the fixed policy
 * "lowest free id first; all rollback frees of the step, in array order, then
 * allocations in array order".  Atomic on error.  n_segs == 0 is an empty step:
 * HAT_OK, nothing is enqueued and no state changes (segs may be NULL then). */
hat_status_t hat_mid_forward(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, void* hip_stream);

/* The same step for hidden states that live in HOST memory (the form in which they
 * arrive from the devices; Sec. 3.3: the transfer of one chunk overlaps the
 * processing of another).  hidden_in / hidden_out of every segment are host
 * pointers here, read and written asynchronously: keep them alive and untouched
 * until hip_stream has been synchronised.  The rows are uploaded on a stream of
 * the library's own into one of two staging slots in the workspace, the step
 * runs on hip_stream once they have arrived, and the results are copied back
 * on hip_stream; the upload of the next call therefore overlaps the
 * computation of this one.  Overlap needs pinned memory (hipHostMalloc); with
 * pageable memory the copies are still correct but serialise.  Validation,
 * errors and atomicity are those of hat_mid_forward. */
hat_status_t hat_mid_forward_host(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, void* hip_stream);

/* After a tree step that started at base_pos: keeps the accepted path.  keep: host
 * array of n_keep node indices of that step, strictly ascending (a path from a root,
 * though only the order is checked), each < HAT_MAX_VERIFY and base_pos + keep[i]
 * below the cache length.  In every layer the K/V row of node keep[i] moves to cache
 * row base_pos + i (a pure copy: the node was rotated for position base_pos + depth,
 * which is base_pos + i on its own path); the cache length becomes base_pos + n_keep
 * and the pages wholly beyond it return to the pool at once.  n_keep == 0 is a plain
 * rollback to base_pos.  Enqueues one small kernel on hip_stream; the next forward
 * of the device on that stream starts at base_pos + n_keep.  On error nothing changes
 * (HAT_EINVAL: bad list; HAT_EPOS: a row beyond the cache; HAT_EDEVICE). */
hat_status_t hat_mid_kv_compact(hat_mid_t* h, int32_t device_id, int32_t base_pos, const int32_t* keep,
                                int32_t n_keep, void* hip_stream);

/* The device left (Sec. 2.1: requests leave the batch): all its pages return to
 * the pool, its length becomes 0.  Unknown-but-valid ids are a no-op. */
hat_status_t hat_mid_release(hat_mid_t* h, int32_t device_id);

/* Frees host-side state (pinned staging, events) after waiting for the handle's own work: its
 * internal copy stream and the stream of its most recent call.  GPU buffers stay with the caller. */
void hat_mid_destroy(hat_mid_t* h);

/* Text of the last error on this handle ("" if none); valid until the next call. */
const char* hat_mid_last_error(const hat_mid_t* h);

/* ---- introspection and fixtures ------------------------------------------ */

/* Cache length and page list of a device.  pages_out (host, may be NULL) receives
 * at most cap ids; *n_pages_out (may be NULL) the number owned. */
hat_status_t hat_mid_kv_query(const hat_mid_t* h, int32_t device_id, int32_t* kv_len, int32_t* pages_out,
                              int32_t cap, int32_t* n_pages_out);

/* Installs n cache rows of one layer at positions pos0..pos0+n-1 from device
 * arrays k, v of shape [n, n_heads, head_dim] bf16 (k already rotated); an fp16
 * cache holds those bf16 values exactly (magnitudes in [2^-17, 65504]).  Rows
 * must extend or overwrite the device's cache contiguously (pos0 <= length); the
 * length becomes max(length, pos0+n) and missing pages are taken with the same
 * lowest-free-id policy as forward.  Every layer has to be imported over the same
 * range before the rows are attended to.  Synchronises the stream (fixture). */
hat_status_t hat_mid_kv_import(hat_mid_t* h, int32_t device_id, int32_t layer, int32_t pos0, int32_t n,
                               const void* k, const void* v, void* hip_stream);

/* Mirror of import: copies rows pos0..pos0+n-1 of one layer out to k, v
 * ([n, n_heads, head_dim] bf16 device arrays); rows of an fp16 cache are rounded
 * to bf16 (to nearest even) on the way out, so imported rows come back unchanged. */
hat_status_t hat_mid_kv_export(hat_mid_t* h, int32_t device_id, int32_t layer, int32_t pos0, int32_t n,
                               void* k, void* v, void* hip_stream);

/* hat_mid_kv_export for callers that may not allocate or synchronise: serving loops that move a
 * device's cache elsewhere (migration, snapshots) from code where hipMalloc is forbidden -- under
 * stream capture, inside tight step loops, in harnesses that ban it.  Same arguments, checks and
 * results as hat_mid_kv_export, but the page ids of the exported rows are staged in an array
 * that the library holds statically on every GPU (16 KB per GPU, for the life of the process)
 * instead of in the workspace, they travel there with an asynchronous copy from a pinned buffer
 * made at create time, and nothing waits for the stream: the call makes no hipMalloc / hipFree,
 * no allocating library call and no stream synchronisation (it waits, on the host, only for the
 * previous call's upload of page ids to have left the pinned buffer).
 * Limit: rows pos0 .. pos0+n-1 may span at most 4096 pages (65 536 rows); more is HAT_EINVAL.
 * All handles of one GPU share the array and it keeps the last call's page ids: calls that
 * overlap on one GPU (different streams without ordering, or several handles at once) race on
 * it -- order them on one stream, as consecutive calls on one handle already must be. */
hat_status_t hat_mid_kv_export_static(hat_mid_t* h, int32_t device_id, int32_t layer, int32_t pos0, int32_t n,
                                      void* k, void* v, void* hip_stream);

/* Rows and GPU time of the last completed step -- the pair the cloud's state
 * monitor records every round (Sec. 3.2, Eq. 1-2).  Synchronises on the step's
 * end event. */
hat_status_t hat_mid_last_step_stats(hat_mid_t* h, int32_t* tokens, float* gpu_ms);

/* ---- per-kernel timing (for roofline measurement) -------------------------- */

typedef enum {
  HAT_K_GATHER = 0,   /* hidden_in rows -> fp32 residual */
  HAT_K_RMSNORM,      /* both norms */
  HAT_K_GEMM_QKV,
  HAT_K_ROPE_APPEND,
  HAT_K_ATTN_CHUNK,
  HAT_K_ATTN_VERIFY,
  HAT_K_ATTN_MERGE,
  HAT_K_GEMM_O,
  HAT_K_GEMM_GATEUP,
  HAT_K_GEMM_DOWN,
  HAT_K_SCATTER,      /* residual -> hidden_out rows */
  HAT_K_COUNT
} hat_kernel_id_t;

/* on != 0: later forwards bracket every kernel launch with HIP events on the
 * launch stream.  Slows the step slightly; off by default. */
hat_status_t hat_mid_set_profiling(hat_mid_t* h, int32_t on);

/* Sums since the last call, per kernel id: GPU milliseconds and launch counts
 * (host arrays of HAT_K_COUNT entries).  Synchronises the recorded events, then
 * resets the sums. */
hat_status_t hat_mid_kernel_times(hat_mid_t* h, float* ms, int32_t* launches);

/* ---- stage dumps (for per-stage parity tests) ------------------------------ */

typedef enum {
  HAT_DUMP_XNORM = 0, /* attention-norm output, [T, d_model] */
  HAT_DUMP_Q,         /* rotated queries, [T, d_model] */
  HAT_DUMP_ATTN,      /* attention output before the O projection, [T, d_model] */
  HAT_DUMP_XNORM2,    /* FFN-norm output (norm of the residual after the attention block), [T, d_model] */
  HAT_DUMP_ACT        /* silu(gate)*up, [T, d_ffn] */
} hat_dump_id_t;

/* Copies one intermediate of the LAST layer of the last forward, rows in batch
 * order, to dst (device pointer, row-major fp32).  Only meaningful right after a
 * forward on the same stream. */
hat_status_t hat_mid_debug_dump(hat_mid_t* h, int32_t which, void* dst, void* hip_stream);

/* ---- planner on its own (tests of the host logic, no GPU needed) ----------------------- */

/* A handle without GPU memory and without any HIP call: it keeps the page and length state
 * of hat_mid_create's handle and accepts hat_mid_debug_plan, hat_mid_kv_query,
 * hat_mid_kv_compact (state only), hat_mid_release, hat_mid_last_error and hat_mid_destroy;
 * the calls that need the GPU (forward, forward_host, kv_import, kv_export, step statistics,
 * profiling, dumps) return HAT_EINVAL. */
hat_status_t hat_mid_debug_create_host_only(const hat_mid_config_t* cfg, hat_mid_t** out);

/* Validates and plans one step exactly as hat_mid_forward does -- same errors, same atomicity,
 * page movements committed on success -- and returns the plan instead of running it.  Host
 * arrays, any of which may be NULL: pos / kv_dst (cap_rows entries: each row's rotary position
 * and page*16 + slot write target, in batch order), the chunk- and verify-attention work items
 * (12 int32 words each: segment, first query row, query rows, first key, end key, first partial
 * row or -1, segment start, first batch row, cache length, page-list offset, and for verify items
 * two words of per-row visibility bytes) and the split-KV merge items (8 words: first batch row,
 * rows, partial row of split 0, splits, partial rows between splits, 3 unused); cap_items bounds
 * each item array.  The segments' hidden pointers are checked for NULL only. */
hat_status_t hat_mid_debug_plan(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, int32_t* pos,
                                int32_t* kv_dst, int32_t cap_rows, int32_t* chunk_items, int32_t* n_chunk_items,
                                int32_t* verify_items, int32_t* n_verify_items, int32_t* merge_items,
                                int32_t* n_merge_items, int32_t cap_items);

/* ---- tuning aid ------------------------------------------------------------------ */

/* Forces the tile shape and K split of one GEMM class in later forwards
 * (which: 0 = QKV, 1 = O, 2 = gate/up, 3 = down; tile: index into the library's
 * tile table, -1 = automatic choice; ksplit: 1 = none, only honoured where the
 * result is accumulated).  For sweeps of launch shapes; results do not change
 * beyond fp32 summation order. */
hat_status_t hat_mid_debug_force_gemm(hat_mid_t* h, int32_t which, int32_t tile, int32_t ksplit);

/* The automatic choice for a GEMM of T rows: Nw = weight rows (padded to 256), Nout = logical
 * output features, K = inner dimension (multiple of 64), epilogue 0 = fp16 output, 1 = SwiGLU,
 * 2 = accumulate into the residual (the only one whose K may be split; part_rows = capacity of
 * the partial-sum buffer in rows, 0 = no buffer).  Host code only, no GPU work; for tests of the
 * planner.  Returns HAT_EINVAL on a null pointer. */
hat_status_t hat_mid_debug_gemm_plan(int32_t T, int32_t Nw, int32_t Nout, int32_t K, int32_t epilogue,
                                     int32_t part_rows, int32_t* tile, int32_t* ksplit);

/* Workgroup counts that the attention work lists aim for (chunk kernel, verify kernel): long key
 * ranges are split over several workgroups until a launch has about that many.  0 keeps a value.
 * For tests that force the split and unsplit paths, and for sweeps; the work-list capacities were
 * sized at create time, so a larger target splits only as far as they allow.  Results change only
 * in fp32 summation order. */
hat_status_t hat_mid_debug_set_attn_targets(hat_mid_t* h, int32_t chunk_target, int32_t verify_target);

/* Lowers the capacity (in 32-bit words) that a step's plan may occupy; 0 restores the real one.
 * Lets a test reach the "plan exceeds capacity" failure, which happens after the step's page
 * movements, and check that they are undone. */
hat_status_t hat_mid_debug_limit_plan(hat_mid_t* h, int64_t max_words);

/* on != 0: later forwards run, in place of verify attention, a kernel that performs exactly its
 * memory accesses (same work items, page-list walk, load instructions and order) and none of its
 * arithmetic.  The step's OUTPUTS ARE THEN MEANINGLESS (the attention output of verify rows is
 * left as it was); the cache is still appended to.  hat_mid_kernel_times reports the probe under
 * HAT_K_ATTN_VERIFY: its duration is the ceiling this access order can reach on the machine. */
hat_status_t hat_mid_debug_set_verify_probe(hat_mid_t* h, int32_t on);

/* Microbenchmarks of the machine (no handle needed): the rates that the instruction mixes used
 * by this library's kernels reach on their own, for reading roofline fractions against measured
 * as well as published peaks.  buf: device scratch of `bytes` (16-byte aligned; at least 1 MiB,
 * for the streaming kinds as large as the stream to be measured, e.g. 1 GiB); iters launches
 * (1..1000) are timed with HIP events on hip_stream after one warm-up launch, and the call waits
 * for them.  *rate: bytes/s (STREAM_READ*, COPY: read + written bytes; LDS_LOAD: bytes moved into
 * LDS by direct-to-LDS loads from a 1 MiB cache-resident region, all CUs together) or FLOP/s
 * (MFMA_F16: 32x32x16 fp16 matrix instructions only, two waves per SIMD). */
typedef enum {
  HAT_PEAK_STREAM_READ = 0,
  HAT_PEAK_STREAM_READ_NT = 1,   /* the same with non-temporal loads */
  HAT_PEAK_COPY = 2,
  HAT_PEAK_MFMA_F16 = 3,
  HAT_PEAK_LDS_LOAD = 4
} hat_peak_kind_t;
hat_status_t hat_mid_debug_peak(int32_t kind, void* buf, size_t bytes, int32_t iters, void* hip_stream, double* rate);

/* Number of entries in the library's GEMM tile table (valid `tile` values of
 * hat_mid_debug_force_gemm are 0 .. count-1).  No GPU work. */
int32_t hat_mid_debug_gemm_tile_count(void);

/* Shape of entry `tile` of that table: output features x token rows of one workgroup tile, its
 * waves, the k extent of one ring stage and the number of stages (host pointers; any may be null).
 * HAT_EINVAL if `tile` is out of range.  No GPU work; for tests of the planner. */
hat_status_t hat_mid_debug_gemm_tile_info(int32_t tile, int32_t* features, int32_t* tokens, int32_t* waves,
                                          int32_t* k_per_stage, int32_t* stages);

#ifdef __cplusplus
}
#endif
#endif /* HAT_MID_H */
