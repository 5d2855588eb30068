// Prefix-causal attention over the paged KV cache, in two launch shapes:
//
//   chunk  -- a prompt chunk of a device in the prefill phase (paper Sec. 2.1
//             chunked prefill, Sec. 3.3): many query rows, matrix-core bound.
//             One workgroup = 256 query rows (8 waves x 32) of one head; K/V tiles
//             of 64 keys are staged in LDS and shared by the eight waves.
//   verify -- the draft sequence of a device in the decode phase verified in one
//             step (Sec. 3.4), or a tree of candidates (Sec. 2.2) given as one
//             visibility byte per row: at most 8 query rows against a long cache, HBM
//             bound.  One workgroup = one (segment, head, key range); each wave
//             streams every 4th pair of pages straight from global memory into
//             MFMA operand registers (the page tiles are stored in operand order,
//             so a wave instruction reads whole contiguous 512 B / 1 KB runs),
//             then the four waves' partial results are merged through LDS.
//
// The cache holds bf16; queries, probabilities and outputs are fp16 like every other
// activation, so K and V are widened bf16 -> fp16 in registers (exact for
// magnitudes in [2^-17, 65504], saturating above) on their way to the MFMA.
// Both compute S^T = K Q^T with v_mfma_f32_32x32x16_f16, so a lane owns ONE query
// column and 16 keys of it: the online softmax is lane-local except for one
// exchange between the two lane halves, and the probabilities are already in the
// B-operand order of O^T += V^T P^T (the V tile is stored in that key order).
// Row at position p sees keys 0..p of its own device.  Long key ranges may be
// split over several workgroups; those write (max, sum, O normalised by that sum, fp16)
// partials that attn_merge combines.
#include <hip/hip_runtime.h>

#include "hat_device_util.h"
#include "hat_kernels.h"
#include "hat_layout.h"

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float kLog2e = 1.4426950408889634f;

struct SegInfo {
  int start, nseg, kv_len, tok0, npages;
  const int32_t* pt;
};

__device__ __forceinline__ SegInfo seg_info(const HatPlanDev& p, const HatAttnItem& it) {
  SegInfo s;
  s.start = it.start;
  s.tok0 = it.tok0;
  s.kv_len = it.kv_len;
  s.nseg = s.kv_len - s.start;
  s.npages = (s.kv_len + 15) >> 4;
  s.pt = p.page_tbl + it.pt_off;
  return s;
}

// max over the two lane halves (lanes n and n + 32 hold the same query column): every lane gets
// max(x[n], x[n + 32]).
// One VALU instruction instead of a trip through the LDS crossbar: v_permlane32_swap exchanges
// the upper half of its first operand with the lower half of its second, so two copies of x
// become {lo, lo} and {hi, hi}.
__device__ __forceinline__ float half_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// 16 bytes of cache that this launch reads exactly once (the verify kernel's page tiles): the
// non-temporal hint keeps the stream from displacing what other kernels left in the caches, and
// measures 11 % faster on the verify-heavy workload (363 -> 325 us per launch).
__device__ __forceinline__ u32x4 stream_load(const u32x4* p) { return __builtin_nontemporal_load(p); }

// Online-softmax update for one 32-key S^T tile held as 16 accumulator values.
// key of value r: key0 + 8*(r/4) + 4*half + r%4.  Returns probabilities as the
// two B operands (keys 0..15 / 16..31 of the tile) and rescales O when the running
// maximum of any row of the wave moved.  MASK = 0 is for tiles that lie wholly
// below every row's causal limit (no compares); 1 = causal (keys up to qpos); 2 = the
// caller supplies the visibility of the lane's keys as a bit set (vis).  Scores are kept unscaled; the
// softmax scale (times log2 e) is folded into the exponent's fma.
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <int NC, int MASK>
__device__ __forceinline__ void softmax_step(const f32x16& s_acc, float scale_log2, int key0, int half, int qpos,
                                             float& m_run, float& l_run, f32x16 (&o)[NC], f16x8& p0, f16x8& p1,
                                             uint32_t vis = 0) {
  float sr[16];
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    if (MASK == 1) {
      const int key = key0 + 8 * (r >> 2) + 4 * half + (r & 3);
      sr[r] = (key <= qpos) ? s_acc[r] : -INFINITY;
    } else if (MASK == 2) {
      // vis: this lane's 16 keys of the tile, bit 8*(r/4) + r%4 = key of value r visible
      sr[r] = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? s_acc[r] : -INFINITY;
    } else {
      sr[r] = s_acc[r];
    }
    mx = fmaxf(mx, sr[r]);
  }
  mx = half_max(mx);
  const float m_new = fmaxf(m_run, mx * scale_log2);   // running maximum in log2 units
  const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
  float ps = 0.f;
  float pv[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    pv[r] = __builtin_amdgcn_exp2f(fmaf(sr[r], scale_log2, -m_safe));
    ps += pv[r];
  }
  if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {   // wave-uniform: some row's maximum moved
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
    l_run *= alpha;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[c][r] *= alpha;
    m_run = m_new;
  }
  l_run += ps;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const f32x2 a = {pv[2 * j], pv[2 * j + 1]}, b = {pv[8 + 2 * j], pv[8 + 2 * j + 1]};
    const f16x2 ha = __builtin_convertvector(a, f16x2), hb = __builtin_convertvector(b, f16x2);
    p0[2 * j] = ha[0]; p0[2 * j + 1] = ha[1];
    p1[2 * j] = hb[0]; p1[2 * j + 1] = hb[1];
  }
}

// zero the V operand elements whose key lies at or beyond kv_len (stale memory
// there may hold NaN patterns, and 0 * NaN would poison the accumulator)
__device__ __forceinline__ f16x8 clean_v(f16x8 v, int page_key0, int half, int kv_len) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int key = page_key0 + 8 * (j >> 2) + 4 * half + (j & 3);
    if (key >= kv_len) v[j] = (_Float16)0.f;
  }
  return v;
}

// 8 bf16 (as loaded from the cache) -> 8 fp16.  bf16 -> fp32 is a shift; fp32 -> fp16
// with round-toward-zero is exact where the value is representable and saturates
// (instead of overflowing to infinity) where it is not.
// With an fp16 cache (KVF16) the elements are operands as they are.
template <bool KVF16>
__device__ __forceinline__ u32x4 kv_to_f16_bits(u32x4 raw) {
  if constexpr (KVF16) return raw;
  u32x4 out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(raw[i] << 16), hi = __uint_as_float(raw[i] & 0xffff0000u);
    out[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
  }
  return out;
}
template <bool KVF16>
__device__ __forceinline__ f16x8 kv_to_f16(u32x4 raw) { return __builtin_bit_cast(f16x8, kv_to_f16_bits<KVF16>(raw)); }

__device__ __forceinline__ _Float16 to_act(float x) { return (_Float16)__builtin_amdgcn_fmed3f(x, -65504.f, 65504.f); }

// ------------------------------------------------------------------ verify
template <int HD, bool KVF16>
__global__ __launch_bounds__(256, 2) void attn_verify_kernel(HatPlanDev p, HatAttn a) {
  constexpr int NS = HD / 16;  // k-steps of Q K^T
  constexpr int NC = HD / 32;  // 32-row blocks of O^T
  constexpr int REC = 2 * 16 * HD;  // elements of one (page, head) record
  __shared__ float lds_o[4][HAT_MAX_VERIFY_ROWS][HD];
  __shared__ float lds_m[4][HAT_MAX_VERIFY_ROWS], lds_l[4][HAT_MAX_VERIFY_ROWS];

  const HatAttnItem it = a.items[blockIdx.x];
  const int head = blockIdx.y;
  const SegInfo sg = seg_info(p, it);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, n = lane & 31;
  const int qi = n < it.nq ? n : it.nq - 1;  // clamp idle columns onto a real row
  const int qrow = sg.tok0 + it.q0 + qi;
  const uint32_t vis = ((qi < 4 ? it.vis_lo : it.vis_hi) >> (8 * (qi & 3))) & 0xffu;  // q0 = 0 for verify items
  const float scale_log2 = kLog2e / sqrtf((float)HD);

  f16x8 qreg[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s)
    qreg[s] = *(const f16x8*)(a.qkv + p32_index(qrow, head * HD + (2 * s + half) * 8, 3 * a.d));

  f32x16 o[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[c][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  int kv_end = it.kv_end < sg.kv_len ? it.kv_end : sg.kv_len;
  const int pair0 = it.kv_begin >> 5, pair1 = (kv_end + 31) >> 5;
  const kv_t* pool = a.pool_layer + (size_t)head * a.n_pages * REC;  // this head's pages are contiguous
  const size_t page_stride = REC;

  // One register stage of raw page data per wave, refilled as early as possible: the loads of
  // the wave's next page pair are issued as soon as the current pair has been widened out of the
  // raw registers, and travel while the current pair is soft-maxed and multiplied.  Two
  // workgroups share a CU (<= 256 VGPRs).
  u32x4 kraw[NS], varaw[NC], vbraw[NC];
  const kv_t *recA = pool, *recB = pool;
  auto page_recs = [&](int pp) {   // wave-uniform: scalar loads of the two page ids
    int ia = 2 * pp, ib = 2 * pp + 1;
    ib = ib < sg.npages ? ib : sg.npages - 1;
    recA = pool + (size_t)sg.pt[ia] * page_stride;
    recB = pool + (size_t)sg.pt[ib] * page_stride;
  };
  auto load_k = [&]() {
    const kv_t* krec = (n < 16) ? recA : recB;
#pragma unroll
    for (int s = 0; s < NS; ++s) kraw[s] = stream_load((const u32x4*)(krec + ((2 * s + half) * 16 + (n & 15)) * 8));
  };
  auto load_v = [&]() {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      varaw[c] = stream_load((const u32x4*)(recA + 16 * HD + c * 512 + lane * 8));
      vbraw[c] = stream_load((const u32x4*)(recB + 16 * HD + c * 512 + lane * 8));
    }
  };
  int pp = pair0 + wave;
  if (pp < pair1) {
    page_recs(pp);
    load_k();
    load_v();
  }
  for (; pp < pair1; pp += 4) {
    const int key0 = pp << 5;
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kv_to_f16<KVF16>(kraw[s]), qreg[s], sacc, 0, 0, 0);
    f16x8 va[NC], vb[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      va[c] = kv_to_f16<KVF16>(varaw[c]);
      vb[c] = kv_to_f16<KVF16>(vbraw[c]);
    }
    if (pp + 4 < pair1) {
      page_recs(pp + 4);
      load_k();
      load_v();
    }
    if (key0 + 32 > sg.kv_len) {
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        va[c] = clean_v(va[c], key0, half, sg.kv_len);
        vb[c] = clean_v(vb[c], key0 + 16, half, sg.kv_len);
      }
    }
    f16x8 p0, p1;
    if (key0 + 31 >= sg.start) {
      // keys start-32 .. start+31 as one 64-bit set: the cache below the segment is visible, the
      // segment's own rows as the query row's byte says, nothing beyond; the tile's 32 keys begin at
      // bit key0 - start + 32 (1..39 here, as start - 31 <= key0 <= start + 7), and this lane
      // holds keys 4*half + {0..3, 8..11, 16..19, 24..27} of them
      const uint64_t window = ((uint64_t)vis << 32) | 0xffffffffull;
      const uint32_t tile_vis = (uint32_t)(window >> (key0 - sg.start + 32)) >> (4 * half);
      softmax_step<NC, 2>(sacc, scale_log2, key0, half, 0, m_run, l_run, o, p0, p1, tile_vis);
    } else {
      softmax_step<NC, 0>(sacc, scale_log2, key0, half, 0, m_run, l_run, o, p0, p1);
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      o[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[c], p0, o[c], 0, 0, 0);
      o[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vb[c], p1, o[c], 0, 0, 0);
    }
  }
  l_run += __shfl_xor(l_run, 32);

  // merge the four waves (each saw a disjoint quarter of the keys)
  if (n < it.nq) {
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) lds_o[wave][n][32 * c + 8 * (r >> 2) + 4 * half + (r & 3)] = o[c][r];
    if (half == 0) {
      lds_m[wave][n] = m_run;
      lds_l[wave][n] = l_run;
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < it.nq * (HD / 4); idx += 256) {
    const int q = idx / (HD / 4), e = (idx % (HD / 4)) * 4;
    float M = fmaxf(fmaxf(lds_m[0][q], lds_m[1][q]), fmaxf(lds_m[2][q], lds_m[3][q]));
    const float Ms = (M == -INFINITY) ? 0.f : M;
    float L = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = exp2f(lds_m[w][q] - Ms);
      L += lds_l[w][q] * f;
      const f32x4 v = *(const f32x4*)&lds_o[w][q][e];
#pragma unroll
      for (int x = 0; x < 4; ++x) acc[x] += v[x] * f;
    }
    if (it.part_row < 0) {
      const float inv = 1.0f / L;
      f16x4 ov;
#pragma unroll
      for (int x = 0; x < 4; ++x) ov[x] = to_act(acc[x] * inv);
      *(f16x4*)(a.outP + p32_index(sg.tok0 + it.q0 + q, head * HD + e, a.d)) = ov;
    } else {
      // a partial result travels normalised by its own sum, in the activation type: the merge
      // weighs it by that sum.  A key range that this row does not see at all has L = 0.
      const size_t pr = (size_t)(it.part_row + q) * a.H + head;
      const float inv = L > 0.f ? 1.0f / L : 0.f;
      f16x4 ov;
#pragma unroll
      for (int x = 0; x < 4; ++x) ov[x] = to_act(acc[x] * inv);
      *(f16x4*)(a.part_o + pr * HD + e) = ov;
      if (e == 0) a.part_ml[pr] = make_float2(M, L);
    }
  }
}

// ------------------------------------------------------------------ verify, loads only
// The verify kernel's memory side on its own: same work items, same page-list walk, same
// non-temporal 16-byte loads in the same order, one register stage per wave -- and no arithmetic
// beyond an XOR of what was loaded.  Its duration is the ceiling that this access order can reach
// on the machine; it writes nothing (the store below never executes for real cache contents).
template <int HD>
__global__ __launch_bounds__(256, 2) void attn_verify_probe_kernel(HatPlanDev p, HatAttn a, uint32_t* sink) {
  constexpr int NS = HD / 16, NC = HD / 32, REC = 2 * 16 * HD;
  const HatAttnItem it = a.items[blockIdx.x];
  const int head = blockIdx.y;
  const SegInfo sg = seg_info(p, it);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = lane >> 5, n = lane & 31;
  int kv_end = it.kv_end < sg.kv_len ? it.kv_end : sg.kv_len;
  const int pair0 = it.kv_begin >> 5, pair1 = (kv_end + 31) >> 5;
  const kv_t* pool = a.pool_layer + (size_t)head * a.n_pages * REC;
  u32x4 acc = {0, 0, 0, 0};
  u32x4 kraw[NS], varaw[NC], vbraw[NC];
  const kv_t *recA = pool, *recB = pool;
  auto page_recs = [&](int pp) {
    int ia = 2 * pp, ib = 2 * pp + 1;
    ib = ib < sg.npages ? ib : sg.npages - 1;
    recA = pool + (size_t)sg.pt[ia] * REC;
    recB = pool + (size_t)sg.pt[ib] * REC;
  };
  auto load_all = [&]() {
    const kv_t* krec = (n < 16) ? recA : recB;
#pragma unroll
    for (int s = 0; s < NS; ++s) kraw[s] = stream_load((const u32x4*)(krec + ((2 * s + half) * 16 + (n & 15)) * 8));
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      varaw[c] = stream_load((const u32x4*)(recA + 16 * HD + c * 512 + lane * 8));
      vbraw[c] = stream_load((const u32x4*)(recB + 16 * HD + c * 512 + lane * 8));
    }
  };
  int pp = pair0 + wave;
  if (pp < pair1) {
    page_recs(pp);
    load_all();
  }
  for (; pp < pair1; pp += 4) {
#pragma unroll
    for (int s = 0; s < NS; ++s) acc ^= kraw[s];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc ^= varaw[c] ^ vbraw[c];
    if (pp + 4 < pair1) {
      page_recs(pp + 4);
      load_all();
    }
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && acc[0] == 0x7f4a7c15u) *sink = 1;
}

// ------------------------------------------------------------------ chunk
// softmax_step in two parts, for the interior stages of the chunk kernel where the
// matrix pipe should stay busy while the VALU does the exponentials: scores -> (maximum,
// exponentials, row sum) touches only the score registers, so it can be scheduled among the
// MFMAs that still accumulate into O; the O rescale and the fp16 pack follow.
__device__ __forceinline__ void softmax_probs(f32x16& s, float scale_log2, float m_run, float& m_new, float& ps) {
  float mx = s[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
  mx = half_max(mx);
  m_new = fmaxf(m_run, mx * scale_log2);
  ps = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2, -m_new));  // scores are finite here: m_new is too
    ps += s[r];
  }
}
__device__ __forceinline__ void probs_to_f16(const f32x16& pv, f16x8& p0, f16x8& p1) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const f32x2 a = {pv[2 * j], pv[2 * j + 1]}, b = {pv[8 + 2 * j], pv[8 + 2 * j + 1]};
    const f16x2 ha = __builtin_convertvector(a, f16x2), hb = __builtin_convertvector(b, f16x2);
    p0[2 * j] = ha[0]; p0[2 * j + 1] = ha[1];
    p1[2 * j] = hb[0]; p1[2 * j + 1] = hb[1];
  }
}

template <int HD, bool KVF16>
__global__ __launch_bounds__(HAT_CHUNK_QROWS * 2) void attn_chunk_kernel(HatPlanDev p, HatAttn a) {
  constexpr int NS = HD / 16;
  constexpr int NC = HD / 32;
  constexpr int REC = 2 * 16 * HD;        // elements of one (page, head) record
  constexpr int RECB = REC * 2;           // bytes
  constexpr int NTH = HAT_CHUNK_QROWS * 2;     // threads: one wave per 32 query rows
  constexpr int LPT = 4 * RECB / 16 / NTH;     // 16-byte loads per thread per 64-key stage
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2][4 * RECB];

  const HatAttnItem it = a.items[blockIdx.x];
  const int head = blockIdx.y;
  const SegInfo sg = seg_info(p, it);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: per-wave decisions become scalar branches
  const int half = lane >> 5, n = lane & 31;
  const int wq0 = it.q0 + 32 * wave;  // first row of this wave, relative to the segment
  int nq_w = it.nq - 32 * wave;       // valid rows of this wave
  nq_w = nq_w > 32 ? 32 : nq_w;
  const bool wave_live = nq_w > 0;
  int qi = wq0 + (n < nq_w ? n : (nq_w > 0 ? nq_w - 1 : 0));
  if (!wave_live) qi = it.q0;  // idle wave: any in-range row
  const int qrow = sg.tok0 + qi;
  const int qpos = sg.start + qi;
  const int wave_last_pos = wave_live ? sg.start + wq0 + nq_w - 1 : -1;
  const int wave_first_pos = sg.start + wq0;
  const float scale_log2 = kLog2e / sqrtf((float)HD);

  f16x8 qreg[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s)
    qreg[s] = *(const f16x8*)(a.qkv + p32_index(qrow, head * HD + (2 * s + half) * 8, 3 * a.d));

  f32x16 o[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[c][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // keys this item needs: [kv_begin, min(kv_end, last row's position + 1))
  int kv_end = it.kv_end;
  const int need = sg.start + it.q0 + it.nq;
  kv_end = kv_end < need ? kv_end : need;
  const int st0 = it.kv_begin >> 6, st1 = (kv_end + 63) >> 6;
  const kv_t* pool = a.pool_layer + (size_t)head * a.n_pages * REC;  // this head's pages are contiguous
  const size_t page_stride = REC;

  // K/V stages travel global -> registers -> (widen to fp16) -> LDS.  The loads of stage
  // st+2 are issued during stage st, right after the registers gave stage st+1 to LDS,
  // and are consumed one whole stage later.
  u32x4 regs[LPT];
  constexpr int UPR = RECB / 16;  // 16-byte units per (page, head) record
  static_assert(UPR % NTH == 0 || NTH == 2 * UPR, "a thread's i-th unit lies in a page that is the same for its whole wave");
  const uint32_t lane_off = (UPR >= NTH ? threadIdx.x : threadIdx.x % UPR) * 16;
  const int tsub = UPR >= NTH ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x / UPR);  // which of the two pages unit i spans
  int pgid[4];  // page ids of the stage to load next (the same for every thread)
  auto load_page_ids = [&](int st) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      int pi = st * 4 + k;
      pi = pi < sg.npages ? pi : sg.npages - 1;
      pgid[k] = sg.pt[pi];
    }
  };
  auto gload_one = [&](auto ic) {
    constexpr int i = decltype(ic)::value;
    int page;
    uint32_t off;
    if constexpr (UPR >= NTH) {  // the same page for the whole workgroup
      constexpr int pg = (i * NTH) / UPR, off0 = (i * NTH) % UPR;
      page = pgid[pg];
      off = lane_off + off0 * 16;
    } else {                     // the workgroup's i-th units span two pages, one per half
      page = tsub ? pgid[2 * i + 1] : pgid[2 * i];
      off = lane_off;
    }
    page = __builtin_amdgcn_readfirstlane(page);
    const unsigned char* rec = (const unsigned char*)pool + (size_t)page * RECB;  // wave-uniform
    regs[i] = *(const u32x4*)(rec + off);
  };
  auto gload = [&](int st) {
    load_page_ids(st);
    hat_static_for<LPT>([&](auto ic) { gload_one(ic); });
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LPT; ++i) *(u32x4*)(&lds[buf][(i * NTH + threadIdx.x) * 16]) = kv_to_f16_bits<KVF16>(regs[i]);
  };
  // general stage: causal masks, ragged ends, waves that skip a 32-key half
  auto compute = [&](int st, int buf) {
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      const int key0 = st * 64 + pr * 32;
      if (key0 > wave_last_pos || key0 >= kv_end) continue;  // wave-uniform
      const unsigned char* recA = &lds[buf][(2 * pr) * RECB];
      const unsigned char* recB = recA + RECB;
      const unsigned char* krec = (n < 16) ? recA : recB;
      f32x16 sacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const f16x8 kk = *(const f16x8*)(krec + ((2 * s + half) * 16 + (n & 15)) * 16);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kk, qreg[s], sacc, 0, 0, 0);
      }
      f16x8 p0, p1;
      if (key0 + 31 > wave_first_pos) softmax_step<NC, 1>(sacc, scale_log2, key0, half, qpos, m_run, l_run, o, p0, p1);
      else softmax_step<NC, 0>(sacc, scale_log2, key0, half, qpos, m_run, l_run, o, p0, p1);
      const bool tail = key0 + 32 > sg.kv_len;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        f16x8 va = *(const f16x8*)(recA + 16 * HD * 2 + c * 1024 + lane * 16);
        f16x8 vb = *(const f16x8*)(recB + 16 * HD * 2 + c * 1024 + lane * 16);
        if (tail) {
          va = clean_v(va, key0, half, sg.kv_len);
          vb = clean_v(vb, key0 + 16, half, sg.kv_len);
        }
        o[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, p0, o[c], 0, 0, 0);
        o[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vb, p1, o[c], 0, 0, 0);
      }
    }
  };
  // interior stage: all 64 keys lie at or below every row of the wave, so there is no
  // mask, no skipping and no ragged end.  Hand-scheduled: the 32 MFMAs go out in 8 groups
  // of 4 (scores of half A, scores of half B, O update with A, O update with B); the LDS
  // operands of group g+1 are fetched before the MFMAs of group g are issued, and between
  // consecutive MFMAs sits a slice of VALU work that does not depend on them -- widening
  // the next stage's K/V registers into LDS under the scores of A, the exponentials of A
  // under the scores of B, the exponentials of B under the O update with A -- so the
  // matrix pipe and the VALU of one wave run at the same time.
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)&lds[0][0];
  const uint32_t kaddr0 = lds_base + (n < 16 ? 0 : RECB) + (half * 16 + (n & 15)) * 16;
  const uint32_t vaddr0 = lds_base + 16 * HD * 2 + lane * 16;
  // MFMAs of a stage in issue order: m in [0, NS): scores of A, k-step m; [NS, 2 NS): scores
  // of B; then 2 NC O updates with A (32-row block c = idx/2, page idx%2 of the pair), then
  // 2 NC with B.  Operands are fetched from LDS GS MFMAs ahead.
  constexpr int GS = 2;
  constexpr int NM = 2 * NS + 4 * NC, NG = NM / GS;
  static_assert(NM % GS == 0 && NS % GS == 0 && (2 * NC) % GS == 0, "groups do not straddle phases");
  auto stage_interior = [&](int st, int buf, bool do_store, bool do_load) {
    const uint32_t ka = kaddr0 + buf * (4 * RECB), va = vaddr0 + buf * (4 * RECB);
    hat_f16x8 op[2][GS];
    f32x16 sA, sB;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f16x8 p0, p1;
    float mx = 0.f, m_new = 0.f, ps = 0.f;
    auto load_operand = [&](auto mc, hat_f16x8& dst) {
      constexpr int m = decltype(mc)::value;
      if constexpr (m < 2 * NS) {
        constexpr int sub = m / NS, ks = m % NS;
        dst = hat_lds_read<sub * 2 * RECB + ks * 512>(ka);
      } else {
        constexpr int idx = m - 2 * NS, sub = idx / (2 * NC), c = (idx % (2 * NC)) / 2, rec = idx % 2;
        dst = hat_lds_read<(sub * 2 + rec) * RECB + c * 1024>(va);
      }
    };
    // exponentials of elements [r0, r1) of a score tile, in place, and their sum
    // (the empty asm statements keep the optimiser from sinking a slice's arithmetic down to
    // where its results are used, which would undo the interleaving)
    auto exps = [&](f32x16& sc, int r0, int r1) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (r >= r0 && r < r1) {
          float e = __builtin_amdgcn_exp2f(fmaf(sc[r], scale_log2, -m_new));
          asm volatile("" : "+v"(e));
          sc[r] = e;
          ps += e;
        }
      asm volatile("" : "+v"(ps));
    };
    // softmax of one 32-key half in NSL slices: 0 = row maximum, 1 = exchange between the lane
    // halves, the rest = exponentials
    auto softmax_slice = [&](f32x16& sc, auto qc, auto nslc) {
      constexpr int q = decltype(qc)::value, NSL = decltype(nslc)::value;
      if constexpr (q == 0) {
        mx = sc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
        asm volatile("" : "+v"(mx));
      } else if constexpr (q == 1) {
        mx = half_max(mx);
        m_new = fmaxf(m_run, mx * scale_log2);
        asm volatile("" : "+v"(m_new));
        ps = 0.f;
      } else {
        constexpr int parts = NSL - 2;
        exps(sc, (q - 2) * 16 / parts, (q - 1) * 16 / parts);
      }
    };
    auto rescale = [&]() {
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {  // wave-uniform: some row's maximum moved
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[c][r] *= alpha;
        m_run = m_new;
      }
      l_run += ps;
    };

    if (do_load) load_page_ids(st + 2);  // consumed under the scores of B, half a stage from here
    hat_static_for<GS>([&](auto jc) { load_operand(jc, op[0][decltype(jc)::value]); });
    hat_static_for<NG>([&](auto gc) {
      constexpr int G = decltype(gc)::value;
      constexpr int cur = G & 1;
      hat_wait_operands(op[cur]);
      if constexpr (G + 1 < NG)
        hat_static_for<GS>([&](auto jc) {
          load_operand(std::integral_constant<int, (G + 1) * GS + decltype(jc)::value>{}, op[cur ^ 1][decltype(jc)::value]);
        });
      if constexpr (G * GS == 2 * NS) {              // scores of A are soft-maxed: pack them for the O update
        rescale();
        probs_to_f16(sA, p0, p1);
      } else if constexpr (G * GS == 2 * NS + 2 * NC) {
        rescale();
        probs_to_f16(sB, p0, p1);
      }
      __builtin_amdgcn_sched_barrier(0);
      hat_static_for<GS>([&](auto jc) {
        constexpr int j = decltype(jc)::value, m = G * GS + j;
        if constexpr (m < NS) {                                  // scores of A | widen next stage into LDS
          sA = __builtin_amdgcn_mfma_f32_32x32x16_f16(op[cur][j], qreg[m], m == 0 ? zero16 : sA, 0, 0, 0);
          if constexpr (m < LPT) {
            if (do_store) *(u32x4*)(&lds[buf ^ 1][(m * NTH + threadIdx.x) * 16]) = kv_to_f16_bits<KVF16>(regs[m]);
          }
        } else if constexpr (m < 2 * NS) {                       // scores of B | loads of stage st+2, softmax of A
          constexpr int q = m - NS;
          sB = __builtin_amdgcn_mfma_f32_32x32x16_f16(op[cur][j], qreg[q], q == 0 ? zero16 : sB, 0, 0, 0);
          if constexpr (q < LPT) {
            if (do_load) gload_one(std::integral_constant<int, q>{});
          }
          softmax_slice(sA, std::integral_constant<int, q>{}, std::integral_constant<int, NS>{});
        } else if constexpr (m < 2 * NS + 2 * NC) {              // O update with A | softmax of B
          constexpr int q = m - 2 * NS, c = q / 2;
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(op[cur][j], (q % 2) ? p1 : p0, o[c], 0, 0, 0);
          softmax_slice(sB, std::integral_constant<int, q>{}, std::integral_constant<int, 2 * NC>{});
        } else {                                                 // O update with B
          constexpr int q = m - 2 * NS - 2 * NC, c = q / 2;
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(op[cur][j], (q % 2) ? p1 : p0, o[c], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    });
  };

  if (st0 < st1) {  // tiles are widened to fp16 once, on their way into LDS
    gload(st0);
    lstore(0);
    if (st0 + 1 < st1) gload(st0 + 1);
  }
  __syncthreads();

  // LDS[buf] holds stage st; the registers hold stage st+1, whose buffer everyone left at
  // the barrier that ended stage st-1.  A wave's interior stages come first (two loops, so
  // that each gets its own register allocation); every wave passes one barrier per stage.
  int st_int = (wave_first_pos + 1) >> 6;
  st_int = st_int < (kv_end >> 6) ? st_int : (kv_end >> 6);
  if (!wave_live || st_int < st0) st_int = st0;
  int st = st0;
  for (; st < st_int; ++st) {
    stage_interior(st, (st - st0) & 1, st + 1 < st1, st + 2 < st1);
    __syncthreads();
  }
  for (; st < st1; ++st) {
    const int buf = (st - st0) & 1;
    if (st + 1 < st1) lstore(buf ^ 1);
    if (st + 2 < st1) gload(st + 2);
    compute(st, buf);
    __syncthreads();
  }
  l_run += __shfl_xor(l_run, 32);

  if (n < nq_w) {
    const int row = wq0 + n;  // relative to segment
    if (it.part_row < 0) {
      const float inv = 1.0f / l_run;
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = to_act(o[c][4 * g + e] * inv);
          *(f16x4*)(a.outP + p32_index(sg.tok0 + row, head * HD + 32 * c + 8 * g + 4 * half, a.d)) = ov;
        }
    } else {
      const size_t prow = (size_t)(it.part_row + 32 * wave + n) * a.H + head;
      const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;   // 0: this key range lies beyond the row's position
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f16x4 ov;
#pragma unroll
          for (int e = 0; e < 4; ++e) ov[e] = to_act(o[c][4 * g + e] * inv);
          *(f16x4*)(a.part_o + prow * HD + 32 * c + 8 * g + 4 * half) = ov;
        }
      if (half == 0) a.part_ml[prow] = make_float2(m_run, l_run);
    }
  }
}

// ------------------------------------------------------------------ merge
// one workgroup per (group of <= 16 rows, head); one thread per (row, 8 features)
template <int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(HatAttn a, const HatMergeItem* __restrict__ items) {
  const HatMergeItem it = items[blockIdx.x];
  const int head = blockIdx.y;
  for (int idx = threadIdx.x; idx < it.nrows * (HD / 8); idx += 256) {
    const int r = idx / (HD / 8), e = (idx % (HD / 8)) * 8;
    // both passes take the key ranges four at a time, loads first: a loop that loads one range per
    // pass waits out a memory round trip per range (the order of the sums is unchanged)
    const size_t pr0 = (size_t)(it.part_row + r) * a.H + head, prs = (size_t)it.stride * a.H;
    float M = -INFINITY;
    for (int s0 = 0; s0 < it.nsplit; s0 += 4) {
      float mx[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (s0 + u < it.nsplit) mx[u] = a.part_ml[pr0 + (s0 + u) * prs].x;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (s0 + u < it.nsplit) M = fmaxf(M, mx[u]);
    }
    float L = 0.f;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int s0 = 0; s0 < it.nsplit; s0 += 4) {
      float2 ml[4];
      f16x8 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (s0 + u < it.nsplit) {
          const size_t pr = pr0 + (s0 + u) * prs;
          ml[u] = a.part_ml[pr];
          v[u] = *(const f16x8*)(a.part_o + pr * HD + e);
        }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (s0 + u < it.nsplit) {
          const float f = ml[u].y * exp2f(ml[u].x - M);   // weight of this key range: its sum, on the common scale
          L += f;
#pragma unroll
          for (int x = 0; x < 8; ++x) acc[x] += (float)v[u][x] * f;
        }
    }
    const float inv = 1.0f / L;
    f16x8 ov;
#pragma unroll
    for (int x = 0; x < 8; ++x) ov[x] = to_act(acc[x] * inv);
    *(f16x8*)(a.outP + p32_index(it.row0 + r, head * HD + e, a.d)) = ov;
  }
}

}  // namespace

hipError_t hat_launch_attn_chunk(const HatPlanDev& p, const HatAttn& a, hipStream_t st) {
  if (a.n_items <= 0) return hipSuccess;
  dim3 grid(a.n_items, a.H);
  if (a.hd == 128 && a.kv_f16) attn_chunk_kernel<128, true><<<grid, HAT_CHUNK_QROWS * 2, 0, st>>>(p, a);
  else if (a.hd == 128) attn_chunk_kernel<128, false><<<grid, HAT_CHUNK_QROWS * 2, 0, st>>>(p, a);
  else if (a.hd == 64 && a.kv_f16) attn_chunk_kernel<64, true><<<grid, HAT_CHUNK_QROWS * 2, 0, st>>>(p, a);
  else if (a.hd == 64) attn_chunk_kernel<64, false><<<grid, HAT_CHUNK_QROWS * 2, 0, st>>>(p, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t hat_launch_attn_verify(const HatPlanDev& p, const HatAttn& a, hipStream_t st) {
  if (a.n_items <= 0) return hipSuccess;
  dim3 grid(a.n_items, a.H);
  if (a.hd == 128 && a.kv_f16) attn_verify_kernel<128, true><<<grid, 256, 0, st>>>(p, a);
  else if (a.hd == 128) attn_verify_kernel<128, false><<<grid, 256, 0, st>>>(p, a);
  else if (a.hd == 64 && a.kv_f16) attn_verify_kernel<64, true><<<grid, 256, 0, st>>>(p, a);
  else if (a.hd == 64) attn_verify_kernel<64, false><<<grid, 256, 0, st>>>(p, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t hat_launch_attn_verify_probe(const HatPlanDev& p, const HatAttn& a, uint32_t* sink, hipStream_t st) {
  if (a.n_items <= 0) return hipSuccess;
  dim3 grid(a.n_items, a.H);
  if (a.hd == 128) attn_verify_probe_kernel<128><<<grid, 256, 0, st>>>(p, a, sink);
  else if (a.hd == 64) attn_verify_probe_kernel<64><<<grid, 256, 0, st>>>(p, a, sink);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t hat_launch_attn_merge(const HatAttn& a, const HatMergeItem* items, int n_items, hipStream_t st) {
  if (n_items <= 0) return hipSuccess;
  dim3 grid(n_items, a.H);
  if (a.hd == 128) attn_merge_kernel<128><<<grid, 256, 0, st>>>(a, items);
  else if (a.hd == 64) attn_merge_kernel<64><<<grid, 256, 0, st>>>(a, items);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
