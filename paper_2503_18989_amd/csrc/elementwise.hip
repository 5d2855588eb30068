// Bandwidth-bound kernels of the decoder layer: RMSNorm, rotary embedding fused
// with the KV-cache append, the ragged gather/scatter between the callers'
// per-device hidden-state arrays and the batch, and the layout conversions used
// at create time and by the fixtures.  (Layer structure: paper Sec. 2.1; KV
// cache: Sec. 2.1; hidden states in / deep hidden states out: Sec. 3.1, Fig. 3.)
#include <hip/hip_runtime.h>

#include "hat_kernels.h"
#include "hat_layout.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// fp32 -> fp16, round to nearest even, saturating instead of overflowing to infinity
__device__ __forceinline__ _Float16 to_act(float x) { return (_Float16)__builtin_amdgcn_fmed3f(x, -65504.f, 65504.f); }
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint16_t kvx8 __attribute__((ext_vector_type(8)));

// eight values -> eight cache elements: bf16 (round to nearest even) or fp16 (the same, saturating)
template <bool KVF16>
__device__ __forceinline__ kvx8 to_kv(const float (&x)[8]) {
  if constexpr (KVF16) {
    f16x8 h;
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = to_act(x[e]);
    return __builtin_bit_cast(kvx8, h);
  } else {
    bf16x8 b;
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = (__bf16)x[e];
    return __builtin_bit_cast(kvx8, b);
  }
}
template <bool KVF16>
__device__ __forceinline__ float kv_to_float(kv_t x) {
  if constexpr (KVF16) return (float)__builtin_bit_cast(_Float16, x);
  else return (float)__builtin_bit_cast(__bf16, x);
}
template <bool KVF16>
__device__ __forceinline__ kv_t float_to_kv(float x) {
  if constexpr (KVF16) return __builtin_bit_cast(kv_t, to_act(x));
  else return __builtin_bit_cast(kv_t, (__bf16)x);
}

namespace {

// ---------------------------------------------------------------- gather/scatter
// one workgroup per batch row; io_dtype 0 = bf16, 1 = f32
__global__ void gather_kernel(HatPlanDev p, float* __restrict__ resid, int d, int io_dtype) {
  const int t = blockIdx.x;
  const int s = p.tok_seg[t];
  const int row = t - p.tok_off[s];
  float* dst = resid + (size_t)t * d;
  if (io_dtype == 0) {
    const bf16_t* src = (const bf16_t*)p.in_ptr[s] + (size_t)row * d;
    for (int i = threadIdx.x * 8; i < d; i += blockDim.x * 8) {
      bf16x8 v = *(const bf16x8*)(src + i);
      f32x4 a, b;
#pragma unroll
      for (int e = 0; e < 4; ++e) { a[e] = (float)v[e]; b[e] = (float)v[4 + e]; }
      *(f32x4*)(dst + i) = a;
      *(f32x4*)(dst + i + 4) = b;
    }
  } else {
    const float* src = (const float*)p.in_ptr[s] + (size_t)row * d;
    for (int i = threadIdx.x * 4; i < d; i += blockDim.x * 4) *(f32x4*)(dst + i) = *(const f32x4*)(src + i);
  }
}

__global__ void scatter_kernel(HatPlanDev p, const float* __restrict__ resid, const float* __restrict__ part,
                               int nparts, int d, int io_dtype) {
  const int t = blockIdx.x;
  const int s = p.tok_seg[t];
  const int row = t - p.tok_off[s];
  const float* src = resid + (size_t)t * d;
  const size_t pstride = (size_t)p.T * d;
  for (int i = threadIdx.x * 4; i < d; i += blockDim.x * 4) {
    f32x4 a = *(const f32x4*)(src + i);
    for (int q = 0; q < nparts; ++q) {
      const f32x4 b = *(const f32x4*)(part + q * pstride + (size_t)t * d + i);
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] += b[e];
    }
    if (io_dtype == 0) {
      bf16_t* dst = (bf16_t*)p.out_ptr[s] + (size_t)row * d;
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (__bf16)a[e];
      *(bf16x4*)(dst + i) = v;
    } else {
      float* dst = (float*)p.out_ptr[s] + (size_t)row * d;
      *(f32x4*)(dst + i) = a;
    }
  }
}

// ---------------------------------------------------------------- rotary table
// table[t][i] = (cos, sin)(pos[t] * inv_freq[i]), angle and functions in double:
// positions reach several thousand radians, where float arguments lose digits.
__global__ void rope_table_kernel(HatPlanDev p, const double* __restrict__ inv_freq, float2* __restrict__ table,
                                  int half) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= p.T * half) return;
  const int t = idx / half, i = idx % half;
  const double ang = (double)p.pos[t] * inv_freq[i];
  double s, c;
  sincos(ang, &s, &c);
  table[idx] = make_float2((float)c, (float)s);
}

// a, b += the 8 floats at pp of each of the nparts split-K partial sums (pstride floats apart), added in
// ascending order of the split.  The loads of four splits are issued before the first of them is
// used: a loop that loads one split per pass waits out a memory round trip per split.
__device__ __forceinline__ void fold_partials(f32x4& a, f32x4& b, const float* __restrict__ pp, size_t pstride, int nparts) {
  for (int q0 = 0; q0 < nparts; q0 += 4) {
    f32x4 pa[4], pb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (q0 + u < nparts) {
        const float* src = pp + (size_t)(q0 + u) * pstride;
        pa[u] = *(const f32x4*)src;
        pb[u] = *(const f32x4*)(src + 4);
      }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (q0 + u < nparts) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { a[e] += pa[u][e]; b[e] += pb[u][e]; }
      }
  }
}

// ---------------------------------------------------------------- RMSNorm
// one workgroup (256 threads) per row: x = resid + pending split-K partial sums
// (written back), y = x * rsqrt(mean(x^2) + eps) * gain as fp16 in P32 layout.
// A row (<= 8192 floats) stays in registers between the two passes.
__global__ __launch_bounds__(256) void rmsnorm_kernel(float* __restrict__ resid, const float* __restrict__ part,
                                                       int nparts, int T, const float* __restrict__ gain,
                                                       act_t* __restrict__ outP, int d, float eps) {
  const int t = blockIdx.x;
  float* x = resid + (size_t)t * d;
  const size_t pstride = (size_t)T * d;
  constexpr int MAXV = 4;  // 256 threads * 8 floats * 4 = 8192 columns held in registers
  f32x4 va[MAXV], vb[MAXV];
  float ss = 0.f;
#pragma unroll
  for (int v = 0; v < MAXV; ++v) {
    const int i = (v * 256 + threadIdx.x) * 8;
    if (i < d) {
      f32x4 a = *(const f32x4*)(x + i), b = *(const f32x4*)(x + i + 4);
      fold_partials(a, b, part + (size_t)t * d + i, pstride, nparts);
      if (nparts > 0) { *(f32x4*)(x + i) = a; *(f32x4*)(x + i + 4) = b; }
#pragma unroll
      for (int e = 0; e < 4; ++e) ss += a[e] * a[e] + b[e] * b[e];
      va[v] = a; vb[v] = b;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = red[0] + red[1] + red[2] + red[3];
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int v = 0; v < MAXV; ++v) {
    const int i = (v * 256 + threadIdx.x) * 8;
    if (i < d) {
      const f32x4 ga = *(const f32x4*)(gain + i), gb = *(const f32x4*)(gain + i + 4);
      f16x8 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) { o[e] = to_act(va[v][e] * r * ga[e]); o[4 + e] = to_act(vb[v][e] * r * gb[e]); }
      *(f16x8*)(outP + p32_index(t, i, d)) = o;
    }
  }
}

// The same for batches of many rows: a workgroup takes R consecutive rows (one wave per row, the
// row in registers between the two passes) and passes the fp16 results through LDS so that a
// store instruction writes, for each 8-feature octet, the R rows' 16-byte pieces that lie next
// to each other in the P32 layout (R x 16 contiguous bytes instead of 16: with one row per
// workgroup the 16-byte stores are two thirds of the kernel's time at thousands of rows;
// measured 34 -> 19 us at 3556 x 4096 and 49 -> 31 us at 4096 x 5120 with R = 4).  The
// 16-byte chunk of octet o of row r sits at chunk position o ^ r of the row, so that both the
// row-wise writes and the octet-wise reads spread over the banks.  Rows of at most MAXD floats.
template <int R, int MAXD>
__global__ __launch_bounds__(256) void rmsnorm_rows_kernel(float* __restrict__ resid, const float* __restrict__ part,
                                                            int nparts, int T, const float* __restrict__ gain,
                                                            act_t* __restrict__ outP, int d, float eps) {
  static_assert(R * MAXD * 2 <= 65536 && MAXD % 512 == 0, "the rows of a group fit in LDS");
  __shared__ __attribute__((aligned(16))) unsigned char tile[R * MAXD * 2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * R;
  const size_t pstride = (size_t)T * d;
  const int noct = d >> 3;
  constexpr int MAXO = MAXD / 8 / 64;   // octets per lane of the longest row
  for (int rr = wave; rr < R; rr += 4) {
    const int t = t0 + rr;
    if (t >= T) break;   // the same for every lane of the wave
    float* x = resid + (size_t)t * d;
    f32x4 va[MAXO], vb[MAXO];
    float ss = 0.f;
#pragma unroll
    for (int v = 0; v < MAXO; ++v) {
      const int i = (v * 64 + lane) * 8;
      if (i < d) {
        f32x4 a = *(const f32x4*)(x + i), b = *(const f32x4*)(x + i + 4);
        fold_partials(a, b, part + (size_t)t * d + i, pstride, nparts);
        if (nparts > 0) { *(f32x4*)(x + i) = a; *(f32x4*)(x + i + 4) = b; }
#pragma unroll
        for (int e = 0; e < 4; ++e) ss += a[e] * a[e] + b[e] * b[e];
        va[v] = a; vb[v] = b;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int v = 0; v < MAXO; ++v) {
      const int oct = v * 64 + lane;
      if (oct < noct) {
        const f32x4 ga = *(const f32x4*)(gain + oct * 8), gb = *(const f32x4*)(gain + oct * 8 + 4);
        f16x8 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) { o[e] = to_act(va[v][e] * r * ga[e]); o[4 + e] = to_act(vb[v][e] * r * gb[e]); }
        *(f16x8*)(tile + (size_t)rr * d * 2 + ((oct ^ rr) << 4)) = o;
      }
    }
  }
  __syncthreads();
  const int rows = (T - t0) < R ? (T - t0) : R;
  for (int idx = threadIdx.x; idx < noct * R; idx += 256) {
    const int rr = idx % R, oct = idx / R;
    if (rr < rows)
      *(f16x8*)(outP + p32_index(t0 + rr, oct * 8, d)) = *(const f16x8*)(tile + (size_t)rr * d * 2 + ((oct ^ rr) << 4));
  }
}

// ---------------------------------------------------------------- RoPE + KV append
// Two kinds of workgroups in one launch.
//  (a) the first n_kblocks: one thread per (row, head, octet pair): octets o and o + hd/16 hold
//      the two halves of 8 rotation pairs.  q is rotated in place (fp16); rotated k is rounded
//      to the cache type and written to the row's (page, slot) of this layer's pool as two
//      16-byte octets.
//  (b) the rest: one workgroup per V tile of an appended (page, head) (two tiles at hd = 64).
//      A thread loads one 16-byte octet of one of the page's 16 rows (consecutive lanes:
//      consecutive rows, 256-byte runs of the P32 layout), scatters its 8 values into an LDS
//      image of the tile (whose order is [hd/32][slot half][feature][8 slots]), and after the
//      barrier writes one 16-byte piece of the image: the workgroup stores the tile as one
//      contiguous run.  Slots that are not new in this step keep their old contents.
template <bool KVF16, int HD>
__global__ __launch_bounds__(256) void rope_append_kernel(HatPlanDev p, act_t* __restrict__ qkv,
                                                           const float2* __restrict__ table, kv_t* __restrict__ pool,
                                                           int n_pages, int H, int n_kblocks) {
  constexpr int hd = HD;
  constexpr int half_oct = hd >> 4;             // octets per half head
  const int d = H * hd, row_len = 3 * d;
  if ((int)blockIdx.x < n_kblocks) {
    const int per_row = H * half_oct;
    const int n_a = p.T * per_row;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n_a) return;
    // consecutive lanes take consecutive rows of one (head, octet pair): 32 rows of a
    // P32 panel are one 512-byte run, and consecutive slots of a K tile are contiguous
    const int t = idx % p.T, rem = idx / p.T;
    const int hh = rem / half_oct, o = rem % half_oct;
    const int c_lo = hh * hd + o * 8, c_hi = c_lo + (hd >> 1);
    const float2* cs = table + (size_t)t * (hd >> 1) + o * 8;

    act_t* q_lo = qkv + p32_index(t, c_lo, row_len);
    act_t* q_hi = qkv + p32_index(t, c_hi, row_len);
    const f16x8 ql = *(f16x8*)q_lo, qh = *(f16x8*)q_hi;
    const f16x8 kl = *(const f16x8*)(qkv + p32_index(t, d + c_lo, row_len));
    const f16x8 kh = *(const f16x8*)(qkv + p32_index(t, d + c_hi, row_len));
    f16x8 rql, rqh;
    float rkl[8], rkh[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float c = cs[e].x, s = cs[e].y;
      const float a = (float)ql[e], b = (float)qh[e];
      rql[e] = to_act(a * c - b * s);
      rqh[e] = to_act(b * c + a * s);
      const float ka = (float)kl[e], kb = (float)kh[e];
      rkl[e] = ka * c - kb * s;
      rkh[e] = kb * c + ka * s;
    }
    *(f16x8*)q_lo = rql;
    *(f16x8*)q_hi = rqh;
    const int dst = p.kv_dst[t];
    const int page = dst >> 4, slot = dst & 15;
    kv_t* kt = pool + ((size_t)hh * n_pages + page) * kv_head_elems(hd);
    *(kvx8*)(kt + ktile_index(slot, o * 8)) = to_kv<KVF16>(rkl);
    *(kvx8*)(kt + ktile_index(slot, o * 8 + (hd >> 1))) = to_kv<KVF16>(rkh);
    return;
  }
  constexpr int PIECES = hd * 2;       // 16-byte pieces of one V tile (16 slots x hd two-byte elements)
  constexpr int TPB = 256 / PIECES;    // tiles per workgroup
  // 16 bytes of padding after every 512 (one slot half of a 32-feature block), so that the two
  // slot halves and neighbouring octets do not fall on the same banks when the rows are scattered
  constexpr int IMG = PIECES * 16 + (PIECES / 32) * 16;
  __shared__ __attribute__((aligned(16))) unsigned char image[TPB][IMG];
  const int tb = threadIdx.x / PIECES, q = threadIdx.x % PIECES;
  const int tix = ((int)blockIdx.x - n_kblocks) * TPB + tb;
  const bool live = tix < p.n_append * H;
  HatAppendItem it{};
  int hh = 0;
  if (live) {
    it = p.append[tix % p.n_append];
    hh = tix / p.n_append;
    const int r = q & 15, o = q >> 4;   // slot and octet of this thread's load
    const int pos = it.pos0 + r;
    if (pos >= it.lo && pos < it.hi) {
      const f16x8 x = *(const f16x8*)(qkv + p32_index(it.row0 + r, 2 * d + hh * hd + o * 8, row_len));
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int byte = vtile_index(r, o * 8 + e) * 2;
        byte += (byte >> 9) * 16;
        const _Float16 xe = x[e];   // (a copy: bit_cast must not be handed the vector element itself)
        *(kv_t*)(&image[tb][byte]) = KVF16 ? __builtin_bit_cast(kv_t, xe) : float_to_kv<false>((float)xe);
      }
    }
  }
  __syncthreads();
  if (!live) return;
  kv_t* dst = pool + ((size_t)hh * n_pages + it.page) * kv_head_elems(hd) + 16 * hd + q * 8;
  kvx8 out = *(const kvx8*)(&image[tb][q * 16 + (q >> 5) * 16]);
  if (it.lo > it.pos0 || it.hi < it.pos0 + 16) {   // a partly new page: the other slots keep what they hold
    const kvx8 old = *(const kvx8*)dst;
    const int h = (q >> 5) & 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int pos = it.pos0 + 8 * (j >> 2) + 4 * h + (j & 3);
      if (pos < it.lo || pos >= it.hi) out[j] = old[j];
    }
  }
  *(kvx8*)dst = out;
}

// ---------------------------------------------------------------- weight re-tiling
__global__ void retile_kernel(act_t* __restrict__ dst, int Nw, int Kd, const bf16_t* __restrict__ s0,
                              const bf16_t* __restrict__ s1, const bf16_t* __restrict__ s2, int n0, int Ks, int mode) {
  // one thread per destination octet
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)Nw * (Kd >> 3);
  if (idx >= total) return;
  // destination order: [panel][octet][row%32]
  const int r32 = (int)(idx & 31);
  const size_t po = idx >> 5;
  const int oct = (int)(po % (size_t)(Kd >> 3));
  const int R = (int)(po / (size_t)(Kd >> 3)) * 32 + r32;
  const bf16_t* src = nullptr;
  int sr = -1;
  if (mode == 0) {
    if (R < n0) { src = s0; sr = R; }
  } else if (mode == 1) {
    if (R < 3 * n0) { src = R < n0 ? s0 : R < 2 * n0 ? s1 : s2; sr = R % n0; }
  } else {
    // gate/up: every 32-row block = 16 gate rows, then the up rows of the same 16 features
    const int blk = R >> 5, w = R & 31;
    const int f = blk * 16 + (w & 15);
    if (f < n0) { src = (w < 16) ? s0 : s1; sr = f; }
  }
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.f;
  if (src) {
    const int k = oct * 8;
    if (k + 8 <= Ks) {
      if ((Ks & 7) == 0) {
        v = *(const bf16x8*)(src + (size_t)sr * Ks + k);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[(size_t)sr * Ks + k + e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (k + e < Ks) v[e] = src[(size_t)sr * Ks + k + e];
    }
  }
  // bf16 -> fp16 through fp32: exact for |w| in [2^-17, 65504] (8 mantissa bits fit in 11);
  // smaller magnitudes keep an absolute error below 2^-25, larger ones saturate
  f16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = to_act((float)v[e]);
  *(f16x8*)(dst + idx * 8) = o;
}

__global__ void bf16_to_f32_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = (float)src[i];
}

// ---------------------------------------------------------------- fixtures
// one thread per (row, head, octet)
template <bool KVF16>
__global__ void kv_import_kernel(kv_t* __restrict__ pool, int n_pages, const int32_t* __restrict__ pages, int pos0, int n,
                                 const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int H, int hd) {
  const int octs = hd >> 3;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * H * octs) return;
  const int o = (int)(idx % octs);
  const int hh = (int)((idx / octs) % H);
  const int r = (int)(idx / ((size_t)octs * H));
  const int pos = pos0 + r;
  const int page = pages[(pos >> 4) - (pos0 >> 4)], slot = pos & 15;
  kv_t* kt = pool + ((size_t)hh * n_pages + page) * kv_head_elems(hd);
  kv_t* vt = kt + 16 * hd;
  const size_t so = ((size_t)r * H + hh) * hd + o * 8;
  const bf16x8 kk = *(const bf16x8*)(k + so);
  const bf16x8 vv = *(const bf16x8*)(v + so);
  float kf[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) kf[e] = (float)kk[e];
  *(kvx8*)(kt + ktile_index(slot, o * 8)) = to_kv<KVF16>(kf);      // bf16 -> bf16 is the identity
#pragma unroll
  for (int e = 0; e < 8; ++e) vt[vtile_index(slot, o * 8 + e)] = float_to_kv<KVF16>((float)vv[e]);
}

template <bool KVF16>
__global__ void kv_export_kernel(const kv_t* __restrict__ pool, int n_pages, const int32_t* __restrict__ pages, int pos0, int n,
                                 bf16_t* __restrict__ k, bf16_t* __restrict__ v, int H, int hd) {
  const int octs = hd >> 3;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * H * octs) return;
  const int o = (int)(idx % octs);
  const int hh = (int)((idx / octs) % H);
  const int r = (int)(idx / ((size_t)octs * H));
  const int pos = pos0 + r;
  const int page = pages[(pos >> 4) - (pos0 >> 4)], slot = pos & 15;
  const kv_t* kt = pool + ((size_t)hh * n_pages + page) * kv_head_elems(hd);
  const kv_t* vt = kt + 16 * hd;
  const size_t so = ((size_t)r * H + hh) * hd + o * 8;
  const kvx8 kk = *(const kvx8*)(kt + ktile_index(slot, o * 8));
  bf16x8 ko, vv;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ko[e] = (__bf16)kv_to_float<KVF16>(kk[e]);
    vv[e] = (__bf16)kv_to_float<KVF16>(vt[vtile_index(slot, o * 8 + e)]);
  }
  *(bf16x8*)(k + so) = ko;
  *(bf16x8*)(v + so) = vv;
}

// One thread per (layer, head, octet of the head): applies the row moves in order.  The moves
// of a kept tree path go to lower-or-equal rows in ascending order, so a destination is never a
// source of a later move, and no two threads touch the same bytes.
__global__ void kv_move_kernel(kv_t* __restrict__ pool, size_t layer_elems, int L, int n_pages, HatRowMoves mv, int H,
                               int hd) {
  const int octs = hd >> 3;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)L * H * octs) return;
  const int o = (int)(idx % octs);
  const int hh = (int)((idx / octs) % H);
  const int l = (int)(idx / ((size_t)octs * H));
  kv_t* base = pool + (size_t)l * layer_elems + (size_t)hh * n_pages * kv_head_elems(hd);
  for (int m = 0; m < mv.n; ++m) {
    kv_t* sp = base + (size_t)(mv.src[m] >> 4) * kv_head_elems(hd);
    kv_t* dp = base + (size_t)(mv.dst[m] >> 4) * kv_head_elems(hd);
    const int ss = mv.src[m] & 15, ds = mv.dst[m] & 15;
    *(kvx8*)(dp + ktile_index(ds, o * 8)) = *(const kvx8*)(sp + ktile_index(ss, o * 8));
#pragma unroll
    for (int e = 0; e < 8; ++e) dp[16 * hd + vtile_index(ds, o * 8 + e)] = sp[16 * hd + vtile_index(ss, o * 8 + e)];
  }
}

__global__ void unpack_p32_kernel(const act_t* __restrict__ srcP, int row_len, int col0, int ncols, int T,
                                  float* __restrict__ dst) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)T * ncols) return;
  const int t = (int)(idx / ncols), c = (int)(idx % ncols);
  dst[idx] = (float)srcP[p32_index(t, col0 + c, row_len)];
}

inline unsigned blocks_for(size_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

}  // namespace

hipError_t hat_launch_gather(const HatPlanDev& p, float* resid, int d, int io_dtype, hipStream_t st) {
  gather_kernel<<<p.T, 256, 0, st>>>(p, resid, d, io_dtype);
  return hipGetLastError();
}
hipError_t hat_launch_scatter(const HatPlanDev& p, const float* resid, const float* part, int nparts, int d,
                              int io_dtype, hipStream_t st) {
  scatter_kernel<<<p.T, 256, 0, st>>>(p, resid, part, nparts, d, io_dtype);
  return hipGetLastError();
}
hipError_t hat_launch_rope_table(const HatPlanDev& p, const double* inv_freq, float2* table, int half,
                                 hipStream_t st) {
  rope_table_kernel<<<blocks_for((size_t)p.T * half, 256), 256, 0, st>>>(p, inv_freq, table, half);
  return hipGetLastError();
}
hipError_t hat_launch_rmsnorm(float* resid, const float* part, int nparts, const float* gain, act_t* outP, int T,
                              int d, float eps, hipStream_t st) {
  if (d > 8192 || (d & 7)) return hipErrorInvalidValue;
  // from about a thousand rows on there are enough groups of rows to fill the chip (at 150-768 rows the
  // one-row kernel measured 10-14 us against 15-20 us)
  const bool groups = T >= 1024 && d % 64 == 0;   // (d / 8 a multiple of 8: the chunk swizzle stays inside the row)
  if (groups && d <= 4096) rmsnorm_rows_kernel<4, 4096><<<(T + 3) / 4, 256, 0, st>>>(resid, part, nparts, T, gain, outP, d, eps);
  else if (groups) rmsnorm_rows_kernel<4, 8192><<<(T + 3) / 4, 256, 0, st>>>(resid, part, nparts, T, gain, outP, d, eps);
  else rmsnorm_kernel<<<T, 256, 0, st>>>(resid, part, nparts, T, gain, outP, d, eps);
  return hipGetLastError();
}
hipError_t hat_launch_rope_append(const HatPlanDev& p, act_t* qkv, const float2* table, kv_t* pool_layer,
                                  int n_pages, int H, int hd, int kv_f16, hipStream_t st) {
  const int n_kblocks = (int)(((size_t)p.T * H * (hd >> 4) + 255) / 256);
  const int tiles = p.n_append * H;
  if (hd == 128) {
    const dim3 grid(n_kblocks + tiles);
    if (kv_f16) rope_append_kernel<true, 128><<<grid, 256, 0, st>>>(p, qkv, table, pool_layer, n_pages, H, n_kblocks);
    else rope_append_kernel<false, 128><<<grid, 256, 0, st>>>(p, qkv, table, pool_layer, n_pages, H, n_kblocks);
  } else if (hd == 64) {
    const dim3 grid(n_kblocks + (tiles + 1) / 2);
    if (kv_f16) rope_append_kernel<true, 64><<<grid, 256, 0, st>>>(p, qkv, table, pool_layer, n_pages, H, n_kblocks);
    else rope_append_kernel<false, 64><<<grid, 256, 0, st>>>(p, qkv, table, pool_layer, n_pages, H, n_kblocks);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
hipError_t hat_launch_retile(act_t* dst, int Nw, int Kd, const bf16_t* src0, const bf16_t* src1, const bf16_t* src2,
                             int n0, int Ks, int mode, hipStream_t st) {
  const size_t n = (size_t)Nw * (Kd >> 3);
  retile_kernel<<<blocks_for(n, 256), 256, 0, st>>>(dst, Nw, Kd, src0, src1, src2, n0, Ks, mode);
  return hipGetLastError();
}
hipError_t hat_launch_bf16_to_f32(const bf16_t* src, float* dst, int n, hipStream_t st) {
  bf16_to_f32_kernel<<<blocks_for(n, 256), 256, 0, st>>>(src, dst, n);
  return hipGetLastError();
}
hipError_t hat_launch_kv_import(kv_t* pool_layer, int n_pages, const int32_t* pages, int pos0, int n,
                                const bf16_t* k, const bf16_t* v, int H, int hd, int kv_f16, hipStream_t st) {
  const size_t cnt = (size_t)n * H * (hd >> 3);
  if (kv_f16) kv_import_kernel<true><<<blocks_for(cnt, 256), 256, 0, st>>>(pool_layer, n_pages, pages, pos0, n, k, v, H, hd);
  else kv_import_kernel<false><<<blocks_for(cnt, 256), 256, 0, st>>>(pool_layer, n_pages, pages, pos0, n, k, v, H, hd);
  return hipGetLastError();
}
hipError_t hat_launch_kv_export(const kv_t* pool_layer, int n_pages, const int32_t* pages, int pos0, int n,
                                bf16_t* k, bf16_t* v, int H, int hd, int kv_f16, hipStream_t st) {
  const size_t cnt = (size_t)n * H * (hd >> 3);
  if (kv_f16) kv_export_kernel<true><<<blocks_for(cnt, 256), 256, 0, st>>>(pool_layer, n_pages, pages, pos0, n, k, v, H, hd);
  else kv_export_kernel<false><<<blocks_for(cnt, 256), 256, 0, st>>>(pool_layer, n_pages, pages, pos0, n, k, v, H, hd);
  return hipGetLastError();
}
hipError_t hat_launch_kv_move(kv_t* pool, size_t layer_elems, int L, int n_pages, const HatRowMoves& mv, int H,
                              int hd, hipStream_t st) {
  if (mv.n <= 0) return hipSuccess;
  const size_t cnt = (size_t)L * H * (hd >> 3);
  kv_move_kernel<<<blocks_for(cnt, 256), 256, 0, st>>>(pool, layer_elems, L, n_pages, mv, H, hd);
  return hipGetLastError();
}
hipError_t hat_launch_unpack_p32(const act_t* srcP, int row_len, int col0, int ncols, int T, float* dst,
                                 hipStream_t st) {
  unpack_p32_kernel<<<blocks_for((size_t)T * ncols, 256), 256, 0, st>>>(srcP, row_len, col0, ncols, T, dst);
  return hipGetLastError();
}
