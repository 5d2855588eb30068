// bf16 MFMA GEMM for the projection and feed-forward matrices of a decoder layer
// (paper Sec. 2.1: self-attention module + feed-forward network; these four
// products are the bulk of a chunk step's arithmetic).
//
//   out[t, f] = sum_k X[t, k] * W[f, k]      X: activations, W: weights [out, in]
//
// Both operands are in the P32 layout (hat_layout.h).  The kernel computes the
// transposed product C^T = W * X^T with v_mfma_f32_32x32x16_bf16: MFMA rows are
// output features, MFMA columns are tokens.  In the accumulator a lane then owns
// one token and runs of 4 consecutive features, which is exactly an 8-byte piece
// of the P32 layout of the *next* operand, so every epilogue stores coalesced.
//
// Tile: BF features x BT tokens per workgroup, BK = 64 per stage, waves arranged
// WF x WT.  Global -> LDS goes through registers with the next stage's loads in
// flight during the MFMAs of the current one (two LDS stages, one barrier per
// stage).  LDS holds each 32-row panel's k-slab contiguously, so an MFMA operand
// is one ds_read_b128 at lane*16 + immediate.
#include <hip/hip_runtime.h>

#include "hat_kernels.h"
#include "hat_layout.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BK = 64;
constexpr int SLAB = (BK / 8) * 512;  // bytes of one panel's k-slab (32 rows x BK)
constexpr int CPS = SLAB / 1024;      // 1 KB wave-chunks per slab

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

template <int BF, int BT, int WF, int WT, int EPI>
__global__ __launch_bounds__(WF* WT * 64) void gemm_kernel(HatGemm g, int ksplit) {
  constexpr int NW = WF * WT;
  constexpr int MI = BF / WF / 32;  // feature blocks per wave
  constexpr int NJ = BT / WT / 32;  // token blocks per wave
  constexpr int PF = BF / 32, PT = BT / 32;
  constexpr int NCH = (PF + PT) * CPS;  // 1 KB chunks per stage
  static_assert(NCH % NW == 0, "chunks must divide over waves");
  constexpr int LPW = NCH / NW;  // chunk loads per wave per stage
  constexpr int STAGE = (PF + PT) * SLAB;

  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wf = wave / WT, wt = wave % WT;

  // workgroup -> tile.  Consecutive hardware ids go round-robin over the 8 XCDs;
  // give each XCD a contiguous run of tiles so that tiles sharing a weight panel
  // meet in one L2.
  const int nT = (g.T + BT - 1) / BT;
  const int nF = g.Nw / BF;
  const int nblk = nT * nF;
  int b = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8;
    const int x = b % 8, i = b / 8;
    // XCD x owns [x*per + min(x,rem), ...) of the logical order
    b = x * per + (x < rem ? x : rem) + i;
  }
  const int ft = b / nT, tt = b % nT;
  const int Tpanels = (g.T + 31) >> 5;

  const int KT = g.K / BK;
  const int kt0 = (int)((long)blockIdx.z * KT / ksplit);
  const int kt1 = (int)((long)(blockIdx.z + 1) * KT / ksplit);

  // per-wave chunk sources
  const bf16_t* src[LPW];
  int dst_off[LPW];
  const size_t krow = (size_t)(g.K >> 3) * 256;  // elements per panel
#pragma unroll
  for (int c = 0; c < LPW; ++c) {
    const int ch = wave * LPW + c;
    const int q = ch / CPS, sub = ch % CPS;
    const bf16_t* base;
    if (q < PF) {
      base = g.W + (size_t)(ft * PF + q) * krow;
    } else {
      int pnl = tt * PT + (q - PF);
      pnl = pnl < Tpanels ? pnl : Tpanels - 1;
      base = g.X + (size_t)pnl * krow;
    }
    src[c] = base + sub * 512 + lane * 8;
    dst_off[c] = ch * 1024 + lane * 16;
  }

  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 stage_regs[LPW];
  auto gload = [&](int kt) {
#pragma unroll
    for (int c = 0; c < LPW; ++c) stage_regs[c] = *(const u32x4*)(src[c] + (size_t)kt * (BK / 8) * 256);
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int c = 0; c < LPW; ++c) *(u32x4*)(lds + buf * STAGE + dst_off[c]) = stage_regs[c];
  };

  if (kt0 < kt1) {
    gload(kt0);
    lstore(0);
  }
  __syncthreads();

  for (int kt = kt0; kt < kt1; ++kt) {
    const int buf = (kt - kt0) & 1;
    if (kt + 1 < kt1) gload(kt + 1);
    const unsigned char* sW = lds + buf * STAGE + (wf * MI) * SLAB + lane * 16;
    const unsigned char* sX = lds + buf * STAGE + (PF + wt * NJ) * SLAB + lane * 16;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[MI], bb[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) a[i] = *(const bf16x8*)(sW + i * SLAB + ks * 1024);
#pragma unroll
      for (int j = 0; j < NJ; ++j) bb[j] = *(const bf16x8*)(sX + j * SLAB + ks * 1024);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < kt1) lstore(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue.  lane: token = t0 + 32j + lane%32 ; feature = f0 + 32i + 8*(r/4) + 4*(lane/32) + r%4
  const int h = lane >> 5, n = lane & 31;
  const int t_base = tt * BT + wt * NJ * 32;
  const int f_base = ft * BF + wf * MI * 32;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int tok = t_base + j * 32 + n;
    if (tok >= g.T) continue;
    if constexpr (EPI == HAT_EPI_P32) {
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int fb = f_base + i * 32;
        if (fb >= g.Nout) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = fb + 8 * q + 4 * h;
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (__bf16)acc[i][j][4 * q + e];
          *(bf16x4*)(g.outP + p32_index(tok, f, g.Nout)) = v;
        }
      }
    } else if constexpr (EPI == HAT_EPI_SWIGLU) {
      static_assert(EPI != HAT_EPI_SWIGLU || MI % 2 == 0, "gate/up blocks come in pairs");
#pragma unroll
      for (int i = 0; i < MI; i += 2) {
        const int fb = (f_base + i * 32) / 2;  // output feature block
        if (fb >= g.Nout) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = fb + 8 * q + 4 * h;
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (__bf16)(silu_f(acc[i][j][4 * q + e]) * acc[i + 1][j][4 * q + e]);
          *(bf16x4*)(g.outP + p32_index(tok, f, g.Nout)) = v;
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int fb = f_base + i * 32;
        if (fb >= g.Nout) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = fb + 8 * q + 4 * h;
          float* p = g.resid + (size_t)tok * g.Nout + f;
          if (ksplit == 1) {
            f32x4 v = *(f32x4*)p;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += acc[i][j][4 * q + e];
            *(f32x4*)p = v;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) atomicAdd(p + e, acc[i][j][4 * q + e]);
          }
        }
      }
    }
  }
}

template <int BF, int BT, int WF, int WT>
constexpr int lds_bytes() {
  return 2 * (BF / 32 + BT / 32) * SLAB;
}

template <int BF, int BT, int WF, int WT, int EPI>
hipError_t launch_cfg(const HatGemm& g, int ksplit, hipStream_t st) {
  const int nT = (g.T + BT - 1) / BT, nF = g.Nw / BF;
  dim3 grid(nT * nF, 1, ksplit);
  constexpr int kLds = lds_bytes<BF, BT, WF, WT>();
  auto kern = gemm_kernel<BF, BT, WF, WT, EPI>;
  kern<<<grid, dim3(WF * WT * 64), kLds, st>>>(g, ksplit);
  return hipGetLastError();
}

template <int BF, int BT, int WF, int WT, int EPI>
hipError_t set_attr() {
  return hipFuncSetAttribute((const void*)gemm_kernel<BF, BT, WF, WT, EPI>,
                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes<BF, BT, WF, WT>());
}

// tile shapes: features x tokens, waves along features x waves along tokens
#define HAT_FOR_TILES(X, EPI) \
  X(256, 256, 2, 2, EPI)      \
  X(256, 128, 2, 2, EPI)      \
  X(256, 64, 4, 1, EPI)       \
  X(256, 32, 4, 1, EPI)       \
  X(128, 128, 2, 2, EPI)      \
  X(128, 64, 2, 2, EPI)       \
  X(128, 32, 2, 1, EPI)

template <int EPI>
hipError_t launch_epi(const HatGemm& g, hipStream_t st) {
  // Pick the tile (and, where the epilogue accumulates into the fp32 residual,
  // a K split) with the smallest estimated time: rounds of 256 workgroups times
  // the work of one workgroup, weighted by how much LDS traffic the wave tile
  // needs per MFMA.
  struct Cand { int bf, bt, wf, wt; };
  static const Cand cands[] = {{256, 256, 2, 2}, {256, 128, 2, 2}, {256, 64, 4, 1}, {256, 32, 4, 1},
                               {128, 128, 2, 2}, {128, 64, 2, 2},  {128, 32, 2, 1}};
  const int KT = g.K / BK;
  double best = 1e300;
  int bi = 0, bks = 1;
  for (int c = 0; c < 7; ++c) {
    const Cand& q = cands[c];
    const int nT = (g.T + q.bt - 1) / q.bt, nF = g.Nw / q.bf;
    const int max_split = (EPI == HAT_EPI_RESID) ? 16 : 1;
    for (int ks = 1; ks <= max_split; ks *= 2) {
      if (ks > 1 && KT / ks < 4) break;
      const double rounds = (double)((nT * nF * ks + 255) / 256);
      const double wtf = q.bf / q.wf, wtt = q.bt / q.wt;
      const double lds_pen = 1.0 + 24.0 * (1.0 / wtf + 1.0 / wtt);
      const double waves_pen = (q.wf * q.wt == 4) ? 1.0 : 1.6;  // fewer waves hide less latency
      const double cost = rounds * ((double)q.bf * q.bt * (KT / ks + 3)) * lds_pen * waves_pen + ks * 1e3;
      if (cost < best) { best = cost; bi = c; bks = ks; }
    }
  }
  const int BF = cands[bi].bf, BT = cands[bi].bt, ksplit = bks;
#define HAT_TRY(bf, bt, wf, wt, epi) \
  if (BF == bf && BT == bt) return launch_cfg<bf, bt, wf, wt, epi>(g, ksplit, st);
  HAT_FOR_TILES(HAT_TRY, EPI)
#undef HAT_TRY
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t hat_gemm_init() {
  hipError_t e;
#define HAT_ATTR(bf, bt, wf, wt, epi) \
  if ((e = set_attr<bf, bt, wf, wt, epi>()) != hipSuccess) return e;
  HAT_FOR_TILES(HAT_ATTR, HAT_EPI_P32)
  HAT_FOR_TILES(HAT_ATTR, HAT_EPI_SWIGLU)
  HAT_FOR_TILES(HAT_ATTR, HAT_EPI_RESID)
#undef HAT_ATTR
  return hipSuccess;
}

hipError_t hat_launch_gemm(const HatGemm& g, hipStream_t st) {
  if (g.T <= 0) return hipSuccess;
  if (g.K % BK != 0 || g.Nw % 256 != 0) return hipErrorInvalidValue;
  switch (g.epilogue) {
    case HAT_EPI_P32: return launch_epi<HAT_EPI_P32>(g, st);
    case HAT_EPI_SWIGLU: return launch_epi<HAT_EPI_SWIGLU>(g, st);
    case HAT_EPI_RESID: return launch_epi<HAT_EPI_RESID>(g, st);
  }
  return hipErrorInvalidValue;
}
