// fp16 MFMA GEMM for the projection and feed-forward matrices of a decoder layer
// (paper Sec. 2.1: self-attention module + feed-forward network; these four
// products are the bulk of a chunk step's arithmetic).
//
//   out[t, f] = sum_k X[t, k] * W[f, k]      X: activations, W: weights [out, in]
//
// Both operands are in the P32 layout (hat_layout.h).  The kernel computes the
// transposed product C^T = W * X^T with v_mfma_f32_32x32x16_f16: MFMA rows are
// output features, MFMA columns are tokens.  In the accumulator a lane then owns
// one token and runs of 4 consecutive features, which is exactly an 8-byte piece
// of the P32 layout of the *next* operand, so every epilogue stores coalesced.
//
// Data movement: global -> LDS with direct-to-LDS loads (global_load_lds_dwordx4),
// no register staging, into a ring of NSTAGE k-tiles.  Measured on MI355X: a CU
// sustains about 36-42 B/clk through these loads, each one holds the issuing wave
// for on the order of a hundred cycles, and the ring depth beyond two tiles does not
// matter -- so the refill is spread thinly between the MFMAs instead of issued in
// bursts, and the tile shape (bytes moved per flop) decides the rest.  Because the
// P32 panel slab of a k-tile is contiguous in memory and is kept contiguous in
// LDS, each wave instruction moves one 1 KB run, and an MFMA operand is one
// ds_read_b128 at lane*16 + immediate, conflict-free without a swizzle.
// LDS reads are issued from inline asm so that the compiler does not serialise
// them behind the outstanding direct-to-LDS loads; the waits are explicit:
// vmcnt for "my loads of this k-tile have landed", a barrier for "everyone's
// have", lgkmcnt for the operand reads.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "hat_device_util.h"
#include "hat_kernels.h"
#include "hat_layout.h"

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }
// fp32 -> fp16, round to nearest even, saturating instead of overflowing to infinity
__device__ __forceinline__ _Float16 to_act(float x) { return (_Float16)__builtin_amdgcn_fmed3f(x, -65504.f, 65504.f); }

template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { hat_static_for<N>(f); }
template <int OFF>
__device__ __forceinline__ f16x8 lds_read(uint32_t addr) { return hat_lds_read<OFF>(addr); }
template <int N>
__device__ __forceinline__ void wait_vmcnt() { hat_wait_vmcnt<N>(); }
template <int N>
__device__ __forceinline__ void wait_operands(f16x8 (&v)[N]) { hat_wait_operands(v); }

template <int BF, int BT, int WF, int WT, int BKT, int NSTAGE>
struct Tile {
  static constexpr int NW = WF * WT;
  static constexpr int MI = BF / WF / 32;   // feature blocks per wave
  static constexpr int NJ = BT / WT / 32;   // token blocks per wave
  static constexpr int PF = BF / 32, PT = BT / 32;
  static constexpr int SLAB = (BKT / 8) * 512;  // bytes of one panel's k-slab
  static constexpr int CPS = SLAB / 1024;       // 1 KB wave-chunks per slab
  static constexpr int NCH = (PF + PT) * CPS;
  static constexpr int LPW = NCH / NW;          // direct-to-LDS loads per wave per stage
  static constexpr int STAGE = (PF + PT) * SLAB;
  static constexpr int KS = BKT / 16;
  static constexpr int LDS_BYTES = NSTAGE * STAGE;
  static_assert(NCH % NW == 0, "chunks must divide over waves");
  static_assert((NSTAGE - 2) * LPW <= 63, "vmcnt is 6 bits");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per workgroup");
};

template <int BF, int BT, int WF, int WT, int BKT, int NSTAGE, int EPI>
__global__ __launch_bounds__(WF* WT * 64) void gemm_kernel(HatGemm g, int ksplit) {
  using TL = Tile<BF, BT, WF, WT, BKT, NSTAGE>;
  constexpr int MI = TL::MI, NJ = TL::NJ, PF = TL::PF, PT = TL::PT, SLAB = TL::SLAB, CPS = TL::CPS;
  constexpr int LPW = TL::LPW, STAGE = TL::STAGE, KS = TL::KS;

  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wf = wave / WT, wt = wave % WT;

  // workgroup -> tile.  Consecutive hardware ids go round-robin over the 8 XCDs;
  // give each XCD a contiguous run of tiles so that tiles sharing a weight panel
  // meet in one L2.
  const int nT = (g.T + BT - 1) / BT;
  const int nF = (g.Nw + BF - 1) / BF;
  const int nblk = nT * nF;
  int b = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8;
    const int x = b % 8, i = b / 8;
    b = x * per + (x < rem ? x : rem) + i;
  }
  // within an XCD's run, walk groups of 4 feature tiles across the token tiles: the ~32
  // workgroups resident on an XCD then form a 4 x 8 patch of tiles (12 distinct operand
  // slabs per k-tile instead of 16+) and more of their loads hit in L2
  int ft, tt;
  {
    constexpr int GF = 4;
    const int grp = b / (GF * nT);
    const int f0 = grp * GF;
    const int gf = (nF - f0) < GF ? (nF - f0) : GF;
    const int r = b - grp * GF * nT;
    ft = f0 + r % gf;
    tt = r / gf;
  }
  const int Tpanels = (g.T + 31) >> 5;

  const int KT = g.K / BKT;
  const int kt0 = (int)((long)blockIdx.z * KT / ksplit);
  const int kt1 = (int)((long)(blockIdx.z + 1) * KT / ksplit);
  const int nkt = kt1 - kt0;

  // per-wave chunk sources (per-lane address); destinations are wave-uniform
  const act_t* src[LPW];
  const size_t krow = (size_t)(g.K >> 3) * 256;  // elements per panel
#pragma unroll
  for (int c = 0; c < LPW; ++c) {
    const int ch = wave * LPW + c;
    const int q = ch / CPS, sub = ch % CPS;
    const act_t* base;
    if (q < PF) {
      int pnl = ft * PF + q;
      pnl = pnl < (g.Nw >> 5) ? pnl : (g.Nw >> 5) - 1;  // ragged last feature tile: same
      base = g.W + (size_t)pnl * krow;
    } else {
      int pnl = tt * PT + (q - PF);
      pnl = pnl < Tpanels ? pnl : Tpanels - 1;  // ragged last tile: re-read a real panel
      base = g.X + (size_t)pnl * krow;
    }
    src[c] = base + (size_t)kt0 * (BKT / 8) * 256 + sub * 512 + lane * 8;
  }
  auto issue = [&](int i) {  // i: k-tile index relative to kt0
    unsigned char* dstb = lds + (i % NSTAGE) * STAGE + wave * (LPW * 1024);
#pragma unroll
    for (int c = 0; c < LPW; ++c)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src[c] + (size_t)i * (BKT / 8) * 256),
          (__attribute__((address_space(3))) void*)(dstb + c * 1024), 16, 0, 0);
  };

  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // One continuous pipeline over k-steps.  The operands of k-step s+1 are read from LDS
  // while the MFMAs of k-step s run, also across k-tile boundaries: at the last k-step of
  // tile i a wave first makes sure tile i+1 has landed (its own loads: vmcnt; everyone's:
  // barrier -- which also says everyone is done reading tile i), reads tile i+1's first
  // operands, and only then issues tile i's last MFMAs.  The direct-to-LDS loads of tile
  // i+NSTAGE (into the buffer tile i just vacated) are slotted between the MFMAs of the
  // following KS k-steps.
  static_assert(KS % 2 == 0, "operand register sets alternate per k-step");
  static_assert((NSTAGE - 1) * LPW <= 63, "vmcnt is 6 bits");
  auto issue_chunk = [&](int i, int c) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(src[c] + (size_t)i * (BKT / 8) * 256),
        (__attribute__((address_space(3))) void*)(lds + (i % NSTAGE) * STAGE + wave * (LPW * 1024) + c * 1024), 16, 0, 0);
  };
  auto wait_pending = [&](int tiles) {  // at most `tiles` k-tiles of my loads still in flight
    switch (tiles) {
      case 0: wait_vmcnt<0>(); break;
      case 1: wait_vmcnt<(NSTAGE >= 2 ? 1 : 0) * LPW>(); break;
      case 2: wait_vmcnt<(NSTAGE >= 3 ? 2 : 0) * LPW>(); break;
      default: wait_vmcnt<(NSTAGE >= 4 ? 3 : 0) * LPW>(); break;
    }
  };
  static_assert(NSTAGE <= 4, "wait_pending covers up to 3 pending tiles");
#pragma unroll
  for (int s = 0; s < NSTAGE; ++s)
    if (s < nkt) issue(s);

  const uint32_t offW = (wf * MI) * SLAB + lane * 16;
  const uint32_t offX = (PF + wt * NJ) * SLAB + lane * 16;
  f16x8 a[2][MI], bb[2][NJ];
  constexpr int NMFMA = MI * NJ;
  constexpr int CPP = (LPW + KS - 1) / KS;  // loads of one refill part (one k-step's share of a tile)

  if (nkt > 0) {
    wait_pending(nkt - 1 < NSTAGE - 1 ? nkt - 1 : NSTAGE - 1);
    __builtin_amdgcn_s_barrier();
    const uint32_t aW = lds_base + offW, aX = lds_base + offX;
    static_for<MI>([&](auto ii) { a[0][ii] = lds_read<ii * SLAB>(aW); });
    static_for<NJ>([&](auto jj) { bb[0][jj] = lds_read<jj * SLAB>(aX); });
  }
  for (int i = 0; i < nkt; ++i) {
    const uint32_t sbase = lds_base + (i % NSTAGE) * STAGE;
    const uint32_t aW = sbase + offW, aX = sbase + offX;
    static_for<KS>([&](auto ks) {
      constexpr int cur = ks & 1;
      wait_operands(a[cur]);
      wait_operands(bb[cur]);
      if constexpr (ks + 1 < KS) {
        static_for<MI>([&](auto ii) { a[cur ^ 1][ii] = lds_read<ii * SLAB + (ks + 1) * 1024>(aW); });
        static_for<NJ>([&](auto jj) { bb[cur ^ 1][jj] = lds_read<jj * SLAB + (ks + 1) * 1024>(aX); });
      } else if (i + 1 < nkt) {
        const int after = nkt - 2 - i;  // tiles issued behind tile i+1
        wait_pending(after < NSTAGE - 2 ? after : NSTAGE - 2);
        __builtin_amdgcn_s_barrier();
        const uint32_t nbase = lds_base + ((i + 1) % NSTAGE) * STAGE;
        const uint32_t nW = nbase + offW, nX = nbase + offX;
        static_for<MI>([&](auto ii) { a[cur ^ 1][ii] = lds_read<ii * SLAB>(nW); });
        static_for<NJ>([&](auto jj) { bb[cur ^ 1][jj] = lds_read<jj * SLAB>(nX); });
      }
      // The refill of the ring is spread thinly over the MFMAs: a direct-to-LDS load holds
      // the issuing wave for on the order of a hundred cycles, so a burst of them would
      // stall the matrix pipe.  The tile going into the buffer vacated at the last
      // boundary is issued in KS parts: part 0 right after that boundary (last k-step of
      // the previous tile), parts 1.. over this tile's k-steps 0..KS-2.
      constexpr int part = (ks + 1) % KS;
      const int rtile = (ks + 1 == KS) ? i + NSTAGE : i - 1 + NSTAGE;
      const bool refill = rtile < nkt && ((ks + 1 == KS) ? (i + 1 < nkt) : (i >= 1));
      // keep the operand reads ahead of this k-step's MFMAs (the scheduler would otherwise
      // sink them behind the MFMAs and expose the LDS latency)
      __builtin_amdgcn_sched_barrier(0);
      static_for<NMFMA>([&](auto n) {
        constexpr int ii = n / NJ, jj = n % NJ;
        acc[ii][jj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[cur][ii], bb[cur][jj], acc[ii][jj], 0, 0, 0);
        static_for<CPP>([&](auto q) {
          constexpr int slot = (q * NMFMA / CPP) < NMFMA ? (q * NMFMA / CPP) : NMFMA - 1;
          constexpr int c = part * CPP + q;
          if constexpr (slot == n && c < LPW) {
            if (refill) issue_chunk(rtile, c);
          }
        });
      });
      __builtin_amdgcn_sched_barrier(0);
    });
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
          f16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = to_act(acc[i][j][4 * q + e]);
          *(f16x4*)(g.outP + p32_index(tok, f, g.Nout)) = v;
        }
      }
    } else if constexpr (EPI == HAT_EPI_SWIGLU) {
      // a 32-row block of W holds 16 gate rows then the 16 up rows of the same features:
      // accumulator elements 4q+e (q = 0,1) and 4(q+2)+e of a lane are gate and up of
      // output feature fb + 8q + 4h + e
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int fb = (f_base + i * 32) / 2;  // output feature block (16 wide)
        if (fb >= g.Nout) continue;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int f = fb + 8 * q + 4 * h;
          f16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = to_act(silu_f(acc[i][j][4 * q + e]) * acc[i][j][4 * (q + 2) + e]);
          *(f16x4*)(g.outP + p32_index(tok, f, g.Nout)) = v;
        }
      }
    } else {
      // fp32 result: added into the residual when K is not split, else stored as this
      // split's partial sum (the next consumer of the residual folds the partials in)
      float* outb = (ksplit == 1) ? g.resid : g.part + (size_t)blockIdx.z * g.T * g.Nout;
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int fb = f_base + i * 32;
        if (fb >= g.Nout) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = fb + 8 * q + 4 * h;
          float* p = outb + (size_t)tok * g.Nout + f;
          f32x4 v;
          if (ksplit == 1) {
            v = *(f32x4*)p;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += acc[i][j][4 * q + e];
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
          }
          *(f32x4*)p = v;
        }
      }
    }
  }
}

// tile table: id, features x tokens, waves along features x tokens, k per stage, stages.
// Heights of 96 and 192 rows exist so that the tile count can match the 256 CUs where
// 128 / 256 leave a quarter or a third of them idle (7B-shaped QKV and gate/up at T <= 256).
// Tile 19 is tile 1 on eight waves (two per SIMD, 64 x 128 each): measured 2-8 % faster
// at T = 512 .. 4096 wherever the 256 x 256 shape is the right one.  Tiles 20-22 take 224, 192
// and 160 token rows: for batches whose row count leaves the last 256-row tile mostly empty
// or the tile count just above a multiple of the 256 CUs (measured up to 25 % at T = 2200).  Tile 23
// (128 x 160) is for batches of 129 .. 160 rows, e.g. 30 devices x 5 draft rows: one token tile
// instead of a full and a nearly empty one (O, gate/up and down 3-13 % faster at 150 rows on the
// 7B shape, 12-20 % on the 13B shape).
#define HAT_FOR_TILES(X, EPI)       \
  X(0, 256, 256, 2, 2, 64, 2, EPI)  \
  X(1, 256, 256, 2, 2, 32, 4, EPI)  \
  X(2, 128, 256, 2, 2, 64, 3, EPI)  \
  X(3, 256, 128, 2, 2, 64, 3, EPI)  \
  X(4, 128, 128, 2, 2, 64, 4, EPI)  \
  X(5, 256, 64, 4, 1, 64, 3, EPI)   \
  X(6, 256, 32, 4, 1, 64, 4, EPI)   \
  X(7, 128, 64, 2, 2, 64, 4, EPI)   \
  X(8, 128, 32, 2, 1, 64, 4, EPI)   \
  X(9, 64, 256, 1, 4, 64, 3, EPI)   \
  X(10, 128, 128, 2, 2, 64, 2, EPI) \
  X(11, 128, 128, 2, 2, 32, 4, EPI) \
  X(12, 128, 64, 2, 2, 64, 3, EPI)  \
  X(13, 192, 128, 2, 2, 64, 3, EPI) \
  X(14, 96, 128, 1, 4, 64, 4, EPI)  \
  X(15, 96, 256, 1, 4, 64, 3, EPI)  \
  X(16, 192, 64, 2, 2, 64, 4, EPI)  \
  X(17, 192, 256, 2, 2, 64, 2, EPI) \
  X(18, 96, 64, 1, 2, 64, 4, EPI)   \
  X(19, 256, 256, 4, 2, 32, 4, EPI) \
  X(20, 256, 224, 4, 1, 64, 2, EPI) \
  X(21, 256, 192, 2, 2, 32, 4, EPI) \
  X(22, 256, 160, 4, 1, 64, 3, EPI) \
  X(23, 128, 160, 4, 1, 64, 3, EPI)
constexpr int kNumTiles = 24;

struct TileInfo { int bf, bt, waves, bkt, nstage; bool planned; float eff; };
// `planned`: offered to the automatic choice; the others are alternative stagings of the
// same shapes, used only when forced
constexpr bool kPlanned[kNumTiles] = {false, true, true, true, true, true, true, true, true, true,
                                      false, false, false, true, true, true, true, true, true, true,
                                      true, true, true, true};
// Share of the matrix peak that a tile's k-loop reaches when it is not load-bound, fitted to
// sweeps at T = 512 .. 5220 (7B shapes, all four products, K split 1 .. 8); 0 = not measured
// there, the tile is only offered to batches of at most kSmallT rows.
constexpr float kEff[kNumTiles] = {0.f, 0.585f, 0.538f, 0.533f, 0.916f, 0.f, 0.f, 0.f, 0.f, 0.f,
                                   0.f, 0.f, 0.f, 0.514f, 0.f, 1.209f, 0.f, 0.504f, 0.f, 0.629f,
                                   0.518f, 0.565f, 0.564f, 0.f};
constexpr int kSmallT = 384;
constexpr TileInfo kTiles[kNumTiles] = {
#define HAT_INFO(id, bf, bt, wf, wt, bkt, ns, epi) {bf, bt, (wf) * (wt), bkt, ns, kPlanned[id], kEff[id]},
    HAT_FOR_TILES(HAT_INFO, 0)
#undef HAT_INFO
};

template <int EPI>
hipError_t launch_epi(const HatGemm& g, const HatGemmPlan& p, hipStream_t st) {
#define HAT_TRY(id, bf, bt, wf, wt, bkt, ns, epi)                       \
  if (p.tile == id) {                                                   \
    using TL = Tile<bf, bt, wf, wt, bkt, ns>;                           \
    dim3 grid(((g.T + bt - 1) / bt) * ((g.Nw + bf - 1) / bf), 1, p.ksplit); \
    auto kern = gemm_kernel<bf, bt, wf, wt, bkt, ns, epi>;              \
    kern<<<grid, dim3(wf * wt * 64), TL::LDS_BYTES, st>>>(g, p.ksplit); \
    return hipGetLastError();                                           \
  }
  HAT_FOR_TILES(HAT_TRY, EPI)
#undef HAT_TRY
  return hipErrorInvalidValue;
}

template <int EPI>
hipError_t attr_epi() {
  hipError_t e;
#define HAT_ATTR(id, bf, bt, wf, wt, bkt, ns, epi)                                                        \
  e = hipFuncSetAttribute((const void*)gemm_kernel<bf, bt, wf, wt, bkt, ns, epi>,                         \
                          hipFuncAttributeMaxDynamicSharedMemorySize, Tile<bf, bt, wf, wt, bkt, ns>::LDS_BYTES); \
  if (e != hipSuccess) return e;
  HAT_FOR_TILES(HAT_ATTR, EPI)
#undef HAT_ATTR
  return hipSuccess;
}

}  // namespace

int hat_gemm_tile_count() { return kNumTiles; }
bool hat_gemm_tile_info(int id, int* bf, int* bt, int* waves, int* bkt, int* nstage) {
  if (id < 0 || id >= kNumTiles) return false;
  const TileInfo& q = kTiles[id];
  if (bf) *bf = q.bf;
  if (bt) *bt = q.bt;
  if (waves) *waves = q.waves;
  if (bkt) *bkt = q.bkt;
  if (nstage) *nstage = q.nstage;
  return true;
}

hipError_t hat_gemm_init() {
  hipError_t e;
  if ((e = attr_epi<HAT_EPI_P32>()) != hipSuccess) return e;
  if ((e = attr_epi<HAT_EPI_SWIGLU>()) != hipSuccess) return e;
  if ((e = attr_epi<HAT_EPI_RESID>()) != hipSuccess) return e;
  return hipSuccess;
}

HatGemmPlan hat_gemm_plan(const HatGemm& g) {
  // Estimated time of a candidate = rounds of 256 workgroups x the larger of the
  // MFMA time and the L2->LDS streaming time of one workgroup; split-K (only where
  // the result is accumulated in fp32) adds the traffic of its partial sums.
  HatGemmPlan best{0, 1};
  if (g.force_tile >= 0 && g.force_tile < kNumTiles) {
    best.tile = g.force_tile;
    best.ksplit = g.force_ksplit > 0 ? g.force_ksplit : 1;
    if (g.epilogue != HAT_EPI_RESID || !g.part) best.ksplit = 1;
    while (best.ksplit > 1 && ((long)best.ksplit * g.T > g.part_rows || g.K / 64 / best.ksplit < 1)) --best.ksplit;
    return best;
  }
  // Two regimes, each with constants fitted to tile sweeps on MI355X (7B shapes).
  // Up to kSmallT rows (T = 32 .. 384) the weight stream decides: a CU moves about 36 B/clk
  // through direct-to-LDS loads, the MFMA loop runs at about 85 % of the matrix peak on its own,
  // and the two overlap only partly (issuing the loads holds the waves that also issue the
  // MFMAs); the weight stream cannot beat ~5.5 TB/s, nor (Little's law) the bytes of W that
  // the resident workgroups' rings keep in flight divided by the ~1.2 us a load from HBM takes
  // under load -- which is what decides between shapes when there are few token rows.
  // Above that (T = 512 .. 5220) a k-tile costs the larger of its MFMA time at the tile's own
  // measured efficiency and its load time at 28 B/clk, a round of workgroups costs ~3.7 us of
  // prologue and drain, and the epilogue's traffic is not hidden: 14 B/clk per CU for the
  // fp16 stores, 6.2 for the read-modify-write of the fp32 residual, 7.2 for split-K partial
  // sums (written here, read back by the consumer of the residual).
  double best_cost = 1e300;
  const int KT = g.K / 64;
  const bool large = g.T > kSmallT;
  for (int c = 0; c < kNumTiles; ++c) {
    const TileInfo& q = kTiles[c];
    if (!q.planned) continue;
    // 160/192/224-row token tiles: large batches only, except the 128 x 160 tile (23), which exists for batches
    // of 129 .. 160 rows (a second, mostly empty 128-row token tile costs them 15-20 %)
    if (large ? q.eff == 0.f : ((q.bt & (q.bt - 1)) != 0 && !(c == 23 && g.T > 128 && g.T <= 160))) continue;
    const int nT = (g.T + q.bt - 1) / q.bt, nF = (g.Nw + q.bf - 1) / q.bf;
    const int max_split = (g.epilogue == HAT_EPI_RESID && g.part) ? 16 : 1;
    const int lds = q.nstage * (q.bf + q.bt) * q.bkt * 2;
    const int per_cu = std::max(1, std::min(160 * 1024 / lds, 8 / q.waves));
    for (int ks = 1; ks <= max_split; ++ks) {
      if (ks > 1 && (KT / ks < 4 || (long)ks * g.T > g.part_rows)) break;
      const double blocks = (double)nT * nF * ks;
      const double rounds = std::ceil(blocks / 256.0);
      const double kt = std::ceil((double)KT / ks) + 2.0;                     // + pipeline fill
      double cyc;
      if (large) {
        const double mfma_cyc = 2.0 * q.bf * q.bt * 64 / (4 * 1017.0 * q.eff);  // per k-tile, 4 SIMDs
        const double load_cyc = (q.bf + q.bt) * 64 * 2 / 28.1;
        const double tile_cyc = std::max(mfma_cyc, load_cyc) + 0.073 * std::min(mfma_cyc, load_cyc);
        cyc = rounds * kt * tile_cyc + rounds * 8938.0;
        const double rows = (double)g.T * g.Nout / 256.0;                     // output elements per CU
        if (g.epilogue != HAT_EPI_RESID) cyc += rows * 2.0 / 14.0;
        else if (ks == 1) cyc += rows * 8.0 / 6.2;
        else cyc += rows * 8.0 * ks / 7.15;
      } else {
        const double mfma_eff = q.waves == 8 ? 0.90 : 0.85;                     // two waves per SIMD fill more of the pipe
        const double mfma_cyc = 2.0 * q.bf * q.bt * 64 / (4 * 1017.0 * mfma_eff);
        const double load_cyc = (q.bf + q.bt) * 64 * 2 / 36.0;
        const double tile_cyc = std::max(mfma_cyc, load_cyc) + 0.45 * std::min(mfma_cyc, load_cyc);
        cyc = rounds * kt * tile_cyc + rounds * 3000.0;
        if (ks > 1) cyc += (double)ks * g.T * g.Nout * 8.0 / 256.0 / 12.0;    // partial write + read, per CU
      }
      const double resident = std::min(blocks, 256.0 * per_cu);
      const double inflight = resident * q.bf * q.bkt * 2.0 * (q.nstage - 1);
      const double bw = std::min(5.5e12, inflight / 1.2e-6);
      const double hbm_cyc = 2.0 * g.Nw * g.K / bw * 2.4e9 + 7000.0;
      const double cost = std::max(cyc, hbm_cyc) + 1e-3 * cyc;                // tie-break below the HBM floor
      if (cost < best_cost) { best_cost = cost; best.tile = c; best.ksplit = ks; }
    }
  }
  return best;
}

hipError_t hat_launch_gemm(const HatGemm& g, const HatGemmPlan& p, hipStream_t st) {
  if (g.T <= 0) return hipSuccess;
  if (g.K % 64 != 0 || g.Nw % 256 != 0) return hipErrorInvalidValue;
  if (p.ksplit > 1 && (g.epilogue != HAT_EPI_RESID || !g.part)) return hipErrorInvalidValue;
  switch (g.epilogue) {
    case HAT_EPI_P32: return launch_epi<HAT_EPI_P32>(g, p, st);
    case HAT_EPI_SWIGLU: return launch_epi<HAT_EPI_SWIGLU>(g, p, st);
    case HAT_EPI_RESID: return launch_epi<HAT_EPI_RESID>(g, p, st);
  }
  return hipErrorInvalidValue;
}
