// Launch interface between the host side of the library and its HIP kernels.
// All pointers are device pointers unless stated otherwise; every function
// enqueues on `st` and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;    // storage type of the callers' weights, of hidden in/out and of imported / exported cache rows
typedef _Float16 act_t;   // arithmetic type of the MFMA operands: re-tiled weights and all activations
typedef uint16_t kv_t;    // one KV-cache element: bf16 or fp16 bits, as the handle's configuration says (kv_f16)

constexpr int HAT_MAX_VERIFY_ROWS = 8;  // query rows of a verify work item
// query rows of one chunk-attention workgroup: 8 waves x 32 rows (the 64-key K/V stage that a
// workgroup loads and widens is shared by all of them)
constexpr int HAT_CHUNK_QROWS = 256;

// ---- GEMM: out[t, f] = sum_k X[t, k] * W[f, k], operands in P32 layout ------
enum HatEpilogue {
  HAT_EPI_P32 = 0,     // fp16 (act_t) result, P32 layout, row length Nout
  HAT_EPI_SWIGLU = 1,  // W rows interleaved (16 gate, 16 up): silu(gate)*up, P32, row length Nout
  HAT_EPI_RESID = 2    // resid[t, f] += result  (fp32 row-major, leading dim Nout)
};

struct HatGemm {
  const act_t* W;   // P32 [Nw, K], Nw multiple of 256, padding rows zero
  const act_t* X;   // P32 [>= roundup(T,32), K]
  int K;            // multiple of 64
  int T;            // valid rows of X
  int Nw;           // rows of W including padding
  int Nout;         // logical output features (EPI_SWIGLU: Nw/2 >= Nout)
  act_t* outP;      // EPI_P32 / EPI_SWIGLU
  float* resid;     // EPI_RESID, K not split: resid[t, f] += result
  float* part;      // EPI_RESID, K split s ways: part[z][t][f] = partial sum of split z (may be null: no split)
  int part_rows;    // capacity of `part` in rows of Nout floats (bounds ksplit * T)
  int epilogue;
  int force_tile;   // >= 0: use this tile id (tuning); -1: choose
  int force_ksplit; // with force_tile: K split (0/1 = none)
};
struct HatGemmPlan {
  int tile;    // index into the tile table of gemm.hip
  int ksplit;  // 1 = K not split
};
HatGemmPlan hat_gemm_plan(const HatGemm& g);
hipError_t hat_launch_gemm(const HatGemm& g, const HatGemmPlan& p, hipStream_t st);
int hat_gemm_tile_count();
// shape of tile `id` (features, tokens, waves, k per stage, stages); false if out of range
bool hat_gemm_tile_info(int id, int* bf, int* bt, int* waves, int* bkt, int* nstage);
hipError_t hat_gemm_init();  // one-time function attributes (dynamic LDS size)

// ---- weight re-tiling (create time) -----------------------------------------
// dst: P32 [Nw, Kd] in act_t (bf16 -> fp16 is exact for |w| in [2^-17, 65504]).  mode 0: row R <- src0[R] (R < n0), else 0.
// mode 1 (qkv): rows [0,n0) <- src0, [n0,2n0) <- src1, [2n0,3n0) <- src2.
// mode 2 (gate/up): row R: blk=R/32, w=R%32; f = 16*blk + w%16; (w<16 ? src0 : src1)[f], zero if f >= n0
// (every 32-row block = 16 gate rows followed by the up rows of the same 16 features).
// Source rows have Ks elements (Ks <= Kd; columns beyond Ks are zero).
hipError_t hat_launch_retile(act_t* dst, int Nw, int Kd, const bf16_t* src0, const bf16_t* src1,
                             const bf16_t* src2, int n0, int Ks, int mode, hipStream_t st);
hipError_t hat_launch_bf16_to_f32(const bf16_t* src, float* dst, int n, hipStream_t st);

// ---- per-step plan as seen by the kernels -----------------------------------
// One KV page touched by this step's append: rows [lo, hi) of the page's 16 positions are new.
struct HatAppendItem {
  int32_t page;   // page id
  int32_t row0;   // batch row that holds position pos0 (may lie before the segment's first row)
  int32_t pos0;   // absolute position of the page's slot 0
  int32_t lo, hi; // new positions of this page: pos0 <= lo < hi <= pos0 + 16
  int32_t pad0, pad1, pad2;
};

struct HatPlanDev {
  int T, S;
  const int32_t* pos;       // [T] absolute position of each row
  const int32_t* kv_dst;    // [T] page*16 + slot where the row's K/V go
  const int32_t* tok_seg;   // [T] segment of each row
  const int32_t* tok_off;   // [S+1] first row of each segment
  const int32_t* seg_start; // [S]
  const int32_t* seg_pt;    // [S] offset of the segment's page list in page_tbl
  const int32_t* page_tbl;
  const uint64_t* in_ptr;   // [S] hidden_in
  const uint64_t* out_ptr;  // [S] hidden_out
  const HatAppendItem* append;  // pages written by this step
  int n_append;
};

hipError_t hat_launch_gather(const HatPlanDev& p, float* resid, int d, int io_dtype, hipStream_t st);
hipError_t hat_launch_scatter(const HatPlanDev& p, const float* resid, const float* part, int nparts, int d,
                              int io_dtype, hipStream_t st);
hipError_t hat_launch_rope_table(const HatPlanDev& p, const double* inv_freq, float2* table, int half, hipStream_t st);
// x = resid + sum of nparts partial sums (part[i][t][:], stride T*d); if nparts > 0 the sum is
// written back to resid.  out = rmsnorm(x) * gain as fp16 (act_t) in P32 layout.
hipError_t hat_launch_rmsnorm(float* resid, const float* part, int nparts, const float* gain, act_t* outP, int T,
                              int d, float eps, hipStream_t st);
// qkv: P32 [., 3d]; rotates q in place, writes rotated k and v into the pool of one layer
hipError_t hat_launch_rope_append(const HatPlanDev& p, act_t* qkv, const float2* table, kv_t* pool_layer,
                                  int n_pages, int H, int hd, int kv_f16, hipStream_t st);

// ---- attention ---------------------------------------------------------------
// One work item = 32*QB query rows of one segment against keys [kv_begin, kv_end).
struct HatAttnItem {
  int32_t seg;       // segment index
  int32_t q0;        // first query row, relative to the segment
  int32_t nq;        // valid query rows in this item
  int32_t kv_begin;  // multiple of 64
  int32_t kv_end;    // exclusive; keys beyond the causal limit are masked
  int32_t part_row;  // >= 0: first row of this item's partial result; -1: write the final output
  // copies of the segment's plan entries, so that a workgroup reaches its first page id
  // after one dependent load instead of three
  int32_t start;     // absolute position of the segment's first row
  int32_t tok0;      // batch row of the segment's first row
  int32_t kv_len;    // cache length after this step's append
  int32_t pt_off;    // offset of the segment's page list in page_tbl
  // verify items: byte i = visibility of the segment's new rows for query row i (bit j: the row
  // stored at cache row start + j is visible); a chain has (2 << i) - 1.  Unused by chunk items.
  uint32_t vis_lo, vis_hi;
};
struct HatMergeItem {
  int32_t row0;      // first batch row of this group
  int32_t nrows;     // rows in the group (<= 16)
  int32_t part_row;  // partial row of split 0 for row0; split i is at part_row + i*stride
  int32_t nsplit;
  int32_t stride;    // partial rows between consecutive splits (= rows of the attention item)
  int32_t pad0, pad1, pad2;
};
struct HatAttn {
  const act_t* qkv;          // P32 [., 3d]; q = columns [0, d)
  const kv_t* pool_layer;    // this layer's pages
  int kv_f16;                // cache elements are fp16 (else bf16, widened to fp16 on their way to the MFMA)
  act_t* outP;               // P32 [., d]
  act_t* part_o;             // [part rows][H][hd] partial outputs, each normalised by its own sum
  float2* part_ml;           // [part rows][H] (running max in log2 units, sum)
  const HatAttnItem* items;
  int n_items;
  int H, hd, d;
  int n_pages;               // pool capacity (pages per head and layer)
};
hipError_t hat_launch_attn_chunk(const HatPlanDev& p, const HatAttn& a, hipStream_t st);
hipError_t hat_launch_attn_verify(const HatPlanDev& p, const HatAttn& a, hipStream_t st);
hipError_t hat_launch_attn_merge(const HatAttn& a, const HatMergeItem* items, int n_items, hipStream_t st);
// the verify kernel's loads without its arithmetic (a measurement aid; writes nothing but *sink, and that never)
hipError_t hat_launch_attn_verify_probe(const HatPlanDev& p, const HatAttn& a, uint32_t* sink, hipStream_t st);

// ---- fixtures ------------------------------------------------------------------
// k, v: [n, H, hd] bf16 plain; pages: device array of the page ids covering the rows.  An fp16 cache
// takes the bf16 values exactly (where fp16 can hold them) and gives them back rounded to bf16.
hipError_t hat_launch_kv_import(kv_t* pool_layer, int n_pages, const int32_t* pages, int pos0, int n,
                                const bf16_t* k, const bf16_t* v, int H, int hd, int kv_f16, hipStream_t st);
// Row moves inside one device's cache, applied in order in every layer and head.
struct HatRowMoves {
  int32_t n;
  int32_t src[HAT_MAX_VERIFY_ROWS], dst[HAT_MAX_VERIFY_ROWS];  // page*16 + slot
};
hipError_t hat_launch_kv_move(kv_t* pool, size_t layer_elems, int L, int n_pages, const HatRowMoves& mv, int H,
                              int hd, hipStream_t st);
hipError_t hat_launch_kv_export(const kv_t* pool_layer, int n_pages, const int32_t* pages, int pos0, int n,
                                bf16_t* k, bf16_t* v, int H, int hd, int kv_f16, hipStream_t st);
// P32 [., ncols_total] columns [col0, col0+ncols) -> fp32 row-major [T, ncols]
hipError_t hat_launch_unpack_p32(const act_t* srcP, int row_len, int col0, int ncols, int T, float* dst,
                                 hipStream_t st);
