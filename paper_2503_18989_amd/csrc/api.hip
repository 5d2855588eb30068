// Host side of the middle-submodel library: configuration, workspace carving,
// the integer planner of a step (positions, page table, attention work lists)
// and the launch sequence of the decoder layers.  Interface and semantics are
// documented in include/hat_mid.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <set>
#include <string>
#include <vector>

#include "../../include/hat_mid.h"
#include "hat_kernels.h"
#include "hat_layout.h"

// ---- static scratch of hat_mid_kv_export_static -------------------------------------------------
// Page ids of the rows being exported, staged here instead of in the caller's workspace.  One copy
// of the array exists on every GPU the library is loaded on (16 KB each, held until the process
// ends).  In host code the array's NAME is only a handle for hipGetSymbolAddress: the address a
// kernel may use is the one that call returns, taken once per device with that device current.
constexpr int kStaticPageIds = 4096;   // 4096 pages = 65 536 cache rows per call
static __device__ __align__(256) int32_t scratch[kStaticPageIds];

namespace {

constexpr int kMaxGpus = 64;
std::mutex g_scratch_mu;
int32_t* g_scratch_ptr[kMaxGpus] = {};   // device address of `scratch` on each GPU (nullptr: not taken yet)

// Address of the current device's copy of `scratch`, taken on first use on that device.
hipError_t static_scratch(int device, int32_t** out) {
  if (device < 0 || device >= kMaxGpus) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = (int32_t*)p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int round_up(int x, int a) { return (x + a - 1) / a * a; }

constexpr int kCapAttnTarget = 2048;  // workgroup target that the work-list capacities are sized for

struct LayerDev {
  act_t *wqkv, *wo, *wgu, *wd;
  float *g_attn, *g_ffn;
};

struct Shapes {
  int L, d, H, hd, F, Fpad;
  int Nqkv, No, Ngu, Nd;  // padded weight rows
  int Tcap;               // row capacity of activation buffers (multiple of 256)
  int attn_target;        // workgroups a chunk-attention launch should reach
  int verify_target;      // workgroups a verify-attention launch should reach
  int chunk_items_cap, verify_items_cap, merge_cap;
  int part_rows_cap;
  int gemm_part_rows;     // rows of the split-K partial-sum buffer
  size_t plan_words;
};

bool valid_cfg(const hat_mid_config_t* c) {
  if (!c) return false;
  if (c->n_layers <= 0 || c->n_heads <= 0 || c->d_ffn <= 0) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->d_model != c->n_heads * c->head_dim || c->d_model % 64 != 0 || c->d_model > 8192) return false;
  if (c->page_size != HAT_PAGE_SIZE || c->n_pages <= 0) return false;
  if (c->max_devices <= 0 || c->max_step_tokens <= 0 || c->max_pos <= 0) return false;
  if (c->io_dtype != HAT_BF16 && c->io_dtype != HAT_F32) return false;
  if (c->kv_dtype != HAT_KV_BF16 && c->kv_dtype != HAT_KV_F16) return false;
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) return false;
  return true;
}

Shapes make_shapes(const hat_mid_config_t& c) {
  Shapes s;
  s.L = c.n_layers; s.d = c.d_model; s.H = c.n_heads; s.hd = c.head_dim; s.F = c.d_ffn;
  s.Fpad = round_up(c.d_ffn, 64);
  s.Nqkv = round_up(3 * s.d, 256);
  s.No = round_up(s.d, 256);
  s.Ngu = round_up(2 * s.Fpad, 256);
  s.Nd = round_up(s.d, 256);
  s.Tcap = round_up(c.max_step_tokens, 256);
  s.attn_target = 256;  // one 8-wave workgroup per CU
  s.verify_target = 2048;
  // capacities are sized for this target; a larger one (hat_mid_debug_set_attn_targets) splits
  // only as far as they allow -- the planner checks every capacity before it splits
  const int per_head = (kCapAttnTarget + s.H - 1) / s.H;
  s.chunk_items_cap = 2 * per_head + s.Tcap / 128 + c.max_devices + 2;
  s.verify_items_cap = 2 * per_head + c.max_devices + 2;
  s.merge_cap = s.Tcap / 16 + s.Tcap / 128 + 2 * c.max_devices + 2;
  s.part_rows_cap = HAT_CHUNK_QROWS * (2 * per_head + 2) + HAT_MAX_VERIFY * s.verify_items_cap;
  s.gemm_part_rows = 4096;
  s.plan_words = (size_t)3 * s.Tcap + 8 * ((size_t)s.Tcap / 16 + 2 * (size_t)c.max_devices + 2) + 8 * (size_t)c.max_devices + 16 + (size_t)c.n_pages + c.max_devices +
                 12 * ((size_t)s.chunk_items_cap + s.verify_items_cap) + 8 * (size_t)s.merge_cap + 64;
  return s;
}

// carve the workspace; with base == nullptr only sizes are computed
struct Carver {
  unsigned char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((unsigned char*)b) {}
  template <class T>
  T* take(size_t n) {
    off = align_up(off, 256);
    T* p = base ? (T*)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

struct Buffers {
  std::vector<LayerDev> layers;
  double* inv_freq;
  float* resid;
  act_t *xn, *xn2, *qkv, *attn, *act;
  float2* table;
  act_t* part_o;
  float2* part_ml;
  float* gemm_part;
  int32_t* plan_dev;
  int32_t* fixture_pages;
  float* stage_in[2];
  float* stage_out;
};

size_t carve(const hat_mid_config_t& c, const Shapes& s, void* base, Buffers* out) {
  Carver cv(base);
  Buffers b;
  b.layers.resize(s.L);
  for (int l = 0; l < s.L; ++l) {
    b.layers[l].wqkv = cv.take<act_t>((size_t)s.Nqkv * s.d);
    b.layers[l].wo = cv.take<act_t>((size_t)s.No * s.d);
    b.layers[l].wgu = cv.take<act_t>((size_t)s.Ngu * s.d);
    b.layers[l].wd = cv.take<act_t>((size_t)s.Nd * s.Fpad);
    b.layers[l].g_attn = cv.take<float>(s.d);
    b.layers[l].g_ffn = cv.take<float>(s.d);
  }
  b.inv_freq = cv.take<double>(s.hd / 2);
  b.resid = cv.take<float>((size_t)s.Tcap * s.d);
  b.xn = cv.take<act_t>((size_t)s.Tcap * s.d);
  b.xn2 = cv.take<act_t>((size_t)s.Tcap * s.d);
  b.qkv = cv.take<act_t>((size_t)s.Tcap * 3 * s.d);
  b.attn = cv.take<act_t>((size_t)s.Tcap * s.d);
  b.act = cv.take<act_t>((size_t)s.Tcap * s.Fpad);
  b.table = cv.take<float2>((size_t)s.Tcap * (s.hd / 2));
  b.part_o = cv.take<act_t>((size_t)s.part_rows_cap * s.d);
  b.part_ml = cv.take<float2>((size_t)s.part_rows_cap * s.H);
  b.gemm_part = cv.take<float>((size_t)s.gemm_part_rows * s.d);
  b.plan_dev = cv.take<int32_t>(s.plan_words);
  b.fixture_pages = cv.take<int32_t>((size_t)(c.max_pos + 15) / 16 + 2);
  // staging for steps whose hidden states live in host memory: two input slots (the upload of the
  // next step overlaps the current one) and one output slot, sized for fp32 rows
  b.stage_in[0] = cv.take<float>((size_t)s.Tcap * s.d);
  b.stage_in[1] = cv.take<float>((size_t)s.Tcap * s.d);
  b.stage_out = cv.take<float>((size_t)s.Tcap * s.d);
  if (out) *out = b;
  return align_up(cv.off, 256);
}

struct DeviceState {
  int len = 0;
  std::vector<int32_t> pages;
};

constexpr int kPlanBufs = 3;

}  // namespace

struct hat_mid {
  hat_mid_config_t cfg;
  Shapes s;
  Buffers b;
  kv_t* pool;
  size_t layer_pool_elems;

  std::set<int32_t> free_pages;
  std::vector<DeviceState> dev;

  int32_t* plan_host[kPlanBufs] = {nullptr, nullptr, nullptr};
  hipEvent_t plan_ev[kPlanBufs] = {nullptr, nullptr, nullptr};
  bool plan_ev_used[kPlanBufs] = {false, false, false};
  int plan_next = 0;

  hipEvent_t ev_begin = nullptr, ev_end = nullptr;
  bool have_step = false;
  int last_tokens = 0;

  bool profiling = false;
  struct Rec { int id; hipEvent_t a, b; };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> ev_pool;

  // steps fed from host memory (hat_mid_forward_host)
  hipStream_t copy_stream = nullptr;
  hipEvent_t up_done[2] = {nullptr, nullptr}, slot_free[2] = {nullptr, nullptr};
  bool slot_used[2] = {false, false};
  int host_slot = 0;

  // what the step being planned has done to the page state, so that a failure after the pages
  // moved (plan capacity, a HIP call while enqueueing) can put everything back
  struct PageOp { int32_t page; bool taken; };   // taken: the page left the free set; else it entered it
  std::vector<PageOp> undo_pages;
  std::vector<std::pair<int32_t, DeviceState>> undo_dev;
  bool undo_on = false;

  // hat_mid_kv_export_static: this GPU's copy of the static scratch array, a pinned host buffer for
  // the page ids on their way there, and the event that says the last upload has read it
  int device = -1;
  int32_t* static_pages_dev = nullptr;
  int32_t* static_pages_host = nullptr;
  hipEvent_t static_ev = nullptr;
  bool static_ev_used = false;

  hipStream_t last_stream = nullptr;       // stream of the most recent enqueue (hat_mid_destroy waits for it)
  bool used_stream = false;
  size_t plan_limit = 0;                   // > 0: lowered plan capacity (hat_mid_debug_limit_plan)
  bool verify_probe = false;               // verify attention replaced by its loads-only twin (hat_mid_debug_set_verify_probe)

  bool host_only = false;                  // built by hat_mid_debug_create_host_only: no GPU memory, no HIP calls
  std::vector<int32_t> host_plan;          // its plan words
  int force_tile[4] = {-1, -1, -1, -1};   // tuning overrides per GEMM class (qkv, o, gate/up, down)
  int force_ksplit[4] = {0, 0, 0, 0};

  std::string err;
};

namespace {

hat_status_t fail(hat_mid* h, hat_status_t st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (h) h->err = buf;
  return st;
}

#define HIP_TRY(h, expr)                                                                          \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return fail(h, HAT_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// node i sees itself and nothing later; its ancestors are one path (each ancestor's own mask is
// the ancestors before it plus itself)
bool valid_tree(const uint8_t* m, int n) {
  for (int i = 0; i < n; ++i) {
    if ((m[i] >> i) != 1) return false;
    unsigned path = 0;
    for (int j = 0; j < i; ++j) {
      if (!((m[i] >> j) & 1)) continue;
      if (m[j] != (path | (1u << j))) return false;
      path |= 1u << j;
    }
  }
  return true;
}

int32_t take_lowest(hat_mid* h) {
  auto it = h->free_pages.begin();
  int32_t id = *it;
  h->free_pages.erase(it);
  if (h->undo_on) h->undo_pages.push_back({id, true});
  return id;
}

void give_back(hat_mid* h, int32_t id) {
  h->free_pages.insert(id);
  if (h->undo_on) h->undo_pages.push_back({id, false});
}

// Page movements of one call are logged between undo_begin and undo_commit; undo_rollback puts
// lengths, page lists and the free set back to what they were at undo_begin.
void undo_begin(hat_mid* h) {
  h->undo_pages.clear();
  h->undo_dev.clear();
  h->undo_on = true;
}
void undo_save_device(hat_mid* h, int32_t id) { h->undo_dev.emplace_back(id, h->dev[id]); }
void undo_commit(hat_mid* h) {
  h->undo_on = false;
  h->undo_pages.clear();
  h->undo_dev.clear();
}
void undo_rollback(hat_mid* h) {
  h->undo_on = false;
  for (auto it = h->undo_pages.rbegin(); it != h->undo_pages.rend(); ++it) {
    if (it->taken) h->free_pages.insert(it->page);
    else h->free_pages.erase(it->page);
  }
  for (auto it = h->undo_dev.rbegin(); it != h->undo_dev.rend(); ++it) h->dev[it->first] = std::move(it->second);
  h->undo_pages.clear();
  h->undo_dev.clear();
}

void note_stream(hat_mid* h, hipStream_t st) {
  h->last_stream = st;
  h->used_stream = true;
}

hipEvent_t get_event(hat_mid* h) {
  if (!h->ev_pool.empty()) {
    hipEvent_t e = h->ev_pool.back();
    h->ev_pool.pop_back();
    return e;
  }
  hipEvent_t e;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// brackets one launch with events when profiling is on
struct Timed {
  hat_mid* h;
  hipStream_t st;
  int id;
  hipEvent_t a = nullptr, b = nullptr;
  Timed(hat_mid* h_, hipStream_t st_, int id_) : h(h_), st(st_), id(id_) {
    if (h->profiling) {
      a = get_event(h);
      b = get_event(h);
      if (a) (void)hipEventRecord(a, st);
    }
  }
  ~Timed() {
    if (h->profiling && a && b) {
      (void)hipEventRecord(b, st);
      h->recs.push_back({id, a, b});
    }
  }
};

#define LAUNCH(h, st, id, call)                                                                      \
  do {                                                                                               \
    hipError_t e_;                                                                                   \
    {                                                                                                \
      Timed t_(h, st, id);                                                                           \
      e_ = (call);                                                                                   \
    }                                                                                                \
    if (e_ != hipSuccess) return fail(h, HAT_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));   \
  } while (0)

}  // namespace

extern "C" {

size_t hat_mid_kv_bytes(const hat_mid_config_t* cfg) {
  if (!valid_cfg(cfg)) return 0;
  return (size_t)cfg->n_layers * cfg->n_pages * kv_page_elems(cfg->n_heads, cfg->head_dim) * sizeof(kv_t);
}

size_t hat_mid_workspace_bytes(const hat_mid_config_t* cfg) {
  if (!valid_cfg(cfg)) return 0;
  Shapes s = make_shapes(*cfg);
  return carve(*cfg, s, nullptr, nullptr);
}

static hat_status_t create_impl(const hat_mid_config_t* cfg, const hat_mid_layer_weights_t* layers, void* kv_pool,
                                void* workspace, void* hip_stream, hat_mid_t** out) {
  if (out) *out = nullptr;
  if (!out || !valid_cfg(cfg) || !layers || !kv_pool || !workspace) return HAT_EINVAL;
  if (((uintptr_t)kv_pool | (uintptr_t)workspace) & 255) return HAT_EINVAL;
  for (int l = 0; l < cfg->n_layers; ++l) {
    const hat_mid_layer_weights_t& w = layers[l];
    if (!w.attn_norm || !w.wq || !w.wk || !w.wv || !w.wo || !w.ffn_norm || !w.w_gate || !w.w_up || !w.w_down)
      return HAT_EINVAL;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  hat_mid* h = new hat_mid();
  h->cfg = *cfg;
  h->s = make_shapes(*cfg);
  carve(*cfg, h->s, workspace, &h->b);
  h->pool = (kv_t*)kv_pool;
  h->layer_pool_elems = (size_t)cfg->n_pages * kv_page_elems(cfg->n_heads, cfg->head_dim);
  for (int i = 0; i < cfg->n_pages; ++i) h->free_pages.insert(i);
  h->dev.resize(cfg->max_devices);

  auto bail = [&](hipError_t e, const char* what) {
    fprintf(stderr, "hat_mid_create: %s: %s\n", what, hipGetErrorString(e));
    hat_mid_destroy(h);
    return HAT_EHIP;
  };
  hipError_t e;
  if ((e = hat_gemm_init()) != hipSuccess) return bail(e, "gemm init");
  for (int i = 0; i < kPlanBufs; ++i) {
    if ((e = hipHostMalloc((void**)&h->plan_host[i], h->s.plan_words * sizeof(int32_t), hipHostMallocDefault)) !=
        hipSuccess)
      return bail(e, "pinned plan buffer");
    if ((e = hipEventCreateWithFlags(&h->plan_ev[i], hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
  }
  if ((e = hipGetDevice(&h->device)) != hipSuccess) return bail(e, "current device");
  if ((e = static_scratch(h->device, &h->static_pages_dev)) != hipSuccess) return bail(e, "address of the static scratch array");
  if ((e = hipHostMalloc((void**)&h->static_pages_host, kStaticPageIds * sizeof(int32_t), hipHostMallocDefault)) != hipSuccess)
    return bail(e, "pinned page-id buffer");
  if ((e = hipEventCreateWithFlags(&h->static_ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
  if ((e = hipStreamCreateWithFlags(&h->copy_stream, hipStreamNonBlocking)) != hipSuccess) return bail(e, "copy stream");
  for (int i = 0; i < 2; ++i) {
    if ((e = hipEventCreateWithFlags(&h->up_done[i], hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
    if ((e = hipEventCreateWithFlags(&h->slot_free[i], hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
  }
  if ((e = hipEventCreate(&h->ev_begin)) != hipSuccess) return bail(e, "event");
  if ((e = hipEventCreate(&h->ev_end)) != hipSuccess) return bail(e, "event");

  // rotary frequencies theta^(-2i/hd), in double
  {
    std::vector<double> f(h->s.hd / 2);
    for (int i = 0; i < h->s.hd / 2; ++i) f[i] = std::pow((double)cfg->rope_theta, -2.0 * i / h->s.hd);
    if ((e = hipMemcpyAsync(h->b.inv_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice, st)) !=
        hipSuccess)
      return bail(e, "inv_freq upload");
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return bail(e, "sync");
  }
  // weights -> P32 tiles
  const Shapes& s = h->s;
  for (int l = 0; l < s.L; ++l) {
    const hat_mid_layer_weights_t& w = layers[l];
    LayerDev& ld = h->b.layers[l];
    if ((e = hat_launch_retile(ld.wqkv, s.Nqkv, s.d, (const bf16_t*)w.wq, (const bf16_t*)w.wk, (const bf16_t*)w.wv,
                               s.d, s.d, 1, st)) != hipSuccess)
      return bail(e, "retile qkv");
    if ((e = hat_launch_retile(ld.wo, s.No, s.d, (const bf16_t*)w.wo, nullptr, nullptr, s.d, s.d, 0, st)) !=
        hipSuccess)
      return bail(e, "retile o");
    if ((e = hat_launch_retile(ld.wgu, s.Ngu, s.d, (const bf16_t*)w.w_gate, (const bf16_t*)w.w_up, nullptr, s.F, s.d,
                               2, st)) != hipSuccess)
      return bail(e, "retile gate/up");
    if ((e = hat_launch_retile(ld.wd, s.Nd, s.Fpad, (const bf16_t*)w.w_down, nullptr, nullptr, s.d, s.F, 0, st)) !=
        hipSuccess)
      return bail(e, "retile down");
    if ((e = hat_launch_bf16_to_f32((const bf16_t*)w.attn_norm, ld.g_attn, s.d, st)) != hipSuccess)
      return bail(e, "gain");
    if ((e = hat_launch_bf16_to_f32((const bf16_t*)w.ffn_norm, ld.g_ffn, s.d, st)) != hipSuccess)
      return bail(e, "gain");
  }
  note_stream(h, st);
  *out = h;
  return HAT_OK;
}

void hat_mid_destroy(hat_mid_t* h) {
  if (!h) return;
  if (h->host_only) {
    delete h;
    return;
  }
  // wait for this handle's work only: its copy stream and the stream of its last enqueue (calls on
  // one handle are stream-ordered, so that covers all of them)
  if (h->copy_stream) (void)hipStreamSynchronize(h->copy_stream);
  if (h->used_stream) (void)hipStreamSynchronize(h->last_stream);
  for (int i = 0; i < kPlanBufs; ++i) {
    if (h->plan_host[i]) (void)hipHostFree(h->plan_host[i]);
    if (h->plan_ev[i]) (void)hipEventDestroy(h->plan_ev[i]);
  }
  if (h->ev_begin) (void)hipEventDestroy(h->ev_begin);
  if (h->ev_end) (void)hipEventDestroy(h->ev_end);
  if (h->static_ev) (void)hipEventDestroy(h->static_ev);
  if (h->static_pages_host) (void)hipHostFree(h->static_pages_host);
  for (int i = 0; i < 2; ++i) {
    if (h->up_done[i]) (void)hipEventDestroy(h->up_done[i]);
    if (h->slot_free[i]) (void)hipEventDestroy(h->slot_free[i]);
  }
  if (h->copy_stream) (void)hipStreamDestroy(h->copy_stream);
  for (auto& r : h->recs) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  for (auto e : h->ev_pool) (void)hipEventDestroy(e);
  delete h;
}

const char* hat_mid_last_error(const hat_mid_t* h) { return h ? h->err.c_str() : "null handle"; }

hat_status_t hat_mid_release(hat_mid_t* h, int32_t device_id) {
  if (!h) return HAT_EINVAL;
  if (device_id < 0 || device_id >= h->cfg.max_devices) return fail(h, HAT_EDEVICE, "device id %d out of range", device_id);
  DeviceState& d = h->dev[device_id];
  for (int32_t p : d.pages) h->free_pages.insert(p);
  d.pages.clear();
  d.len = 0;
  return HAT_OK;
}

hat_status_t hat_mid_kv_compact(hat_mid_t* h, int32_t device_id, int32_t base_pos, const int32_t* keep,
                                int32_t n_keep, void* hip_stream) {
  if (!h) return HAT_EINVAL;
  const hat_mid_config_t& c = h->cfg;
  if (device_id < 0 || device_id >= c.max_devices) return fail(h, HAT_EDEVICE, "device id %d out of range", device_id);
  if (base_pos < 0 || n_keep < 0 || n_keep > HAT_MAX_VERIFY || (n_keep > 0 && !keep))
    return fail(h, HAT_EINVAL, "bad compact arguments");
  for (int i = 0; i < n_keep; ++i)
    if (keep[i] < 0 || keep[i] >= HAT_MAX_VERIFY || (i > 0 && keep[i] <= keep[i - 1]))
      return fail(h, HAT_EINVAL, "kept nodes must be ascending indices below %d", HAT_MAX_VERIFY);
  DeviceState& d = h->dev[device_id];
  if (base_pos > d.len || (n_keep > 0 && base_pos + keep[n_keep - 1] >= d.len))
    return fail(h, HAT_EPOS, "kept row beyond cache length %d", d.len);
  HatRowMoves mv{};
  for (int i = 0; i < n_keep; ++i) {
    const int src = base_pos + keep[i], dst = base_pos + i;
    if (src == dst) continue;
    mv.src[mv.n] = d.pages[src >> 4] * 16 + (src & 15);
    mv.dst[mv.n] = d.pages[dst >> 4] * 16 + (dst & 15);
    ++mv.n;
  }
  if (!h->host_only) note_stream(h, (hipStream_t)hip_stream);
  if (!h->host_only)
    HIP_TRY(h, hat_launch_kv_move(h->pool, h->layer_pool_elems, c.n_layers, c.n_pages, mv, c.n_heads, c.head_dim,
                                  (hipStream_t)hip_stream));
  d.len = base_pos + n_keep;
  const size_t want = (size_t)(d.len + 15) / 16;
  while (d.pages.size() > want) {
    h->free_pages.insert(d.pages.back());
    d.pages.pop_back();
  }
  return HAT_OK;
}

hat_status_t hat_mid_kv_query(const hat_mid_t* h, int32_t device_id, int32_t* kv_len, int32_t* pages_out, int32_t cap,
                              int32_t* n_pages_out) {
  if (!h) return HAT_EINVAL;
  if (device_id < 0 || device_id >= h->cfg.max_devices) return HAT_EDEVICE;
  const DeviceState& d = h->dev[device_id];
  if (kv_len) *kv_len = d.len;
  if (n_pages_out) *n_pages_out = (int32_t)d.pages.size();
  if (pages_out)
    for (int i = 0; i < cap && i < (int)d.pages.size(); ++i) pages_out[i] = d.pages[i];
  return HAT_OK;
}

// What the planning half of a step hands to the enqueueing half: where each array lies in the
// plan words, and how many work items there are.
struct StepPlan {
  int T = 0, S = 0, n_append = 0;
  size_t o_pos = 0, o_dst = 0, o_tseg = 0, o_toff = 0, o_sstart = 0, o_spt = 0, o_in = 0, o_out = 0, o_pt = 0, o_app = 0;
  size_t o_ci = 0, o_vi = 0, o_mi = 0, words = 0;
  int n_citems = 0, n_vitems = 0, n_mitems = 0;
};

// Host half of a step: validates every segment, commits the page movements, and writes the plan
// (positions, write targets, page lists, attention work lists) into P (capacity: plan_words).
// No GPU call: the same code serves the host-only handles that the planner's CPU tests use.
static hat_status_t plan_step(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, int32_t* P, StepPlan* sp) {
  if (!segs || n_segs < 0) return fail(h, HAT_EINVAL, "no segments");
  const hat_mid_config_t& c = h->cfg;
  const Shapes& s = h->s;

  // ---- validate everything before touching state
  if (n_segs > c.max_devices) return fail(h, HAT_EINVAL, "more segments (%d) than devices", n_segs);
  std::vector<char> seen(c.max_devices, 0);
  long total = 0;
  for (int i = 0; i < n_segs; ++i) {
    const hat_mid_segment_t& g = segs[i];
    if (g.device_id < 0 || g.device_id >= c.max_devices)
      return fail(h, HAT_EDEVICE, "segment %d: device id %d out of range", i, g.device_id);
    if ((g.kind != HAT_SEG_CHUNK && g.kind != HAT_SEG_VERIFY) || g.n <= 0 || g.start_pos < 0)
      return fail(h, HAT_EINVAL, "segment %d: bad kind/n/start", i);
    if (g.kind == HAT_SEG_VERIFY && g.n > HAT_MAX_VERIFY)
      return fail(h, HAT_EINVAL, "segment %d: verify segment of %d rows (max %d)", i, g.n, HAT_MAX_VERIFY);
    if (g.tree_mask) {
      if (g.kind != HAT_SEG_VERIFY) return fail(h, HAT_EINVAL, "segment %d: a tree needs a verify segment", i);
      if (!valid_tree(g.tree_mask, g.n)) return fail(h, HAT_EINVAL, "segment %d: tree_mask is not a parents-first forest", i);
    }
    if ((long)g.start_pos + g.n > c.max_pos) return fail(h, HAT_EINVAL, "segment %d: beyond max_pos", i);
    if (!g.hidden_in || !g.hidden_out) return fail(h, HAT_EINVAL, "segment %d: null hidden pointer", i);
    if (seen[g.device_id]) return fail(h, HAT_EDUP, "segment %d: device %d twice in one step", i, g.device_id);
    seen[g.device_id] = 1;
    if (g.start_pos > h->dev[g.device_id].len)
      return fail(h, HAT_EPOS, "segment %d: start %d beyond cache length %d", i, g.start_pos, h->dev[g.device_id].len);
    total += g.n;
  }
  if (total > c.max_step_tokens) return fail(h, HAT_EINVAL, "step of %ld rows exceeds max_step_tokens", total);
  {
    long free_after = (long)h->free_pages.size(), need = 0;
    for (int i = 0; i < n_segs; ++i) {
      const hat_mid_segment_t& g = segs[i];
      const long have = (long)h->dev[g.device_id].pages.size();
      const long keep = (g.start_pos + 15) / 16;
      free_after += have - keep;
      need += (g.start_pos + g.n + 15) / 16 - keep;
    }
    if (need > free_after) return fail(h, HAT_ENOMEM, "KV pool exhausted: need %ld pages, %ld free", need, free_after);
  }

  // ---- move the pages: all rollbacks, then all allocations.  Logged: the caller commits the
  // step once it has been planned and enqueued, and rolls it back otherwise.
  undo_begin(h);
  for (int i = 0; i < n_segs; ++i) undo_save_device(h, segs[i].device_id);
  for (int i = 0; i < n_segs; ++i) {
    DeviceState& d = h->dev[segs[i].device_id];
    const size_t keep = (size_t)(segs[i].start_pos + 15) / 16;
    while (d.pages.size() > keep) {
      give_back(h, d.pages.back());
      d.pages.pop_back();
    }
    d.len = segs[i].start_pos;
  }
  const int T = (int)total, S = n_segs;
  int np_total = 0;
  for (int i = 0; i < n_segs; ++i) {
    DeviceState& d = h->dev[segs[i].device_id];
    const size_t want = (size_t)(segs[i].start_pos + segs[i].n + 15) / 16;
    while (d.pages.size() < want) d.pages.push_back(take_lowest(h));
    d.len = segs[i].start_pos + segs[i].n;
    np_total += (int)d.pages.size();
  }

  // ---- plan words
  size_t w = 0;
  auto take = [&](size_t n, size_t align_words) {
    w = align_up(w, align_words);
    size_t o = w;
    w += n;
    return o;
  };
  const size_t o_pos = take(T, 1), o_dst = take(T, 1), o_tseg = take(T, 1);
  const size_t o_toff = take(S + 1, 1), o_sstart = take(S, 1), o_spt = take(S, 1);
  const size_t o_in = take(2 * (size_t)S, 2), o_out = take(2 * (size_t)S, 2);
  const size_t o_pt = take(np_total, 1);
  int n_append = 0;
  for (int i = 0; i < S; ++i) n_append += ((segs[i].start_pos + segs[i].n - 1) >> 4) - (segs[i].start_pos >> 4) + 1;
  const size_t o_app = take(8 * (size_t)n_append, 4);

  std::vector<HatAttnItem> citems, vitems;
  std::vector<HatMergeItem> mitems;
  {
    int t = 0, pt = 0;
    for (int i = 0; i < S; ++i) {
      const hat_mid_segment_t& g = segs[i];
      const DeviceState& d = h->dev[g.device_id];
      P[o_toff + i] = t;
      P[o_sstart + i] = g.start_pos;
      P[o_spt + i] = pt;
      uint64_t ip = (uint64_t)(uintptr_t)g.hidden_in, op = (uint64_t)(uintptr_t)g.hidden_out;
      memcpy(&P[o_in + 2 * i], &ip, 8);
      memcpy(&P[o_out + 2 * i], &op, 8);
      for (size_t k = 0; k < d.pages.size(); ++k) P[o_pt + pt + k] = d.pages[k];
      for (int r = 0; r < g.n; ++r) {
        const int q = g.start_pos + r;   // cache row; also the position unless the rows form a tree
        P[o_pos + t] = g.tree_mask ? g.start_pos + __builtin_popcount(g.tree_mask[r]) - 1 : q;
        P[o_dst + t] = d.pages[q >> 4] * 16 + (q & 15);
        P[o_tseg + t] = i;
        ++t;
      }
      pt += (int)d.pages.size();
    }
    P[o_toff + S] = T;
    HatAppendItem* ap = (HatAppendItem*)&P[o_app];
    for (int i = 0; i < S; ++i) {
      const hat_mid_segment_t& g = segs[i];
      const DeviceState& d = h->dev[g.device_id];
      for (int pg = g.start_pos >> 4; pg <= (g.start_pos + g.n - 1) >> 4; ++pg) {
        HatAppendItem a{};
        a.page = d.pages[pg]; a.pos0 = pg * 16; a.row0 = P[o_toff + i] + (a.pos0 - g.start_pos);
        a.lo = std::max(g.start_pos, a.pos0); a.hi = std::min(g.start_pos + g.n, a.pos0 + 16);
        *ap++ = a;
      }
    }
  }

  // ---- attention work lists
  {
    const int per_head = (s.verify_target + s.H - 1) / s.H;  // verify items wanted
    int part_row = 0;
    // rows of a split item are merged in groups of 16 (one workgroup per group and head)
    auto push_merge = [&](int row0, int nrows, int prow, int nsplit) {
      for (int g0 = 0; g0 < nrows; g0 += 16) {
        HatMergeItem m{};
        m.row0 = row0 + g0; m.nrows = std::min(16, nrows - g0); m.part_row = prow + g0; m.nsplit = nsplit;
        m.stride = nrows;
        mitems.push_back(m);
      }
    };
    // verify segments: split each cache into key ranges of about equal size
    long vkeys = 0;
    int nver = 0;
    for (int i = 0; i < S; ++i)
      if (segs[i].kind == HAT_SEG_VERIFY) { vkeys += segs[i].start_pos + segs[i].n; ++nver; }
    if (nver) {
      long ch = (vkeys + per_head - 1) / per_head;
      ch = std::max<long>(256, (ch + 127) / 128 * 128);
      for (int i = 0; i < S; ++i) {
        if (segs[i].kind != HAT_SEG_VERIFY) continue;
        const int len = segs[i].start_pos + segs[i].n;
        int ns = (int)((len + ch - 1) / ch);
        ns = std::min(ns, 64);
        if ((int)vitems.size() + ns > s.verify_items_cap - 1 || part_row + ns * segs[i].n > s.part_rows_cap) ns = 1;
        const int step = round_up((len + ns - 1) / ns, 64);
        ns = (len + step - 1) / step;
        for (int k = 0; k < ns; ++k) {
          HatAttnItem it{};
          it.seg = i; it.q0 = 0; it.nq = segs[i].n;
          it.start = segs[i].start_pos; it.tok0 = P[o_toff + i]; it.kv_len = len; it.pt_off = P[o_spt + i];
          it.kv_begin = k * step; it.kv_end = std::min(len, (k + 1) * step);
          it.part_row = ns > 1 ? part_row + k * segs[i].n : -1;
          for (int r = 0; r < segs[i].n; ++r) {
            const uint32_t vis = segs[i].tree_mask ? segs[i].tree_mask[r] : (2u << r) - 1;
            (r < 4 ? it.vis_lo : it.vis_hi) |= vis << (8 * (r & 3));
          }
          vitems.push_back(it);
        }
        if (ns > 1) {
          push_merge(P[o_toff + i], segs[i].n, part_row, ns);
          part_row += ns * segs[i].n;
        }
      }
    }
    // chunk segments: tiles of HAT_CHUNK_QROWS rows, split along the keys so that no work item
    // is larger than a third of one workgroup slot's share of the launch (all heads do the same
    // work, so a head has attn_target / H slots): the items, sorted by cost, then pack evenly.
    double total_cost = 0;
    for (int i = 0; i < S; ++i) {
      if (segs[i].kind != HAT_SEG_CHUNK) continue;
      for (int q0 = 0; q0 < segs[i].n; q0 += HAT_CHUNK_QROWS) {
        const int nq = std::min(HAT_CHUNK_QROWS, segs[i].n - q0);
        total_cost += (double)nq * (segs[i].start_pos + q0 + 0.5 * nq);
      }
    }
    if (total_cost > 0) {
      const double slots = std::max(1, s.attn_target / s.H);
      const double cost_cap = std::max(256.0 * 256.0, total_cost / (3.0 * slots));
      for (int i = 0; i < S; ++i) {
        if (segs[i].kind != HAT_SEG_CHUNK) continue;
        for (int q0 = 0; q0 < segs[i].n; q0 += HAT_CHUNK_QROWS) {
          const int nq = std::min(HAT_CHUNK_QROWS, segs[i].n - q0);
          const int need = segs[i].start_pos + q0 + nq;
          const double cost = (double)nq * (need - 0.5 * nq);
          int ns = (int)std::ceil(cost / cost_cap);
          ns = std::max(1, std::min(std::min(ns, std::max(1, need / 256)), 16));
          if ((int)citems.size() + ns > s.chunk_items_cap - 1 || part_row + ns * nq > s.part_rows_cap ||
              (int)mitems.size() + 9 >= s.merge_cap)
            ns = 1;
          const int step = round_up((need + ns - 1) / ns, 64);
          ns = (need + step - 1) / step;
          for (int k = 0; k < ns; ++k) {
            HatAttnItem it{};
            it.seg = i; it.q0 = q0; it.nq = nq;
            it.start = segs[i].start_pos; it.tok0 = P[o_toff + i]; it.kv_len = segs[i].start_pos + segs[i].n;
            it.pt_off = P[o_spt + i];
            it.kv_begin = k * step; it.kv_end = std::min(need, (k + 1) * step);
            it.part_row = ns > 1 ? part_row + k * nq : -1;
            citems.push_back(it);
          }
          if (ns > 1) {
            push_merge(P[o_toff + i] + q0, nq, part_row, ns);
            part_row += ns * nq;
          }
        }
      }
    }
    auto by_cost = [](const HatAttnItem& a, const HatAttnItem& b) {
      return (long)(a.kv_end - a.kv_begin) * a.nq > (long)(b.kv_end - b.kv_begin) * b.nq;
    };
    std::stable_sort(citems.begin(), citems.end(), by_cost);
    std::stable_sort(vitems.begin(), vitems.end(), by_cost);
  }
  const size_t o_ci = take(12 * citems.size(), 4), o_vi = take(12 * vitems.size(), 4), o_mi = take(8 * mitems.size(), 8);
  const size_t plan_cap = h->plan_limit ? std::min(h->plan_limit, s.plan_words) : s.plan_words;
  if (w > plan_cap) {
    undo_rollback(h);
    return fail(h, HAT_EINVAL, "internal: plan of %zu words exceeds capacity %zu", w, plan_cap);
  }
  static_assert(sizeof(HatAttnItem) == 48 && sizeof(HatMergeItem) == 32, "plan item sizes");
  if (!citems.empty()) memcpy(&P[o_ci], citems.data(), citems.size() * sizeof(HatAttnItem));
  if (!vitems.empty()) memcpy(&P[o_vi], vitems.data(), vitems.size() * sizeof(HatAttnItem));
  if (!mitems.empty()) memcpy(&P[o_mi], mitems.data(), mitems.size() * sizeof(HatMergeItem));

  sp->T = T; sp->S = S; sp->n_append = n_append;
  sp->o_pos = o_pos; sp->o_dst = o_dst; sp->o_tseg = o_tseg; sp->o_toff = o_toff; sp->o_sstart = o_sstart;
  sp->o_spt = o_spt; sp->o_in = o_in; sp->o_out = o_out; sp->o_pt = o_pt; sp->o_app = o_app;
  sp->o_ci = o_ci; sp->o_vi = o_vi; sp->o_mi = o_mi; sp->words = w;
  sp->n_citems = (int)citems.size(); sp->n_vitems = (int)vitems.size(); sp->n_mitems = (int)mitems.size();
  return HAT_OK;
}

// Device half of a step: uploads the plan and enqueues the kernels of every layer on st.
static hat_status_t enqueue_step(hat_mid_t* h, const StepPlan& sp, const int32_t* P, int bi, hipStream_t st) {
  const hat_mid_config_t& c = h->cfg;
  const Shapes& s = h->s;
  const int T = sp.T, S = sp.S, n_append = sp.n_append;
  const size_t o_pos = sp.o_pos, o_dst = sp.o_dst, o_tseg = sp.o_tseg, o_toff = sp.o_toff, o_sstart = sp.o_sstart;
  const size_t o_spt = sp.o_spt, o_in = sp.o_in, o_out = sp.o_out, o_pt = sp.o_pt, o_app = sp.o_app;
  const size_t o_ci = sp.o_ci, o_vi = sp.o_vi, o_mi = sp.o_mi, w = sp.words;

  HIP_TRY(h, hipEventRecord(h->ev_begin, st));
  HIP_TRY(h, hipMemcpyAsync(h->b.plan_dev, P, w * sizeof(int32_t), hipMemcpyHostToDevice, st));
  HIP_TRY(h, hipEventRecord(h->plan_ev[bi], st));
  h->plan_ev_used[bi] = true;

  const int32_t* D = h->b.plan_dev;
  HatPlanDev pd;
  pd.T = T; pd.S = S;
  pd.pos = D + o_pos; pd.kv_dst = D + o_dst; pd.tok_seg = D + o_tseg; pd.tok_off = D + o_toff;
  pd.seg_start = D + o_sstart; pd.seg_pt = D + o_spt; pd.page_tbl = D + o_pt;
  pd.in_ptr = (const uint64_t*)(D + o_in); pd.out_ptr = (const uint64_t*)(D + o_out);
  pd.append = (const HatAppendItem*)(D + o_app); pd.n_append = n_append;

  LAUNCH(h, st, HAT_K_GATHER, hat_launch_gather(pd, h->b.resid, s.d, c.io_dtype, st));
  LAUNCH(h, st, HAT_K_ROPE_APPEND, hat_launch_rope_table(pd, h->b.inv_freq, h->b.table, s.hd / 2, st));

  int nparts = 0;  // split-K partial sums of the previous residual GEMM still to be folded in
  auto run_gemm = [&](int id, HatGemm& g, int* ksplit_out) -> hat_status_t {
    const int cls = id == HAT_K_GEMM_QKV ? 0 : id == HAT_K_GEMM_O ? 1 : id == HAT_K_GEMM_GATEUP ? 2 : 3;
    g.force_tile = h->force_tile[cls];
    g.force_ksplit = h->force_ksplit[cls];
    const HatGemmPlan gp = hat_gemm_plan(g);
    if (ksplit_out) *ksplit_out = gp.ksplit;
    LAUNCH(h, st, id, hat_launch_gemm(g, gp, st));
    return HAT_OK;
  };
  for (int l = 0; l < s.L; ++l) {
    const LayerDev& ld = h->b.layers[l];
    kv_t* pool_l = h->pool + (size_t)l * h->layer_pool_elems;
    LAUNCH(h, st, HAT_K_RMSNORM,
           hat_launch_rmsnorm(h->b.resid, h->b.gemm_part, nparts, ld.g_attn, h->b.xn, T, s.d, c.rms_eps, st));
    nparts = 0;
    HatGemm g{};
    g.W = ld.wqkv; g.X = h->b.xn; g.K = s.d; g.T = T; g.Nw = s.Nqkv; g.Nout = 3 * s.d; g.outP = h->b.qkv;
    g.epilogue = HAT_EPI_P32;
    hat_status_t rc = run_gemm(HAT_K_GEMM_QKV, g, nullptr);
    if (rc != HAT_OK) return rc;
    LAUNCH(h, st, HAT_K_ROPE_APPEND, hat_launch_rope_append(pd, h->b.qkv, h->b.table, pool_l, c.n_pages, s.H, s.hd, c.kv_dtype == HAT_KV_F16, st));
    HatAttn a{};
    a.qkv = h->b.qkv; a.pool_layer = pool_l; a.outP = h->b.attn; a.part_o = h->b.part_o; a.part_ml = h->b.part_ml;
    a.H = s.H; a.hd = s.hd; a.d = s.d; a.n_pages = c.n_pages; a.kv_f16 = c.kv_dtype == HAT_KV_F16;
    if (sp.n_citems > 0) {
      a.items = (const HatAttnItem*)(D + o_ci); a.n_items = sp.n_citems;
      LAUNCH(h, st, HAT_K_ATTN_CHUNK, hat_launch_attn_chunk(pd, a, st));
    }
    if (sp.n_vitems > 0) {
      a.items = (const HatAttnItem*)(D + o_vi); a.n_items = sp.n_vitems;
      if (h->verify_probe)
        LAUNCH(h, st, HAT_K_ATTN_VERIFY, hat_launch_attn_verify_probe(pd, a, (uint32_t*)h->b.fixture_pages, st));
      else
        LAUNCH(h, st, HAT_K_ATTN_VERIFY, hat_launch_attn_verify(pd, a, st));
    }
    if (sp.n_mitems > 0)
      LAUNCH(h, st, HAT_K_ATTN_MERGE, hat_launch_attn_merge(a, (const HatMergeItem*)(D + o_mi), sp.n_mitems, st));
    g = HatGemm{};
    g.W = ld.wo; g.X = h->b.attn; g.K = s.d; g.T = T; g.Nw = s.No; g.Nout = s.d; g.resid = h->b.resid;
    g.part = h->b.gemm_part; g.part_rows = s.gemm_part_rows;
    g.epilogue = HAT_EPI_RESID;
    int ks = 1;
    if ((rc = run_gemm(HAT_K_GEMM_O, g, &ks)) != HAT_OK) return rc;
    nparts = ks > 1 ? ks : 0;
    LAUNCH(h, st, HAT_K_RMSNORM,
           hat_launch_rmsnorm(h->b.resid, h->b.gemm_part, nparts, ld.g_ffn, h->b.xn2, T, s.d, c.rms_eps, st));
    nparts = 0;
    g = HatGemm{};
    g.W = ld.wgu; g.X = h->b.xn2; g.K = s.d; g.T = T; g.Nw = s.Ngu; g.Nout = s.Fpad; g.outP = h->b.act;
    g.epilogue = HAT_EPI_SWIGLU;
    if ((rc = run_gemm(HAT_K_GEMM_GATEUP, g, nullptr)) != HAT_OK) return rc;
    g = HatGemm{};
    g.W = ld.wd; g.X = h->b.act; g.K = s.Fpad; g.T = T; g.Nw = s.Nd; g.Nout = s.d; g.resid = h->b.resid;
    g.part = h->b.gemm_part; g.part_rows = s.gemm_part_rows;
    g.epilogue = HAT_EPI_RESID;
    if ((rc = run_gemm(HAT_K_GEMM_DOWN, g, &ks)) != HAT_OK) return rc;
    nparts = ks > 1 ? ks : 0;
  }
  LAUNCH(h, st, HAT_K_SCATTER, hat_launch_scatter(pd, h->b.resid, h->b.gemm_part, nparts, s.d, c.io_dtype, st));
  HIP_TRY(h, hipEventRecord(h->ev_end, st));
  h->have_step = true;
  h->last_tokens = T;
  return HAT_OK;
}

static hat_status_t forward_impl(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, void* hip_stream) {
  if (!h) return HAT_EINVAL;
  if (n_segs == 0) return HAT_OK;  // an empty step: no work, no state change
  if (h->host_only) return fail(h, HAT_EINVAL, "a host-only handle plans steps, it does not run them");
  hipStream_t st = (hipStream_t)hip_stream;
  // the pinned plan buffers rotate; this one was last read by the upload of three steps ago
  const int bi = h->plan_next;
  if (h->plan_ev_used[bi]) HIP_TRY(h, hipEventSynchronize(h->plan_ev[bi]));
  int32_t* P = h->plan_host[bi];
  StepPlan sp;
  const hat_status_t prc = plan_step(h, segs, n_segs, P, &sp);
  if (prc != HAT_OK) return prc;   // nothing moved (plan_step undoes its own page movements)
  note_stream(h, st);
  const hat_status_t erc = enqueue_step(h, sp, P, bi, st);
  if (erc != HAT_OK) {
    // a HIP call failed part-way: lengths and pages go back to where they were; kernels already
    // enqueued may still write cache rows at or beyond the segments' start positions
    undo_rollback(h);
    return erc;
  }
  undo_commit(h);
  h->plan_next = (bi + 1) % kPlanBufs;
  return HAT_OK;
}

// No exception crosses the ABI: the entry points that allocate host memory (vectors, the handle)
// turn an allocation failure into a status.
hat_status_t hat_mid_create(const hat_mid_config_t* cfg, const hat_mid_layer_weights_t* layers, void* kv_pool,
                            void* workspace, void* hip_stream, hat_mid_t** out) {
  try {
    return create_impl(cfg, layers, kv_pool, workspace, hip_stream, out);
  } catch (...) {
    if (out) *out = nullptr;
    return HAT_EHIP;
  }
}

hat_status_t hat_mid_forward(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, void* hip_stream) {
  try {
    return forward_impl(h, segs, n_segs, hip_stream);
  } catch (...) {
    if (h && h->undo_on) undo_rollback(h);
    return fail(h, HAT_EHIP, "host allocation failed while planning the step");
  }
}

hat_status_t hat_mid_last_step_stats(hat_mid_t* h, int32_t* tokens, float* gpu_ms) {
  if (!h) return HAT_EINVAL;
  if (!h->have_step) return fail(h, HAT_EINVAL, "no step has run yet");
  HIP_TRY(h, hipEventSynchronize(h->ev_end));
  float ms = 0.f;
  HIP_TRY(h, hipEventElapsedTime(&ms, h->ev_begin, h->ev_end));
  if (tokens) *tokens = h->last_tokens;
  if (gpu_ms) *gpu_ms = ms;
  return HAT_OK;
}

hat_status_t hat_mid_set_profiling(hat_mid_t* h, int32_t on) {
  if (!h) return HAT_EINVAL;
  if (h->host_only) return fail(h, HAT_EINVAL, "a host-only handle has no GPU side");
  h->profiling = on != 0;
  return HAT_OK;
}

hat_status_t hat_mid_kernel_times(hat_mid_t* h, float* ms, int32_t* launches) {
  if (!h || !ms || !launches) return HAT_EINVAL;
  for (int i = 0; i < HAT_K_COUNT; ++i) { ms[i] = 0.f; launches[i] = 0; }
  for (auto& r : h->recs) {
    HIP_TRY(h, hipEventSynchronize(r.b));
    float t = 0.f;
    HIP_TRY(h, hipEventElapsedTime(&t, r.a, r.b));
    ms[r.id] += t;
    launches[r.id] += 1;
    h->ev_pool.push_back(r.a);
    h->ev_pool.push_back(r.b);
  }
  h->recs.clear();
  return HAT_OK;
}

static hat_status_t fixture_pages(hat_mid_t* h, const DeviceState& d, int pos0, int n, hipStream_t st) {
  const int p0 = pos0 >> 4, p1 = (pos0 + n - 1) >> 4;
  HIP_TRY(h, hipStreamSynchronize(st));  // the staging area below is reused by every fixture call
  HIP_TRY(h, hipMemcpy(h->b.fixture_pages, d.pages.data() + p0, (size_t)(p1 - p0 + 1) * sizeof(int32_t),
                       hipMemcpyHostToDevice));
  return HAT_OK;
}

static hat_status_t forward_host_impl(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, void* hip_stream) {
  if (!h) return HAT_EINVAL;
  if (h->host_only) return fail(h, HAT_EINVAL, "a host-only handle has no GPU side");
  if (n_segs == 0) return HAT_OK;
  if (!segs || n_segs < 0) return fail(h, HAT_EINVAL, "no segments");
  if (n_segs > h->cfg.max_devices) return fail(h, HAT_EINVAL, "more segments (%d) than devices", n_segs);
  const Shapes& s = h->s;
  const size_t rowb = (size_t)s.d * (h->cfg.io_dtype == HAT_F32 ? 4 : 2);
  long total = 0;
  for (int i = 0; i < n_segs; ++i) {
    if (segs[i].n <= 0 || !segs[i].hidden_in || !segs[i].hidden_out)
      return fail(h, HAT_EINVAL, "segment %d: n = %d or a null host pointer", i, segs[i].n);
    total += segs[i].n;
  }
  if (total > s.Tcap) return fail(h, HAT_EINVAL, "step of %ld rows exceeds max_step_tokens %d", total, s.Tcap);
  hipStream_t st = (hipStream_t)hip_stream;
  const int slot = h->host_slot;
  h->host_slot ^= 1;
  // this input slot was last read by the step two calls back
  if (h->slot_used[slot]) HIP_TRY(h, hipStreamWaitEvent(h->copy_stream, h->slot_free[slot], 0));
  std::vector<hat_mid_segment_t> dsegs(segs, segs + n_segs);
  unsigned char* in = (unsigned char*)h->b.stage_in[slot];
  unsigned char* out = (unsigned char*)h->b.stage_out;
  size_t off = 0;
  for (int i = 0; i < n_segs; ++i) {
    const size_t nb = (size_t)segs[i].n * rowb;
    HIP_TRY(h, hipMemcpyAsync(in + off, segs[i].hidden_in, nb, hipMemcpyHostToDevice, h->copy_stream));
    dsegs[i].hidden_in = in + off;
    dsegs[i].hidden_out = out + off;
    off += nb;
  }
  HIP_TRY(h, hipEventRecord(h->up_done[slot], h->copy_stream));
  HIP_TRY(h, hipStreamWaitEvent(st, h->up_done[slot], 0));
  const hat_status_t rc = forward_impl(h, dsegs.data(), n_segs, hip_stream);
  HIP_TRY(h, hipEventRecord(h->slot_free[slot], st));
  h->slot_used[slot] = true;
  if (rc != HAT_OK) return rc;
  off = 0;
  for (int i = 0; i < n_segs; ++i) {
    const size_t nb = (size_t)segs[i].n * rowb;
    HIP_TRY(h, hipMemcpyAsync(segs[i].hidden_out, out + off, nb, hipMemcpyDeviceToHost, st));
    off += nb;
  }
  return HAT_OK;
}

hat_status_t hat_mid_forward_host(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, void* hip_stream) {
  try {
    return forward_host_impl(h, segs, n_segs, hip_stream);
  } catch (...) {
    if (h && h->undo_on) undo_rollback(h);
    return fail(h, HAT_EHIP, "host allocation failed while planning the step");
  }
}

hat_status_t hat_mid_kv_import(hat_mid_t* h, int32_t device_id, int32_t layer, int32_t pos0, int32_t n, const void* k,
                               const void* v, void* hip_stream) {
  if (!h) return HAT_EINVAL;
  if (h->host_only) return fail(h, HAT_EINVAL, "a host-only handle has no GPU side");
  const hat_mid_config_t& c = h->cfg;
  if (device_id < 0 || device_id >= c.max_devices) return fail(h, HAT_EDEVICE, "device id %d out of range", device_id);
  if (layer < 0 || layer >= c.n_layers || n <= 0 || pos0 < 0 || !k || !v) return fail(h, HAT_EINVAL, "bad import arguments");
  if ((long)pos0 + n > c.max_pos) return fail(h, HAT_EINVAL, "import beyond max_pos");
  DeviceState& d = h->dev[device_id];
  if (pos0 > d.len) return fail(h, HAT_EPOS, "import at %d beyond cache length %d", pos0, d.len);
  const size_t want = (size_t)(pos0 + n + 15) / 16;
  if (want > d.pages.size() && want - d.pages.size() > h->free_pages.size())
    return fail(h, HAT_ENOMEM, "KV pool exhausted on import");
  undo_begin(h);
  undo_save_device(h, device_id);
  while (d.pages.size() < want) d.pages.push_back(take_lowest(h));
  d.len = std::max(d.len, pos0 + n);
  hipStream_t st = (hipStream_t)hip_stream;
  note_stream(h, st);
  hat_status_t rc = fixture_pages(h, d, pos0, n, st);
  if (rc == HAT_OK) {
    const hipError_t e = hat_launch_kv_import(h->pool + (size_t)layer * h->layer_pool_elems, c.n_pages, h->b.fixture_pages,
                                              pos0, n, (const bf16_t*)k, (const bf16_t*)v, c.n_heads, c.head_dim, c.kv_dtype == HAT_KV_F16, st);
    if (e != hipSuccess) rc = fail(h, HAT_EHIP, "kv import launch failed: %s", hipGetErrorString(e));
  }
  if (rc != HAT_OK) {
    undo_rollback(h);   // the pages taken for this import return to the pool, the length is as before
    return rc;
  }
  undo_commit(h);
  return HAT_OK;
}

hat_status_t hat_mid_kv_export(hat_mid_t* h, int32_t device_id, int32_t layer, int32_t pos0, int32_t n, void* k,
                               void* v, void* hip_stream) {
  if (!h) return HAT_EINVAL;
  if (h->host_only) return fail(h, HAT_EINVAL, "a host-only handle has no GPU side");
  const hat_mid_config_t& c = h->cfg;
  if (device_id < 0 || device_id >= c.max_devices) return fail(h, HAT_EDEVICE, "device id %d out of range", device_id);
  if (layer < 0 || layer >= c.n_layers || n <= 0 || pos0 < 0 || !k || !v) return fail(h, HAT_EINVAL, "bad export arguments");
  const DeviceState& d = h->dev[device_id];
  if (pos0 + n > d.len) return fail(h, HAT_EPOS, "export of rows %d..%d beyond cache length %d", pos0, pos0 + n, d.len);
  hipStream_t st = (hipStream_t)hip_stream;
  note_stream(h, st);
  hat_status_t rc = fixture_pages(h, d, pos0, n, st);
  if (rc != HAT_OK) return rc;
  HIP_TRY(h, hat_launch_kv_export(h->pool + (size_t)layer * h->layer_pool_elems, c.n_pages, h->b.fixture_pages, pos0, n,
                                  (bf16_t*)k, (bf16_t*)v, c.n_heads, c.head_dim, c.kv_dtype == HAT_KV_F16, st));
  return HAT_OK;
}

hat_status_t hat_mid_kv_export_static(hat_mid_t* h, int32_t device_id, int32_t layer, int32_t pos0, int32_t n, void* k,
                                      void* v, void* hip_stream) {
  if (!h) return HAT_EINVAL;
  if (h->host_only) return fail(h, HAT_EINVAL, "a host-only handle has no GPU side");
  const hat_mid_config_t& c = h->cfg;
  if (device_id < 0 || device_id >= c.max_devices) return fail(h, HAT_EDEVICE, "device id %d out of range", device_id);
  if (layer < 0 || layer >= c.n_layers || n <= 0 || pos0 < 0 || !k || !v) return fail(h, HAT_EINVAL, "bad export arguments");
  const DeviceState& d = h->dev[device_id];
  if ((long)pos0 + n > d.len) return fail(h, HAT_EPOS, "export of rows %d..%ld beyond cache length %d", pos0, (long)pos0 + n, d.len);
  const int p0 = pos0 >> 4, p1 = (pos0 + n - 1) >> 4, np = p1 - p0 + 1;
  if (np > kStaticPageIds)
    return fail(h, HAT_EINVAL, "export of %d rows spans %d pages: the static scratch holds %d page ids (%d rows)", n, np,
                kStaticPageIds, kStaticPageIds * HAT_PAGE_SIZE);
  hipStream_t st = (hipStream_t)hip_stream;
  // the pinned buffer is free again once the previous call's upload has read it
  if (h->static_ev_used) HIP_TRY(h, hipEventSynchronize(h->static_ev));
  memcpy(h->static_pages_host, d.pages.data() + p0, (size_t)np * sizeof(int32_t));
  note_stream(h, st);
  // from here on only the address taken with hipGetSymbolAddress is used for the array
  HIP_TRY(h, hipMemcpyAsync(h->static_pages_dev, h->static_pages_host, (size_t)np * sizeof(int32_t), hipMemcpyHostToDevice, st));
  HIP_TRY(h, hipEventRecord(h->static_ev, st));
  h->static_ev_used = true;
  HIP_TRY(h, hat_launch_kv_export(h->pool + (size_t)layer * h->layer_pool_elems, c.n_pages, h->static_pages_dev, pos0, n,
                                  (bf16_t*)k, (bf16_t*)v, c.n_heads, c.head_dim, c.kv_dtype == HAT_KV_F16, st));
  return HAT_OK;
}

hat_status_t hat_mid_debug_create_host_only(const hat_mid_config_t* cfg, hat_mid_t** out) {
  if (out) *out = nullptr;
  if (!out || !valid_cfg(cfg)) return HAT_EINVAL;
  try {
    hat_mid* h = new hat_mid();
    h->host_only = true;
    h->cfg = *cfg;
    h->s = make_shapes(*cfg);
    h->pool = nullptr;
    h->layer_pool_elems = (size_t)cfg->n_pages * kv_page_elems(cfg->n_heads, cfg->head_dim);
    for (int i = 0; i < cfg->n_pages; ++i) h->free_pages.insert(i);
    h->dev.resize(cfg->max_devices);
    h->host_plan.resize(h->s.plan_words);
    *out = h;
    return HAT_OK;
  } catch (...) {
    return HAT_EHIP;
  }
}

hat_status_t hat_mid_debug_plan(hat_mid_t* h, const hat_mid_segment_t* segs, int32_t n_segs, int32_t* pos,
                                int32_t* kv_dst, int32_t cap_rows, int32_t* chunk_items, int32_t* n_chunk_items,
                                int32_t* verify_items, int32_t* n_verify_items, int32_t* merge_items,
                                int32_t* n_merge_items, int32_t cap_items) {
  if (!h) return HAT_EINVAL;
  if (!h->host_only) return fail(h, HAT_EINVAL, "hat_mid_debug_plan needs a host-only handle");
  if (n_chunk_items) *n_chunk_items = 0;
  if (n_verify_items) *n_verify_items = 0;
  if (n_merge_items) *n_merge_items = 0;
  if (n_segs == 0) return HAT_OK;
  try {
    StepPlan sp;
    const int32_t* P = h->host_plan.data();
    const hat_status_t rc = plan_step(h, segs, n_segs, h->host_plan.data(), &sp);
    if (rc != HAT_OK) return rc;
    undo_commit(h);
    if (sp.T > cap_rows || std::max(sp.n_citems, std::max(sp.n_vitems, sp.n_mitems)) > cap_items)
      return fail(h, HAT_EINVAL, "output arrays too small for %d rows / %d, %d, %d items (the step has been planned)", sp.T,
                  sp.n_citems, sp.n_vitems, sp.n_mitems);
    if (pos) memcpy(pos, P + sp.o_pos, sp.T * sizeof(int32_t));
    if (kv_dst) memcpy(kv_dst, P + sp.o_dst, sp.T * sizeof(int32_t));
    if (chunk_items) memcpy(chunk_items, P + sp.o_ci, (size_t)sp.n_citems * sizeof(HatAttnItem));
    if (verify_items) memcpy(verify_items, P + sp.o_vi, (size_t)sp.n_vitems * sizeof(HatAttnItem));
    if (merge_items) memcpy(merge_items, P + sp.o_mi, (size_t)sp.n_mitems * sizeof(HatMergeItem));
    if (n_chunk_items) *n_chunk_items = sp.n_citems;
    if (n_verify_items) *n_verify_items = sp.n_vitems;
    if (n_merge_items) *n_merge_items = sp.n_mitems;
    return HAT_OK;
  } catch (...) {
    if (h->undo_on) undo_rollback(h);
    return fail(h, HAT_EHIP, "host allocation failed while planning the step");
  }
}

hat_status_t hat_mid_debug_force_gemm(hat_mid_t* h, int32_t which, int32_t tile, int32_t ksplit) {
  if (!h || which < 0 || which > 3) return HAT_EINVAL;
  h->force_tile[which] = tile;
  h->force_ksplit[which] = ksplit;
  return HAT_OK;
}

int32_t hat_mid_debug_gemm_tile_count(void) { return hat_gemm_tile_count(); }

hat_status_t hat_mid_debug_gemm_tile_info(int32_t tile, int32_t* features, int32_t* tokens, int32_t* waves,
                                          int32_t* k_per_stage, int32_t* stages) {
  int bf, bt, w, bk, ns;
  if (!hat_gemm_tile_info(tile, &bf, &bt, &w, &bk, &ns)) return HAT_EINVAL;
  if (features) *features = bf;
  if (tokens) *tokens = bt;
  if (waves) *waves = w;
  if (k_per_stage) *k_per_stage = bk;
  if (stages) *stages = ns;
  return HAT_OK;
}

hat_status_t hat_mid_debug_set_attn_targets(hat_mid_t* h, int32_t chunk_target, int32_t verify_target) {
  if (!h || chunk_target < 0 || verify_target < 0) return HAT_EINVAL;
  if (chunk_target > 0) h->s.attn_target = chunk_target;
  if (verify_target > 0) h->s.verify_target = verify_target;
  return HAT_OK;
}

hat_status_t hat_mid_debug_set_verify_probe(hat_mid_t* h, int32_t on) {
  if (!h) return HAT_EINVAL;
  if (h->host_only) return fail(h, HAT_EINVAL, "a host-only handle has no GPU side");
  h->verify_probe = on != 0;
  return HAT_OK;
}

hat_status_t hat_mid_debug_limit_plan(hat_mid_t* h, int64_t max_words) {
  if (!h || max_words < 0) return HAT_EINVAL;
  h->plan_limit = (size_t)max_words;
  return HAT_OK;
}

hat_status_t hat_mid_debug_gemm_plan(int32_t T, int32_t Nw, int32_t Nout, int32_t K, int32_t epilogue,
                                     int32_t part_rows, int32_t* tile, int32_t* ksplit) {
  if (!tile || !ksplit) return HAT_EINVAL;
  HatGemm g{};
  static float dummy;   // only its non-nullness is looked at
  g.T = T; g.Nw = Nw; g.Nout = Nout; g.K = K; g.epilogue = epilogue;
  g.part = part_rows > 0 ? &dummy : nullptr;
  g.part_rows = part_rows;
  g.force_tile = -1;
  const HatGemmPlan p = hat_gemm_plan(g);
  *tile = p.tile;
  *ksplit = p.ksplit;
  return HAT_OK;
}

hat_status_t hat_mid_debug_dump(hat_mid_t* h, int32_t which, void* dst, void* hip_stream) {
  if (!h || !dst) return HAT_EINVAL;
  if (!h->have_step) return fail(h, HAT_EINVAL, "no step has run yet");
  const Shapes& s = h->s;
  hipStream_t st = (hipStream_t)hip_stream;
  const int T = h->last_tokens;
  switch (which) {
    case HAT_DUMP_XNORM: HIP_TRY(h, hat_launch_unpack_p32(h->b.xn, s.d, 0, s.d, T, (float*)dst, st)); break;
    case HAT_DUMP_Q: HIP_TRY(h, hat_launch_unpack_p32(h->b.qkv, 3 * s.d, 0, s.d, T, (float*)dst, st)); break;
    case HAT_DUMP_ATTN: HIP_TRY(h, hat_launch_unpack_p32(h->b.attn, s.d, 0, s.d, T, (float*)dst, st)); break;
    case HAT_DUMP_XNORM2: HIP_TRY(h, hat_launch_unpack_p32(h->b.xn2, s.d, 0, s.d, T, (float*)dst, st)); break;
    case HAT_DUMP_ACT: HIP_TRY(h, hat_launch_unpack_p32(h->b.act, s.Fpad, 0, s.F, T, (float*)dst, st)); break;
    default: return fail(h, HAT_EINVAL, "unknown dump id %d", which);
  }
  return HAT_OK;
}

}  // extern "C"
