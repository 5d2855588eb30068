// Runs the library's step planner (host code of api.hip) under AddressSanitizer +
// UndefinedBehaviorSanitizer through a host-only handle: random traffic of chunks, chains with
// rollback, trees with compaction, departures and malformed steps.  The kernels' launch functions
// are stubbed out here -- a host-only handle never reaches them -- so that only api.hip is built.
// Exit status 0 = every call returned a status the header allows and the sanitizers saw nothing.
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../include/hat_mid.h"
#include "../paper_2503_18989_amd/csrc/hat_kernels.h"

HatGemmPlan hat_gemm_plan(const HatGemm&) { return HatGemmPlan{0, 1}; }
hipError_t hat_launch_gemm(const HatGemm&, const HatGemmPlan&, hipStream_t) { return hipErrorUnknown; }
int hat_gemm_tile_count() { return 0; }
bool hat_gemm_tile_info(int, int*, int*, int*, int*, int*) { return false; }
hipError_t hat_gemm_init() { return hipErrorUnknown; }
hipError_t hat_launch_retile(act_t*, int, int, const bf16_t*, const bf16_t*, const bf16_t*, int, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_bf16_to_f32(const bf16_t*, float*, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_gather(const HatPlanDev&, float*, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_scatter(const HatPlanDev&, const float*, const float*, int, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_rope_table(const HatPlanDev&, const double*, float2*, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_rmsnorm(float*, const float*, int, const float*, act_t*, int, int, float, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_rope_append(const HatPlanDev&, act_t*, const float2*, kv_t*, int, int, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_attn_chunk(const HatPlanDev&, const HatAttn&, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_attn_verify(const HatPlanDev&, const HatAttn&, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_attn_merge(const HatAttn&, const HatMergeItem*, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_attn_verify_probe(const HatPlanDev&, const HatAttn&, uint32_t*, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_kv_import(kv_t*, int, const int32_t*, int, int, const bf16_t*, const bf16_t*, int, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_kv_move(kv_t*, size_t, int, int, const HatRowMoves&, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_kv_export(const kv_t*, int, const int32_t*, int, int, bf16_t*, bf16_t*, int, int, int, hipStream_t) { return hipErrorUnknown; }
hipError_t hat_launch_unpack_p32(const act_t*, int, int, int, int, float*, hipStream_t) { return hipErrorUnknown; }

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main() {
  hat_mid_config_t cfg{};
  cfg.n_layers = 30; cfg.d_model = 4096; cfg.n_heads = 32; cfg.head_dim = 128; cfg.d_ffn = 11008;
  cfg.rms_eps = 1e-6f; cfg.rope_theta = 1e4f; cfg.page_size = 16; cfg.n_pages = 3000; cfg.max_devices = 12;
  cfg.max_step_tokens = 4096; cfg.max_pos = 6000; cfg.io_dtype = HAT_BF16;
  hat_mid_t* h = nullptr;
  CHECK(hat_mid_debug_create_host_only(nullptr, &h) == HAT_EINVAL && h == nullptr);
  CHECK(hat_mid_debug_create_host_only(&cfg, &h) == HAT_OK && h != nullptr);
  uint64_t state = 777;
  auto rnd = [&](int n) { state = state * 6364136223846793005ull + 1442695040888963407ull; return (int)((state >> 33) % (uint64_t)n); };
  const int cap_rows = 4096, cap_items = 1024;
  std::vector<int32_t> pos(cap_rows), dst(cap_rows), ci(12 * cap_items), vi(12 * cap_items), mi(8 * cap_items);
  std::vector<int> len(cfg.max_devices, 0);
  int dummy = 0, ok_steps = 0, bad_steps = 0;
  for (int step = 0; step < 400; ++step) {
    std::vector<hat_mid_segment_t> segs;
    std::vector<std::vector<uint8_t>> masks(cfg.max_devices);
    int rows = 0;
    const bool poison = rnd(10) == 0;       // now and then a malformed step
    for (int d = 0; d < cfg.max_devices; ++d) {
      if (rnd(3) == 0) continue;
      if (len[d] + 1100 > cfg.max_pos || rnd(20) == 0) { CHECK(hat_mid_release(h, d) == HAT_OK); len[d] = 0; continue; }
      hat_mid_segment_t s{};
      s.device_id = d; s.hidden_in = &dummy; s.hidden_out = &dummy;
      const int r = rnd(3);
      if (len[d] == 0 || r == 0) { s.kind = HAT_SEG_CHUNK; s.start_pos = len[d]; s.n = 1 + rnd(700); }
      else if (r == 1) { s.kind = HAT_SEG_VERIFY; const int back = rnd(5) < len[d] ? rnd(5) : 0; s.start_pos = len[d] - back; s.n = 1 + rnd(8); }
      else {
        s.kind = HAT_SEG_VERIFY; s.start_pos = len[d]; s.n = 1 + rnd(8);
        masks[d].resize(s.n);
        for (int i = 0; i < s.n; ++i) { const int p = rnd(i + 1) - 1; masks[d][i] = (uint8_t)((1u << i) | (p >= 0 ? masks[d][p] : 0)); }
        s.tree_mask = masks[d].data();
      }
      if (rows + s.n > cfg.max_step_tokens) continue;
      rows += s.n;
      segs.push_back(s);
    }
    if (poison && !segs.empty()) {
      hat_mid_segment_t& s = segs[rnd((int)segs.size())];
      switch (rnd(5)) {
        case 0: s.start_pos += 3; break;                 // a gap
        case 1: s.n = 0; break;
        case 2: s.device_id = cfg.max_devices; break;
        case 3: s.kind = HAT_SEG_VERIFY; s.n = 9; s.tree_mask = nullptr; break;
        default: s.hidden_in = nullptr; break;
      }
    }
    int32_t nc = 0, nv = 0, nm = 0;
    const hat_status_t rc = hat_mid_debug_plan(h, segs.data(), (int32_t)segs.size(), pos.data(), dst.data(), cap_rows, ci.data(),
                                               &nc, vi.data(), &nv, mi.data(), &nm, cap_items);
    if (rc == HAT_OK) {
      ++ok_steps;
      for (const hat_mid_segment_t& s : segs) len[s.device_id] = s.start_pos + s.n;
      for (const hat_mid_segment_t& s : segs)
        if (s.tree_mask && rnd(2)) {                     // keep a path of the tree: ascending indices
          std::vector<int32_t> keep;
          for (int i = 0; i < s.n; ++i) if (rnd(3) == 0) keep.push_back(i);
          CHECK(hat_mid_kv_compact(h, s.device_id, s.start_pos, keep.data(), (int32_t)keep.size(), nullptr) == HAT_OK);
          len[s.device_id] = s.start_pos + (int)keep.size();
        }
    } else {
      ++bad_steps;
      CHECK(rc == HAT_EINVAL || rc == HAT_EPOS || rc == HAT_EDEVICE || rc == HAT_ENOMEM || rc == HAT_EDUP);
      CHECK(hat_mid_last_error(h)[0] != 0);
    }
    for (int d = 0; d < cfg.max_devices; ++d) {
      int32_t l = -1, np = -1;
      CHECK(hat_mid_kv_query(h, d, &l, nullptr, 0, &np) == HAT_OK && l == len[d] && np == (len[d] + 15) / 16);
    }
  }
  CHECK(hat_mid_forward(h, nullptr, 1, nullptr) == HAT_EINVAL);   // a host-only handle runs nothing
  hat_mid_destroy(h);
  CHECK(ok_steps > 200 && bad_steps > 10);
  std::printf("planner sanitizer driver: ok (%d steps planned, %d rejected)\n", ok_steps, bad_steps);
  return 0;
}
