// Microbenchmarks of what this chip delivers through the instruction mixes the kernels of this
// library are built from: streaming reads (plain and non-temporal), a copy, a matrix-core-only
// loop, and the direct-to-LDS load path from cache-resident data.  They give the "measured peak"
// next to the published one when a kernel's roofline fraction is read, and are reached through
// hat_mid_debug_peak (include/hat_mid.h); bench.py --peaks prints them.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "../../include/hat_mid.h"

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;

// Every wave owns a contiguous span and reads it in steps of 16 KB (16 loads of 16 bytes per lane in
// flight, as the verify-attention kernel keeps per wave); the XOR of what it read is stored only if it
// equals a value that the data never produces, so the loads cannot be dropped.
template <bool NT>
__global__ __launch_bounds__(kThreads) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink) {
  constexpr int INFLIGHT = 16;
  u32x4 acc = {0, 0, 0, 0};
  const int lane = threadIdx.x & 63;
  const size_t waves = (size_t)gridDim.x * (kThreads / 64);
  const size_t wave = (size_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  const size_t steps = n16 / (64 * INFLIGHT);                     // 16 KB steps in the whole buffer
  const size_t s0 = steps * wave / waves, s1 = steps * (wave + 1) / waves;
  for (size_t s = s0; s < s1; ++s) {
    const u32x4* p = src + s * (64 * INFLIGHT) + lane;
    u32x4 v[INFLIGHT];
#pragma unroll
    for (int u = 0; u < INFLIGHT; ++u) v[u] = NT ? __builtin_nontemporal_load(p + u * 64) : p[u * 64];
#pragma unroll
    for (int u = 0; u < INFLIGHT; ++u) acc ^= v[u];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && acc[1] == 0x7f4a7c15u) *sink = 1;
}

__global__ __launch_bounds__(kThreads) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// matrix cores only: every wave keeps NACC independent 32x32x16 fp16 MFMA chains going
template <int NACC>
__global__ __launch_bounds__(kThreads) void mfma_kernel(int iters, float* sink) {
  f32x16 acc[NACC];
#pragma unroll
  for (int a = 0; a < NACC; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
  f16x8 x, y;
#pragma unroll
  for (int e = 0; e < 8; ++e) { x[e] = (_Float16)(0.001f * (threadIdx.x + e)); y[e] = (_Float16)(0.002f * (e + 1)); }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int a = 0; a < NACC; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, acc[a], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < NACC; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[a][r];
  if (s == 12345.678f) *sink = s;
}

// direct-to-LDS loads (16 bytes per lane, 1 KB per wave instruction) from a region small enough
// to stay in cache: what one compute unit can pull through its load path.  Each wave keeps 16
// loads in flight into its own 16 KB of LDS (the oldest is waited for before the next is issued);
// nothing is read back from LDS.
__global__ __launch_bounds__(kThreads) void lds_load_kernel(const unsigned char* __restrict__ src, size_t region_bytes, int iters) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const size_t pieces = region_bytes / 1024;
  size_t p = ((size_t)blockIdx.x * 4 + wave) % pieces;
  auto load = [&](int slot) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + p * 1024 + lane * 16),
                                     (__attribute__((address_space(3))) void*)(lds + (wave * 16 + slot) * 1024), 16, 0, 0);
    p += 37;                       // another piece each time, all of them inside the region
    if (p >= pieces) p -= pieces;
  };
#pragma unroll
  for (int u = 0; u < 16; ++u) load(u);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      asm volatile("s_waitcnt vmcnt(15)" ::: "memory");
      load(u);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

}  // namespace

extern "C" hat_status_t hat_mid_debug_peak(int32_t kind, void* buf, size_t bytes, int32_t iters, void* hip_stream,
                                           double* rate) {
  if (!rate || iters <= 0 || iters > 1000) return HAT_EINVAL;
  *rate = 0.0;
  hipStream_t st = (hipStream_t)hip_stream;
  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return HAT_EHIP;
  const int cus = prop.multiProcessorCount;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return HAT_EHIP;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return HAT_EHIP; }
  hat_status_t rc = HAT_OK;
  double work = 0.0;   // bytes or flops of one launch
  auto launch = [&]() -> bool {
    switch (kind) {
      case HAT_PEAK_STREAM_READ:
      case HAT_PEAK_STREAM_READ_NT: {
        if (!buf || bytes < (1u << 20) || ((uintptr_t)buf & 15)) return false;
        const size_t n16 = (bytes - 256) / 16;
        uint32_t* sink = (uint32_t*)((unsigned char*)buf + n16 * 16);
        if (kind == HAT_PEAK_STREAM_READ) stream_read_kernel<false><<<cus * 8, kThreads, 0, st>>>((const u32x4*)buf, n16, sink);
        else stream_read_kernel<true><<<cus * 8, kThreads, 0, st>>>((const u32x4*)buf, n16, sink);
        work = (double)n16 * 16;
        return true;
      }
      case HAT_PEAK_COPY: {
        if (!buf || bytes < (2u << 20) || ((uintptr_t)buf & 15)) return false;
        const size_t n16 = bytes / 32;
        copy_kernel<<<cus * 8, kThreads, 0, st>>>((const u32x4*)buf, (u32x4*)buf + n16, n16);
        work = (double)n16 * 32;   // read + write
        return true;
      }
      case HAT_PEAK_MFMA_F16: {
        if (!buf || bytes < 256) return false;
        const int loops = 4096;
        mfma_kernel<8><<<cus * 2, kThreads, 0, st>>>(loops, (float*)buf);   // two workgroups = two waves per SIMD
        work = (double)cus * 2 * 4 * loops * 8 * (2.0 * 32 * 32 * 16);
        return true;
      }
      case HAT_PEAK_LDS_LOAD: {
        if (!buf || bytes < (1u << 20)) return false;
        const int loops = 256;
        const size_t region = 1u << 20;   // 1 MB: stays in every L2
        lds_load_kernel<<<cus, kThreads, 64 * 1024, st>>>((const unsigned char*)buf, region, loops);
        work = (double)cus * 4 * (loops + 1) * 16 * 1024;
        return true;
      }
      default: return false;
    }
  };
  if (!launch() || hipGetLastError() != hipSuccess) rc = HAT_EINVAL;   // also the warm-up
  if (rc == HAT_OK) {
    if (hipEventRecord(e0, st) != hipSuccess) rc = HAT_EHIP;
    for (int i = 0; i < iters && rc == HAT_OK; ++i)
      if (!launch() || hipGetLastError() != hipSuccess) rc = HAT_EHIP;
    if (rc == HAT_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess)) rc = HAT_EHIP;
    float ms = 0.f;
    if (rc == HAT_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = HAT_EHIP;
    if (rc == HAT_OK && ms > 0.f) *rate = work * iters / (ms * 1e-3);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}
