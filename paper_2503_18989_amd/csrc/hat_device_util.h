// Device-side helpers shared by the hand-scheduled kernels: compile-time loops, LDS
// operand reads issued from inline asm (so that their waits can be placed by hand) and
// the waits that go with them.
#ifndef HAT_DEVICE_UTIL_H
#define HAT_DEVICE_UTIL_H
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

typedef _Float16 hat_f16x8 __attribute__((ext_vector_type(8)));

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <class F, int... I>
__device__ __forceinline__ void hat_static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void hat_static_for(F&& f) {
  hat_static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// 16 bytes per lane from LDS at addr + OFF (an immediate, 16 bits)
template <int OFF>
__device__ __forceinline__ hat_f16x8 hat_lds_read(uint32_t addr) {
  static_assert(OFF >= 0 && OFF < 65536, "ds_read offset field is 16 bits");
  hat_f16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
// "operands have arrived": the wait is tied to the first register, the others are
// threaded through empty asm statements (volatile asm keeps its order) so that no
// MFMA using them can be scheduled above the wait.
template <int N>
__device__ __forceinline__ void hat_wait_operands(hat_f16x8 (&v)[N]) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(v[0]));
#pragma unroll
  for (int i = 1; i < N; ++i) asm volatile("" : "+v"(v[i]));
}
template <int N>
__device__ __forceinline__ void hat_wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
#endif
