// Helpers shared by the GEMM kernels that stage their operands in LDS with asynchronous global -> LDS
// copies (csrc/fg_gemm_stream.hip, csrc/fg_gemm_f16w.hip).
#pragma once
#include "fg_common.h"

namespace fg {
namespace {

// first unit of workgroup p when `total` units are cut into `grid` equal contiguous ranges
__device__ __forceinline__ int64_t work_begin(int64_t total, int grid, int p) { return (total * p) / grid; }
__device__ __forceinline__ int swz(int row, int kc) { return kc ^ ((row >> 1) & 7); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// The compiler orders every LDS read it can see behind ALL outstanding asynchronous global -> LDS
// copies (it cannot tell which copy an address belongs to), which would drain the prefetch queue on
// every step.  The stages are therefore read with hand-placed ds_read instructions; the explicit
// vmcnt wait plus the barrier at the top of each step are what make the data visible.
template <int OFF>
__device__ __forceinline__ u4_t lds_read128(uint32_t addr) {
  u4_t r;
  __asm__ volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
template <int OFF>
__device__ __forceinline__ float2 lds_read64(uint32_t addr) {
  float2 r;
  __asm__ volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
template <int OFF>
__device__ __forceinline__ uint32_t lds_read32(uint32_t addr) {
  uint32_t r;
  __asm__ volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// all ds_reads issued so far have landed
__device__ __forceinline__ void lds_wait() { __asm__ volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// makes later uses of v depend on a point after the preceding lds_wait()
template <class T>
__device__ __forceinline__ void lds_landed(T& v) {
  __asm__ volatile("" : "+v"(v));
}
template <int I>
struct IdxC {
  static constexpr int value = I;
};
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(IdxC<B>{});
    static_for<B + 1, E>(f);
  }
}

}  // namespace
}  // namespace fg
