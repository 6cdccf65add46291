// Device helpers shared by the kernel files (kernels_bf16.hip, kernels_xcache.hip, kernels_generic.hip): vector types,
// the clamped sequence length, the in-register 8 x 8 transposition that turns a lane's block of a
// row-major tile into MFMA operands, and loop helpers whose register buffers are picked at compile time.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <type_traits>

namespace slim {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr float NEG_INF = -INFINITY;

__device__ __forceinline__ int seq_len_of(const int32_t* lens, int b, int T) {
  if (!lens) return T;
  const int n = lens[b];
  return n < 0 ? 0 : (n > T ? T : n);
}

// 8 rows x 8 bf16 columns per lane  ->  8 operands (one per column), each 8 rows of that column.
__device__ __forceinline__ void transpose8x8(const u32x4 (&kt)[8], u32x4 (&a)[8]) {
#pragma unroll
  for (int jp = 0; jp < 4; ++jp) {
    const u32x4 lo = kt[2 * jp], hi = kt[2 * jp + 1];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      a[2 * c][jp] = __builtin_amdgcn_perm(hi[c], lo[c], 0x05040100u);      // even column: low halves
      a[2 * c + 1][jp] = __builtin_amdgcn_perm(hi[c], lo[c], 0x07060302u);  // odd column: high halves
    }
  }
}

// f(k + I, integral_constant<I>) for I = 0 .. N-1 while k + I < end: loop bodies whose register
// buffers are chosen by a compile-time index.
template <int I, int N, class F>
__device__ __forceinline__ void unrolled_steps(int k, int end, F& f) {
  if constexpr (I < N) {
    if (k + I < end) f(k + I, std::integral_constant<int, I>{});
    unrolled_steps<I + 1, N>(k, end, f);
  }
}

// The same without the bound checks, for whole groups of N steps (straight-line code: the compiler can
// then count the loads in flight across steps).
template <int I, int N, class F>
__device__ __forceinline__ void full_steps(int k, F& f) {
  if constexpr (I < N) {
    f(k + I, std::integral_constant<int, I>{});
    full_steps<I + 1, N>(k, f);
  }
}

}  // namespace slim
