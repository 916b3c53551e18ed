// Shared constants and small device helpers of the gfx950 CNN library.
// Network and parameter layout: arXiv 1912.05234, Section 3, listing `forward`.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cnn.h"

namespace cnn {

// activation sizes per image
constexpr int NI = 28 * 28;        // input image
constexpr int NC1 = 6 * 24 * 24;   // C1 output
constexpr int NS1 = 6 * 12 * 12;   // S1 output
constexpr int NC2 = 12 * 8 * 8;    // C2 output
constexpr int NS2 = 12 * 4 * 4;    // S2 output
constexpr int NY = 10;             // network output

// flat parameter vector: k1[6,5,5] b1[6] k2[12,6,5,5] b2[12] fc[10,192] b[10]
constexpr int OFF_K1 = 0;
constexpr int OFF_B1 = 150;
constexpr int OFF_K2 = 156;
constexpr int OFF_B2 = 1956;
constexpr int OFF_FC = 1968;
constexpr int OFF_B = 3888;
constexpr int NPARAM = 3898;
static_assert(NPARAM == CNN_NPARAM, "parameter count");

// One row of per-workgroup partial results: 3898 gradient sums, the loss sum
// in slot LOSS_SLOT, padding up to a multiple of 64 floats.
constexpr int LOSS_SLOT = NPARAM;
constexpr int PSTRIDE = 3904;

// Logistic function of Section 3 (listing `sigmoid`), 1/(1+exp(-x)), through the
// hardware base-2 exponential and reciprocal (each about 1 ulp).  Finite for
// every finite x: exp2 overflows to +inf and 1/inf = 0; it underflows to 0 and
// 1/1 = 1.
constexpr float NEG_LOG2E = -1.44269504088896340736f;
__device__ __forceinline__ float logistic(float x) {
  const float e = __builtin_amdgcn_exp2f(x * NEG_LOG2E);
  return __builtin_amdgcn_rcpf(1.0f + e);
}
// The same function of z = -log2(e) * x: the convolution layers keep their weights and biases
// multiplied by that constant in the expanded operand table, so their sums arrive already scaled.
__device__ __forceinline__ float logistic_of_scaled(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z));
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace cnn

#define CNN_HIP_TRY(expr)                 \
  do {                                    \
    hipError_t e__ = (expr);              \
    if (e__ != hipSuccess) {              \
      (void)hipGetLastError();            \
      return CNN_EHIP;                    \
    }                                     \
  } while (0)
