// The fully connected layer's three calls for the network's own shape (192 inputs, 10 outputs), each
// wave working straight from global memory (arXiv 1912.05234, Section 3: the layer is `mconv` with a
// kernel as large as its input; its backward forms are backin, backweights and backbias).  A row of
// this layer is 768 bytes in and 40 bytes out, so the calls are bound by memory and by their own
// set-up; the general kernels (cnn_igemm.h) stage groups of images in LDS for four waves that share
// them, which costs barriers and staging time that rows this small do not need.  Here the operands
// of v_mfma_f32_16x16x4_f32 are loaded in the instruction's own layout, the K index permuted so that a
// lane's four K elements are 16 consecutive bytes:
//   forward          D[o][image] = sum_i w[o][i] in[image][i]: M = 10(16) outputs, N = 16 images per tile,
//                    K = 192 in 48 steps; lane (q, n16) holds in[image n16][16 t + 4 q + r] for step (t, r)
//   input gradient   D[i][image] = sum_o w[o][i] d_out[image][o]: M = 192 in twelve tiles, N = 16 images,
//                    K = 10(12) in three steps; a lane's four results are 16 consecutive bytes of d_in
//   weight gradient  D[o][i] = sum_image d_out[image][o] in[image][i]: M = 10(16), N = 192 in twelve tiles,
//                    K = images four per step; column n16 of tile nt is input 64 (nt / 4) + 4 n16 + nt % 4,
//                    so that a lane reads three 16-byte pieces per image; the sums stay in registers
//                    over a wave's steps, the eight waves of a workgroup are added through LDS in a
//                    fixed order and the workgroup writes one set of partial tiles in the layout of
//                    the general kernel, whose second kernel adds the workgroups' partials.
#pragma once

#include "cnn_wave.h"

namespace cnn {
namespace fc {

constexpr int IN = NS2, OUT = 10;  // 192 inputs (the pooled output of the second convolution), ten outputs
static_assert(IN % 64 == 0 && OUT <= 12, "twelve column tiles, three K steps of four outputs");
inline bool shape_fits(int I, int O) { return I == IN && O == OUT; }

constexpr int WAVES_PER_GROUP = 4, THREADS = 64 * WAVES_PER_GROUP;
constexpr int TILE = 16;  // images per tile of the forward and input-gradient kernels

// out[n][o] = bias[o] + sum_i w[o][i] in[n][i]; bias may be null.
__global__ __launch_bounds__(THREADS) void forward_kernel(const float* __restrict__ in, const float* __restrict__ w,
                                                          const float* __restrict__ bias, float* __restrict__ out,
                                                          int B) {
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  // A[row o = n16][k = q] of step (s, r) = w[o][16 s + 4 q + r]; rows 10..15 are zero
  f4 a[IN / 16];
  {
    const float* row = w + (n16 < OUT ? n16 : 0) * IN + 4 * q;
#pragma unroll
    for (int s = 0; s < IN / 16; ++s) {
      a[s] = *reinterpret_cast<const f4*>(row + 16 * s);
      if (n16 >= OUT) a[s] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    }
  }
  f4 start = f4{0.0f, 0.0f, 0.0f, 0.0f};  // result row 4 q + r
  if (bias) {
#pragma unroll
    for (int r = 0; r < 4; ++r) start[r] = 4 * q + r < OUT ? bias[4 * q + r] : 0.0f;
  }
  const int tiles = (B + TILE - 1) / TILE, G = gridDim.x * WAVES_PER_GROUP;
  // B[k = q][column n16] = in[image n16 of the tile][16 s + 4 q + r]; images past the end re-read the last one
  auto load = [&](int T, f4 (&x)[IN / 16]) {
    const int n = TILE * T + n16 < B ? TILE * T + n16 : B - 1;
    const float* row = in + (size_t)n * IN + 4 * q;
#pragma unroll
    for (int s = 0; s < IN / 16; ++s) x[s] = *reinterpret_cast<const f4*>(row + 16 * s);
  };
  f4 x[IN / 16], xn[IN / 16];
  int T = blockIdx.x * WAVES_PER_GROUP + wave;
  if (T < tiles) load(T, x);
  for (; T < tiles; T += G) {
    if (T + G < tiles) load(T + G, xn);  // in flight during this tile
    // four independent sums (one per r), joined at the end
    f4 acc[4] = {start, f4{0.0f, 0.0f, 0.0f, 0.0f}, f4{0.0f, 0.0f, 0.0f, 0.0f}, f4{0.0f, 0.0f, 0.0f, 0.0f}};
#pragma unroll
    for (int s = 0; s < IN / 16; ++s)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[r] = mfma16(a[s][r], x[s][r], acc[r]);
    const f4 d = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    const int n = TILE * T + n16;
    if (n < B && q < 3) {  // outputs 4 q .. 4 q + 3 of image n (two of them in the last quarter)
      float* dst = out + (size_t)n * OUT + 4 * q;
      *reinterpret_cast<float2*>(dst) = float2{d[0], d[1]};
      if (q < 2) *reinterpret_cast<float2*>(dst + 2) = float2{d[2], d[3]};
    }
#pragma unroll
    for (int s = 0; s < IN / 16; ++s) x[s] = xn[s];
  }
}

// d_in[n][i] = sum_o w[o][i] d_out[n][o].
__global__ __launch_bounds__(THREADS) void bwd_input_kernel(const float* __restrict__ d_out,
                                                            const float* __restrict__ w, float* __restrict__ d_in,
                                                            int B) {
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  // A[row i = 16 mt + n16][k = q] of step s = w[o = 4 s + q][i]; outputs 10, 11 are zero
  float a[IN / 16][3];
#pragma unroll
  for (int mt = 0; mt < IN / 16; ++mt)
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      const int o = 4 * s + q;
      a[mt][s] = w[(o < OUT ? o : 0) * IN + 16 * mt + n16];
      if (o >= OUT) a[mt][s] = 0.0f;
    }
  const int tiles = (B + TILE - 1) / TILE, G = gridDim.x * WAVES_PER_GROUP;
  // B[k = q][column n16] of step s = d_out[image n16 of the tile][4 s + q]
  auto load = [&](int T, float (&b)[3]) {
    const int n = TILE * T + n16 < B ? TILE * T + n16 : B - 1;
    const float* row = d_out + (size_t)n * OUT;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      const int o = 4 * s + q;
      b[s] = row[o < OUT ? o : 0];
      if (o >= OUT) b[s] = 0.0f;
    }
  };
  float b[3], bn[3];
  int T = blockIdx.x * WAVES_PER_GROUP + wave;
  if (T < tiles) load(T, b);
  for (; T < tiles; T += G) {
    if (T + G < tiles) load(T + G, bn);
    const int n = TILE * T + n16;
    float* dst = d_in + (size_t)(n < B ? n : 0) * IN + 4 * q;
#pragma unroll
    for (int mt = 0; mt < IN / 16; ++mt) {
      f4 acc = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int s = 0; s < 3; ++s) acc = mfma16(a[mt][s], b[s], acc);
      if (n < B) *reinterpret_cast<f4*>(dst + 16 * mt) = acc;  // inputs 16 mt + 4 q .. + 3 of image n
    }
#pragma unroll
    for (int s = 0; s < 3; ++s) b[s] = bn[s];
  }
}

// ---- weight and bias gradient --------------------------------------------------------------------------
constexpr int WGRAD_WAVES = 8, WGRAD_THREADS = 64 * WGRAD_WAVES;
constexpr int NT = IN / 16;               // twelve column tiles
constexpr int ACC_FLOATS = NT * 4 * 64;   // a wave's sums: [tile nt][register r][lane]
constexpr int AHEAD = 4;                  // K steps (of four images) whose loads are one memory round trip
struct __align__(16) WgradLds {
  float comb[WGRAD_WAVES / 2][ACC_FLOATS];  // cross-wave sums
  float bsum[WGRAD_WAVES][64];
};
// part: [gridDim.x][12 tiles][16 rows o][16 columns] then the bias rows [gridDim.x][16] (the layout
// igemm::wgrad_reduce_kernel reads with MT = 1, NT = 12, P = 1).
__global__ __launch_bounds__(WGRAD_THREADS) void bwd_weight_kernel(const float* __restrict__ in,
                                                                   const float* __restrict__ d_out,
                                                                   float* __restrict__ part, int B) {
  __shared__ WgradLds lds;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  f4 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  float g_b = 0.0f;
  const int steps = (B + 3) / 4, G = gridDim.x * WGRAD_WAVES;
  for (int S0 = blockIdx.x * WGRAD_WAVES + wave; S0 < steps; S0 += AHEAD * G) {
    // A[row o = n16][k = q] = d_out[image 4 S + q][o]; B[k = q][column n16 of tile 4 g + c] =
    // in[image 4 S + q][64 g + 4 n16 + c].  A step or an image past the end contributes a zero A
    // operand (its B operand re-reads image 0).
    float av[AHEAD];
    f4 xv[AHEAD][IN / 64];
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) {
      const int S = S0 + k * G;
      const long long n = 4LL * S + q;
      const bool real = S < steps && n < B;
      const size_t nn = real ? (size_t)n : 0;
      av[k] = d_out[nn * OUT + (n16 < OUT ? n16 : 0)];
      if (!real || n16 >= OUT) av[k] = 0.0f;
#pragma unroll
      for (int g = 0; g < IN / 64; ++g) xv[k][g] = *reinterpret_cast<const f4*>(in + nn * IN + 64 * g + 4 * n16);
    }
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) {
      g_b += av[k];
#pragma unroll
      for (int g = 0; g < IN / 64; ++g)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[4 * g + c] = mfma16(av[k], xv[k][g][c], acc[4 * g + c]);
    }
  }
  // ---- the eight waves' sums in a fixed order: (w, w + 4), then (w, w + 2), then (0, 1) ----
  lds.bsum[wave][l] = g_b;
#pragma unroll
  for (int half = WGRAD_WAVES / 2; half >= 1; half >>= 1) {
    __syncthreads();
    if (wave >= half && wave < 2 * half) {
      float* dst = lds.comb[wave - half];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[(4 * nt + r) * 64 + l] = acc[nt][r];
    }
    __syncthreads();
    if (wave < half) {
      const float* src = lds.comb[wave];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[nt][r] += src[(4 * nt + r) * 64 + l];
    }
  }
  if (wave == 0) {
    float* tiles = part + (size_t)blockIdx.x * NT * 256;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int i = 64 * (nt >> 2) + 4 * n16 + (nt & 3);  // the input this lane's column of tile nt stands for
#pragma unroll
      for (int r = 0; r < 4; ++r) tiles[(i >> 4) * 256 + (4 * q + r) * 16 + (i & 15)] = acc[nt][r];  // row o = 4 q + r
    }
  } else if (wave == 1 && l < 16) {
    // bias gradient of output l: the four lane quarters of the eight waves, in wave order
    float s = 0.0f;
    if (l < OUT)
      for (int w = 0; w < WGRAD_WAVES; ++w) s += (lds.bsum[w][l] + lds.bsum[w][l + 16]) + (lds.bsum[w][l + 32] + lds.bsum[w][l + 48]);
    part[(size_t)gridDim.x * NT * 256 + (size_t)blockIdx.x * 16 + l] = s;
  }
}
inline size_t bwd_weight_workspace_bytes(unsigned groups) { return sizeof(float) * (size_t)groups * (NT * 256 + 16); }

}  // namespace fc
}  // namespace cnn
