// Input gradient of a 5 x 5 convolution with twelve output and six input maps on a 12 x 12 input
// (the shape of the network's second convolution), in the col2im form of `backin` (arXiv
// 1912.05234, Section 3, "Backpropagating Convolution"):
//   T[(c,u,v), p] = sum_j k[j,c,u,v] * d_out[j,p],      d_in[c, y(p)+u, x(p)+v] += T[(c,u,v), p]
// one wave per image.  The 150 rows of T fill ten 16-row tiles of v_mfma_f32_16x16x4_f32 (K = 12
// output maps in three steps, four tiles of sixteen pixels): 120 matrix instructions per image, where
// the general kernel (cnn_igemm.h: a forward convolution over the bordered error) needs 414.  T is
// added into an LDS copy of d_in in rounds of read-add-write whose targets cannot collide; the
// tiling of the taps, the two halves of the maps 4 and 5 and the rounds are those of the fused
// training step and are described there (cnn_wave.h: bwd_tap, bwd_packed_source, phase 6 of
// wave_image); only the index helpers are shared.
#pragma once

#include "cnn_wave.h"

namespace cnn {
namespace col2im {

constexpr int WAVES_PER_GROUP = 8;
constexpr int ENTRIES = 18 + 12;   // plain tiles V(0..4), U4 of the maps 0..3; packed tiles PV(0..2), PU
constexpr int ACC_FLOATS = NS1 + 304;  // d_in[6][12][12] and the second copy of the maps 4, 5 (with its reach)
struct __align__(16) Lds {
  float tab[ENTRIES * 64];                    // A operands, [entry = tile * 3 + K step][lane]
  float acc[WAVES_PER_GROUP][ACC_FLOATS];
};
constexpr int COUT = 12, CIN = 6, OUT_PIXELS = 64, IN_FLOATS = NS1, OUT_FLOATS = COUT * OUT_PIXELS;

__global__ __launch_bounds__(64 * WAVES_PER_GROUP) void conv_bwd_input_kernel(const float* __restrict__ d_out,
                                                                             const float* __restrict__ k,
                                                                             float* __restrict__ d_in, int B) {
  __shared__ Lds lds;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  // ---- A operands: lane (q, n16) of entry (tile, s) holds k[j = 4 s + q][c][tap] of tile row n16 ----
  for (int i = t; i < ENTRIES * 64; i += 64 * WAVES_PER_GROUP) {
    const int e = i >> 6, lane = i & 63, j = 4 * (e % 3) + (lane >> 4), row = lane & 15;
    int src;  // 25 c + tap, or -1
    if (e < 18) {
      const int tap = bwd_tap(e / 3, row & 3);
      src = 25 * (row >> 2) + tap;
    } else {
      src = bwd_packed_source((e - 18) / 3, row >> 2, row & 3);
    }
    lds.tab[i] = src >= 0 ? k[j * (CIN * 25) + src] : 0.0f;
  }
  __syncthreads();
  const float* tl = lds.tab + l;
  float* acc = lds.acc[wave];
  float* copy = acc + NS1;
  // pixel 16 nt + n16 of tile nt is (y, x) = (2 nt + (n16 % 4) / 2, 2 (n16 / 4) + n16 % 2): a lane's element of d_out
  const int lane_src = q * OUT_PIXELS + ((n16 & 3) >> 1) * 8 + 2 * (n16 >> 2) + (n16 & 1);
  const int pp = 12 * ((n16 & 3) >> 1) + 2 * (n16 >> 2) + (n16 & 1);
  auto load_image = [&](size_t n, float (&bd)[3][4]) {
    const float* src = d_out + n * OUT_FLOATS + lane_src;
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) bd[s][nt] = src[4 * s * OUT_PIXELS + 16 * nt];
  };
  const size_t G = (size_t)gridDim.x * WAVES_PER_GROUP, first = (size_t)blockIdx.x * WAVES_PER_GROUP + wave;
  float bd[3][4], next[3][4];
  if (first < (size_t)B) load_image(first, bd);
  for (size_t n = first; n < (size_t)B; n += G) {
    if (n + G < (size_t)B) load_image(n + G, next);  // in flight during this image
    for (int e = l; e < ACC_FLOATS / 4; e += 64) reinterpret_cast<f4*>(acc)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    wave_sync();
    auto tiles = [&](int first_entry, f4 (&out)[4]) {
      float av[3];
#pragma unroll
      for (int s = 0; s < 3; ++s) av[s] = tl[(first_entry + s) * 64];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        f4 a = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < 3; ++s) a = mfma16(av[s], bd[s][nt], a);
        out[nt] = a;
      }
    };
    // level = 2 nt + u: all even levels of a tap column in one round, then all odd ones
    auto rounds = [&](const f4 (&tv)[4], const float (&u4)[4], float* dst) {
      {
        float e[6], old[6];
#pragma unroll
        for (int m = 0; m < 6; ++m) {
          float a = 0.0f;
          if (m < 4) a = tv[m < 4 ? m : 0][0];
          if (m >= 1 && m <= 4) a += tv[m >= 1 ? m - 1 : 0][2];
          if (m >= 2) a += u4[m >= 2 ? m - 2 : 0];
          e[m] = a;
          old[m] = dst[24 * m];
        }
#pragma unroll
        for (int m = 0; m < 6; ++m) dst[24 * m] = old[m] + e[m];
      }
      wave_sync();
      {
        float e[5], old[5];
#pragma unroll
        for (int m = 0; m < 5; ++m) {
          float a = 0.0f;
          if (m < 4) a = tv[m < 4 ? m : 0][1];
          if (m >= 1) a += tv[m >= 1 ? m - 1 : 0][3];
          e[m] = a;
          old[m] = dst[24 * m + 12];
        }
#pragma unroll
        for (int m = 0; m < 5; ++m) dst[24 * m + 12] = old[m] + e[m];
      }
      wave_sync();
    };
    f4 tu[4];
    tiles(18 + kTilePU * 3, tu);
    {  // maps 0..3: lane quarter q owns map q
      f4 t4[4], tv[4], tn[4];
      tiles(kTileU4 * 3, t4);
      float* tgt = acc + 144 * q + pp;
      tiles(kTileV0 * 3, tv);
#pragma unroll
      for (int v = 0; v < 5; ++v) {
        if (v < 4) tiles((kTileV0 + v + 1) * 3, tn);
        float u4[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) u4[nt] = v < 4 ? t4[nt][v < 4 ? v : 0] : tu[nt][3];
        rounds(tv, u4, tgt + v);
        if (v < 4) {
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) tv[nt] = tn[nt];
        }
      }
    }
    {  // maps 4, 5: quarters 0, 1 for the tap columns 0..2 into d_in, quarters 2, 3 for 3, 4 into the copy
      float* tgt = q < 2 ? acc + 144 * (4 + q) + pp : copy + 144 * (q - 2) + pp + 3;
      f4 tv[4], tn[4];
      tiles(18 + kTilePV0 * 3, tv);
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        if (r < 2) tiles(18 + (kTilePV0 + r + 1) * 3, tn);
        float u4[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) u4[nt] = tu[nt][r];
        rounds(tv, u4, tgt + r);
        if (r < 2) {
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) tv[nt] = tn[nt];
        }
      }
    }
    // ---- d_in of this image: 864 consecutive floats, the two halves of the maps 4, 5 joined ----
    float* dst = d_in + n * IN_FLOATS;
    for (int e = l; e < IN_FLOATS; e += 64) {
      float v = acc[e];
      if (e >= 4 * 144) v += copy[e - 4 * 144];
      dst[e] = v;
    }
    wave_sync();  // the reads above come before the next image's clearing
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) bd[s][nt] = next[s][nt];
  }
}

inline bool shape_fits(int Cin, int H, int W, int Cout, int KH, int KW) {
  return Cin == CIN && Cout == COUT && KH == 5 && KW == 5 && H == 12 && W == 12;
}

}  // namespace col2im
}  // namespace cnn
