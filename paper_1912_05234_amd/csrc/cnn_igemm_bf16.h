// Reduced-precision variant of the implicit-GEMM convolution: operands rounded to bfloat16
// (round to nearest, ties to even), products summed in fp32 on v_mfma_f32_16x16x32_bf16.
// Tensors in memory stay fp32, NCHW; only the arithmetic changes, which is why these are separate
// entry points with their own tolerance.  (The paper computes in `float` throughout, Section 3;
// this is the reduced-precision matrix-core form of its `conv` / `backin`.)
//
// The instruction takes, per lane, eight consecutive K elements of A's row (lane % 16) and of B's
// column (lane % 16), K elements 8 (lane / 16) .. + 7 of a block of 32.  The K index is therefore
// ordered (u, v, c) with the channels padded to a multiple of eight, and the staged tensor is held
// in LDS channel-last as bf16 [row][column][C8]: a lane's eight B values are then one aligned
// 16-byte LDS read at (byte offset of the tap and channel chunk) + (byte offset of the pixel).
#pragma once

#include <hip/hip_runtime.h>

#include "cnn_igemm.h"

namespace cnn {
namespace igemm16 {

using igemm::THREADS;
using igemm::WAVES;
using igemm::f4;
using igemm::i4;
using igemm::divmod;
using igemm::lds_barrier;
using bf8 = __bf16 __attribute__((ext_vector_type(8)));

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ unsigned short to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
// two at once: lo in bits 0..15, hi in bits 16..31 (the conversion of a float pair is one
// instruction on gfx950, same rounding)
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  using f2v = float __attribute__((ext_vector_type(2)));
  using bf2v = __bf16 __attribute__((ext_vector_type(2)));
  const bf2v r = __builtin_convertvector(f2v{lo, hi}, bf2v);
  return __builtin_bit_cast(unsigned, r);
}

struct Args {
  const float* src;   // [B][SC][SH][SW]
  const float* w;     // [Cout][Cin][KH][KW]
  const float* bias;  // M values or null
  float* dst;         // [B][M][OH][OW]
  int B, M, SC, SH, SW, KH, KW, OH, OW;
  int pady, padx;     // border of zeros around a staged plane
  int flip;           // 0: A[m][(u,v,c)] = w[m][c][u][v];  1: A[m][(u,v,c)] = w[c][m][KH-1-u][KW-1-v]
  int C8, K, NBK;     // channels padded to 8; reduction length KH*KW*C8; blocks of 32
  int RS;             // bytes of a row of the weight table
  int LW, LPIX;       // pixels of a staged row, of a staged image
  int NB, groups, MT;
  float inv_kp, inv_c8, inv_kw, inv_ohow, inv_ow, inv_chhw, inv_hw, inv_sw;
};
// LDS layout in bytes, in this order (every part a multiple of 16).
struct Lds {
  int wt, koff, bias, poff, ooff, x, total;
};
__host__ __device__ inline int up16(int v) { return (v + 15) & ~15; }
__host__ __device__ inline Lds lds_layout(const Args& a) {
  Lds l;
  l.wt = 0;                                     // bf16 [16 MT rows][RS / 2]
  l.koff = l.wt + 16 * a.MT * a.RS;             // int [NBK][4]: byte offset in x of K elements 32 b + 8 q ..
  l.bias = l.koff + 16 * a.NBK;                 // float [16 MT]
  l.poff = l.bias + 64 * a.MT;                  // int [NB*OH*OW]: byte offset of the column's pixel in x
  l.ooff = l.poff + up16(4 * a.NB * a.OH * a.OW);  // int [NB*OH*OW]: float offset of the column in dst
  l.x = l.ooff + up16(4 * a.NB * a.OH * a.OW);  // bf16 [NB][LPIX][C8]
  l.total = l.x + up16(2 * a.NB * a.LPIX * a.C8);
  return l;
}

template <int TP>
__global__ __launch_bounds__(THREADS) void conv_kernel(const Args g) {
  extern __shared__ __align__(16) char smem[];
  const Lds L = lds_layout(g);
  int* koff = reinterpret_cast<int*>(smem + L.koff);
  float* bl = reinterpret_cast<float*>(smem + L.bias);
  int* poff = reinterpret_cast<int*>(smem + L.poff);
  int* ooff = reinterpret_cast<int*>(smem + L.ooff);
  char* x = smem + L.x;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, j = l & 15;
  const int KHKW = g.KH * g.KW, OHOW = g.OH * g.OW, HW = g.SH * g.SW, per_image = g.SC * HW;
  const int KP = 32 * g.NBK;  // K elements of a table row

  // ---- tables, once per workgroup ----
  for (int e0 = t; e0 < 16 * g.MT * KP; e0 += 8 * THREADS) {  // eight independent loads in flight per thread
    float val[8];
    int where[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int e = e0 + i * THREADS;
      val[i] = 0.0f, where[i] = -1;
      if (e < 16 * g.MT * KP) {
        int m, kk, tap, c, u, v;
        divmod(e, KP, g.inv_kp, m, kk);
        divmod(kk, g.C8, g.inv_c8, tap, c);
        divmod(tap, g.KW, g.inv_kw, u, v);
        where[i] = m * g.RS + 2 * kk;
        if (m < g.M && kk < g.K && c < g.SC)
          val[i] = !g.flip ? g.w[((size_t)m * g.SC + c) * KHKW + u * g.KW + v]
                           : g.w[((size_t)c * g.M + m) * KHKW + (g.KH - 1 - u) * g.KW + (g.KW - 1 - v)];
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (where[i] >= 0) *reinterpret_cast<unsigned short*>(smem + L.wt + where[i]) = to_bf16(val[i]);
  }
  for (int e = t; e < 4 * g.NBK; e += THREADS) {
    const int kk = 8 * e;  // 32 (e / 4) + 8 (e % 4)
    int off = 0;
    if (kk < g.K) {
      int tap, c, u, v;
      divmod(kk, g.C8, g.inv_c8, tap, c);
      divmod(tap, g.KW, g.inv_kw, u, v);
      off = 2 * ((u * g.LW + v) * g.C8 + c);
    }
    koff[e] = off;
  }
  for (int m = t; m < 16 * g.MT; m += THREADS) bl[m] = (g.bias && m < g.M) ? g.bias[m] : 0.0f;
  for (int n = t; n < g.NB * OHOW; n += THREADS) {
    int img, r, y, xx;
    divmod(n, OHOW, g.inv_ohow, img, r);
    divmod(r, g.OW, g.inv_ow, y, xx);
    poff[n] = 2 * (img * g.LPIX + y * g.LW + xx) * g.C8;
    ooff[n] = img * g.M * OHOW + r;
  }
  // borders and padding channels stay zero for the whole kernel
  for (int e = t; e < (g.NB * g.LPIX * g.C8) >> 3; e += THREADS) reinterpret_cast<f4*>(x)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};

  // Staging of a group: one item = one pixel's eight channels of a chunk, read from the eight
  // channel planes (a wave reads 256 consecutive bytes of each), rounded, packed and written as one
  // 16-byte LDS item; two items per thread in flight.  There is no hand-over through registers
  // across the matrix work here: the workgroups are small, and the other resident ones cover the
  // load latency.
  const int CH = g.C8 >> 3;
  auto stage = [&](int grp) {
    const int b0 = grp * g.NB, items = min(g.NB, g.B - b0) * CH * HW;
    const float* src = g.src + (size_t)b0 * per_image;
    for (int e0 = t; e0 < items; e0 += 2 * THREADS) {
      float v[2][8];
      int where[2];
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int e = e0 + k * THREADS;
        where[k] = -1;
        if (e < items) {
          int img, r, chunk, p, y, xx;
          divmod(e, CH * HW, g.inv_chhw, img, r);
          divmod(r, HW, g.inv_hw, chunk, p);
          divmod(p, g.SW, g.inv_sw, y, xx);
          where[k] = 2 * ((img * g.LPIX + (y + g.pady) * g.LW + g.padx + xx) * g.C8 + 8 * chunk);
          const float* sp = src + (size_t)img * per_image + (size_t)(8 * chunk) * HW + p;
#pragma unroll
          for (int cc = 0; cc < 8; ++cc) v[k][cc] = 8 * chunk + cc < g.SC ? sp[cc * HW] : 0.0f;
        }
      }
#pragma unroll
      for (int k = 0; k < 2; ++k)
        if (where[k] >= 0) {
          i4 packed;
#pragma unroll
          for (int h = 0; h < 4; ++h) packed[h] = (int)pack_bf16(v[k][2 * h], v[k][2 * h + 1]);
          *reinterpret_cast<i4*>(x + where[k]) = packed;
        }
    }
  };

  for (int grp = blockIdx.x; grp < g.groups; grp += gridDim.x) {
    const int b0 = grp * g.NB, nb = min(g.NB, g.B - b0);
    lds_barrier();  // tables and zeros (first pass) / the previous group's reads are complete
    stage(grp);
    lds_barrier();

    const int N = nb * OHOW, PT = (N + 15) >> 4, PG = (PT + TP - 1) / TP;
    float* dst = g.dst + (size_t)b0 * g.M * OHOW;
    for (int job = wave; job < PG * g.MT; job += WAVES) {
      const int pg = job / g.MT, mt = job - pg * g.MT;
      int po[TP], oo[TP];
      f4 acc[TP];
      const f4 binit = *reinterpret_cast<const f4*>(&bl[16 * mt + 4 * q]);
#pragma unroll
      for (int tt = 0; tt < TP; ++tt) {
        const int n = 16 * (pg * TP + tt) + j, nn = n < N ? n : N - 1;
        po[tt] = poff[nn];
        oo[tt] = ooff[nn];
      }
      const char* arow = smem + L.wt + (16 * mt + j) * g.RS + 16 * q;
      // Block 0 starts the sums from the bias; then two blocks per trip, the reads of one under the
      // MFMAs of the other.  The byte offset of a block's K elements is fetched two blocks ahead, so
      // that no read waits for another, and a trip has no branches: block numbers past the end are
      // clamped to the last block, whose operands are then read again and not used.
      const int last = g.NBK - 1;
      const int* kq = koff + q;
      bf8 a0, a1, b0v[TP], b1v[TP];
      int k2 = kq[4 * min(2, last)], k3 = kq[4 * min(3, last)];
      {
        const int k0 = kq[0], k1 = kq[4 * min(1, last)];
        a0 = *reinterpret_cast<const bf8*>(arow);
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) b0v[tt] = *reinterpret_cast<const bf8*>(x + po[tt] + k0);
        a1 = *reinterpret_cast<const bf8*>(arow + 64 * min(1, last));
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) b1v[tt] = *reinterpret_cast<const bf8*>(x + po[tt] + k1);
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b0v[tt], binit, 0, 0, 0);
      }
      int b = 1;  // block b is in a1, b1v
      for (; b + 1 < g.NBK; b += 2) {
        const int k4 = kq[4 * min(b + 3, last)], k5 = kq[4 * min(b + 4, last)];
        a0 = *reinterpret_cast<const bf8*>(arow + 64 * (b + 1));
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) b0v[tt] = *reinterpret_cast<const bf8*>(x + po[tt] + k2);
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1v[tt], acc[tt], 0, 0, 0);
        a1 = *reinterpret_cast<const bf8*>(arow + 64 * min(b + 2, last));
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) b1v[tt] = *reinterpret_cast<const bf8*>(x + po[tt] + k3);
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b0v[tt], acc[tt], 0, 0, 0);
        k2 = k4, k3 = k5;
      }
      if (b < g.NBK) {  // one block left: it is already in a1, b1v
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b1v[tt], acc[tt], 0, 0, 0);
      }
      // lane (q, j) holds rows 16 mt + 4 q + r of column j
      const int m0 = 16 * mt + 4 * q;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (m0 + r < g.M) {
#pragma unroll
          for (int tt = 0; tt < TP; ++tt)
            if (16 * (pg * TP + tt) + j < N) dst[oo[tt] + (m0 + r) * OHOW] = acc[tt][r];
        }
    }
  }
}

}  // namespace igemm16
}  // namespace cnn
