// Reduced-precision variant of the implicit-GEMM convolution: operands rounded to bfloat16
// (round to nearest, ties to even), products summed in fp32 on v_mfma_f32_16x16x32_bf16.
// Tensors in memory stay fp32, NCHW; only the arithmetic changes, which is why these are separate
// entry points with their own tolerance.  (The paper computes in `float` throughout, Section 3;
// this is the reduced-precision matrix-core form of its `conv` / `backin` and, further down, of
// `backweights` / `backbias`.)
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

// fp32 -> bf16 bits, round to nearest even; a NaN stays a (quiet) NaN instead of having its
// mantissa carried into the exponent
__device__ __forceinline__ unsigned short to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
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
  int P, MR, KWP, OWP;  // column packing as in the fp32 kernel: P pixels per column, rows (m, sh) = M*P,
                       // shifted taps v' < KW+P-1 with A[(m,sh)][(u,v',c)] = w[m][c][u][v'-sh], OW/P columns per row
  int C8, K, NBK;     // channels padded to 8; reduction length KH*KWP*C8; blocks of 32
  int RS;             // bytes of a row of the weight table
  int LW, LPIX;       // pixels of a staged row, of a staged image
  int NB, groups, MT;
  float inv_kp, inv_c8, inv_kwp, inv_cols, inv_owp, inv_chhw, inv_hw, inv_sw, inv_p;
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
  l.poff = l.bias + 64 * a.MT;                  // int [NB*OH*OWP]: byte offset of the column's first pixel in x
  l.ooff = l.poff + up16(4 * a.NB * a.OH * a.OWP);  // int [NB*OH*OWP]: float offset of the column in dst (channel 0, sh 0)
  l.x = l.ooff + up16(4 * a.NB * a.OH * a.OWP);  // bf16 [NB][LPIX][C8]
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
        int mrow, kk, tap, c, u, vp, m, sh;
        divmod(e, KP, g.inv_kp, mrow, kk);
        divmod(kk, g.C8, g.inv_c8, tap, c);
        divmod(tap, g.KWP, g.inv_kwp, u, vp);
        divmod(mrow, g.P, g.inv_p, m, sh);
        const int v = vp - sh;
        where[i] = mrow * g.RS + 2 * kk;
        if (mrow < g.MR && kk < g.K && c < g.SC && v >= 0 && v < g.KW)
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
      int tap, c, u, vp;
      divmod(kk, g.C8, g.inv_c8, tap, c);
      divmod(tap, g.KWP, g.inv_kwp, u, vp);
      off = 2 * ((u * g.LW + vp) * g.C8 + c);
    }
    koff[e] = off;
  }
  for (int mrow = t; mrow < 16 * g.MT; mrow += THREADS) {
    int m, sh;
    divmod(mrow, g.P, g.inv_p, m, sh);
    bl[mrow] = (g.bias && mrow < g.MR) ? g.bias[m] : 0.0f;
  }
  const int COLS = g.OH * g.OWP;
  for (int n = t; n < g.NB * COLS; n += THREADS) {
    int img, r, y, xx;
    divmod(n, COLS, g.inv_cols, img, r);
    divmod(r, g.OWP, g.inv_owp, y, xx);
    poff[n] = 2 * (img * g.LPIX + y * g.LW + g.P * xx) * g.C8;
    ooff[n] = img * g.M * OHOW + y * g.OW + g.P * xx;
  }
  // float offset in dst of this lane's result register r in M tile 0 (packed forms have one M tile)
  int ro0[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int m, sh;
    divmod(4 * q + r, g.P, g.inv_p, m, sh);
    ro0[r] = m * OHOW + sh;
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

    const int N = nb * COLS, PT = (N + 15) >> 4, PG = (PT + TP - 1) / TP;
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
      // lane (q, j) holds rows 16 mt + 4 q + r of column j; row (m, sh) is channel m, pixel P X + sh
      const int m0 = 16 * mt + 4 * q;
      if ((g.P & 3) == 0 && 16 * (pg * TP + TP) <= N) {
        // four (or a multiple of four) pixels per column: the four registers are neighbours in memory
        if (m0 < g.MR) {
#pragma unroll
          for (int tt = 0; tt < TP; ++tt) *reinterpret_cast<f4*>(dst + oo[tt] + ro0[0]) = acc[tt];
        }
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (m0 + r < g.MR) {
#pragma unroll
            for (int tt = 0; tt < TP; ++tt)
              if (16 * (pg * TP + tt) + j < N) dst[oo[tt] + ro0[r] + 16 * mt * OHOW] = acc[tt][r];
          }
      }
    }
  }
}

// ---- weight and bias gradient ----------------------------------------------------------------------
// T[co][(c,u,v)] = sum over pixels of d_out[co][y][x] * in[c][y+u][x+v], operands rounded to bf16.
// K runs over pixel slots: a row of the output is cut into XG = ceil(Wo / 8) runs of eight pixels
// (the last one padded with zeros of d_out), a slot run g = (image, y, xg) is what one lane group q
// of a K block of 32 takes, so a lane's eight A values are eight neighbouring pixels of one channel
// row: d_out is staged as bf16 [channel][slot].  Its eight B values are the image pixels
// in[c][y+u][8 xg + v .. + 7], which start at any pixel: the images are therefore held KW times,
// copy v shifted left by v pixels, bf16 [v][image][c][row][WP = 8 XG], and the read is the aligned
// 16 bytes at (byte offset of the tap in copy v) + (byte offset of the slot run).  The copies are
// made inside LDS from one unshifted bf16 image (two 16-byte reads, a funnel shift per output
// word, one 16-byte write per copy), which itself arrives by coalesced loads of four pixels per
// lane; kernels wider than eight columns take the plain kernel.
// Workgroup (bx, by) sums the groups bx, bx + gridDim.x, ... for M tile mt = by / NTG and tap tiles
// 16 (by % NTG) + wave + 4 i; partial tiles and bias sums go to the caller's workspace in the layout
// of the fp32 kernel (part[bx][mt][nt][16][16], then bpart[bx][16 mt + c]) and the same second
// kernel adds them.  The bias gradient is the sum of the rounded d_out, taken from the A operands.
struct WArgs {
  const float* in;
  const float* d_out;
  float* part;
  int B, Cin, H, W, Cout, Ho, Wo, KH, KW;
  int K;            // taps Cin*KH*KW
  int MT, NT, NTG;  // tiles of the output channels and of the taps; groups of 16 tap tiles
  int XG, WP;       // runs of eight pixels per output row; 8 XG
  int WR, W4;       // pixels of a row of the unshifted staged image (a multiple of 8, >= WP + 8 and >= W); ceil(W / 4)
  int NB, groups;
  int NBK;          // K blocks of 32 slots of a full group
  int RSD, DR;      // bytes of a row of the staged d_out; its rows: min(16, Cout)
  float inv_khkw, inv_kw, inv_xg, inv_hoxg, inv_hxg, inv_cinhxg, inv_w4, inv_hw4, inv_cinhw4;
};
struct WLds {
  int goff, dy, x, raw, total;
};
__host__ __device__ inline WLds wlds_layout(const WArgs& a) {
  WLds l;
  l.goff = 0;                                // int [NBK][4]: byte offset of slot run 4 blk + q inside a copy
  l.dy = l.goff + 16 * a.NBK;                // bf16 [DR rows: the channels of the workgroup's M tile][RSD / 2]
  l.x = l.dy + a.DR * a.RSD;                 // bf16 [KW][NB][Cin][H][WP]: the shifted copies
  l.raw = l.x + 2 * a.KW * a.NB * a.Cin * a.H * a.WP;  // bf16 [NB][Cin][H][WR]: the images as they are
  l.total = l.raw + 2 * a.NB * a.Cin * a.H * a.WR;
  return l;
}

__global__ __launch_bounds__(THREADS) void wgrad_kernel(const WArgs g) {
  extern __shared__ __align__(16) char smem[];
  const WLds L = wlds_layout(g);
  int* goff = reinterpret_cast<int*>(smem + L.goff);
  char* dy = smem + L.dy;
  char* x = smem + L.x;
  char* raw = smem + L.raw;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, j = l & 15;
  const int KHKW = g.KH * g.KW, HoWo = g.Ho * g.Wo, HW = g.H * g.W, per_image = g.Cin * HW;
  const int RUNS = g.Ho * g.XG;  // slot runs per image
  const int mt = blockIdx.y / g.NTG, ntg = blockIdx.y - mt * g.NTG;
  const int rows = min(16, g.Cout - 16 * mt);

  for (int e = t; e < 4 * g.NBK; e += THREADS) {
    int off = 0;
    if (e < g.NB * RUNS) {
      int img, r, y, xg;
      divmod(e, RUNS, g.inv_hoxg, img, r);
      divmod(r, g.XG, g.inv_xg, y, xg);
      off = 2 * ((img * g.Cin * g.H + y) * g.WP + 8 * xg);
    }
    goff[e] = off;
  }
  // everything staged starts as zeros: padding rows and slots of d_out stay so, image cells that
  // a ragged first group never writes must read as finite numbers
  for (int e = t; e < (L.total - L.dy) >> 4; e += THREADS) reinterpret_cast<f4*>(dy)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};

  // this wave's tap tiles; this lane's tap of each: byte offset inside the copies
  int toff[4], ntile = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int nt = 16 * ntg + wave + 4 * i, col = 16 * nt + j;
    if (nt < g.NT) ntile = i + 1;
    toff[i] = 0;
    if (col < g.K) {
      int c, rem, u, v;
      divmod(col, KHKW, g.inv_khkw, c, rem);
      divmod(rem, g.KW, g.inv_kw, u, v);
      toff[i] = 2 * (((v * g.NB * g.Cin + c) * g.H + u) * g.WP);
    }
  }
  f4 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  const bool sums_bias = ntg == 0 && wave == 0;  // wave-uniform
  float asum = 0.0f;
  const char* arow = dy + (j < rows ? j : 0) * g.RSD + 16 * q;  // padding rows of D read row 0: never stored
  const int* gq = goff + q;

  auto stage = [&](int grp) {
    const int b0 = grp * g.NB, nb = min(g.NB, g.B - b0);
    // d_out: item (image, channel of this M tile, y, xg) -> eight pixels of one row
    const int ditems = nb * rows * RUNS;
    const float* dsrc = g.d_out + ((size_t)b0 * g.Cout + 16 * mt) * HoWo;
    for (int e = t; e < ditems; e += THREADS) {
      int img, r, co, r2, y, xg;
      divmod(e, rows * RUNS, 1.0f / (float)(rows * RUNS), img, r);
      divmod(r, RUNS, g.inv_hoxg, co, r2);
      divmod(r2, g.XG, g.inv_xg, y, xg);
      const float* sp = dsrc + ((size_t)img * g.Cout + co) * HoWo + y * g.Wo + 8 * xg;
      float v[8];
      if ((g.Wo & 3) == 0) {  // rows of whole 16-byte items
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const f4 p = 8 * xg + 4 * h < g.Wo ? reinterpret_cast<const f4*>(sp)[h] : f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int k = 0; k < 4; ++k) v[4 * h + k] = p[k];
        }
      } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = 8 * xg + k < g.Wo ? sp[k] : 0.0f;
      }
      i4 packed;
#pragma unroll
      for (int h = 0; h < 4; ++h) packed[h] = (int)pack_bf16(v[2 * h], v[2 * h + 1]);
      *reinterpret_cast<i4*>(dy + co * g.RSD + 2 * ((img * g.Ho + y) * g.WP + 8 * xg)) = packed;
    }
    // slots of images the group does not have (a ragged last group) read as zero
    const int have = nb * RUNS, missing = (g.NB - nb) * RUNS;  // in runs of eight slots
    if (missing > 0)
      for (int e = t; e < rows * missing; e += THREADS) {
        int co, k;
        divmod(e, missing, 1.0f / (float)missing, co, k);
        *reinterpret_cast<i4*>(dy + co * g.RSD + 16 * (have + k)) = i4{0, 0, 0, 0};
      }
    // images, unshifted: item (image, c, row, x4) -> four pixels, one 8-byte LDS write
    const int ritems = nb * g.Cin * g.H * g.W4;
    const float* xsrc = g.in + (size_t)b0 * per_image;
    const bool aligned_rows = (g.W & 3) == 0;
    for (int e = t; e < ritems; e += THREADS) {
      int img, r, c, r2, yy, x4;
      divmod(e, g.Cin * g.H * g.W4, g.inv_cinhw4, img, r);
      divmod(r, g.H * g.W4, g.inv_hw4, c, r2);
      divmod(r2, g.W4, g.inv_w4, yy, x4);
      const float* sp = xsrc + (size_t)img * per_image + c * HW + yy * g.W + 4 * x4;
      f4 p;
      if (aligned_rows) {
        p = *reinterpret_cast<const f4*>(sp);
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) p[k] = 4 * x4 + k < g.W ? sp[k] : 0.0f;
      }
      using i2 = int __attribute__((ext_vector_type(2)));
      *reinterpret_cast<i2*>(raw + 2 * (((img * g.Cin + c) * g.H + yy) * g.WR + 4 * x4)) =
          i2{(int)pack_bf16(p[0], p[1]), (int)pack_bf16(p[2], p[3])};
    }
  };
  // The KW shifted copies of the group's images from the unshifted one: item (image, c, row, xg).
  auto shift_copies = [&](int grp) {
    const int nb = min(g.NB, g.B - grp * g.NB), items = nb * g.Cin * g.H * g.XG;
    for (int e = t; e < items; e += THREADS) {
      int img, r, c, r2, yy, xg;
      divmod(e, g.Cin * g.H * g.XG, g.inv_cinhxg, img, r);
      divmod(r, g.H * g.XG, g.inv_hxg, c, r2);
      divmod(r2, g.XG, g.inv_xg, yy, xg);
      const int row = (img * g.Cin + c) * g.H + yy;
      const i4* rp = reinterpret_cast<const i4*>(raw + 2 * (row * g.WR + 8 * xg));
      const i4 lo = rp[0], hi = rp[1];  // pixels 8 xg .. 8 xg + 15 (WR >= WP + 8)
      const int d[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      char* dst = x + 2 * (row * g.WP + 8 * xg);
      const int copy_bytes = 2 * g.NB * g.Cin * g.H * g.WP;
#pragma unroll
      for (int v = 0; v < 8; ++v)
        if (v < g.KW) {
          i4 o;
#pragma unroll
          for (int h = 0; h < 4; ++h)
            o[h] = (v & 1) ? (int)__builtin_amdgcn_alignbit((unsigned)d[(v + 1) / 2 + h], (unsigned)d[v / 2 + h], 16)
                           : d[v / 2 + h];
          *reinterpret_cast<i4*>(dst + v * copy_bytes) = o;
        }
    }
  };

  for (int grp = blockIdx.x; grp < g.groups; grp += gridDim.x) {
    const int nb = min(g.NB, g.B - grp * g.NB), nbk = (nb * RUNS + 3) >> 2;
    lds_barrier();  // table and zeros (first pass) / the previous group's reads are complete
    stage(grp);
    lds_barrier();  // the unshifted images are complete
    shift_copies(grp);
    lds_barrier();
    if (ntile == 0) continue;  // fewer tap tiles than waves: this wave only helps with the staging
    // one block per trip; the operands of block b + 1 are read under the MFMAs of block b
    bf8 a = *reinterpret_cast<const bf8*>(arow);
    int go = gq[0];
    bf8 bv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) bv[i] = *reinterpret_cast<const bf8*>(x + toff[i] + go);
    for (int b = 0; b < nbk; ++b) {
      const int nxt = min(b + 1, nbk - 1);
      const bf8 an = *reinterpret_cast<const bf8*>(arow + 64 * nxt);
      go = gq[4 * nxt];
      bf8 bn[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) bn[i] = *reinterpret_cast<const bf8*>(x + toff[i] + go);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < ntile) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bv[i], acc[i], 0, 0, 0);
      if (sums_bias) {
        const i4 bits = __builtin_bit_cast(i4, a);
#pragma unroll
        for (int h = 0; h < 4; ++h)
          asum += __uint_as_float((unsigned)bits[h] << 16) + __uint_as_float((unsigned)bits[h] & 0xffff0000u);
      }
      a = an;
#pragma unroll
      for (int i = 0; i < 4; ++i) bv[i] = bn[i];
    }
  }
  if (sums_bias) {  // lane (j, q) summed channel j over its quarter of every block: add the four q
    asum += __shfl_xor(asum, 16, 64);
    asum += __shfl_xor(asum, 32, 64);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int nt = 16 * ntg + wave + 4 * i;
    if (i < ntile) {
      float* o = g.part + (((size_t)blockIdx.x * g.MT + mt) * g.NT + nt) * 256 + 64 * q + j;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[16 * r] = acc[i][r];
    }
  }
  if (sums_bias && q == 0) {
    float* bpart = g.part + (size_t)gridDim.x * g.MT * g.NT * 256;
    bpart[(size_t)blockIdx.x * g.MT * 16 + 16 * mt + j] = j < rows ? asum : 0.0f;
  }
}

}  // namespace igemm16
}  // namespace cnn
