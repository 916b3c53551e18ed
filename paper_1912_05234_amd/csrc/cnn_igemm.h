// General-shape convolution kernels on the fp32 matrix cores (v_mfma_f32_16x16x4_f32, wave64).
// Definitions: arXiv 1912.05234, Section 3 -- listings conv / mconv (forward), backin (input
// gradient), backweights and backbias (weight and bias gradients).  A fully connected layer is the
// same operation with a kernel as large as its input (Section 3), here H = W = KH = KW = 1.
//
// Every operation is an implicit GEMM D[M x N] = A[M x K] * B[K x N] in 16 x 16 tiles with K taken four
// at a time; lane l = 16 q + j of a wave supplies A[i = j][k = q] and B[k = q][j] and receives
// D[i = 4 q + r][j] in result register r.  The operand that is gathered (image patches) is staged in
// LDS once per group of images and addressed as (offset of the K index) + (offset of the N or M
// index), both from small LDS tables, so no index arithmetic is left in the inner loop.
//
//   forward          M = Cout          K = Cin*KH*KW        N = pixels of the group's outputs
//   input gradient   M = Cin           K = Cout*KH*KW       N = pixels of the group's inputs; the
//                    output error is staged with a zero border of (KH-1, KW-1) and the kernel is
//                    read flipped, which turns backin into a forward convolution
//   weight gradient  M = Cout          K = pixels of all images   N = Cin*KH*KW taps + one column of
//                    ones (the bias gradient)
#pragma once

#include "cnn_common.h"

namespace cnn {
namespace igemm {

using f4 = float __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f4 mfma16(float a, float b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

constexpr int THREADS = 256;  // four waves per workgroup
constexpr int WAVES = THREADS / 64;

// e / d and e % d for 0 <= e < 2^22, d >= 1, inv = 1.0f / d: the float estimate is off by at most
// one and is corrected.
__device__ __forceinline__ void divmod(int e, int d, float inv, int& quo, int& rem) {
  int qv = (int)((float)e * inv);
  int rv = e - qv * d;
  if (rv < 0) {
    --qv;
    rv += d;
  } else if (rv >= d) {
    ++qv;
    rv -= d;
  }
  quo = qv;
  rem = rv;
}

// ---- forward and input gradient -----------------------------------------------------------------------
// The staged tensor src[B][SC][SH][SW] is held in LDS per image as SC planes of LP floats with rows
// of LW floats and the data at (pady, padx) inside each plane; dst[B][M][OH][OW].
struct ConvArgs {
  const float* src;
  const float* w;     // [Cout][Cin][KH][KW]
  const float* bias;  // M values or null
  float* dst;
  int B, M, K;         // images, rows of D, reduction length SC*KH*KW
  int SC, SH, SW;      // staged tensor: channels, rows, columns
  int LW, LP, LI;      // LDS strides: row, plane, image (LI = SC*LP)
  int pady, padx;      // origin of the data inside a plane
  int KH, KW, OH, OW;  // kernel and output extents
  int NB, groups;      // images per group, number of groups
  int MT, S;           // tiles of M, steps of K
  int flip;            // 0: A[m][(c,u,v)] = w[m][c][u][v];  1: A[m][(c,u,v)] = w[c][m][KH-1-u][KW-1-v]
  int zero_fill;       // the planes have a border that must read as zero
  float inv_khkw, inv_kw, inv_ohow, inv_ow, inv_sw, inv_sh;
};
// LDS layout (floats / ints), in this order; sizes are rounded up to multiples of 4.
struct ConvLds {
  int wt, koff, bias, poff, ooff, x, total;
};
__host__ __device__ inline int round4(int v) { return (v + 3) & ~3; }
__host__ __device__ inline ConvLds conv_lds(const ConvArgs& a) {
  ConvLds l;
  l.wt = 0;                              // [MT][S][64] A operand in lane order
  l.koff = l.wt + a.MT * a.S * 64;       // [4 S] LDS offset of K index kk (0 for padding)
  l.bias = l.koff + 4 * a.S;             // [16 MT]
  l.poff = l.bias + 16 * a.MT;           // [NB*OH*OW] LDS offset of output pixel n
  l.ooff = l.poff + round4(a.NB * a.OH * a.OW);  // [NB*OH*OW] offset of pixel n in dst (channel 0)
  l.x = l.ooff + round4(a.NB * a.OH * a.OW);     // [NB*LI] staged images
  l.total = l.x + round4(a.NB * a.LI);
  return l;
}

// TP pixel tiles against the M tile whose A operands start at `wa` (lane part included): the
// operands of step s + 1 and the K offset of step s + 2 are read while step s issues.
template <int TP>
__device__ __forceinline__ void conv_tiles(f4 (&acc)[TP], const float* wa, const int* ko, const float* x,
                                           const int (&po)[TP], int S) {
  int k1 = ko[0], k2 = ko[S > 1 ? 4 : 0];
  float a = wa[0], b[TP];
#pragma unroll
  for (int t = 0; t < TP; ++t) b[t] = x[k1 + po[t]];
  for (int s = 0; s < S; ++s) {
    const int s1 = s + 1 < S ? s + 1 : S - 1, s2 = s + 2 < S ? s + 2 : S - 1;
    const int k3 = ko[4 * s2];
    const float an = wa[64 * s1];
    float bn[TP];
#pragma unroll
    for (int t = 0; t < TP; ++t) bn[t] = x[k2 + po[t]];
#pragma unroll
    for (int t = 0; t < TP; ++t) acc[t] = mfma16(a, b[t], acc[t]);
    a = an;
    k2 = k3;
#pragma unroll
    for (int t = 0; t < TP; ++t) b[t] = bn[t];
  }
}

template <int TP>
__global__ __launch_bounds__(THREADS) void conv_kernel(const ConvArgs g) {
  extern __shared__ __align__(16) float lds[];
  const ConvLds L = conv_lds(g);
  float* wt = lds + L.wt;
  int* koff = reinterpret_cast<int*>(lds + L.koff);
  float* bl = lds + L.bias;
  int* poff = reinterpret_cast<int*>(lds + L.poff);
  int* ooff = reinterpret_cast<int*>(lds + L.ooff);
  float* x = lds + L.x;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, j = l & 15;
  const int KHKW = g.KH * g.KW, OHOW = g.OH * g.OW;

  // ---- tables, once per workgroup ----
  for (int e = t; e < g.MT * g.S * 64; e += THREADS) {
    const int lane = e & 63, sidx = e >> 6, s = sidx % g.S, mt = sidx / g.S;
    const int m = 16 * mt + (lane & 15), kk = 4 * s + (lane >> 4);
    float v = 0.0f;
    if (m < g.M && kk < g.K) {
      if (!g.flip) {
        v = g.w[(size_t)m * g.K + kk];
      } else {
        int c, rem, u, vv;
        divmod(kk, KHKW, g.inv_khkw, c, rem);
        divmod(rem, g.KW, g.inv_kw, u, vv);
        v = g.w[((size_t)c * g.M + m) * KHKW + (g.KH - 1 - u) * g.KW + (g.KW - 1 - vv)];
      }
    }
    wt[e] = v;
  }
  for (int kk = t; kk < 4 * g.S; kk += THREADS) {
    int off = 0;
    if (kk < g.K) {
      int c, rem, u, vv;
      divmod(kk, KHKW, g.inv_khkw, c, rem);
      divmod(rem, g.KW, g.inv_kw, u, vv);
      off = c * g.LP + u * g.LW + vv;
    }
    koff[kk] = off;
  }
  for (int m = t; m < 16 * g.MT; m += THREADS) bl[m] = (g.bias && m < g.M) ? g.bias[m] : 0.0f;
  for (int n = t; n < g.NB * OHOW; n += THREADS) {
    int img, r, y, xx;
    divmod(n, OHOW, g.inv_ohow, img, r);
    divmod(r, g.OW, g.inv_ow, y, xx);
    poff[n] = img * g.LI + y * g.LW + xx;
    ooff[n] = img * g.M * OHOW + r;
  }
  if (g.zero_fill)
    for (int e = t; e < g.NB * g.LI; e += THREADS) x[e] = 0.0f;

  const int per_image = g.SC * g.SH * g.SW;
  for (int grp = blockIdx.x; grp < g.groups; grp += gridDim.x) {
    const int b0 = grp * g.NB, nb = min(g.NB, g.B - b0);
    const float* src = g.src + (size_t)b0 * per_image;
    __syncthreads();  // tables (first pass) / the previous group's reads are complete
    const int count = nb * per_image;
    if (!g.zero_fill) {
      for (int e = t; e < count; e += THREADS) x[e] = src[e];  // LI == per_image: a flat copy
    } else {
      for (int e = t; e < count; e += THREADS) {
        int row, xx, ic, y;
        divmod(e, g.SW, g.inv_sw, row, xx);
        divmod(row, g.SH, g.inv_sh, ic, y);
        x[ic * g.LP + (y + g.pady) * g.LW + g.padx + xx] = src[e];
      }
    }
    __syncthreads();

    const int N = nb * OHOW, PT = (N + 15) >> 4, PG = (PT + TP - 1) / TP;
    float* dst = g.dst + (size_t)b0 * g.M * OHOW;
    for (int job = wave; job < PG * g.MT; job += WAVES) {
      const int pg = job / g.MT, mt = job - pg * g.MT;
      int po[TP];
      f4 acc[TP];
      const f4 binit = *reinterpret_cast<const f4*>(&bl[16 * mt + 4 * q]);
#pragma unroll
      for (int tt = 0; tt < TP; ++tt) {
        const int n = 16 * (pg * TP + tt) + j;
        po[tt] = poff[n < N ? n : N - 1];
        acc[tt] = binit;
      }
      conv_tiles<TP>(acc, wt + (size_t)mt * g.S * 64 + l, koff + q, x, po, g.S);
#pragma unroll
      for (int tt = 0; tt < TP; ++tt) {
        const int n = 16 * (pg * TP + tt) + j;
        if (n < N) {
          float* o = dst + ooff[n] + (size_t)(16 * mt + 4 * q) * OHOW;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (16 * mt + 4 * q + r < g.M) o[(size_t)r * OHOW] = acc[tt][r];
        }
      }
    }
  }
}

// ---- weight and bias gradient --------------------------------------------------------------------------
// in[B][Cin][H][W], d_out[B][Cout][Ho][Wo].  Workgroup (bx, by) sums the images of groups bx, bx +
// gridDim.x, ... into the D tiles of M tile mt = by / NTG and N tiles 16 (by % NTG) + wave + 4 i
// (i < 4), and writes them to part[bx][mt][nt][16][16].  Column K of D is the bias gradient.
struct WgradArgs {
  const float* in;
  const float* d_out;
  float* part;
  int B, Cin, H, W, Cout, Ho, Wo, KH, KW;
  int K;          // Cin*KH*KW taps
  int MT, NT;     // tiles of Cout and of K + 1 columns
  int NTG;        // groups of 16 N tiles
  int NB, groups;
  int NP;         // pixel slots of a group: NB*Ho*Wo rounded up to a multiple of 4
  int NPS;        // row stride of the staged error, NP rounded up to 2 mod 32 (conflict-free A reads)
  float inv_khkw, inv_kw, inv_howo, inv_wo;
};
struct WgradLds {
  int pb, so, dy, x, total;
};
__host__ __device__ inline WgradLds wgrad_lds(const WgradArgs& a) {
  WgradLds l;
  l.pb = 0;                 // [NP] LDS offset of pixel slot n in x (0 for padding slots)
  l.so = l.pb + a.NP;       // [NP] offset of pixel slot n in d_out (channel 0), -1 for padding slots
  l.dy = l.so + a.NP;       // [16][NPS] output error of the M tile, zero in padding slots
  l.x = l.dy + 16 * a.NPS;  // [NB][Cin*H*W]
  l.total = l.x + round4(a.NB * a.Cin * a.H * a.W);
  return l;
}

template <int TW>
__device__ __forceinline__ void wgrad_tiles(f4 (&acc)[4], const float* da, const int* pb, const float* x,
                                            const int (&toff)[4], const bool (&ones)[4], int S) {
  int p1 = pb[0], p2 = pb[S > 1 ? 4 : 0];
  float a = da[0], b[TW];
#pragma unroll
  for (int i = 0; i < TW; ++i) b[i] = ones[i] ? 1.0f : x[p1 + toff[i]];
  for (int s = 0; s < S; ++s) {
    const int s1 = s + 1 < S ? s + 1 : S - 1, s2 = s + 2 < S ? s + 2 : S - 1;
    const int p3 = pb[4 * s2];
    const float an = da[4 * s1];
    float bn[TW];
#pragma unroll
    for (int i = 0; i < TW; ++i) bn[i] = ones[i] ? 1.0f : x[p2 + toff[i]];
#pragma unroll
    for (int i = 0; i < TW; ++i) acc[i] = mfma16(a, b[i], acc[i]);
    a = an;
    p2 = p3;
#pragma unroll
    for (int i = 0; i < TW; ++i) b[i] = bn[i];
  }
}

__global__ __launch_bounds__(THREADS) void wgrad_kernel(const WgradArgs g) {
  extern __shared__ __align__(16) float lds[];
  const WgradLds L = wgrad_lds(g);
  int* pb = reinterpret_cast<int*>(lds + L.pb);
  int* so = reinterpret_cast<int*>(lds + L.so);
  float* dy = lds + L.dy;
  float* x = lds + L.x;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, j = l & 15;
  const int KHKW = g.KH * g.KW, HoWo = g.Ho * g.Wo, HW = g.H * g.W, per_image = g.Cin * HW;
  const int mt = blockIdx.y / g.NTG, ntg = blockIdx.y - mt * g.NTG;

  for (int n = t; n < g.NP; n += THREADS) {
    int pbv = 0, sov = -1;
    if (n < g.NB * HoWo) {
      int img, r, y, xx;
      divmod(n, HoWo, g.inv_howo, img, r);
      divmod(r, g.Wo, g.inv_wo, y, xx);
      pbv = img * per_image + y * g.W + xx;
      sov = img * g.Cout * HoWo + r;
    }
    pb[n] = pbv;
    so[n] = sov;
  }
  // this lane's column of each of the wave's tiles
  int toff[4], nvalid = 0;
  bool ones[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int nt = 16 * ntg + wave + 4 * i, col = 16 * nt + j;
    if (nt < g.NT) nvalid = i + 1;
    toff[i] = 0;
    ones[i] = col == g.K;
    if (col < g.K) {
      int c, rem, u, vv;
      divmod(col, KHKW, g.inv_khkw, c, rem);
      divmod(rem, g.KW, g.inv_kw, u, vv);
      toff[i] = c * HW + u * g.W + vv;
    }
  }
  f4 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = f4{0.0f, 0.0f, 0.0f, 0.0f};

  for (int grp = blockIdx.x; grp < g.groups; grp += gridDim.x) {
    const int b0 = grp * g.NB, nb = min(g.NB, g.B - b0);
    __syncthreads();
    const float* src = g.in + (size_t)b0 * per_image;
    for (int e = t; e < g.NB * per_image; e += THREADS) x[e] = e < nb * per_image ? src[e] : 0.0f;
    const float* dsrc = g.d_out + (size_t)b0 * g.Cout * HoWo;
    const int nvalid_px = nb * HoWo;
    for (int c = 0; c < 16; ++c) {
      const int co = 16 * mt + c;
      for (int n = t; n < g.NP; n += THREADS)
        dy[c * g.NPS + n] = (co < g.Cout && n < nvalid_px) ? dsrc[so[n] + (size_t)co * HoWo] : 0.0f;
    }
    __syncthreads();
    const int S = (nvalid_px + 3) >> 2;  // slots past nvalid_px up to the next multiple of 4 are zero
    const float* da = dy + j * g.NPS + q;
    switch (nvalid) {
      case 4: wgrad_tiles<4>(acc, da, pb + q, x, toff, ones, S); break;
      case 3: wgrad_tiles<3>(acc, da, pb + q, x, toff, ones, S); break;
      case 2: wgrad_tiles<2>(acc, da, pb + q, x, toff, ones, S); break;
      case 1: wgrad_tiles<1>(acc, da, pb + q, x, toff, ones, S); break;
      default: break;
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int nt = 16 * ntg + wave + 4 * i;
    if (nt < g.NT) {
      float* o = g.part + (((size_t)blockIdx.x * g.MT + mt) * g.NT + nt) * 256 + 64 * q + j;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[16 * r] = acc[i][r];
    }
  }
}

// d_k[co][tap] and d_bias[co] = sum over the G partial tiles in ascending order of g within sixteen
// interleaved strands, the strands then combined by a fixed tree: one thread strand per output.
__global__ __launch_bounds__(THREADS) void wgrad_reduce_kernel(const float* __restrict__ part, int G, int MT,
                                                               int NT, int Cout, int K,
                                                               float* __restrict__ d_k,
                                                               float* __restrict__ d_bias) {
  __shared__ float red[THREADS];
  const int strand = threadIdx.x >> 4, el = blockIdx.x * 16 + (threadIdx.x & 15);
  const int total = Cout * (K + 1);
  float sum = 0.0f;
  int co = 0, col = 0;
  if (el < total) {
    co = el / (K + 1);
    col = el - co * (K + 1);
    const float* p = part + ((size_t)(co >> 4) * NT + (col >> 4)) * 256 + (co & 15) * 16 + (col & 15);
    const size_t gstride = (size_t)MT * NT * 256;
    for (int gi = strand; gi < G; gi += 16) sum += p[gi * gstride];
  }
  red[threadIdx.x] = sum;
  __syncthreads();
  for (int s = 8; s > 0; s >>= 1) {
    if (strand < s) red[threadIdx.x] += red[threadIdx.x + 16 * s];
    __syncthreads();
  }
  if (strand == 0 && el < total) {
    if (col < K)
      d_k[(size_t)co * K + col] = red[threadIdx.x];
    else if (d_bias)
      d_bias[co] = red[threadIdx.x];
  }
}

}  // namespace igemm
}  // namespace cnn
