// General-shape convolution kernels on the fp32 matrix cores (v_mfma_f32_16x16x4_f32, wave64).
// Definitions: arXiv 1912.05234, Section 3 -- listings conv / mconv (forward), backin (input
// gradient), backweights and backbias (weight and bias gradients).  A fully connected layer is the
// same operation with a kernel as large as its input (Section 3), here H = W = KH = KW = 1.
//
// Every operation is an implicit GEMM D[M x N] = A[M x K] * B[K x N] in 16 x 16 tiles with K taken four
// at a time (one "step"); lane l = 16 q + j of a wave supplies A[i = j][k = q] and B[k = q][j] and
// receives D[i = 4 q + r][j] in result register r.  The operand that is gathered (image patches) is
// staged in LDS once per group of images and addressed as (offset of the K index) + (offset of the N
// index), both from small LDS tables, so no index arithmetic is left in the inner loop.  Steps are
// taken in blocks of four: the dense operand and the K offsets of a block are one 16-byte LDS read
// each, and the reads of block i + 1 are issued under the matrix instructions of block i.
//
//   forward          M = Cout          K = Cin*KH*KW        N = pixels of the group's outputs
//   input gradient   M = Cin           K = Cout*KH*KW       N = pixels of the group's inputs; the
//                    output error is staged with a zero border of (KH-1, KW-1) and the kernel is
//                    read flipped, which turns backin into a forward convolution
//   weight gradient  M = Cout          K = pixels of all images   N = Cin*KH*KW taps; the bias
//                    gradient is summed while the output error is staged
//
// Column packing (forward and input gradient, few output channels): P horizontally adjacent output
// pixels x = P X + sh share one GEMM column (y, X) and take P rows (m, sh) instead.  With v' = v + sh
// the gathered operand staged[c][y+u][P X + v'] does not depend on sh, so
//   D[(m,sh)][(y,X)] = sum_{c,u,v' < KW+P-1} W[(m,sh)][(c,u,v')] * staged[c][y+u][P X + v'],
//   W[(m,sh)][(c,u,v')] = k[m][c][u][v'-sh]  (zero where v'-sh is outside 0..KW-1):
// a 16-row tile is filled by M*P rows and the number of matrix instructions falls by
// P*KW / (KW+P-1).  P = 1 is the plain form.
#pragma once

#include "cnn_common.h"

namespace cnn {
namespace igemm {

using f4 = float __attribute__((ext_vector_type(4)));
using f2 = float __attribute__((ext_vector_type(2)));
using i4 = int __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f4 mfma16(float a, float b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

constexpr int THREADS = 256;  // four waves per workgroup
constexpr int WAVES = THREADS / 64;
// Forward and input-gradient kernel: staged data of the next group of images travels through
// registers while the current group is computed, up to PFV 16-byte items or PFS 4-byte items per
// thread; what a larger group has beyond that follows in further passes of the same size after the
// group's turn has come, without overlap.  Stage modes (the weight-gradient kernel stages with
// direct global-to-LDS loads instead):
constexpr int PFV = 8, PFS = 16;  // the scalar items live in the first PFS / 4 vector registers
constexpr int STAGE_VECTOR = 1, STAGE_SCALAR = 2;

// Workgroup barrier that orders LDS accesses only: global loads and stores stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

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
__host__ __device__ inline int round4(int v) { return (v + 3) & ~3; }
// Row stride (floats) of a table read 16 bytes per lane with one row per lane: a multiple of 4 that
// is not a multiple of 8, so that eight consecutive rows start in eight different groups of four banks.
__host__ __device__ inline int row_stride(int blocks) { return 4 * blocks + ((blocks & 1) ? 0 : 4); }

// One block (four steps) of matrix instructions for NTILE accumulators: a[s] against b[s][t].
template <int NTILE>
__device__ __forceinline__ void block_mfma(f4 (&acc)[NTILE], const f4& a, const float (&b)[4][NTILE]) {
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int t = 0; t < NTILE; ++t) acc[t] = mfma16(a[s], b[s][t], acc[t]);
}
// The gathered operand of one block: b[s][t] = staged[k[s] + off[t]] (byte offsets).
template <int NTILE>
__device__ __forceinline__ void block_gather(float (&b)[4][NTILE], const char* staged, const i4& k,
                                             const int (&off)[NTILE]) {
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int t = 0; t < NTILE; ++t) b[s][t] = *reinterpret_cast<const float*>(staged + k[s] + off[t]);
}
// Asks the scheduler to issue one LDS read after each matrix instruction of a block.
template <int NTILE>
__device__ __forceinline__ void block_interleave() {
#pragma unroll
  for (int i = 0; i < 4 * NTILE; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
}
// Blocks first, first + stride, ... (count of them) of a GEMM for NTILE tiles that share the dense
// operand: `dense` points at the lane's 16-byte entry of block 0, the entries of consecutive blocks
// DSTEP entries apart; `koff` is the row of its q, indexed by block; `last` is the highest block index
// that may be read (prefetches are clamped to it).  With ASUM the lane's dense operands are also
// summed into *asum (each block once, in block order).
template <int NTILE, int DSTEP, bool ASUM = false>
__device__ __forceinline__ void gemm_blocks(f4 (&acc)[NTILE], const f4* dense, const i4* koff,
                                            const char* staged, const int (&off)[NTILE], int first,
                                            int stride, int count, int last, float* asum = nullptr) {
  if (count <= 0) return;
  auto at = [&](int i) {
    const int b = first + i * stride;
    return b < last ? b : last;
  };
  auto add = [&](const f4& a) {
    if (ASUM) *asum += (a[0] + a[1]) + (a[2] + a[3]);
  };
  i4 k0 = koff[at(0)], k1 = koff[at(1)];
  f4 a0 = dense[DSTEP * at(0)], a1;
  float b0[4][NTILE], b1[4][NTILE];
  block_gather<NTILE>(b0, staged, k0, off);
  int i = 0;
  for (; i + 2 < count; i += 2) {  // two blocks per trip; at least one more block follows
    a1 = dense[DSTEP * at(i + 1)];
    block_gather<NTILE>(b1, staged, k1, off);
    k0 = koff[at(i + 2)];
    block_mfma<NTILE>(acc, a0, b0);
    add(a0);
    block_interleave<NTILE>();
    a0 = dense[DSTEP * at(i + 2)];
    block_gather<NTILE>(b0, staged, k0, off);
    k1 = koff[at(i + 3)];
    block_mfma<NTILE>(acc, a1, b1);
    add(a1);
    block_interleave<NTILE>();
  }
  if (i + 2 == count) {  // the last two blocks: nothing left to fetch ahead
    a1 = dense[DSTEP * at(i + 1)];
    block_gather<NTILE>(b1, staged, k1, off);
    block_mfma<NTILE>(acc, a0, b0);
    add(a0);
    block_interleave<NTILE>();
    block_mfma<NTILE>(acc, a1, b1);
    add(a1);
  } else {
    block_mfma<NTILE>(acc, a0, b0);
    add(a0);
  }
}

// ---- forward and input gradient -----------------------------------------------------------------------
// The staged tensor src[B][SC][SH][SW] is held in LDS per image as SC planes of LP floats with rows
// of LW floats and the data at (pady, padx) inside each plane; dst[B][M][OH][OW].
struct ConvArgs {
  const float* src;
  const float* w;     // [Cout][Cin][KH][KW]
  const float* bias;  // M values or null
  float* dst;
  int B, M, K;         // images, output channels, reduction length SC*KH*(KW+P-1)
  int P, MR, KWP, OWP; // column packing: pixels per column, rows of D = M*P, KW+P-1, OW/P
  int SC, SH, SW;      // staged tensor: channels, rows, columns
  int LW, LP, LI;      // LDS strides: row, plane, image (LI = SC*LP)
  int pady, padx;      // origin of the data inside a plane
  int KH, KW, OH, OW;  // kernel and output extents
  int NB, groups;      // images per group, number of groups
  int MT, R;           // tiles of the MR rows; rows of a tile held in LDS: min(16, MR), row R stays zero
  int NBK, SP;         // blocks of four K steps; row stride of the two K-indexed tables (floats)
  int flip;            // 0: A[m][(c,u,v)] = w[m][c][u][v];  1: A[m][(c,u,v)] = w[c][m][KH-1-u][KW-1-v]
  int zero_fill;       // the planes have a border that must read as zero
  int stage, passes;   // STAGE_*: VECTOR needs SC*SH*SW % 4 == 0 and no border; register loads per group
  float inv_sp, inv_r1, inv_p, inv_khkwp, inv_kwp, inv_ohowp, inv_owp, inv_sw, inv_sh;
};
// LDS layout in floats, in this order.
struct ConvLds {
  int wt, koff, bias, poff, ooff, x, total;
};
__host__ __device__ inline ConvLds conv_lds(const ConvArgs& a) {
  ConvLds l;
  l.wt = 0;  // [MT*(R+1)*4 rows: M tile, row i, q][SP]: A[i][4 s + q] at [s]
  l.koff = l.wt + a.MT * (a.R + 1) * 4 * a.SP;  // [4 rows: q][SP]: byte offset of K index 4 s + q (0 for padding)
  l.bias = l.koff + 4 * a.SP;          // [16 MT]
  l.poff = l.bias + 16 * a.MT;         // [NB*OH*OWP] byte offset of column n in the staged images
  l.ooff = l.poff + round4(a.NB * a.OH * a.OWP);  // [NB*OH*OWP] offset of column n in dst (channel 0, sh 0)
  l.x = l.ooff + round4(a.NB * a.OH * a.OWP);     // [NB*LI] staged images
  l.total = l.x + round4(a.NB * a.LI);
  return l;
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
  const int KHKW = g.KH * g.KW, KHKWP = g.KH * g.KWP, OHOW = g.OH * g.OW, OHOWP = g.OH * g.OWP;

  // ---- tables, once per workgroup ----
  const int wt_total = g.MT * (g.R + 1) * 4 * g.SP;
  for (int e0 = t; e0 < wt_total; e0 += 4 * THREADS) {  // four independent loads in flight per thread
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + u * THREADS;
      v[u] = 0.0f;
      if (e < wt_total) {
        int row, s, tile, ri;
        divmod(e, g.SP, g.inv_sp, row, s);
        divmod(row >> 2, g.R + 1, g.inv_r1, tile, ri);
        const int mrow = 16 * tile + ri, kk = 4 * s + (row & 3);
        if (ri < g.R && mrow < g.MR && kk < g.K) {
          int m, sh, c, rem, uu, vp;
          divmod(mrow, g.P, g.inv_p, m, sh);
          divmod(kk, KHKWP, g.inv_khkwp, c, rem);
          divmod(rem, g.KWP, g.inv_kwp, uu, vp);
          const int vv = vp - sh;
          if (vv >= 0 && vv < g.KW)
            v[u] = !g.flip ? g.w[((size_t)m * g.SC + c) * KHKW + uu * g.KW + vv]
                           : g.w[((size_t)c * g.M + m) * KHKW + (g.KH - 1 - uu) * g.KW + (g.KW - 1 - vv)];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (e0 + u * THREADS < wt_total) wt[e0 + u * THREADS] = v[u];
  }
  for (int e = t; e < 4 * g.SP; e += THREADS) {
    int qq, s;
    divmod(e, g.SP, g.inv_sp, qq, s);
    const int kk = 4 * s + qq;
    int off = 0;
    if (kk < g.K) {
      int c, rem, u, vp;
      divmod(kk, KHKWP, g.inv_khkwp, c, rem);
      divmod(rem, g.KWP, g.inv_kwp, u, vp);
      off = 4 * (c * g.LP + u * g.LW + vp);
    }
    koff[e] = off;
  }
  for (int mrow = t; mrow < 16 * g.MT; mrow += THREADS) {
    int m, sh;
    divmod(mrow, g.P, g.inv_p, m, sh);
    bl[mrow] = (g.bias && mrow < g.MR) ? g.bias[m] : 0.0f;
  }
  for (int n = t; n < g.NB * OHOWP; n += THREADS) {
    int img, r, y, xx;
    divmod(n, OHOWP, g.inv_ohowp, img, r);
    divmod(r, g.OWP, g.inv_owp, y, xx);
    poff[n] = 4 * (img * g.LI + y * g.LW + g.P * xx);
    ooff[n] = img * g.M * OHOW + y * g.OW + g.P * xx;
  }
  // byte offset in dst of this lane's result register r in M tile 0 (packed forms have one M tile)
  unsigned ro0[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int m, sh;
    divmod(4 * q + r, g.P, g.inv_p, m, sh);
    ro0[r] = 4u * (unsigned)(m * OHOW + sh);
  }
  if (g.zero_fill)
    for (int e = t; e < g.NB * g.LI; e += THREADS) x[e] = 0.0f;

  const int per_image = g.SC * g.SH * g.SW;
  // LDS index of staged element e of a group (flat, or into the bordered planes)
  auto target = [&](int e) {
    if (!g.zero_fill) return e;
    int row, xx, ic, y;
    divmod(e, g.SW, g.inv_sw, row, xx);
    divmod(row, g.SH, g.inv_sh, ic, y);
    return ic * g.LP + (y + g.pady) * g.LW + g.padx + xx;
  };
  f4 pv[PFV];
  int ptgt[PFS];
  if (g.stage == STAGE_SCALAR) {
#pragma unroll
    for (int i = 0; i < PFS; ++i) {
      const int e = t + THREADS * i;
      ptgt[i] = e < g.NB * per_image ? target(e) : 0;
    }
  }
  // Pass r over group grp: loads into registers ...
  auto issue = [&](int grp, int r) {
    const int b0 = grp * g.NB, count = min(g.NB, g.B - b0) * per_image;
    const float* src = g.src + (size_t)b0 * per_image;
    if (g.stage == STAGE_VECTOR) {
      const int first = r * (THREADS * PFV) + t;
#pragma unroll
      for (int i = 0; i < PFV; ++i)
        if (first + THREADS * i < count >> 2) pv[i] = reinterpret_cast<const f4*>(src)[first + THREADS * i];
    } else {
      const int first = r * (THREADS * PFS) + t;
#pragma unroll
      for (int i = 0; i < PFS; ++i)
        if (first + THREADS * i < count) pv[i >> 2][i & 3] = src[first + THREADS * i];
    }
  };
  // ... and from there into LDS (the targets of the first pass are kept in registers).
  auto commit = [&](int grp, int r) {
    const int b0 = grp * g.NB, count = min(g.NB, g.B - b0) * per_image;
    if (g.stage == STAGE_VECTOR) {
      const int first = r * (THREADS * PFV) + t;
#pragma unroll
      for (int i = 0; i < PFV; ++i)
        if (first + THREADS * i < count >> 2) reinterpret_cast<f4*>(x)[first + THREADS * i] = pv[i];
    } else if (r == 0) {
#pragma unroll
      for (int i = 0; i < PFS; ++i)
        if (t + THREADS * i < count) x[ptgt[i]] = pv[i >> 2][i & 3];
    } else {
      const int first = r * (THREADS * PFS) + t;
#pragma unroll
      for (int i = 0; i < PFS; ++i)
        if (first + THREADS * i < count) x[target(first + THREADS * i)] = pv[i >> 2][i & 3];
    }
  };

  if ((int)blockIdx.x < g.groups) issue(blockIdx.x, 0);
  for (int grp = blockIdx.x; grp < g.groups; grp += gridDim.x) {
    const int b0 = grp * g.NB, nb = min(g.NB, g.B - b0);
    lds_barrier();  // tables (first pass) / the previous group's reads are complete
    commit(grp, 0);
    for (int r = 1; r < g.passes; ++r) {  // what did not fit into the registers: no overlap
      issue(grp, r);
      commit(grp, r);
    }
    lds_barrier();
    if (grp + (int)gridDim.x < g.groups) issue(grp + gridDim.x, 0);

    const int N = nb * OHOWP, PT = (N + 15) >> 4, PG = (PT + TP - 1) / TP;
    char* dst = reinterpret_cast<char*>(g.dst + (size_t)b0 * g.M * OHOW);  // byte offsets below fit 32 bits
    for (int job = wave; job < PG * g.MT; job += WAVES) {
      const int pg = job / g.MT, mt = job - pg * g.MT;
      const int nrow = g.MR - 16 * mt - 4 * q;  // result registers r < nrow of this lane are rows of D
      unsigned ro[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) ro[r] = ro0[r] + 64u * (unsigned)(mt * OHOW);
      const bool full = 16 * (pg * TP + TP) <= N;  // no padding pixels in this job's tiles
      int po[TP];
      unsigned oo[TP];
      f4 acc[TP];
      const f4 binit = *reinterpret_cast<const f4*>(&bl[16 * mt + 4 * q]);
#pragma unroll
      for (int tt = 0; tt < TP; ++tt) {
        const int n = 16 * (pg * TP + tt) + j, nn = n < N ? n : N - 1;
        po[tt] = poff[nn];
        oo[tt] = 4u * (unsigned)ooff[nn];
        acc[tt] = binit;
      }
      const int arow = (mt * (g.R + 1) + (16 * mt + j < g.MR ? j : g.R)) * 4 + q;
      gemm_blocks<TP, 1>(acc, reinterpret_cast<const f4*>(wt + (size_t)arow * g.SP),
                      reinterpret_cast<const i4*>(koff + q * g.SP), reinterpret_cast<const char*>(x), po, 0, 1,
                      g.NBK, g.NBK - 1);
      if (full && (g.P & 3) == 0) {
        // four (or a multiple of four) pixels per column: the lane's four result registers are
        // horizontal neighbours of one channel, stored as one 16-byte item (the wide stores carry
        // the non-temporal hint: worth 5 % where the kernel is bound by its stores; the 4-byte
        // stores below must not, they rely on the cache to merge them into lines)
        if (nrow > 0) {
#pragma unroll
          for (int tt = 0; tt < TP; ++tt)
            __builtin_nontemporal_store(acc[tt], reinterpret_cast<f4*>(dst + (oo[tt] + ro[0])));
        }
      } else if (full && OHOW == 1 && (g.M & 3) == 0) {
        // one pixel per image (the fully connected form): the lane's four result registers are
        // four consecutive channels, which are neighbours in memory
        if (nrow > 0) {
#pragma unroll
          for (int tt = 0; tt < TP; ++tt) *reinterpret_cast<f4*>(dst + (oo[tt] + ro[0])) = acc[tt];
        }
      } else if (full && (g.P & 1) == 0) {
        // an even number of pixels per column: result registers (0, 1) and (2, 3) are horizontal
        // neighbours of one channel, stored as 8-byte items (sixteen lanes fill 128 consecutive
        // bytes when P = 2)
#pragma unroll
        for (int r = 0; r < 4; r += 2)
          if (r < nrow) {
#pragma unroll
            for (int tt = 0; tt < TP; ++tt)
              __builtin_nontemporal_store(f2{acc[tt][r], acc[tt][r + 1]},
                                          reinterpret_cast<f2*>(dst + (oo[tt] + ro[r])));
          }
      } else if (full) {  // wave-uniform: the common case carries no per-pixel predicates
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (r < nrow) {
#pragma unroll
            for (int tt = 0; tt < TP; ++tt)
              *reinterpret_cast<float*>(dst + (oo[tt] + ro[r])) = acc[tt][r];
          }
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (r < nrow) {
#pragma unroll
            for (int tt = 0; tt < TP; ++tt)
              if (16 * (pg * TP + tt) + j < N)
                *reinterpret_cast<float*>(dst + (oo[tt] + ro[r])) = acc[tt][r];
          }
      }
    }
  }
}

// ---- weight and bias gradient --------------------------------------------------------------------------
// in[B][Cin][H][W], d_out[B][Cout][Ho][Wo].  Workgroup (bx, by) sums the images of groups bx, bx +
// gridDim.x, ... for M tile mt = by / NTG and the tap tiles of group ntg = by % NTG.  With three or
// more tap tiles in all, wave w owns tiles 16 ntg + w + 4 i (i < 4) and KS = 1; with two (one) tap
// tiles the waves split the pixels as well: tile w % 2 (0), K slice w / 2 (w) of KS = 2 (4), a slice
// taking every KS-th block; the slices of a tile are added through LDS at the end.  Results go to
// part[bx][mt][nt][16][16]; the waves that own tile 0 also sum their A operands, the bias gradient,
// into bpart[bx][16 mt + c] (bpart follows part).
//
// With column packing (few output channels, P > 1) the rows are (co, sh), a pixel slot is the group
// (y, X) of P adjacent pixels and the columns are the shifted taps (ci, u, v' < KW+P-1):
//   T[(co,sh)][(ci,u,v')] = sum_{slots} d_out[co][y][P X + sh] * in[ci][y+u][P X + v'],
//   d_k[co][ci][u][v] = sum_sh T[(co,sh)][(ci,u,v+sh)]        (the second kernel adds the P terms).
//
// K runs over the pixel slots n of a group (image-major, padded with zeros to whole blocks of 16).
// Step s4 of block blk takes, in lane group q, slot n = 16 blk + 4 q + s4: a lane's four A values of a
// block are then consecutive pixels of one channel, so the output error is staged as it lies in
// memory, one row per channel.
//
// Staging uses the direct global-to-LDS load: a wave's instruction moves 64 items of 16 or 4 bytes
// (4 when an image or a map is not a multiple of four floats, or the rows are packed) from per-lane
// addresses to consecutive bytes of LDS, with no registers and no LDS write instructions in between.  Two LDS
// buffers alternate: the loads of group i + 1 are issued before the matrix instructions of group i.
struct WgradArgs {
  const float* in;
  const float* d_out;
  float* part;
  int B, Cin, H, W, Cout, Ho, Wo, KH, KW;
  int P, MR, KWP, WOP;  // column packing as in the forward form: rows (co, sh) = Cout*P, KW+P-1, Wo/P
  int K;          // columns of D: the Cin*KH*KWP (shifted) taps
  int MT, NT;     // tiles of the MR rows and of the K columns
  int NTG;        // groups of 16 column tiles
  int KS;         // K slices per workgroup
  int R;          // rows of the staged error: min(16, MR); row R stays zero
  int NB, groups;
  int NBK, NPS;   // blocks of 16 pixel slots per full group; row stride of the staged error (floats)
  int XS;         // floats of one staged image buffer (whole load instructions)
  int vec_x;      // 16-byte items for the images (Cin*H*W a multiple of 4), else 4-byte
  int vec_d;      // 16-byte items for the output error (P = 1 and Ho*Wo a multiple of 4), else 4-byte
  float inv_p, inv_khkwp, inv_kwp, inv_spi, inv_wop;
};
struct WgradLds {
  int pb, buf, dy, x, buf_floats, total;  // dy and x are offsets inside a buffer
};
// Row stride of the staged error: 16-byte reads by eight lanes of consecutive channels then fall
// into eight different groups of four banks.
__host__ __device__ inline int error_row_stride(int blocks) { return 16 * blocks + 4; }
__host__ __device__ inline WgradLds wgrad_lds(const WgradArgs& a) {
  WgradLds l;
  l.pb = 0;                  // [4 rows: q][NBK][4] byte offset in x of slot 16 blk + 4 q + s4 (0 for padding)
  l.buf = l.pb + 16 * a.NBK;  // two buffers of buf_floats each:
  l.dy = 0;                  //   [R + 1 rows: channel][NPS] output error by pixel slot
  l.x = (a.R + 1) * a.NPS;   //   [XS] images of the group
  l.buf_floats = l.x + a.XS;
  l.total = l.buf + 2 * l.buf_floats;
  const int handover = l.buf + WAVES * (256 + 16);  // the K slices' tiles and bias sums meet here at the end
  if (l.total < handover) l.total = handover;
  return l;
}

// One direct global-to-LDS load: lane l moves VB bytes from its own address `src` to lds_base + l VB
// (lds_base must be the same in every lane).  Counted by vmcnt like any vector memory load.
template <int VB>
__device__ __forceinline__ void load_to_lds(const float* src, float* lds_base);
template <>
__device__ __forceinline__ void load_to_lds<16>(const float* src, float* lds_base) {
  __builtin_amdgcn_global_load_lds(src, lds_base, 16, 0, 0);
}
template <>
__device__ __forceinline__ void load_to_lds<4>(const float* src, float* lds_base) {
  __builtin_amdgcn_global_load_lds(src, lds_base, 4, 0, 0);
}

template <int VBX, int VBD>  // bytes per lane of a staging load: images, output error
__global__ __launch_bounds__(THREADS) void wgrad_kernel(const WgradArgs g) {
  extern __shared__ __align__(16) float lds[];
  constexpr int VX = VBX / 4, CHX = 64 * VX;  // floats per lane and per load instruction, images
  constexpr int VD = VBD / 4, CHD = 64 * VD;  // ... output error
  const WgradLds L = wgrad_lds(g);
  int* pb = reinterpret_cast<int*>(lds + L.pb);
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, j = l & 15;
  const int KHKWP = g.KH * g.KWP, HoWo = g.Ho * g.Wo, SPI = g.Ho * g.WOP, HW = g.H * g.W, per_image = g.Cin * HW;
  const int mt = blockIdx.y / g.NTG, ntg = blockIdx.y - mt * g.NTG;
  const int rows = min(16, g.MR - 16 * mt);

  for (int n = t; n < 16 * g.NBK; n += THREADS) {
    int pbv = 0;
    if (n < g.NB * SPI) {
      int img, r, y, xx;
      divmod(n, SPI, g.inv_spi, img, r);
      divmod(r, g.WOP, g.inv_wop, y, xx);
      pbv = 4 * (img * per_image + y * g.W + g.P * xx);
    }
    pb[((((n >> 2) & 3) * g.NBK + (n >> 4)) << 2) + (n & 3)] = pbv;
  }
  // Both buffers start as zeros: the zero row stays so, and image cells that a ragged first group
  // never loads must read as finite numbers (they meet zeros of the output error).
  for (int e = t; e < 2 * L.buf_floats; e += THREADS) lds[L.buf + e] = 0.0f;
  lds_barrier();

  // this wave's tiles and K slice; this lane's column (tap) of each tile
  const int tile0 = g.KS == 1 ? wave : g.KS == 2 ? (wave & 1) : 0;
  const int slice = g.KS == 1 ? 0 : g.KS == 2 ? (wave >> 1) : wave;
  int toff[4], ntile = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int nt = 16 * ntg + tile0 + 4 * i, col = 16 * nt + j;
    if (nt < g.NT && (g.KS == 1 || i == 0)) ntile = i + 1;
    toff[i] = 0;
    if (col < g.K) {
      int c, rem, u, vp;
      divmod(col, KHKWP, g.inv_khkwp, c, rem);
      divmod(rem, g.KWP, g.inv_kwp, u, vp);
      toff[i] = 4 * (c * HW + u * g.W + vp);
    }
  }
  f4 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  const bool sums_bias = ntg == 0 && tile0 == 0;  // wave-uniform
  float asum = 0.0f;
  const int arow = (j < rows ? j : g.R) * g.NPS + 4 * q;
  const i4* koff = reinterpret_cast<const i4*>(pb) + q * g.NBK;

  // Source offset (floats, channel 0 and shift 0 of the group) of the lane's item in chunk
  // wave + 4 i of a row of the output error: fixed for the whole kernel.
  constexpr int DCH = 4;  // chunks of a row per wave: rows of up to 16 CHD slots
  int soff[DCH];
#pragma unroll
  for (int i = 0; i < DCH; ++i) {
    const int n = (wave + WAVES * i) * CHD + l * VD;
    soff[i] = 0;
    if (n < g.NB * SPI) {
      int img, r, y, xx;
      divmod(n, SPI, g.inv_spi, img, r);
      divmod(r, g.WOP, g.inv_wop, y, xx);
      soff[i] = img * g.Cout * HoWo + y * g.Wo + g.P * xx;
    }
  }
  // Loads of group grp into buffer `buf` (LDS float offset).
  auto issue = [&](int grp, int buf) {
    const int b0 = grp * g.NB, nb = min(g.NB, g.B - b0), count = nb * per_image, npx = nb * SPI;
    const float* src = g.in + (size_t)b0 * per_image;
    // images: items past the group's data re-read its last item (the cells they fill meet zeros)
    for (int c = wave; c * CHX < count; c += WAVES) {
      const int e = min(c * CHX + l * VX, count - VX);
      load_to_lds<VBX>(src + e, lds + buf + L.x + c * CHX);
    }
    // output error: row by row, lanes past the group's slots load nothing (zeroed below)
    // (packed rows exist only with one M tile, so row r of the tile is row r of D)
    const float* dsrc = g.d_out + ((size_t)b0 * g.Cout + 16 * mt) * HoWo;  // row 0: channel 16 mt, shift 0
    for (int r = 0, sh = 0; r < rows; ++r) {
      if (r > 0) {  // next row: the next shift of the same channel, or the next channel
        if (++sh == g.P) {
          sh = 0;
          dsrc += HoWo - (g.P - 1);
        } else {
          dsrc += 1;
        }
      }
#pragma unroll
      for (int i = 0; i < DCH; ++i) {
        const int c = wave + WAVES * i;
        if (c * CHD < npx) {  // wave-uniform
          if (c * CHD + l * VD < npx) load_to_lds<VBD>(dsrc + soff[i], lds + buf + L.dy + r * g.NPS + c * CHD);
        }
      }
    }
    // slots npx .. 16 nbk - 1 of every row read as zero
    const int nbk = (npx + 15) >> 4, tail = 16 * nbk - npx;
    for (int e = t; e < rows * tail; e += THREADS) {
      int r, k;
      divmod(e, tail, 1.0f / (float)tail, r, k);
      lds[buf + L.dy + r * g.NPS + npx + k] = 0.0f;
    }
  };

  int cur = L.buf;
  if ((int)blockIdx.x < g.groups) issue(blockIdx.x, cur);
  for (int grp = blockIdx.x; grp < g.groups; grp += gridDim.x) {
    const int nbk = (min(g.NB, g.B - grp * g.NB) * SPI + 15) >> 4;
    __builtin_amdgcn_s_waitcnt(0);  // this wave's loads have landed in LDS
    lds_barrier();                  // ... and everybody's; the other buffer is no longer read
    const int nxt = cur == L.buf ? L.buf + L.buf_floats : L.buf;
    if (grp + (int)gridDim.x < g.groups) issue(grp + gridDim.x, nxt);
    const int count = nbk > slice ? (nbk - slice + g.KS - 1) / g.KS : 0;
    const f4* dense = reinterpret_cast<const f4*>(lds + cur + L.dy + arow);
    const char* xb = reinterpret_cast<const char*>(lds + cur + L.x);
    if (sums_bias) {
      switch (ntile) {
        case 4: gemm_blocks<4, 4, true>(acc, dense, koff, xb, toff, slice, g.KS, count, nbk - 1, &asum); break;
        case 3: {
          f4(&a3)[3] = reinterpret_cast<f4(&)[3]>(acc);
          const int(&t3)[3] = reinterpret_cast<const int(&)[3]>(toff);
          gemm_blocks<3, 4, true>(a3, dense, koff, xb, t3, slice, g.KS, count, nbk - 1, &asum);
          break;
        }
        case 2: {
          f4(&a2)[2] = reinterpret_cast<f4(&)[2]>(acc);
          const int(&t2)[2] = reinterpret_cast<const int(&)[2]>(toff);
          gemm_blocks<2, 4, true>(a2, dense, koff, xb, t2, slice, g.KS, count, nbk - 1, &asum);
          break;
        }
        case 1: {
          f4(&a1)[1] = reinterpret_cast<f4(&)[1]>(acc);
          const int(&t1)[1] = reinterpret_cast<const int(&)[1]>(toff);
          gemm_blocks<1, 4, true>(a1, dense, koff, xb, t1, slice, g.KS, count, nbk - 1, &asum);
          break;
        }
        default: break;
      }
    } else {
      switch (ntile) {
        case 4: gemm_blocks<4, 4>(acc, dense, koff, xb, toff, slice, g.KS, count, nbk - 1); break;
        case 3: {
          f4(&a3)[3] = reinterpret_cast<f4(&)[3]>(acc);
          const int(&t3)[3] = reinterpret_cast<const int(&)[3]>(toff);
          gemm_blocks<3, 4>(a3, dense, koff, xb, t3, slice, g.KS, count, nbk - 1);
          break;
        }
        case 2: {
          f4(&a2)[2] = reinterpret_cast<f4(&)[2]>(acc);
          const int(&t2)[2] = reinterpret_cast<const int(&)[2]>(toff);
          gemm_blocks<2, 4>(a2, dense, koff, xb, t2, slice, g.KS, count, nbk - 1);
          break;
        }
        case 1: {
          f4(&a1)[1] = reinterpret_cast<f4(&)[1]>(acc);
          const int(&t1)[1] = reinterpret_cast<const int(&)[1]>(toff);
          gemm_blocks<1, 4>(a1, dense, koff, xb, t1, slice, g.KS, count, nbk - 1);
          break;
        }
        default: break;
      }
    }
    cur = nxt;
  }
  if (sums_bias) {  // lane (j, q) summed channel j over its quarter of every block: add the four q
    asum += __shfl_xor(asum, 16, 64);
    asum += __shfl_xor(asum, 32, 64);
  }
  if (g.KS > 1) {
    // The K slices of a tile meet in LDS (the staging buffers are dead): slices 1.. hand their tile
    // (one per wave when K is split) and bias sums to the wave of slice 0, which adds them in
    // slice order, so the workgroup writes one partial per tile.
    float* xch = lds + L.buf;
    lds_barrier();  // every wave has left the buffers
    if (slice > 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) xch[wave * 256 + 64 * r + l] = acc[0][r];
      if (sums_bias && q == 0) xch[WAVES * 256 + wave * 16 + j] = asum;
    }
    lds_barrier();
    if (slice == 0) {
      for (int sl = 1; sl < g.KS; ++sl) {
        const int other = g.KS == 2 ? wave + 2 * sl : sl;  // the wave that ran slice sl of this tile
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[0][r] += xch[other * 256 + 64 * r + l];
        if (sums_bias && q == 0) asum += xch[WAVES * 256 + other * 16 + j];
      }
    }
  }
  if (slice == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int nt = 16 * ntg + tile0 + 4 * i;
      if (i < ntile) {
        float* o = g.part + (((size_t)blockIdx.x * g.MT + mt) * g.NT + nt) * 256 + 64 * q + j;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[16 * r] = acc[i][r];
      }
    }
    if (sums_bias && q == 0) {
      float* bpart = g.part + (size_t)gridDim.x * g.MT * g.NT * 256;
      bpart[(size_t)blockIdx.x * g.MT * 16 + 16 * mt + j] = asum;
    }
  }
}

// d_k[co][ci][u][v] = sum over the GP partial tiles and the P shifts of T[(co,sh)][(ci,u,v+sh)];
// d_bias[co] = sum over the GP partial bias rows and the P shifts.  A workgroup takes `epw` outputs
// (4, 8 or 16: few outputs are spread over more workgroups); THREADS / epw interleaved strands walk
// the partials in ascending order, eight loads in flight (the walk is bound by load latency), and
// are combined by a fixed tree.
__global__ __launch_bounds__(THREADS) void wgrad_reduce_kernel(const float* __restrict__ part, int GP, int MT,
                                                               int NT, int Cout, int Cin, int KH, int KW,
                                                               int P, int epw, float* __restrict__ d_k,
                                                               float* __restrict__ d_bias) {
  __shared__ float red[THREADS];
  const int strands = THREADS / epw;
  const int strand = threadIdx.x / epw, el = blockIdx.x * epw + threadIdx.x % epw;
  const int KWP = KW + P - 1, nk = Cout * Cin * KH * KW, total = nk + (d_bias ? Cout : 0);
  float sum = 0.0f;
  if (el < total) {
    for (int sh = 0; sh < P; ++sh) {
      const float* p;
      size_t stride;
      if (el < nk) {
        const int v = el % KW, cu = (el / KW) % (Cin * KH), co = el / (KW * Cin * KH);
        const int row = co * P + sh, col = cu * KWP + v + sh;
        p = part + ((size_t)(row >> 4) * NT + (col >> 4)) * 256 + (row & 15) * 16 + (col & 15);
        stride = (size_t)MT * NT * 256;
      } else {
        p = part + (size_t)GP * MT * NT * 256 + (size_t)(el - nk) * P + sh;
        stride = (size_t)MT * 16;
      }
      int gi = strand;
      for (; gi + 7 * strands < GP; gi += 8 * strands) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = p[(gi + strands * k) * stride];
#pragma unroll
        for (int k = 0; k < 8; ++k) sum += v[k];
      }
      for (; gi < GP; gi += strands) sum += p[gi * stride];
    }
  }
  red[threadIdx.x] = sum;
  __syncthreads();
  for (int s = strands / 2; s > 0; s >>= 1) {
    if (strand < s) red[threadIdx.x] += red[threadIdx.x + epw * s];
    __syncthreads();
  }
  if (strand == 0 && el < total) {
    if (el < nk)
      d_k[el] = red[threadIdx.x];
    else
      d_bias[el - nk] = red[threadIdx.x];
  }
}

}  // namespace igemm
}  // namespace cnn
