// Convolution calls for the shapes of the network's own two convolution layers, ONE WAVE PER IMAGE,
// in the GEMM forms of the fused training step (arXiv 1912.05234, Section 3: listings conv / mconv,
// backweights, backbias).  An image of these layers is small enough for one wave to hold in its LDS,
// which saves the barriers and the staging for shared groups of images that the general kernels
// (cnn_igemm.h) pay; eight waves per workgroup, two workgroups per compute unit.
//
// namespace conv2: six input and twelve output maps, 5 x 5 kernel, 12 x 12 input
//   forward          M = 64 output pixels in four tiles, N = 12(16) maps, K = 150(152) taps: 152
//                    v_mfma_f32_16x16x4_f32 per image; the image's 864 inputs are staged in the
//                    wave's LDS, the weights sit in LDS as the instruction's B operand
//   weight gradient  M = 12(16) maps, N = 150(160) taps in ten tiles, K = 64 pixels: 160 per image;
//                    the output error is the A operand straight from global memory, the sums stay
//                    in registers over all of a wave's images; the eight waves of a workgroup are
//                    added through LDS in a fixed order and the workgroup writes one set of partial
//                    tiles in the layout of the general kernel, whose second kernel adds the
//                    workgroups' partials
//   (the input gradient of this shape is cnn_col2im.h)
// namespace conv1: one input and six output maps, 5 x 5 kernel, 28 x 28 input: forward and weight
//   gradient as GEMMs over pixel pairs, 144 per image each, and the input gradient on the vector
//   unit; see there.
// Pixel order and operand layouts are those of cnn_wave.h (fwd_tap, fwd_imm, c1f_*, c1g_*); only such
// index helpers and GEMM inner loops are shared with the fused step.
#pragma once

#include "cnn_wave.h"

namespace cnn {
namespace conv2 {

constexpr int WAVES_PER_GROUP = 8, THREADS = 64 * WAVES_PER_GROUP;
constexpr int CIN = 6, COUT = 12, TAPS = CIN * 25, IN_FLOATS = NS1, OUT_FLOATS = COUT * 64;
inline bool shape_fits(int Cin, int H, int W, int Cout, int KH, int KW) {
  return Cin == CIN && Cout == COUT && KH == 5 && KW == 5 && H == 12 && W == 12;
}

// One image's input as 216 16-byte pieces in registers (the fourth only in lanes 0..23).
struct Input {
  f4 a, b, c, d;
};
__device__ __forceinline__ Input load_input(const float* __restrict__ in, size_t n) {
  const f4* src = reinterpret_cast<const f4*>(in + n * IN_FLOATS);
  const int l = threadIdx.x & 63;
  Input x;
  x.a = src[l];
  x.b = src[l + 64];
  x.c = src[l + 128];
  x.d = src[l < 24 ? l + 192 : l];
  return x;
}
__device__ __forceinline__ void store_input(float* lds, const Input& x) {
  const int l = threadIdx.x & 63;
  f4* dst = reinterpret_cast<f4*>(lds);
  dst[l] = x.a;
  dst[l + 64] = x.b;
  dst[l + 128] = x.c;
  if (l < 24) dst[l + 192] = x.d;
}

// ---- forward ---------------------------------------------------------------------------------------------
constexpr int FWD_IN = IN_FLOATS + 288;  // the padded K steps read up to 1152 floats from the start (zero weights)
struct __align__(16) FwdLds {
  float tab[38 * 64];  // B operand, [K step][lane]: k[j = lane % 16][fwd_tap(step, lane / 16)]
  float bias[16];
  float in[WAVES_PER_GROUP][FWD_IN];
};
__global__ __launch_bounds__(THREADS) void forward_kernel(const float* __restrict__ in, const float* __restrict__ k,
                                                          const float* __restrict__ bias, float* __restrict__ out,
                                                          int B) {
  __shared__ FwdLds lds;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  for (int i = t; i < 38 * 64; i += THREADS) {
    const int lane = i & 63, tap = fwd_tap(i >> 6, lane >> 4), j = lane & 15;
    lds.tab[i] = j < COUT && tap >= 0 ? k[j * TAPS + tap] : 0.0f;
  }
  if (t < 16) lds.bias[t] = bias && t < COUT ? bias[t] : 0.0f;
  float* x = lds.in[wave];
  for (int e = IN_FLOATS + l; e < FWD_IN; e += 64) x[e] = 0.0f;  // finite filler behind the image
  __syncthreads();
  const float* tl = lds.tab + l;
  const int pp = 12 * ((n16 & 3) >> 1) + 2 * (n16 >> 2) + (n16 & 1);
  const float* a12 = x + pp + 12 * q;
  const float* a1 = x + pp + q;
  const float* a144 = x + pp + 144 * q;
  const float b2 = lds.bias[n16];
  const size_t G = (size_t)gridDim.x * WAVES_PER_GROUP, first = (size_t)blockIdx.x * WAVES_PER_GROUP + wave;
  Input cur;
  if (first < (size_t)B) cur = load_input(in, first);
  for (size_t n = first; n < (size_t)B; n += G) {
    store_input(x, cur);
    wave_sync();
    if (n + G < (size_t)B) cur = load_input(in, n + G);  // in flight during this image
    f4 acc[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[mt] = f4{b2, b2, b2, b2};
    float opa[3][4], opw[3];
    auto load_step = [&](int s, float (&oa)[4], float& ow) {
      const float* base = s < 30 ? a12 : s < 36 ? a1 : a144;
      ow = tl[s * 64];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) oa[mt] = base[fwd_imm(s) + 24 * mt];
    };
    load_step(0, opa[0], opw[0]);
    load_step(1, opa[1], opw[1]);
#pragma unroll
    for (int s = 0; s < 38; ++s) {
      if (s + 2 < 38) load_step(s + 2, opa[(s + 2) % 3], opw[(s + 2) % 3]);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) acc[mt] = mfma16(opa[s % 3][mt], opw[s % 3], acc[mt]);
      if (s + 2 < 38) __builtin_amdgcn_sched_group_barrier(0x100, 5, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
    wave_sync();  // the reads of this image come before the next image's stores
    // register r of tile mt is pixel (y, x) = (2 mt + r / 2, 2 q + r % 2) of map n16: two 8-byte stores per tile
    if (n16 < COUT) {
      float* dst = out + n * OUT_FLOATS + n16 * 64 + 2 * q;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        *reinterpret_cast<float2*>(dst + 16 * mt) = float2{acc[mt][0], acc[mt][1]};
        *reinterpret_cast<float2*>(dst + 16 * mt + 8) = float2{acc[mt][2], acc[mt][3]};
      }
    }
  }
}

// ---- weight and bias gradient -------------------------------------------------------------------------------
constexpr int ACC_FLOATS = 10 * 4 * 64;  // a wave's sums: [tile nt][register r][lane]
struct __align__(16) WgradLds {
  int k2b[10][64];                           // first s1 cell of tap 16 nt + lane % 16 for pixel quarter lane / 16
  float x[WAVES_PER_GROUP][IN_FLOATS];
  float comb[WAVES_PER_GROUP / 2][ACC_FLOATS];  // cross-wave sums
  float bsum[WAVES_PER_GROUP][64];
};
// part: [gridDim.x][10 tiles][16 rows j][16 columns] then the bias rows [gridDim.x][16] (the layout
// igemm::wgrad_reduce_kernel reads with MT = 1, NT = 10, P = 1).
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void bwd_weight_kernel(const float* __restrict__ in,
                                                             const float* __restrict__ d_out,
                                                             float* __restrict__ part, int B) {
  __shared__ WgradLds lds;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  for (int e = t; e < 640; e += THREADS) {
    const int nt = e >> 6, lane = e & 63, tap = 16 * nt + (lane & 15);
    const int c = tap / 25, rem = tap - 25 * c, u = rem / 5, v = rem - 5 * u;
    lds.k2b[nt][lane] = (tap < TAPS ? c * 144 + u * 12 + v : 0) + 2 * (lane >> 4);
  }
  __syncthreads();
  float* x = lds.x[wave];
  const float* bsrc[10];
#pragma unroll
  for (int nt = 0; nt < 10; ++nt) bsrc[nt] = x + lds.k2b[nt][l];
  // A operand: lane (q, n16) holds d_out[map n16][pixel 16 S + 4 q + r] = (y, x) = (2 S + r / 2, 2 q + r % 2);
  // the lanes of the padding rows 12..15 read map 11 (their result rows are never stored)
  const int lane_src = (n16 < COUT ? n16 : COUT - 1) * 64 + 2 * q;
  auto load_error = [&](size_t n, f4 (&d)[4]) {
    const float* src = d_out + n * OUT_FLOATS + lane_src;
#pragma unroll
    for (int S = 0; S < 4; ++S) {
      const float2 lo = *reinterpret_cast<const float2*>(src + 16 * S), hi = *reinterpret_cast<const float2*>(src + 16 * S + 8);
      d[S] = f4{lo.x, lo.y, hi.x, hi.y};
    }
  };
  f4 acc[10];
#pragma unroll
  for (int nt = 0; nt < 10; ++nt) acc[nt] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  float g_b = 0.0f;
  const size_t G = (size_t)gridDim.x * WAVES_PER_GROUP, first = (size_t)blockIdx.x * WAVES_PER_GROUP + wave;
  Input cur;
  f4 d[4], dn[4];
  if (first < (size_t)B) {
    cur = load_input(in, first);
    load_error(first, d);
  }
  for (size_t n = first; n < (size_t)B; n += G) {
    store_input(x, cur);
    wave_sync();
    if (n + G < (size_t)B) {  // in flight during this image
      cur = load_input(in, n + G);
      load_error(n + G, dn);
    }
#pragma unroll
    for (int S = 0; S < 4; ++S) g_b += (d[S][0] + d[S][1]) + (d[S][2] + d[S][3]);
    float bv[2][10];
    auto load_step = [&](int step, float (&o)[10]) {
      const int S = step >> 2, r = step & 3, imm = 24 * S + 12 * (r >> 1) + (r & 1);
#pragma unroll
      for (int nt = 0; nt < 10; ++nt) o[nt] = bsrc[nt][imm];
    };
    load_step(0, bv[0]);
#pragma unroll
    for (int step = 0; step < 16; ++step) {
      if (step < 15) load_step(step + 1, bv[(step + 1) & 1]);
#pragma unroll
      for (int nt = 0; nt < 10; ++nt) acc[nt] = mfma16(d[step >> 2][step & 3], bv[step & 1][nt], acc[nt]);
      if (step < 15) __builtin_amdgcn_sched_group_barrier(0x100, 10, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 10, 0);
    }
    wave_sync();  // the reads of this image come before the next image's stores
#pragma unroll
    for (int S = 0; S < 4; ++S) d[S] = dn[S];
  }
  // ---- the eight waves' sums in a fixed order: (w, w + 4), then (w, w + 2), then (0, 1) ----
  lds.bsum[wave][l] = g_b;
#pragma unroll
  for (int half = WAVES_PER_GROUP / 2; half >= 1; half >>= 1) {
    __syncthreads();
    if (wave >= half && wave < 2 * half) {
      float* dst = lds.comb[wave - half];
#pragma unroll
      for (int nt = 0; nt < 10; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[(4 * nt + r) * 64 + l] = acc[nt][r];
    }
    __syncthreads();
    if (wave < half) {
      const float* src = lds.comb[wave];
#pragma unroll
      for (int nt = 0; nt < 10; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[nt][r] += src[(4 * nt + r) * 64 + l];
    }
  }
  if (wave == 0) {
    float* tile = part + (size_t)blockIdx.x * 10 * 256;
#pragma unroll
    for (int nt = 0; nt < 10; ++nt)
#pragma unroll
      for (int r = 0; r < 4; ++r) tile[nt * 256 + (4 * q + r) * 16 + n16] = acc[nt][r];  // row j = 4 q + r, column n16
  } else if (wave == 1 && l < 16) {
    // bias gradient of map l: the four lane quarters of the eight waves, in wave order
    float s = 0.0f;
    if (l < COUT)
      for (int w = 0; w < WAVES_PER_GROUP; ++w) s += (lds.bsum[w][l] + lds.bsum[w][l + 16]) + (lds.bsum[w][l + 32] + lds.bsum[w][l + 48]);
    part[(size_t)gridDim.x * 10 * 256 + (size_t)blockIdx.x * 16 + l] = s;
  }
}
inline size_t bwd_weight_workspace_bytes(unsigned groups) { return sizeof(float) * (size_t)groups * (10 * 256 + 16); }

}  // namespace conv2

// ---- the first convolution's shape: one input map 28 x 28, six output maps, 5 x 5 kernel -----------------
// Forward pass, one wave per image, as the GEMM over pixel pairs of cnn_wave.h (c1f_*: rows (map, x
// parity), K = 30 shifted taps, 18 tiles of 16 pixel pairs): 144 matrix instructions per image.  The
// operation moves 3.1 KB in and 13.8 KB out per image and is bound by those stores: the three tiles of
// a band of four pixel rows are collected in LDS as out[6][4][24] and leave as six runs of 384
// consecutive bytes in 16-byte items with the non-temporal hint (8-byte stores straight from the
// result registers were 8 % slower than the general kernel once the output no longer fits the
// last-level cache).
namespace conv1 {

constexpr int WAVES_PER_GROUP = 8, THREADS = 64 * WAVES_PER_GROUP;
inline bool shape_fits(int Cin, int H, int W, int Cout, int KH, int KW) {
  return Cin == 1 && Cout == 6 && KH == 5 && KW == 5 && H == 28 && W == 28;
}
constexpr int BAND = 6 * 4 * 24;  // one band of the output: six maps, four rows
struct __align__(16) FwdLds {
  float wa[C1F_KSTEPS * 64];  // A operand, [K step][lane]
  float bias[8];
  float img[WAVES_PER_GROUP][NI];
  float band[WAVES_PER_GROUP][BAND];
};
__global__ __launch_bounds__(THREADS) void forward_kernel(const float* __restrict__ in, const float* __restrict__ k,
                                                          const float* __restrict__ bias, float* __restrict__ out,
                                                          int B) {
  __shared__ FwdLds lds;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  if (t < C1F_KSTEPS * 64) {
    const int src = c1f_weight(t >> 6, t & 63);  // index into the flat parameter vector, k1 first
    lds.wa[t] = src >= 0 ? k[src - OFF_K1] : 0.0f;
  }
  if (t < 8) lds.bias[t] = bias && t < 6 ? bias[t] : 0.0f;
  __syncthreads();
  float wa[C1F_KSTEPS];
#pragma unroll
  for (int ks = 0; ks < C1F_KSTEPS; ++ks) wa[ks] = lds.wa[ks * 64 + l];
  f4 binit = f4{0.0f, 0.0f, 0.0f, 0.0f};
  if (q < 3) binit = f4{lds.bias[2 * q], lds.bias[2 * q], lds.bias[2 * q + 1], lds.bias[2 * q + 1]};
  const C1Lane ln = c1f_lane();
  // maps 2 q and 2 q + 1 at the lane's pixel pair inside a band (lanes q = 3 hold padding rows)
  const int lane_band = 2 * q * 96 + (((n16 >> 1) & 1) * 2 + (n16 & 1)) * 24 + 2 * (n16 >> 2);
  float* img = lds.img[wave];
  float* band = lds.band[wave];
  const size_t G = (size_t)gridDim.x * WAVES_PER_GROUP, first = (size_t)blockIdx.x * WAVES_PER_GROUP + wave;
  Pixels px;
  if (first < (size_t)B) px = load_pixels(in + first * NI);
  for (size_t n = first; n < (size_t)B; n += G) {
    store_pixels(img, px);
    wave_sync();
    if (n + G < (size_t)B) px = load_pixels(in + (n + G) * NI);  // in flight during this image
    float* dst = out + n * NC1;
#pragma unroll
    for (int ty = 0; ty < 6; ++ty) {
      f4 d0, d1, d2;
      c1f_gemm_pair(wa, ln, img + c1f_tile_img(3 * ty), img + c1f_tile_img(3 * ty + 1), binit, d0, d1);
      c1f_gemm_one(wa, ln, img + c1f_tile_img(3 * ty + 2), binit, d2);
      if (q < 3) {
        float* p = band + lane_band;
        *reinterpret_cast<float2*>(p) = float2{d0[0], d0[1]};
        *reinterpret_cast<float2*>(p + 96) = float2{d0[2], d0[3]};
        *reinterpret_cast<float2*>(p + 8) = float2{d1[0], d1[1]};
        *reinterpret_cast<float2*>(p + 8 + 96) = float2{d1[2], d1[3]};
        *reinterpret_cast<float2*>(p + 16) = float2{d2[0], d2[1]};
        *reinterpret_cast<float2*>(p + 16 + 96) = float2{d2[2], d2[3]};
      }
      wave_sync();
      // the band: map m's four rows are 96 consecutive floats of the output
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const int e = l + 64 * i;  // 16-byte piece of the band
        if (e < BAND / 4) {
          const int m = e / 24, piece = e - 24 * m;
          __builtin_nontemporal_store(reinterpret_cast<const f4*>(band)[e],
                                      reinterpret_cast<f4*>(dst + m * 576 + ty * 96) + piece);
        }
      }
      wave_sync();  // the band is read before the next one is written
    }
  }
}

// Weight and bias gradient of the same shape, one wave per image: the GEMM over pixel pairs of
// cnn_wave.h (c1g_accumulate: rows (map, x parity), columns the 30 shifted taps, K = 288 pixel
// pairs; the padding column 30 sums the error itself, i.e. the bias gradient): 144 matrix
// instructions per image.  The output error (13.8 KB per image, the bulk of what the operation
// reads) comes in three chunks of eight rows, d1c[6][8][24] with the maps D1C_MAP apart, the next
// chunk in registers while the current one is multiplied.  The sums stay in registers over all of
// a wave's images; the workgroup's eight waves are added in a fixed order and one set of partial
// tiles goes to the workspace in the general kernel's layout for P = 2 (rows 2 m + sh, columns
// 6 u + v'; bias rows 2 m + sh), which its second kernel joins and adds.
constexpr int CHUNK_PIECES = 6 * 8 * 24 / 4;  // 16-byte pieces of an error chunk
struct __align__(16) WgradLds {
  float ones[C1G_ONES];
  float img[WAVES_PER_GROUP][NI];
  float d1c[WAVES_PER_GROUP][6 * D1C_MAP + 8];  // after the last image: the wave's sums, [8 registers][64 lanes]
};
static_assert(6 * D1C_MAP + 8 >= 8 * 64, "a wave's chunk area holds its sums");
struct Chunk {
  f4 v[5];  // pieces l, l + 64, .. (the fifth only in lanes 0..31)
};
__device__ __forceinline__ Chunk load_chunk(const float* __restrict__ d_out, size_t n, int gp) {
  const int l = threadIdx.x & 63;
  Chunk c;
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    const int e = l + 64 * i, ee = e < CHUNK_PIECES ? e : 0, m = ee / 48, piece = ee - 48 * m;
    c.v[i] = reinterpret_cast<const f4*>(d_out + n * NC1 + m * 576 + gp * 192)[piece];
  }
  return c;
}
__device__ __forceinline__ void store_chunk(float* d1c, const Chunk& c) {
  const int l = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    const int e = l + 64 * i, m = e / 48, piece = e - 48 * m;
    if (e < CHUNK_PIECES) *reinterpret_cast<f4*>(d1c + m * D1C_MAP + 4 * piece) = c.v[i];
  }
}
__global__ __launch_bounds__(THREADS) void bwd_weight_kernel(const float* __restrict__ in,
                                                             const float* __restrict__ d_out,
                                                             float* __restrict__ part, int B) {
  __shared__ WgradLds lds;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15;
  for (int e = t; e < C1G_ONES; e += THREADS) lds.ones[e] = 1.0f;
  __syncthreads();
  float* img = lds.img[wave];
  float* d1c = lds.d1c[wave];
  f4 acc[2] = {f4{0.0f, 0.0f, 0.0f, 0.0f}, f4{0.0f, 0.0f, 0.0f, 0.0f}};
  const size_t G = (size_t)gridDim.x * WAVES_PER_GROUP, first = (size_t)blockIdx.x * WAVES_PER_GROUP + wave;
  Pixels px;
  Chunk ch;
  if (first < (size_t)B) {
    px = load_pixels(in + first * NI);
    ch = load_chunk(d_out, first, 0);
  }
  for (size_t n = first; n < (size_t)B; n += G) {
    store_pixels(img, px);
    const bool more = n + G < (size_t)B;
    if (more) px = load_pixels(in + (n + G) * NI);  // in flight during this image
#pragma unroll
    for (int gp = 0; gp < 3; ++gp) {
      store_chunk(d1c, ch);
      wave_sync();
      // the next chunk (of this image, or the first of the next image) is in flight during the GEMM
      if (gp < 2)
        ch = load_chunk(d_out, n, gp + 1);
      else if (more)
        ch = load_chunk(d_out, n + G, 0);
      c1g_accumulate<C1G_STEPS / 3, D1C_MAP>(acc, d1c, img + 8 * 28 * gp, l, lds.ones);
      wave_sync();  // the reads of this chunk come before the next chunk's (and image's) stores
    }
  }
  // ---- the eight waves' sums in wave order; T[row i = 4 q + r][column 16 nt + n16] ----
  float* mine = lds.d1c[wave];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int r = 0; r < 4; ++r) mine[(4 * nt + r) * 64 + l] = acc[nt][r];
  __syncthreads();
  if (wave < 2) {  // wave nt adds and stores tile nt
    float* tile = part + ((size_t)blockIdx.x * 2 + wave) * 256;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float sum = 0.0f;
      for (int w = 0; w < WAVES_PER_GROUP; ++w) sum += lds.d1c[w][(4 * wave + r) * 64 + l];
      tile[(4 * q + r) * 16 + n16] = sum;
      // column 30 (tile 1, n16 = 14) holds the sums of the error by (map, x parity): the bias rows
      if (wave == 1 && n16 == 14) part[(size_t)gridDim.x * 2 * 256 + (size_t)blockIdx.x * 16 + 4 * q + r] = sum;
    }
  }
}
inline size_t bwd_weight_workspace_bytes(unsigned groups) { return sizeof(float) * (size_t)groups * (2 * 256 + 16); }

// Input gradient of the same shape (listing `backin`, summed over the six maps of the output error):
//   d_in[p][q] = sum_m sum_{u,v} k[m][u][v] * d_out[m][p-u][q-v]          (terms inside the 24 x 24 error only)
// One output map and six input maps: a matrix tile has nothing to share between rows (the general
// kernel packs fourteen pixels into a column to fill one and needs 476 matrix instructions per
// image), so this runs on the fp32 vector unit, one wave per image.  A lane owns half a row of the
// output, fourteen neighbouring pixels (56 lanes): for a map and a kernel row it reads the eighteen
// error values its strip can reach, as nine 8-byte items, and does 70 multiply-adds, the 25 weights of
// the map in registers (broadcast reads, once per map).  LDS reads are what bounds this kernel: a
// 4-byte read of 64 lanes takes the LDS four cycles, an 8-byte read as well, hence strips whose
// reads are 8-byte aligned.  The error lies in the wave's LDS in rows of 28 floats, four zeros and
// the 24 values: the zeros of the next row are the right border, so no column is tested; a row
// above or below the map is replaced by one row of zeros (chosen per lane and kernel row when the
// kernel starts).
constexpr int BI_STRIDE = 28, BI_MAP = 24 * BI_STRIDE, BI_ZERO = 6 * BI_MAP, BI_FLOATS = BI_ZERO + 32;
constexpr int BI_KPAD = 28;                  // a map's 25 weights as seven 16-byte pieces
constexpr int BI_PIECES = 6 * 24 * 24 / 4;  // 16-byte pieces of an image's error
constexpr int BI_ROUNDS = (BI_PIECES + 63) / 64;
struct __align__(16) BwdInputLds {
  float k[6 * BI_KPAD];
  float d[WAVES_PER_GROUP][BI_FLOATS];
};
__global__ __launch_bounds__(THREADS) void bwd_input_kernel(const float* __restrict__ d_out,
                                                            const float* __restrict__ k, float* __restrict__ d_in,
                                                            int B) {
  __shared__ BwdInputLds lds;
  const int t = threadIdx.x, wave = t >> 6, l = t & 63;
  for (int e = t; e < 6 * BI_KPAD; e += THREADS) {
    const int m = e / BI_KPAD, tap = e - BI_KPAD * m;
    lds.k[e] = tap < 25 ? k[m * 25 + tap] : 0.0f;
  }
  float* d = lds.d[wave];
  for (int e = l; e < BI_FLOATS; e += 64) d[e] = 0.0f;  // the borders stay zero, the values are replaced per image
  __syncthreads();
  // the lane's strip: row p, columns 14 hx .. 14 hx + 13; kernel row u reads error row p - u, whose first
  // value for this strip is column 14 hx - 4, i.e. float 14 hx of the padded row
  const bool live = l < 56;
  const int p = live ? l >> 1 : 0, hx = l & 1, out_at = 28 * p + 14 * hx;
  int off[5], step[5];
#pragma unroll
  for (int u = 0; u < 5; ++u) {
    const int y = p - u;
    const bool inside = y >= 0 && y < 24;
    off[u] = (inside ? y * BI_STRIDE : BI_ZERO) + 14 * hx;
    step[u] = inside ? BI_MAP : 0;
  }
  // where the lane's 16-byte pieces of the error go: piece e = (map, row, four columns)
  int put[BI_ROUNDS];
#pragma unroll
  for (int j = 0; j < BI_ROUNDS; ++j) {
    const int e = l + 64 * j, ee = e < BI_PIECES ? e : 0, m = ee / 144, rem = ee - 144 * m, y = rem / 6, x4 = rem - 6 * y;
    put[j] = m * BI_MAP + y * BI_STRIDE + 4 + 4 * x4;
  }
  auto load_error = [&](size_t n, f4 (&v)[BI_ROUNDS]) {
    const f4* src = reinterpret_cast<const f4*>(d_out + n * NC1);
#pragma unroll
    for (int j = 0; j < BI_ROUNDS; ++j) v[j] = src[l + 64 * j < BI_PIECES ? l + 64 * j : l];
  };
  const size_t G = (size_t)gridDim.x * WAVES_PER_GROUP, first = (size_t)blockIdx.x * WAVES_PER_GROUP + wave;
  f4 cur[BI_ROUNDS];
  if (first < (size_t)B) load_error(first, cur);
  for (size_t n = first; n < (size_t)B; n += G) {
#pragma unroll
    for (int j = 0; j < BI_ROUNDS; ++j)
      if (l + 64 * j < BI_PIECES) *reinterpret_cast<f4*>(d + put[j]) = cur[j];  // 16-byte aligned: rows of 28 floats
    wave_sync();
    if (n + G < (size_t)B) load_error(n + G, cur);  // in flight during this image
    float acc[14];
#pragma unroll
    for (int i = 0; i < 14; ++i) acc[i] = 0.0f;
    int at[5];
#pragma unroll
    for (int u = 0; u < 5; ++u) at[u] = off[u];
#pragma unroll 1
    for (int m = 0; m < 6; ++m) {
      float w[BI_KPAD];  // the map's weights, every lane the same (broadcast reads)
#pragma unroll
      for (int i = 0; i < BI_KPAD / 4; ++i) {
        const f4 piece = *reinterpret_cast<const f4*>(&lds.k[m * BI_KPAD + 4 * i]);
        w[4 * i] = piece[0];
        w[4 * i + 1] = piece[1];
        w[4 * i + 2] = piece[2];
        w[4 * i + 3] = piece[3];
      }
      // the eighteen values of kernel row u + 1 are read while the 70 multiply-adds of row u issue (the
      // scheduling groups pin that order)
      float x[2][18];
      auto load_row = [&](int u, float (&o)[18]) {
        const float2* src = reinterpret_cast<const float2*>(d + at[u]);
#pragma unroll
        for (int j = 0; j < 9; ++j) {
          const float2 two = src[j];
          o[2 * j] = two.x;
          o[2 * j + 1] = two.y;
        }
        at[u] += step[u];
      };
      load_row(0, x[0]);
#pragma unroll
      for (int u = 0; u < 5; ++u) {
        if (u < 4) load_row(u + 1, x[(u + 1) & 1]);
#pragma unroll
        for (int v = 0; v < 5; ++v)
#pragma unroll
          for (int i = 0; i < 14; ++i) acc[i] = fmaf(w[5 * u + v], x[u & 1][i - v + 4], acc[i]);
        if (u < 4) __builtin_amdgcn_sched_group_barrier(0x100, 9, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 70, 0);
      }
    }
    if (live) {
      float2* dst = reinterpret_cast<float2*>(d_in + n * NI + out_at);
#pragma unroll
      for (int i = 0; i < 7; ++i) dst[i] = float2{acc[2 * i], acc[2 * i + 1]};
    }
    wave_sync();  // the reads of this image come before the next image's stores
  }
}

}  // namespace conv1
}  // namespace cnn
