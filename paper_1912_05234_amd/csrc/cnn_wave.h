// Device code of the fused step: ONE WAVEFRONT (64 lanes) OWNS ONE IMAGE from the
// pixel load to the last gradient term.  Definitions: arXiv 1912.05234, Section 3
// (forward, conv, mconv, sigmoid, avgpool, backweights, backbias, backin,
// backavgpool); the backward driver is the chain rule over those.
//
// Where the arithmetic runs
//   C1 forward            fp32 VALU, weights broadcast from LDS
//   C2 forward            v_mfma_f32_16x16x4_f32: M = 16 pixels, N = 12(16) maps, K = 150(152) taps
//   C2 weight gradient    v_mfma_f32_16x16x4_f32: M = 12(16) maps, N = 16 taps, K = 64 pixels
//   C2 input error        v_mfma_f32_16x16x4_f32: T[tap,pixel] = k2^T * d_c2 (K = 12 maps), then T is
//                         added into d_s1 at (y+u, x+v) (the col2im form of `backin`: no zero padding)
//                         in rounds of plain LDS read-add-write whose targets cannot collide
//   C1 weight gradient    v_mfma_f32_16x16x4_f32: M = 12(16) rows (map, x parity), N = 30(32) shifted taps,
//                         K = 288 pixel pairs; the C1 error is staged in LDS as d1[6][24][24]
//   FC weight gradient    v_mfma_f32_4x4x1_f32 rank-1 updates
//   FC, pooling, sigmoid  fp32 VALU
//
// A workgroup is four such waves.  They share nothing but a read-only table of MFMA operands in
// LDS (the C2 and FC weights, laid out [entry][lane] exactly as the instructions consume them),
// copied once per kernel from its ready-made image in global memory; after that single workgroup
// barrier the waves do not synchronise with each other until they join their gradient sums at
// the end of the kernel.  The same table, helpers and GEMM formulations serve the small-batch
// kernel (cnn_group.h), where eight waves share one image and C1 forward is a GEMM too.
//
// Pixel order.  A lane quad (4 consecutive lanes) is one 2x2 pooling window, so
// avgpool is a sum inside the quad (C1) or inside a lane's four MFMA result
// registers (C2) and never needs an LDS round trip.
//   C1: group g < 9, lane l: window w = 16 g + l/4 of the 12x12 windows, sub-pixel l%4.
//   C2: pixel index p = 4 w + sub, w = 4 wy + wx over the 4x4 windows; tile mt covers p in [16mt, 16mt+16).
// MFMA operand layouts (64 lanes, q = lane/16, n16 = lane%16):
//   16x16x4: A[i=n16][k=q], B[k=q][j=n16], D[i=4q+r][j=n16] in result register r.
//   4x4x1  : D_r(lane) += A(4*(lane/4)+r) * B(lane).
#pragma once

#include <type_traits>

#include "cnn_common.h"

// Hook for a cycle-counter probe at phase boundaries; empty in the library build.
#ifndef CNN_PHASE
#define CNN_PHASE_DECL
#define CNN_PHASE(k)
#define CNN_PHASE_FLUSH
#define CNN_KERNEL_MARK(k)
#endif
#ifndef CNN_GROUP_MARK
#define CNN_GROUP_MARK(k)
#endif

namespace cnn {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int WAVES = 4;  // waves (= images in flight) per workgroup
constexpr int D2S = 68;   // row stride of the C2 error array in LDS (floats)

// Per-wave LDS of the forward pass.  Padded K steps of the C2 forward read up to 1152 floats
// past the start of s1; those cells are zero or finite and meet zero weights.
struct __align__(16) FwdLds {
  float img[NI];
  float pool[NS1 + 288 + NS2];  // s1 at P_S1, s2 at P_S2
};
// LDS of the small-batch training step (cnn_group.h; one image per workgroup).  d_s1 comes first:
// the col2im rows of the two padding maps (c = 6, 7) add 0.0 at offsets up to 1152 floats past its
// start, which stays inside the struct.  `pool` holds, at the P_* offsets, the arrays that are dead
// by the time the C1 weight gradient runs; that phase reuses the whole pool for the staged C1 error.
constexpr int P_S1 = 0;                 // s1[6][12][12] + 288 (padded K steps of the C2 forward read them)
constexpr int P_S2 = P_S1 + NS1 + 288;  // s2[192]
constexpr int P_DS2 = P_S2 + NS2;       // d_s2[192] + 64 (rows of the padding maps of the C2 tiles)
constexpr int P_D2 = P_DS2 + NS2 + 64;  // d2[16][D2S]: error at C2's pre-activation, [map][pixel p]
constexpr int P_END = P_D2 + 16 * D2S;
// The C1 error is staged over the whole pool as d1[6][24][24] with the maps D1_MAP floats apart: the
// gradient GEMM's A operand reads all six maps in one instruction, and a map stride of 576 (a
// multiple of the 32 banks) would put them on the same four banks.
constexpr int D1_MAP = 24 * 24 + 4;
constexpr int POOL_FLOATS = 6 * D1_MAP + 32;
static_assert(POOL_FLOATS >= P_END, "pool holds the forward/C2 arrays");
struct __align__(16) TrainLds {
  float d_s1[NS1];  // error at S1 (col2im target)
  float img[NI];
  float pool[POOL_FLOATS];
};
// Per-wave LDS of the large-batch training step (one wave per image, two waves per SIMD): the same
// arrays packed into exactly one partial row's worth of floats (15.25 KB), so that eight waves and
// the operand table share a compute unit's 160 KB.  The padded K steps of the C2 forward read up
// to 1152 floats past the start of s1: s2, d_s2 and d2, all finite.  d2 has no rows for the
// padding maps.  The C1 error is staged in three chunks of eight image rows, d1c[6][8][24] with
// the maps D1C_MAP apart (a stride of 192 would be a multiple of the 32 banks), over s1 .. d_s2,
// which are dead by then.  The col2im rows of the padding maps add 0.0 to d_s1 offsets up to
// 1152 + 144 + 100, i.e. inside img or the pool's first cells: re-written with their own values.
constexpr int W_S1 = 0;                  // s1[6][12][12]
constexpr int W_S2 = W_S1 + NS1;         // s2[192]
constexpr int W_DS2 = W_S2 + NS2;        // d_s2[192] + 64
constexpr int W_D2 = W_DS2 + NS2 + 64;   // d2[12][D2S]
constexpr int W_END = W_D2 + 12 * D2S;
constexpr int W_DS1_COPY = 304;          // second copy of d_s1's maps 4, 5 over d2: 2 x 144 + the reach of a padding column
static_assert(W_DS1_COPY % 4 == 0 && W_DS1_COPY <= 12 * D2S, "the copy fits over d2");
constexpr int D1C_MAP = 8 * 24 + 4;
constexpr int WPOOL_FLOATS = PSTRIDE - NS1 - NI;
static_assert(WPOOL_FLOATS >= W_END && 6 * D1C_MAP <= W_D2, "pool holds the arrays; a d1 chunk ends before d2");
struct __align__(16) WaveTrainLds {
  float d_s1[NS1];
  float img[NI];
  float pool[WPOOL_FLOATS];
};
static_assert(sizeof(WaveTrainLds) == sizeof(float) * PSTRIDE, "a wave's LDS area holds one partial row");
// Shared operand table, [entry][lane].
constexpr int TAB_BF = 0;          // 38: C2 forward B operand, k2[j = n16][tap(s, q)]
constexpr int TAB_FCW = 38;        // 30: fc[o][lane + 64 k] at entry 3 o + k
constexpr int TAB_FWD_ENTRIES = 68;
constexpr int TAB_AB = 68;         // 21: C2 input-error A operand of input maps 0..3, entry tile*3 + s
constexpr int TAB_AB1 = 89;        // 21: the same for input maps 4..7 (the small-batch kernel)
constexpr int TAB_C1A = 110;       // 8: C1 forward A operand of the small-batch kernel, W[(m,sh) = n16][tap 4 ks + q]
constexpr int TAB_TRAIN_ENTRIES = 118;  // all of them; what the small-batch kernel reads
// The one-wave-per-image training kernel reads BF, FCW and AB from the table and keeps, right after
// them in its LDS copy, twelve entries that exist only there: input maps 4, 5 with two taps per tile
// (bwd_packed_source), entry tile*3 + s, gathered from the AB / AB1 slots of global memory when the
// kernel starts (packed_table_slot).
constexpr int TAB_PK = TAB_AB1;
constexpr int TAB_PK_COUNT = 12;
constexpr int TAB_WAVE_ENTRIES = TAB_PK + TAB_PK_COUNT;
// After the [entry][lane] part: C1 weights by tap, k1t[tap][8] = k1[0..5][tap], 0, 0 for tap < 25 and
// the biases b1 in row 25; every lane reads the same row (an LDS broadcast).
constexpr int K1T_FLOATS = 26 * 8;
// Last: the biases read per image, bias[0..11] = b2, bias[16..25] = b, zeros elsewhere.
constexpr int TAB_BIAS_FLOATS = 32;
constexpr int TAB_BIAS_B = 16, TAB_BIAS_B1 = 26;  // bias[16..25] = b, bias[26..31] = b1
template <int ENTRIES>
struct __align__(16) OperandTable {
  float e[ENTRIES * 64];
  float k1t[K1T_FLOATS];
  float bias[TAB_BIAS_FLOATS];
};
// The table is kept expanded in global memory next to the flat parameter vector (all 110 entries,
// then k1t, then bias); a kernel copies the part it needs into LDS with 16-byte loads.
constexpr int TABG_K1T = TAB_TRAIN_ENTRIES * 64;
constexpr int TABG_BIAS = TABG_K1T + K1T_FLOATS;
constexpr int TABG_FLOATS = TABG_BIAS + TAB_BIAS_FLOATS;
static_assert(TABG_K1T % 4 == 0 && K1T_FLOATS % 4 == 0, "16-byte pieces");

enum Mode { kForward = 0, kForwardDump = 1, kTrain = 2 };
template <int MODE>
struct LdsOf {
  typedef FwdLds type;
  static constexpr int entries = TAB_FWD_ENTRIES;
  static constexpr int S1 = P_S1, S2 = P_S2;
};
template <>
struct LdsOf<kTrain> {
  typedef WaveTrainLds type;
  static constexpr int entries = TAB_WAVE_ENTRIES;
  static constexpr int S1 = W_S1, S2 = W_S2;
};
__device__ __forceinline__ float quad_xor1(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float quad_xor2(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_row_half_mirror(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_row_mirror(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
}
// Sum over the 64 lanes in a fixed order, same value in every lane: quad, 8, 16 lanes by DPP,
// then the four rows of 16 through scalar registers.
__device__ __forceinline__ float wave_sum(float v) {
  v += quad_xor1(v);
  v += quad_xor2(v);
  v += dpp_row_half_mirror(v);
  v += dpp_row_mirror(v);
  const int iv = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ f4 mfma16(float a, float b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f4 mfma4(float a, float b, f4 c) {
  return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
}
// Ordering point inside ONE wave: LDS writes issued before it by any lane are seen by LDS reads
// issued after it by any lane of the same wave.  The LDS unit executes one wave's instructions in
// order, so nothing has to be waited for; the fences only stop the compiler from moving LDS
// accesses across this point.  No other wave is involved.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- K order of the C2 forward GEMM: step s < 38, lane quarter q -> tap (c,u,v) -------------
// steps 0..29: (c = s/5, v = s%5), u = q            LDS offset c*144 + v      + 12 q
// steps 30..35: c = s-30, u = 4, v = q               LDS offset c*144 + 48     + q
// steps 36,37: u = v = 4, c = 4(s-36) + q (c < 6)    LDS offset 576(s-36) + 52 + 144 q
__host__ __device__ constexpr int fwd_tap(int s, int q) {
  return s < 30 ? (s / 5) * 25 + q * 5 + (s % 5)
                : s < 36 ? (s - 30) * 25 + 20 + q : (4 * (s - 36) + q < 6 ? (4 * (s - 36) + q) * 25 + 24 : -1);
}
__host__ __device__ constexpr int fwd_imm(int s) {
  return s < 30 ? (s / 5) * 144 + (s % 5) : s < 36 ? (s - 30) * 144 + 48 : 576 * (s - 36) + 52;
}
// ---- M tiles of the C2 input-error GEMM.  Row i = 4 qi + ri of every tile belongs to input map
// c = 4 cg + qi (cg = 0, 1; maps 6, 7 are zero padding) and to the tap
//   tile V(v), v < 5 : (u = ri, v)        tile U4 : (u = 4, v = ri)        tile C : (4, 4) in ri = 0 only.
// A lane's result register r of tile (cg, .) therefore lands in d_s1[c = 4 cg + q] at row y+u, column x+v.
enum BwdTile { kTileV0 = 0, kTileU4 = 5, kTileC = 6 };  // V(v) = kTileV0 + v; tile C is used by the small-batch kernel only
__host__ __device__ constexpr int bwd_tap(int tile, int ri) {
  return tile < 5 ? 5 * ri + tile : tile == kTileU4 ? 20 + ri : (ri == 0 ? 24 : -1);
}
// Packed tiles for input maps 4 and 5 (a plain tile would leave the rows of maps 6, 7 empty): rows
// qi = 0, 1 belong to map 4 + qi and the taps of columns v = 0, 1, 2; rows qi = 2, 3 to map 4 + (qi - 2)
// again and the taps of columns v = 3, 4, whose terms are added into a second copy of the two maps
// (lanes of both halves would otherwise meet in the same cells within a round).
//   tile PV(s), s < 3 : qi < 2: (u = ri, v = s)       qi >= 2: (u = ri, v = 3 + s) for s < 2, nothing for s = 2
//   tile PU           : qi < 2: (4, v = ri), ri < 3   qi >= 2: ri = 0: (4, 3), ri = 1: (4, 4)
// so that in round s every lane finds "its" u = 4 term in result register s of PU.  Register 3 of
// PU is used by no round: its rows (qi, ri = 3) take tap (4, 4) of the maps 0..3, map qi, which puts
// the term into the very lane that owns map qi when those maps are summed (the plain tile C of
// those maps would use four rows of sixteen).
// Returns 25 c + tap, or -1 for a zero row.
enum PackedTile { kTilePV0 = 0, kTilePU = 3 };
__host__ __device__ constexpr int bwd_packed_source(int tile, int qi, int ri) {
  const int c = 4 + (qi & 1);
  if (tile < 3) return qi < 2 ? 25 * c + 5 * ri + tile : (tile < 2 ? 25 * c + 5 * ri + 3 + tile : -1);
  if (ri == 3) return 25 * qi + 24;
  if (qi < 2) return 25 * c + 20 + ri;
  return ri < 2 ? 25 * c + 23 + ri : -1;
}
// Slot of the expanded table (float index) that holds what lane `lane` of packed entry e = tile*3 + s
// needs, or -1 for a zero: the same weight sits in the plain tiles of AB (maps 0..3) or AB1 (maps 4..7).
__host__ __device__ constexpr int packed_table_slot(int e, int lane) {
  const int sidx = e % 3, q = lane >> 4, n16 = lane & 15, src = bwd_packed_source(e / 3, n16 >> 2, n16 & 3);
  if (src < 0) return -1;
  const int c = src / 25, tap = src % 25;
  const int tile = tap < 20 ? tap % 5 : tap < 24 ? (int)kTileU4 : (int)kTileC, ri = tap < 20 ? tap / 5 : tap < 24 ? tap - 20 : 0;
  return ((c < 4 ? TAB_AB : TAB_AB1) + tile * 3 + sidx) * 64 + q * 16 + (c & 3) * 4 + ri;
}
// ---- C1 forward as a GEMM (16x16x4 MFMA) -----------------------------------------------------------
// Output pixels are taken in horizontal pairs x = 2X + sh (sh = 0, 1).  With v' = v + sh the image
// factor img[y+u][2X+v'] does not depend on sh:
//   pre[(m,sh)][(y,X)] = b1[m] + sum_{u < 5, v' < 6} W[(m,sh)][(u,v')] * img[y+u][2X+v'],
//   W[(m,sh)][(u,v')] = k1[m][u][v'-sh]  (zero where v'-sh is outside 0..4).
// M = 12 rows (m,sh), i = 2m + sh, in one 16-row tile; K = 30 taps t = 6u + v' in 8 steps of four
// (t = 4 ks + q); N = 288 pixel pairs in 18 tiles of 16.  Tile T = 3 ty + tx covers the 2 x 4 block of
// pooling windows wy = 2 ty + a, wx = 4 tx + bx; column j = lane%16 = 4 bx + 2 a + dy is the pair
// (y = 2 wy + dy, X = wx).  Lanes j and j^1 are the two rows of one window and a lane's result
// registers of one map (sh = 0, 1) are its two columns, so avgpool is two adds and one DPP add.
//   A[i = lane%16][k = q] = W[i][4 ks + q]      (rows 12..15 and taps 30, 31 are zero)
//   B[k = q][j = lane%16] = img[y + u][2X + v']
//   D[i = 4q + r][j]: map m = 2q + r/2, sh = r%2, in result register r (lanes q = 3 hold padding rows).
constexpr int C1F_TILES = 18, C1F_KSTEPS = 8;
__host__ __device__ constexpr int c1f_weight(int ks, int lane) {  // flat parameter index or -1
  const int q = lane >> 4, i = lane & 15, t = 4 * ks + q;
  if (t >= 30 || i >= 12) return -1;
  const int u = t / 6, v = t % 6 - (i & 1);
  return v >= 0 && v < 5 ? OFF_K1 + (i >> 1) * 25 + u * 5 + v : -1;
}
// Offsets (floats) that depend on the tile only: image, pooled [6][12][12] arrays, [6][24][24] arrays.
__host__ __device__ constexpr int c1f_tile_img(int T) { return (T / 3) * 112 + (T % 3) * 8; }
__host__ __device__ constexpr int c1f_tile_s1(int T) { return (T / 3) * 24 + (T % 3) * 4; }
__host__ __device__ constexpr int c1f_tile_c1(int T) { return (T / 3) * 96 + (T % 3) * 8; }
// Offsets that depend on the lane only.
struct C1Lane {
  int img[C1F_KSTEPS];  // B operand of K step ks
  int s1;               // map 2q of a pooled array (map 2q + 1 is 144 further)
  int c1;               // map 2q, sh = 0 of the staged d1 (map 2q + 1 is D1_MAP further)
};
__device__ __forceinline__ C1Lane c1f_lane() {
  const int l = threadIdx.x & 63, q = l >> 4, n16 = l & 15;
  const int dy = n16 & 1, a = (n16 >> 1) & 1, bx = n16 >> 2;
  C1Lane o;
#pragma unroll
  for (int ks = 0; ks < C1F_KSTEPS; ++ks) {
    const int t = 4 * ks + q, tt = t < 30 ? t : 0;
    o.img[ks] = (2 * a + dy + tt / 6) * 28 + 2 * bx + tt % 6;
  }
  o.s1 = 2 * q * 144 + a * 12 + bx;
  o.c1 = 2 * q * D1_MAP + (2 * a + dy) * 24 + 2 * bx;
  return o;
}
// Pre-activations of two tiles at once (two independent accumulation chains); img0 / img1 point at
// the tiles' origins in the image.  The B operand of step ks + 1 is read while step ks issues.
__device__ __forceinline__ void c1f_gemm_pair(const float (&wa)[C1F_KSTEPS], const C1Lane& ln, const float* img0,
                                              const float* img1, f4 binit, f4& d0, f4& d1) {
  d0 = binit;
  d1 = binit;
  float x0[3], x1[3];
  x0[0] = img0[ln.img[0]];
  x1[0] = img1[ln.img[0]];
  x0[1] = img0[ln.img[1]];
  x1[1] = img1[ln.img[1]];
#pragma unroll
  for (int ks = 0; ks < C1F_KSTEPS; ++ks) {
    if (ks + 2 < C1F_KSTEPS) {
      x0[(ks + 2) % 3] = img0[ln.img[ks + 2]];
      x1[(ks + 2) % 3] = img1[ln.img[ks + 2]];
    }
    d0 = mfma16(wa[ks], x0[ks % 3], d0);
    d1 = mfma16(wa[ks], x1[ks % 3], d1);
  }
}
// The same for a single tile (one chain).
__device__ __forceinline__ void c1f_gemm_one(const float (&wa)[C1F_KSTEPS], const C1Lane& ln, const float* img0,
                                             f4 binit, f4& d0) {
  d0 = binit;
  float x0[3];
  x0[0] = img0[ln.img[0]];
  x0[1] = img0[ln.img[1]];
#pragma unroll
  for (int ks = 0; ks < C1F_KSTEPS; ++ks) {
    if (ks + 2 < C1F_KSTEPS) x0[(ks + 2) % 3] = img0[ln.img[ks + 2]];
    d0 = mfma16(wa[ks], x0[ks % 3], d0);
  }
}
// sigmoid in place, then S1 = avgpool for the tile's windows: s1 points at the tile's origin in the
// pooled array.  Lanes j and j^1 store the same value to the same cell; the padding rows of lanes
// q = 3 land in the (finite, never used) cells behind the sixth map.
__device__ __forceinline__ void c1f_finish(f4& d, const C1Lane& ln, float* s1) {
#pragma unroll
  for (int r = 0; r < 4; ++r) d[r] = logistic(d[r]);
  float p0 = d[0] + d[1], p1 = d[2] + d[3];
  p0 += quad_xor1(p0);
  p1 += quad_xor1(p1);
  s1[ln.s1] = 0.25f * p0;
  s1[ln.s1 + 144] = 0.25f * p1;
}

// Flat parameter index whose value slot i of the expanded table holds, or -1 for a zero.
__host__ __device__ constexpr int table_source(int i) {
  if (i < TABG_K1T) {
    const int e = i >> 6, l = i & 63, q = l >> 4, n16 = l & 15;
    if (e < TAB_FCW) {
      const int tap = fwd_tap(e, q);
      return n16 < 12 && tap >= 0 ? OFF_K2 + n16 * 150 + tap : -1;
    }
    if (e < TAB_AB) {
      const int o = (e - TAB_FCW) / 3, k = (e - TAB_FCW) % 3;
      return OFF_FC + o * NS2 + l + 64 * k;
    }
    if (e >= TAB_C1A) return c1f_weight(e - TAB_C1A, l);
    const int cg = e >= TAB_AB1 ? 1 : 0, t = e - (cg ? TAB_AB1 : TAB_AB), sidx = t % 3, tile = t / 3;
    const int c = 4 * cg + (n16 >> 2), tap = bwd_tap(tile, n16 & 3);
    return c < 6 && tap >= 0 ? OFF_K2 + (4 * sidx + q) * 150 + c * 25 + tap : -1;
  }
  if (i < TABG_BIAS) {
    const int tap = (i - TABG_K1T) >> 3, m = (i - TABG_K1T) & 7;
    return m < 6 ? (tap < 25 ? OFF_K1 + m * 25 + tap : OFF_B1 + m) : -1;
  }
  const int k = i - TABG_BIAS;
  return k < 12 ? OFF_B2 + k
                : k >= TAB_BIAS_B && k < TAB_BIAS_B + NY ? OFF_B + (k - TAB_BIAS_B)
                                                         : k >= TAB_BIAS_B1 ? OFF_B1 + (k - TAB_BIAS_B1) : -1;
}
// Factor a slot holds its parameter multiplied by: the forward weights and biases of both
// convolution layers carry -log2(e) (see logistic_of_scaled); the C2 input-error operand carries the
// 1/4 of the average pooling below it (backavgpool, Section 3), which the C1 error then does not apply.
__host__ __device__ constexpr float table_scale(int i) {
  if (i < TABG_K1T) {
    const int e = i >> 6;
    return e < TAB_FCW ? NEG_LOG2E : e >= TAB_AB && e < TAB_C1A ? 0.25f : 1.0f;
  }
  if (i < TABG_BIAS) return NEG_LOG2E;
  return i - TABG_BIAS < 12 ? NEG_LOG2E : 1.0f;
}
// No parameter sits in more than four slots (a C1 weight: once by tap, twice as shifted GEMM operand):
// the SGD kernel refreshes the expanded table by writing every updated parameter to its recorded places.
constexpr int TABLE_MAX_DEST = 4;
constexpr int table_max_multiplicity() {
  int count[NPARAM] = {};
  int most = 0;
  for (int i = 0; i < TABG_FLOATS; ++i) {
    const int p = table_source(i);
    if (p >= 0 && ++count[p] > most) most = count[p];
  }
  return most;
}

// Copies the expanded table from global memory into the workgroup's LDS in two halves, so that a
// kernel can do other set-up work while the loads are in flight: `fetch` issues all of a thread's
// 16-byte loads, `commit` stores them to LDS.  All THREADS threads of the workgroup take part and
// the caller follows the commit with a workgroup barrier.
// COHERENT: the table was written by other compute units during this kernel (the device-side
// epoch loop): its 16-byte pieces are fetched with agent-scope loads, which do not take stale lines
// from this XCD's L2 cache.
// ENTRIES counts the entries of the LDS copy, of which the first LOADED come from global memory.
// FIRST: the entry whose pieces are fetched first; `commit_first` stores those (one round of loads)
// and the tail, `commit_rest` the others, each followed by a barrier of the caller's.
template <int ENTRIES, int THREADS, bool COHERENT = false, int LOADED = ENTRIES, int FIRST = 0>
struct TableLoad {
  static constexpr int PIECES = LOADED * 16, ROUNDS = (PIECES + THREADS - 1) / THREADS;
  static constexpr int TAIL = (K1T_FLOATS + TAB_BIAS_FLOATS) / 4;
  typedef OperandTable<ENTRIES> Table;
  static_assert(offsetof(Table, bias) == offsetof(Table, k1t) + sizeof(float) * K1T_FLOATS,
                "k1t and bias are copied as one run");
  static_assert(TAIL <= THREADS, "one thread per piece of the tail");
  static_assert(FIRST >= 0 && FIRST < LOADED, "the entry fetched first is one of the loaded ones");
  f4 v[ROUNDS], tail;
  // 16-byte piece of the table that this thread moves in round r (the same in global memory and in
  // LDS), or -1: the pieces are taken in the order FIRST * 16, .., PIECES - 1, 0, .., FIRST * 16 - 1, so
  // that round 0 brings the entries from FIRST on (what the caller needs first) and loads return in
  // the order they are issued
  static __device__ __forceinline__ int piece(int r) {
    const int i = r * THREADS + (int)threadIdx.x, at = i + FIRST * 16;
    return i < PIECES ? (at < PIECES ? at : at - PIECES) : -1;
  }
  // Issue order: round 0, the tail (k1t, biases), the other rounds.
  __device__ __forceinline__ void fetch(const float* __restrict__ tabg) {
    const int t = threadIdx.x;
    if (COHERENT) {
      const __amdgpu_buffer_rsrc_t rs =
          __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(tabg), 0, sizeof(float) * TABG_FLOATS, 0x00020000);
      constexpr int AGENT_SCOPE = 16;  // the sc1 bit of the cache policy
      typedef unsigned u4 __attribute__((ext_vector_type(4)));
      auto load = [&](int byte) { return __builtin_bit_cast(f4, (u4)__builtin_amdgcn_raw_buffer_load_b128(rs, byte, 0, AGENT_SCOPE)); };
      { const int i = piece(0); v[0] = load(16 * (i >= 0 ? i : 0)); }
      tail = load(4 * TABG_K1T + 16 * (t < TAIL ? t : 0));
#pragma unroll
      for (int r = 1; r < ROUNDS; ++r) {
        const int i = piece(r);
        v[r] = load(16 * (i >= 0 ? i : 0));
      }
      return;
    }
    const f4* src = reinterpret_cast<const f4*>(tabg);
    { const int i = piece(0); v[0] = src[i >= 0 ? i : 0]; }
    tail = src[TABG_K1T / 4 + (t < TAIL ? t : 0)];
#pragma unroll
    for (int r = 1; r < ROUNDS; ++r) {
      const int i = piece(r);
      v[r] = src[i >= 0 ? i : 0];
    }
  }
  // Round 0 and the tail: the entries FIRST .. (and the first ones again, as far as a round reaches).
  __device__ __forceinline__ void commit_first(Table& tab) const {
    const int t = threadIdx.x, i = piece(0);
    if (i >= 0) reinterpret_cast<f4*>(tab.e)[i] = v[0];
    if (t < TAIL) reinterpret_cast<f4*>(tab.k1t)[t] = tail;
  }
  __device__ __forceinline__ void commit_rest(Table& tab) const {
#pragma unroll
    for (int r = 1; r < ROUNDS; ++r) {
      const int i = piece(r);
      if (i >= 0) reinterpret_cast<f4*>(tab.e)[i] = v[r];
    }
  }
  __device__ __forceinline__ void commit(Table& tab) const {
    commit_first(tab);
    commit_rest(tab);
  }
};
template <int ENTRIES, int THREADS, int LOADED = ENTRIES>
__device__ __forceinline__ void load_tables(OperandTable<ENTRIES>& tab, const float* __restrict__ tabg) {
  TableLoad<ENTRIES, THREADS, false, LOADED> ld;
  ld.fetch(tabg);
  ld.commit(tab);
}

// ---- C1 weight gradient as one GEMM per image (16x16x4 MFMA) ------------------------------------
//   g_k1[m][u][v] = sum_{y,x < 24} d1[m][y][x] * img[y+u][x+v]            (backweights, Section 3)
// Pixels are taken in horizontal pairs x = 2X + sh (sh = 0, 1).  With v' = v + sh the image factor
// img[y+u][2X+v'] no longer depends on sh, so
//   T[(m,sh)][(u,v')] = sum_{y,X} d1[m][y][2X+sh] * img[y+u][2X+v'],   g_k1[m][u][v] = T[(m,0)][(u,v)] + T[(m,1)][(u,v+1)]
// is a GEMM with M = 12 rows (m,sh) in one 16-row tile, N = 30 columns (u,v'), c = 6u + v', in two
// 16-column tiles, and K = 288 pixel pairs in 72 steps of four: step kk covers row y = kk / 3 and
// pairs X = 4 (kk % 3) + q, q = lane / 16.  d1 is staged in LDS as d1[m][24][24], maps D1_MAP apart.
//   A[i = lane%16][k = q] = d1[m = (i/2) % 6][y][2X + i%2]     (rows 12..15 repeat rows 0..3, dropped)
//   B[k = q][j = lane%16] = img[y + u][2X + v'], c = 16 nt + j  (columns 30, 31 read tap 0, dropped)
//   D[i = 4q + r][j]: register r of tile nt.
constexpr int C1G_STEPS = 72;
constexpr int C1G_PARK = 16 * 32;  // floats: T as [row i][column c]
__host__ __device__ constexpr int c1g_imm_a(int kk) { return 24 * (kk / 3) + 8 * (kk % 3); }
__host__ __device__ constexpr int c1g_imm_b(int kk) { return 28 * (kk / 3) + 8 * (kk % 3); }
// Lane parts of the operand addresses (floats): d1 (maps MAP floats apart) and the two image tiles.
template <int MAP = D1_MAP>
__device__ __forceinline__ void c1g_lane_offsets(int& a, int (&bt)[2], int l) {
  const int q = l >> 4, n16 = l & 15;
  a = ((n16 >> 1) % 6) * MAP + (n16 & 1) + 2 * q;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const int c = 16 * nt + n16;
    bt[nt] = (c < 30 ? (c / 6) * 28 + c % 6 : 0) + 2 * q;
  }
}
// STEPS steps of the GEMM from the given origins of d1 and the image: operands of step kk + 2 are
// read while the two MFMAs of step kk issue.
// With `ones` (C1G_ONES floats of 1.0): the two padding columns 30, 31 read 1.0 instead of image
// pixels, so that column 30 of the result is the sum of the A operand over all steps,
//   T[(m,sh)][30] = sum_{y,X} d1[m][y][2X+sh],   g_b1[m] = T[(m,0)][30] + T[(m,1)][30]      (backbias, Section 3)
// at no cost in instructions.
constexpr int C1G_ONES = 224;  // the reach of a lane's B operand over eight image rows: 28 * 7 + 16 + 6 + 1
template <int STEPS, int MAP = D1_MAP>
__device__ __forceinline__ void c1g_accumulate(f4 (&acc)[2], const float* d1, const float* img, int lane,
                                               const float* ones = nullptr) {
  static_assert(28 * ((STEPS - 1) / 3) + 8 * 2 + 6 < C1G_ONES || STEPS > 24, "the ones cover a padding lane's reads");
  int a, bt[2];
  c1g_lane_offsets<MAP>(a, bt, lane);
  const float* pa = d1 + a;
  const float* pb0 = img + bt[0];
  const float* pb1 = ones && (lane & 15) >= 14 ? ones + 2 * (lane >> 4) : img + bt[1];
  float oa[3], ob0[3], ob1[3];
  auto load_step = [&](int kk, int slot) {
    oa[slot] = pa[c1g_imm_a(kk)];
    ob0[slot] = pb0[c1g_imm_b(kk)];
    ob1[slot] = pb1[c1g_imm_b(kk)];
  };
  load_step(0, 0);
  if (STEPS > 1) load_step(1, 1);
#pragma unroll
  for (int kk = 0; kk < STEPS; ++kk) {
    if (kk + 2 < STEPS) load_step(kk + 2, (kk + 2) % 3);
    acc[0] = mfma16(oa[kk % 3], ob0[kk % 3], acc[0]);
    acc[1] = mfma16(oa[kk % 3], ob1[kk % 3], acc[1]);
    if (kk + 2 < STEPS) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
  }
}
// The same GEMM restricted to the K steps of NT tiles of the C1 forward tiling (c1f_tile_*): tile T
// covers four pixel rows and one group of four pixel pairs, i.e. four K steps whose operand
// offsets are the tile's origin plus 24 (d1) or 28 (image) floats per row.  d1t[k] / imgt[k] point
// at the origins of tile k.
template <int NT>
__device__ __forceinline__ void c1g_accumulate_tiles(f4 (&acc)[2], const float* const (&d1t)[3],
                                                     const float* const (&imgt)[3]) {
  int a, bt[2];
  c1g_lane_offsets(a, bt, threadIdx.x & 63);
  float oa[3], ob0[3], ob1[3];
  auto load_step = [&](int st, int slot) {
    const int k = st >> 2, row = st & 3;
    oa[slot] = d1t[k][a + 24 * row];
    ob0[slot] = imgt[k][bt[0] + 28 * row];
    ob1[slot] = imgt[k][bt[1] + 28 * row];
  };
  load_step(0, 0);
  load_step(1, 1);
#pragma unroll
  for (int st = 0; st < 4 * NT; ++st) {
    if (st + 2 < 4 * NT) load_step(st + 2, (st + 2) % 3);
    acc[0] = mfma16(oa[st % 3], ob0[st % 3], acc[0]);
    acc[1] = mfma16(oa[st % 3], ob1[st % 3], acc[1]);
    if (st + 2 < 4 * NT) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
  }
}
// Parks T: park[i * 32 + c] for the lane's rows i = 4q + r and columns c = 16 nt + lane%16.
__device__ __forceinline__ void c1g_park(const f4 (&acc)[2], float* park) {
  const int l = threadIdx.x & 63, q = l >> 4, n16 = l & 15;
#pragma unroll
  for (int nt = 0; nt < 2; ++nt)
#pragma unroll
    for (int r = 0; r < 4; ++r) park[(4 * q + r) * 32 + 16 * nt + n16] = acc[nt][r];
}
// g_k1 element e = m * 25 + 5 u + v from a parked T.
__device__ __forceinline__ float c1g_combine(const float* park, int e) {
  const int m = e / 25, tap = e - 25 * m, u = tap / 5, v = tap - 5 * u;
  return park[(2 * m) * 32 + 6 * u + v] + park[(2 * m + 1) * 32 + 6 * u + v + 1];
}

// Offsets of the origin of pooling window win = 12 wy + wx, shared by the waves of a training
// workgroup and read per image (registers are what the training kernel is short of): .x inside the
// 28 x 28 image, .y inside a 24 x 24 map.
constexpr int NWIN = 144;
struct WindowTable {
  int2 o[NWIN];
  // C2 weight gradient: offset (floats, inside s1) of the s1 cell that lane l reads first for tap tile
  // nt, i.e. of tap 16 nt + l % 16 = (c, u, v) at pixel quarter l / 16: c * 144 + u * 12 + v + 2 (l / 16)
  // (0 + 2 (l / 16) for the padding taps 150..159)
  int k2b[10][64];
  float ones[C1G_ONES];  // 1.0: B operand of the padding columns of the C1 weight-gradient GEMM (c1g_accumulate)
};
// Filled by all THREADS threads of the workgroup (the caller's barrier follows).
template <int THREADS>
__device__ __forceinline__ void window_table_init(WindowTable& w) {
  const int t = threadIdx.x;
#pragma unroll
  for (int r = 0; r < (NWIN + THREADS - 1) / THREADS; ++r) {
    const int win = t + r * THREADS;
    if (win < NWIN) w.o[win] = int2{56 * (win / 12) + 2 * (win % 12), 48 * (win / 12) + 2 * (win % 12)};
  }
#pragma unroll
  for (int r = 0; r < (640 + THREADS - 1) / THREADS; ++r) {
    const int e = t + r * THREADS;
    const int nt = e >> 6, l = e & 63, tap = 16 * nt + (l & 15);
    const int c = tap / 25, rem = tap - 25 * c, u = rem / 5, v = rem - 5 * u;
    if (e < 640) w.k2b[nt][l] = (tap < 150 ? c * 144 + u * 12 + v : 0) + 2 * (l >> 4);
  }
#pragma unroll
  for (int r = 0; r < (C1G_ONES + THREADS - 1) / THREADS; ++r)
    if (t + r * THREADS < C1G_ONES) w.ones[t + r * THREADS] = 1.0f;
}

// What the FC weight gradient needs of one image, kept in global memory until the wave has done all
// its images: s2 (192 floats), then delta in [192, 202) and zeros up to 208; rows of 256 floats, so
// that no two images share a cache line.  The gradient is then ONE GEMM per wave over its images,
//   g_fc[o][i] = sum_n delta_n[o] * s2_n[i]                                   (backweights, Section 3)
// with M = 10(16) outputs, N = 192 inputs in twelve tiles, K = the wave's images four at a time:
// three matrix instructions per image instead of thirty multiply-adds on sums that no register or LDS
// space is left for.
constexpr int FC_HIST = 256;        // floats per image
constexpr int FC_HIST_DELTA = 192;  // delta[0..9], then six zeros
// Everything a wave keeps in registers across its images.
template <int MODE>
struct WaveState {
  int pix0[9];    // forward only: LDS offset of the origin of this lane's pooling window in pixel group g
  float bias2;    // b2[n16]
  // training only
  f4 acc_k2[10];  // sum over images of d_c2 (x) s1 patches, D[j = 4q+r][tap = 16 nt + n16]
  f4 acc_k1[2];   // C1 weight gradient GEMM result T[(m,sh) = 4q+r][c = 16 nt + n16]; column 30: the C1 bias gradient
  float g_b;      // FC bias gradient: lane o < 10 holds b[o]
  float g_b2, loss;
};

template <int MODE>
__device__ __forceinline__ void wave_init(WaveState<MODE>& st, typename LdsOf<MODE>::type& s) {
  const int l = threadIdx.x & 63, b = l >> 2;
  // all of this wave's LDS starts finite: padded GEMM steps multiply it by zero weights
  static_assert(sizeof(s) % 16 == 0, "LDS struct is a whole number of 16-byte pieces");
  f4* raw = reinterpret_cast<f4*>(&s);
  for (int e = l; e < (int)(sizeof(s) / 16); e += 64) raw[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int g = 0; g < 9; ++g) {
    const int win = 16 * g + b;
    st.pix0[g] = 2 * (win / 12) * 28 + 2 * (win % 12);  // unused when training (see WindowTable)
  }
  st.bias2 = 0.0f;  // read from the operand table once it is complete
  if (MODE == kTrain) {
#pragma unroll
    for (int nt = 0; nt < 10; ++nt) st.acc_k2[nt] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    st.acc_k1[0] = st.acc_k1[1] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    st.g_b2 = 0.0f;
    st.loss = 0.0f;
    st.g_b = 0.0f;
  }
}

// Optional per-image outputs of the forward pass.
struct DumpPtrs {
  float *c1, *s1, *c2, *s2;
};

// The 196 16-byte pieces of one image as four float4 registers per lane (the fourth only in lanes
// 0..3).  Kept as separate values so that they stay in registers.
struct Pixels {
  f4 a, b, c, d;
};
__device__ __forceinline__ Pixels load_pixels(const float* __restrict__ image) {
  const f4* src = reinterpret_cast<const f4*>(image);
  const int l = threadIdx.x & 63;
  Pixels px;
  px.a = src[l];  // consecutive lanes -> consecutive 16 bytes
  px.b = src[l + 64];
  px.c = src[l + 128];
  px.d = src[l < 4 ? l + 192 : l];  // lanes >= 4 re-read a piece they already have (no divergence)
  return px;
}

// The lane index as a phase of the training step sees it: through a register the compiler cannot
// see through, so that the address arithmetic built on it is redone in every phase of every image
// instead of being computed once per kernel and held in (scarce) registers for its whole life.
// The forward-only kernels have registers to spare and keep the hoisting.
template <int MODE>
__device__ __forceinline__ int phase_lane() {
  int l = threadIdx.x & 63;
  if (MODE == kTrain) asm volatile("" : "+v"(l));
  return l;
}
#define CNN_PHASE_LANES                                              \
  const int l = phase_lane<MODE>();                                  \
  const int q = l >> 4, n16 = l & 15, b = l >> 2, sub = l & 3;       \
  const int pp = 12 * ((n16 & 3) >> 1) + 2 * (n16 >> 2) + (n16 & 1); \
  const float* tl = tab.e + l;                                       \
  (void)q, (void)n16, (void)b, (void)sub, (void)pp, (void)tl

__device__ __forceinline__ void store_pixels(float* img, const Pixels& px) {
  const int l = threadIdx.x & 63;
  f4* dst = reinterpret_cast<f4*>(img);
  dst[l] = px.a;
  dst[l + 64] = px.b;
  dst[l + 128] = px.c;
  if (l < 4) dst[l + 192] = px.d;
}
// Touches the 25 cache lines of an image so that they are on their way into the L2 cache; the value
// is not used (the asm keeps the load alive and costs no instruction).
__device__ __forceinline__ void touch_pixels(const float* __restrict__ image) {
  const int l = threadIdx.x & 63;
  float v = image[l < 25 ? 32 * l : 0];
  asm volatile("" ::"v"(v));
}

// One image through forward (and, when MODE == kTrain, backward).  Forward only: `px` holds this
// image's pixels on entry; if `next_image` is not null its pixels are loaded into `px` while this
// image is still being worked on, so the HBM latency of the only per-image global read is hidden.
// Training: the image is in s.img on entry and `next_image` (never null: the caller passes any
// valid image when there is no next one) is in s.img on return; `px` is not used.  Returns yhat in y[10]
// (wave-uniform).  `label` is only read when training; `hist` is the image's history row (FC_HIST
// floats, training only).
template <int MODE>
__device__ __forceinline__ void wave_image(WaveState<MODE>& st, typename LdsOf<MODE>::type& s,
                                           const OperandTable<LdsOf<MODE>::entries>& tab, Pixels& px,
                                           const float* __restrict__ next_image, int label,
                                           float (&y)[10], const DumpPtrs& dump,
                                           size_t n, const WindowTable* wt = nullptr, float* hist = nullptr) {
  constexpr int P_S1 = LdsOf<MODE>::S1, P_S2 = LdsOf<MODE>::S2;
  const int l = threadIdx.x & 63, q = l >> 4, n16 = l & 15, b = l >> 2, sub = l & 3;
  const int pp = 12 * ((n16 & 3) >> 1) + 2 * (n16 >> 2) + (n16 & 1);
  const float* tl = tab.e + l;  // this lane's column of the operand table

  CNN_PHASE_DECL;
  CNN_PHASE(0);
  if (MODE != kTrain) {
    store_pixels(s.img, px);
    wave_sync();
    if (next_image) px = load_pixels(next_image);
  }
  // (training: the image is in LDS already, stored by the kernel or at the end of the previous image)

  CNN_PHASE(1);
  // ---- C1 = sigmoid(mconv(I, k1, b1)), S1 = avgpool(C1).  Tap-outer: the six weights of a tap are
  //      wave-uniform scalars, every lane holds its nine pixels' accumulators for all six maps. ----
  float c1[9][6];
  {
    CNN_PHASE_LANES;
    const float* ip[9];
    // training: the window origins come from the shared table, re-read per image
#pragma unroll
    for (int g = 0; g < 9; ++g)
      ip[g] = s.img + (MODE == kTrain ? wt->o[16 * g + b].x : st.pix0[g]) + (sub >> 1) * 28 + (sub & 1);
    // One kernel row u: 45 pixel reads, 10 broadcast weight reads and 270 multiply-adds.  The reads
    // of tap v + 1 are issued before the multiply-adds of tap v and no earlier (two sets of nine
    // pixels and six weights in registers, not five).  FIRST: the sums start here, at the biases.
    auto kernel_row = [&](int u, auto first) {
      constexpr bool FIRST = decltype(first)::value;
      const float* ku = tab.k1t + u * 40;
      float x[2][9], wt[2][6], bias[6];
      if (FIRST) {
        const f4 ba = *reinterpret_cast<const f4*>(&tab.k1t[25 * 8]);
        const float2 bb = *reinterpret_cast<const float2*>(&tab.k1t[25 * 8 + 4]);
        bias[0] = ba[0]; bias[1] = ba[1]; bias[2] = ba[2]; bias[3] = ba[3]; bias[4] = bb.x; bias[5] = bb.y;
      }
      auto load_tap = [&](int v, float (&xx)[9], float (&ww)[6]) {
        const f4 wa = *reinterpret_cast<const f4*>(&ku[v * 8]);
        const float2 wb = *reinterpret_cast<const float2*>(&ku[v * 8 + 4]);
        ww[0] = wa[0]; ww[1] = wa[1]; ww[2] = wa[2]; ww[3] = wa[3]; ww[4] = wb.x; ww[5] = wb.y;
#pragma unroll
        for (int g = 0; g < 9; ++g) xx[g] = ip[g][u * 28 + v];
      };
      load_tap(0, x[0], wt[0]);
      __builtin_amdgcn_sched_group_barrier(0x100, FIRST ? 13 : 11, 0);
#pragma unroll
      for (int v = 0; v < 5; ++v) {
        if (v < 4) load_tap(v + 1, x[(v + 1) & 1], wt[(v + 1) & 1]);
#pragma unroll
        for (int i = 0; i < 6; ++i)
#pragma unroll
          for (int g = 0; g < 9; ++g) c1[g][i] = fmaf(wt[v & 1][i], x[v & 1][g], FIRST && v == 0 ? bias[i] : c1[g][i]);
        if (v < 4) __builtin_amdgcn_sched_group_barrier(0x100, 11, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 54, 0);
      }
    };
    // Row 0 is written out; rows 1..4 are a real loop with the 54 sums carried around it, which keeps
    // the compiler from hoisting all 225 reads (and their registers) or serialising the sums.
    kernel_row(0, std::true_type());
#pragma unroll 1
    for (int u = 1; u < 5; ++u) kernel_row(u, std::false_type());
    // sigmoid, then S1 = avgpool(C1): the four lanes of a quad are the four pixels of one window.
    // A butterfly with selects leaves the window sum of map `sub` in lane `sub`, so one unmasked
    // store per group writes four maps (no divergent store, nothing for the scheduler to trip on).
    const bool odd = sub & 1, hi = sub & 2;
#pragma unroll
    for (int g = 0; g < 9; ++g) {
#pragma unroll
      for (int i = 0; i < 6; ++i) {
        c1[g][i] = logistic_of_scaled(c1[g][i]);
        if (MODE == kForwardDump && dump.c1) {
          const int win = 16 * g + b;
          dump.c1[n * NC1 + i * 576 + (2 * (win / 12) + (sub >> 1)) * 24 + 2 * (win % 12) + (sub & 1)] = c1[g][i];
        }
      }
      const float s01 = (odd ? c1[g][1] : c1[g][0]) + quad_xor1(odd ? c1[g][0] : c1[g][1]);
      const float s23 = (odd ? c1[g][3] : c1[g][2]) + quad_xor1(odd ? c1[g][2] : c1[g][3]);
      const float tot = (hi ? s23 : s01) + quad_xor2(hi ? s01 : s23);
      s.pool[P_S1 + sub * 144 + 16 * g + b] = 0.25f * tot;
    }
    // maps 4 and 5 of two groups at a time: lane sub -> map 4 + (sub & 1) of group (sub & 2 ? g1 : g0)
#pragma unroll
    for (int gp = 0; gp < 5; ++gp) {
      const int g0 = 2 * gp, g1 = gp < 4 ? 2 * gp + 1 : 8;
      const float sa = (odd ? c1[g0][5] : c1[g0][4]) + quad_xor1(odd ? c1[g0][4] : c1[g0][5]);
      const float sb = (odd ? c1[g1][5] : c1[g1][4]) + quad_xor1(odd ? c1[g1][4] : c1[g1][5]);
      const float tot = (hi ? sb : sa) + quad_xor2(hi ? sa : sb);
      s.pool[P_S1 + (4 + (sub & 1)) * 144 + 16 * (hi ? g1 : g0) + b] = 0.25f * tot;
    }
  }
  wave_sync();
  if (MODE == kForwardDump && dump.s1)
    for (int e = l; e < NS1; e += 64) dump.s1[n * NS1 + e] = s.pool[P_S1 + e];

  CNN_PHASE(2);
  if (MODE == kTrain) touch_pixels(next_image);
  // ---- C2 = sigmoid(mconv(S1, k2, b2)) as a 64 x 16 x 152 GEMM, S2 = avgpool(C2) ------------------
  f4 c2v[4];
  {
    CNN_PHASE_LANES;
    const float* a12 = s.pool + P_S1 + pp + 12 * q;
    const float* a1 = s.pool + P_S1 + pp + q;
    const float* a144 = s.pool + P_S1 + pp + 144 * q;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) c2v[mt] = f4{st.bias2, st.bias2, st.bias2, st.bias2};
    // operands of K step s+2 are read while the MFMAs of step s issue (three rotating buffers);
    // the scheduling groups pin that order, which the compiler would otherwise collapse
    float opa[3][4], opw[3];
    auto load_step = [&](int sidx, float (&oa)[4], float& ow) {
      const float* base = sidx < 30 ? a12 : sidx < 36 ? a1 : a144;
      ow = tl[(TAB_BF + sidx) * 64];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) oa[mt] = base[fwd_imm(sidx) + 24 * mt];
    };
    load_step(0, opa[0], opw[0]);
    load_step(1, opa[1], opw[1]);
#pragma unroll
    for (int sidx = 0; sidx < 38; ++sidx) {
      if (sidx + 2 < 38) load_step(sidx + 2, opa[(sidx + 2) % 3], opw[(sidx + 2) % 3]);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) c2v[mt] = mfma16(opa[sidx % 3][mt], opw[sidx % 3], c2v[mt]);
      if (sidx + 2 < 38) __builtin_amdgcn_sched_group_barrier(0x100, 5, 0);  // 5 LDS reads of step s+2
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);                     // 4 MFMAs of step s
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) c2v[mt][r] = logistic_of_scaled(c2v[mt][r]);
      if (n16 < 12) s.pool[P_S2 + n16 * 16 + 4 * mt + q] = 0.25f * ((c2v[mt][0] + c2v[mt][1]) + (c2v[mt][2] + c2v[mt][3]));
      if (MODE == kForwardDump && dump.c2 && n16 < 12)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          dump.c2[n * NC2 + n16 * 64 + (2 * mt + (r >> 1)) * 8 + 2 * q + (r & 1)] = c2v[mt][r];
    }
  }
  wave_sync();
  if (MODE == kForwardDump && dump.s2)
    for (int e = l; e < NS2; e += 64) dump.s2[n * NS2 + e] = s.pool[P_S2 + e];

  CNN_PHASE(3);
  // ---- output = sigmoid(mconv(S2, fc, b)): lane owns inputs lane, lane+64, lane+128 ----------------
  float sv[3];
  {
    CNN_PHASE_LANES;
#pragma unroll
    for (int k = 0; k < 3; ++k) sv[k] = s.pool[P_S2 + l + 64 * k];
#pragma unroll
    for (int o = 0; o < 10; ++o) {
      float p = tl[(TAB_FCW + 3 * o) * 64] * sv[0];
      p = fmaf(tl[(TAB_FCW + 3 * o + 1) * 64], sv[1], p);
      p = fmaf(tl[(TAB_FCW + 3 * o + 2) * 64], sv[2], p);
      y[o] = logistic(wave_sum(p) + tab.bias[TAB_BIAS_B + o]);
    }
  }
  if constexpr (MODE == kTrain) {
    // ---- output error, FC backweights / backbias / backin ------------------------------------------
    float delta[10];
    {
      float lsum = 0.0f;
#pragma unroll
      for (int o = 0; o < 10; ++o) {
        const float e = y[o] - (o == label ? 1.0f : 0.0f);
        lsum = fmaf(e, e, lsum);
        delta[o] = e * fmaf(-y[o], y[o], y[o]);  // y (1 - y) as y - y^2: one instruction
      }
      st.loss = fmaf(0.5f, lsum, st.loss);
    }
    // backweights: s2 and delta go to the image's history row, the products are taken once per
    // wave (wave_fc_gradient); backbias: lane o keeps the sum of delta[o].
    {
      CNN_PHASE_LANES;
      float mine = 0.0f;
#pragma unroll
      for (int o = 0; o < 10; ++o) mine = l == o ? delta[o] : mine;
      st.g_b += mine;
#pragma unroll
      for (int k = 0; k < 3; ++k) hist[l + 64 * k] = sv[k];
      if (l < 16) hist[FC_HIST_DELTA + l] = mine;  // zero in lanes 10..15
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        float d = 0.0f;
#pragma unroll
        for (int o = 0; o < 10; ++o) d = fmaf(tl[(TAB_FCW + 3 * o + k) * 64], delta[o], d);
        s.pool[W_DS2 + l + 64 * k] = d;
      }
      // clear the col2im target of the C2 input error
      for (int e = l; e < NS1 / 4; e += 64) reinterpret_cast<f4*>(s.d_s1)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    wave_sync();

    CNN_PHASE(4);
    // ---- backavgpool through S2 and the derivative of C2's sigmoid; d_c2 stays in the MFMA result
    //      layout, which is exactly the A-operand layout of the weight-gradient GEMM; the rows of the
    //      twelve real maps also go to LDS as the B operand of the input-error GEMM ---------------------
    f4 d2v[4];
    {
    CNN_PHASE_LANES;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      const float up = s.pool[W_DS2 + n16 * 16 + 4 * mt + q] * 0.25f;  // rows n16 >= 12 read finite filler
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float c = c2v[mt][r];
        d2v[mt][r] = up * fmaf(-c, c, c);
      }
      if (n16 < 12) *reinterpret_cast<f4*>(&s.pool[W_D2 + n16 * D2S + 16 * mt + 4 * q]) = d2v[mt];
      st.g_b2 += (d2v[mt][0] + d2v[mt][1]) + (d2v[mt][2] + d2v[mt][3]);
    }
    }
    wave_sync();

    CNN_PHASE(5);
    // ---- C2 backweights: G[j, tap] += sum_p d_c2[j, p] * s1[c, y(p)+u, x(p)+v];  K step = (S, r):
    //      the four pixels 16 S + 4 q + r of lane quarter q ------------------------------------------
    {
      CNN_PHASE_LANES;
      const float* bsrc[10];  // s1 patch element of tap 16 nt + n16 for pixel quarter q
#pragma unroll
      for (int nt = 0; nt < 10; ++nt) bsrc[nt] = s.pool + W_S1 + wt->k2b[nt][l];
      // the ten s1 reads of step + 1 are issued under the ten MFMAs of a step and no earlier
      float bv[2][10];
      auto load_step = [&](int step, float (&o)[10]) {
        const int S = step >> 2, r = step & 3, imm = 24 * S + 12 * (r >> 1) + (r & 1);
#pragma unroll
        for (int nt = 0; nt < 10; ++nt) o[nt] = bsrc[nt][imm];
      };
      load_step(0, bv[0]);
      __builtin_amdgcn_sched_group_barrier(0x100, 10, 0);
#pragma unroll
      for (int step = 0; step < 16; ++step) {
        if (step < 15) load_step(step + 1, bv[(step + 1) & 1]);
#pragma unroll
        for (int nt = 0; nt < 10; ++nt)
          st.acc_k2[nt] = mfma16(d2v[step >> 2][step & 3], bv[step & 1][nt], st.acc_k2[nt]);
        if (step < 15) __builtin_amdgcn_sched_group_barrier(0x100, 10, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 10, 0);
      }
    }

    CNN_PHASE(6);
    // ---- C2 backin summed over the twelve maps, col2im form:
    //        T[(c,u,v), p] = sum_j k2[j,c,u,v] * d_c2[j,p];   d_s1[c, y(p)+u, x(p)+v] += T[(c,u,v), p].
    //      With level = 2 nt + u (nt = pixel tile = row pair of p), two terms of one map touch the
    //      same cells only if their levels differ by at most 1; equal level and equal v means the very
    //      same cells.  So for each v: terms of equal level are added in registers, then all even
    //      levels go to LDS in one round of read-add-write, then all odd levels.  Within a round no two
    //      lanes share an address (maps are 144 floats apart, levels 24, pixels of a tile distinct).
    //      The two groups of four input maps (cg) are taken one after the other: half the registers.
    {
      CNN_PHASE_LANES;
      float bd[3][4];
#pragma unroll
      for (int sidx = 0; sidx < 3; ++sidx)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) bd[sidx][nt] = s.pool[W_D2 + (4 * sidx + q) * D2S + 16 * nt + n16];
      // the second copy of maps 4 and 5 (see bwd_packed_tap) lies over d2, which is in registers now
      float* copy = s.pool + W_D2;
      wave_sync();
      for (int e = l; e < W_DS1_COPY / 4; e += 64) reinterpret_cast<f4*>(copy)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
      wave_sync();
      // One round pair (even levels, then odd levels) for the tiles tv of one tap column: `u4` is the
      // u = 4 term per pixel tile, `dst` the lane's cell of level 0 for that column.
      auto rounds = [&](const f4 (&tv)[4], const float (&u4)[4], float* dst) {
        // even levels 2m, m < 6: (nt = m, u = 0) + (m-1, 2) + (m-2, 4)
        {
          float e[6], old[6];
#pragma unroll
          for (int m = 0; m < 6; ++m) {
            float acc = 0.0f;
            if (m < 4) acc = tv[m < 4 ? m : 0][0];
            if (m >= 1 && m <= 4) acc += tv[m >= 1 ? m - 1 : 0][2];
            if (m >= 2) acc += u4[m >= 2 ? m - 2 : 0];
            e[m] = acc;
            old[m] = dst[24 * m];
          }
#pragma unroll
          for (int m = 0; m < 6; ++m) dst[24 * m] = old[m] + e[m];
        }
        wave_sync();
        // odd levels 2m+1, m < 5: (nt = m, u = 1) + (m-1, 3)
        {
          float e[5], old[5];
#pragma unroll
          for (int m = 0; m < 5; ++m) {
            float acc = 0.0f;
            if (m < 4) acc = tv[m < 4 ? m : 0][1];
            if (m >= 1) acc += tv[m >= 1 ? m - 1 : 0][3];
            e[m] = acc;
            old[m] = dst[24 * m + 12];
          }
#pragma unroll
          for (int m = 0; m < 5; ++m) dst[24 * m + 12] = old[m] + e[m];
        }
        wave_sync();
      };
      // the four pixel tiles of one M tile: entry `first` + sidx of the table
      auto tiles = [&](int first, f4 (&out)[4]) {
        float av[3];
#pragma unroll
        for (int sidx = 0; sidx < 3; ++sidx) av[sidx] = tl[(first + sidx) * 64];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
          f4 a = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int sidx = 0; sidx < 3; ++sidx) a = mfma16(av[sidx], bd[sidx][nt], a);
          out[nt] = a;
        }
      };
      // ---- input maps 0..3: lane quarter q owns map q; tiles V(0..4) and U4; tap (4, 4) rides in
      //      register 3 of the packed tile PU of the maps 4, 5 below ----
      f4 tu[4];
      tiles(TAB_PK + kTilePU * 3, tu);
      {
        f4 t4[4];  // taps (4, v), v < 4, in register v
        tiles(TAB_AB + kTileU4 * 3, t4);
        float* tgt = s.d_s1 + 144 * q + pp;
        // tile V(v+1) is issued before the rounds of V(v), so its MFMAs run under the LDS round trips
        f4 tv[4], tn[4];  // taps (u, v), u < 4, in register u
        tiles(TAB_AB + kTileV0 * 3, tv);
#pragma unroll
        for (int v = 0; v < 5; ++v) {
          if (v < 4) tiles(TAB_AB + (kTileV0 + v + 1) * 3, tn);
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
      // ---- input maps 4, 5, packed: lane quarters 0, 1 own them for tap columns 0..2 and add into
      //      d_s1, quarters 2, 3 own them again for columns 3, 4 and add into the copy; in round s a
      //      lane's column is s or 3 + s (quarters 2, 3 have nothing in round 2: their tile rows are
      //      zero and they re-write cells with their own values) ----
      {
        // (tu: the u = 4 term of round r in register r)
        float* tgt = q < 2 ? s.d_s1 + 144 * (4 + q) + pp : copy + 144 * (q - 2) + pp + 3;
        f4 tv[4], tn[4];
        tiles(TAB_PK + kTilePV0 * 3, tv);
#pragma unroll
        for (int r = 0; r < 3; ++r) {
          if (r < 2) tiles(TAB_PK + (kTilePV0 + r + 1) * 3, tn);
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
    }

    CNN_PHASE(7);
    // ---- backavgpool through S1 and the derivative of C1's sigmoid, then C1 backweights as a GEMM
    //      over pixel pairs, in three chunks of eight image rows (pixel groups 3 gp .. 3 gp + 2): the
    //      chunk's error is staged in LDS as d1c[m][8][24] over s1 .. d_s2 (dead by now) and the GEMM
    //      runs the 24 K steps of those rows ---------------------------------------------------------
    {
      CNN_PHASE_LANES;
      const int lane_d1 = (sub >> 1) * 24 + (sub & 1);
#pragma unroll
      for (int gp = 0; gp < 3; ++gp) {
        float up[3][6];
        int off[3];
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          off[k] = wt->o[16 * (3 * gp + k) + b].y - 192 * gp + lane_d1;
#pragma unroll
          for (int i = 0; i < 6; ++i) up[k][i] = s.d_s1[i * 144 + 16 * (3 * gp + k) + b];
          // maps 4 and 5 were summed in two halves (the copy lies over d2, beyond the staged chunk)
#pragma unroll
          for (int i = 4; i < 6; ++i) up[k][i] += s.pool[W_D2 + (i - 4) * 144 + 16 * (3 * gp + k) + b];
        }
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          const int g = 3 * gp + k;
          float* dst = s.pool + off[k];
#pragma unroll
          for (int i = 0; i < 6; ++i) {
            const float c = c1[g][i];
            // c (1 - c); the pooling's 1/4 is in the operand table.  (backbias: the GEMM below sums d1
            // in its padding column.)
            dst[i * D1C_MAP] = up[k][i] * fmaf(-c, c, c);
          }
        }
        wave_sync();
        CNN_PHASE(8);
        // the next image's pixels (touched into the L2 cache long ago) are fetched under the last
        // chunk's GEMM, when the fewest registers are in use, and take this image's place after it
        // (through an offset the compiler cannot see before this point: it would otherwise start
        // the loads, and occupy their sixteen registers, phases earlier)
        Pixels nx;
        if (gp == 2) {
          int zero = 0;
          asm volatile("" : "+v"(zero));
          nx = load_pixels(next_image + zero);
        }
        c1g_accumulate<C1G_STEPS / 3, D1C_MAP>(st.acc_k1, s.pool, s.img + 8 * 28 * gp, phase_lane<MODE>(), wt->ones);
        wave_sync();
        if (gp == 2) {
          store_pixels(s.img, nx);
          wave_sync();
        }
      }
    }
    CNN_PHASE(9);
  }
}

// FC weight gradient of a wave from the history rows of its images (see FC_HIST).  One K step of the
// GEMM takes up to four images: lane (q, n16) supplies A[o = n16][k = q] = delta of the step's q-th
// image and B[k = q][i = n16] = its s2[16 nt + n16] for the twelve tiles nt.  Result tile nt,
// register r of lane (q, n16): g_fc[o = 4 q + r][i = 16 nt + n16].
struct FcStepOperands {
  float a, b[12];
};
// rows[k] points at the row of the step's k-th image, or at any valid row when the step has fewer
// than four (`count` says how many are real: the others contribute delta = 0).
__device__ __forceinline__ void fc_step_load(FcStepOperands& op, const float* const (&rows)[4], int count) {
  const int l = threadIdx.x & 63, q = l >> 4, n16 = l & 15;
  const float* mine = q == 0 ? rows[0] : q == 1 ? rows[1] : q == 2 ? rows[2] : rows[3];
  op.a = mine[FC_HIST_DELTA + n16];
  if (q >= count) op.a = 0.0f;
#pragma unroll
  for (int nt = 0; nt < 12; ++nt) op.b[nt] = mine[16 * nt + n16];
}
__device__ __forceinline__ void fc_step_mfma(f4 (&g_fc)[12], const FcStepOperands& op) {
#pragma unroll
  for (int nt = 0; nt < 12; ++nt) g_fc[nt] = mfma16(op.a, op.b[nt], g_fc[nt]);
}

// Writes the wave's gradient sums as one partial row (PSTRIDE floats in parameter order, the loss
// in LOSS_SLOT, zeros after it) to `row`, every slot by exactly one lane.  `row` may be the start
// of the wave's own LDS area (all of it is dead once the wave's images are done); `park` is
// C1G_PARK floats of LDS outside the row that no other wave uses; `g_fc` is wave_fc_gradient's result.
__device__ __forceinline__ void wave_flush(WaveState<kTrain>& st, const f4 (&g_fc)[12], float* row, float* park) {
  const int l = threadIdx.x & 63, q = l >> 4, n16 = l & 15;
  // The stores are grouped by the lanes that take part (one branch per group, not one per store):
  // FC rows o = 4 q + r < 10 are registers 0, 1 of the quarters 0..2 and registers 2, 3 of the quarters
  // 0, 1; C2 rows j = 4 q + r < 12 are every register of the quarters 0..2, and of the last tap tile
  // only the columns n16 < 6 are taps.
  {
    float* fc = row + OFF_FC + 4 * q * NS2 + n16;
    if (q < 3) {
#pragma unroll
      for (int nt = 0; nt < 12; ++nt)
#pragma unroll
        for (int r = 0; r < 2; ++r) fc[r * NS2 + 16 * nt] = g_fc[nt][r];
    }
    if (q < 2) {
#pragma unroll
      for (int nt = 0; nt < 12; ++nt)
#pragma unroll
        for (int r = 2; r < 4; ++r) fc[r * NS2 + 16 * nt] = g_fc[nt][r];
    }
  }
  if (l < 10) row[OFF_B + l] = st.g_b;
  if (l < PSTRIDE - LOSS_SLOT) row[LOSS_SLOT + l] = l == 0 ? st.loss : 0.0f;
  if (q < 3) {
    float* k2 = row + OFF_K2 + 4 * q * 150 + n16;
#pragma unroll
    for (int nt = 0; nt < 9; ++nt)
#pragma unroll
      for (int r = 0; r < 4; ++r) k2[r * 150 + 16 * nt] = st.acc_k2[nt][r];
    if (n16 < 150 - 16 * 9) {
#pragma unroll
      for (int r = 0; r < 4; ++r) k2[r * 150 + 16 * 9] = st.acc_k2[9][r];
    }
  }
  {
    float v = st.g_b2;  // lane (q, j): sum over the four lane quarters
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    if (q == 0 && n16 < 12) row[OFF_B2 + n16] = v;
  }
  // C1 weights: the two shifted halves of the GEMM result are joined through LDS
  c1g_park(st.acc_k1, park);
  wave_sync();
#pragma unroll
  for (int round = 0; round < 3; ++round) {
    const int e = l + 64 * round;
    if (e < 150) row[OFF_K1 + e] = c1g_combine(park, e);
  }
  // C1 biases: column 30 of the same result holds the sums of d1 by (map, x parity)
  if (l < 6) row[OFF_B1 + l] = park[(2 * l) * 32 + 30] + park[(2 * l + 1) * 32 + 30];
}

}  // namespace cnn
