// Stateless per-operation kernels (general shapes) and their C entry points.
// Definitions: arXiv 1912.05234, Section 3 -- listings conv, mconv, sigmoid,
// avgpool, backweights, backbias, backin, backavgpool.  Convolutions and fully
// connected layers whose operands fit in LDS run as implicit GEMMs on the matrix
// cores (cnn_igemm.h); the plain one-thread-per-output kernels below serve every
// other shape.  The fused training step lives in cnn_fused.hip.
#include <mutex>

#include "cnn_common.h"
#include "cnn_igemm.h"
#include "cnn_igemm_bf16.h"
#include "cnn_col2im.h"
#include "cnn_conv_wave.h"
#include "cnn_fc_wave.h"

namespace {

using namespace cnn;

constexpr int TPB = 256;

inline unsigned grid_for(size_t n) {
  size_t g = (n + TPB - 1) / TPB;
  const size_t cap = 256 * 32;  // grid-stride beyond this
  return (unsigned)(g < cap ? (g ? g : 1) : cap);
}

// Streaming kernels: one item per thread (neighbouring workgroups then touch neighbouring memory,
// which the memory system likes better than a few workgroups striding far: 6.2 against 5.0 TB/s for
// a 566 MB copy), and outputs written with the non-temporal hint (+ 4 to 20 %): nothing here reads
// its own output again.
inline unsigned grid_stream(size_t n) {
  size_t g = (n + TPB - 1) / TPB;
  const size_t cap = 0x7fffffff;
  return (unsigned)(g < cap ? (g ? g : 1) : cap);
}
typedef float vec2 __attribute__((ext_vector_type(2)));
typedef float vec4 __attribute__((ext_vector_type(4)));

// An operand as the arithmetic sees it: itself, or rounded to bfloat16 (nearest even).
template <bool BF16>
__device__ __forceinline__ float operand(float v) {
  return BF16 ? __uint_as_float((unsigned)igemm16::to_bf16(v) << 16) : v;
}

// out[b,co,y,x] = bias[co] + sum_{ci,u,v} in[b,ci,y+u,x+v] * k[co,ci,u,v]
template <bool BF16>
__global__ __launch_bounds__(TPB) void conv_fwd_kernel(const float* __restrict__ in,
                                                       const float* __restrict__ k,
                                                       const float* __restrict__ bias,
                                                       float* __restrict__ out, size_t total, int Cin,
                                                       int H, int W, int Cout, int KH, int KW) {
  const int Ho = H - KH + 1, Wo = W - KW + 1;
  for (size_t o = blockIdx.x * (size_t)TPB + threadIdx.x; o < total; o += (size_t)gridDim.x * TPB) {
    const int x = (int)(o % Wo);
    const int y = (int)((o / Wo) % Ho);
    const int co = (int)((o / ((size_t)Wo * Ho)) % Cout);
    const size_t b = o / ((size_t)Wo * Ho * Cout);
    float acc = bias ? bias[co] : 0.0f;
    for (int ci = 0; ci < Cin; ++ci) {
      const float* ip = in + ((b * Cin + ci) * H + y) * (size_t)W + x;
      const float* kp = k + ((size_t)co * Cin + ci) * KH * KW;
      for (int u = 0; u < KH; ++u)
        for (int v = 0; v < KW; ++v) acc = fmaf(operand<BF16>(ip[u * W + v]), operand<BF16>(kp[u * KW + v]), acc);
    }
    out[o] = acc;
  }
}

// d_in[b,ci,p,q] = sum_co sum_{u,v valid} k[co,ci,u,v] * d_out[b,co,p-u,q-v]
template <bool BF16>
__global__ __launch_bounds__(TPB) void conv_bwd_input_kernel(const float* __restrict__ d_out,
                                                             const float* __restrict__ k,
                                                             float* __restrict__ d_in, size_t total,
                                                             int Cin, int H, int W, int Cout, int KH,
                                                             int KW) {
  const int Ho = H - KH + 1, Wo = W - KW + 1;
  for (size_t o = blockIdx.x * (size_t)TPB + threadIdx.x; o < total; o += (size_t)gridDim.x * TPB) {
    const int q = (int)(o % W);
    const int p = (int)((o / W) % H);
    const int ci = (int)((o / ((size_t)W * H)) % Cin);
    const size_t b = o / ((size_t)W * H * Cin);
    const int u_lo = max(0, p - Ho + 1), u_hi = min(KH - 1, p);
    const int v_lo = max(0, q - Wo + 1), v_hi = min(KW - 1, q);
    float acc = 0.0f;
    for (int co = 0; co < Cout; ++co) {
      const float* dp = d_out + (b * Cout + co) * (size_t)Ho * Wo;
      const float* kp = k + ((size_t)co * Cin + ci) * KH * KW;
      for (int u = u_lo; u <= u_hi; ++u)
        for (int v = v_lo; v <= v_hi; ++v)
          acc = fmaf(operand<BF16>(kp[u * KW + v]), operand<BF16>(dp[(p - u) * Wo + (q - v)]), acc);
    }
    d_in[o] = acc;
  }
}

// Fixed-order reduction of one value per thread over the workgroup.
__device__ __forceinline__ float block_sum(float v, float* red) {
  red[threadIdx.x] = v;
  __syncthreads();
  for (int s = TPB / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  const float r = red[0];
  __syncthreads();
  return r;
}

// One workgroup per weight (blocks [0, Cout*Cin*KH*KW)) or per bias (the next Cout
// blocks): d_k[co,ci,u,v] = sum_{b,y,x} in[b,ci,y+u,x+v] * d_out[b,co,y,x].
template <bool BF16>
__global__ __launch_bounds__(TPB) void conv_bwd_weight_kernel(const float* __restrict__ in,
                                                              const float* __restrict__ d_out,
                                                              float* __restrict__ d_k,
                                                              float* __restrict__ d_bias, int B, int Cin,
                                                              int H, int W, int Cout, int KH, int KW) {
  __shared__ float red[TPB];
  const int Ho = H - KH + 1, Wo = W - KW + 1;
  const int nk = Cout * Cin * KH * KW;
  const size_t dom = (size_t)B * Ho * Wo;
  const int id = blockIdx.x;
  float acc = 0.0f;
  if (id < nk) {
    const int v = id % KW, u = (id / KW) % KH, ci = (id / (KW * KH)) % Cin, co = id / (KW * KH * Cin);
    for (size_t e = threadIdx.x; e < dom; e += TPB) {
      const int x = (int)(e % Wo), y = (int)((e / Wo) % Ho);
      const size_t b = e / ((size_t)Wo * Ho);
      acc = fmaf(operand<BF16>(in[((b * Cin + ci) * H + y + u) * (size_t)W + x + v]),
                 operand<BF16>(d_out[((b * Cout + co) * Ho + y) * (size_t)Wo + x]), acc);
    }
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) d_k[id] = acc;
  } else {
    const int co = id - nk;
    for (size_t e = threadIdx.x; e < dom; e += TPB) {
      const size_t b = e / ((size_t)Wo * Ho), r = e % ((size_t)Wo * Ho);
      acc += operand<BF16>(d_out[(b * Cout + co) * (size_t)Ho * Wo + r]);
    }
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) d_bias[co] = acc;
  }
}

// One thread per output element.  With rows counted over all maps (r = map * Ho + p) the 2x2
// window of output (r, q) is rows 2 r, 2 r + 1 and columns 2 q, 2 q + 1 of the input, so one division
// per element suffices and the two columns move as one 8-byte item (W is even).
__global__ __launch_bounds__(TPB) void avgpool_fwd_kernel(const float* __restrict__ in,
                                                          float* __restrict__ out, size_t total, int W) {
  const size_t Wo = (size_t)(W / 2);
  for (size_t o = blockIdx.x * (size_t)TPB + threadIdx.x; o < total; o += (size_t)gridDim.x * TPB) {
    const size_t r = o / Wo, q = o - r * Wo;
    const float2* ip = reinterpret_cast<const float2*>(in + 2 * r * W + 2 * q);
    const float2 a = ip[0], b = ip[W / 2];
    out[o] = (a.x + a.y + b.x + b.y) * 0.25f;
  }
}

// One thread per element of d_out: it writes the 2x2 block it spreads into (same row arithmetic).
__global__ __launch_bounds__(TPB) void avgpool_bwd_kernel(const float* __restrict__ d_out,
                                                          float* __restrict__ d_in, size_t total, int Wo) {
  const size_t W = 2 * (size_t)Wo;
  for (size_t e = blockIdx.x * (size_t)TPB + threadIdx.x; e < total; e += (size_t)gridDim.x * TPB) {
    const size_t r = e / Wo, q = e - r * Wo;
    const float v = d_out[e] * 0.25f;
    float2* op = reinterpret_cast<float2*>(d_in + 2 * r * W + 2 * q);
    op[0] = float2{v, v};
    op[Wo] = float2{v, v};
  }
}

__global__ __launch_bounds__(TPB) void fc_fwd_kernel(const float* __restrict__ in,
                                                     const float* __restrict__ w,
                                                     const float* __restrict__ bias,
                                                     float* __restrict__ out, size_t total, int I, int O) {
  for (size_t e = blockIdx.x * (size_t)TPB + threadIdx.x; e < total; e += (size_t)gridDim.x * TPB) {
    const int o = (int)(e % O);
    const size_t b = e / O;
    float acc = bias ? bias[o] : 0.0f;
    for (int i = 0; i < I; ++i) acc = fmaf(in[b * I + i], w[(size_t)o * I + i], acc);
    out[e] = acc;
  }
}

__global__ __launch_bounds__(TPB) void fc_bwd_input_kernel(const float* __restrict__ d_out,
                                                           const float* __restrict__ w,
                                                           float* __restrict__ d_in, size_t total, int I,
                                                           int O) {
  for (size_t e = blockIdx.x * (size_t)TPB + threadIdx.x; e < total; e += (size_t)gridDim.x * TPB) {
    const int i = (int)(e % I);
    const size_t b = e / I;
    float acc = 0.0f;
    for (int o = 0; o < O; ++o) acc = fmaf(w[(size_t)o * I + i], d_out[b * O + o], acc);
    d_in[e] = acc;
  }
}

// One workgroup per weight (blocks [0, O*I)) or per bias (next O blocks).
__global__ __launch_bounds__(TPB) void fc_bwd_weight_kernel(const float* __restrict__ in,
                                                            const float* __restrict__ d_out,
                                                            float* __restrict__ d_w,
                                                            float* __restrict__ d_bias, int B, int I,
                                                            int O) {
  __shared__ float red[TPB];
  const int id = blockIdx.x;
  float acc = 0.0f;
  if (id < O * I) {
    const int i = id % I, o = id / I;
    for (size_t b = threadIdx.x; b < (size_t)B; b += TPB) acc = fmaf(d_out[b * O + o], in[b * I + i], acc);
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) d_w[id] = acc;
  } else {
    const int o = id - O * I;
    for (size_t b = threadIdx.x; b < (size_t)B; b += TPB) acc += d_out[b * O + o];
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) d_bias[o] = acc;
  }
}

// Four elements per thread as one 16-byte item; the last n % 4 elements one by one.
__global__ __launch_bounds__(TPB) void logistic_fwd_kernel(const float* __restrict__ x,
                                                           float* __restrict__ y, size_t n) {
  const size_t n4 = n / 4, stride = (size_t)gridDim.x * TPB, first = blockIdx.x * (size_t)TPB + threadIdx.x;
  for (size_t e = first; e < n4; e += stride) {
    const float4 v = reinterpret_cast<const float4*>(x)[e];
    __builtin_nontemporal_store(vec4{logistic(v.x), logistic(v.y), logistic(v.z), logistic(v.w)},
                                reinterpret_cast<vec4*>(y) + e);
  }
  for (size_t e = 4 * n4 + first; e < n; e += stride) y[e] = logistic(x[e]);
}

__global__ __launch_bounds__(TPB) void logistic_bwd_kernel(const float* __restrict__ y,
                                                           const float* __restrict__ d_y,
                                                           float* __restrict__ d_x, size_t n) {
  const size_t n4 = n / 4, stride = (size_t)gridDim.x * TPB, first = blockIdx.x * (size_t)TPB + threadIdx.x;
  for (size_t e = first; e < n4; e += stride) {
    const float4 v = reinterpret_cast<const float4*>(y)[e], d = reinterpret_cast<const float4*>(d_y)[e];
    __builtin_nontemporal_store(vec4{d.x * v.x * (1.0f - v.x), d.y * v.y * (1.0f - v.y),
                                     d.z * v.z * (1.0f - v.z), d.w * v.w * (1.0f - v.w)},
                                reinterpret_cast<vec4*>(d_x) + e);
  }
  for (size_t e = 4 * n4 + first; e < n; e += stride) {
    const float v = y[e];
    d_x[e] = d_y[e] * v * (1.0f - v);
  }
}

inline int launched() { return hipGetLastError() == hipSuccess ? CNN_OK : CNN_EHIP; }

// ---- launch plans of the matrix-core kernels ----------------------------------------------------
constexpr int LDS_LIMIT = 64 * 1024 - 512;  // bytes of dynamic LDS one workgroup may ask for
constexpr int LDS_TARGET = 48 * 1024;       // preferred, so that three workgroups share a compute unit
constexpr int WGRAD_LDS_TARGET = 36 * 1024; // both buffers of the weight gradient: four workgroups per compute unit
constexpr int CU_LDS = 160 * 1024;
constexpr int NUM_CU = 256;
constexpr int MAX_GROUP = 64;               // images per group
constexpr int MAX_PARTIALS = 1024;          // workgroup columns (partial sums) of the weight gradient

// Workgroups that keep every compute unit as full as the LDS use allows (at most eight each).
unsigned resident_workgroups(size_t lds_bytes) {
  size_t per_cu = CU_LDS / (lds_bytes + 512);
  if (per_cu > 8) per_cu = 8;
  if (per_cu < 1) per_cu = 1;
  return (unsigned)(NUM_CU * per_cu);
}

// LDS cycles of the gathered-operand reads of the first two column tiles over the first K steps, in
// a model of the 64 four-byte banks (measured: a 64-lane read of every second word costs what a read of
// consecutive words costs, every fourth word twice as much): a wave's read is served in two halves of
// 32 lanes, and a half takes as many cycles as the largest number of different words that fall into one bank.
// Lane (q, j) of K step s reads word koff(4 s + q) + poff(16 tile + j).
constexpr int LDS_BANKS = 64;
int gather_read_cost(int LW, int LP, int LI, int KH, int KWP, int K, int OWP, int COLS, int P) {
  const int steps = (K + 3) / 4 < 16 ? (K + 3) / 4 : 16;
  int cost = 0;
  for (int tile = 0; tile < 2; ++tile)
    for (int s = 0; s < steps; ++s)
      for (int half = 0; half < 2; ++half) {
        int word[32], worst = 0;
        for (int l = 0; l < 32; ++l) {
          const int kk = 4 * s + 2 * half + (l >> 4), n = 16 * tile + (l & 15);
          const int c = kk / (KH * KWP), rem = kk % (KH * KWP), img = n / COLS, r = n % COLS;
          word[l] = (kk < K ? c * LP + (rem / KWP) * LW + rem % KWP : 0) + img * LI + (r / OWP) * LW + P * (r % OWP);
        }
        int per_bank[LDS_BANKS] = {0};  // different words per bank: each word counted at its first lane
        for (int l = 0; l < 32; ++l) {
          bool first = true;
          for (int e = 0; e < l; ++e) first = first && word[e] != word[l];
          if (first && ++per_bank[word[l] & (LDS_BANKS - 1)] > worst) worst = per_bank[word[l] & (LDS_BANKS - 1)];
        }
        cost += worst;
      }
  return cost;
}

// Row stride (floats) of a bordered plane: the natural one or up to eight floats more, whichever the
// model above likes best.  (C1's input error, 24 + 2*4 = 32 columns: every row starts in the same
// bank and the read takes 14 cycles instead of 2; 36 columns make it conflict-free.)  Remembered per
// shape, since a call should not pay for the search.
int bordered_row_stride(int SC, int SH, int SW, int KH, int KW, int OH, int OW, int pady, int padx, int P) {
  struct Entry {
    int key[10], LW;
  };
  static Entry memo[16];
  static int used = 0, next = 0;
  static std::mutex guard;
  const int key[10] = {SC, SH, SW, KH, KW, OH, OW, pady, padx, P};
  std::lock_guard<std::mutex> lock(guard);
  for (int i = 0; i < used; ++i) {
    bool same = true;
    for (int e = 0; e < 10; ++e) same = same && memo[i].key[e] == key[e];
    if (same) return memo[i].LW;
  }
  const int base = SW + 2 * padx, rows = SH + 2 * pady, KWP = KW + P - 1, OWP = OW / P;
  int best_lw = base, best_cost = -1;
  for (int LW = base; LW <= base + 8; ++LW) {
    const int LP = rows * LW, cost = gather_read_cost(LW, LP, SC * LP, KH, KWP, SC * KH * KWP, OWP, OH * OWP, P);
    if (best_cost < 0 || cost < best_cost) best_cost = cost, best_lw = LW;
  }
  Entry& slot = memo[next];
  next = (next + 1) % 16;
  if (used < 16) ++used;
  for (int e = 0; e < 10; ++e) slot.key[e] = key[e];
  slot.LW = best_lw;
  return best_lw;
}

struct ConvPlan {
  igemm::ConvArgs a;
  int tp = 0;  // pixel tiles per wave job; 0: the shape does not fit, use the plain kernel
  unsigned grid = 0;
  size_t lds_bytes = 0;
};

// dst[B][M][OH][OW] from src[B][SC][SH][SW] staged with a border of (pady, padx), P output pixels
// per GEMM column.  tp = 0 when the operands do not fit in LDS.
ConvPlan plan_conv_layout(const float* src, const float* w, const float* bias, float* dst, int B, int M,
                          int SC, int SH, int SW, int KH, int KW, int OH, int OW, int pady, int padx, int flip,
                          int P, long long LW) {
  ConvPlan p;
  igemm::ConvArgs& a = p.a;
  a.src = src, a.w = w, a.bias = bias, a.dst = dst;
  a.B = B, a.M = M, a.SC = SC, a.SH = SH, a.SW = SW, a.KH = KH, a.KW = KW, a.OH = OH, a.OW = OW;
  a.pady = pady, a.padx = padx, a.flip = flip, a.zero_fill = (pady || padx) ? 1 : 0;
  a.P = P, a.MR = M * P, a.KWP = KW + P - 1, a.OWP = OW / P;
  const long long K = (long long)SC * KH * a.KWP, LP = (SH + 2LL * pady) * LW, LI = SC * LP;
  const long long COLS = (long long)OH * a.OWP, MT = ((long long)a.MR + 15) / 16, NBK = (K + 15) / 16;
  const long long R = a.MR < 16 ? a.MR : 16;
  if ((MT * (R + 1) * 4 + 4) * (4 * NBK + 4) + 16 * MT + LI + 2 * COLS + 16 > LDS_LIMIT / 4) return p;  // not even one image
  a.K = (int)K, a.LW = (int)LW, a.LP = (int)LP, a.LI = (int)LI, a.MT = (int)MT, a.R = (int)R, a.NBK = (int)NBK;
  a.SP = igemm::row_stride(a.NBK);
  auto bytes = [&](int nb) {
    a.NB = nb;
    return (long long)igemm::conv_lds(a).total * 4;
  };
  if (bytes(1) > LDS_LIMIT) return p;
  // Images per group: enough for four column tiles, more when the batch is large, within the LDS
  // target; among the admissible sizes the one that wastes the fewest matrix instructions on
  // padding tiles and idle waves.
  const int nb_tiles = (int)((64 + COLS - 1) / COLS);
  int nb_want = (B + 2047) / 2048;
  if (nb_want < nb_tiles) nb_want = nb_tiles;
  if (nb_want > MAX_GROUP) nb_want = MAX_GROUP;
  if (nb_want > B) nb_want = B;
  double best = -1.0;
  int best_nb = 1, best_tp = 1;
  for (int nb = 1; nb <= nb_want; ++nb) {
    const long long by = bytes(nb);
    if (by > LDS_LIMIT || (by > LDS_TARGET && nb > nb_tiles)) break;
    for (int tp = 1; tp <= 4; tp <<= 1) {
      const long long PT = (nb * COLS + 15) / 16, jobs = ((PT + tp - 1) / tp) * MT;
      const double used = (double)nb * COLS / 16.0 * MT, slots = (double)((jobs + 3) / 4) * 4 * tp;
      const double score = used / slots * (1.0 + 0.005 * tp);  // near ties: share the dense operand
      if (score >= best) best = score, best_nb = nb, best_tp = tp;
    }
  }
  a.NB = best_nb;
  p.tp = best_tp;
  a.groups = (B + a.NB - 1) / a.NB;
  p.lds_bytes = (size_t)bytes(a.NB);
  const unsigned resident = resident_workgroups(p.lds_bytes);
  p.grid = (unsigned)a.groups < resident ? (unsigned)a.groups : resident;
  // How a group reaches LDS: through registers that are loaded while the previous group is
  // multiplied, as 16-byte items when the images are borderless multiples of four floats.
  const long long per_image = (long long)SC * SH * SW, per_group = a.NB * per_image;
  if (!a.zero_fill && per_image % 4 == 0) {
    a.stage = igemm::STAGE_VECTOR;
    a.passes = (int)((per_group / 4 + igemm::THREADS * igemm::PFV - 1) / (igemm::THREADS * igemm::PFV));
  } else {
    a.stage = igemm::STAGE_SCALAR;
    a.passes = (int)((per_group + igemm::THREADS * igemm::PFS - 1) / (igemm::THREADS * igemm::PFS));
  }
  a.inv_sp = 1.0f / (float)a.SP, a.inv_r1 = 1.0f / (float)(a.R + 1), a.inv_p = 1.0f / (float)P;
  a.inv_khkwp = 1.0f / (float)(KH * a.KWP), a.inv_kwp = 1.0f / (float)a.KWP;
  a.inv_ohowp = 1.0f / (float)COLS, a.inv_owp = 1.0f / (float)a.OWP;
  a.inv_sw = 1.0f / (float)SW, a.inv_sh = 1.0f / (float)SH;
  return p;
}

// Bordered planes get the row stride the bank model prefers when the operands still fit with it.
ConvPlan plan_conv_packed(const float* src, const float* w, const float* bias, float* dst, int B, int M,
                          int SC, int SH, int SW, int KH, int KW, int OH, int OW, int pady, int padx, int flip,
                          int P) {
  const long long natural = SW + 2LL * padx, K = (long long)SC * KH * (KW + P - 1);
  // the search works in int: only for planes that could fit in LDS at all
  if ((pady || padx) && SC * (SH + 2LL * pady) * natural < LDS_LIMIT / 4 && K < (1 << 20)) {
    const long long LW = bordered_row_stride(SC, SH, SW, KH, KW, OH, OW, pady, padx, P);
    if (LW != natural) {
      const ConvPlan p = plan_conv_layout(src, w, bias, dst, B, M, SC, SH, SW, KH, KW, OH, OW, pady, padx, flip, P, LW);
      if (p.tp) return p;
    }
  }
  return plan_conv_layout(src, w, bias, dst, B, M, SC, SH, SW, KH, KW, OH, OW, pady, padx, flip, P, natural);
}

// The packing factor: the largest divisor P of OW with M*P <= 16 whose operands fit in LDS (a wider
// kernel row costs LDS for the weight table); 1 for kernels one column wide, where packing gains nothing.
ConvPlan plan_conv(const float* src, const float* w, const float* bias, float* dst, int B, int M, int SC,
                   int SH, int SW, int KH, int KW, int OH, int OW, int pady, int padx, int flip) {
  if (KW > 1)
    for (int P = 16 / M; P >= 2; --P) {
      if (OW % P) continue;
      const ConvPlan p = plan_conv_packed(src, w, bias, dst, B, M, SC, SH, SW, KH, KW, OH, OW, pady, padx, flip, P);
      if (p.tp) return p;
    }
  return plan_conv_packed(src, w, bias, dst, B, M, SC, SH, SW, KH, KW, OH, OW, pady, padx, flip, 1);
}

int launch_conv(const ConvPlan& p, hipStream_t stream) {
  switch (p.tp) {
    case 4: igemm::conv_kernel<4><<<p.grid, igemm::THREADS, p.lds_bytes, stream>>>(p.a); break;
    case 2: igemm::conv_kernel<2><<<p.grid, igemm::THREADS, p.lds_bytes, stream>>>(p.a); break;
    default: igemm::conv_kernel<1><<<p.grid, igemm::THREADS, p.lds_bytes, stream>>>(p.a); break;
  }
  return launched();
}

struct WgradPlan {
  igemm::WgradArgs a;
  bool fits = false;
  bool one_wave_per_image = false;  // the shape of one of the network's convolutions: conv1:: / conv2::bwd_weight_kernel, gx workgroups
  bool fc_rows = false;             // the shape of the network's fully connected layer: fc::bwd_weight_kernel, gx workgroups
  unsigned gx = 0, gy = 0;
  size_t lds_bytes = 0, workspace_bytes = 0;
};

WgradPlan plan_wgrad_packed(int B, int Cin, int H, int W, int Cout, int KH, int KW, int P) {
  WgradPlan p;
  igemm::WgradArgs& a = p.a;
  a.in = nullptr, a.d_out = nullptr, a.part = nullptr;
  a.B = B, a.Cin = Cin, a.H = H, a.W = W, a.Cout = Cout, a.KH = KH, a.KW = KW;
  a.Ho = H - KH + 1, a.Wo = W - KW + 1;
  a.P = P, a.MR = Cout * P, a.KWP = KW + P - 1, a.WOP = a.Wo / P;
  const long long K = (long long)Cin * KH * a.KWP, HoWo = (long long)a.Ho * a.Wo, SPI = (long long)a.Ho * a.WOP;
  const long long per_image = (long long)Cin * H * W;
  if (2 * (per_image + 2 * SPI) > LDS_LIMIT / 4 || K > (1 << 20)) return p;
  a.K = (int)K, a.MT = (a.MR + 15) / 16, a.NT = (int)((K + 15) / 16), a.NTG = (a.NT + 15) / 16;
  a.KS = a.NT >= 3 ? 1 : a.NT == 2 ? 2 : 4;
  a.R = a.MR < 16 ? a.MR : 16;
  a.vec_x = per_image % 4 == 0 ? 1 : 0;
  a.vec_d = (P == 1 && HoWo % 4 == 0) ? 1 : 0;
  const int chunk_x = a.vec_x ? 256 : 64, chunk_d = a.vec_d ? 256 : 64;  // floats per staging load instruction
  auto bytes = [&](int nb) {
    a.NB = nb;
    a.NBK = (int)((nb * SPI + 15) / 16);
    a.NPS = igemm::error_row_stride(a.NBK);
    a.XS = (int)((nb * per_image + chunk_x - 1) / chunk_x * chunk_x);
    return (long long)igemm::wgrad_lds(a).total * 4;
  };
  if (SPI > 16LL * chunk_d || bytes(1) > LDS_LIMIT) return p;
  int nb = 1;
  const int nb_fill = (B + MAX_PARTIALS - 1) / MAX_PARTIALS;
  // more images per group while the partial sums stay at MAX_PARTIALS columns, the two buffers stay
  // within the LDS target and a row of the output error within sixteen load instructions
  for (int c = 2; c <= MAX_GROUP && c <= B && c <= nb_fill && bytes(c) <= WGRAD_LDS_TARGET && c * SPI <= 16LL * chunk_d;
       ++c)
    nb = c;
  p.lds_bytes = (size_t)bytes(nb);
  a.groups = (B + nb - 1) / nb;
  unsigned gx = resident_workgroups(p.lds_bytes) / (unsigned)(a.MT * a.NTG);
  if (gx < 1) gx = 1;
  if (gx > MAX_PARTIALS) gx = MAX_PARTIALS;
  if (gx > (unsigned)a.groups) gx = (unsigned)a.groups;
  p.gx = gx;
  p.gy = (unsigned)(a.MT * a.NTG);
  p.workspace_bytes = ((size_t)gx * a.MT * a.NT * 256 + (size_t)gx * a.MT * 16) * sizeof(float);
  a.inv_p = 1.0f / (float)P, a.inv_khkwp = 1.0f / (float)(KH * a.KWP), a.inv_kwp = 1.0f / (float)a.KWP;
  a.inv_spi = 1.0f / (float)SPI, a.inv_wop = 1.0f / (float)a.WOP;
  p.fits = true;
  return p;
}

// The packing factor that needs the fewest matrix instructions per image (column tiles x blocks of
// pixel slots) among the divisors P of Wo with Cout*P <= 16; 1 for kernels one column wide.
WgradPlan plan_wgrad(int B, int Cin, int H, int W, int Cout, int KH, int KW) {
  if (conv1::shape_fits(Cin, H, W, Cout, KH, KW)) {
    WgradPlan p;
    igemm::WgradArgs& a = p.a;
    a.in = nullptr, a.d_out = nullptr, a.part = nullptr;
    a.B = B, a.Cin = Cin, a.H = H, a.W = W, a.Cout = Cout, a.KH = KH, a.KW = KW;
    a.P = 2, a.MT = 1, a.NT = 2;  // rows (map, x parity), columns the shifted taps: what the second kernel joins
    p.fits = p.one_wave_per_image = true;
    const unsigned groups = (unsigned)((B + conv1::WAVES_PER_GROUP - 1) / conv1::WAVES_PER_GROUP);
    p.gx = groups < 2u * NUM_CU ? groups : 2u * NUM_CU;
    p.gy = 1;
    p.workspace_bytes = conv1::bwd_weight_workspace_bytes(p.gx);
    return p;
  }
  if (H == 1 && W == 1 && KH == 1 && KW == 1 && fc::shape_fits(Cin, Cout)) {
    WgradPlan p;
    igemm::WgradArgs& a = p.a;
    a.in = nullptr, a.d_out = nullptr, a.part = nullptr;
    a.B = B, a.Cin = Cin, a.H = H, a.W = W, a.Cout = Cout, a.KH = KH, a.KW = KW;
    a.P = 1, a.MT = 1, a.NT = fc::NT;  // what the second kernel needs to find the partial tiles
    p.fits = p.fc_rows = true;
    // a wave takes fc::AHEAD steps of four images per memory round trip
    const int per_group = 4 * fc::AHEAD * fc::WGRAD_WAVES;
    const unsigned groups = (unsigned)((B + per_group - 1) / per_group);
    p.gx = groups < 2u * NUM_CU ? groups : 2u * NUM_CU;
    p.gy = 1;
    p.workspace_bytes = fc::bwd_weight_workspace_bytes(p.gx);
    return p;
  }
  if (conv2::shape_fits(Cin, H, W, Cout, KH, KW)) {
    WgradPlan p;
    igemm::WgradArgs& a = p.a;
    a.in = nullptr, a.d_out = nullptr, a.part = nullptr;
    a.B = B, a.Cin = Cin, a.H = H, a.W = W, a.Cout = Cout, a.KH = KH, a.KW = KW;
    a.P = 1, a.MT = 1, a.NT = 10;  // what the second kernel needs to find the partial tiles
    p.fits = p.one_wave_per_image = true;
    const unsigned groups = (unsigned)((B + conv2::WAVES_PER_GROUP - 1) / conv2::WAVES_PER_GROUP);
    p.gx = groups < 2u * NUM_CU ? groups : 2u * NUM_CU;  // two workgroups per compute unit are resident
    p.gy = 1;
    p.workspace_bytes = conv2::bwd_weight_workspace_bytes(p.gx);
    return p;
  }
  int best = 1;
  if (KW > 1) {
    const long long Ho = H - KH + 1, Wo = W - KW + 1;
    long long best_cost = -1;
    for (int P = 1; P * Cout <= 16; ++P) {
      if (Wo % P) continue;
      const long long cost = (((long long)Cin * KH * (KW + P - 1) + 15) / 16) * ((Ho * (Wo / P) + 15) / 16);
      if (best_cost < 0 || cost < best_cost) best_cost = cost, best = P;
    }
  }
  for (int P = best; P > 1; --P) {
    if ((W - KW + 1) % P) continue;
    const WgradPlan p = plan_wgrad_packed(B, Cin, H, W, Cout, KH, KW, P);
    if (p.fits) return p;
  }
  return plan_wgrad_packed(B, Cin, H, W, Cout, KH, KW, 1);
}

// ---- reduced precision: the bf16 matrix-core kernel ------------------------------------------------
struct Conv16Plan {
  igemm16::Args a;
  int tp = 0;  // pixel tiles per wave job; 0: the shape does not fit, use the plain kernel
  unsigned grid = 0;
  size_t lds_bytes = 0;
};

Conv16Plan plan_conv16_packed(const float* src, const float* w, const float* bias, float* dst, int B, int M, int SC,
                              int SH, int SW, int KH, int KW, int OH, int OW, int pady, int padx, int flip, int P) {
  Conv16Plan p;
  igemm16::Args& a = p.a;
  a.src = src, a.w = w, a.bias = bias, a.dst = dst;
  a.B = B, a.M = M, a.SC = SC, a.SH = SH, a.SW = SW, a.KH = KH, a.KW = KW, a.OH = OH, a.OW = OW;
  a.pady = pady, a.padx = padx, a.flip = flip;
  a.P = P, a.MR = M * P, a.KWP = KW + P - 1, a.OWP = OW / P;
  const long long C8 = ((long long)SC + 7) & ~7LL, K = (long long)KH * a.KWP * C8, NBK = (K + 31) / 32;
  const long long LW = SW + 2LL * padx, LPIX = (SH + 2LL * pady) * LW, MT = ((long long)a.MR + 15) / 16;
  const long long COLS = (long long)OH * a.OWP;
  // first in 64 bits: one image and the tables must fit before anything is narrowed to int
  if (16 * MT * (64 * NBK + 16) + 16 * NBK + 64 * MT + 8 * COLS + 2 * LPIX * C8 + 64 > LDS_LIMIT) return p;
  a.C8 = (int)C8, a.K = (int)K, a.NBK = (int)NBK, a.RS = (int)(64 * NBK + 16), a.LW = (int)LW, a.LPIX = (int)LPIX;
  a.MT = (int)MT;
  auto bytes = [&](int nb) {
    a.NB = nb;
    return (long long)igemm16::lds_layout(a).total;
  };
  if (bytes(1) > LDS_LIMIT) return p;
  const int nb_tiles = (int)((64 + COLS - 1) / COLS);
  int nb_want = (B + 2047) / 2048;
  if (nb_want < nb_tiles) nb_want = nb_tiles;
  if (nb_want > MAX_GROUP) nb_want = MAX_GROUP;
  if (nb_want > B) nb_want = B;
  double best = -1.0;
  int best_nb = 1, best_tp = 1;
  for (int nb = 1; nb <= nb_want; ++nb) {
    const long long by = bytes(nb);
    if (by > LDS_LIMIT || (by > LDS_TARGET && nb > nb_tiles)) break;
    for (int tp = 1; tp <= 4; tp <<= 1) {
      const long long PT = (nb * COLS + 15) / 16, jobs = ((PT + tp - 1) / tp) * MT;
      const double used = (double)nb * COLS / 16.0 * MT, slots = (double)((jobs + 3) / 4) * 4 * tp;
      // this kernel is bound by LDS reads, not by matrix slots: a job reads 1 KB of weights per
      // block once for its tp tiles and 1 KB of pixels per tile
      const double score = used / slots * tp / (tp + 1.0);
      if (score >= best) best = score, best_nb = nb, best_tp = tp;
    }
  }
  a.NB = best_nb;
  p.tp = best_tp;
  a.groups = (B + a.NB - 1) / a.NB;
  p.lds_bytes = (size_t)bytes(a.NB);
  const unsigned resident = resident_workgroups(p.lds_bytes);
  p.grid = (unsigned)a.groups < resident ? (unsigned)a.groups : resident;
  a.inv_kp = 1.0f / (float)(32 * a.NBK), a.inv_c8 = 1.0f / (float)a.C8, a.inv_kwp = 1.0f / (float)a.KWP;
  a.inv_cols = 1.0f / (float)COLS, a.inv_owp = 1.0f / (float)a.OWP, a.inv_p = 1.0f / (float)P, a.inv_chhw = 1.0f / (float)(C8 / 8 * SH * SW);
  a.inv_hw = 1.0f / (float)(SH * SW), a.inv_sw = 1.0f / (float)SW;
  return p;
}

// Column packing as in the fp32 kernel (P pixels of a row per column, rows (m, sh)): among the
// divisors P of OW with M*P <= 16 the one with the fewest 16-byte pixel reads per image, tiles x
// K blocks; 1 for kernels one column wide.
Conv16Plan plan_conv16(const float* src, const float* w, const float* bias, float* dst, int B, int M, int SC,
                       int SH, int SW, int KH, int KW, int OH, int OW, int pady, int padx, int flip) {
  Conv16Plan best = plan_conv16_packed(src, w, bias, dst, B, M, SC, SH, SW, KH, KW, OH, OW, pady, padx, flip, 1);
  if (KW == 1) return best;
  auto cost = [&](const Conv16Plan& p) { return (double)OH * p.a.OWP / 16.0 * p.a.NBK; };
  for (int P = 2; P * M <= 16; ++P) {
    if (OW % P) continue;
    const Conv16Plan p = plan_conv16_packed(src, w, bias, dst, B, M, SC, SH, SW, KH, KW, OH, OW, pady, padx, flip, P);
    if (p.tp && (!best.tp || cost(p) < cost(best))) best = p;
  }
  return best;
}

int launch_conv16(const Conv16Plan& p, hipStream_t stream) {
  switch (p.tp) {
    case 4: igemm16::conv_kernel<4><<<p.grid, igemm::THREADS, p.lds_bytes, stream>>>(p.a); break;
    case 2: igemm16::conv_kernel<2><<<p.grid, igemm::THREADS, p.lds_bytes, stream>>>(p.a); break;
    default: igemm16::conv_kernel<1><<<p.grid, igemm::THREADS, p.lds_bytes, stream>>>(p.a); break;
  }
  return launched();
}

struct Wgrad16Plan {
  igemm16::WArgs a;
  bool fits = false;
  unsigned gx = 0, gy = 0;
  size_t lds_bytes = 0, workspace_bytes = 0;
};

Wgrad16Plan plan_wgrad16(int B, int Cin, int H, int W, int Cout, int KH, int KW) {
  Wgrad16Plan p;
  igemm16::WArgs& a = p.a;
  a.in = nullptr, a.d_out = nullptr, a.part = nullptr;
  a.B = B, a.Cin = Cin, a.H = H, a.W = W, a.Cout = Cout, a.KH = KH, a.KW = KW;
  a.Ho = H - KH + 1, a.Wo = W - KW + 1;
  const long long K = (long long)Cin * KH * KW, NT = (K + 15) / 16, MT = ((long long)Cout + 15) / 16;
  const long long XG = (a.Wo + 7) / 8, WP = 8 * XG, RUNS = a.Ho * XG;
  const long long WR = WP + 8 > (((long long)W + 7) & ~7LL) ? WP + 8 : (((long long)W + 7) & ~7LL), W4 = (W + 3) / 4;
  if (KW > 8) return p;  // the shifted copies are made for at most eight kernel columns
  // in 64 bits first: one image must fit
  if (16 * (16 * ((RUNS + 3) / 4 * 4) + 16) + 2 * Cin * (long long)H * (KW * WP + WR) + 64 > LDS_LIMIT || NT > (1 << 20)) return p;
  a.K = (int)K, a.NT = (int)NT, a.MT = (int)MT, a.NTG = (int)((NT + 15) / 16), a.XG = (int)XG, a.WP = (int)WP;
  a.WR = (int)WR, a.W4 = (int)W4, a.DR = Cout < 16 ? Cout : 16;
  auto bytes = [&](int nb) {
    a.NB = nb;
    a.NBK = (int)((nb * RUNS + 3) / 4);
    a.RSD = 64 * a.NBK + 16;
    return (long long)igemm16::wlds_layout(a).total;
  };
  if (bytes(1) > LDS_LIMIT) return p;
  p.fits = true;
  int nb = 1;
  const int nb_fill = (B + MAX_PARTIALS - 1) / MAX_PARTIALS;
  for (int c = 2; c <= MAX_GROUP && c <= B && c <= (nb_fill > 4 ? nb_fill : 4) && bytes(c) <= WGRAD_LDS_TARGET; ++c) nb = c;
  p.lds_bytes = (size_t)bytes(nb);
  a.groups = (B + nb - 1) / nb;
  unsigned gx = resident_workgroups(p.lds_bytes) / (unsigned)(a.MT * a.NTG);
  if (gx < 1) gx = 1;
  if (gx > 2 * MAX_PARTIALS) gx = 2 * MAX_PARTIALS;  // every resident workgroup: this kernel lives on hidden latency
  if (gx > (unsigned)a.groups) gx = (unsigned)a.groups;
  p.gx = gx;
  p.gy = (unsigned)(a.MT * a.NTG);
  p.workspace_bytes = ((size_t)gx * a.MT * a.NT * 256 + (size_t)gx * a.MT * 16) * sizeof(float);
  a.inv_khkw = 1.0f / (float)(KH * KW), a.inv_kw = 1.0f / (float)KW, a.inv_xg = 1.0f / (float)XG;
  a.inv_hoxg = 1.0f / (float)RUNS, a.inv_hxg = 1.0f / (float)(H * XG);
  a.inv_cinhxg = 1.0f / (float)(Cin * H * XG), a.inv_w4 = 1.0f / (float)W4, a.inv_hw4 = 1.0f / (float)(H * W4);
  a.inv_cinhw4 = 1.0f / (float)(Cin * H * W4);
  return p;
}

inline bool conv_args_ok(int B, int Cin, int H, int W, int Cout, int KH, int KW) {
  return B >= 1 && Cin >= 1 && Cout >= 1 && KH >= 1 && KW >= 1 && H >= KH && W >= KW &&
         (size_t)Cout * Cin * KH * KW + (size_t)Cout < (size_t)1 << 30;
}

inline bool wgrad_args_ok(const float* in, const float* d_out, const float* d_k, const float* d_bias, int B, int Cin,
                          int H, int W, int Cout, int KH, int KW) {
  return in && d_out && d_k && conv_args_ok(B, Cin, H, W, Cout, KH, KW) && aligned16(in) && aligned16(d_out) &&
         aligned16(d_k) && (!d_bias || aligned16(d_bias));
}

// The matrix-core weight gradient: partial tiles per workgroup column into `part`, then the
// fixed-order sum of the columns.
int launch_wgrad(WgradPlan& p, const float* in, const float* d_out, float* d_k, float* d_bias, float* part,
                 hipStream_t st) {
  p.a.in = in, p.a.d_out = d_out, p.a.part = part;
  const dim3 grid(p.gx, p.gy);
  if (p.fc_rows)
    fc::bwd_weight_kernel<<<p.gx, fc::WGRAD_THREADS, 0, st>>>(in, d_out, part, p.a.B);
  else if (p.one_wave_per_image && p.a.Cin == 1)
    conv1::bwd_weight_kernel<<<p.gx, conv1::THREADS, 0, st>>>(in, d_out, part, p.a.B);
  else if (p.one_wave_per_image)
    conv2::bwd_weight_kernel<<<p.gx, conv2::THREADS, 0, st>>>(in, d_out, part, p.a.B);
  else if (p.a.vec_x && p.a.vec_d)
    igemm::wgrad_kernel<16, 16><<<grid, igemm::THREADS, p.lds_bytes, st>>>(p.a);
  else if (p.a.vec_x)
    igemm::wgrad_kernel<16, 4><<<grid, igemm::THREADS, p.lds_bytes, st>>>(p.a);
  else if (p.a.vec_d)
    igemm::wgrad_kernel<4, 16><<<grid, igemm::THREADS, p.lds_bytes, st>>>(p.a);
  else
    igemm::wgrad_kernel<4, 4><<<grid, igemm::THREADS, p.lds_bytes, st>>>(p.a);
  const igemm::WgradArgs& a = p.a;
  const size_t outputs = (size_t)a.Cout * a.Cin * a.KH * a.KW + a.Cout;
  const int epw = outputs >= 2048 ? 16 : outputs >= 512 ? 8 : 4;  // outputs per workgroup of the second kernel
  igemm::wgrad_reduce_kernel<<<(unsigned)((outputs + epw - 1) / epw), igemm::THREADS, 0, st>>>(
      a.part, (int)p.gx, a.MT, a.NT, a.Cout, a.Cin, a.KH, a.KW, a.P, epw, d_k, d_bias);
  return launched();
}

int launch_wgrad_plain(const float* in, const float* d_out, float* d_k, float* d_bias, int B, int Cin, int H, int W,
                       int Cout, int KH, int KW, hipStream_t st) {
  const unsigned blocks = (unsigned)(Cout * Cin * KH * KW + (d_bias ? Cout : 0));
  conv_bwd_weight_kernel<false><<<blocks, TPB, 0, st>>>(in, d_out, d_k, d_bias, B, Cin, H, W, Cout, KH, KW);
  return launched();
}

// ---- built-in scratch for callers that cannot allocate ----------------------------------------------
// Device memory that belongs to the loaded code object: every GPU the library runs on holds its own
// copy at its own address until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; kernels get the address that call returned for the current device.
constexpr size_t SCRATCH_FLOATS = CNN_STATIC_SCRATCH_BYTES / sizeof(float);
static __device__ __align__(256) float scratch[SCRATCH_FLOATS];
constexpr int SCRATCH_MAX_DEVICES = 64;

// The current device's copy of `scratch`, looked up once per device.
int scratch_of_current_device(float** out) {
  static float* ptr[SCRATCH_MAX_DEVICES] = {};
  static std::mutex guard;
  int dev = -1;
  CNN_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= SCRATCH_MAX_DEVICES) return CNN_EINVAL;
  std::lock_guard<std::mutex> lock(guard);
  if (!ptr[dev]) {
    void* p = nullptr;
    CNN_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return CNN_EHIP;
    ptr[dev] = static_cast<float*>(p);
  }
  *out = ptr[dev];
  return CNN_OK;
}

// Workgroups of the fully connected layer's row kernels: one tile of sixteen rows per wave while the
// machine has room, then the waves loop.
unsigned fc_groups(int B) {
  const long long tiles = ((long long)B + fc::TILE - 1) / fc::TILE;
  const long long groups = (tiles + fc::WAVES_PER_GROUP - 1) / fc::WAVES_PER_GROUP, resident = 4LL * NUM_CU;
  return (unsigned)(groups < resident ? groups : resident);
}

}  // namespace

extern "C" {

int cnn_conv_fwd(const float* in, const float* k, const float* bias, float* out, int B, int Cin, int H,
                 int W, int Cout, int KH, int KW, void* hip_stream) {
  if (!in || !k || !out || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(k) || !aligned16(out) || (bias && !aligned16(bias))) return CNN_EINVAL;
  if (conv1::shape_fits(Cin, H, W, Cout, KH, KW)) {  // the network's first convolution: one wave per image
    const int groups = (B + conv1::WAVES_PER_GROUP - 1) / conv1::WAVES_PER_GROUP, resident = 2 * NUM_CU;
    conv1::forward_kernel<<<groups < resident ? groups : resident, conv1::THREADS, 0, (hipStream_t)hip_stream>>>(
        in, k, bias, out, B);
    return launched();
  }
  if (conv2::shape_fits(Cin, H, W, Cout, KH, KW)) {  // the network's second convolution: one wave per image
    // (two workgroups per compute unit; one, three or four measured the same: the kernel is bound by its matrix instructions)
    const int groups = (B + conv2::WAVES_PER_GROUP - 1) / conv2::WAVES_PER_GROUP, resident = 2 * NUM_CU;
    conv2::forward_kernel<<<groups < resident ? groups : resident, conv2::THREADS, 0, (hipStream_t)hip_stream>>>(
        in, k, bias, out, B);
    return launched();
  }
  const ConvPlan p = plan_conv(in, k, bias, out, B, Cout, Cin, H, W, KH, KW, H - KH + 1, W - KW + 1, 0, 0, 0);
  if (p.tp) return launch_conv(p, (hipStream_t)hip_stream);
  const size_t total = (size_t)B * Cout * (H - KH + 1) * (W - KW + 1);
  conv_fwd_kernel<false><<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(in, k, bias, out, total, Cin,
                                                                                H, W, Cout, KH, KW);
  return launched();
}

int cnn_conv_bwd_input(const float* d_out, const float* k, float* d_in, int B, int Cin, int H, int W,
                       int Cout, int KH, int KW, void* hip_stream) {
  if (!d_out || !k || !d_in || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(k) || !aligned16(d_in)) return CNN_EINVAL;
  if (col2im::shape_fits(Cin, H, W, Cout, KH, KW)) {
    // the shape of the network's second convolution: col2im form, 120 instead of 414 matrix instructions per image
    const int groups = (B + col2im::WAVES_PER_GROUP - 1) / col2im::WAVES_PER_GROUP;
    const int resident = 2 * NUM_CU;  // 112 registers per lane: four waves per SIMD, two workgroups per compute unit
    col2im::conv_bwd_input_kernel<<<groups < resident ? groups : resident, 64 * col2im::WAVES_PER_GROUP, 0,
                                    (hipStream_t)hip_stream>>>(d_out, k, d_in, B);
    return launched();
  }
  if (conv1::shape_fits(Cin, H, W, Cout, KH, KW)) {
    // the shape of the network's first convolution: one output map, nothing for a matrix tile to share
    const int groups = (B + conv1::WAVES_PER_GROUP - 1) / conv1::WAVES_PER_GROUP;
    conv1::bwd_input_kernel<<<groups < NUM_CU ? groups : NUM_CU, conv1::THREADS, 0, (hipStream_t)hip_stream>>>(
        d_out, k, d_in, B);  // 128 KB of LDS: one workgroup per compute unit
    return launched();
  }
  const ConvPlan p = plan_conv(d_out, k, nullptr, d_in, B, Cin, Cout, H - KH + 1, W - KW + 1, KH, KW, H, W,
                               KH - 1, KW - 1, 1);
  if (p.tp) return launch_conv(p, (hipStream_t)hip_stream);
  const size_t total = (size_t)B * Cin * H * W;
  conv_bwd_input_kernel<false><<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, k, d_in, total,
                                                                                      Cin, H, W, Cout, KH, KW);
  return launched();
}

int cnn_conv_fwd_valu(const float* in, const float* k, const float* bias, float* out, int B, int Cin, int H,
                      int W, int Cout, int KH, int KW, void* hip_stream) {
  if (!in || !k || !out || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(k) || !aligned16(out) || (bias && !aligned16(bias))) return CNN_EINVAL;
  const size_t total = (size_t)B * Cout * (H - KH + 1) * (W - KW + 1);
  conv_fwd_kernel<false><<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(in, k, bias, out, total, Cin,
                                                                                H, W, Cout, KH, KW);
  return launched();
}

int cnn_conv_bwd_input_valu(const float* d_out, const float* k, float* d_in, int B, int Cin, int H, int W,
                            int Cout, int KH, int KW, void* hip_stream) {
  if (!d_out || !k || !d_in || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(k) || !aligned16(d_in)) return CNN_EINVAL;
  const size_t total = (size_t)B * Cin * H * W;
  conv_bwd_input_kernel<false><<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, k, d_in, total,
                                                                                      Cin, H, W, Cout, KH, KW);
  return launched();
}

int cnn_conv_fwd_bf16(const float* in, const float* k, const float* bias, float* out, int B, int Cin, int H,
                      int W, int Cout, int KH, int KW, void* hip_stream) {
  if (!in || !k || !out || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(k) || !aligned16(out) || (bias && !aligned16(bias))) return CNN_EINVAL;
  const Conv16Plan p = plan_conv16(in, k, bias, out, B, Cout, Cin, H, W, KH, KW, H - KH + 1, W - KW + 1, 0, 0, 0);
  if (p.tp) return launch_conv16(p, (hipStream_t)hip_stream);
  const size_t total = (size_t)B * Cout * (H - KH + 1) * (W - KW + 1);
  conv_fwd_kernel<true><<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(in, k, bias, out, total, Cin,
                                                                               H, W, Cout, KH, KW);
  return launched();
}

int cnn_conv_bwd_input_bf16(const float* d_out, const float* k, float* d_in, int B, int Cin, int H, int W,
                            int Cout, int KH, int KW, void* hip_stream) {
  if (!d_out || !k || !d_in || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(k) || !aligned16(d_in)) return CNN_EINVAL;
  const Conv16Plan p = plan_conv16(d_out, k, nullptr, d_in, B, Cin, Cout, H - KH + 1, W - KW + 1, KH, KW, H, W,
                                   KH - 1, KW - 1, 1);
  if (p.tp) return launch_conv16(p, (hipStream_t)hip_stream);
  const size_t total = (size_t)B * Cin * H * W;
  conv_bwd_input_kernel<true><<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, k, d_in, total,
                                                                                     Cin, H, W, Cout, KH, KW);
  return launched();
}

size_t cnn_conv_bwd_weight_workspace_bytes(int B, int Cin, int H, int W, int Cout, int KH, int KW) {
  if (!conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return 0;
  return plan_wgrad(B, Cin, H, W, Cout, KH, KW).workspace_bytes;
}

int cnn_conv_bwd_weight(const float* in, const float* d_out, float* d_k, float* d_bias, int B, int Cin,
                        int H, int W, int Cout, int KH, int KW, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  if (!wgrad_args_ok(in, d_out, d_k, d_bias, B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (workspace && !aligned16(workspace)) return CNN_EINVAL;
  WgradPlan p = plan_wgrad(B, Cin, H, W, Cout, KH, KW);
  if (p.fits && workspace && workspace_bytes >= p.workspace_bytes)
    return launch_wgrad(p, in, d_out, d_k, d_bias, static_cast<float*>(workspace), (hipStream_t)hip_stream);
  return launch_wgrad_plain(in, d_out, d_k, d_bias, B, Cin, H, W, Cout, KH, KW, (hipStream_t)hip_stream);
}

int cnn_conv_bwd_weight_static(const float* in, const float* d_out, float* d_k, float* d_bias, int B, int Cin,
                               int H, int W, int Cout, int KH, int KW, void* hip_stream) {
  if (!wgrad_args_ok(in, d_out, d_k, d_bias, B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  WgradPlan p = plan_wgrad(B, Cin, H, W, Cout, KH, KW);
  if (!p.fits)  // only the kernel without partial sums serves this shape: it needs no scratch at all
    return launch_wgrad_plain(in, d_out, d_k, d_bias, B, Cin, H, W, Cout, KH, KW, (hipStream_t)hip_stream);
  if (p.workspace_bytes > sizeof(float) * SCRATCH_FLOATS) return CNN_ESCRATCH;
  float* part = nullptr;
  const int rc = scratch_of_current_device(&part);
  if (rc != CNN_OK) return rc;
  // every partial tile and bias row the second kernel reads is written by the first one in the same
  // call, so nothing of the previous call's contents has to be cleared
  return launch_wgrad(p, in, d_out, d_k, d_bias, part, (hipStream_t)hip_stream);
}

size_t cnn_conv_bwd_weight_bf16_workspace_bytes(int B, int Cin, int H, int W, int Cout, int KH, int KW) {
  if (!conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return 0;
  return plan_wgrad16(B, Cin, H, W, Cout, KH, KW).workspace_bytes;
}

int cnn_conv_bwd_weight_bf16(const float* in, const float* d_out, float* d_k, float* d_bias, int B, int Cin,
                             int H, int W, int Cout, int KH, int KW, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  if (!in || !d_out || !d_k || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(d_out) || !aligned16(d_k) || (d_bias && !aligned16(d_bias)))
    return CNN_EINVAL;
  if (workspace && !aligned16(workspace)) return CNN_EINVAL;
  Wgrad16Plan p = plan_wgrad16(B, Cin, H, W, Cout, KH, KW);
  if (p.fits && workspace && workspace_bytes >= p.workspace_bytes) {
    p.a.in = in, p.a.d_out = d_out, p.a.part = static_cast<float*>(workspace);
    hipStream_t st = (hipStream_t)hip_stream;
    igemm16::wgrad_kernel<<<dim3(p.gx, p.gy), igemm::THREADS, p.lds_bytes, st>>>(p.a);
    const size_t outputs = (size_t)Cout * Cin * KH * KW + Cout;
    const int epw = outputs >= 2048 ? 16 : outputs >= 512 ? 8 : 4;
    igemm::wgrad_reduce_kernel<<<(unsigned)((outputs + epw - 1) / epw), igemm::THREADS, 0, st>>>(
        p.a.part, (int)p.gx, p.a.MT, p.a.NT, Cout, Cin, KH, KW, 1, epw, d_k, d_bias);
    return launched();
  }
  const unsigned blocks = (unsigned)(Cout * Cin * KH * KW + (d_bias ? Cout : 0));
  conv_bwd_weight_kernel<true><<<blocks, TPB, 0, (hipStream_t)hip_stream>>>(in, d_out, d_k, d_bias, B, Cin, H,
                                                                            W, Cout, KH, KW);
  return launched();
}

int cnn_avgpool_fwd(const float* in, float* out, int B, int C, int H, int W, void* hip_stream) {
  if (!in || !out || B < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(out)) return CNN_EINVAL;
  const size_t total = (size_t)B * C * (H / 2) * (W / 2);
  avgpool_fwd_kernel<<<grid_stream(total), TPB, 0, (hipStream_t)hip_stream>>>(in, out, total, W);
  return launched();
}

int cnn_avgpool_bwd(const float* d_out, float* d_in, int B, int C, int Ho, int Wo, void* hip_stream) {
  if (!d_out || !d_in || B < 1 || C < 1 || Ho < 1 || Wo < 1) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(d_in)) return CNN_EINVAL;
  const size_t total = (size_t)B * C * Ho * Wo;
  avgpool_bwd_kernel<<<grid_stream(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, d_in, total, Wo);
  return launched();
}

int cnn_fc_fwd(const float* in, const float* w, const float* bias, float* out, int B, int I, int O,
               void* hip_stream) {
  if (!in || !w || !out || B < 1 || I < 1 || O < 1) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(w) || !aligned16(out) || (bias && !aligned16(bias))) return CNN_EINVAL;
  if (fc::shape_fits(I, O)) {
    // the shape of the network's own layer: every wave takes tiles of sixteen rows straight from global memory
    fc::forward_kernel<<<fc_groups(B), fc::THREADS, 0, (hipStream_t)hip_stream>>>(in, w, bias, out, B);
    return launched();
  }
  const ConvPlan p = plan_conv(in, w, bias, out, B, O, I, 1, 1, 1, 1, 1, 1, 0, 0, 0);
  if (p.tp) return launch_conv(p, (hipStream_t)hip_stream);
  const size_t total = (size_t)B * O;
  fc_fwd_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(in, w, bias, out, total, I, O);
  return launched();
}

int cnn_fc_bwd_input(const float* d_out, const float* w, float* d_in, int B, int I, int O,
                     void* hip_stream) {
  if (!d_out || !w || !d_in || B < 1 || I < 1 || O < 1) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(w) || !aligned16(d_in)) return CNN_EINVAL;
  if (fc::shape_fits(I, O)) {
    fc::bwd_input_kernel<<<fc_groups(B), fc::THREADS, 0, (hipStream_t)hip_stream>>>(d_out, w, d_in, B);
    return launched();
  }
  const ConvPlan p = plan_conv(d_out, w, nullptr, d_in, B, I, O, 1, 1, 1, 1, 1, 1, 0, 0, 1);
  if (p.tp) return launch_conv(p, (hipStream_t)hip_stream);
  const size_t total = (size_t)B * I;
  fc_bwd_input_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, w, d_in, total, I, O);
  return launched();
}

size_t cnn_fc_bwd_weight_workspace_bytes(int B, int I, int O) {
  return cnn_conv_bwd_weight_workspace_bytes(B, I, 1, 1, O, 1, 1);
}

int cnn_fc_bwd_weight(const float* in, const float* d_out, float* d_w, float* d_bias, int B, int I, int O,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!in || !d_out || !d_w || B < 1 || I < 1 || O < 1 || (size_t)I * O + O >= (size_t)1 << 30)
    return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(d_out) || !aligned16(d_w) || (d_bias && !aligned16(d_bias)))
    return CNN_EINVAL;
  if (workspace && workspace_bytes >= cnn_fc_bwd_weight_workspace_bytes(B, I, O) &&
      cnn_fc_bwd_weight_workspace_bytes(B, I, O) > 0)
    return cnn_conv_bwd_weight(in, d_out, d_w, d_bias, B, I, 1, 1, O, 1, 1, workspace, workspace_bytes,
                               hip_stream);
  const unsigned blocks = (unsigned)(O * I + (d_bias ? O : 0));
  fc_bwd_weight_kernel<<<blocks, TPB, 0, (hipStream_t)hip_stream>>>(in, d_out, d_w, d_bias, B, I, O);
  return launched();
}

int cnn_logistic_fwd(const float* x, float* y, size_t n, void* hip_stream) {
  if (!x || !y || n < 1 || !aligned16(x) || !aligned16(y)) return CNN_EINVAL;
  logistic_fwd_kernel<<<grid_stream((n + 3) / 4), TPB, 0, (hipStream_t)hip_stream>>>(x, y, n);
  return launched();
}

int cnn_logistic_bwd(const float* y, const float* d_y, float* d_x, size_t n, void* hip_stream) {
  if (!y || !d_y || !d_x || n < 1 || !aligned16(y) || !aligned16(d_y) || !aligned16(d_x))
    return CNN_EINVAL;
  logistic_bwd_kernel<<<grid_stream((n + 3) / 4), TPB, 0, (hipStream_t)hip_stream>>>(y, d_y, d_x, n);
  return launched();
}

}  // extern "C"
