// Fused forward / forward+backward kernels of the whole network, the
// deterministic gradient reduction with the SGD update, and the context-based
// C entry points.  Definitions: arXiv 1912.05234, Section 3 (forward, conv,
// mconv, sigmoid, avgpool, backweights, backbias, backin, backavgpool) and
// Section 2 (batch gradient descent, w := w - eta * sum_i grad F_i).
//
// One workgroup of 256 lanes owns one image at a time.  The image, every
// activation (C1, S1, C2, S2, output) and every error array stay in LDS from
// the first load to the last gradient term; the only HBM traffic per image is
// its 3136-byte pixel block and its label.  A workgroup walks the images
// n = g, g+G, g+2G, ... and keeps its share of the 3898 gradient sums in
// registers (every gradient element has exactly one owning lane), so the
// per-workgroup partial needs no atomics and its value does not depend on
// scheduling.  A second kernel adds the G partials in a fixed order and applies
// the update.
#include <new>
#include <vector>

#include "cnn_common.h"

namespace {

using namespace cnn;

constexpr int TPB = 256;
constexpr int GCAP = 1024;  // most workgroups (= gradient partials) per step

struct __align__(16) Lds {
  float w[PSTRIDE];   // all parameters
  float img[NI];
  float c1[NC1];      // C1 output, later the error at C1's pre-activation
  float s1[NS1];
  float c2[NC2];      // C2 output, later the error at C2's pre-activation
  float s2[NS2];
  float d_s1[NS1];    // error at S1
  float d_s2[NS2];    // error at S2
  float y[16];
  float delta[16];    // error at the output pre-activation
};

__device__ __forceinline__ void load_weights(Lds& s, const float* __restrict__ w) {
  for (int p = threadIdx.x; p < PSTRIDE / 4; p += TPB)
    reinterpret_cast<float4*>(s.w)[p] = reinterpret_cast<const float4*>(w)[p];
}

// 784 floats = 196 aligned 16-byte loads, consecutive lanes -> consecutive addresses
__device__ __forceinline__ void load_image(Lds& s, const float* __restrict__ images, size_t n) {
  const float4* src = reinterpret_cast<const float4*>(images + n * NI);
  if (threadIdx.x < NI / 4) reinterpret_cast<float4*>(s.img)[threadIdx.x] = src[threadIdx.x];
}

// C1 .. output layer of listing `forward`; activations left in LDS.
__device__ __forceinline__ void forward_phases(Lds& s) {
  const int t = threadIdx.x;
  // C1 = sigmoid(mconv(I, k1, b1)): bias and sigmoid folded into the convolution's epilogue
  for (int o = t; o < NC1; o += TPB) {
    const int i = o / 576, r = o % 576, y = r / 24, x = r % 24;
    float acc = s.w[OFF_B1 + i];
    const float* ip = s.img + y * 28 + x;
    const float* kp = s.w + OFF_K1 + i * 25;
#pragma unroll
    for (int u = 0; u < 5; ++u)
#pragma unroll
      for (int v = 0; v < 5; ++v) acc = fmaf(ip[u * 28 + v], kp[u * 5 + v], acc);
    s.c1[o] = logistic(acc);
  }
  __syncthreads();
  // S1 = avgpool(C1)
  for (int o = t; o < NS1; o += TPB) {
    const int m = o / 144, r = o % 144, p = r / 12, q = r % 12;
    const float* cp = s.c1 + m * 576 + 2 * p * 24 + 2 * q;
    s.s1[o] = (cp[0] + cp[1] + cp[24] + cp[25]) * 0.25f;
  }
  __syncthreads();
  // C2 = sigmoid(mconv(S1, k2, b2)): every output map sums over all six input maps
  for (int o = t; o < NC2; o += TPB) {
    const int j = o / 64, r = o % 64, y = r / 8, x = r % 8;
    float acc = s.w[OFF_B2 + j];
    for (int c = 0; c < 6; ++c) {
      const float* ip = s.s1 + c * 144 + y * 12 + x;
      const float* kp = s.w + OFF_K2 + j * 150 + c * 25;
#pragma unroll
      for (int u = 0; u < 5; ++u)
#pragma unroll
        for (int v = 0; v < 5; ++v) acc = fmaf(ip[u * 12 + v], kp[u * 5 + v], acc);
    }
    s.c2[o] = logistic(acc);
  }
  __syncthreads();
  // S2 = avgpool(C2)
  if (t < NS2) {
    const int m = t / 16, r = t % 16, p = r / 4, q = r % 4;
    const float* cp = s.c2 + m * 64 + 2 * p * 8 + 2 * q;
    s.s2[t] = (cp[0] + cp[1] + cp[8] + cp[9]) * 0.25f;
  }
  __syncthreads();
  // output = sigmoid(mconv(S2, fc, b)): ten dot products of length 192, 16 lanes each
  {
    const int o = t >> 4, part = t & 15;
    float acc = 0.0f;
    if (o < NY) {
      const float* wp = s.w + OFF_FC + o * NS2 + part * 12;
      const float* ip = s.s2 + part * 12;
#pragma unroll
      for (int i = 0; i < 12; ++i) acc = fmaf(ip[i], wp[i], acc);
    }
    acc += __shfl_xor(acc, 8, 16);
    acc += __shfl_xor(acc, 4, 16);
    acc += __shfl_xor(acc, 2, 16);
    acc += __shfl_xor(acc, 1, 16);
    if (o < NY && part == 0) s.y[o] = logistic(acc + s.w[OFF_B + o]);
  }
  __syncthreads();
}

__device__ __forceinline__ float image_loss(const float* y, int label) {
  float l = 0.0f;
#pragma unroll
  for (int o = 0; o < NY; ++o) {
    const float e = y[o] - (o == label ? 1.0f : 0.0f);
    l = fmaf(e, e, l);
  }
  return 0.5f * l;
}

// ------------------------------------------------------------------ forward only
// Optional outputs: yhat[B,10], the four activation arrays, and (with labels) one
// (correct count, loss sum) pair per workgroup in eval_partial[G][2].
__global__ __launch_bounds__(TPB) void forward_kernel(const float* __restrict__ images,
                                                      const int32_t* __restrict__ labels, int B,
                                                      const float* __restrict__ w, float* __restrict__ yhat,
                                                      float* __restrict__ c1o, float* __restrict__ s1o,
                                                      float* __restrict__ c2o, float* __restrict__ s2o,
                                                      float* __restrict__ eval_partial) {
  __shared__ Lds s;
  const int t = threadIdx.x;
  load_weights(s, w);
  float n_ok = 0.0f, loss = 0.0f;  // lane 0 only
  for (size_t n = blockIdx.x; n < (size_t)B; n += gridDim.x) {
    load_image(s, images, n);
    __syncthreads();
    forward_phases(s);
    if (yhat && t < NY) yhat[n * NY + t] = s.y[t];
    if (c1o)
      for (int o = t; o < NC1; o += TPB) c1o[n * NC1 + o] = s.c1[o];
    if (s1o)
      for (int o = t; o < NS1; o += TPB) s1o[n * NS1 + o] = s.s1[o];
    if (c2o)
      for (int o = t; o < NC2; o += TPB) c2o[n * NC2 + o] = s.c2[o];
    if (s2o && t < NS2) s2o[n * NS2 + t] = s.s2[t];
    if (labels && t == 0) {
      const int label = labels[n];
      int best = 0;
#pragma unroll
      for (int o = 1; o < NY; ++o)
        if (s.y[o] > s.y[best]) best = o;  // strict '>' keeps the lowest index on ties
      n_ok += (best == label) ? 1.0f : 0.0f;
      loss += image_loss(s.y, label);
    }
    __syncthreads();
  }
  if (eval_partial && t == 0) {
    eval_partial[2 * blockIdx.x] = n_ok;  // exact: at most 2^24 images per workgroup
    eval_partial[2 * blockIdx.x + 1] = loss;
  }
}

// Sums the G (count, loss) pairs in index order.
__global__ void eval_reduce_kernel(const float* __restrict__ eval_partial, int G,
                                   int64_t* __restrict__ n_correct, float* __restrict__ loss_sum) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int64_t ok = 0;
    float loss = 0.0f;
    for (int g = 0; g < G; ++g) {
      ok += (int64_t)eval_partial[2 * g];
      loss += eval_partial[2 * g + 1];
    }
    if (n_correct) *n_correct = ok;
    if (loss_sum) *loss_sum = loss;
  }
}

// ------------------------------------------------------------- forward + backward
__global__ __launch_bounds__(TPB) void train_kernel(const float* __restrict__ images,
                                                    const int32_t* __restrict__ labels, int B,
                                                    const float* __restrict__ w,
                                                    float* __restrict__ partial) {
  __shared__ Lds s;
  const int t = threadIdx.x;
  load_weights(s, w);

  // Gradient sums owned by this lane (summed over this workgroup's images).
  float g_fc[8];   // fc[p], p = t + 256 r, r < 8 (p < 1920)
  float g_b = 0.0f;   // b[t], t < 10
  float g_k2[10];  // k2[j0 + a][c][u][v], a < 2, v < 5, for lanes t < 180
  float g_b2[2] = {0.0f, 0.0f};  // b2[j0 + a], lanes t < 6
  float g_k1[5];   // k1[i][u][v] over this lane's rows, lanes t < 240
  float g_b1 = 0.0f;  // b1[i] over this lane's rows, lanes with u == 0
  float loss = 0.0f;  // lane 0
#pragma unroll
  for (int r = 0; r < 8; ++r) g_fc[r] = 0.0f;
#pragma unroll
  for (int r = 0; r < 10; ++r) g_k2[r] = 0.0f;
#pragma unroll
  for (int r = 0; r < 5; ++r) g_k1[r] = 0.0f;

  // lane roles for the two weight-gradient convolutions
  const int k2_c = t / 30, k2_u = (t % 30) / 6, k2_j0 = 2 * (t % 6);  // valid for t < 180
  const int k1_i = t / 40, k1_u = (t % 40) / 8, k1_ys = t % 8;         // valid for t < 240

  for (size_t n = blockIdx.x; n < (size_t)B; n += gridDim.x) {
    load_image(s, images, n);
    const int label = labels[n];
    __syncthreads();
    forward_phases(s);

    // error at the output pre-activation: (yhat - onehot) * yhat * (1 - yhat)
    if (t < NY) {
      const float y = s.y[t];
      s.delta[t] = (y - (t == label ? 1.0f : 0.0f)) * y * (1.0f - y);
    }
    if (t == 0) loss += image_loss(s.y, label);
    __syncthreads();

    // FC layer: backweights (outer product), backbias, backin (fc^T delta)
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int p = t + TPB * r;
      if (p < 1920) g_fc[r] = fmaf(s.delta[p / NS2], s.s2[p % NS2], g_fc[r]);
    }
    if (t < NY) g_b += s.delta[t];
    if (t < NS2) {
      float acc = 0.0f;
#pragma unroll
      for (int o = 0; o < NY; ++o) acc = fmaf(s.w[OFF_FC + o * NS2 + t], s.delta[o], acc);
      s.d_s2[t] = acc;
    }
    __syncthreads();

    // backavgpool through S2, then the derivative of C2's sigmoid (in place over C2)
    for (int o = t; o < NC2; o += TPB) {
      const int j = o / 64, r = o % 64, y = r / 8, x = r % 8;
      const float c = s.c2[o];
      s.c2[o] = s.d_s2[j * 16 + (y >> 1) * 4 + (x >> 1)] * 0.25f * c * (1.0f - c);
    }
    __syncthreads();

    // C2 layer, backweights: g_k2[j,c,u,v] += sum_{y,x} s1[c,y+u,x+v] * d_c2[j,y,x]
    if (t < 180) {
      float acc[10];
#pragma unroll
      for (int r = 0; r < 10; ++r) acc[r] = 0.0f;
      float bsum0 = 0.0f, bsum1 = 0.0f;
      for (int y = 0; y < 8; ++y) {
        const float* ip = s.s1 + k2_c * 144 + (y + k2_u) * 12;
        const float* d0 = s.c2 + k2_j0 * 64 + y * 8;
        float in[12];
#pragma unroll
        for (int x = 0; x < 12; ++x) in[x] = ip[x];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const float e0 = d0[x], e1 = d0[64 + x];
          bsum0 += e0;
          bsum1 += e1;
#pragma unroll
          for (int v = 0; v < 5; ++v) {
            acc[v] = fmaf(in[x + v], e0, acc[v]);
            acc[5 + v] = fmaf(in[x + v], e1, acc[5 + v]);
          }
        }
      }
#pragma unroll
      for (int r = 0; r < 10; ++r) g_k2[r] += acc[r];
      // backbias: one lane per pair of maps (the lanes with c == 0 and u == 0)
      if (t < 6) {
        g_b2[0] += bsum0;
        g_b2[1] += bsum1;
      }
    }
    // C2 layer, backin summed over the twelve output maps:
    //   d_s1[c,p,q] = sum_j sum_{u,v : 0<=p-u<8, 0<=q-v<8} k2[j,c,u,v] * d_c2[j,p-u,q-v]
    for (int o = t; o < NS1; o += TPB) {
      const int c = o / 144, r = o % 144, p = r / 12, q = r % 12;
      const int u_lo = max(0, p - 7), u_hi = min(4, p), v_lo = max(0, q - 7), v_hi = min(4, q);
      float acc = 0.0f;
      for (int j = 0; j < 12; ++j) {
        const float* kp = s.w + OFF_K2 + j * 150 + c * 25;
        const float* dp = s.c2 + j * 64;
        for (int u = u_lo; u <= u_hi; ++u)
          for (int v = v_lo; v <= v_hi; ++v) acc = fmaf(kp[u * 5 + v], dp[(p - u) * 8 + (q - v)], acc);
      }
      s.d_s1[o] = acc;
    }
    __syncthreads();

    // backavgpool through S1, then the derivative of C1's sigmoid (in place over C1)
    for (int o = t; o < NC1; o += TPB) {
      const int i = o / 576, r = o % 576, y = r / 24, x = r % 24;
      const float c = s.c1[o];
      s.c1[o] = s.d_s1[i * 144 + (y >> 1) * 12 + (x >> 1)] * 0.25f * c * (1.0f - c);
    }
    __syncthreads();

    // C1 layer, backweights and backbias (its input error is not needed):
    //   g_k1[i,u,v] += sum_{y,x} I[y+u,x+v] * d_c1[i,y,x]; lane (i,u,ys) takes rows ys, ys+8, ys+16
    if (t < 240) {
      float acc[5] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
      float bsum = 0.0f;
      for (int y = k1_ys; y < 24; y += 8) {
        const float* ip = s.img + (y + k1_u) * 28;
        const float* dp = s.c1 + k1_i * 576 + y * 24;
        float win[5];
#pragma unroll
        for (int v = 0; v < 4; ++v) win[v + 1] = ip[v];
        for (int x = 0; x < 24; ++x) {
#pragma unroll
          for (int v = 0; v < 4; ++v) win[v] = win[v + 1];
          win[4] = ip[x + 4];
          const float e = dp[x];
          bsum += e;
#pragma unroll
          for (int v = 0; v < 5; ++v) acc[v] = fmaf(win[v], e, acc[v]);
        }
      }
#pragma unroll
      for (int v = 0; v < 5; ++v) g_k1[v] += acc[v];
      if (k1_u == 0) g_b1 += bsum;
    }
    __syncthreads();  // LDS is reused by the next image
  }

  // ---- write this workgroup's partial: every slot has exactly one writer ----
  float* out = partial + (size_t)blockIdx.x * PSTRIDE;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int p = t + TPB * r;
    if (p < 1920) out[OFF_FC + p] = g_fc[r];
  }
  if (t < NY) out[OFF_B + t] = g_b;
  if (t < 180) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int v = 0; v < 5; ++v) out[OFF_K2 + (k2_j0 + a) * 150 + k2_c * 25 + k2_u * 5 + v] = g_k2[a * 5 + v];
  }
  if (t < 6) {
    out[OFF_B2 + k2_j0] = g_b2[0];
    out[OFF_B2 + k2_j0 + 1] = g_b2[1];
  }
  // the eight row-slices (ys = lane & 7) of a C1 weight are added in a fixed butterfly order
#pragma unroll
  for (int v = 0; v < 5; ++v) {
    float a = g_k1[v];
    a += __shfl_xor(a, 4, 8);
    a += __shfl_xor(a, 2, 8);
    a += __shfl_xor(a, 1, 8);
    if (t < 240 && k1_ys == 0) out[OFF_K1 + k1_i * 25 + k1_u * 5 + v] = a;
  }
  {
    float a = g_b1;
    a += __shfl_xor(a, 4, 8);
    a += __shfl_xor(a, 2, 8);
    a += __shfl_xor(a, 1, 8);
    if (t < 240 && k1_ys == 0 && k1_u == 0) out[OFF_B1 + k1_i] = a;
  }
  if (t == 0) out[LOSS_SLOT] = loss;
}

// Adds the G partial rows in a fixed order (four interleaved strands, then a
// fixed tree over the strands) and either applies  w <- w - scale * g  (grad_out
// == nullptr) or stores g.  One workgroup per 64 parameters; lanes of a wave
// read 64 consecutive floats of a row.
__global__ __launch_bounds__(TPB) void reduce_update_kernel(const float* __restrict__ partial, int G,
                                                            float scale, float* __restrict__ w,
                                                            float* __restrict__ grad_out,
                                                            float* __restrict__ loss_sum) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, strand = threadIdx.x >> 6;
  const int p = blockIdx.x * 64 + lane;
  float acc = 0.0f;
  for (int g = strand; g < G; g += 4) acc += partial[(size_t)g * PSTRIDE + p];
  red[strand][lane] = acc;
  __syncthreads();
  if (strand == 0) {
    const float total = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
    if (p < NPARAM) {
      if (grad_out)
        grad_out[p] = total;
      else
        w[p] = fmaf(-scale, total, w[p]);
    } else if (p == LOSS_SLOT && loss_sum) {
      *loss_sum = total;
    }
  }
}

}  // namespace

// ------------------------------------------------------------------- C ABI
struct cnn_ctx {
  hipStream_t stream;
  int max_batch;
  int gcap;
  float* w;             // [PSTRIDE]
  float* partial;       // [gcap][PSTRIDE]
  float* eval_partial;  // [gcap][2]
  std::vector<hipEvent_t> ev;  // 2 per recorded step (before, after the fused kernel)
  int ev_used = 0;             // recorded steps
};

namespace {

constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int gcap_for(int max_batch) { return max_batch < GCAP ? max_batch : GCAP; }

struct Layout {
  size_t w, partial, eval_partial, total;
};

inline Layout layout_for(int max_batch) {
  Layout l;
  const size_t g = (size_t)gcap_for(max_batch);
  l.w = 0;
  l.partial = align_up(l.w + sizeof(float) * PSTRIDE, 256);
  l.eval_partial = align_up(l.partial + sizeof(float) * PSTRIDE * g, 256);
  l.total = align_up(l.eval_partial + sizeof(float) * 2 * g, 256);
  return l;
}

const int kParamOff[6] = {OFF_K1, OFF_B1, OFF_K2, OFF_B2, OFF_FC, OFF_B};
const int kParamLen[6] = {150, 6, 1800, 12, 1920, 10};

inline bool batch_ok(const cnn_ctx* ctx, int B) { return ctx && B >= 1 && B <= ctx->max_batch; }

inline int grid_for(const cnn_ctx* ctx, int B) { return B < ctx->gcap ? B : ctx->gcap; }

int run_forward(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float* yhat, float* c1,
                float* s1, float* c2, float* s2, bool eval) {
  const int G = grid_for(ctx, B);
  forward_kernel<<<G, TPB, 0, ctx->stream>>>(images, labels, B, ctx->w, yhat, c1, s1, c2, s2,
                                             eval ? ctx->eval_partial : nullptr);
  if (hipGetLastError() != hipSuccess) return CNN_EHIP;
  return G;
}

int run_backward(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float scale,
                 float* grad_out, float* loss_sum) {
  const int G = grid_for(ctx, B);
  const bool timed = (size_t)(2 * ctx->ev_used + 1) < ctx->ev.size();
  if (timed) CNN_HIP_TRY(hipEventRecord(ctx->ev[2 * ctx->ev_used], ctx->stream));
  train_kernel<<<G, TPB, 0, ctx->stream>>>(images, labels, B, ctx->w, ctx->partial);
  if (hipGetLastError() != hipSuccess) return CNN_EHIP;
  if (timed) {
    CNN_HIP_TRY(hipEventRecord(ctx->ev[2 * ctx->ev_used + 1], ctx->stream));
    ++ctx->ev_used;
  }
  reduce_update_kernel<<<PSTRIDE / 64, TPB, 0, ctx->stream>>>(ctx->partial, G, scale, ctx->w, grad_out,
                                                              loss_sum);
  if (hipGetLastError() != hipSuccess) return CNN_EHIP;
  return CNN_OK;
}

}  // namespace

extern "C" {

const char* cnn_strerror(int code) {
  switch (code) {
    case CNN_OK: return "ok";
    case CNN_EINVAL: return "invalid argument (null or misaligned pointer, size out of range)";
    case CNN_EWORKSPACE: return "workspace too small";
    case CNN_EHIP: return "HIP runtime call or kernel launch failed";
    default: return "unknown error code";
  }
}

size_t cnn_workspace_bytes(int max_batch) { return max_batch < 1 ? 0 : layout_for(max_batch).total; }

int cnn_set_weights(cnn_ctx* ctx, const float* k1, const float* b1, const float* k2, const float* b2,
                    const float* fc, const float* b) {
  if (!ctx) return CNN_EINVAL;
  const float* src[6] = {k1, b1, k2, b2, fc, b};
  for (int a = 0; a < 6; ++a)
    if (src[a])
      CNN_HIP_TRY(hipMemcpyAsync(ctx->w + kParamOff[a], src[a], sizeof(float) * kParamLen[a],
                                 hipMemcpyDeviceToDevice, ctx->stream));
  return CNN_OK;
}

int cnn_get_weights(cnn_ctx* ctx, float* k1, float* b1, float* k2, float* b2, float* fc, float* b) {
  if (!ctx) return CNN_EINVAL;
  float* dst[6] = {k1, b1, k2, b2, fc, b};
  for (int a = 0; a < 6; ++a)
    if (dst[a])
      CNN_HIP_TRY(hipMemcpyAsync(dst[a], ctx->w + kParamOff[a], sizeof(float) * kParamLen[a],
                                 hipMemcpyDeviceToDevice, ctx->stream));
  return CNN_OK;
}

int cnn_init(cnn_ctx** out, void* workspace, size_t workspace_bytes, int max_batch, const float* k1,
             const float* b1, const float* k2, const float* b2, const float* fc, const float* b,
             void* hip_stream) {
  if (!out) return CNN_EINVAL;
  *out = nullptr;
  if (!workspace || max_batch < 1 || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return CNN_EINVAL;
  const Layout l = layout_for(max_batch);
  if (workspace_bytes < l.total) return CNN_EWORKSPACE;
  cnn_ctx* ctx = new (std::nothrow) cnn_ctx;
  if (!ctx) return CNN_EINVAL;
  char* base = static_cast<char*>(workspace);
  ctx->stream = (hipStream_t)hip_stream;
  ctx->max_batch = max_batch;
  ctx->gcap = gcap_for(max_batch);
  ctx->w = reinterpret_cast<float*>(base + l.w);
  ctx->partial = reinterpret_cast<float*>(base + l.partial);
  ctx->eval_partial = reinterpret_cast<float*>(base + l.eval_partial);
  if (hipMemsetAsync(ctx->w, 0, sizeof(float) * PSTRIDE, ctx->stream) != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return CNN_EHIP;
  }
  const int rc = cnn_set_weights(ctx, k1, b1, k2, b2, fc, b);
  if (rc != CNN_OK) {
    delete ctx;
    return rc;
  }
  *out = ctx;
  return CNN_OK;
}

int cnn_profile_begin(cnn_ctx* ctx, int capacity) {
  if (!ctx || capacity < 0 || capacity > (1 << 20)) return CNN_EINVAL;
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  ctx->ev.clear();
  ctx->ev_used = 0;
  for (int i = 0; i < 2 * capacity; ++i) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) {
      (void)hipGetLastError();
      for (hipEvent_t d : ctx->ev) (void)hipEventDestroy(d);
      ctx->ev.clear();
      return CNN_EHIP;
    }
    ctx->ev.push_back(e);
  }
  return CNN_OK;
}

int cnn_profile_read(cnn_ctx* ctx, float* ms, int capacity, int* n_recorded) {
  if (!ctx || !ms || !n_recorded || capacity < 0) return CNN_EINVAL;
  CNN_HIP_TRY(hipStreamSynchronize(ctx->stream));
  const int n = ctx->ev_used < capacity ? ctx->ev_used : capacity;
  for (int i = 0; i < n; ++i) CNN_HIP_TRY(hipEventElapsedTime(&ms[i], ctx->ev[2 * i], ctx->ev[2 * i + 1]));
  *n_recorded = n;
  ctx->ev_used = 0;
  return CNN_OK;
}

void cnn_destroy(cnn_ctx* ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  delete ctx;
}

int cnn_forward(cnn_ctx* ctx, const float* images, int B, float* yhat) {
  if (!batch_ok(ctx, B) || !images || !yhat || !aligned16(images) || !aligned16(yhat)) return CNN_EINVAL;
  const int rc = run_forward(ctx, images, nullptr, B, yhat, nullptr, nullptr, nullptr, nullptr, false);
  return rc < 0 ? rc : CNN_OK;
}

int cnn_forward_activations(cnn_ctx* ctx, const float* images, int B, float* c1, float* s1, float* c2,
                            float* s2, float* yhat) {
  if (!batch_ok(ctx, B) || !images || !aligned16(images)) return CNN_EINVAL;
  const float* outs[5] = {c1, s1, c2, s2, yhat};
  for (const float* p : outs)
    if (p && !aligned16(p)) return CNN_EINVAL;
  const int rc = run_forward(ctx, images, nullptr, B, yhat, c1, s1, c2, s2, false);
  return rc < 0 ? rc : CNN_OK;
}

int cnn_evaluate(cnn_ctx* ctx, const float* images, const int32_t* labels, int N, int64_t* n_correct,
                 float* loss_sum) {
  if (!batch_ok(ctx, N) || !images || !labels || !n_correct || !aligned16(images)) return CNN_EINVAL;
  const int G = run_forward(ctx, images, labels, N, nullptr, nullptr, nullptr, nullptr, nullptr, true);
  if (G < 0) return G;
  eval_reduce_kernel<<<1, 64, 0, ctx->stream>>>(ctx->eval_partial, G, n_correct, loss_sum);
  return hipGetLastError() == hipSuccess ? CNN_OK : CNN_EHIP;
}

int cnn_gradient(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float* grad,
                 float* loss_sum) {
  if (!batch_ok(ctx, B) || !images || !labels || !grad || !aligned16(images) || !aligned16(grad))
    return CNN_EINVAL;
  return run_backward(ctx, images, labels, B, 0.0f, grad, loss_sum);
}

int cnn_train_batch(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float lr,
                    float* loss_sum) {
  if (!batch_ok(ctx, B) || !images || !labels || !aligned16(images)) return CNN_EINVAL;
  return run_backward(ctx, images, labels, B, lr / (float)B, nullptr, loss_sum);
}

}  // extern "C"
