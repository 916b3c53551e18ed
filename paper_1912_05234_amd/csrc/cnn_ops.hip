// Stateless per-operation kernels (general shapes) and their C entry points.
// Definitions: arXiv 1912.05234, Section 3 -- listings conv, mconv, sigmoid,
// avgpool, backweights, backbias, backin, backavgpool.  These are the plain,
// one-thread-per-output forms; the fused training step lives in cnn_fused.hip.
#include "cnn_common.h"

namespace {

using namespace cnn;

constexpr int TPB = 256;

inline unsigned grid_for(size_t n) {
  size_t g = (n + TPB - 1) / TPB;
  const size_t cap = 256 * 32;  // grid-stride beyond this
  return (unsigned)(g < cap ? (g ? g : 1) : cap);
}

// out[b,co,y,x] = bias[co] + sum_{ci,u,v} in[b,ci,y+u,x+v] * k[co,ci,u,v]
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
        for (int v = 0; v < KW; ++v) acc = fmaf(ip[u * W + v], kp[u * KW + v], acc);
    }
    out[o] = acc;
  }
}

// d_in[b,ci,p,q] = sum_co sum_{u,v valid} k[co,ci,u,v] * d_out[b,co,p-u,q-v]
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
          acc = fmaf(kp[u * KW + v], dp[(p - u) * Wo + (q - v)], acc);
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
      acc = fmaf(in[((b * Cin + ci) * H + y + u) * (size_t)W + x + v],
                 d_out[((b * Cout + co) * Ho + y) * (size_t)Wo + x], acc);
    }
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) d_k[id] = acc;
  } else {
    const int co = id - nk;
    for (size_t e = threadIdx.x; e < dom; e += TPB) {
      const size_t b = e / ((size_t)Wo * Ho), r = e % ((size_t)Wo * Ho);
      acc += d_out[(b * Cout + co) * (size_t)Ho * Wo + r];
    }
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) d_bias[co] = acc;
  }
}

__global__ __launch_bounds__(TPB) void avgpool_fwd_kernel(const float* __restrict__ in,
                                                          float* __restrict__ out, size_t total, int H,
                                                          int W) {
  const int Ho = H / 2, Wo = W / 2;
  for (size_t o = blockIdx.x * (size_t)TPB + threadIdx.x; o < total; o += (size_t)gridDim.x * TPB) {
    const int q = (int)(o % Wo), p = (int)((o / Wo) % Ho);
    const size_t m = o / ((size_t)Wo * Ho);
    const float* ip = in + (m * H + 2 * p) * (size_t)W + 2 * q;
    out[o] = (ip[0] + ip[1] + ip[W] + ip[W + 1]) * 0.25f;
  }
}

__global__ __launch_bounds__(TPB) void avgpool_bwd_kernel(const float* __restrict__ d_out,
                                                          float* __restrict__ d_in, size_t total, int Ho,
                                                          int Wo) {
  const int H = 2 * Ho, W = 2 * Wo;
  for (size_t o = blockIdx.x * (size_t)TPB + threadIdx.x; o < total; o += (size_t)gridDim.x * TPB) {
    const int x = (int)(o % W), y = (int)((o / W) % H);
    const size_t m = o / ((size_t)W * H);
    d_in[o] = d_out[(m * Ho + y / 2) * (size_t)Wo + x / 2] * 0.25f;
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

__global__ __launch_bounds__(TPB) void logistic_fwd_kernel(const float* __restrict__ x,
                                                           float* __restrict__ y, size_t n) {
  for (size_t e = blockIdx.x * (size_t)TPB + threadIdx.x; e < n; e += (size_t)gridDim.x * TPB)
    y[e] = logistic(x[e]);
}

__global__ __launch_bounds__(TPB) void logistic_bwd_kernel(const float* __restrict__ y,
                                                           const float* __restrict__ d_y,
                                                           float* __restrict__ d_x, size_t n) {
  for (size_t e = blockIdx.x * (size_t)TPB + threadIdx.x; e < n; e += (size_t)gridDim.x * TPB) {
    const float v = y[e];
    d_x[e] = d_y[e] * v * (1.0f - v);
  }
}

inline int launched() { return hipGetLastError() == hipSuccess ? CNN_OK : CNN_EHIP; }

inline bool conv_args_ok(int B, int Cin, int H, int W, int Cout, int KH, int KW) {
  return B >= 1 && Cin >= 1 && Cout >= 1 && KH >= 1 && KW >= 1 && H >= KH && W >= KW &&
         (size_t)Cout * Cin * KH * KW + (size_t)Cout < (size_t)1 << 30;
}

}  // namespace

extern "C" {

int cnn_conv_fwd(const float* in, const float* k, const float* bias, float* out, int B, int Cin, int H,
                 int W, int Cout, int KH, int KW, void* hip_stream) {
  if (!in || !k || !out || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(k) || !aligned16(out) || (bias && !aligned16(bias))) return CNN_EINVAL;
  const size_t total = (size_t)B * Cout * (H - KH + 1) * (W - KW + 1);
  conv_fwd_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(in, k, bias, out, total, Cin, H,
                                                                         W, Cout, KH, KW);
  return launched();
}

int cnn_conv_bwd_input(const float* d_out, const float* k, float* d_in, int B, int Cin, int H, int W,
                       int Cout, int KH, int KW, void* hip_stream) {
  if (!d_out || !k || !d_in || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(k) || !aligned16(d_in)) return CNN_EINVAL;
  const size_t total = (size_t)B * Cin * H * W;
  conv_bwd_input_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, k, d_in, total, Cin,
                                                                               H, W, Cout, KH, KW);
  return launched();
}

int cnn_conv_bwd_weight(const float* in, const float* d_out, float* d_k, float* d_bias, int B, int Cin,
                        int H, int W, int Cout, int KH, int KW, void* hip_stream) {
  if (!in || !d_out || !d_k || !conv_args_ok(B, Cin, H, W, Cout, KH, KW)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(d_out) || !aligned16(d_k) || (d_bias && !aligned16(d_bias)))
    return CNN_EINVAL;
  const unsigned blocks = (unsigned)(Cout * Cin * KH * KW + (d_bias ? Cout : 0));
  conv_bwd_weight_kernel<<<blocks, TPB, 0, (hipStream_t)hip_stream>>>(in, d_out, d_k, d_bias, B, Cin, H,
                                                                      W, Cout, KH, KW);
  return launched();
}

int cnn_avgpool_fwd(const float* in, float* out, int B, int C, int H, int W, void* hip_stream) {
  if (!in || !out || B < 1 || C < 1 || H < 2 || W < 2 || (H & 1) || (W & 1)) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(out)) return CNN_EINVAL;
  const size_t total = (size_t)B * C * (H / 2) * (W / 2);
  avgpool_fwd_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(in, out, total, H, W);
  return launched();
}

int cnn_avgpool_bwd(const float* d_out, float* d_in, int B, int C, int Ho, int Wo, void* hip_stream) {
  if (!d_out || !d_in || B < 1 || C < 1 || Ho < 1 || Wo < 1) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(d_in)) return CNN_EINVAL;
  const size_t total = (size_t)B * C * Ho * Wo * 4;
  avgpool_bwd_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, d_in, total, Ho, Wo);
  return launched();
}

int cnn_fc_fwd(const float* in, const float* w, const float* bias, float* out, int B, int I, int O,
               void* hip_stream) {
  if (!in || !w || !out || B < 1 || I < 1 || O < 1) return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(w) || !aligned16(out) || (bias && !aligned16(bias))) return CNN_EINVAL;
  const size_t total = (size_t)B * O;
  fc_fwd_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(in, w, bias, out, total, I, O);
  return launched();
}

int cnn_fc_bwd_input(const float* d_out, const float* w, float* d_in, int B, int I, int O,
                     void* hip_stream) {
  if (!d_out || !w || !d_in || B < 1 || I < 1 || O < 1) return CNN_EINVAL;
  if (!aligned16(d_out) || !aligned16(w) || !aligned16(d_in)) return CNN_EINVAL;
  const size_t total = (size_t)B * I;
  fc_bwd_input_kernel<<<grid_for(total), TPB, 0, (hipStream_t)hip_stream>>>(d_out, w, d_in, total, I, O);
  return launched();
}

int cnn_fc_bwd_weight(const float* in, const float* d_out, float* d_w, float* d_bias, int B, int I, int O,
                      void* hip_stream) {
  if (!in || !d_out || !d_w || B < 1 || I < 1 || O < 1 || (size_t)I * O + O >= (size_t)1 << 30)
    return CNN_EINVAL;
  if (!aligned16(in) || !aligned16(d_out) || !aligned16(d_w) || (d_bias && !aligned16(d_bias)))
    return CNN_EINVAL;
  const unsigned blocks = (unsigned)(O * I + (d_bias ? O : 0));
  fc_bwd_weight_kernel<<<blocks, TPB, 0, (hipStream_t)hip_stream>>>(in, d_out, d_w, d_bias, B, I, O);
  return launched();
}

int cnn_logistic_fwd(const float* x, float* y, size_t n, void* hip_stream) {
  if (!x || !y || n < 1 || !aligned16(x) || !aligned16(y)) return CNN_EINVAL;
  logistic_fwd_kernel<<<grid_for(n), TPB, 0, (hipStream_t)hip_stream>>>(x, y, n);
  return launched();
}

int cnn_logistic_bwd(const float* y, const float* d_y, float* d_x, size_t n, void* hip_stream) {
  if (!y || !d_y || !d_x || n < 1 || !aligned16(y) || !aligned16(d_y) || !aligned16(d_x))
    return CNN_EINVAL;
  logistic_bwd_kernel<<<grid_for(n), TPB, 0, (hipStream_t)hip_stream>>>(y, d_y, d_x, n);
  return launched();
}

}  // extern "C"
