// CPU oracle for the CNN of "Array Languages Make Neural Networks Fast"
// (arXiv 1912.05234), Section 3 (CNN).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
// definition the GPU library is checked against.  It shares no code with the
// GPU library and must never be reached from it: only the tests, the smoke
// check and the benchmark's CPU-baseline leg may load it.
//
// Every function is the paper's definition written out as nested scalar
// loops, with no blocking, fusion or reordering.  Two instances are built
// from the one template:
//   *_f32: storage float (the paper's `float`), every sum and every sigmoid
//          evaluated in double and rounded once to float;
//   *_f64: storage and arithmetic double (for finite-difference checks).
//
// Arrays are row-major.  "Rank-polymorphic" functions of the paper are
// written for rank 4; lower ranks are reached by padding the shape with
// leading unit axes, which leaves the memory image unchanged (Section 3,
// Convolution: the remark that a reshape that removes a unit axis does not
// alter the representation).
//
// Pins (tests/test_oracle_*.py): brute force on tiny inputs, closed forms,
// adjoint identities, a second formulation of backin, invariants, central
// finite differences of the whole loss, and a float64 autograd cross-check.
// Nothing here is "parity unpinned".

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

constexpr int R = 4;  // working rank

struct Shape {
  int d[R];
  long size() const { return (long)d[0] * d[1] * d[2] * d[3]; }
  long at(int a, int b, int c, int e) const {
    return (((long)a * d[1] + b) * d[2] + c) * d[3] + e;
  }
};

// ---------------------------------------------------------------------------
// Section 3, paragraph "Convolution", listing `conv`:
//   out[iv] = sum over ov < shape(k) of I[iv+ov] * k[ov],
//   shape(out) = shape(I) - shape(k) + 1.
// No kernel flip (a cross-correlation), valid region only.
template <class T, class A>
void conv(const T* I, Shape si, const T* k, Shape sk, T* out) {
  Shape so;
  for (int a = 0; a < R; ++a) so.d[a] = si.d[a] - sk.d[a] + 1;
  for (int i0 = 0; i0 < so.d[0]; ++i0)
    for (int i1 = 0; i1 < so.d[1]; ++i1)
      for (int i2 = 0; i2 < so.d[2]; ++i2)
        for (int i3 = 0; i3 < so.d[3]; ++i3) {
          A acc = 0;
          for (int o0 = 0; o0 < sk.d[0]; ++o0)
            for (int o1 = 0; o1 < sk.d[1]; ++o1)
              for (int o2 = 0; o2 < sk.d[2]; ++o2)
                for (int o3 = 0; o3 < sk.d[3]; ++o3)
                  acc += (A)I[si.at(i0 + o0, i1 + o1, i2 + o2, i3 + o3)] *
                         (A)k[sk.at(o0, o1, o2, o3)];
          out[so.at(i0, i1, i2, i3)] = (T)acc;
        }
}

// Section 3, "Convolution", listing `mconv`:
//   out[i] = conv(I, k[i]) + b[i]  for i < shape(b).
// The bias is added to the rounded result of conv, as the listing composes
// the two functions.
template <class T, class A>
void mconv(const T* I, Shape si, const T* k, int n, Shape sk, const T* b, T* out) {
  Shape so;
  for (int a = 0; a < R; ++a) so.d[a] = si.d[a] - sk.d[a] + 1;
  const long ksz = sk.size(), osz = so.size();
  for (int i = 0; i < n; ++i) {
    conv<T, A>(I, si, k + i * ksz, sk, out + i * osz);
    for (long e = 0; e < osz; ++e) out[i * osz + e] = (T)((A)out[i * osz + e] + (A)b[i]);
  }
}

// Section 3, "Convolution", listing `sigmoid`: 1 / (1 + exp(-x)) elementwise.
template <class T, class A>
void sigmoid(const T* in, long n, T* out) {
  for (long e = 0; e < n; ++e) out[e] = (T)((A)1 / ((A)1 + std::exp(-(A)in[e])));
}

// Derived (the paper does not print it): the derivative of the logistic
// function expressed through its output y, d_in = d_out * y * (1 - y).
template <class T, class A>
void sigmoid_back(const T* y, const T* d_out, long n, T* d_in) {
  for (long e = 0; e < n; ++e) d_in[e] = (T)((A)d_out[e] * (A)y[e] * ((A)1 - (A)y[e]));
}

// Section 3, "Average Pooling", listing `avgpool` (2-d) and its generic
// wrapper over all leading axes: out[iv] = average(in[2*iv + ov], ov < [2,2]),
// shape(out) = shape(in) / 2.
template <class T, class A>
void avgpool(const T* in, long lead, int H, int W, T* out) {
  const int Ho = H / 2, Wo = W / 2;
  for (long m = 0; m < lead; ++m)
    for (int p = 0; p < Ho; ++p)
      for (int q = 0; q < Wo; ++q) {
        A acc = 0;
        for (int a = 0; a < 2; ++a)
          for (int b = 0; b < 2; ++b) acc += (A)in[(m * H + 2 * p + a) * W + 2 * q + b];
        out[(m * Ho + p) * Wo + q] = (T)(acc / (A)4);
      }
}

// Section 3, "Backpropagating Average Pooling", listing `backavgpool`:
//   out[iv] = d_out[iv / 2] / 4,  shape(out) = 2 * shape(d_out).
template <class T, class A>
void backavgpool(const T* d_out, long lead, int Ho, int Wo, T* d_in) {
  const int H = 2 * Ho, W = 2 * Wo;
  for (long m = 0; m < lead; ++m)
    for (int y = 0; y < H; ++y)
      for (int x = 0; x < W; ++x)
        d_in[(m * H + y) * W + x] = (T)((A)d_out[(m * Ho + y / 2) * Wo + x / 2] / (A)4);
}

// Section 3, "Backpropagating Convolution", listing `backweights`:
//   backweights(d_out, in) = conv(in, d_out).
template <class T, class A>
void backweights(const T* d_out, Shape sd, const T* in, Shape si, T* out) {
  conv<T, A>(in, si, d_out, sd, out);
}

// Section 3, "Backpropagating Convolution", listing `backbias`: sum(d_out).
template <class T, class A>
T backbias(const T* d_out, long n) {
  A acc = 0;
  for (long e = 0; e < n; ++e) acc += (A)d_out[e];
  return (T)acc;
}

// Section 3, "Backpropagating Convolution", `backin`: the error with respect
// to the input of conv.  The text defines it as the sum of k[ov]*d_out[iv-ov]
// over exactly those ov for which iv-ov lies inside d_out (inner elements see
// every weight, boundary elements fewer).  That sentence is implemented here;
// the printed index arithmetic is not transcribed because its bounds leave
// d_out when shape(d_out) < shape(k) - 1 on an axis, which happens on the
// channel axis of C2 and in FC.
template <class T, class A>
void backin(const T* d_out, Shape sd, const T* k, Shape sk, Shape si, T* d_in) {
  // per axis, the weights ov with 0 <= iv-ov < shape(d_out): lo(iv) <= ov <= hi(iv)
  auto lo = [&](int axis, int iv) { int v = iv - sd.d[axis] + 1; return v > 0 ? v : 0; };
  auto hi = [&](int axis, int iv) { return iv < sk.d[axis] - 1 ? iv : sk.d[axis] - 1; };
  for (int i0 = 0; i0 < si.d[0]; ++i0)
    for (int i1 = 0; i1 < si.d[1]; ++i1)
      for (int i2 = 0; i2 < si.d[2]; ++i2)
        for (int i3 = 0; i3 < si.d[3]; ++i3) {
          A acc = 0;
          for (int o0 = lo(0, i0); o0 <= hi(0, i0); ++o0)
            for (int o1 = lo(1, i1); o1 <= hi(1, i1); ++o1)
              for (int o2 = lo(2, i2); o2 <= hi(2, i2); ++o2)
                for (int o3 = lo(3, i3); o3 <= hi(3, i3); ++o3)
                  acc += (A)k[sk.at(o0, o1, o2, o3)] *
                         (A)d_out[sd.at(i0 - o0, i1 - o1, i2 - o2, i3 - o3)];
          d_in[si.at(i0, i1, i2, i3)] = (T)acc;
        }
}

// ---------------------------------------------------------------------------
// The network.  Parameter shapes as in the listing `forward` (Section 3):
//   k1[6,5,5] b1[6] k2[12,6,5,5] b2[12] fc[10,12,1,4,4] b[10].
constexpr int NK1 = 150, NB1 = 6, NK2 = 1800, NB2 = 12, NFC = 1920, NB = 10;
constexpr int NPARAM = NK1 + NB1 + NK2 + NB2 + NFC + NB;  // 3898
constexpr int OFF_K1 = 0, OFF_B1 = OFF_K1 + NK1, OFF_K2 = OFF_B1 + NB1, OFF_B2 = OFF_K2 + NK2,
              OFF_FC = OFF_B2 + NB2, OFF_B = OFF_FC + NFC;
constexpr int NI = 784, NC1 = 3456, NS1 = 864, NC2 = 768, NS2 = 192, NY = 10;

template <class T>
struct Acts {
  T c1[NC1], s1[NS1], c2[NC2], s2[NS2], y[NY];
};

const Shape S_I = {{1, 1, 28, 28}}, S_K1 = {{1, 1, 5, 5}}, S_C1MAP = {{1, 1, 24, 24}};
const Shape S_S1 = {{1, 6, 12, 12}}, S_K2 = {{1, 6, 5, 5}}, S_C2MAP = {{1, 1, 8, 8}};
const Shape S_S2 = {{1, 12, 4, 4}}, S_FC = {{1, 12, 4, 4}}, S_ONE = {{1, 1, 1, 1}};

// Section 3, listing `forward`.
template <class T, class A>
void forward(const T* I, const T* w, Acts<T>& a) {
  std::vector<T> pre(NC1);
  mconv<T, A>(I, S_I, w + OFF_K1, 6, S_K1, w + OFF_B1, pre.data());
  sigmoid<T, A>(pre.data(), NC1, a.c1);
  avgpool<T, A>(a.c1, 6, 24, 24, a.s1);
  mconv<T, A>(a.s1, S_S1, w + OFF_K2, 12, S_K2, w + OFF_B2, pre.data());
  sigmoid<T, A>(pre.data(), NC2, a.c2);
  avgpool<T, A>(a.c2, 12, 8, 8, a.s2);
  mconv<T, A>(a.s2, S_S2, w + OFF_FC, 10, S_FC, w + OFF_B, pre.data());
  sigmoid<T, A>(pre.data(), NY, a.y);
}

// Loss of one image, Section 3 "Backpropagating Convolution":
//   L = 1/2 * sum_o (y_o - f_o)^2 with y the one-hot target of the label.
template <class T, class A>
A loss_of(const T* yhat, int label) {
  A acc = 0;
  for (int o = 0; o < NY; ++o) {
    const A t = (o == label) ? (A)1 : (A)0;
    const A e = (A)yhat[o] - t;
    acc += e * e;
  }
  return acc / (A)2;
}

// Gradient of that loss for one image, assembled from the paper's building
// blocks by the chain rule (the paper defers the driver to its repository):
// output error -> FC -> backavgpool -> sigmoid' -> C2 -> backavgpool ->
// sigmoid' -> C1.  Through mconv, backweights/backbias apply per output map
// and backin is summed over the output maps.  Adds into g[NPARAM] (type A).
template <class T, class A>
A grad_image(const T* I, int label, const T* w, A* g, Acts<T>& a) {
  forward<T, A>(I, w, a);
  // derivative of the loss through the output sigmoid
  T e[NY], d_fc[NY];
  for (int o = 0; o < NY; ++o) e[o] = (T)((A)a.y[o] - ((o == label) ? (A)1 : (A)0));
  sigmoid_back<T, A>(a.y, e, NY, d_fc);

  // FC layer
  std::vector<T> tmp(NFC > NK2 ? NFC : NK2), d_s2(NS2), part(NC1);
  std::vector<A> acc(NC1);
  std::fill(acc.begin(), acc.begin() + NS2, (A)0);
  for (int o = 0; o < NY; ++o) {
    backweights<T, A>(d_fc + o, S_ONE, a.s2, S_S2, tmp.data());
    for (int e2 = 0; e2 < NS2; ++e2) g[OFF_FC + o * NS2 + e2] += (A)tmp[e2];
    g[OFF_B + o] += (A)backbias<T, A>(d_fc + o, 1);
    backin<T, A>(d_fc + o, S_ONE, w + OFF_FC + o * NS2, S_FC, S_S2, part.data());
    for (int e2 = 0; e2 < NS2; ++e2) acc[e2] += (A)part[e2];
  }
  for (int e2 = 0; e2 < NS2; ++e2) d_s2[e2] = (T)acc[e2];

  // S2 and the sigmoid of C2
  std::vector<T> up(NC1), d_c2(NC2), d_s1(NS1), d_c1(NC1);
  backavgpool<T, A>(d_s2.data(), 12, 4, 4, up.data());
  sigmoid_back<T, A>(a.c2, up.data(), NC2, d_c2.data());

  // C2 layer
  std::fill(acc.begin(), acc.begin() + NS1, (A)0);
  for (int j = 0; j < 12; ++j) {
    backweights<T, A>(d_c2.data() + j * 64, S_C2MAP, a.s1, S_S1, tmp.data());
    for (int e2 = 0; e2 < 150; ++e2) g[OFF_K2 + j * 150 + e2] += (A)tmp[e2];
    g[OFF_B2 + j] += (A)backbias<T, A>(d_c2.data() + j * 64, 64);
    backin<T, A>(d_c2.data() + j * 64, S_C2MAP, w + OFF_K2 + j * 150, S_K2, S_S1, part.data());
    for (int e2 = 0; e2 < NS1; ++e2) acc[e2] += (A)part[e2];
  }
  for (int e2 = 0; e2 < NS1; ++e2) d_s1[e2] = (T)acc[e2];

  // S1 and the sigmoid of C1
  backavgpool<T, A>(d_s1.data(), 6, 12, 12, up.data());
  sigmoid_back<T, A>(a.c1, up.data(), NC1, d_c1.data());

  // C1 layer (its input error is not needed: nothing precedes it)
  for (int i = 0; i < 6; ++i) {
    backweights<T, A>(d_c1.data() + i * 576, S_C1MAP, I, S_I, tmp.data());
    for (int e2 = 0; e2 < 25; ++e2) g[OFF_K1 + i * 25 + e2] += (A)tmp[e2];
    g[OFF_B1 + i] += (A)backbias<T, A>(d_c1.data() + i * 576, 576);
  }
  return loss_of<T, A>(a.y, label);
}

// One training step on a batch: gradients of every image with the weights as
// they were before the step, summed over the batch (Section 2: F = sum_i F_i),
// then one update  w <- w - (rate / B) * sum_i grad_i  (listing
// `weights = weights - rate*backweights(d_out,in)`, with the batch mean).
template <class T, class A>
A train_batch(const T* images, const int32_t* labels, int B, double rate, T* w, A* g_out) {
  std::vector<A> g(NPARAM, (A)0);
  Acts<T>* a = new Acts<T>;
  A loss = 0;
  for (int n = 0; n < B; ++n) loss += grad_image<T, A>(images + (long)n * NI, labels[n], w, g.data(), *a);
  delete a;
  const A scale = (A)rate / (A)B;
  for (int p = 0; p < NPARAM; ++p) w[p] = (T)((A)w[p] - scale * g[p]);
  if (g_out)
    for (int p = 0; p < NPARAM; ++p) g_out[p] = g[p];
  return loss;
}

// Forward-only classification: prediction = index of the largest output,
// lowest index on ties.
template <class T, class A>
void evaluate(const T* images, const int32_t* labels, long N, const T* w, T* yhat,
              int64_t* n_correct, A* loss_sum) {
  Acts<T>* a = new Acts<T>;
  int64_t ok = 0;
  A loss = 0;
  for (long n = 0; n < N; ++n) {
    forward<T, A>(images + n * NI, w, *a);
    if (yhat) std::memcpy(yhat + n * NY, a->y, sizeof(T) * NY);
    if (labels) {
      int best = 0;
      for (int o = 1; o < NY; ++o)
        if (a->y[o] > a->y[best]) best = o;
      ok += (best == labels[n]);
      loss += loss_of<T, A>(a->y, labels[n]);
    }
  }
  delete a;
  if (n_correct) *n_correct = ok;
  if (loss_sum) *loss_sum = loss;
}

Shape shape_of(const int* s) { return Shape{{s[0], s[1], s[2], s[3]}}; }

}  // namespace

// ---------------------------------------------------------------------------
// C entry points (host pointers only), one set per instance.
#define ORACLE_INSTANCE(SUF, T, A)                                                              \
  extern "C" void oracle_conv_##SUF(const T* I, const int* si, const T* k, const int* sk,       \
                                    T* out) {                                                   \
    conv<T, A>(I, shape_of(si), k, shape_of(sk), out);                                          \
  }                                                                                             \
  extern "C" void oracle_mconv_##SUF(const T* I, const int* si, const T* k, int n,              \
                                     const int* sk, const T* b, T* out) {                       \
    mconv<T, A>(I, shape_of(si), k, n, shape_of(sk), b, out);                                   \
  }                                                                                             \
  extern "C" void oracle_sigmoid_##SUF(const T* in, long n, T* out) { sigmoid<T, A>(in, n, out); } \
  extern "C" void oracle_sigmoid_back_##SUF(const T* y, const T* d_out, long n, T* d_in) {      \
    sigmoid_back<T, A>(y, d_out, n, d_in);                                                      \
  }                                                                                             \
  extern "C" void oracle_avgpool_##SUF(const T* in, long lead, int H, int W, T* out) {          \
    avgpool<T, A>(in, lead, H, W, out);                                                         \
  }                                                                                             \
  extern "C" void oracle_backavgpool_##SUF(const T* d_out, long lead, int Ho, int Wo, T* d_in) { \
    backavgpool<T, A>(d_out, lead, Ho, Wo, d_in);                                               \
  }                                                                                             \
  extern "C" void oracle_backweights_##SUF(const T* d_out, const int* sd, const T* in,          \
                                           const int* si, T* out) {                             \
    backweights<T, A>(d_out, shape_of(sd), in, shape_of(si), out);                              \
  }                                                                                             \
  extern "C" T oracle_backbias_##SUF(const T* d_out, long n) { return backbias<T, A>(d_out, n); } \
  extern "C" void oracle_backin_##SUF(const T* d_out, const int* sd, const T* k, const int* sk, \
                                      const int* si, T* d_in) {                                 \
    backin<T, A>(d_out, shape_of(sd), k, shape_of(sk), shape_of(si), d_in);                     \
  }                                                                                             \
  extern "C" void oracle_forward_##SUF(const T* I, const T* w, T* c1, T* s1, T* c2, T* s2,      \
                                       T* y) {                                                  \
    Acts<T>* a = new Acts<T>;                                                                   \
    forward<T, A>(I, w, *a);                                                                    \
    if (c1) std::memcpy(c1, a->c1, sizeof(a->c1));                                              \
    if (s1) std::memcpy(s1, a->s1, sizeof(a->s1));                                              \
    if (c2) std::memcpy(c2, a->c2, sizeof(a->c2));                                              \
    if (s2) std::memcpy(s2, a->s2, sizeof(a->s2));                                              \
    if (y) std::memcpy(y, a->y, sizeof(a->y));                                                  \
    delete a;                                                                                   \
  }                                                                                             \
  extern "C" double oracle_grad_image_##SUF(const T* I, int label, const T* w, double* g) {     \
    std::vector<A> acc(NPARAM, (A)0);                                                           \
    Acts<T>* a = new Acts<T>;                                                                   \
    A loss = grad_image<T, A>(I, label, w, acc.data(), *a);                                     \
    delete a;                                                                                   \
    for (int p = 0; p < NPARAM; ++p) g[p] = (double)acc[p];                                     \
    return (double)loss;                                                                        \
  }                                                                                             \
  extern "C" double oracle_train_batch_##SUF(const T* images, const int32_t* labels, int B,     \
                                             double rate, T* w, double* g_out) {                \
    std::vector<A> g(NPARAM);                                                                   \
    A loss = train_batch<T, A>(images, labels, B, rate, w, g_out ? g.data() : nullptr);         \
    if (g_out)                                                                                  \
      for (int p = 0; p < NPARAM; ++p) g_out[p] = (double)g[p];                                 \
    return (double)loss;                                                                        \
  }                                                                                             \
  extern "C" void oracle_evaluate_##SUF(const T* images, const int32_t* labels, long N,         \
                                        const T* w, T* yhat, int64_t* n_correct,                \
                                        double* loss_sum) {                                     \
    A loss = 0;                                                                                 \
    evaluate<T, A>(images, labels, N, w, yhat, n_correct, &loss);                               \
    if (loss_sum) *loss_sum = (double)loss;                                                     \
  }

ORACLE_INSTANCE(f32, float, double)
ORACLE_INSTANCE(f64, double, double)

extern "C" int oracle_nparam(void) { return NPARAM; }

// Nearest bfloat16 (1 sign, 8 exponent, 7 fraction bits: float's exponent range with an 8-bit
// significand), ties to the even significand, returned as a float.  Written from the format's
// definition with frexp / nearbyint (the default rounding mode is to nearest even); used to state
// what the reduced-precision convolution computes: the plain definition applied to rounded operands.
// Pins: hand-computed ties and neighbours, idempotence, an independent library conversion.
extern "C" void oracle_round_bf16(const float* in, long n, float* out) {
  for (long i = 0; i < n; ++i) {
    const double x = in[i];
    if (x == 0.0 || !std::isfinite(x)) {
      out[i] = in[i];
      continue;
    }
    int e;
    std::frexp(x, &e);               // |x| = m * 2^e with m in [0.5, 1)
    int q = e - 8;                    // spacing of 8-bit significands at this magnitude: 2^(e-8)
    if (q < -133) q = -133;           // subnormals: fixed spacing 2^-126 * 2^-7
    const double step = std::ldexp(1.0, q);
    out[i] = (float)(std::nearbyint(x / step) * step);  // exact in double; may round up to infinity
  }
}
