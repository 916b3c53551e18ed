/* C ABI of the MI355X (gfx950) library for one training step of the CNN of
 * arXiv 1912.05234 ("Array Languages Make Neural Networks Fast"), Section 3.
 *
 * Network (listing `forward`): image I[28,28] -> C1 = sigmoid(mconv(I, k1[6,5,5], b1[6]))
 * [6,24,24] -> S1 = avgpool [6,12,12] -> C2 = sigmoid(mconv(S1, k2[12,6,5,5], b2[12]))
 * [12,8,8] -> S2 = avgpool [12,4,4] -> yhat = sigmoid(mconv(S2, fc[10,12,1,4,4], b[10])) [10].
 * Loss of one image: 1/2 * sum_o (yhat_o - t_o)^2 with t the one-hot label
 * (paragraph "Backpropagating Convolution").
 *
 * General rules for every entry point
 *  - All data pointers are DEVICE pointers (HIP global memory on the current
 *    device), fp32 / int32 / int64 as typed, contiguous, row-major, and at
 *    least 16-byte aligned.  The library never allocates, frees or keeps
 *    caller memory except the workspace handed to cnn_init.
 *  - Work is enqueued on the given HIP stream (a hipStream_t passed as void*;
 *    NULL = the default stream) and the call returns without waiting.
 *    Results, including scalars, are written to device memory.
 *  - Return value: CNN_OK (0) or a negative CNN_E* code; nothing is enqueued
 *    when an argument check fails.  cnn_strerror names a code.
 *  - Labels must lie in 0..9; this is a precondition, not checked on the device.
 *  - Parameter layout is the paper's: k1[i][u][v], k2[j][c][u][v],
 *    fc[o][c][y][x] (flat input index c*16 + y*4 + x), biases one per map.
 */
#ifndef PAPER_1912_05234_CNN_H
#define PAPER_1912_05234_CNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CNN_OK 0
#define CNN_EINVAL (-1)     /* null / misaligned pointer, size out of range, odd pooling extent */
#define CNN_EWORKSPACE (-2) /* workspace too small for max_batch */
#define CNN_EHIP (-3)       /* a HIP call or kernel launch failed */
#define CNN_ESCRATCH (-4)   /* the problem needs more than the library's built-in scratch buffer */
#define CNN_ETIMEOUT (-5)   /* a bounded wait inside the device-side epoch loop was given up */

#define CNN_NPARAM 3898     /* 150 + 6 + 1800 + 12 + 1920 + 10 */

typedef struct cnn_ctx cnn_ctx; /* opaque, host memory owned by the library */

const char* cnn_strerror(int code);

/* Device bytes cnn_init needs for batches of up to max_batch images (weights, their copy laid out
 * as the kernels' matrix operands, per-workgroup gradient partials, reduction scratch, and for
 * max_batch above 640 one KiB per image: the pooled C2 output and the output error of every image of
 * a batch, from which the fully connected layer's weight gradient is taken once per batch).
 * 0 if max_batch < 1. */
size_t cnn_workspace_bytes(int max_batch);

/* Creates a context over caller-owned device `workspace` (>= cnn_workspace_bytes(max_batch),
 * 256-byte aligned; must outlive the context) and copies the six parameter
 * arrays into it (device pointers; a NULL array means zeros, the usual start
 * for the biases).  All later calls on the context run on `hip_stream`.  Unlike the other calls,
 * cnn_init also makes one small synchronous host-to-device copy (an index table). */
int cnn_init(cnn_ctx** out, void* workspace, size_t workspace_bytes, int max_batch,
             const float* k1, const float* b1, const float* k2, const float* b2,
             const float* fc, const float* b, void* hip_stream);

/* Frees the host-side context (not the workspace).  NULL is allowed. */
void cnn_destroy(cnn_ctx* ctx);

/* Copy the current parameters out to / in from device arrays; NULL skips an array.  The arrays
 * are those of listing `forward` (Section 3): k1[6,5,5], b1[6], k2[12,6,5,5], b2[12],
 * fc[10,12,1,4,4], b[10].  The paper has no such calls; they stand in for checkpointing. */
int cnn_get_weights(cnn_ctx* ctx, float* k1, float* b1, float* k2, float* b2, float* fc, float* b);
int cnn_set_weights(cnn_ctx* ctx, const float* k1, const float* b1, const float* k2,
                    const float* b2, const float* fc, const float* b);

/* Listing `forward` over a batch: images[B,28,28] -> yhat[B,10].  1 <= B <= max_batch. */
int cnn_forward(cnn_ctx* ctx, const float* images, int B, float* yhat);

/* As cnn_forward, also storing every layer's activations (any may be NULL):
 * c1[B,6,24,24], s1[B,6,12,12], c2[B,12,8,8], s2[B,12,4,4], yhat[B,10]. */
int cnn_forward_activations(cnn_ctx* ctx, const float* images, int B, float* c1, float* s1,
                            float* c2, float* s2, float* yhat);

/* Sum over the batch of the loss gradient with respect to all parameters
 * (order k1,b1,k2,b2,fc,b; grad[3898]) without touching the weights: the
 * backweights / backbias / backin / backavgpool chain of Section 3 applied per
 * image and summed (Section 2: F = sum_i F_i).  loss_sum (nullable) receives
 * sum_n L_n. */
int cnn_gradient(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float* grad,
                 float* loss_sum);

/* One SGD step: the gradient above, then w <- w - (lr / B) * grad for every
 * parameter, all gradients taken at the weights from before the step
 * (listing `weights = weights - rate*backweights(d_out,in)`; batch mean).
 * loss_sum (nullable, device) receives sum_n L_n at the old weights.
 * Bitwise reproducible for equal inputs and equal B. */
int cnn_train_batch(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float lr,
                    float* loss_sum);

/* One epoch of mini-batch gradient descent (Section 4.2: the training set is walked in batches,
 * one update per batch): step k = 0 .. ceil(N / batch) - 1 is cnn_train_batch on the images
 * [k * batch, min(N, (k + 1) * batch)) in index order, each with its own size as B (the last
 * step may be shorter).  1 <= batch <= max_batch, N >= 1.  loss_sums (nullable, device,
 * ceil(N / batch) floats) receives each step's sum_n L_n at the weights from before that step.
 * Enqueues 2 * ceil(N / batch) kernels on the context's stream and returns without waiting; the
 * result is bitwise the same as the equivalent sequence of cnn_train_batch calls. */
int cnn_train_epoch(cnn_ctx* ctx, const float* images, const int32_t* labels, int N, int batch,
                    float lr, float* loss_sums);

/* How cnn_train_epoch runs (the answer to the launch-orchestration problem of Section 4.3).
 * device_loop = 0 (default): two kernels per step, enqueued back to back.  device_loop = 1: for
 * batch <= 256 (and no more workgroups than the GPU holds at once) all floor(N / batch) whole steps
 * run inside ONE kernel whose workgroups meet at two grid-wide barriers per step; a shorter last
 * step, larger batches and every other call still use the two-kernel step.  Same arithmetic in the
 * same order: the weights are bitwise those of the default mode.  The kernel needs the GPU to
 * itself (all its workgroups resident): every wait at a barrier is bounded by wait_seconds (0 ..
 * 3600); a workgroup that waits longer sets an error word and all leave, with the weights somewhere
 * between two steps.  never_arrives != 0 makes every barrier wait for a workgroup that does not
 * exist (a way to exercise the give-up path; the first barrier then fails before any update).
 * cnn_epoch_status waits for the context's stream and returns CNN_OK, or CNN_ETIMEOUT once after a
 * kernel gave up (it then re-arms the barrier state; set the weights again before training on). */
int cnn_epoch_mode(cnn_ctx* ctx, int device_loop, double wait_seconds, int never_arrives);
int cnn_epoch_status(cnn_ctx* ctx);

/* Forward-only classification of N images (1 <= N <= max_batch), the pass over the test images
 * that ends the paper's runs (Section 4.2): n_correct (device int64) = number of images whose
 * largest output (lowest index on ties; the paper does not say) equals the label; loss_sum
 * (nullable) = sum_n L_n.  The count is summed in integers: exact for any N. */
int cnn_evaluate(cnn_ctx* ctx, const float* images, const int32_t* labels, int N,
                 int64_t* n_correct, float* loss_sum);

/* Timing aid for callers that cannot see inside a step.  After cnn_profile_begin(ctx, capacity)
 * each cnn_train_batch / cnn_gradient call records one pair of HIP events around its fused
 * forward+backward kernel on the context's stream (the first `capacity` calls; later ones are
 * not recorded).  A pair's reading is the kernel's duration plus the dispatch latency between
 * the two records (about a microsecond), so it is an upper bound on the kernel time.
 * cnn_profile_read waits for the context's stream, writes the elapsed milliseconds of each
 * recorded pair to ms (a HOST array of at least `capacity` floats) and the number of recorded
 * steps to *n_recorded (HOST), and restarts recording from zero.  capacity == 0 stops recording
 * and frees the events.  No device memory is involved. */
int cnn_profile_begin(cnn_ctx* ctx, int capacity);
int cnn_profile_read(cnn_ctx* ctx, float* ms, int capacity, int* n_recorded);

/* ---- Stateless per-operation entry points (batch axis first, NCHW). ----------
 * No context, no device state: results depend on the arguments alone.  (The host keeps one small
 * cache of launch parameters per tensor shape -- an LDS row stride chosen by a bank-conflict
 * model, a pure function of the shape -- guarded by a mutex; calls from several threads are fine.)
 * conv = valid cross-correlation, no kernel flip (listing `conv`), over all Cin
 * input maps per output map plus bias (listing `mconv`), no activation:
 *   out[b,co,y,x] = bias[co] + sum_{ci,u,v} in[b,ci,y+u,x+v] * k[co,ci,u,v]
 * with Ho = H-KH+1, Wo = W-KW+1 (both must be >= 1).  bias may be NULL.  All tensors are device
 * memory, 16-byte aligned, fp32, and finite: the matrix-core kernels multiply padding lanes by
 * zero, which a NaN or infinity in the input would turn into NaN.  (The shapes of the network's own
 * layers have kernels of their own: Cin = 6, Cout = 12, KH = KW = 5, H = W = 12, the second
 * convolution, and Cin = 1, Cout = 6, KH = KW = 5, H = W = 28, the first, for all three convolution
 * calls; I = 192, O = 10 for the three cnn_fc_* calls.  Same
 * definitions, sums in another order.) */
int cnn_conv_fwd(const float* in, const float* k, const float* bias, float* out, int B, int Cin,
                 int H, int W, int Cout, int KH, int KW, void* hip_stream);
/* `backin` summed over output maps: d_in[b,ci,p,q] = sum_co sum_{u,v : 0<=p-u<Ho, 0<=q-v<Wo}
 * k[co,ci,u,v] * d_out[b,co,p-u,q-v].  (The shapes of the network's two convolutions have kernels of
 * their own, see cnn_conv_fwd; same definition, sums in another order.) */
int cnn_conv_bwd_input(const float* d_out, const float* k, float* d_in, int B, int Cin, int H,
                       int W, int Cout, int KH, int KW, void* hip_stream);
/* The two calls above on the fp32 vector unit alone (one thread per output element, plain
 * multiply-adds in the order of the listings `conv` / `backin`, no matrix cores, no LDS): the
 * comparison leg of the per-layer measurement (is the implicit-GEMM form on the matrix cores
 * faster than the vector unit?), and the form to call when the data may hold NaN or infinity:
 * it multiplies nothing by padding zeros.  Same arguments and results to rounding; any shape.
 * (For the weight gradient the same role is played by cnn_conv_bwd_weight with a NULL workspace.) */
int cnn_conv_fwd_valu(const float* in, const float* k, const float* bias, float* out, int B, int Cin,
                      int H, int W, int Cout, int KH, int KW, void* hip_stream);
int cnn_conv_bwd_input_valu(const float* d_out, const float* k, float* d_in, int B, int Cin, int H,
                            int W, int Cout, int KH, int KW, void* hip_stream);
/* Reduced-precision forms of cnn_conv_fwd and cnn_conv_bwd_input, same arguments, same fp32 tensors: every operand
 * (input or output error, and kernel) is rounded to bfloat16 (nearest, ties to even) as it is read,
 * products are summed in fp32 on the bf16 matrix cores, bias and result stay fp32.  The paper
 * computes in `float` (Section 3, listings `conv` and `backin`); these trade its 1e-5 agreement for
 * matrix-core throughput: the result is the plain definition applied to the rounded operands, to
 * fp32 summation accuracy.  Shapes that do not fit in LDS run a plain kernel with the same rounding. */
int cnn_conv_fwd_bf16(const float* in, const float* k, const float* bias, float* out, int B, int Cin,
                      int H, int W, int Cout, int KH, int KW, void* hip_stream);
int cnn_conv_bwd_input_bf16(const float* d_out, const float* k, float* d_in, int B, int Cin, int H,
                            int W, int Cout, int KH, int KW, void* hip_stream);
/* `backweights` and `backbias`, summed over the batch:
 *   d_k[co,ci,u,v] = sum_{b,y,x} in[b,ci,y+u,x+v] * d_out[b,co,y,x];  d_bias[co] = sum d_out[:,co].
 * d_bias may be NULL.  `workspace` is device memory (16-byte aligned) for partial sums that the call
 * may overwrite; with at least cnn_conv_bwd_weight_workspace_bytes() bytes the matrix-core kernel
 * runs, with NULL or fewer bytes a slower kernel that needs none.  The summation order is fixed in
 * either case (the two orders differ).  The size query returns 0 for invalid arguments and for
 * shapes only the slower kernel serves. */
size_t cnn_conv_bwd_weight_workspace_bytes(int B, int Cin, int H, int W, int Cout, int KH, int KW);
int cnn_conv_bwd_weight(const float* in, const float* d_out, float* d_k, float* d_bias, int B,
                        int Cin, int H, int W, int Cout, int KH, int KW, void* workspace,
                        size_t workspace_bytes, void* hip_stream);
/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): cnn_conv_bwd_weight with the partial sums in
 * a buffer of CNN_STATIC_SCRATCH_BYTES that is part of the loaded library (one copy per GPU, held
 * until the process ends) instead of a caller workspace.  Same kernels, same summation order and
 * therefore bitwise the same d_k / d_bias as cnn_conv_bwd_weight with a sufficient workspace.  The
 * call allocates and frees nothing.  Returns CNN_ESCRATCH, with nothing enqueued, when the shape
 * would need more partial sums than the buffer holds (cnn_conv_bwd_weight_workspace_bytes() tells:
 * the network's layers need 2 MiB (C1) and 10.1 MiB (C2) at any batch size); shapes that only the
 * slower kernel serves need no scratch and are accepted.  All calls on one GPU share that GPU's
 * buffer: two calls whose kernels may overlap on one GPU (different streams, different threads)
 * race, so serialise them.  The buffer's address on a device is looked up at the first call on
 * that device (no allocation either). */
#define CNN_STATIC_SCRATCH_BYTES (16u << 20)
int cnn_conv_bwd_weight_static(const float* in, const float* d_out, float* d_k, float* d_bias, int B,
                               int Cin, int H, int W, int Cout, int KH, int KW, void* hip_stream);
/* Reduced-precision form of cnn_conv_bwd_weight, same arguments and workspace rules (its own size
 * query): `in` and `d_out` are rounded to bfloat16 as they are read, products are summed in fp32 on
 * the bf16 matrix cores; d_bias is the fp32 sum of the rounded d_out. */
size_t cnn_conv_bwd_weight_bf16_workspace_bytes(int B, int Cin, int H, int W, int Cout, int KH, int KW);
int cnn_conv_bwd_weight_bf16(const float* in, const float* d_out, float* d_k, float* d_bias, int B,
                             int Cin, int H, int W, int Cout, int KH, int KW, void* workspace,
                             size_t workspace_bytes, void* hip_stream);
/* Listing `avgpool` over [B,C,H,W] (H, W even) -> [B,C,H/2,W/2]. */
int cnn_avgpool_fwd(const float* in, float* out, int B, int C, int H, int W, void* hip_stream);
/* Listing `backavgpool`: d_out[B,C,Ho,Wo] -> d_in[B,C,2Ho,2Wo] = d_out[..,y/2,x/2] / 4. */
int cnn_avgpool_bwd(const float* d_out, float* d_in, int B, int C, int Ho, int Wo, void* hip_stream);
/* Fully connected layer (mconv with kernel shape = input shape):
 *   out[b,o] = bias[o] + sum_i in[b,i] * w[o,i];  bias may be NULL. */
int cnn_fc_fwd(const float* in, const float* w, const float* bias, float* out, int B, int I, int O,
               void* hip_stream);
/* Listing `backin` for that layer (kernel shape = input shape, so the error of an output is a
 * single number and every product is valid), summed over the outputs:
 *   d_in[b,i] = sum_o w[o,i] * d_out[b,o]. */
int cnn_fc_bwd_input(const float* d_out, const float* w, float* d_in, int B, int I, int O,
                     void* hip_stream);
/* Listings `backweights` (= conv(in, d_out) with a one-element d_out) and `backbias` for that
 * layer, summed over the batch:
 *   d_w[o,i] = sum_b d_out[b,o] * in[b,i];  d_bias[o] = sum_b d_out[b,o] (nullable).  Workspace as
 * for cnn_conv_bwd_weight. */
size_t cnn_fc_bwd_weight_workspace_bytes(int B, int I, int O);
int cnn_fc_bwd_weight(const float* in, const float* d_out, float* d_w, float* d_bias, int B, int I,
                      int O, void* workspace, size_t workspace_bytes, void* hip_stream);
/* Listing `sigmoid`: y = 1 / (1 + exp(-x)), n elements. */
int cnn_logistic_fwd(const float* x, float* y, size_t n, void* hip_stream);
/* Its derivative through the stored output: d_x = d_y * y * (1 - y).  Not printed in the paper
 * (the back-propagation driver is left to its repository); derived from the listing above. */
int cnn_logistic_bwd(const float* y, const float* d_y, float* d_x, size_t n, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
