// Kernels of the fused step, the deterministic gradient reduction with the SGD
// update, and the context-based C entry points.  Definitions: arXiv 1912.05234,
// Section 3 (forward, conv, mconv, sigmoid, avgpool, backweights, backbias,
// backin, backavgpool) and Section 2 (batch gradient descent,
// w := w - eta * sum_i grad F_i).
//
// One wavefront owns one image at a time (cnn_wave.h): the pixels, every
// activation and every error array stay in that wave's LDS and registers; the
// only HBM traffic per image is its 3136-byte pixel block and its label.  A
// workgroup is a single wave, walks the images n = g, g+G, g+2G, ... and keeps
// its 3898 gradient sums in registers, so no atomics touch memory shared between
// waves and a partial's value does not depend on scheduling.  A second kernel
// adds the G partials in a fixed order and applies the update.
#include <new>
#include <vector>

#include "cnn_wave.h"
#include "cnn_group.h"

namespace {

using namespace cnn;

constexpr int GCAP = 1024;      // waves of a full machine at one per SIMD (256 compute units)
constexpr int TRAIN_BLOCKS = 256;  // most workgroups (= gradient partials) of the large-batch training kernel: one per compute unit
constexpr int FWD_GCAP = 3072;  // most forward-only waves: three per SIMD
// Batches up to this size give each image to a workgroup of eight waves (lower latency per image;
// up to two such workgroups share a compute unit); larger ones give each image to a single wave
// (more images in flight, no barriers).  Measured crossover: 21.7 against 27.9 us per step at batch
// 512, 30.8 against 28.8 us at batch 768.
constexpr int GROUP_MAX_BATCH = 640;
// Device-side epoch loop: one barrier flag per workgroup (a batch of at most EPOCH_MAX_BATCH images:
// thread t of a 512-thread workgroup polls flag t), one flag nobody sets, the error word.
constexpr int EPOCH_MAX_BATCH = 256;
constexpr int SYNC_PHANTOM = EPOCH_MAX_BATCH, SYNC_ERROR = EPOCH_MAX_BATCH + 1, SYNC_WORDS = EPOCH_MAX_BATCH + 2;

// Forward-only: yhat[B,10], optional activation dump, optional (count, loss) per wave.
// Wave gw = 4 * blockIdx.x + wave walks the images gw, gw + G, gw + 2G, ... (G = waves in the grid).
template <int MODE>
__global__ __launch_bounds__(64 * WAVES, 2) void forward_kernel(const float* __restrict__ images,
                                                            const int32_t* __restrict__ labels, int B,
                                                            const float* __restrict__ tabg,
                                                            float* __restrict__ yhat, DumpPtrs dump,
                                                            float* __restrict__ eval_partial) {
  __shared__ OperandTable<TAB_FWD_ENTRIES> tab;
  __shared__ FwdLds lds[WAVES];
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63;
  FwdLds& s = lds[wave];
  WaveState<MODE> st;
  const size_t gw = (size_t)blockIdx.x * WAVES + wave, G = (size_t)gridDim.x * WAVES;
  Pixels px = load_pixels(images + (gw < (size_t)B ? gw : 0) * NI);  // in flight during the set-up
  load_tables<TAB_FWD_ENTRIES, 64 * WAVES>(tab, tabg);
  wave_init(st, s);
  __syncthreads();  // the only workgroup-wide barrier: the operand table is complete
  st.bias2 = tab.bias[l & 15];
  float n_ok = 0.0f, loss = 0.0f;
  for (size_t n = gw; n < (size_t)B; n += G) {
    float y[10];
    const size_t nn = n + G;
    wave_image<MODE>(st, s, tab, px, nn < (size_t)B ? images + nn * NI : nullptr, 0, y, dump, n);
    if (yhat) {
#pragma unroll
      for (int o = 0; o < NY; ++o)
        if (l == o) yhat[n * NY + o] = y[o];
    }
    if (labels) {
      const int label = labels[n];
      int best = 0;
      float bestv = y[0], lsum = 0.0f;
#pragma unroll
      for (int o = 0; o < NY; ++o) {
        if (o > 0 && y[o] > bestv) {  // strict '>' keeps the lowest index on ties
          bestv = y[o];
          best = o;
        }
        const float e = y[o] - (o == label ? 1.0f : 0.0f);
        lsum = fmaf(e, e, lsum);
      }
      n_ok += (best == label) ? 1.0f : 0.0f;
      loss = fmaf(0.5f, lsum, loss);
    }
    wave_sync();
  }
  if (eval_partial && l == 0) {
    eval_partial[2 * gw] = n_ok;  // exact: far fewer than 2^24 images per wave
    eval_partial[2 * gw + 1] = loss;
  }
}

// Sums the G (count, loss) pairs: 1024 interleaved strands (at most three pairs each for the 3072
// waves of the forward kernel, so the loads are one memory round trip), then a fixed tree over the
// strands.  The counts are whole numbers (each wave's is far below 2^24, so exact in its float) and
// are added as 64-bit integers.
constexpr int EVAL_REDUCE_THREADS = 1024;
__global__ __launch_bounds__(EVAL_REDUCE_THREADS) void eval_reduce_kernel(const float* __restrict__ eval_partial,
                                                                          int G, int64_t* __restrict__ n_correct,
                                                                          float* __restrict__ loss_sum) {
  __shared__ long long counts[EVAL_REDUCE_THREADS];
  __shared__ float losses[EVAL_REDUCE_THREADS];
  const int t = threadIdx.x;
  long long ok = 0;
  float loss = 0.0f;
  for (int g = t; g < G; g += EVAL_REDUCE_THREADS) {
    const float2 pair = reinterpret_cast<const float2*>(eval_partial)[g];
    ok += (long long)pair.x;
    loss += pair.y;
  }
  counts[t] = ok;
  losses[t] = loss;
  __syncthreads();
  for (int half = EVAL_REDUCE_THREADS / 2; half >= 1; half >>= 1) {
    if (t < half) {
      counts[t] += counts[t + half];
      losses[t] += losses[t + half];
    }
    __syncthreads();
  }
  if (t == 0) {
    if (n_correct) *n_correct = (int64_t)counts[0];
    if (loss_sum) *loss_sum = losses[0];
  }
}

// Forward + backward over each wave's images: eight waves per workgroup, one workgroup per compute
// unit, i.e. two waves per SIMD.  (One wave alone issues a vector instruction every 2.4 ns, two
// together one every 1.4 ns, and the matrix instructions of one run under the LDS waits of the
// other; the price is 256 registers and 15.25 KB of LDS per wave.)  Workgroup b owns the images
// b + gridDim.x * k, k < K; WaveShare says which of them each wave takes.  The eight waves then add
// their gradient sums through LDS in a fixed order and the workgroup writes ONE partial row,
// partial[blockIdx.x][PSTRIDE], with 16-byte stores (a wave without images contributes zeros).
constexpr int TWAVES = 8;
// Which of a workgroup's K images each wave takes.  The images are dealt in rounds: a full round
// gives one image to each of the eight waves, a half round one to each of waves 0..3 only; the
// pattern of SHARE_ROUNDS rounds repeats every SHARE_PERIOD images.  A function of K and the wave
// alone, so the grouping of the gradient sums (and with it every rounding) is the same in every run.
// Why not full rounds only: the two waves of a SIMD do not advance at the same rate.  The one in
// the lower slot wins the issue arbitration more often and needs about 64 thousand clocks per
// image where its partner needs 88 (51 thousand for a wave that has the SIMD to itself), in every
// workgroup alike, so an equal split leaves the SIMD to one wave for the last sixth of the kernel.
// A batch that does not fill the machine (K < 8) still leaves waves 4..7 idle rather than two
// waves on one SIMD and none on another: the first round is a full one.
constexpr unsigned SHARE_PATTERN = 0xB;  // rounds F F H F (first round in bit 0): 4 images to 3
constexpr int SHARE_ROUNDS = 4;
constexpr bool share_full(int r) { return (SHARE_PATTERN >> r) & 1; }
constexpr int share_start(int r) {  // first image of round r inside a period
  int at = 0;
  for (int i = 0; i < r; ++i) at += share_full(i) ? 8 : 4;
  return at;
}
constexpr int SHARE_PERIOD = share_start(SHARE_ROUNDS);
constexpr int share_full_rounds() {
  int n = 0;
  for (int r = 0; r < SHARE_ROUNDS; ++r) n += share_full(r);
  return n;
}
constexpr int SHARE_FULL = share_full_rounds();
static_assert(share_full(0), "the first round deals to all eight waves");
struct ShareSlots {  // start of the j-th round that deals to waves 0..3 (every round) / to waves 4..7 (full rounds)
  int low[SHARE_ROUNDS], high[SHARE_ROUNDS];
  constexpr ShareSlots() : low(), high() {
    int nh = 0;
    for (int r = 0; r < SHARE_ROUNDS; ++r) {
      low[r] = share_start(r);
      if (share_full(r)) high[nh++] = share_start(r);
    }
    for (; nh < SHARE_ROUNDS; ++nh) high[nh] = SHARE_PERIOD;  // never reached
  }
};
__device__ constexpr ShareSlots SHARE_SLOTS = ShareSlots();
// How many of K images wave w takes.
__device__ __forceinline__ int share_count(int K, int w) {
  const int per = w < 4 ? SHARE_ROUNDS : SHARE_FULL, rest = K % SHARE_PERIOD;
  int n = per * (K / SHARE_PERIOD);
#pragma unroll
  for (int j = 0; j < SHARE_ROUNDS; ++j)
    if (j < per && (w < 4 ? SHARE_SLOTS.low[j] : SHARE_SLOTS.high[j]) + w < rest) ++n;
  return n;
}
// Walks wave w's images: k() is the current one, left how many remain including it.
struct WaveShare {
  int base, j, per, left, w;
  __device__ __forceinline__ WaveShare(int K, int wave) : base(0), j(0), per(wave < 4 ? SHARE_ROUNDS : SHARE_FULL), left(share_count(K, wave)), w(wave) {}
  __device__ __forceinline__ int k() const { return base + (w < 4 ? SHARE_SLOTS.low[j] : SHARE_SLOTS.high[j]) + w; }
  __device__ __forceinline__ void advance() {
    --left;
    if (++j == per) {
      j = 0;
      base += SHARE_PERIOD;
    }
  }
};
__global__ __launch_bounds__(64 * TWAVES) __attribute__((amdgpu_waves_per_eu(2, 2))) void train_kernel(
    const float* __restrict__ images, const int32_t* __restrict__ labels, int B, const float* __restrict__ tabg,
    float* __restrict__ partial, float* fc_hist) {
  __shared__ OperandTable<TAB_WAVE_ENTRIES> tab;
  __shared__ WaveTrainLds lds[TWAVES];
  __shared__ WindowTable wt;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // in a scalar register: addresses built on it are wave-uniform
  WaveTrainLds& s = lds[wave];
  WaveState<kTrain> st;
  CNN_KERNEL_MARK(0);
  const int K = B > (int)blockIdx.x ? (B - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
  WaveShare mine(K, wave);
  const bool has_images = mine.left > 0;
  auto image_index = [&](int k) { return (size_t)blockIdx.x + (size_t)gridDim.x * (size_t)k; };
  Pixels px = load_pixels(images + (has_images ? image_index(mine.k()) : 0) * NI);  // in flight during the set-up
  // every load of the set-up is issued before anything waits for one: the table proper (BF, FCW, AB,
  // k1t, biases) in 16-byte pieces, and the packed entries, gathered one float at a time
  TableLoad<TAB_WAVE_ENTRIES, 64 * TWAVES, false, TAB_PK> table;
  table.fetch(tabg);
  constexpr int PK_ROUNDS = (TAB_PK_COUNT * 64 + 64 * TWAVES - 1) / (64 * TWAVES);
  float pk[PK_ROUNDS];
#pragma unroll
  for (int r = 0; r < PK_ROUNDS; ++r) {
    const int e = r * TWAVES + wave;  // a wave gathers one entry per round (wave-uniform: scalar arithmetic)
    const int slot = e < TAB_PK_COUNT ? packed_table_slot(e, threadIdx.x & 63) : -1;
    pk[r] = tabg[slot >= 0 ? slot : 0];
    if (slot < 0) pk[r] = 0.0f;
  }
  window_table_init<64 * TWAVES>(wt);
  // waves without images skip their set-up and their row
  if (has_images) {
    wave_init(st, s);
    store_pixels(s.img, px);
  }
  table.commit(tab);
#pragma unroll
  for (int r = 0; r < PK_ROUNDS; ++r) {
    const int i = r * 64 * TWAVES + threadIdx.x;
    if (i < TAB_PK_COUNT * 64) tab.e[TAB_PK * 64 + i] = pk[r];
  }
  __syncthreads();  // the operand and window tables are complete
  st.bias2 = tab.bias[threadIdx.x & 15];
  const DumpPtrs none = {nullptr, nullptr, nullptr, nullptr};
  CNN_KERNEL_MARK(1);
  while (mine.left > 0) {
    float y[10];
    const size_t n = image_index(mine.k());
    mine.advance();
    const size_t nn = mine.left > 0 ? image_index(mine.k()) : n;
    wave_image<kTrain>(st, s, tab, px, images + nn * NI, labels[n], y, none, n, &wt, fc_hist + n * FC_HIST);
  }
  CNN_KERNEL_MARK(2);
  // FC weight gradient: a second walk over this wave's images, four per K step (the history rows
  // have left the L2 cache by now; a wave that is done early does this while the others still work)
  f4 g_fc[12];
  if (has_images) {
#pragma unroll
    for (int nt = 0; nt < 12; ++nt) g_fc[nt] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    // this wave's stores to its history rows are complete before it reads them back
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    WaveShare again(K, wave);
    const float* row = fc_hist;  // overwritten before use: has_images
    // operands of one K step (the next four images, fewer at the end)
    auto load_step = [&](FcStepOperands& op) {
      const float* rows[4];
      const int count = again.left < 4 ? again.left : 4;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (again.left > 0) {
          row = fc_hist + image_index(again.k()) * FC_HIST;
          again.advance();
        }
        rows[k] = row;  // past the last image: the last one again (count masks its delta)
      }
      fc_step_load(op, rows, count);
    };
    // eight steps (32 images) at a time while there are that many, then four, two, one: the loads of
    // a group are one memory round trip (the registers of the image loop are free by now)
    auto steps = [&](auto group) {
      constexpr int N = decltype(group)::value;
      FcStepOperands ops[N];
#pragma unroll
      for (int g = 0; g < N; ++g) load_step(ops[g]);
#pragma unroll
      for (int g = 0; g < N; ++g) fc_step_mfma(g_fc, ops[g]);
    };
    while (again.left > 28) steps(std::integral_constant<int, 8>());
    if (again.left > 12) steps(std::integral_constant<int, 4>());
    if (again.left > 12) steps(std::integral_constant<int, 4>());
    if (again.left > 4) steps(std::integral_constant<int, 2>());
    if (again.left > 4) steps(std::integral_constant<int, 2>());
    if (again.left > 0) steps(std::integral_constant<int, 1>());
    if (again.left > 0) steps(std::integral_constant<int, 1>());
  }
  __syncthreads();  // every wave is done with the operand table: its storage parks the C1 GEMM results
  if (has_images) wave_flush(st, g_fc, reinterpret_cast<float*>(&s), tab.e + wave * C1G_PARK);
  __syncthreads();
  {
    // rows of the waves that had images in a fixed tree; an idle wave's row counts as zeros (the
    // first round deals image k to wave k, so wave k has images exactly when K > k)
    const f4* r = reinterpret_cast<const f4*>(&lds[0]);
    constexpr int RF4 = PSTRIDE / 4;  // a wave's area is exactly one row
    f4* dst = reinterpret_cast<f4*>(partial + (size_t)blockIdx.x * PSTRIDE);
    const f4 zero = f4{0.0f, 0.0f, 0.0f, 0.0f};
    for (int i = threadIdx.x; i < RF4; i += 64 * TWAVES) {
      f4 v[TWAVES];
#pragma unroll
      for (int k = 0; k < TWAVES; ++k) v[k] = K > k ? r[i + k * RF4] : zero;
      dst[i] = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
    }
  }
  CNN_KERNEL_MARK(3);
  CNN_PHASE_FLUSH;
}

// Small batches: eight waves share one image (cnn_group.h); one partial row per workgroup.
__global__ __launch_bounds__(64 * GWAVES) void train_group_kernel(const float* __restrict__ images,
                                                              const int32_t* __restrict__ labels, int B,
                                                              const float* __restrict__ tabg,
                                                              float* __restrict__ partial) {
  __shared__ OperandTable<TAB_TRAIN_ENTRIES> tab;
  __shared__ TrainLds s;
  __shared__ __align__(16) float d_s1b[D_S1B_FLOATS];
  __shared__ float ybuf[16];
  group_train<false>(images + (size_t)blockIdx.x * NI, labels + blockIdx.x, tabg,
                     partial + (size_t)blockIdx.x * PSTRIDE, tab, s, d_s1b, ybuf);
}

// Expanded operand table from the flat parameter vector: tabg[i] = table_scale(i) * w[table_source(i)] or 0.
__global__ __launch_bounds__(256) void expand_kernel(const float* __restrict__ w, float* __restrict__ tabg) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < TABG_FLOATS) {
    const int p = table_source(i);
    tabg[i] = p >= 0 ? table_scale(i) * w[p] : 0.0f;
  }
}

// Adds the G partial rows in a fixed order (sixteen interleaved strands, each summed in row
// order, then a fixed tree over the strands) and either applies  w <- w - scale * g  (grad_out ==
// nullptr) or stores g.  An updated parameter is also written to its slots of the expanded operand
// table, dest[p][0..3] (-1 = none).  One block of work per 64 parameters, `block` < PSTRIDE / 64; the
// lanes of a wave read 64 consecutive floats of a row, and a strand keeps eight row reads in flight.
// THREADS = 1024: one strand per wave; 512: every wave takes strands s and s + 8, one after the
// other (same sums, same order).  COHERENT (device-side epoch loop: rows, weights and table are
// written and read by different compute units within one kernel): agent-scope loads and stores.
constexpr int RSTRANDS = 16;
template <bool COHERENT>
__device__ __forceinline__ float ld_shared(const float* p) {
  return COHERENT ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
}
template <bool COHERENT>
__device__ __forceinline__ void st_shared(float* p, float v) {
  if (COHERENT)
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    *p = v;
}
template <int THREADS, bool COHERENT>
__device__ __forceinline__ void reduce_update_block(int block, float (&red)[RSTRANDS][64],
                                                    const float* __restrict__ partial, int G, float scale,
                                                    float* __restrict__ w, const int32_t* __restrict__ dest,
                                                    float* __restrict__ tabg, float* __restrict__ grad_out,
                                                    float* __restrict__ loss_sum) {
  static_assert(THREADS == 64 * RSTRANDS || THREADS == 32 * RSTRANDS, "one or two strands per wave");
  constexpr int WAVES_HERE = THREADS / 64, PASSES = RSTRANDS / WAVES_HERE;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int p = block * 64 + lane;
  // what the update needs besides the sum is fetched first, so that it arrives during the reduction
  float w_old = 0.0f;
  int4 d = int4{-1, -1, -1, -1};
  if (wave == 0 && !grad_out && p < NPARAM) {
    w_old = ld_shared<COHERENT>(w + p);
    d = reinterpret_cast<const int4*>(dest)[p];
  }
  const float* src = partial + p;
#pragma unroll
  for (int pass = 0; pass < PASSES; ++pass) {
    const int strand = wave + WAVES_HERE * pass;
    // eight row reads in flight per strand; a row index past G reads nothing and adds 0.0
    float a[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int g = strand; g < G; g += 8 * RSTRANDS) {
      float r[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int row = g + k * RSTRANDS;
        r[k] = row < G ? ld_shared<COHERENT>(src + (size_t)row * PSTRIDE) : 0.0f;
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) a[k] += r[k];
    }
    red[strand][lane] = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
  }
  __syncthreads();
  if (wave == 0) {
    float t[RSTRANDS];
#pragma unroll
    for (int k = 0; k < RSTRANDS; ++k) t[k] = red[k][lane];
#pragma unroll
    for (int step = 1; step < RSTRANDS; step *= 2)
#pragma unroll
      for (int k = 0; k < RSTRANDS; k += 2 * step) t[k] += t[k + step];
    const float total = t[0];
    if (p < NPARAM) {
      if (grad_out) {
        grad_out[p] = total;
      } else {
        const float wn = fmaf(-scale, total, w_old);
        st_shared<COHERENT>(w + p, wn);
        if (d.x >= 0) st_shared<COHERENT>(tabg + d.x, table_scale(d.x) * wn);
        if (d.y >= 0) st_shared<COHERENT>(tabg + d.y, table_scale(d.y) * wn);
        if (d.z >= 0) st_shared<COHERENT>(tabg + d.z, table_scale(d.z) * wn);
        if (d.w >= 0) st_shared<COHERENT>(tabg + d.w, table_scale(d.w) * wn);
      }
    } else if (p == LOSS_SLOT && loss_sum) {
      *loss_sum = total;
    }
  }
}

__global__ __launch_bounds__(64 * RSTRANDS) void reduce_update_kernel(const float* __restrict__ partial, int G,
                                                                     float scale, float* __restrict__ w,
                                                                     const int32_t* __restrict__ dest,
                                                                     float* __restrict__ tabg,
                                                                     float* __restrict__ grad_out,
                                                                     float* __restrict__ loss_sum) {
  __shared__ float red[RSTRANDS][64];
  reduce_update_block<64 * RSTRANDS, false>(blockIdx.x, red, partial, G, scale, w, dest, tabg, grad_out, loss_sum);
}

// ---- device-side epoch loop ---------------------------------------------------------------------------
// Every step of an epoch inside ONE kernel, for batches small enough that all workgroups (one per
// image of a batch, eight waves each) are resident at once.  Per step: the fused forward + backward
// of the workgroup's image (cnn_group.h) -> its partial row; grid barrier; the workgroups 0 ..
// PSTRIDE/64 - 1 sum their 64 parameters over the rows in the order of reduce_update_kernel, update
// them and the expanded operand table; grid barrier; next step (which re-reads the table).
// Rows, weights and table travel between compute units (whose L2 caches are not coherent with each
// other) as agent-scope loads and stores.
//
// Grid barrier: workgroup b publishes the number of the barrier in flags[b] once all its threads'
// stores have completed; thread t < G of every workgroup polls flags[t].  No read-modify-write: a
// central counter costs 3.2 us per barrier at 100 workgroups, this form 2.5 us.  Every wait is
// bounded: after `limit` ticks of the 100 MHz wall clock (or when another workgroup has given up)
// the workgroup sets the error word and leaves; so do, in turn, all others.  flags[phantom] with
// phantom >= 0 is a flag nobody sets: the host's way to force the give-up path in a test.
struct GridSync {
  unsigned* flags;
  unsigned* error;
  unsigned G, epoch;
  long long limit;
  int phantom;
};
__device__ __forceinline__ bool grid_barrier(GridSync& gs, int* dead) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's agent-scope stores have been performed
  __syncthreads();
  ++gs.epoch;
  const unsigned t = threadIdx.x;
  if (t == 0) __hip_atomic_store(&gs.flags[blockIdx.x], gs.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (t < gs.G || (gs.phantom >= 0 && t == gs.G)) {
    const unsigned* flag = &gs.flags[t < gs.G ? t : (unsigned)gs.phantom];
    const long long t0 = wall_clock64();
    unsigned polls = 0;
    while ((int)(__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - gs.epoch) < 0) {
      if ((++polls & 7) == 0 &&
          (wall_clock64() - t0 > gs.limit ||
           __hip_atomic_load(gs.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
        __hip_atomic_store(gs.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *dead = 1;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
  }
  __syncthreads();
  return *dead == 0;
}

__global__ __launch_bounds__(64 * GWAVES) void train_epoch_kernel(const float* __restrict__ images,
                                                              const int32_t* __restrict__ labels, int steps,
                                                              float scale, float* __restrict__ w,
                                                              const int32_t* __restrict__ dest,
                                                              float* __restrict__ tabg,
                                                              float* __restrict__ partial,
                                                              float* __restrict__ loss_sums, unsigned* flags,
                                                              unsigned* error, unsigned epoch_base,
                                                              long long limit, int phantom) {
  __shared__ OperandTable<TAB_TRAIN_ENTRIES> tab;
  __shared__ TrainLds s;
  __shared__ __align__(16) float d_s1b[D_S1B_FLOATS];
  __shared__ float ybuf[16];
  __shared__ float red[RSTRANDS][64];
  __shared__ int dead;
  if (threadIdx.x == 0) dead = 0;
  GridSync gs{flags, error, gridDim.x, epoch_base, limit, phantom};
  const int B = gridDim.x;  // images per step = workgroups
  // a launch that follows one that gave up does nothing (the host resets the error word)
  if (__hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
  float* row = partial + (size_t)blockIdx.x * PSTRIDE;
  for (int k = 0; k < steps; ++k) {
    const size_t n = (size_t)k * B + blockIdx.x;
    group_train<true>(images + n * NI, labels + n, tabg, row, tab, s, d_s1b, ybuf);
    if (!grid_barrier(gs, &dead)) return;  // every row of the step is in memory
    for (int j = blockIdx.x; j < PSTRIDE / 64; j += gridDim.x) {  // (a batch below 61 images: several blocks each)
      reduce_update_block<64 * GWAVES, true>(j, red, partial, B, scale, w, dest, tabg, nullptr,
                                            loss_sums ? loss_sums + k : nullptr);
      __syncthreads();  // `red` is free again
    }
    if (!grid_barrier(gs, &dead)) return;  // weights and table of the next step are in memory
  }
}

}  // namespace

// ------------------------------------------------------------------- C ABI
struct cnn_ctx {
  hipStream_t stream;
  int max_batch;
  int gcap;      // cap on training waves
  int fwd_gcap;  // cap on forward-only waves
  float* w;             // [PSTRIDE]
  float* tabg;          // [TABG_FLOATS]: the operand table expanded from w, kept in step with it
  int32_t* dest;        // [PSTRIDE][TABLE_MAX_DEST]: slots of tabg that hold parameter p
  float* partial;       // [partial_rows_for(max_batch)][PSTRIDE]
  float* eval_partial;  // [gcap][2]
  float* fc_hist;       // [max_batch][FC_HIST] when max_batch > GROUP_MAX_BATCH: per image, what the FC weight gradient needs
  unsigned* sync;       // [SYNC_WORDS]: barrier flags of the device-side epoch loop, then its error word
  int epoch_mode = 0;         // 1: cnn_train_epoch runs as one kernel where it can
  long long wait_ticks = 0;   // longest wait at a grid barrier, in ticks of the 100 MHz wall clock
  int phantom = -1;           // test hook: also wait for this flag, which nobody sets
  unsigned barrier_count = 0; // barriers passed by every workgroup so far (flags hold such counts)
  int resident_limit = -1;    // most workgroups of train_epoch_kernel resident at once (-1: not asked yet)
  std::vector<hipEvent_t> ev;  // 2 per recorded step (before, after the fused kernel)
  int ev_used = 0;             // recorded steps
};

namespace {

constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Cap on waves, rounded up to whole workgroups.
inline int gcap_for(int max_batch, int cap = GCAP) {
  const int g = max_batch < cap ? max_batch : cap;
  return (g + WAVES - 1) / WAVES * WAVES;
}

struct Layout {
  size_t w, tabg, dest, partial, eval_partial, fc_hist, sync, total;
};

// Partial rows a step can write: one per workgroup, in the one-wave-per-image kernel (four waves
// per workgroup) or in the small-batch kernel (one workgroup per image).
inline int partial_rows_for(int max_batch) {
  const int by_wave = max_batch < TRAIN_BLOCKS ? max_batch : TRAIN_BLOCKS;
  const int by_group = max_batch < GROUP_MAX_BATCH ? max_batch : GROUP_MAX_BATCH;
  return by_wave > by_group ? by_wave : by_group;
}

inline Layout layout_for(int max_batch) {
  Layout l;
  const size_t g = (size_t)partial_rows_for(max_batch);
  l.w = 0;
  l.tabg = align_up(l.w + sizeof(float) * PSTRIDE, 256);
  l.dest = align_up(l.tabg + sizeof(float) * TABG_FLOATS, 256);
  l.partial = align_up(l.dest + sizeof(int32_t) * TABLE_MAX_DEST * PSTRIDE, 256);
  l.eval_partial = align_up(l.partial + sizeof(float) * PSTRIDE * g, 256);
  l.fc_hist = align_up(l.eval_partial + sizeof(float) * 2 * (size_t)gcap_for(max_batch, FWD_GCAP), 256);
  // only the large-batch kernel keeps sums in global memory; it never launches more workgroups than images
  const size_t hist_rows = max_batch > GROUP_MAX_BATCH ? (size_t)max_batch : 0;
  l.sync = align_up(l.fc_hist + sizeof(float) * FC_HIST * hist_rows, 256);
  l.total = align_up(l.sync + sizeof(unsigned) * SYNC_WORDS, 256);
  return l;
}

const int kParamOff[6] = {OFF_K1, OFF_B1, OFF_K2, OFF_B2, OFF_FC, OFF_B};
const int kParamLen[6] = {150, 6, 1800, 12, 1920, 10};

inline bool batch_ok(const cnn_ctx* ctx, int B) { return ctx && B >= 1 && B <= ctx->max_batch; }

// Workgroups to launch for B images: one wave per image up to the cap on waves.  The forward-only
// kernel may keep one, two or three waves per SIMD resident; the grid is the multiple of a full
// machine (1024 SIMDs) that gives the busiest SIMD the least work.  A SIMD's throughput with w
// resident waves was measured as 120 : 141 : 145 (w = 1, 2, 3), so its time is proportional to
// w * ceil(B / (1024 w)) / rate(w); e.g. 10000 images take 10 image slots per SIMD with two waves
// against 12 with three.
inline int blocks_for(const cnn_ctx* ctx, int B, bool forward_only) {
  const int cap = forward_only ? ctx->fwd_gcap : ctx->gcap;
  int waves = B < cap ? B : cap;
  if (forward_only && B > GCAP) {
    static const float kRate[3] = {120.0f, 141.0f, 145.0f};
    float best = 0.0f;
    for (int w = 1; w <= 3 && GCAP * w <= cap; ++w) {
      const int g = GCAP * w, per_wave = (B + g - 1) / g;
      const float t = (float)(w * per_wave) / kRate[w - 1];
      if (w == 1 || t < best) {
        best = t;
        waves = g;
      }
    }
  }
  return (waves + WAVES - 1) / WAVES;
}

int run_forward(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float* yhat, float* c1,
                float* s1, float* c2, float* s2, bool eval) {
  const int blocks = blocks_for(ctx, B, true);
  const DumpPtrs dump = {c1, s1, c2, s2};
  if (c1 || s1 || c2 || s2)
    forward_kernel<kForwardDump><<<blocks, 64 * WAVES, 0, ctx->stream>>>(images, labels, B, ctx->tabg, yhat,
                                                                          dump, nullptr);
  else
    forward_kernel<kForward><<<blocks, 64 * WAVES, 0, ctx->stream>>>(images, labels, B, ctx->tabg, yhat, dump,
                                                                      eval ? ctx->eval_partial : nullptr);
  if (hipGetLastError() != hipSuccess) return CNN_EHIP;
  return blocks * WAVES;
}

int run_backward(cnn_ctx* ctx, const float* images, const int32_t* labels, int B, float scale,
                 float* grad_out, float* loss_sum) {
  const bool grouped = B <= GROUP_MAX_BATCH;
  // small batches: one workgroup per image; large ones: one workgroup of eight waves per compute unit
  const int blocks = grouped ? B : (B < TRAIN_BLOCKS ? B : TRAIN_BLOCKS);
  const int G = blocks;  // one partial row per workgroup in both kernels
  const bool timed = (size_t)(2 * ctx->ev_used + 1) < ctx->ev.size();
  if (timed) CNN_HIP_TRY(hipEventRecord(ctx->ev[2 * ctx->ev_used], ctx->stream));
  if (grouped)
    train_group_kernel<<<blocks, 64 * GWAVES, 0, ctx->stream>>>(images, labels, B, ctx->tabg, ctx->partial);
  else
    train_kernel<<<blocks, 64 * TWAVES, 0, ctx->stream>>>(images, labels, B, ctx->tabg, ctx->partial, ctx->fc_hist);
  if (hipGetLastError() != hipSuccess) return CNN_EHIP;
  if (timed) {
    CNN_HIP_TRY(hipEventRecord(ctx->ev[2 * ctx->ev_used + 1], ctx->stream));
    ++ctx->ev_used;
  }
  reduce_update_kernel<<<PSTRIDE / 64, 64 * RSTRANDS, 0, ctx->stream>>>(ctx->partial, G, scale, ctx->w, ctx->dest,
                                                              ctx->tabg, grad_out, loss_sum);
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
    case CNN_ESCRATCH: return "the problem needs more than the library's built-in scratch buffer";
    case CNN_ETIMEOUT: return "a wait between workgroups of the device-side epoch loop was given up";
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
  expand_kernel<<<(TABG_FLOATS + 255) / 256, 256, 0, ctx->stream>>>(ctx->w, ctx->tabg);
  return hipGetLastError() == hipSuccess ? CNN_OK : CNN_EHIP;
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
  ctx->fwd_gcap = gcap_for(max_batch, FWD_GCAP);
  ctx->w = reinterpret_cast<float*>(base + l.w);
  ctx->tabg = reinterpret_cast<float*>(base + l.tabg);
  ctx->dest = reinterpret_cast<int32_t*>(base + l.dest);
  ctx->partial = reinterpret_cast<float*>(base + l.partial);
  ctx->eval_partial = reinterpret_cast<float*>(base + l.eval_partial);
  ctx->fc_hist = reinterpret_cast<float*>(base + l.fc_hist);
  ctx->sync = reinterpret_cast<unsigned*>(base + l.sync);
  ctx->wait_ticks = 100000000ll;  // one second
  {
    // inverse of table_source: where each parameter sits in the expanded table
    static_assert(TABLE_MAX_DEST == 4 && table_max_multiplicity() <= TABLE_MAX_DEST,
                  "the update kernel reads a parameter's table slots as one int4");
    std::vector<int32_t> dest(TABLE_MAX_DEST * PSTRIDE, -1);
    for (int i = 0; i < TABG_FLOATS; ++i) {
      const int p = table_source(i);
      if (p < 0) continue;
      int k = 0;
      while (dest[TABLE_MAX_DEST * p + k] >= 0) ++k;  // < TABLE_MAX_DEST by the assertion above
      dest[TABLE_MAX_DEST * p + k] = i;
    }
    // synchronous copy: the host vector may go away as soon as the call returns
    if (hipMemcpy(ctx->dest, dest.data(), sizeof(int32_t) * dest.size(), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemsetAsync(ctx->w, 0, sizeof(float) * PSTRIDE, ctx->stream) != hipSuccess ||
        hipMemsetAsync(ctx->sync, 0, sizeof(unsigned) * SYNC_WORDS, ctx->stream) != hipSuccess) {
      (void)hipGetLastError();
      delete ctx;
      return CNN_EHIP;
    }
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
  eval_reduce_kernel<<<1, EVAL_REDUCE_THREADS, 0, ctx->stream>>>(ctx->eval_partial, G, n_correct, loss_sum);
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

int cnn_train_epoch(cnn_ctx* ctx, const float* images, const int32_t* labels, int N, int batch, float lr,
                    float* loss_sums) {
  if (!ctx || N < 1 || !batch_ok(ctx, batch) || !images || !labels || !aligned16(images)) return CNN_EINVAL;
  int first = 0, k = 0;
  if (ctx->epoch_mode == 1 && batch <= EPOCH_MAX_BATCH && N >= batch) {
    // the whole steps as ONE kernel, if all its workgroups can be resident at once
    if (ctx->resident_limit < 0) {
      int per_cu = 0, dev = 0, cus = 0;
      CNN_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, train_epoch_kernel, 64 * GWAVES, 0));
      CNN_HIP_TRY(hipGetDevice(&dev));
      CNN_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
      ctx->resident_limit = per_cu * cus;
    }
    const int steps = N / batch;
    if (batch <= ctx->resident_limit && ctx->barrier_count < 0x7f000000u - 2u * (unsigned)steps) {
      train_epoch_kernel<<<batch, 64 * GWAVES, 0, ctx->stream>>>(
          images, labels, steps, lr / (float)batch, ctx->w, ctx->dest, ctx->tabg, ctx->partial, loss_sums,
          ctx->sync, ctx->sync + SYNC_ERROR, ctx->barrier_count, ctx->wait_ticks, ctx->phantom);
      if (hipGetLastError() != hipSuccess) return CNN_EHIP;
      ctx->barrier_count += 2u * (unsigned)steps;
      first = steps * batch;
      k = steps;
    }
  }
  for (; first < N; ++k, first += batch) {
    const int B = N - first < batch ? N - first : batch;
    const int rc = run_backward(ctx, images + (size_t)first * NI, labels + first, B, lr / (float)B, nullptr,
                                loss_sums ? loss_sums + k : nullptr);
    if (rc != CNN_OK) return rc;
  }
  return CNN_OK;
}

int cnn_epoch_mode(cnn_ctx* ctx, int device_loop, double wait_seconds, int never_arrives) {
  if (!ctx || (device_loop != 0 && device_loop != 1) || !(wait_seconds >= 0.0) || wait_seconds > 3600.0)
    return CNN_EINVAL;
  ctx->epoch_mode = device_loop;
  ctx->wait_ticks = (long long)(wait_seconds * 1e8);
  ctx->phantom = never_arrives ? SYNC_PHANTOM : -1;
  return CNN_OK;
}

int cnn_epoch_status(cnn_ctx* ctx) {
  if (!ctx) return CNN_EINVAL;
  unsigned err = 0;
  CNN_HIP_TRY(hipMemcpyAsync(&err, ctx->sync + SYNC_ERROR, sizeof(err), hipMemcpyDeviceToHost, ctx->stream));
  CNN_HIP_TRY(hipStreamSynchronize(ctx->stream));
  if (err == 0) return CNN_OK;
  // start over: the flags of a kernel that gave up hold different counts
  CNN_HIP_TRY(hipMemsetAsync(ctx->sync, 0, sizeof(unsigned) * SYNC_WORDS, ctx->stream));
  ctx->barrier_count = 0;
  return CNN_ETIMEOUT;
}

}  // extern "C"
