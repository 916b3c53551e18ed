// Small-batch form of the fused step: EIGHT WAVEFRONTS (two per SIMD of a compute unit) SHARE ONE
// IMAGE.  Same arithmetic, same operand table, same LDS arrays and the same MFMA formulations as
// cnn_wave.h (arXiv 1912.05234, Section 3); only the division of labour differs, to cut the latency
// of a single image when there are too few images to give every SIMD its own.  Two waves per SIMD
// because one wave alone issues a vector instruction only every ~5 cycles, two reach ~2.4.
//
//   C1 forward and C1 error      GEMM tiles T = wave, wave + 8 (waves 0, 1 also T = wave + 16), cnn_wave.h
//   C1 weight gradient           the GEMM's K steps that belong to the wave's own C1 tiles
//   C2 forward, C2 error         waves 0..3: pixel tile mt = wave
//   output layer                 outputs o = wave and wave + 8
//   FC weight gradient           waves 0..2 take the three 4-output row tiles
//   C2 input error (col2im)      waves 0..3: input maps 4 cg .. 4 cg + 3, cg = wave % 2, and pixel tiles
//                                nt = 2 h, 2 h + 1, h = wave / 2; half h adds into its own copy of d_s1,
//                                so no two waves ever touch the same cell; the C1 error reads both copies
//   C2 weight gradient           waves 4..7: tap tiles nt = 0-1, 2-3, 4-6, 7-9 over all 64 pixels (each wave
//                                owns whole columns of the result, so nothing has to be added across waves)
//
// Phases that hand data between waves are separated by workgroup barriers (six, plus one in the
// final cross-wave sums).  A workgroup handles exactly one image: the grid is one workgroup per
// image of the batch.
#pragma once

#include "cnn_wave.h"

namespace cnn {

constexpr int GWAVES = 8;  // waves per workgroup of the small-batch kernel
// Second col2im target: [6][12][12] plus the cells behind it that the rows of the padding maps 6, 7
// rewrite with themselves (+ 0.0), as they do behind the first target inside TrainLds.
constexpr int D_S1B_FLOATS = NS1 + 304;

// Tap tiles of the C2 weight gradient owned by wave 4 + i: first tile and count.
__host__ __device__ constexpr int k2_first(int i) { return i < 2 ? 2 * i : 3 * i - 2; }
__host__ __device__ constexpr int k2_count(int i) { return i < 2 ? 2 : 3; }

struct GroupState {
  float bias2;      // b2[n16]
  f4 acc_k2[3];     // waves 4..7: C2 weight gradient tiles nt = k2_first(wave - 4) + k
  f4 acc_k1[2];     // C1 weight gradient GEMM over the K steps of this wave's tiles, T[(m,sh)][c]
  f4 acc_fc[3];     // waves 0..2: FC weight gradient rows o = 4 wave + r, columns lane + 64 k
  float g_bq;       // waves 0..2: FC bias gradient b[4 wave + lane % 4]
  float g_b1[2];    // C1 bias gradient of maps 2q, 2q + 1 over this lane's pixels
  float g_b2, loss;
};

// C1 forward + S1 for this wave's NT tiles T = wave + 8 k of the C1 GEMM (cnn_wave.h): returns the
// activations in c1[k].  All MFMAs first (two independent chains at a time), then the sigmoids and
// the pooling.
template <int NT>
__device__ __forceinline__ void group_c1_forward(TrainLds& s, const OperandTable<TAB_TRAIN_ENTRIES>& tab, int wave,
                                                 const C1Lane& ln, f4 (&c1)[3]) {
  const int l = threadIdx.x & 63, q = l >> 4;
  float wa[C1F_KSTEPS];
#pragma unroll
  for (int ks = 0; ks < C1F_KSTEPS; ++ks) wa[ks] = tab.e[(TAB_C1A + ks) * 64 + l];
  f4 binit = f4{0.0f, 0.0f, 0.0f, 0.0f};
  if (q < 3) {
    const float2 bq = *reinterpret_cast<const float2*>(&tab.bias[TAB_BIAS_B1 + 2 * q]);
    binit = f4{bq.x, bq.x, bq.y, bq.y};
  }
  c1f_gemm_pair(wa, ln, s.img + c1f_tile_img(wave), s.img + c1f_tile_img(wave + 8), binit, c1[0], c1[1]);
  if (NT == 3) c1f_gemm_one(wa, ln, s.img + c1f_tile_img(wave + 16), binit, c1[2]);
#pragma unroll
  for (int k = 0; k < NT; ++k) c1f_finish(c1[k], ln, s.pool + P_S1 + c1f_tile_s1(wave + 8 * k));
}

// C1 error of this wave's tiles into the staged d1[6][24][24]; the error at S1 is the sum of the two
// col2im copies.  Lanes q = 3 hold padding rows.
template <int NT>
__device__ __forceinline__ void group_c1_error(GroupState& st, TrainLds& s, const float* d_s1b, int wave,
                                               const C1Lane& ln, const f4 (&c1)[3]) {
  const int q = (threadIdx.x & 63) >> 4;
  if (q < 3) {
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      const int T = wave + 8 * k, o = ln.s1 + c1f_tile_s1(T);
      // (the average pooling's 1/4 is in the col2im operand of the table)
      const float up0 = s.d_s1[o] + d_s1b[o], up1 = s.d_s1[o + 144] + d_s1b[o + 144];
      const f4 c = c1[k];
      const float2 da = float2{up0 * c[0] * (1.0f - c[0]), up0 * c[1] * (1.0f - c[1])};
      const float2 db = float2{up1 * c[2] * (1.0f - c[2]), up1 * c[3] * (1.0f - c[3])};
      st.g_b1[0] += da.x + da.y;
      st.g_b1[1] += db.x + db.y;
      float* dst = s.pool + ln.c1 + c1f_tile_c1(T);
      *reinterpret_cast<float2*>(dst) = da;
      *reinterpret_cast<float2*>(dst + D1_MAP) = db;
    }
  }
}

// C2 weight gradient for COUNT tap tiles over all four pixel tiles: sixteen K steps in one straight
// line (no branches), so that the operand reads of later steps are issued under the MFMAs of
// earlier ones.  bsrc[k] points at the lane's tap of tile k in s1.
template <int COUNT>
__device__ __forceinline__ void group_k2_gradient(f4 (&acc)[3], const TrainLds& s, const float* const (&bsrc)[3]) {
  const int l = threadIdx.x & 63, q = l >> 4, n16 = l & 15;
  f4 a[4];
#pragma unroll
  for (int S = 0; S < 4; ++S) a[S] = *reinterpret_cast<const f4*>(&s.pool[P_D2 + n16 * D2S + 16 * S + 4 * q]);
#pragma unroll
  for (int step = 0; step < 16; ++step) {
    const int S = step >> 2, r = step & 3, off = 24 * S + 12 * (r >> 1) + (r & 1);
#pragma unroll
    for (int k = 0; k < COUNT; ++k) acc[k] = mfma16(a[S][r], bsrc[k][off], acc[k]);
  }
}

// A value of the partial row.  COHERENT (the device-side epoch loop, where other compute units read
// the row during the same kernel): an agent-scope store, written through to memory.
template <bool COHERENT>
__device__ __forceinline__ void put_row(float* p, float v) {
  if (COHERENT)
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    *p = v;
}

// The whole step for the workgroup's image (`image`, `label` point at it); one partial row, `out`.
// `d_s1b` is the second col2im target (D_S1B_FLOATS floats), `ybuf` 16 floats of LDS for the network
// output.  COHERENT: see put_row and TableLoad.
template <bool COHERENT>
__device__ __forceinline__ void group_train(const float* __restrict__ image,
                                            const int32_t* __restrict__ label_ptr,
                                            const float* __restrict__ tabg, float* __restrict__ out,
                                            OperandTable<TAB_TRAIN_ENTRIES>& tab, TrainLds& s, float* d_s1b,
                                            float* ybuf) {
  const int t = threadIdx.x, wave = t >> 6, l = t & 63, q = l >> 4, n16 = l & 15, sub = l & 3;
  const int pp = 12 * ((n16 & 3) >> 1) + 2 * (n16 >> 2) + (n16 & 1);
  const float* tl = tab.e + l;
  const int pix = t < NI / 4 ? t : 0;  // the 16-byte piece of the image this thread moves
  CNN_GROUP_MARK(0);

  f4 px = reinterpret_cast<const f4*>(image)[pix];
  const int label = *label_ptr;  // in flight during the set-up too
  // the C1 forward operands (the table's last entries) and the biases come first: see barrier (1)
  TableLoad<TAB_TRAIN_ENTRIES, 64 * GWAVES, COHERENT, TAB_TRAIN_ENTRIES, TAB_C1A> table;
  table.fetch(tabg);
  // every LDS cell that padded GEMM steps may read starts finite, and both col2im targets start at
  // zero (the image area is written below, before the first barrier, so it is left alone here)
  for (int e = t; e < D_S1B_FLOATS / 4; e += 64 * GWAVES) {
    if (e < NS1 / 4) reinterpret_cast<f4*>(s.d_s1)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    reinterpret_cast<f4*>(d_s1b)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  }
  for (int e = t; e < POOL_FLOATS / 4; e += 64 * GWAVES) reinterpret_cast<f4*>(s.pool)[e] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  GroupState st;
  const C1Lane ln = c1f_lane();
#pragma unroll
  for (int k = 0; k < 3; ++k) st.acc_k2[k] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  st.acc_k1[0] = st.acc_k1[1] = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int k = 0; k < 3; ++k) st.acc_fc[k] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  st.g_bq = 0.0f;
  st.g_b1[0] = st.g_b1[1] = 0.0f;
  st.g_b2 = 0.0f;
  st.loss = 0.0f;
  CNN_GROUP_MARK(1);
  // The lane-invariant address arithmetic of the phases below is independent of the table, so the
  // compiler is free to run it while the table's loads are still in flight; barrier (1) publishes
  // the image together with what the C1 forward pass reads of the table (its own operands and the
  // biases, fetched first); the rest of the table arrives during that pass and is published by
  // barrier (2).
  {
    table.commit_first(tab);
    if (t < NI / 4) reinterpret_cast<f4*>(s.img)[t] = px;
    CNN_GROUP_MARK(2);
    __syncthreads();  // (1) image, C1 forward operands and biases in LDS
    st.bias2 = tab.bias[n16];

    // ---- C1 forward + S1 for this wave's tiles ---------------------------------------------------------
    f4 c1[3];
    if (wave < 2)
      group_c1_forward<3>(s, tab, wave, ln, c1);
    else
      group_c1_forward<2>(s, tab, wave, ln, c1);
    table.commit_rest(tab);
    CNN_GROUP_MARK(3);
    __syncthreads();  // (2) S1 and the operand table complete

    // ---- C2 forward for pixel tile mt = wave, S2 (waves 0..3) -----------------------------------------
    f4 c2v = f4{st.bias2, st.bias2, st.bias2, st.bias2};
    if (wave < 4) {
      const float* a12 = s.pool + P_S1 + pp + 12 * q + 24 * wave;
      const float* a1 = s.pool + P_S1 + pp + q + 24 * wave;
      const float* a144 = s.pool + P_S1 + pp + 144 * q + 24 * wave;
      // operands of step s + AHEAD are read while step s issues: an LDS read takes longer than three
      // matrix instructions, and with eight waves per image there are registers to spare
      constexpr int AHEAD = 6, SLOTS = 8;
      float opa[SLOTS], opw[SLOTS];
      auto load_step = [&](int sidx, float& oa, float& ow) {
        const float* base = sidx < 30 ? a12 : sidx < 36 ? a1 : a144;
        ow = tl[(TAB_BF + sidx) * 64];
        oa = base[fwd_imm(sidx)];
      };
#pragma unroll
      for (int sidx = 0; sidx < AHEAD; ++sidx) load_step(sidx, opa[sidx], opw[sidx]);
      // even and odd K steps in two sums: a matrix instruction waits for the previous one of its own
      // chain only
      f4 odd = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int sidx = 0; sidx < 38; ++sidx) {
        if (sidx + AHEAD < 38) load_step(sidx + AHEAD, opa[(sidx + AHEAD) % SLOTS], opw[(sidx + AHEAD) % SLOTS]);
        if (sidx & 1)
          odd = mfma16(opa[sidx % SLOTS], opw[sidx % SLOTS], odd);
        else
          c2v = mfma16(opa[sidx % SLOTS], opw[sidx % SLOTS], c2v);
        if (sidx + AHEAD < 38) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) c2v[r] = logistic_of_scaled(c2v[r] + odd[r]);
      if (n16 < 12) s.pool[P_S2 + n16 * 16 + 4 * wave + q] = 0.25f * ((c2v[0] + c2v[1]) + (c2v[2] + c2v[3]));
    }
    CNN_GROUP_MARK(4);
    __syncthreads();  // (3) S2 complete

    // ---- output layer: this wave's outputs o = wave, wave + 8 -----------------------------------------
    float sv[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) sv[k] = s.pool[P_S2 + l + 64 * k];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int o = wave + GWAVES * j;  // wave-uniform
      if (o < NY) {
        float p = tl[(TAB_FCW + 3 * o) * 64] * sv[0];
        p = fmaf(tl[(TAB_FCW + 3 * o + 1) * 64], sv[1], p);
        p = fmaf(tl[(TAB_FCW + 3 * o + 2) * 64], sv[2], p);
        const float yo = logistic(wave_sum(p) + tab.bias[TAB_BIAS_B + o]);
        if (l == 0) ybuf[o] = yo;
      }
    }
    CNN_GROUP_MARK(5);
    __syncthreads();  // (4) yhat complete
    if (wave < 4) {
      float delta[10];
      {
        float lsum = 0.0f;
#pragma unroll
        for (int o = 0; o < 10; ++o) {
          const float yo = ybuf[o];
          const float e = yo - (o == label ? 1.0f : 0.0f);
          lsum = fmaf(e, e, lsum);
          delta[o] = e * yo * (1.0f - yo);
        }
        if (wave == 0) st.loss = fmaf(0.5f, lsum, st.loss);
      }
      if (wave < 3) {  // FC backweights / backbias, row tile mt = wave
        float d[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float v = 0.0f;
#pragma unroll
          for (int mt = 0; mt < 3; ++mt)
            if (4 * mt + r < 10) v = wave == mt ? delta[4 * mt + r] : v;
          d[r] = v;
        }
        const float aq = (sub & 2) ? ((sub & 1) ? d[3] : d[2]) : ((sub & 1) ? d[1] : d[0]);
        st.g_bq += aq;
#pragma unroll
        for (int k = 0; k < 3; ++k) st.acc_fc[k] = mfma4(aq, sv[k], st.acc_fc[k]);
      }
      // ---- error at C2 for this wave's tile: the lane's own element of the error at S2,
      //      d_s2[i] = sum_o fc[o][i] delta[o] with i = 16 n16 + 4 wave + q, then backavgpool and sigmoid' --
      {
        const int i = n16 * 16 + 4 * wave + q;
        const float* fcw = tab.e + (TAB_FCW + (i >> 6)) * 64 + (i & 63);
        float up = 0.0f;
#pragma unroll
        for (int o = 0; o < 10; ++o) up = fmaf(fcw[3 * o * 64], delta[o], up);
        up *= 0.25f;
        f4 d2v;
#pragma unroll
        for (int r = 0; r < 4; ++r) d2v[r] = n16 < 12 ? up * c2v[r] * (1.0f - c2v[r]) : 0.0f;
        *reinterpret_cast<f4*>(&s.pool[P_D2 + n16 * D2S + 16 * wave + 4 * q]) = d2v;
        st.g_b2 += (d2v[0] + d2v[1]) + (d2v[2] + d2v[3]);
      }
    }
    CNN_GROUP_MARK(6);
    __syncthreads();  // (5) d_c2 complete

    if (wave < 4) {
      // ---- C2 input error for input maps 4 cg .. 4 cg + 3 from the pixel tiles nt = 2 h, 2 h + 1
      //      (col2im rounds of cnn_wave.h restricted to those tiles: levels 4 h .. 4 h + 6) ---------------
      const int cg = wave & 1, h = wave >> 1;
      float bd[3][2];
#pragma unroll
      for (int sidx = 0; sidx < 3; ++sidx)
#pragma unroll
        for (int j = 0; j < 2; ++j) bd[sidx][j] = s.pool[P_D2 + (4 * sidx + q) * D2S + 16 * (2 * h + j) + n16];
      const float* ta = tl + (cg ? TAB_AB1 : TAB_AB) * 64;
      f4 t4[2];
      float t44[2];
      {
        float au[3], ac[3];
#pragma unroll
        for (int sidx = 0; sidx < 3; ++sidx) {
          au[sidx] = ta[(kTileU4 * 3 + sidx) * 64];
          ac[sidx] = ta[(kTileC * 3 + sidx) * 64];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          f4 a = f4{0.0f, 0.0f, 0.0f, 0.0f}, c = a;
#pragma unroll
          for (int sidx = 0; sidx < 3; ++sidx) {
            a = mfma16(au[sidx], bd[sidx][j], a);
            c = mfma16(ac[sidx], bd[sidx][j], c);
          }
          t4[j] = a;
          t44[j] = c[0];
        }
      }
      float* tgt = (h ? d_s1b : s.d_s1) + 144 * q + pp + 576 * cg + 48 * h;
#pragma unroll
      for (int v = 0; v < 5; ++v) {
        f4 tv[2];
        {
          float av[3];
#pragma unroll
          for (int sidx = 0; sidx < 3; ++sidx) av[sidx] = ta[((kTileV0 + v) * 3 + sidx) * 64];
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            f4 a = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int sidx = 0; sidx < 3; ++sidx) a = mfma16(av[sidx], bd[sidx][j], a);
            tv[j] = a;
          }
        }
        const float tu4[2] = {v < 4 ? t4[0][v < 4 ? v : 0] : t44[0], v < 4 ? t4[1][v < 4 ? v : 0] : t44[1]};
        {  // even levels 2 (2 h + mm), mm < 4: (j = mm, u = 0) + (mm - 1, 2) + (mm - 2, 4)
          const float e[4] = {tv[0][0], tv[1][0] + tv[0][2], tv[1][2] + tu4[0], tu4[1]};
          float old[4];
#pragma unroll
          for (int mm = 0; mm < 4; ++mm) old[mm] = tgt[24 * mm + v];
#pragma unroll
          for (int mm = 0; mm < 4; ++mm) tgt[24 * mm + v] = old[mm] + e[mm];
        }
        wave_sync();
        {  // odd levels 2 (2 h + mm) + 1, mm < 3: (j = mm, u = 1) + (mm - 1, 3)
          const float e[3] = {tv[0][1], tv[1][1] + tv[0][3], tv[1][3]};
          float old[3];
#pragma unroll
          for (int mm = 0; mm < 3; ++mm) old[mm] = tgt[24 * mm + 12 + v];
#pragma unroll
          for (int mm = 0; mm < 3; ++mm) tgt[24 * mm + 12 + v] = old[mm] + e[mm];
        }
        wave_sync();
      }
    } else {
      // ---- C2 weight gradient: this wave's tap tiles over all four pixel tiles ---------------------------
      const int first = k2_first(wave - 4), count = k2_count(wave - 4);  // wave-uniform
      const float* bsrc[3];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const int tap = 16 * (first + (k < count ? k : 0)) + n16;
        const int c = tap / 25, rem = tap - 25 * c, u = rem / 5, v = rem - 5 * u;
        bsrc[k] = s.pool + P_S1 + (tap < 150 ? c * 144 + u * 12 + v : 0) + 2 * q;
      }
      if (count == 3)
        group_k2_gradient<3>(st.acc_k2, s, bsrc);
      else
        group_k2_gradient<2>(st.acc_k2, s, bsrc);
    }
    CNN_GROUP_MARK(7);
    __syncthreads();  // (6) both d_s1 copies complete; s1, d_c2 no longer needed

    // ---- C1 error for this wave's tiles, then the K steps of the C1 weight gradient GEMM that belong
    //      to the same tiles: a wave reads only the d1 cells it staged itself, so no barrier -------------
    const float* d1t[3];
    const float* imgt[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int T = wave + 8 * k < C1F_TILES ? wave + 8 * k : wave;
      d1t[k] = s.pool + c1f_tile_c1(T);
      imgt[k] = s.img + c1f_tile_img(T);
    }
    if (wave < 2) {
      group_c1_error<3>(st, s, d_s1b, wave, ln, c1);
      wave_sync();
      c1g_accumulate_tiles<3>(st.acc_k1, d1t, imgt);
    } else {
      group_c1_error<2>(st, s, d_s1b, wave, ln, c1);
      wave_sync();
      c1g_accumulate_tiles<2>(st.acc_k1, d1t, imgt);
    }
    CNN_GROUP_MARK(8);
  }

  // ---- one partial row per workgroup: cross-wave sums through LDS in a fixed order -------------------
  // Nothing has read the operand table since barrier (6); its storage takes the parked values.
  float* k1s = tab.e;                               // [8 waves][16][32]: parked C1 weight GEMM results
  float* b1s = tab.e + GWAVES * C1G_PARK;           // [8 waves][8]: C1 bias sums (256 floats reserved)
  float* b2s = b1s + 256;                           // [4 waves][64]: per-lane C2 bias sums
  static_assert(GWAVES * C1G_PARK + 256 + 256 <= TAB_TRAIN_ENTRIES * 64, "flush scratch fits the table");
  c1g_park(st.acc_k1, k1s + wave * C1G_PARK);
  CNN_GROUP_MARK(11);
#pragma unroll
  for (int k = 0; k < 2; ++k) {  // C1 biases: lanes (q, .) hold maps 2q, 2q + 1
    float v = st.g_b1[k];
    v += quad_xor1(v);
    v += quad_xor2(v);
    v += dpp_row_half_mirror(v);
    v += dpp_row_mirror(v);
    if (n16 == 0 && q < 3) b1s[wave * 8 + 2 * q + k] = v;
  }
  if (wave < 4) b2s[wave * 64 + l] = st.g_b2;  // lane (q, j) of this wave's pixel tile
  CNN_GROUP_MARK(9);
  __syncthreads();
  CNN_GROUP_MARK(12);
  // (stores grouped by the lanes that take part: one branch per group, not one per store)
  if (wave >= 4) {  // C2 weights: every wave stores the columns (tap tiles) it owns; rows j = 4 q + r < 12
    const int first = k2_first(wave - 4), count = k2_count(wave - 4);
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int tap = 16 * (first + k) + n16;
      if (k < count && q < 3 && tap < 150) {
        float* dst = out + OFF_K2 + 4 * q * 150 + tap;
#pragma unroll
        for (int r = 0; r < 4; ++r) put_row<COHERENT>(dst + r * 150, st.acc_k2[k][r]);
      }
    }
  }
  if (wave < 3) {  // FC rows o = 4 wave + r < 10: wave 2 has two
    float* dst = out + OFF_FC + 4 * wave * NS2 + l;
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
      for (int r = 0; r < 2; ++r) put_row<COHERENT>(dst + r * NS2 + 64 * k, st.acc_fc[k][r]);
    if (wave < 2) {
#pragma unroll
      for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int r = 2; r < 4; ++r) put_row<COHERENT>(dst + r * NS2 + 64 * k, st.acc_fc[k][r]);
    }
    if (l < 4 && 4 * wave + l < 10) put_row<COHERENT>(out + OFF_B + 4 * wave + l, st.g_bq);
  }
  CNN_GROUP_MARK(13);
  if (wave >= 6 || (wave == 3 && l >= 32)) {
    // one thread per C1 weight (waves 6, 7 have nothing else to store; 22 lanes of wave 3 take the
    // rest): the eight waves' shares of the GEMM, both shifted halves
    const int e = wave >= 6 ? t - 384 : 96 + l;
    if (e < 150) {
      float x[GWAVES];
#pragma unroll
      for (int k = 0; k < GWAVES; ++k) x[k] = c1g_combine(k1s + k * C1G_PARK, e);
      put_row<COHERENT>(out + OFF_K1 + e, ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7])));
    }
  }
  if (wave == 3) {
    if (l < 6) {  // C1 biases: the eight waves' sums
      float x[GWAVES];
#pragma unroll
      for (int k = 0; k < GWAVES; ++k) x[k] = b1s[k * 8 + l];
      put_row<COHERENT>(out + OFF_B1 + l, ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7])));
    } else if (l >= 16 && l < 28) {  // C2 biases: 4 waves x 4 lane quarters
      const int j = l - 16;
      float x[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) x[k] = b2s[k * 16 + j];
#pragma unroll
      for (int k = 0; k < 16; k += 4) x[k] = (x[k] + x[k + 1]) + (x[k + 2] + x[k + 3]);
      put_row<COHERENT>(out + OFF_B2 + j, (x[0] + x[4]) + (x[8] + x[12]));
    }
  }
  if (t == 0) put_row<COHERENT>(out + LOSS_SLOT, st.loss);
  CNN_GROUP_MARK(10);
}

}  // namespace cnn
