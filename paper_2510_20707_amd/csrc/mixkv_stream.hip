// The two kernels that stream the cache: window-attention statistics + key/value statistics
// (stats_kernel) and the normalised attention column sums + diversity dot products (attn_kernel).
//
// Both are MFMA kernels built the same way.  A workgroup walks runs of consecutive key chunks of
// one unit (one layer, batch item and KV head).  The G*W window-query rows are split into tiles of
// 32 and every wave keeps its TQ tiles in registers for the whole run ("query-stationary"); the
// keys (and values) stream through LDS: tiles of 32 rows are fetched with direct global->LDS loads
// (whole rows, bank-rotated) into a ring of tile images, a few tile steps ahead of their use.
//
// Fragment form.  The contraction index d of Q.K^T may be visited in any order as long as both
// operands agree, so a lane (key or row = lane % 32, half = lane / 32) simply owns every other
// 16-byte piece of its row: piece c of the lane covers elements [(2c + half) * EPC, +EPC) with
// EPC = 8 (bf16) or 4 (f32).  One piece feeds one v_mfma_f32_32x32x16_bf16 (or four
// v_mfma_f32_32x32x2f32).  The same registers serve as the A or the B operand, which lets the
// first kernel put keys on the output rows (softmax statistics stay inside a lane) and the second
// put keys on the output columns (the sum over query rows stays inside a lane).
//
// Softmax runs in the log2 domain: x = (q.k) * softmax_scale * log2(e), weights are exp2(x - b_r)
// with b_r = max_r + log2(sum_r * G*W), so one fused multiply-add and one v_exp_f32 per element
// give the weight already divided by the row sum and by the number of rows
// (paper Sec. 3.2, extrinsic importance: mean over the window queries of the attention weights).
#include "mixkv_stream.h"

namespace mixkv {

// ------------------------------------------------------------------------------------------------
// stats_kernel: first pass over K (and the only pass over V).
//   * running softmax (max, sum) of every window-query row over the run's keys: keys on the MFMA
//     output rows, query rows on the columns, so a lane follows one query row per tile;
//   * 1/|K_i| and the partial sum of the normalised keys (paper Sec. 3.2 diversity metrics,
//     Sec. 3.3 Eq. 3-4: only the sum of normalised keys is needed, never the T x T matrix);
//   * |V_i| (Sec. 3.2, VNorm intrinsic importance).
// Per-run partials go to the workspace; fold_kernel folds them per unit.
// With GIVEN_LSE the caller already has the softmax normalisers of the window rows (the prefill
// attention produced them), so the kernel takes no queries and only the key and value statistics
// remain: a plain streaming pass.
// ------------------------------------------------------------------------------------------------
// Waves per SIMD the register allocation of stats_kernel aims at: two workgroups per compute unit
// where their two rings fit in LDS together (tiles of up to 8 KB), one otherwise.
__host__ __device__ constexpr int stats_waves_per_simd(int dtype, int D, int waves, int tq) {
  const int tile_bytes = D * (dtype == MIXKV_BF16 ? 2 : 4) * 32;
  const int wgs = (tile_bytes <= 8192 && !(waves == 8 && tq == 2)) ? 2 : 1;   // 8 waves x 2 tiles need 256 registers
  return waves / 4 * wgs;
}

template <int DT, int D, int WAVES, int TQ, bool GIVEN_LSE = false>
__global__ __launch_bounds__(WAVES * 64, stats_waves_per_simd(DT, D, WAVES, TQ)) void stats_kernel(
    Shape s, LayerInTable in, char *ws, Workspace w, int64_t unit0, int nunits, int64_t slot0) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), PPR = D * EB / 16;
  constexpr int NT = WAVES * 64, KT = chunk_tiles(DT, D), TILE = 32 * PPR;
  constexpr int VPT = (TILE + NT - 1) / NT;               // V pieces per thread and key tile
  constexpr int KL = (TILE / 64 + WAVES - 1) / WAVES;     // requests per wave, tile and tensor
  __shared__ uint4 kring[kRing * TILE], vring[kRing * TILE];
  __shared__ float ks_s[WAVES * D];

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps its address math scalar
  const int N = s.N, Nc = s.Nc, QTR = s.QT * 32;
  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;      // keys <= this are visible to every row
  const int nq = GIVEN_LSE ? 0 : max(0, min(TQ, s.QT - wave * TQ));  // query tiles this wave owns
  const bool use_v = s.intrinsic == MIXKV_INTRINSIC_VNORM;
  const bool use_k = s.kstats != 0;                  // key norms and the sum of normalised keys have a reader
  // bf16 heads that leave the last wave without a query tile: that wave takes the value norms (see the tile step)
  const bool v_by_last = DT == MIXKV_BF16 && !GIVEN_LSE && s.QT <= (WAVES - 1) * TQ;
  // Waves without a query tile (the workgroup has more tile slots than the head has tiles, or the
  // normalisers are given) run no matrix or softmax work.
  const uint32_t kring_a = lds_base_of(kring), vring_a = lds_base_of(vring);
  const int64_t T = (int64_t)nunits * s.nchunks;
  int64_t item = wg_first_item(blockIdx.x, gridDim.x, T);
  const int64_t item_end = wg_first_item(blockIdx.x + 1, gridDim.x, T);

  while (item < item_end) {
    const int ul = (int)(item / s.nchunks), c0 = (int)(item - (int64_t)ul * s.nchunks);
    const int nit = (int)min((int64_t)(s.nchunks - c0), item_end - item);
    const int64_t unit = unit0 + ul;
    const UnitCoord uc = unit_coord(s, ul);
    const LayerIn L = in.l[uc.layer];
    const int64_t head_off = ((int64_t)uc.b * L.sb + (int64_t)uc.h * L.sh) * EB;
    const char *Kb = reinterpret_cast<const char *>(L.K) + head_off;
    const char *Vb = reinterpret_cast<const char *>(L.V) + head_off;
    const char *Qb = reinterpret_cast<const char *>(L.Q) + ((int64_t)(uc.b * s.hq + uc.h * s.G) * s.W * D) * EB;
    const int64_t row_bytes = L.sn * EB;
    float *invnorm = reinterpret_cast<float *>(ws + w.invnorm) + unit * s.Npad;
    float *vnorm = reinterpret_cast<float *>(ws + w.vnorm) + unit * s.Npad;
    const int key0 = c0 * KT * 32;                                   // first key of the run
    const int nt = min(nit * KT, (N - key0 + 31) / 32);              // tiles of the run that hold keys

    // Request tile tr of the run (keys, and values if they are needed) into its ring image.
    const int64_t tile_bytes = 32 * row_bytes;
    auto request = [&](int tr) {
      const int tbr = key0 + tr * 32;
      const uint32_t off = (uint32_t)(tr & (kRing - 1)) * (TILE * 16);
      fetch_tile<DT, D, WAVES>(Kb + tbr * row_bytes, row_bytes, tbr, N, kring_a + off, wave, lane);
      if (use_v) fetch_tile<DT, D, WAVES>(Vb + tbr * row_bytes, row_bytes, tbr, N, vring_a + off, wave, lane);
    };
    // first rows of the tile the next step of the loop requests (tile t + kLead at step t)
    const char *Kreq = Kb + (key0 + kLead * 32) * row_bytes, *Vreq = Vb + (key0 + kLead * 32) * row_bytes;
    lds_barrier();                                     // the previous run is done with LDS
#pragma unroll
    for (int j = 0; j < kLead; ++j)
      if (j < nt) request(j);

    // this wave's query tiles, in fragment form, for the whole run (tiles past QT are zero)
    Frag qf[TQ][NCHK];
    int lim[TQ];
    float m[TQ], l[TQ];
#pragma unroll
    for (int q = 0; q < (GIVEN_LSE ? 0 : TQ); ++q) {
      const int row = (wave * TQ + q) * 32 + l32;
      const bool live = row < s.GW;
      const char *qrow = Qb + ((int64_t)(live ? row : 0) * D) * EB + half * 16;
#pragma unroll
      for (int c = 0; c < NCHK; ++c) {
        uint4 v = *reinterpret_cast<const uint4 *>(qrow + c * 32);
        qf[q][c].q = live ? v : make_uint4(0, 0, 0, 0);
      }
      lim[q] = s.causal ? Nc + row % s.W : N - 1;     // last key this row attends to
      m[q] = -INFINITY;
      l[q] = 0.f;
    }
    // Nothing may be pending when the tile loop is entered: its waits count the requests issued
    // inside it.
    wait_vm<0>();

    // Sum of normalised keys: lane (lrow, lq) adds up piece lq (elements [lq*EPC, +EPC)) of the
    // rows it visits, so nothing crosses lanes before the end of the run.
    float ksacc[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) ksacc[e] = 0.f;

    // One tile step.  The loop is unrolled over the ring, so the ring slot of a step (t mod kRing) is
    // a constant and the LDS addresses of its reads are a loop-invariant lane offset plus an immediate.
    auto tile_step = [&](auto slot_c, int t) {
      constexpr int SLOT = decltype(slot_c)::value;
      __builtin_amdgcn_sched_barrier(0);
      if (use_v) wait_tile<2 * KL>(t, nt); else wait_tile<KL>(t, nt);
      lds_barrier();
      if (t + kLead < nt) {                            // tile t + kLead goes into the image tile t - 1 has left
        constexpr uint32_t off = (uint32_t)((SLOT + kLead) & (kRing - 1)) * (TILE * 16);
        const int tbr = key0 + (t + kLead) * 32;
        fetch_tile<DT, D, WAVES>(Kreq, row_bytes, tbr, N, kring_a + off, wave, lane);
        if (use_v) fetch_tile<DT, D, WAVES>(Vreq, row_bytes, tbr, N, vring_a + off, wave, lane);
      }
      Kreq += tile_bytes;
      Vreq += tile_bytes;
      __builtin_amdgcn_sched_barrier(0);

      const int tb = key0 + t * 32;
      const uint4 *img = kring + SLOT * TILE;
      const uint4 *vimg = vring + SLOT * TILE;

      // ---- |V_i| on the wave without a query tile (before the score accumulators exist: the two never live together)
      if (use_v && v_by_last) {
        // The last wave has no query tile: it takes the squared norms of all 32 value rows off the
        // diagonal of V V^T (eight matrix instructions on the tile's fragments, exact products, fp32
        // sums) and the other waves do nothing for V.  Row r's diagonal element sits in lane r of the
        // half-wave (r / 4) % 2, accumulator register 4 (r / 8) + r % 4.
        if (wave == WAVES - 1) {
          f32x16 va;
#pragma unroll
          for (int i = 0; i < 16; ++i) va[i] = 0.f;
#pragma unroll
          for (int c = 0; c < NCHK; ++c) {
            Frag vf;
            vf.q = read_key_frag<DT, D>(vimg, 0, c, l32, half);
            va = mma<DT>(vf, vf, va);
          }
          float ss = 0.f;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float x = va[4 * q];
#pragma unroll
            for (int j = 1; j < 4; ++j) x = (l32 & 3) == j ? va[4 * q + j] : x;
            ss = (l32 >> 3) == q ? x : ss;
          }
          const int key = tb + l32;
          if (half == ((l32 >> 2) & 1) && key < Nc) vnorm[key] = __builtin_amdgcn_sqrtf(ss);
        }
      }

      // ---- softmax statistics of all TQ tiles; the MFMA chains are independent
      f32x16 acc[TQ];
      if (nq > 0) {
        Frag kf[NCHK];
#pragma unroll
        for (int c = 0; c < NCHK; ++c) kf[c].q = read_key_frag<DT, D>(img, 0, c, l32, half);
#pragma unroll
        for (int q = 0; q < TQ; ++q)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[q][i] = 0.f;
#pragma unroll
        for (int c = 0; c < NCHK; ++c)
#pragma unroll
          for (int q = 0; q < TQ; ++q) acc[q] = mma<DT>(kf[c], qf[q][c], acc[q]);
      }

      // ---- key norms and the sum of normalised keys (independent of the MFMA results, so it can
      // fill the vector ALU while the matrix core runs).  The tile image is walked 64 pieces at a
      // time (RPL whole rows), steps dealt round-robin to the waves; PPR consecutive lanes hold
      // one key.
      constexpr int STEPS = TILE / 64, RPL = 64 / PPR;
      const int lrow = lane / PPR, lq = lane % PPR;
#pragma unroll
      for (int jj = 0; jj < (STEPS + WAVES - 1) / WAVES; ++jj) {
        if (!use_k) break;
        const int j = jj * WAVES + wave;
        if (STEPS % WAVES != 0 && j >= STEPS) break;
        const int row = j * RPL + lrow, key = tb + row;
        Frag f;
        f.q = img[row * PPR + (lq ^ tile_swz<DT, D>(row))];
        const float ss = seg_sum<PPR>(piece_sumsq<DT>(f));
        const bool valid = key < N;
        const float inv = valid ? inv_norm<DT>(ss) : 0.f;
        if (valid && lq == 0) invnorm[key] = inv;
#pragma unroll
        for (int e = 0; e < EPC; ++e) ksacc[e] = fmaf(inv, frag_elem<DT>(f, e), ksacc[e]);
      }

      // ---- |V_i|: PPR consecutive lanes hold one row (which piece of the row a lane gets does
      // not matter for a sum of squares, so the image is read without undoing the rotation)
      if (use_v && !v_by_last) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          const int p = i * NT + tid, key = tb + p / PPR;
          Frag f;
          f.q = vimg[p < TILE ? p : 0];
          const float ss = seg_sum<PPR>(piece_sumsq<DT>(f));
          if (p % PPR == 0 && p < TILE && key < Nc) vnorm[key] = __builtin_amdgcn_sqrtf(ss);
        }
      }

      if (nq > 0 && tb + 31 > free_limit) {        // tile reaches into the window or past N: mask
#pragma unroll
        for (int q = 0; q < TQ; ++q)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            int kidx = tb + 8 * (i >> 2) + 4 * half + (i & 3);
            acc[q][i] = (kidx > lim[q]) ? -INFINITY : acc[q][i];
          }
      }
#pragma unroll
      for (int q = 0; q < TQ; ++q) {
        if (nq == 0) break;                               // wave-uniform: this wave has no query tile
        // The offset m of a row only has to keep the terms inside the range of a float: exp2 of
        // (logit - m) may be far above 1.  So the terms are formed with the offset as it stands,
        // and only if a row's sum comes out infinite or undefined (a term or the sum overflowed, or the
        // row has no offset yet: m = -inf gives inf or NaN for every key) does the wave take the tile's
        // maximum, move the offset there, rescale the sum and form the terms again.  After a
        // row's first tile that takes a logit 88 above everything the row has seen before.
        float sum[4];                                     // four chains: the adds do not wait on each other
        {
          const float nmu = -m[q];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float term = fast_exp2(fmaf(acc[q][i], c2, nmu));
            sum[i & 3] = i < 4 ? term : sum[i & 3] + term;          // the first term starts its chain
          }
        }
        float lnew = l[q] + ((sum[0] + sum[1]) + (sum[2] + sum[3]));
        if (__builtin_amdgcn_ballot_w64(!(lnew < INFINITY)) != 0) {
          float tmax = fmaxf(acc[q][0], acc[q][1]);
#pragma unroll
          for (int i = 2; i < 16; i += 2) tmax = fmaxf(fmaxf(tmax, acc[q][i]), acc[q][i + 1]);
          const float mn = fmaxf(m[q], tmax * c2);          // c2 > 0: scaling commutes with max
          const float mu = (mn == -INFINITY) ? 0.f : mn;    // nothing visible yet: every term is exp2(-inf) = 0
          float s2[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int i = 0; i < 16; ++i) s2[i & 3] += fast_exp2(fmaf(acc[q][i], c2, -mu));
          lnew = l[q] * fast_exp2(m[q] - mu) + ((s2[0] + s2[1]) + (s2[2] + s2[3]));
          m[q] = mn;
        }
        l[q] = lnew;
      }
    };
    static_assert(kRing == 4, "unrolled four times below");
    for (int t = 0; t < nt; t += kRing) {
      tile_step(std::integral_constant<int, 0>{}, t);
      if (t + 1 < nt) tile_step(std::integral_constant<int, 1>{}, t + 1);
      if (t + 2 < nt) tile_step(std::integral_constant<int, 2>{}, t + 2);
      if (t + 3 < nt) tile_step(std::integral_constant<int, 3>{}, t + 3);
    }

    // ---- run partials to global
    const int64_t slot = slot0 + blockIdx.x + ul;
    float2 *part_ml = reinterpret_cast<float2 *>(ws + w.part_ml) + slot * QTR;
#pragma unroll
    for (int q = 0; q < (GIVEN_LSE ? 0 : TQ); ++q) {
      // The sum may be far from 1 (the offset is not the maximum): bring it back to [0.5, 1) so that
      // the merges below and in the fold cannot overflow.
      {
        int e;
        l[q] = frexpf(l[q], &e);
        m[q] += (float)e;
      }
      ml_merge(m[q], l[q], __shfl_xor(m[q], 32), __shfl_xor(l[q], 32));
      if (q < nq && half == 0) part_ml[(wave * TQ + q) * 32 + l32] = make_float2(m[q], l[q]);
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      float x = ksacc[e];
#pragma unroll
      for (int off = PPR; off < 64; off <<= 1) x += __shfl_xor(x, off);   // rows of one step, fixed order
      if (lane < PPR) ks_s[wave * D + lane * EPC + e] = x;
    }
    lds_barrier();                                     // ks_s complete
    float *part_ks = reinterpret_cast<float *>(ws + w.part_ksum) + slot * D;
    for (int d = tid; d < D; d += NT) {
      float a = 0.f;
      for (int wv = 0; wv < WAVES; ++wv) a += ks_s[wv * D + d];   // fixed order
      part_ks[d] = a;
    }
    item += nit;
  }
}

// ------------------------------------------------------------------------------------------------
// fold_kernel: one workgroup per unit folds the per-run partials that stats_kernel (grid G1) left
// for the unit, in run order:
//   * per window-query row the exponent offset -b_r, b_r = max_r + log2(sum_r * G*W), so that
//     exp2(x - b_r) is the softmax weight already divided by the number of rows (-inf past G*W);
//     with the caller's log-sum-exp of the row, b_r = lse_r * log2(e) + log2(G*W) instead;
//   * the mean normalised key as two rows of 16-byte pieces: row 0 its bf16 head, row 1 the bf16
//     remainder (zero for f32), piece (c, half) of row r at index (c * 2 + half) * 2 + r;
//   * the redundancy r (paper Sec. 3.3, Eq. 3-4).
// Workgroup g of the stats grid owned the items [g*T1/G1, (g+1)*T1/G1) and wrote one partial per
// unit it touched, at slot g + unit_local.  The unit's items are [first, last): the first workgroup
// touching it is the largest g with g*T1/G1 <= first, the last one the largest g with g*T1/G1 < last.
// ------------------------------------------------------------------------------------------------
constexpr int kFoldThreads = 256;

template <int DT, int D>
__global__ __launch_bounds__(kFoldThreads) void fold_kernel(Shape s, LayerOutTable out, LseTable lse, char *ws, Workspace w,
                                                            int64_t unit0, int nunits, int G1, int ipu, int64_t slot0) {
  constexpr int EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), NW = kFoldThreads / 64;
  __shared__ float kbar_f[D];
  __shared__ double red_s[NW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ul = blockIdx.x;
  const int64_t unit = unit0 + ul;
  const UnitCoord uc = unit_coord(s, ul);
  const int N = s.N, QTR = s.QT * 32;
  const int64_t T1 = (int64_t)nunits * ipu, first = (int64_t)ul * ipu, last = first + ipu;
  const int g_lo = (int)(((first + 1) * G1 + T1 - 1) / T1) - 1, g_hi = (int)((last * G1 + T1 - 1) / T1) - 1;

  const float2 *all_ml = reinterpret_cast<const float2 *>(ws + w.part_ml) + (slot0 + ul) * QTR;
  float *nb = reinterpret_cast<float *>(ws + w.nb) + unit * s.nb_rows;
  // rows of this head's group are consecutive in [batch, n_q_heads, W]
  const float *lse_u = lse.l[uc.layer] ? lse.l[uc.layer] + (int64_t)(uc.b * s.hq + uc.h * s.G) * s.W : nullptr;
  for (int r = tid; r < s.nb_rows; r += kFoldThreads) {
    float b = INFINITY;                                // rows past G*W: weight 0
    if (r < s.GW && lse_u) {
      b = lse_u[r] * 1.4426950408889634f + log2f((float)s.GW);
    } else if (r < s.GW) {
      float m = -INFINITY, l = 0.f;
      for (int g0 = g_lo; g0 <= g_hi; g0 += 8) {       // batches of eight independent loads
        float2 p[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) p[j] = (g0 + j <= g_hi) ? all_ml[(int64_t)(g0 + j) * QTR + r] : make_float2(-INFINITY, 0.f);
#pragma unroll
        for (int j = 0; j < 8; ++j) ml_merge(m, l, p[j].x, p[j].y);
      }
      b = m + log2f(l) + log2f((float)s.GW);
    }
    nb[r] = -b;
  }
  const float *all_ks = reinterpret_cast<const float *>(ws + w.part_ksum) + (slot0 + ul) * D;
  double sq = 0.0;
  for (int d = tid; d < D; d += kFoldThreads) {
    float a = 0.f;
    for (int g0 = g_lo; g0 <= g_hi; g0 += 8) {
      float p[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) p[j] = (g0 + j <= g_hi) ? all_ks[(int64_t)(g0 + j) * D + d] : 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) a += p[j];
    }
    kbar_f[d] = a / (float)N;
    sq += (double)a * (double)a;
  }
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) sq += __shfl_xor(sq, sft);
  if (lane == 0) red_s[wave] = sq;
  __syncthreads();
  if (tid == 0) {
    double tot = 0.0;
    for (int wv = 0; wv < NW; ++wv) tot += red_s[wv];
    // Eq. 4: (T^2 |Kbar|^2 - T) / (T (T - 1)) with T^2 |Kbar|^2 = |sum of normalised keys|^2
    const float r = (float)((tot - (double)N) / ((double)N * (double)(N - 1)));
    reinterpret_cast<float *>(ws + w.rbar)[unit] = r;
    float *red_out = out.l[uc.layer].redundancy;
    if (red_out) red_out[uc.b * s.hkv + uc.h] = r;
  }
  uint4 *kbarp = reinterpret_cast<uint4 *>(ws + w.kbarp) + unit * (NCHK * 4);
  for (int p = tid; p < NCHK * 4; p += kFoldThreads) {
    const int row = p & 1, hf = (p >> 1) & 1, c = p >> 2;
    const float *src = kbar_f + (2 * c + hf) * EPC;
    Frag f;
    f.q = make_uint4(0, 0, 0, 0);
    if constexpr (DT == MIXKV_BF16) {
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        float v = src[e];
        uint16_t hi = f32_to_bf16_rne(v);
        uint16_t bits = hi;
        if (row == 1) bits = f32_to_bf16_rne(v - __uint_as_float((uint32_t)hi << 16));
        f.u[e >> 1] |= (uint32_t)bits << ((e & 1) * 16);
      }
    } else {
      if (row == 0) f.q = *reinterpret_cast<const uint4 *>(src);
    }
    kbarp[p] = f.q;
  }
}

// ------------------------------------------------------------------------------------------------
// attn_kernel: second pass over K.
//   a_i    = (1 / (G*W)) * sum over window rows of softmax weights on key i   (Sec. 3.2, extrinsic)
//   kdot_i = K_i . Kbar; the mix kernel turns it into -(K_i . Kbar) / |K_i|   (Sec. 3.2, diversity)
// Query rows on the MFMA output rows, keys on the columns: a wave's sum over its rows is a register
// sum; the waves' partial column sums meet in LDS and are added in a fixed order.  The mean key is
// two more "query" rows (hi + lo bf16 halves, so the dot keeps fp32 accuracy).  When the padded
// query block has a spare tile they sit in its rows 0 and 1 and cost nothing; otherwise every wave
// applies a separate mean-key tile to every WAVES-th key tile.
//
// The exponent offsets and the mean key come from fold_kernel.  The fragments of the next key tile
// are read from LDS into a second set of registers while the current tile is being worked on.
// ------------------------------------------------------------------------------------------------
// Waves per SIMD the register allocation of attn_kernel aims at: two, i.e. two four-wave workgroups
// per compute unit (an eight-wave workgroup is two per SIMD by itself).  Four waves with two query
// tiles of 128-element f32 rows do not fit 256 registers (their fragments are twice as wide as bf16
// ones, and the tile loop then reloads some three hundred spilled registers per step), so they run one
// workgroup per compute unit on the full register file.
__host__ __device__ constexpr int attn_waves_per_simd(int dtype, int D, int waves, int tq) {
  return (dtype == MIXKV_F32 && D == 128 && waves == 4 && tq == 2) ? 1 : 2;
}

template <int DT, int D, int WAVES, int TQ, bool SPARE>
__global__ __launch_bounds__(WAVES * 64, attn_waves_per_simd(DT, D, WAVES, TQ)) void attn_kernel(Shape s, LayerInTable in, LayerOutTable out, char *ws,
                                                            Workspace w, int64_t unit0, int nunits) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), PPR = D * EB / 16;
  constexpr int NT = WAVES * 64, KT = chunk_tiles(DT, D), CH = KT * 32, TILE = 32 * PPR;
  constexpr int KL = (TILE / 64 + WAVES - 1) / WAVES;        // requests per wave and tile
  __shared__ uint4 kring[kRing * TILE];
  __shared__ uint4 kbar_s[NCHK * 4];                         // mean-key rows 0/1 x halves, 16-byte pieces
  __shared__ float cs_s[2 * WAVES * CH];                     // [2][WAVES][CH] partial column sums
  __shared__ int lim_s[WAVES * TQ * 32];                     // last key each query row attends to
  __shared__ float kd_s[SPARE ? 1 : 2 * WAVES * CH];         // [2][WAVES][CH] partial K_i . Kbar (no spare tile)

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps its address math scalar
  const int N = s.N, Nc = s.Nc;
  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;
  // the mean key rides in rows 0/1 of the first tile past the live rows, if the block has one
  // (SPARE, chosen by the launcher: QT < WAVES * TQ)
  constexpr bool spare = SPARE;
  const int kb_wave = s.QT / TQ, kb_q = s.QT % TQ;
  const uint32_t kring_a = lds_base_of(kring);
  for (int r = tid; r < WAVES * TQ * 32; r += NT) lim_s[r] = s.causal ? Nc + r % s.W : N - 1;
  const int64_t T = (int64_t)nunits * s.nchunks;
  int64_t item = wg_first_item(blockIdx.x, gridDim.x, T);
  const int64_t item_end = wg_first_item(blockIdx.x + 1, gridDim.x, T);

  while (item < item_end) {
    const int ul = (int)(item / s.nchunks), c0 = (int)(item - (int64_t)ul * s.nchunks);
    const int nit = (int)min((int64_t)(s.nchunks - c0), item_end - item);
    const int64_t unit = unit0 + ul;
    const UnitCoord uc = unit_coord(s, ul);
    const LayerIn L = in.l[uc.layer];
    const char *Kb = reinterpret_cast<const char *>(L.K) + ((int64_t)uc.b * L.sb + (int64_t)uc.h * L.sh) * EB;
    const char *Qb = reinterpret_cast<const char *>(L.Q) + ((int64_t)(uc.b * s.hq + uc.h * s.G) * s.W * D) * EB;
    const int64_t row_bytes = L.sn * EB;
    float *araw = reinterpret_cast<float *>(ws + w.araw) + unit * s.Npad;
    float *kdot = reinterpret_cast<float *>(ws + w.sdiv) + unit * s.Npad;   // K_i . Kbar, not yet normalised
    const float *nb = reinterpret_cast<const float *>(ws + w.nb) + unit * s.nb_rows;
    const uint4 *kbarp = reinterpret_cast<const uint4 *>(ws + w.kbarp) + unit * (NCHK * 4);
    const int key0 = c0 * CH;                                        // first key of the run
    const int nt = min(nit * KT, (N - key0 + 31) / 32);              // tiles of the run that hold keys

    const int64_t tile_bytes = 32 * row_bytes;
    auto request = [&](int tr) {
      fetch_tile<DT, D, WAVES>(Kb + (key0 + tr * 32) * row_bytes, row_bytes, key0 + tr * 32, N,
                               kring_a + (uint32_t)(tr & (kRing - 1)) * (TILE * 16), wave, lane);
    };
    // first row of the tile the next step of the loop requests (tile t + 1 + kLead at step t)
    const char *Kreq = Kb + (key0 + (1 + kLead) * 32) * row_bytes;
    lds_barrier();                                     // the previous run is done with LDS
#pragma unroll
    for (int j = 0; j <= kLead; ++j)
      if (j < nt) request(j);
    static_assert(kLead + 1 == kRing && kRing % KT == 0, "the tile loop below is unrolled over the ring");

    // query tiles in fragment form (tiles past QT are zero, except for the two mean-key rows) and
    // the exponent offset of each of the lane's 16 rows per tile
    Frag qf[TQ][NCHK];
    float nbv[TQ][16];
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
      const int row = (wave * TQ + q) * 32 + l32;
      const bool live = row < s.GW;
      const bool mean_rows = spare && wave == kb_wave && q == kb_q && l32 < 2;
      const char *qrow = Qb + ((int64_t)(live ? row : 0) * D) * EB + half * 16;
#pragma unroll
      for (int c = 0; c < NCHK; ++c) {
        const uint4 *src = live ? reinterpret_cast<const uint4 *>(qrow + c * 32) : kbarp + (c * 2 + half) * 2 + (l32 & 1);
        const uint4 v = *src;
        qf[q][c].q = (live || mean_rows) ? v : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4) {
        const float4 v = *reinterpret_cast<const float4 *>(nb + (wave * TQ + q) * 32 + 8 * k4 + 4 * half);
        nbv[q][4 * k4 + 0] = v.x; nbv[q][4 * k4 + 1] = v.y; nbv[q][4 * k4 + 2] = v.z; nbv[q][4 * k4 + 3] = v.w;
      }
    }
    if (!spare)
      for (int p = tid; p < NCHK * 4; p += NT) kbar_s[p] = kbarp[p];
    // Nothing may be pending when the tile loop is entered: its waits count the requests issued
    // inside it.
    wait_vm<0>();
    lds_barrier();                                     // tiles 0 .. kLead of the run (and kbar_s) are visible

    // add the waves' partial column sums of chunk `chunk` (buffer pb) in a fixed order
    auto flush_colsums = [&](int chunk, int pb) {
      for (int i = tid; i < CH; i += NT) {
        const int key = chunk * CH + i;
        float a = 0.f;
        for (int wv = 0; wv < WAVES; ++wv) a += cs_s[(pb * WAVES + wv) * CH + i];
        if (key < Nc) araw[key] = a;
        if constexpr (!SPARE) {
          float d = 0.f;
          for (int wv = 0; wv < WAVES; ++wv) d += kd_s[(pb * WAVES + wv) * CH + i];
          if (key < Nc) kdot[key] = d;
        }
      }
    };

    // Where the mean key has no spare query rows it is a tile of its own (rows 0 and 1), and its
    // contraction with a key tile is dealt over the waves by contraction chunk: wave w takes the
    // NOWN chunks w, w + WAVES, ... (none if there are fewer chunks than waves: its mean-key rows
    // are then zero), so every wave issues the same few extra matrix instructions in every step,
    // at fixed places of the instruction stream (the chunk is a run-time index into LDS, the code
    // has no branch), and the waves' partial dot products meet in LDS like the column sums.
    constexpr int NOWN = NCHK >= WAVES ? NCHK / WAVES : 1;
    auto own_chunk = [&](int j) { return (wave + j * WAVES) % NCHK; };
    auto mean_key_frag = [&](int j) {
      Frag kbf;
      kbf.q = kbar_s[(own_chunk(j) * 2 + half) * 2 + (l32 & 1)];
      if (l32 >= 2 || wave >= NCHK) kbf.q = make_uint4(0, 0, 0, 0);
      return kbf;
    };
    // Scores of the key tile in image `img` into accN: NCHK fragment reads, each feeding the TQ chains
    // (and this wave's share of the mean-key tile: kdN).
    auto scores = [&](const uint4 *img, f32x16 (&accN)[TQ], float &kdN) {
      f32x16 acd;
#pragma unroll
      for (int i = 0; i < 16; ++i) acd[i] = 0.f;
#pragma unroll
      for (int q = 0; q < TQ; ++q)
#pragma unroll
        for (int i = 0; i < 16; ++i) accN[q][i] = 0.f;
#pragma unroll
      for (int c = 0; c < NCHK; ++c) {
        Frag kf;
        kf.q = read_key_frag<DT, D>(img, 0, c, l32, half);
#pragma unroll
        for (int q = 0; q < TQ; ++q) accN[q] = mma<DT>(qf[q][c], kf, accN[q]);
      }
      if constexpr (!SPARE) {
#pragma unroll
        for (int j = 0; j < NOWN; ++j) {
          Frag kx;
          kx.q = read_key_frag<DT, D>(img, 0, own_chunk(j), l32, half);
          acd = mma<DT>(mean_key_frag(j), kx, acd);
        }
        kdN = acd[0] + acd[1];
      }
    };

    // One tile step.  At its start the images of tiles <= t + 1 are visible to every wave and the
    // scores of tile t are in accC (their matrix instructions were issued a step ago).  The step
    // issues the matrix instructions of tile t + 1 into accN and, in their shadow, turns the scores
    // of tile t into weights and column sums: a wave's matrix and vector work overlap although
    // the one feeds the other.  Tile t + 1 + kLead is requested into the image of tile t, which
    // nobody reads any more (its fragments were read a step ago).  After the last tile of a run the
    // "next" image holds an older tile: its scores are computed and never used.
    // The loop is unrolled over the ring, so the ring slot of a step (t mod kRing) is a constant and
    // the LDS addresses of its reads are a loop-invariant lane offset plus an immediate.
    auto step = [&](auto slot_c, int t, f32x16 (&accC)[TQ], f32x16 (&accN)[TQ], float &kdC, float &kdN) {
      constexpr int SLOT = decltype(slot_c)::value;
      __builtin_amdgcn_sched_barrier(0);
      wait_tile<KL>(t + 1, nt);
      lds_barrier();                                   // every wave has read the fragments of tile t: its image is free
      if (t + 1 + kLead < nt)                          // tile t + kRing goes into the image of tile t
        fetch_tile<DT, D, WAVES>(Kreq, row_bytes, key0 + (t + 1 + kLead) * 32, N, kring_a + (uint32_t)SLOT * (TILE * 16), wave,
                                 lane);
      Kreq += tile_bytes;
      const int k = SLOT % KT, g = t / KT;             // tile within its chunk, chunk within the run
      if (k == 0 && g > 0) flush_colsums(c0 + g - 1, (g - 1) & 1);
      float *cs = cs_s + ((g & 1) * WAVES + wave) * CH;
      const int tb = key0 + t * 32, key = tb + l32;
      const uint4 *imgn = kring + ((SLOT + 1) & (kRing - 1)) * TILE;

      // straight-line body, once with and once without the mask of the tiles that reach into the
      // window or past N, so that the scheduler sees matrix and vector work in one block
      auto body = [&](auto mask_c) {
        constexpr bool MASK = decltype(mask_c)::value;
        __builtin_amdgcn_sched_barrier(0);
        // ---- K_i . Kbar: rows 0 and 1 (half 0) of the spare tile (taken before the mask touches them)
        float kd = kdC;                                  // no spare tile: this wave's share, from a step ago
        bool kd_mine = false;
        if constexpr (SPARE) {
          const float kd0 = accC[0][0] + accC[0][1], kd1 = accC[TQ - 1][0] + accC[TQ - 1][1];
          kd = kb_q == 0 ? kd0 : kd1;
          kd_mine = wave == kb_wave;
        }
        if constexpr (MASK) {
#pragma unroll
          for (int q = 0; q < TQ; ++q)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int row = (wave * TQ + q) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
              accC[q][i] = (key <= lim_s[row]) ? accC[q][i] : -INFINITY;
            }
        }
        // The matrix instructions of tile t + 1 and the weights of tile t, slice by slice: one
        // matrix instruction, then its share of the step's TQ * 16 weights (fma, exp, add), with
        // the order of the slices fixed so that the vector work is issued while the matrix core
        // runs.  The fragment of the next contraction chunk is read one chunk ahead.
        constexpr int EPS = 16 / NCHK;                   // weights per slice
        static_assert(16 % NCHK == 0, "a whole number of weights per matrix instruction");
        // Fragments are read one contraction chunk ahead into two rotating register sets.
        Frag kfr[2];
        kfr[0].q = read_key_frag<DT, D>(imgn, 0, 0, l32, half);
        float cs4[4];                                    // four chains: the adds do not wait on each other
        f32x16 acd;
        Frag kx, kbx;                                    // this wave's next chunk of the mean-key tile
        if constexpr (!SPARE) {
#pragma unroll
          for (int i = 0; i < 16; ++i) acd[i] = 0.f;
        }
#pragma unroll
        for (int c = 0; c < NCHK; ++c) {
          if (c + 1 < NCHK) kfr[(c + 1) & 1].q = read_key_frag<DT, D>(imgn, 0, c + 1, l32, half);
          if constexpr (!SPARE) {
            // own chunk j is read under slice (j + 1) * NCHK / NOWN - 2 and used one slice later
            if ((c + 2) % (NCHK / NOWN) == 0) {
              const int j = (c + 2) / (NCHK / NOWN) - 1;
              kx.q = read_key_frag<DT, D>(imgn, 0, own_chunk(j), l32, half);
              kbx = mean_key_frag(j);
            }
          }
#pragma unroll
          for (int q = 0; q < TQ; ++q) {
            if (c == 0) {
#pragma unroll
              for (int i = 0; i < 16; ++i) accN[q][i] = 0.f;
            }
            accN[q] = mma<DT>(qf[q][c], kfr[c & 1], accN[q]);
#pragma unroll
            for (int j = 0; j < EPS; ++j) {
              const int n = (c * TQ + q) * EPS + j, qq = n / 16, i = n % 16;
              const float wgt = fast_exp2(fmaf(accC[qq][i], c2, nbv[qq][i]));
              cs4[i & 3] = n < 4 ? wgt : cs4[i & 3] + wgt;        // the first term starts its chain
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          if constexpr (!SPARE) {
            if ((c + 1) % (NCHK / NOWN) == 0) {
              acd = mma<DT>(kbx, kx, acd);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
        if constexpr (!SPARE) kdN = acd[0] + acd[1];
        float colsum = (cs4[0] + cs4[1]) + (cs4[2] + cs4[3]);
        colsum += __shfl_xor(colsum, 32);
        __builtin_amdgcn_sched_barrier(0);
        if (half == 0) cs[k * 32 + l32] = colsum;
        if constexpr (SPARE) {
          if (kd_mine && half == 0 && key < Nc) kdot[key] = kd;
        } else {
          if (half == 0) kd_s[((g & 1) * WAVES + wave) * CH + k * 32 + l32] = kd;
        }
      };
      if (tb + 31 > free_limit) body(std::true_type{});
      else body(std::false_type{});
    };

    f32x16 accA[TQ], accB[TQ];
    float kdA = 0.f, kdB = 0.f;
    scores(kring, accA, kdA);                           // tile 0
    for (int t = 0; t < nt; t += kRing) {
      step(std::integral_constant<int, 0>{}, t, accA, accB, kdA, kdB);
      if (t + 1 < nt) step(std::integral_constant<int, 1>{}, t + 1, accB, accA, kdB, kdA);
      if (t + 2 < nt) step(std::integral_constant<int, 2>{}, t + 2, accA, accB, kdA, kdB);
      if (t + 3 < nt) step(std::integral_constant<int, 3>{}, t + 3, accB, accA, kdB, kdA);
    }
    lds_barrier();
    flush_colsums(c0 + (nt - 1) / KT, ((nt - 1) / KT) & 1);
    item += nit;
  }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
int stream_chunk_keys(int dtype, int D) { return chunk_tiles(dtype, D) * 32; }

// Waves per workgroup and query tiles per wave for a given number of query tiles.
static void stream_config(int QT, int *waves, int *tq) {
  *waves = QT <= 8 ? 4 : 8;
  *tq = QT <= 4 ? 1 : 2;
}
// stats_kernel needs fewer registers per query tile than attn_kernel: up to 8 query tiles it runs
// eight waves of one tile each, four waves per SIMD, which hides more of its latencies; waves
// without a query tile share the key and value statistics (with four tiles: 124 us against 128 us
// for four waves on 8 layers of a 16K-token, 8-KV-head cache).
static void stats_config(int QT, int *waves, int *tq) {
  stream_config(QT, waves, tq);
  if (QT <= 8) { *waves = 8; *tq = 1; }
}

// Grid of the two streaming kernels: enough workgroups to fill the chip once, never more than items.
int stream_grid(const Shape &s, int nunits, int num_cus) {
  int waves, tq;
  stream_config(s.QT, &waves, &tq);
  const int64_t T = (int64_t)nunits * s.nchunks;
  int64_t cap = (int64_t)num_cus * (waves == 4 ? 2 : 1);
  if (cap > kMaxStreamGrid) cap = kMaxStreamGrid;
  return (int)(T < cap ? T : cap);
}

template <int DT, int D, int WAVES, int TQ, bool GIVEN_LSE = false>
static hipError_t launch_stats_c(const Shape &s, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                                 int nunits, int grid, int64_t slot0, hipStream_t st) {
  auto kern = stats_kernel<DT, D, WAVES, TQ, GIVEN_LSE>;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES * 64), 0, st, s, in, ws, w, unit0, nunits, slot0);
  return hipGetLastError();
}

template <int DT, int D, int WAVES, int TQ>
static hipError_t launch_attn_c(const Shape &s, const LayerInTable &in, const LayerOutTable &out, const LseTable &,
                                char *ws, const Workspace &w, int64_t unit0, int nunits, int grid, int64_t,
                                hipStream_t st) {
  // with a spare query tile in the padded block the mean key rides in its first two rows
  if (s.QT < WAVES * TQ) {
    auto kern = attn_kernel<DT, D, WAVES, TQ, true>;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES * 64), 0, st, s, in, out, ws, w, unit0, nunits);
  } else {
    auto kern = attn_kernel<DT, D, WAVES, TQ, false>;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES * 64), 0, st, s, in, out, ws, w, unit0, nunits);
  }
  return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_stats_t(const Shape &s, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                                 int nunits, int grid, int64_t slot0, bool given_lse, hipStream_t st) {
  int waves, tq;
  // without the logits the pass is a plain stream: eight waves per workgroup keep more loads in flight
  if (given_lse) return launch_stats_c<DT, D, 8, 1, true>(s, in, ws, w, unit0, nunits, grid, slot0, st);
  stats_config(s.QT, &waves, &tq);                   // always eight waves; one or two query tiles each
  if (tq == 1) return launch_stats_c<DT, D, 8, 1>(s, in, ws, w, unit0, nunits, grid, slot0, st);
  return launch_stats_c<DT, D, 8, 2>(s, in, ws, w, unit0, nunits, grid, slot0, st);
}

template <int DT, int D>
static hipError_t launch_attn_t(const Shape &s, const LayerInTable &in, const LayerOutTable &out, const LseTable &lse,
                                char *ws, const Workspace &w, int64_t unit0, int nunits, int grid, int64_t slot0,
                                hipStream_t st) {
  int waves, tq;
  stream_config(s.QT, &waves, &tq);
  if (waves == 4 && tq == 1) return launch_attn_c<DT, D, 4, 1>(s, in, out, lse, ws, w, unit0, nunits, grid, slot0, st);
  if (waves == 4) return launch_attn_c<DT, D, 4, 2>(s, in, out, lse, ws, w, unit0, nunits, grid, slot0, st);
  return launch_attn_c<DT, D, 8, 2>(s, in, out, lse, ws, w, unit0, nunits, grid, slot0, st);
}

// `grid` workgroups of the first pass split `items_per_unit` items per unit among themselves.
hipError_t launch_fold(const Shape &s, int dtype, const LayerOutTable &out, const LseTable &lse, char *ws, const Workspace &w,
                       int64_t unit0, int nunits, int grid, int items_per_unit, int64_t slot0, hipStream_t st) {
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(nunits), dim3(kFoldThreads), 0, st, s, out, lse, ws, w, unit0, nunits, grid, items_per_unit, slot0);
    return hipGetLastError();
  };
  if (dtype == MIXKV_BF16) return s.D == 128 ? go(fold_kernel<MIXKV_BF16, 128>) : go(fold_kernel<MIXKV_BF16, 64>);
  return s.D == 128 ? go(fold_kernel<MIXKV_F32, 128>) : go(fold_kernel<MIXKV_F32, 64>);
}

hipError_t launch_stats(const Shape &s, int dtype, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                        int nunits, int grid, int64_t slot0, bool given_lse, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_stats_t<MIXKV_BF16, 128>(s, in, ws, w, unit0, nunits, grid, slot0, given_lse, st);
    return launch_stats_t<MIXKV_BF16, 64>(s, in, ws, w, unit0, nunits, grid, slot0, given_lse, st);
  }
  if (s.D == 128) return launch_stats_t<MIXKV_F32, 128>(s, in, ws, w, unit0, nunits, grid, slot0, given_lse, st);
  return launch_stats_t<MIXKV_F32, 64>(s, in, ws, w, unit0, nunits, grid, slot0, given_lse, st);
}

// `grid` must be the grid stats_kernel ran with: both kernels split the same items the same way,
// and attn_kernel uses it to find the partials of its units.
hipError_t launch_attn(const Shape &s, int dtype, const LayerInTable &in, const LayerOutTable &out, const LseTable &lse,
                       char *ws, const Workspace &w, int64_t unit0, int nunits, int grid, int64_t slot0, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_attn_t<MIXKV_BF16, 128>(s, in, out, lse, ws, w, unit0, nunits, grid, slot0, st);
    return launch_attn_t<MIXKV_BF16, 64>(s, in, out, lse, ws, w, unit0, nunits, grid, slot0, st);
  }
  if (s.D == 128) return launch_attn_t<MIXKV_F32, 128>(s, in, out, lse, ws, w, unit0, nunits, grid, slot0, st);
  return launch_attn_t<MIXKV_F32, 64>(s, in, out, lse, ws, w, unit0, nunits, grid, slot0, st);
}

}  // namespace mixkv
