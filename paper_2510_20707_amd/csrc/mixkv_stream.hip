// The two kernels that stream the cache: window-attention statistics + key/value statistics
// (stats_kernel) and the normalised attention column sums + diversity dot products (attn_kernel).
//
// Both are MFMA kernels.  A workgroup owns `chunk` consecutive keys of one unit (one layer,
// batch item and KV head); each wave owns TPW tiles of 32 keys, held in registers in MFMA
// fragment form, and sweeps the G*W window-query rows in tiles of 32 that live in LDS.
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
#include "mixkv_internal.h"

#ifndef MIXKV_PREFETCH
#define MIXKV_PREFETCH 0   // register double-buffering of the next chunk spills at 2 waves per SIMD
#endif

namespace mixkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

union Frag {
  uint4 q;
  uint32_t u[4];
  float f[4];
  bf16x8 h;
};

template <int DT> struct Tr;
template <> struct Tr<MIXKV_F32> { static constexpr int EB = 4, EPC = 4; };
template <> struct Tr<MIXKV_BF16> { static constexpr int EB = 2, EPC = 8; };

template <int DT>
__device__ __forceinline__ f32x16 mma(const Frag &a, const Frag &b, f32x16 acc) {
  if constexpr (DT == MIXKV_BF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.h, b.h, acc, 0, 0, 0);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.f[i], b.f[i], acc, 0, 0, 0);
    return acc;
  }
}

template <int DT>
__device__ __forceinline__ float frag_elem(const Frag &f, int j) {
  if constexpr (DT == MIXKV_BF16) {
    uint32_t u = f.u[j >> 1];
    return __uint_as_float((j & 1) ? (u & 0xffff0000u) : (u << 16));
  } else {
    return f.f[j];
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Merge two running (max, sum) pairs of a softmax row (log2 domain).  A pair that has seen no
// key is (-inf, 0).
__device__ __forceinline__ void ml_merge(float &m, float &l, float m2, float l2) {
  float mn = fmaxf(m, m2);
  float mu = (mn == -INFINITY) ? 0.f : mn;
  l = l * fast_exp2(m - mu) + l2 * fast_exp2(m2 - mu);
  m = mn;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

struct UnitCoord {
  int layer, b, h;
};
__device__ __forceinline__ UnitCoord unit_coord(const Shape &s, int ul) {
  UnitCoord c;
  c.layer = ul / s.units_per_layer;
  int rem = ul - c.layer * s.units_per_layer;
  c.b = rem / s.hkv;
  c.h = rem - c.b * s.hkv;
  return c;
}

// LDS slot of lane (half, r) inside fragment c: rotating the row by 2c + half keeps both the
// fragment reads (consecutive lanes of one half) and the staging writes (the 16 pieces of one row)
// free of bank conflicts.
__device__ __forceinline__ int frag_slot(int c, int half, int r) { return half * 32 + ((r + 2 * c + half) & 31); }

// Stage the [QT*32, D] query block of one KV head into LDS in fragment order:
// fragment (t, c) is 64 slots x 16 bytes.  Rows >= GW are zero.
template <int DT, int D>
__device__ __forceinline__ void stage_queries(const Shape &s, const char *Qb, uint4 *qs, int tid, int nthreads) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), PPR = D * EB / 16;
  const int pieces = s.QT * 32 * PPR;
  for (int p = tid; p < pieces; p += nthreads) {
    int row = p / PPR, piece = p - row * PPR;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < s.GW) v = *reinterpret_cast<const uint4 *>(Qb + ((int64_t)row * D) * EB + piece * 16);
    int c = piece >> 1, half = piece & 1;
    qs[((row >> 5) * NCHK + c) * 64 + frag_slot(c, half, row & 31)] = v;
  }
}

template <int DT, int D>
__device__ __forceinline__ void load_key_tile(const char *Kb, int64_t row_bytes, int key, int half, Frag *kf) {
  constexpr int EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC);
  const char *p = Kb + key * row_bytes + half * 16;
#pragma unroll
  for (int c = 0; c < NCHK; ++c) kf[c].q = *reinterpret_cast<const uint4 *>(p + c * 32);
}

// Work split of the two streaming kernels.  An item is one chunk of one unit (item = unit_local *
// nchunks + chunk); workgroup g of G owns the contiguous items [g*T/G, (g+1)*T/G) and walks them in
// runs that stay inside one unit, so the unit's queries are staged once per run.
__device__ __forceinline__ int64_t wg_first_item(int64_t g, int64_t G, int64_t T) { return g * T / G; }

// ------------------------------------------------------------------------------------------------
// stats_kernel: first pass over K (and the only pass over V).
//   * running softmax (max, sum) of every window-query row over the run's keys;
//   * 1/|K_i| and the partial sum of the normalised keys (paper Sec. 3.2 diversity metrics,
//     Sec. 3.3 Eq. 3-4: only the sum of normalised keys is needed, never the T x T matrix);
//   * |V_i| (Sec. 3.2, VNorm intrinsic importance).
// Per-run partials go to the workspace slot of the run's first item; finalize_kernel folds them.
// ------------------------------------------------------------------------------------------------
template <int DT, int D, int WAVES, int TPW>
__global__ __launch_bounds__(WAVES * 64, 2) void stats_kernel(Shape s, LayerInTable in, char *ws, Workspace w,
                                                          int64_t unit0, int nunits) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), NE = D / 2, PPR = D * EB / 16;
  constexpr int NT = WAVES * 64, CH = WAVES * TPW * 32;
  constexpr int VB = 4, VPT = CH * PPR / NT / VB;      // V pieces per thread: VB batches of VPT
  static_assert(CH * PPR % (NT * VB) == 0, "V tiling");
  extern __shared__ uint4 smem[];
  const int QTR = s.QT * 32;
  uint4 *qs = smem;                                                       // [QT * NCHK * 64]
  float2 *ml_s = reinterpret_cast<float2 *>(smem + s.QT * NCHK * 64);     // [WAVES][QTR]
  float *ks_s = reinterpret_cast<float *>(ml_s + WAVES * QTR);            // [WAVES][D]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int N = s.N, Nc = s.Nc;
  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;      // keys <= this are visible to every row
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
    const bool use_v = s.intrinsic == MIXKV_INTRINSIC_VNORM;

    __syncthreads();                       // the previous run is done with LDS
    stage_queries<DT, D>(s, Qb, qs, tid, NT);
    for (int r = lane; r < QTR; r += 64) ml_s[wave * QTR + r] = make_float2(-INFINITY, 0.f);
    for (int d = lane; d < D; d += 64) ks_s[wave * D + d] = 0.f;

    Frag kfa[TPW][NCHK], kfb[TPW][NCHK];
    auto load_chunk = [&](int chunk, Frag (&kf)[TPW][NCHK]) {
#pragma unroll
      for (int j = 0; j < TPW; ++j) {
        const int key = chunk * CH + (wave * TPW + j) * 32 + l32;
        load_key_tile<DT, D>(Kb, row_bytes, min(key, N - 1), half, kf[j]);
      }
    };
    load_chunk(c0, kfa);
    __syncthreads();                       // queries staged

    // one chunk: kf holds its keys, the next chunk's keys are fetched into kn meanwhile
    auto do_chunk = [&](int chunk, bool has_next, Frag (&kf)[TPW][NCHK], Frag (&kn)[TPW][NCHK]) {
      const int cbase = chunk * CH;
      if (has_next) load_chunk(chunk + 1, kn);
      // ---- |V_i|: VB batches of VPT 16-byte pieces per thread, consumed one q-tile later than issued
      Frag vb[VPT];
      auto v_issue = [&](int b) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          const int p = (b * VPT + i) * NT + tid, key = cbase + p / PPR;
          vb[i].q = make_uint4(0, 0, 0, 0);
          if (key < Nc) vb[i].q = *reinterpret_cast<const uint4 *>(Vb + key * row_bytes + (p % PPR) * 16);
        }
      };
      auto v_consume = [&](int b) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          const int p = (b * VPT + i) * NT + tid, key = cbase + p / PPR;
          float ss = 0.f;
#pragma unroll
          for (int e = 0; e < EPC; ++e) {
            float x = frag_elem<DT>(vb[i], e);
            ss = fmaf(x, x, ss);
          }
#pragma unroll
          for (int sft = PPR / 2; sft >= 1; sft >>= 1) ss += __shfl_xor(ss, sft);
          if (p % PPR == 0 && key < Nc) vnorm[key] = sqrtf(ss);
        }
      };
      if (use_v) v_issue(0);

      // ---- key norms and the sum of normalised keys
      {
        float inv[TPW];
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
          const int key = cbase + (wave * TPW + j) * 32 + l32;
          float ss = 0.f;
#pragma unroll
          for (int c = 0; c < NCHK; ++c)
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
              float v = frag_elem<DT>(kf[j][c], e);
              ss = fmaf(v, v, ss);
            }
          ss += __shfl_xor(ss, 32);
          const bool valid = key < N;
          inv[j] = valid ? 1.f / fmaxf(sqrtf(ss), 1e-30f) : 0.f;
          if (valid && half == 0) invnorm[key] = inv[j];
        }
        // Groups of 32 accumulators (to bound register use).  Fixed-order butterfly over the 32
        // lanes of a half: every step halves the number of accumulators a lane carries; a lane
        // ends with one, summed over all 32 keys.
        constexpr int NG = 32, NGRP = NE / NG, CG = NCHK / NGRP;
#pragma unroll
        for (int grp = 0; grp < NGRP; ++grp) {
          float ks[NG];
#pragma unroll
          for (int e = 0; e < NG; ++e) ks[e] = 0.f;
#pragma unroll
          for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int c = 0; c < CG; ++c)
#pragma unroll
              for (int e = 0; e < EPC; ++e)
                ks[c * EPC + e] = fmaf(inv[j], frag_elem<DT>(kf[j][grp * CG + c], e), ks[c * EPC + e]);
          int n = NG, start = 0;
#pragma unroll
          for (int sft = 16; sft >= 1; sft >>= 1) {
            const int hn = n >> 1;
            const bool up = (lane & sft) != 0;
#pragma unroll
            for (int i = 0; i < hn; ++i) {
              float send = up ? ks[i] : ks[i + hn];
              float keep = up ? ks[i + hn] : ks[i];
              ks[i] = keep + __shfl_xor(send, sft);
            }
            start += up ? hn : 0;
            n = hn;
          }
#pragma unroll
          for (int i = 0; i < NG / 32; ++i) {
            int e = start + i, c = grp * CG + e / EPC, jj = e % EPC;
            ks_s[wave * D + (2 * c + half) * EPC + jj] += ks[i];    // this lane owns the slot
          }
        }
      }

      // ---- softmax statistics: keys on the MFMA output rows, query rows on the columns (lane % 32)
      for (int t = 0; t < s.QT; ++t) {
        Frag qf[NCHK];
#pragma unroll
        for (int c = 0; c < NCHK; ++c) qf[c].q = qs[(t * NCHK + c) * 64 + frag_slot(c, half, l32)];
        const int row = t * 32 + l32;
        const int lim = s.causal ? Nc + row % s.W : N - 1;   // last key this row attends to
        float2 ml = ml_s[wave * QTR + t * 32 + l32 + 0 * half];
        float m = ml.x, l = ml.y;
        if (half) { m = -INFINITY; l = 0.f; }                // the running pair lives in half 0
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
          const int tb = cbase + (wave * TPW + j) * 32;
          if (tb >= N) continue;
          f32x16 acc;
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
          for (int c = 0; c < NCHK; ++c) acc = mma<DT>(kf[j][c], qf[c], acc);
          if (tb + 31 > free_limit) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              int kidx = tb + 8 * (i >> 2) + 4 * half + (i & 3);
              if (kidx > lim) acc[i] = -INFINITY;
            }
          }
          float tmax = fmaxf(acc[0], acc[1]);
#pragma unroll
          for (int i = 2; i < 16; i += 2) tmax = fmaxf(fmaxf(tmax, acc[i]), acc[i + 1]);
          const float mn = fmaxf(m, tmax * c2);              // c2 > 0: scaling commutes with max
          const float mu = (mn == -INFINITY) ? 0.f : mn;
          float sum = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(acc[i], c2, -mu));
          l = l * fast_exp2(m - mu) + sum;
          m = mn;
        }
        ml_merge(m, l, __shfl_xor(m, 32), __shfl_xor(l, 32));
        if (half == 0) ml_s[wave * QTR + row] = make_float2(m, l);
        if (use_v && t < VB) {
          v_consume(t);
          if (t + 1 < VB) v_issue(t + 1);
        }
      }
      if (use_v)
        for (int b = min(s.QT, VB); b < VB; ++b) {
          if (b > 0) v_issue(b);       // batch 0 was issued before the q-tile loop
          v_consume(b);
        }
    };

#if MIXKV_PREFETCH
    for (int it = 0; it < nit; it += 2) {
      do_chunk(c0 + it, it + 1 < nit, kfa, kfb);
      if (it + 1 < nit) do_chunk(c0 + it + 1, it + 2 < nit, kfb, kfa);
    }
#else
    for (int it = 0; it < nit; ++it) {
      if (it > 0) load_chunk(c0 + it, kfa);
      do_chunk(c0 + it, false, kfa, kfb);
    }
#endif
    __syncthreads();   // ml_s, ks_s complete

    // ---- run partials to global, waves folded in a fixed order
    float2 *part_ml = reinterpret_cast<float2 *>(ws + w.part_ml) + (unit0 * s.nchunks + item) * QTR;
    for (int r = tid; r < QTR; r += NT) {
      float m = -INFINITY, l = 0.f;
      for (int wv = 0; wv < WAVES; ++wv) {
        float2 p = ml_s[wv * QTR + r];
        ml_merge(m, l, p.x, p.y);
      }
      part_ml[r] = make_float2(m, l);
    }
    float *part_ks = reinterpret_cast<float *>(ws + w.part_ksum) + (unit0 * s.nchunks + item) * D;
    for (int d = tid; d < D; d += NT) {
      float a = 0.f;
      for (int wv = 0; wv < WAVES; ++wv) a += ks_s[wv * D + d];
      part_ks[d] = a;
    }
    item += nit;
  }
}

// ------------------------------------------------------------------------------------------------
// finalize_kernel: one workgroup per unit folds the per-run partials of stats_kernel, in run
// order, into the per-row exponent offsets b_r = max_r + log2(sum_r * G*W), the mean normalised
// key and the redundancy r (paper Sec. 3.3, Eq. 3-4).  It recomputes the work split of
// stats_kernel (grid size G over T items) to find the runs of its unit.  A kernel boundary orders
// it after every workgroup of stats_kernel, so no fences or atomics are needed.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void finalize_kernel(Shape s, LayerOutTable out, char *ws, Workspace w,
                                                      int64_t unit0, int nunits, int G) {
  __shared__ double red_s[4];
  __shared__ int g_lo_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NT = 256;
  const int ul = blockIdx.x;
  const int64_t unit = unit0 + ul;
  const UnitCoord uc = unit_coord(s, ul);
  const int QTR = s.QT * 32, D = s.D, N = s.N;
  const int64_t T = (int64_t)nunits * s.nchunks, first = (int64_t)ul * s.nchunks, last = first + s.nchunks;
  // Workgroup g of stats_kernel wrote, for this unit, one partial at slot max(start(g), first) if its
  // item range [start(g), start(g+1)) meets [first, last).  g_lo is the workgroup owning item `first`.
  if (tid == 0) {
    int64_t g = first * G / T;
    while (g > 0 && wg_first_item(g, G, T) > first) --g;
    while (wg_first_item(g + 1, G, T) <= first) ++g;
    g_lo_s = (int)g;
  }
  __syncthreads();
  const int g_lo = g_lo_s;
  const float2 *all_ml = reinterpret_cast<const float2 *>(ws + w.part_ml) + unit0 * s.nchunks * QTR;
  float *brow = reinterpret_cast<float *>(ws + w.brow) + unit * QTR;
  for (int r = tid; r < QTR; r += NT) {
    float m = -INFINITY, l = 0.f;
    for (int64_t g = g_lo; g < G; ++g) {
      const int64_t a = max(wg_first_item(g, G, T), first), b = min(wg_first_item(g + 1, G, T), last);
      if (a >= last) break;
      if (b <= a) continue;
      float2 p = all_ml[a * QTR + r];
      ml_merge(m, l, p.x, p.y);
    }
    brow[r] = (r < s.GW) ? m + log2f(l) + log2f((float)s.GW) : INFINITY;
  }
  const float *all_ks = reinterpret_cast<const float *>(ws + w.part_ksum) + unit0 * s.nchunks * D;
  float *kbar = reinterpret_cast<float *>(ws + w.kbar) + unit * D;
  double sq = 0.0;
  for (int d = tid; d < D; d += NT) {
    float a = 0.f;
    for (int64_t g = g_lo; g < G; ++g) {
      const int64_t ia = max(wg_first_item(g, G, T), first), ib = min(wg_first_item(g + 1, G, T), last);
      if (ia >= last) break;
      if (ib <= ia) continue;
      a += all_ks[ia * D + d];
    }
    kbar[d] = a / (float)N;
    sq += (double)a * (double)a;
  }
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) sq += __shfl_xor(sq, sft);
  if (lane == 0) red_s[wave] = sq;
  __syncthreads();
  if (tid == 0) {
    double tot = red_s[0] + red_s[1] + red_s[2] + red_s[3];
    // Eq. 4: (T^2 |Kbar|^2 - T) / (T (T - 1)) with T^2 |Kbar|^2 = |sum of normalised keys|^2
    float r = (float)((tot - (double)N) / ((double)N * (double)(N - 1)));
    reinterpret_cast<float *>(ws + w.rbar)[unit] = r;
    float *red_out = out.l[uc.layer].redundancy;
    if (red_out) red_out[uc.b * s.hkv + uc.h] = r;
  }
}

// ------------------------------------------------------------------------------------------------
// attn_kernel: second pass over K.
//   a_i   = (1 / (G*W)) * sum over window rows of softmax weights on key i   (Sec. 3.2, extrinsic)
//   sdiv_i = -(K_i . Kbar) / |K_i|                                          (Sec. 3.2, diversity)
// Query rows on the MFMA output rows, keys on the columns: the sum over rows is a register sum.
// The mean key rides along as one more tile of "query" rows (split hi + lo for bf16 so that the
// dot product keeps fp32 accuracy).
// ------------------------------------------------------------------------------------------------
template <int DT, int D, int WAVES, int TPW>
__global__ __launch_bounds__(WAVES * 64, 2) void attn_kernel(Shape s, LayerInTable in, char *ws, Workspace w,
                                                         int64_t unit0, int nunits) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC);
  constexpr int NT = WAVES * 64, CH = WAVES * TPW * 32;
  extern __shared__ uint4 smem[];
  const int QTR = s.QT * 32;
  uint4 *qs = smem;                                                          // [(QT + 1) * NCHK * 64]
  float *brow_s = reinterpret_cast<float *>(smem + (s.QT + 1) * NCHK * 64);  // [QTR]
  int *lim_s = reinterpret_cast<int *>(brow_s + QTR);                        // [QTR]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int N = s.N, Nc = s.Nc;
  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;
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
    const float *invnorm = reinterpret_cast<const float *>(ws + w.invnorm) + unit * s.Npad;
    float *araw = reinterpret_cast<float *>(ws + w.araw) + unit * s.Npad;
    float *sdiv = reinterpret_cast<float *>(ws + w.sdiv) + unit * s.Npad;

    Frag kfa[TPW][NCHK], kfb[TPW][NCHK];
    auto load_chunk = [&](int chunk, Frag (&kf)[TPW][NCHK]) {
#pragma unroll
      for (int j = 0; j < TPW; ++j) {
        const int key = chunk * CH + (wave * TPW + j) * 32 + l32;
        load_key_tile<DT, D>(Kb, row_bytes, min(key, N - 1), half, kf[j]);
      }
    };
    load_chunk(c0, kfa);                   // in flight while the queries are staged

    __syncthreads();                       // the previous run is done with LDS
    stage_queries<DT, D>(s, Qb, qs, tid, NT);
    {
      // extra tile: row 0 (and row 1 for bf16) carry the mean normalised key
      const float *kbar = reinterpret_cast<const float *>(ws + w.kbar) + unit * D;
      uint4 *xt = qs + s.QT * NCHK * 64;
      for (int p = tid; p < NCHK * 64; p += NT) {
        const int c = p >> 6, ln = p & 63, row = ln & 31, hf = ln >> 5;
        Frag f;
        f.q = make_uint4(0, 0, 0, 0);
        if (row < 2) {
          const float *src = kbar + (2 * c + hf) * EPC;
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
            if (row == 0)
#pragma unroll
              for (int e = 0; e < EPC; ++e) f.f[e] = src[e];
          }
        }
        xt[c * 64 + frag_slot(c, hf, row)] = f.q;
      }
      const float *brow = reinterpret_cast<const float *>(ws + w.brow) + unit * QTR;
      for (int r = tid; r < QTR; r += NT) {
        brow_s[r] = brow[r];
        lim_s[r] = s.causal ? Nc + r % s.W : N - 1;
      }
    }
    __syncthreads();

    auto do_chunk = [&](int chunk, bool has_next, Frag (&kf)[TPW][NCHK], Frag (&kn)[TPW][NCHK]) {
      const int cbase = chunk * CH;
      if (has_next) load_chunk(chunk + 1, kn);
      float colsum[TPW];
#pragma unroll
      for (int j = 0; j < TPW; ++j) colsum[j] = 0.f;
      for (int t = 0; t < s.QT; ++t) {
        Frag qf[NCHK];
#pragma unroll
        for (int c = 0; c < NCHK; ++c) qf[c].q = qs[(t * NCHK + c) * 64 + frag_slot(c, half, l32)];
        float nb[16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float4 b4 = *reinterpret_cast<const float4 *>(&brow_s[t * 32 + 8 * k + 4 * half]);
          nb[4 * k + 0] = -b4.x; nb[4 * k + 1] = -b4.y; nb[4 * k + 2] = -b4.z; nb[4 * k + 3] = -b4.w;
        }
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
          const int tb = cbase + (wave * TPW + j) * 32;
          if (tb >= N) continue;
          f32x16 acc;
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
          for (int c = 0; c < NCHK; ++c) acc = mma<DT>(qf[c], kf[j][c], acc);
          float sum = 0.f;
          if (tb + 31 > free_limit) {
            const int key = tb + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int row = t * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
              float p = fast_exp2(fmaf(acc[i], c2, nb[i]));
              sum += (key <= lim_s[row]) ? p : 0.f;
            }
          } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(acc[i], c2, nb[i]));
          }
          colsum[j] += sum;
        }
      }
      // diversity dot products and write-out
      Frag qf[NCHK];
#pragma unroll
      for (int c = 0; c < NCHK; ++c) qf[c].q = qs[(s.QT * NCHK + c) * 64 + frag_slot(c, half, l32)];
#pragma unroll
      for (int j = 0; j < TPW; ++j) {
        const int tb = cbase + (wave * TPW + j) * 32;
        if (tb >= N) continue;
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int c = 0; c < NCHK; ++c) acc = mma<DT>(qf[c], kf[j][c], acc);
        const float dot = acc[0] + acc[1];                       // rows 0 and 1 live in half 0
        const float a = colsum[j] + __shfl_xor(colsum[j], 32);
        const int key = tb + l32;
        if (half == 0 && key < Nc) {
          araw[key] = a;
          sdiv[key] = -dot * invnorm[key];
        }
      }
    };

#if MIXKV_PREFETCH
    for (int it = 0; it < nit; it += 2) {
      do_chunk(c0 + it, it + 1 < nit, kfa, kfb);
      if (it + 1 < nit) do_chunk(c0 + it + 1, it + 2 < nit, kfb, kfa);
    }
#else
    for (int it = 0; it < nit; ++it) {
      if (it > 0) load_chunk(c0 + it, kfa);
      do_chunk(c0 + it, false, kfa, kfb);
    }
#endif
    item += nit;
  }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
constexpr int kWaves = 4;
constexpr int kWgPerCu = 2;           // resident workgroups per CU the grid is sized for
// Key tiles per wave: two where a tile's fragments take 32 registers, one for f32 with D = 128.
template <int DT, int D> struct Tpw { static constexpr int v = (D * Tr<DT>::EB > 256) ? 1 : 2; };

int stream_chunk_keys(int dtype, int D) {
  const int tpw = (D * (dtype == MIXKV_BF16 ? 2 : 4) > 256) ? 1 : 2;
  return kWaves * tpw * kTileKeys;
}

// Grid of the two streaming kernels: enough workgroups to fill the chip once, never more than items.
int stream_grid(const Shape &s, int nunits, int num_cus) {
  const int64_t T = (int64_t)nunits * s.nchunks;
  const int64_t cap = (int64_t)num_cus * kWgPerCu;
  return (int)(T < cap ? T : cap);
}

template <int DT, int D>
static hipError_t launch_stats_t(const Shape &s, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                                 int nunits, int grid, hipStream_t st) {
  constexpr int NCHK = D / (2 * Tr<DT>::EPC);
  const int QTR = s.QT * 32;
  size_t lds = (size_t)s.QT * NCHK * 1024 + (size_t)kWaves * QTR * 8 + (size_t)kWaves * D * 4;
  auto kern = stats_kernel<DT, D, kWaves, Tpw<DT, D>::v>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kWaves * 64), lds, st, s, in, ws, w, unit0, nunits);
  return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_attn_t(const Shape &s, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                                int nunits, int grid, hipStream_t st) {
  constexpr int NCHK = D / (2 * Tr<DT>::EPC);
  const int QTR = s.QT * 32;
  size_t lds = (size_t)(s.QT + 1) * NCHK * 1024 + (size_t)QTR * 8;
  auto kern = attn_kernel<DT, D, kWaves, Tpw<DT, D>::v>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kWaves * 64), lds, st, s, in, ws, w, unit0, nunits);
  return hipGetLastError();
}

hipError_t launch_stats(const Shape &s, int dtype, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                        int nunits, int grid, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_stats_t<MIXKV_BF16, 128>(s, in, ws, w, unit0, nunits, grid, st);
    return launch_stats_t<MIXKV_BF16, 64>(s, in, ws, w, unit0, nunits, grid, st);
  }
  if (s.D == 128) return launch_stats_t<MIXKV_F32, 128>(s, in, ws, w, unit0, nunits, grid, st);
  return launch_stats_t<MIXKV_F32, 64>(s, in, ws, w, unit0, nunits, grid, st);
}

hipError_t launch_finalize(const Shape &s, const LayerOutTable &out, char *ws, const Workspace &w, int64_t unit0,
                           int nunits, int grid, hipStream_t st) {
  hipLaunchKernelGGL(finalize_kernel, dim3(nunits), dim3(256), 0, st, s, out, ws, w, unit0, nunits, grid);
  return hipGetLastError();
}

hipError_t launch_attn(const Shape &s, int dtype, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                       int nunits, int grid, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_attn_t<MIXKV_BF16, 128>(s, in, ws, w, unit0, nunits, grid, st);
    return launch_attn_t<MIXKV_BF16, 64>(s, in, ws, w, unit0, nunits, grid, st);
  }
  if (s.D == 128) return launch_attn_t<MIXKV_F32, 128>(s, in, ws, w, unit0, nunits, grid, st);
  return launch_attn_t<MIXKV_F32, 64>(s, in, ws, w, unit0, nunits, grid, st);
}

}  // namespace mixkv
