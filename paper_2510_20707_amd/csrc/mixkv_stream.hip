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

// Stage the [QT*32, D] query block of one KV head into LDS in fragment order:
// fragment (t, c) is 64 lanes x 16 bytes, lane = half * 32 + row % 32.  Rows >= GW are zero.
template <int DT, int D>
__device__ __forceinline__ void stage_queries(const Shape &s, const char *Qb, uint4 *qs, int tid, int nthreads) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), PPR = D * EB / 16;
  const int pieces = s.QT * 32 * PPR;
  for (int p = tid; p < pieces; p += nthreads) {
    int row = p / PPR, piece = p - row * PPR;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < s.GW) v = *reinterpret_cast<const uint4 *>(Qb + ((int64_t)row * D) * EB + piece * 16);
    int c = piece >> 1, half = piece & 1;
    qs[((row >> 5) * NCHK + c) * 64 + half * 32 + (row & 31)] = v;
  }
}

template <int DT, int D>
__device__ __forceinline__ void load_key_tile(const char *Kb, int64_t row_bytes, int key, int half, Frag *kf) {
  constexpr int EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC);
  const char *p = Kb + key * row_bytes + half * 16;
#pragma unroll
  for (int c = 0; c < NCHK; ++c) kf[c].q = *reinterpret_cast<const uint4 *>(p + c * 32);
}

// ------------------------------------------------------------------------------------------------
// stats_kernel: first pass over K (and the only pass over V).
//   * running softmax (max, sum) of every window-query row over this workgroup's keys;
//   * 1/|K_i| and the partial sum of the normalised keys (paper Sec. 3.2 diversity metrics,
//     Sec. 3.3 Eq. 3-4: only the sum of normalised keys is needed, never the T x T matrix);
//   * |V_i| (Sec. 3.2, VNorm intrinsic importance).
// The last workgroup of a unit to finish folds the partials into the per-row exponent offsets,
// the mean normalised key and the redundancy r (Eq. 4).
// ------------------------------------------------------------------------------------------------
template <int DT, int D, int WAVES, int TPW>
__global__ __launch_bounds__(WAVES * 64) void stats_kernel(Shape s, LayerInTable in, LayerOutTable out, char *ws,
                                                          Workspace w, int64_t unit0) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), NE = D / 2, PPR = D * EB / 16;
  constexpr int NT = WAVES * 64;
  extern __shared__ uint4 smem[];
  const int QTR = s.QT * 32;
  uint4 *qs = smem;                                                       // [QT * NCHK * 64]
  float2 *ml_s = reinterpret_cast<float2 *>(smem + s.QT * NCHK * 64);     // [WAVES][QTR]
  float *ks_s = reinterpret_cast<float *>(ml_s + WAVES * QTR);            // [WAVES][D]
  __shared__ int ticket_s;
  __shared__ double red_s[NT / 64];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int chunk = blockIdx.x % s.nchunks, ul = blockIdx.x / s.nchunks;
  const int64_t unit = unit0 + ul;
  const UnitCoord uc = unit_coord(s, ul);
  const LayerIn L = in.l[uc.layer];
  const int64_t head_off = ((int64_t)uc.b * L.sb + (int64_t)uc.h * L.sh) * EB;
  const char *Kb = reinterpret_cast<const char *>(L.K) + head_off;
  const char *Vb = reinterpret_cast<const char *>(L.V) + head_off;
  const char *Qb = reinterpret_cast<const char *>(L.Q) + ((int64_t)(uc.b * s.hq + uc.h * s.G) * s.W * D) * EB;
  const int64_t row_bytes = L.sn * EB;
  const int N = s.N, Nc = s.Nc;
  const int cbase = chunk * s.chunk;

  stage_queries<DT, D>(s, Qb, qs, tid, NT);

  // ---- this wave's key tiles: fragments, norms, sum of normalised keys
  Frag kf[TPW][NCHK];
  float ks[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) ks[e] = 0.f;
  float *invnorm = reinterpret_cast<float *>(ws + w.invnorm) + unit * s.Npad;
#pragma unroll
  for (int j = 0; j < TPW; ++j) {
    const int tb = cbase + (wave * TPW + j) * 32;
    const int key = tb + l32;
    load_key_tile<DT, D>(Kb, row_bytes, min(key, N - 1), half, kf[j]);
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
    const float inv = valid ? 1.f / fmaxf(sqrtf(ss), 1e-30f) : 0.f;
    if (valid && half == 0) invnorm[key] = inv;
#pragma unroll
    for (int c = 0; c < NCHK; ++c)
#pragma unroll
      for (int e = 0; e < EPC; ++e) ks[c * EPC + e] = fmaf(inv, frag_elem<DT>(kf[j][c], e), ks[c * EPC + e]);
  }
  // Fixed-order butterfly over the 32 lanes of a half: every step halves the number of
  // accumulators a lane carries; a lane ends with NE/32 of them, summed over all 32 keys.
  {
    int n = NE, start = 0;
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
    for (int i = 0; i < NE / 32; ++i) {
      int e = start + i, c = e / EPC, jj = e - c * EPC;
      ks_s[wave * D + (2 * c + half) * EPC + jj] = ks[i];
    }
  }
  __syncthreads();   // queries staged, ks_s complete

  // ---- softmax statistics: keys on the MFMA output rows, query rows on the columns (lane % 32)
  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;      // keys <= this are visible to every row
  for (int t = 0; t < s.QT; ++t) {
    Frag qf[NCHK];
#pragma unroll
    for (int c = 0; c < NCHK; ++c) qf[c].q = qs[(t * NCHK + c) * 64 + lane];
    const int row = t * 32 + l32;
    const int lim = s.causal ? Nc + row % s.W : N - 1;   // last key this row attends to
    float m = -INFINITY, l = 0.f;
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
      const int tb = cbase + (wave * TPW + j) * 32;
      if (tb >= N) continue;
      f32x16 acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
      for (int c = 0; c < NCHK; ++c) acc = mma<DT>(kf[j][c], qf[c], acc);
      float x[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = acc[i] * c2;
      if (tb + 31 > free_limit) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int kidx = tb + 8 * (i >> 2) + 4 * half + (i & 3);
          if (kidx > lim) x[i] = -INFINITY;
        }
      }
      float tmax = x[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, x[i]);
      const float mn = fmaxf(m, tmax);
      const float mu = (mn == -INFINITY) ? 0.f : mn;
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) sum += fast_exp2(x[i] - mu);
      l = l * fast_exp2(m - mu) + sum;
      m = mn;
    }
    ml_merge(m, l, __shfl_xor(m, 32), __shfl_xor(l, 32));
    if (half == 0) ml_s[wave * QTR + row] = make_float2(m, l);
  }

  // ---- |V_i| for the candidates of this chunk: PPR lanes per row, 16 bytes each
  if (s.intrinsic == MIXKV_INTRINSIC_VNORM) {
    float *vnorm = reinterpret_cast<float *>(ws + w.vnorm) + unit * s.Npad;
    const int piece = tid % PPR, rsub = tid / PPR;
    for (int r = rsub; r < s.chunk; r += NT / PPR) {
      const int key = cbase + r;
      Frag v;
      v.q = make_uint4(0, 0, 0, 0);
      if (key < Nc) v.q = *reinterpret_cast<const uint4 *>(Vb + key * row_bytes + piece * 16);
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        float x = frag_elem<DT>(v, e);
        ss = fmaf(x, x, ss);
      }
#pragma unroll
      for (int sft = PPR / 2; sft >= 1; sft >>= 1) ss += __shfl_xor(ss, sft);
      if (piece == 0 && key < Nc) vnorm[key] = sqrtf(ss);
    }
  }
  __syncthreads();   // ml_s complete

  // ---- workgroup partials to global, in a fixed order
  float2 *part_ml = reinterpret_cast<float2 *>(ws + w.part_ml) + (unit * s.nchunks + chunk) * QTR;
  for (int r = tid; r < QTR; r += NT) {
    float m = -INFINITY, l = 0.f;
    for (int wv = 0; wv < WAVES; ++wv) {
      float2 p = ml_s[wv * QTR + r];
      ml_merge(m, l, p.x, p.y);
    }
    part_ml[r] = make_float2(m, l);
  }
  float *part_ks = reinterpret_cast<float *>(ws + w.part_ksum) + (unit * s.nchunks + chunk) * D;
  for (int d = tid; d < D; d += NT) {
    float a = 0.f;
    for (int wv = 0; wv < WAVES; ++wv) a += ks_s[wv * D + d];
    part_ks[d] = a;
  }

  // ---- last workgroup of the unit folds the partials
  __threadfence();
  __syncthreads();
  if (tid == 0) ticket_s = atomicAdd(reinterpret_cast<int *>(ws + w.counters) + unit, 1);
  __syncthreads();
  if (ticket_s != s.nchunks - 1) return;
  __threadfence();

  const float2 *all_ml = reinterpret_cast<const float2 *>(ws + w.part_ml) + unit * s.nchunks * QTR;
  float *brow = reinterpret_cast<float *>(ws + w.brow) + unit * QTR;
  for (int r = tid; r < QTR; r += NT) {
    float m = -INFINITY, l = 0.f;
    for (int ch = 0; ch < s.nchunks; ++ch) {
      float2 p = all_ml[ch * QTR + r];
      ml_merge(m, l, p.x, p.y);
    }
    brow[r] = (r < s.GW) ? m + log2f(l) + log2f((float)s.GW) : INFINITY;
  }
  const float *all_ks = reinterpret_cast<const float *>(ws + w.part_ksum) + unit * s.nchunks * D;
  float *kbar = reinterpret_cast<float *>(ws + w.kbar) + unit * D;
  double sq = 0.0;
  for (int d = tid; d < D; d += NT) {
    float a = 0.f;
    for (int ch = 0; ch < s.nchunks; ++ch) a += all_ks[ch * D + d];
    kbar[d] = a / (float)N;
    sq += (double)a * (double)a;
  }
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) sq += __shfl_xor(sq, sft);
  if (lane == 0) red_s[wave] = sq;
  __syncthreads();
  if (tid == 0) {
    double tot = 0.0;
    for (int wv = 0; wv < WAVES; ++wv) tot += red_s[wv];
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
__global__ __launch_bounds__(WAVES * 64) void attn_kernel(Shape s, LayerInTable in, char *ws, Workspace w,
                                                         int64_t unit0) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), PPR = D * EB / 16;
  constexpr int NT = WAVES * 64;
  extern __shared__ uint4 smem[];
  const int QTR = s.QT * 32;
  uint4 *qs = smem;                                                          // [(QT + 1) * NCHK * 64]
  float *brow_s = reinterpret_cast<float *>(smem + (s.QT + 1) * NCHK * 64);  // [QTR]
  int *lim_s = reinterpret_cast<int *>(brow_s + QTR);                        // [QTR]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int chunk = blockIdx.x % s.nchunks, ul = blockIdx.x / s.nchunks;
  const int64_t unit = unit0 + ul;
  const UnitCoord uc = unit_coord(s, ul);
  const LayerIn L = in.l[uc.layer];
  const char *Kb = reinterpret_cast<const char *>(L.K) + ((int64_t)uc.b * L.sb + (int64_t)uc.h * L.sh) * EB;
  const char *Qb = reinterpret_cast<const char *>(L.Q) + ((int64_t)(uc.b * s.hq + uc.h * s.G) * s.W * D) * EB;
  const int64_t row_bytes = L.sn * EB;
  const int N = s.N, Nc = s.Nc;
  const int cbase = chunk * s.chunk;

  // keys first, so the loads are in flight while the queries are staged
  Frag kf[TPW][NCHK];
#pragma unroll
  for (int j = 0; j < TPW; ++j) {
    const int key = cbase + (wave * TPW + j) * 32 + l32;
    load_key_tile<DT, D>(Kb, row_bytes, min(key, N - 1), half, kf[j]);
  }

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
      xt[p] = f.q;
    }
    const float *brow = reinterpret_cast<const float *>(ws + w.brow) + unit * QTR;
    for (int r = tid; r < QTR; r += NT) {
      brow_s[r] = brow[r];
      lim_s[r] = s.causal ? Nc + r % s.W : N - 1;
    }
  }
  __syncthreads();

  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;
  float colsum[TPW];
#pragma unroll
  for (int j = 0; j < TPW; ++j) colsum[j] = 0.f;

  for (int t = 0; t < s.QT; ++t) {
    Frag qf[NCHK];
#pragma unroll
    for (int c = 0; c < NCHK; ++c) qf[c].q = qs[(t * NCHK + c) * 64 + lane];
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
  {
    Frag qf[NCHK];
#pragma unroll
    for (int c = 0; c < NCHK; ++c) qf[c].q = qs[(s.QT * NCHK + c) * 64 + lane];
    const float *invnorm = reinterpret_cast<const float *>(ws + w.invnorm) + unit * s.Npad;
    float *araw = reinterpret_cast<float *>(ws + w.araw) + unit * s.Npad;
    float *sdiv = reinterpret_cast<float *>(ws + w.sdiv) + unit * s.Npad;
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
  }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
constexpr int kWaves = 4, kTPW = 2;   // 256 keys per workgroup

int stream_chunk_keys() { return kWaves * kTPW * kTileKeys; }

template <int DT, int D>
static hipError_t launch_stats_t(const Shape &s, const LayerInTable &in, const LayerOutTable &out, char *ws,
                                 const Workspace &w, int64_t unit0, int nunits, hipStream_t st) {
  constexpr int NCHK = D / (2 * Tr<DT>::EPC);
  const int QTR = s.QT * 32;
  size_t lds = (size_t)s.QT * NCHK * 1024 + (size_t)kWaves * QTR * 8 + (size_t)kWaves * D * 4;
  auto kern = stats_kernel<DT, D, kWaves, kTPW>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(nunits * s.nchunks)), dim3(kWaves * 64), lds, st, s, in, out, ws, w, unit0);
  return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_attn_t(const Shape &s, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                                int nunits, hipStream_t st) {
  constexpr int NCHK = D / (2 * Tr<DT>::EPC);
  const int QTR = s.QT * 32;
  size_t lds = (size_t)(s.QT + 1) * NCHK * 1024 + (size_t)QTR * 8;
  auto kern = attn_kernel<DT, D, kWaves, kTPW>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(nunits * s.nchunks)), dim3(kWaves * 64), lds, st, s, in, ws, w, unit0);
  return hipGetLastError();
}

hipError_t launch_stats(const Shape &s, int dtype, const LayerInTable &in, const LayerOutTable &out, char *ws,
                        const Workspace &w, int64_t unit0, int nunits, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_stats_t<MIXKV_BF16, 128>(s, in, out, ws, w, unit0, nunits, st);
    return launch_stats_t<MIXKV_BF16, 64>(s, in, out, ws, w, unit0, nunits, st);
  }
  if (s.D == 128) return launch_stats_t<MIXKV_F32, 128>(s, in, out, ws, w, unit0, nunits, st);
  return launch_stats_t<MIXKV_F32, 64>(s, in, out, ws, w, unit0, nunits, st);
}

hipError_t launch_attn(const Shape &s, int dtype, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                       int nunits, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_attn_t<MIXKV_BF16, 128>(s, in, ws, w, unit0, nunits, st);
    return launch_attn_t<MIXKV_BF16, 64>(s, in, ws, w, unit0, nunits, st);
  }
  if (s.D == 128) return launch_attn_t<MIXKV_F32, 128>(s, in, ws, w, unit0, nunits, st);
  return launch_attn_t<MIXKV_F32, 64>(s, in, ws, w, unit0, nunits, st);
}

}  // namespace mixkv
