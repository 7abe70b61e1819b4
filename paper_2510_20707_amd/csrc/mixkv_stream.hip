// The two kernels that stream the cache: window-attention statistics + key/value statistics
// (stats_kernel) and the normalised attention column sums + diversity dot products (attn_kernel).
//
// Both are MFMA kernels built the same way.  A workgroup walks runs of consecutive key chunks of
// one unit (one layer, batch item and KV head).  The G*W window-query rows are split into tiles of
// 32 and every wave keeps its TQ tiles in registers for the whole run ("query-stationary"); the
// keys stream through LDS: each chunk is fetched with direct global->LDS loads (whole rows,
// bank-rotated) into one of two buffers while the other is being consumed by all waves.
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
#include "mixkv_wave.h"

#ifdef MIXKV_TIMING
// Developer aid, compiled out by default: cycle totals of wave 0 of every workgroup of attn_kernel.
__device__ unsigned long long mixkv_dbg[1024 * 16];
#define TSTAMP(v) unsigned long long v = __builtin_readcyclecounter()
#define TACC(slot, a, b) tacc[slot] += (b) - (a)
#define TDECL unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define TFLUSH do { if (threadIdx.x == 0) for (int i_ = 0; i_ < 8; ++i_) mixkv_dbg[blockIdx.x * 16 + 8 + i_] = tacc[i_]; } while (0)
extern "C" int mixkv_debug_read(unsigned long long *host, int clear) {
  if (hipMemcpyFromSymbol(host, HIP_SYMBOL(mixkv_dbg), sizeof(mixkv_dbg)) != hipSuccess) return 1;
  if (clear) { static unsigned long long z[1024 * 16]; return hipMemcpyToSymbol(HIP_SYMBOL(mixkv_dbg), z, sizeof(z)) != hipSuccess; }
  return 0;
}
#else
#define TSTAMP(v)
#define TACC(slot, a, b)
#define TDECL
#define TFLUSH
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

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

// Key tiles per chunk: at most four, and few enough that two workgroups (two key buffers, the
// mean-key tile and the column-sum scratch each) fit in the 160 KB of LDS of a CU.
__host__ __device__ constexpr int chunk_tiles(int dtype, int D) {
  const int tile_bytes = D * (dtype == MIXKV_BF16 ? 2 : 4) * 32;
  return tile_bytes <= 8192 ? 4 : 1;
}

// Work split of the two streaming kernels.  An item is one chunk of one unit (item = unit_local *
// nchunks + chunk); workgroup g of G owns the contiguous items [g*T/G, (g+1)*T/G) and walks them in
// runs that stay inside one unit.  Run (g, unit_local) writes its partials to slot g + unit_local,
// which is unique because both grow along the global order of runs.
__device__ __forceinline__ int64_t wg_first_item(int64_t g, int64_t G, int64_t T) { return g * T / G; }

// LDS image of a key tile: 32 rows of D*EB bytes, row-major, with the 16-byte pieces of row r
// stored at piece index (p ^ swz(r)).  The rotation makes the MFMA fragment reads (16 consecutive
// rows, one piece index) hit 16 different bank groups, while a direct-to-LDS load instruction
// (64 consecutive 16-byte slots) still covers whole rows of global memory.
template <int DT, int D>
__device__ __forceinline__ int tile_swz(int r) {
  constexpr int PPR = D * Tr<DT>::EB / 16;
  return PPR == 8 ? (r >> 1) & 7 : r & 15;
}

// Issue the direct-to-LDS loads of key tile k of the chunk that starts at key cbase.  Load j covers
// slots [64j, 64j+64) of the tile image; lane i fetches the piece that belongs in slot 64j + i.
// Waves take loads round-robin.  The address is a wave-uniform 64-bit base plus a 32-bit lane
// offset.  In the last chunk of a sequence, keys past N-1 re-read key N-1 (their results are
// masked or discarded).
template <int DT, int D, int WAVES>
__device__ __forceinline__ void fetch_tile(const char *Kb, int64_t row_bytes, int cbase, int k, int N, uint4 *buf,
                                           int wave, int lane) {
  constexpr int PPR = D * Tr<DT>::EB / 16, LOADS = 32 * PPR / 64;      // loads per tile
  constexpr int RPL = 64 / PPR > 0 ? 64 / PPR : 1;                      // rows per load (PPR <= 32)
  static_assert(PPR <= 64 && 64 % PPR == 0, "row pieces must divide a load");
  const int lrow = lane / PPR, lq = lane % PPR;
  const uint32_t rb = (uint32_t)row_bytes;
  const int tb = cbase + k * 32;
  uint4 *tile = buf + k * 32 * PPR;
  if (tb + 32 <= N) {
#pragma unroll
    for (int jj = 0; jj < (LOADS + WAVES - 1) / WAVES; ++jj) {
      const int j = jj * WAVES + wave;
      if (LOADS % WAVES != 0 && j >= LOADS) break;
      const char *base = Kb + (int64_t)(tb + j * RPL) * row_bytes;               // wave-uniform
      const uint32_t off = (uint32_t)lrow * rb + (uint32_t)((lq ^ tile_swz<DT, D>(j * RPL + lrow)) * 16);
      __builtin_amdgcn_global_load_lds((glb_void_t *)(base + off), (lds_void_t *)(tile + j * 64), 16, 0, 0);
    }
  } else {
#pragma unroll
    for (int jj = 0; jj < (LOADS + WAVES - 1) / WAVES; ++jj) {
      const int j = jj * WAVES + wave;
      if (LOADS % WAVES != 0 && j >= LOADS) break;
      const int row = j * RPL + lrow;
      const int krow = min(tb + row, N - 1);
      const char *src = Kb + (int64_t)krow * row_bytes + (lq ^ tile_swz<DT, D>(row)) * 16;
      __builtin_amdgcn_global_load_lds((glb_void_t *)src, (lds_void_t *)(tile + j * 64), 16, 0, 0);
    }
  }
}

template <int DT, int D, int WAVES>
__device__ __forceinline__ void fetch_chunk(const char *Kb, int64_t row_bytes, int cbase, int N, uint4 *buf, int wave,
                                            int lane) {
#pragma unroll
  for (int k = 0; k < chunk_tiles(DT, D); ++k) fetch_tile<DT, D, WAVES>(Kb, row_bytes, cbase, k, N, buf, wave, lane);
}

// Fragment c of key tile k for lane (row l32, half): piece 2c + half of row l32.
template <int DT, int D>
__device__ __forceinline__ uint4 read_key_frag(const uint4 *kb, int k, int c, int l32, int half) {
  constexpr int PPR = D * Tr<DT>::EB / 16;
  return kb[(k * 32 + l32) * PPR + ((2 * c + half) ^ tile_swz<DT, D>(l32))];
}

// ------------------------------------------------------------------------------------------------
// stats_kernel: first pass over K (and the only pass over V).
//   * running softmax (max, sum) of every window-query row over the run's keys: keys on the MFMA
//     output rows, query rows on the columns, so a lane follows one query row per tile;
//   * 1/|K_i| and the partial sum of the normalised keys (paper Sec. 3.2 diversity metrics,
//     Sec. 3.3 Eq. 3-4: only the sum of normalised keys is needed, never the T x T matrix);
//   * |V_i| (Sec. 3.2, VNorm intrinsic importance).
// Per-run partials go to the workspace; attn_kernel folds them at the start of its runs.
// ------------------------------------------------------------------------------------------------
template <int DT, int D, int WAVES, int TQ>
__global__ __launch_bounds__(WAVES * 64, 2) void stats_kernel(Shape s, LayerInTable in, char *ws, Workspace w,
                                                             int64_t unit0, int nunits, int64_t slot0) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC), NE = D / 2, PPR = D * EB / 16;
  constexpr int NT = WAVES * 64, KT = chunk_tiles(DT, D), CH = KT * 32, FRAGS = KT * NCHK;
  constexpr int VPT = (32 * PPR + NT - 1) / NT;           // V pieces per thread and key tile
  // Two separately declared key buffers: the compiler can then tell that reads of one do not
  // depend on the direct-to-LDS loads in flight into the other.
  __shared__ uint4 kbuf_a[FRAGS * 64], kbuf_b[FRAGS * 64];
  __shared__ float ks_s[WAVES * D];

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps its address math scalar
  const int N = s.N, Nc = s.Nc, QTR = s.QT * 32;
  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;      // keys <= this are visible to every row
  const int nq = max(0, min(TQ, s.QT - wave * TQ));  // query tiles this wave owns
  const bool use_v = s.intrinsic == MIXKV_INTRINSIC_VNORM;
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

    __syncthreads();                                   // the previous run is done with LDS
    fetch_chunk<DT, D, WAVES>(Kb, row_bytes, c0 * CH, N, kbuf_a, wave, lane);
    for (int d = lane; d < D; d += 64) ks_s[wave * D + d] = 0.f;

    // this wave's query tiles, in fragment form, for the whole run (tiles past QT are zero)
    Frag qf[TQ][NCHK];
    int lim[TQ];
    float m[TQ], l[TQ];
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
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

    // one chunk: its keys are in `kb`; the next chunk streams into `kn` meanwhile
    auto do_chunk = [&](int it, const uint4 *kb, uint4 *kn) {
      const int cbase = (c0 + it) * CH;
      __builtin_amdgcn_s_waitcnt(0);                   // this wave's share of the chunk has landed
      __syncthreads();                                 // ... and everybody else's; the other buffer is free
      const bool has_next = it + 1 < nit;

      // |V_i| rides along: the rows of key tile k are requested one tile ahead of their use, and
      // always *before* the slice of the next chunk's keys issued in the same tile step.  The
      // memory counter retires in order, so waiting for value rows only ever waits for key loads
      // that are at least one tile step old.
      Frag vb[VPT], vn[VPT];                           // rows in use / rows in flight
      auto v_issue = [&](int k) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          const int p = i * NT + tid, key = cbase + k * 32 + p / PPR;
          const bool on = p < 32 * PPR && key < Nc;
          uint4 v = *reinterpret_cast<const uint4 *>(Vb + (int64_t)(on ? key : 0) * row_bytes + (p % PPR) * 16);
          vn[i].q = on ? v : make_uint4(0, 0, 0, 0);
        }
      };
      auto v_consume = [&](int k) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          const int p = i * NT + tid, key = cbase + k * 32 + p / PPR;
          float ss = 0.f;
#pragma unroll
          for (int e = 0; e < EPC; ++e) {
            float x = frag_elem<DT>(vb[i], e);
            ss = fmaf(x, x, ss);
          }
          ss = seg_sum<PPR>(ss);                       // PPR consecutive lanes hold one row
          if (p % PPR == 0 && p < 32 * PPR && key < Nc) vnorm[key] = sqrtf(ss);
        }
      };
      if (use_v) v_issue(0);

#pragma unroll 1
      for (int k = 0; k < KT; ++k) {
        const int tb = cbase + k * 32;
        if (use_v) {
#pragma unroll
          for (int i = 0; i < VPT; ++i) vb[i] = vn[i];
          if (k + 1 < KT) v_issue(k + 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (has_next) fetch_tile<DT, D, WAVES>(Kb, row_bytes, cbase + CH, k, N, kn, wave, lane);
        __builtin_amdgcn_sched_barrier(0);
        if (tb < N) {
          Frag kf[NCHK];
#pragma unroll
          for (int c = 0; c < NCHK; ++c) kf[c].q = read_key_frag<DT, D>(kb, k, c, l32, half);

          // ---- softmax statistics of all TQ tiles; the MFMA chains are independent
          f32x16 acc[TQ];
#pragma unroll
          for (int q = 0; q < TQ; ++q)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[q][i] = 0.f;
#pragma unroll
          for (int c = 0; c < NCHK; ++c)
#pragma unroll
            for (int q = 0; q < TQ; ++q) acc[q] = mma<DT>(kf[c], qf[q][c], acc[q]);
          if (tb + 31 > free_limit) {                  // tile reaches into the window or past N: mask
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
            float tmax = fmaxf(acc[q][0], acc[q][1]);
#pragma unroll
            for (int i = 2; i < 16; i += 2) tmax = fmaxf(fmaxf(tmax, acc[q][i]), acc[q][i + 1]);
            const float mn = fmaxf(m[q], tmax * c2);          // c2 > 0: scaling commutes with max
            const float mu = (mn == -INFINITY) ? 0.f : mn;
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(acc[q][i], c2, -mu));
            l[q] = l[q] * fast_exp2(m[q] - mu) + sum;
            m[q] = mn;
          }

          // ---- key norms and the sum of normalised keys: one wave per tile, round-robin
          if ((k + it * KT) % WAVES == wave) {
            const int key = tb + l32;
            float ss = 0.f;
#pragma unroll
            for (int c = 0; c < NCHK; ++c)
#pragma unroll
              for (int e = 0; e < EPC; ++e) {
                float v = frag_elem<DT>(kf[c], e);
                ss = fmaf(v, v, ss);
              }
            ss += __shfl_xor(ss, 32);
            const bool valid = key < N;
            const float inv = valid ? 1.f / fmaxf(sqrtf(ss), 1e-30f) : 0.f;
            if (valid && half == 0) invnorm[key] = inv;
            // Groups of 32 accumulators (to bound register use).  Fixed-order butterfly over the
            // 32 lanes of a half: every step halves the number of accumulators a lane carries; a
            // lane ends with one, summed over all 32 keys.
            constexpr int NG = 32, NGRP = NE / NG, CG = NCHK / NGRP;
#pragma unroll
            for (int grp = 0; grp < NGRP; ++grp) {
              float ks[NG];
#pragma unroll
              for (int c = 0; c < CG; ++c)
#pragma unroll
                for (int e = 0; e < EPC; ++e) ks[c * EPC + e] = inv * frag_elem<DT>(kf[grp * CG + c], e);
              int n = NG, start = 0;
#pragma unroll
              for (int sft = 16; sft >= 1; sft >>= 1) {
                const int hn = n >> 1;
                const bool up = (lane & sft) != 0;
                const uint32_t um = up ? 0xffffffffu : 0u;    // bit select: keeps the accumulators in registers
#pragma unroll
                for (int i = 0; i < hn; ++i) {
                  const uint32_t lo = __float_as_uint(ks[i]), hi = __float_as_uint(ks[i + hn]);
                  const float send = __uint_as_float((lo & um) | (hi & ~um));
                  const float keep = __uint_as_float((hi & um) | (lo & ~um));
                  ks[i] = keep + __shfl_xor(send, sft);
                }
                start += up ? hn : 0;
                n = hn;
              }
              const int c = grp * CG + start / EPC, jj = start % EPC;
              ks_s[wave * D + (2 * c + half) * EPC + jj] += ks[0];    // this lane owns the slot
            }
          }
        }
        if (use_v) v_consume(k);
      }
    };
    for (int it = 0; it < nit; it += 2) {
      do_chunk(it, kbuf_a, kbuf_b);
      if (it + 1 < nit) do_chunk(it + 1, kbuf_b, kbuf_a);
    }

    // ---- run partials to global
    const int64_t slot = slot0 + blockIdx.x + ul;
    float2 *part_ml = reinterpret_cast<float2 *>(ws + w.part_ml) + slot * QTR;
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
      ml_merge(m[q], l[q], __shfl_xor(m[q], 32), __shfl_xor(l[q], 32));
      if (q < nq && half == 0) part_ml[(wave * TQ + q) * 32 + l32] = make_float2(m[q], l[q]);
    }
    __syncthreads();                                   // ks_s complete
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
// attn_kernel: second pass over K.
//   a_i    = (1 / (G*W)) * sum over window rows of softmax weights on key i   (Sec. 3.2, extrinsic)
//   kdot_i = K_i . Kbar; the mix kernel turns it into -(K_i . Kbar) / |K_i|   (Sec. 3.2, diversity)
// Query rows on the MFMA output rows, keys on the columns: a wave's sum over its rows is a register
// sum; the waves' partial column sums meet in LDS and are added in a fixed order.  The mean key is
// two more "query" rows (hi + lo bf16 halves, so the dot keeps fp32 accuracy).  When the padded
// query block has a spare tile they sit in its rows 0 and 1 and cost nothing; otherwise every wave
// applies a separate mean-key tile to every WAVES-th key tile.
//
// At the start of a run the workgroup folds the per-run partials that stats_kernel (grid G1) left
// for its unit, in run order: per-row exponent offsets b_r = max_r + log2(sum_r * G*W), the mean
// normalised key, and - in the workgroup that owns the unit's first chunk - the redundancy r
// (paper Sec. 3.3, Eq. 3-4).  The kernel boundary orders this after all of stats_kernel.
// ------------------------------------------------------------------------------------------------
template <int DT, int D, int WAVES, int TQ>
__global__ __launch_bounds__(WAVES * 64, 2) void attn_kernel(Shape s, LayerInTable in, LayerOutTable out, char *ws,
                                                            Workspace w, int64_t unit0, int nunits, int G1,
                                                            int64_t slot0) {
  constexpr int EB = Tr<DT>::EB, EPC = Tr<DT>::EPC, NCHK = D / (2 * EPC);
  constexpr int NT = WAVES * 64, KT = chunk_tiles(DT, D), CH = KT * 32, FRAGS = KT * NCHK;
  __shared__ uint4 kbuf_a[FRAGS * 64], kbuf_b[FRAGS * 64];   // separate objects, see stats_kernel
  __shared__ uint4 kbar_s[NCHK * 4];                         // mean-key rows 0/1 x halves, 16-byte pieces
  __shared__ float cs_s[2 * WAVES * CH];                     // [2][WAVES][CH] partial column sums
  __shared__ float nb_s[WAVES * TQ * 32];                    // -b_r per query row (-inf rows give weight 0)
  __shared__ int lim_s[WAVES * TQ * 32];                     // last key each query row attends to
  __shared__ float kbar_f[D];                                // mean normalised key
  __shared__ double red_s[WAVES];
  __shared__ int g_lo_s, g_hi_s;

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps its address math scalar
  const int N = s.N, Nc = s.Nc, QTR = s.QT * 32;
  const float c2 = s.scale_log2e;
  const int free_limit = s.causal ? Nc : N - 1;
  for (int r = tid; r < WAVES * TQ * 32; r += NT) lim_s[r] = s.causal ? Nc + r % s.W : N - 1;
  // the mean key rides in rows 0/1 of the first tile past the live rows, if the block has one
  const bool spare = s.QT < WAVES * TQ;
  const int kb_wave = s.QT / TQ, kb_q = s.QT % TQ;
  const int64_t T = (int64_t)nunits * s.nchunks;
  int64_t item = wg_first_item(blockIdx.x, gridDim.x, T);
  const int64_t item_end = wg_first_item(blockIdx.x + 1, gridDim.x, T);
  TDECL;
#ifdef MIXKV_TIMING
  if (threadIdx.x == 0) { mixkv_dbg[blockIdx.x * 16 + 4] = wall_clock64(); mixkv_dbg[blockIdx.x * 16 + 6] = __builtin_readcyclecounter(); }
#endif

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

    TSTAMP(p0);
    __syncthreads();                                   // the previous run is done with LDS
    fetch_chunk<DT, D, WAVES>(Kb, row_bytes, c0 * CH, N, kbuf_a, wave, lane);
    TSTAMP(p1);

    // ---- fold the partials of stats_kernel for this unit.  Workgroup g of its grid owned the items
    // [g*T1/G1, (g+1)*T1/G1) and wrote one partial per unit it touched, at slot g + unit_local.
    if (tid == 0) {
      const int64_t T1 = (int64_t)nunits * s.nchunks, first = (int64_t)ul * s.nchunks, last = first + s.nchunks;
      int64_t g = first * G1 / T1;
      while (g > 0 && wg_first_item(g, G1, T1) > first) --g;
      while (wg_first_item(g + 1, G1, T1) <= first) ++g;
      g_lo_s = (int)g;
      while (g + 1 < G1 && wg_first_item(g + 1, G1, T1) < last) ++g;
      g_hi_s = (int)g;
    }
    __syncthreads();
    {
      const int g_lo = g_lo_s, g_hi = g_hi_s;
      const float2 *all_ml = reinterpret_cast<const float2 *>(ws + w.part_ml) + (slot0 + ul) * QTR;
      for (int r = tid; r < WAVES * TQ * 32; r += NT) {
        float b = INFINITY;                            // rows past G*W: weight 0
        if (r < s.GW) {
          float m = -INFINITY, l = 0.f;
          for (int g0 = g_lo; g0 <= g_hi; g0 += 4) {   // batches of four independent loads
            float2 p[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) p[j] = (g0 + j <= g_hi) ? all_ml[(int64_t)(g0 + j) * QTR + r] : make_float2(-INFINITY, 0.f);
#pragma unroll
            for (int j = 0; j < 4; ++j) ml_merge(m, l, p[j].x, p[j].y);
          }
          b = m + log2f(l) + log2f((float)s.GW);
        }
        nb_s[r] = -b;
      }
      const float *all_ks = reinterpret_cast<const float *>(ws + w.part_ksum) + (slot0 + ul) * D;
      double sq = 0.0;
      for (int d = tid; d < D; d += NT) {
        float a = 0.f;
        for (int g0 = g_lo; g0 <= g_hi; g0 += 4) {
          float p[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) p[j] = (g0 + j <= g_hi) ? all_ks[(int64_t)(g0 + j) * D + d] : 0.f;
#pragma unroll
          for (int j = 0; j < 4; ++j) a += p[j];
        }
        kbar_f[d] = a / (float)N;
        sq += (double)a * (double)a;
      }
      if (c0 == 0) {                                   // one workgroup per unit publishes r
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) sq += __shfl_xor(sq, sft);
        if (lane == 0) red_s[wave] = sq;
      }
    }
    __syncthreads();                                   // kbar_f, nb_s, red_s visible
    if (c0 == 0 && tid == 0) {
      double tot = 0.0;
      for (int wv = 0; wv < WAVES; ++wv) tot += red_s[wv];
      // Eq. 4: (T^2 |Kbar|^2 - T) / (T (T - 1)) with T^2 |Kbar|^2 = |sum of normalised keys|^2
      const float r = (float)((tot - (double)N) / ((double)N * (double)(N - 1)));
      reinterpret_cast<float *>(ws + w.rbar)[unit] = r;
      float *red_out = out.l[uc.layer].redundancy;
      if (red_out) red_out[uc.b * s.hkv + uc.h] = r;
    }

    // The mean key as two rows of 16-byte pieces: row 0 carries the mean key (its bf16 head), row 1
    // the bf16 remainder (zero for f32).  Piece (c, half) of row r sits at kbar_s[(c * 2 + half) * 2 + r].
    for (int p = tid; p < NCHK * 4; p += NT) {
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
      kbar_s[p] = f.q;
    }
    TSTAMP(p2);
    __syncthreads();                                   // kbar_s visible
    TSTAMP(p3);

    // this wave's query tiles, in fragment form, for the whole run (tiles past QT are zero,
    // except for the two mean-key rows)
    Frag qf[TQ][NCHK];
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
      const int row = (wave * TQ + q) * 32 + l32;
      const bool live = row < s.GW;
      const bool mean_rows = spare && wave == kb_wave && q == kb_q && l32 < 2;
      const char *qrow = Qb + ((int64_t)(live ? row : 0) * D) * EB + half * 16;
#pragma unroll
      for (int c = 0; c < NCHK; ++c) {
        uint4 v = *reinterpret_cast<const uint4 *>(qrow + c * 32);
        uint4 mk = kbar_s[(c * 2 + half) * 2 + (l32 & 1)];
        qf[q][c].q = live ? v : (mean_rows ? mk : make_uint4(0, 0, 0, 0));
      }
    }

    TSTAMP(p4);
    TACC(4, p0, p1); TACC(5, p1, p2); TACC(6, p2, p3); TACC(7, p3, p4);
    // add the waves' partial column sums of chunk `chunk` (buffer pb) in a fixed order
    auto flush_colsums = [&](int chunk, int pb) {
      for (int i = tid; i < CH; i += NT) {
        const int key = chunk * CH + i;
        float a = 0.f;
        for (int wv = 0; wv < WAVES; ++wv) a += cs_s[(pb * WAVES + wv) * CH + i];
        if (key < Nc) araw[key] = a;
      }
    };

    auto do_chunk = [&](int it, const uint4 *kb, uint4 *kn) {
      const int cbase = (c0 + it) * CH;
      TSTAMP(t0);
      __builtin_amdgcn_s_waitcnt(0);
      TSTAMP(t1);
      __syncthreads();
      TSTAMP(t2);
      const bool has_next = it + 1 < nit;
      if (it > 0) flush_colsums(c0 + it - 1, (it - 1) & 1);
      float *cs = cs_s + ((it & 1) * WAVES + wave) * CH;
      TSTAMP(t3);
      TACC(0, t0, t1); TACC(1, t1, t2); TACC(2, t2, t3);

      Frag kf[NCHK];
#pragma unroll
      for (int c = 0; c < NCHK; ++c) kf[c].q = read_key_frag<DT, D>(kb, 0, c, l32, half);
#pragma unroll 1
      for (int k = 0; k < KT; ++k) {
        const int tb = cbase + k * 32;
        // the next chunk streams in one tile per tile step, so its loads never queue up
#ifndef MIXKV_NODMA   // developer switch: time the arithmetic alone (results are then meaningless)
        if (has_next) fetch_tile<DT, D, WAVES>(Kb, row_bytes, cbase + CH, k, N, kn, wave, lane);
#endif
        __builtin_amdgcn_sched_barrier(0);
        f32x16 acc[TQ];
#pragma unroll
        for (int q = 0; q < TQ; ++q)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[q][i] = 0.f;
#pragma unroll
        for (int c = 0; c < NCHK; ++c)
#pragma unroll
          for (int q = 0; q < TQ; ++q) acc[q] = mma<DT>(qf[q][c], kf[c], acc[q]);
        float kd = 0.f;
        if (!spare) {
          // no spare tile: a separate mean-key tile on every WAVES-th key tile
          if ((k + it * KT) % WAVES == wave) {
            f32x16 acd;
#pragma unroll
            for (int i = 0; i < 16; ++i) acd[i] = 0.f;
#pragma unroll
            for (int c = 0; c < NCHK; ++c) {
              Frag kbf;
              kbf.q = kbar_s[(c * 2 + half) * 2 + (l32 & 1)];
              if (l32 >= 2) kbf.q = make_uint4(0, 0, 0, 0);
              acd = mma<DT>(kbf, kf[c], acd);
            }
            kd = acd[0] + acd[1];
          }
        }
        // the fragments of the next tile travel LDS -> registers under this tile's arithmetic
        if (k + 1 < KT) {
#pragma unroll
          for (int c = 0; c < NCHK; ++c) kf[c].q = read_key_frag<DT, D>(kb, k + 1, c, l32, half);
        }
        if (spare) kd = (kb_q == 0 ? acc[0][0] + acc[0][1] : acc[TQ - 1][0] + acc[TQ - 1][1]);   // rows 0, 1: half 0
        const bool kd_mine = spare ? wave == kb_wave : (k + it * KT) % WAVES == wave;
        const int key = tb + l32;
        if (kd_mine && half == 0 && key < Nc) kdot[key] = kd;

        if (tb + 31 > free_limit) {                    // tile reaches into the window or past N: mask
#pragma unroll
          for (int q = 0; q < TQ; ++q)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int row = (wave * TQ + q) * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
              acc[q][i] = (key <= lim_s[row]) ? acc[q][i] : -INFINITY;
            }
        }
        float colsum = 0.f;
#pragma unroll
        for (int q = 0; q < TQ; ++q)
#pragma unroll
          for (int k4 = 0; k4 < 4; ++k4) {
            const float4 nb = *reinterpret_cast<const float4 *>(&nb_s[(wave * TQ + q) * 32 + 8 * k4 + 4 * half]);
            colsum += fast_exp2(fmaf(acc[q][4 * k4 + 0], c2, nb.x)) + fast_exp2(fmaf(acc[q][4 * k4 + 1], c2, nb.y)) +
                      fast_exp2(fmaf(acc[q][4 * k4 + 2], c2, nb.z)) + fast_exp2(fmaf(acc[q][4 * k4 + 3], c2, nb.w));
          }
        colsum += __shfl_xor(colsum, 32);
        if (half == 0) cs[k * 32 + l32] = (tb < N) ? colsum : 0.f;
      }
      TSTAMP(t4);
      TACC(3, t3, t4);
    };
    // Fast path for chunks that no row has to mask (everything before the window): the work is cut
    // into blocks (key tile k, query tile q); the MFMA chain of block j+1 is issued interleaved with
    // the exp2/sum arithmetic on the finished block j, so the matrix core and the vector ALU of the
    // SIMD run at the same time.  Two accumulators alternate; the fragments of the next key tile
    // replace the current ones as soon as the tile's last chain has consumed them.
    auto do_chunk_fast = [&](int it, const uint4 *kb, uint4 *kn) {
      constexpr int NB = KT * TQ;
      const int cbase = (c0 + it) * CH;
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      const bool has_next = it + 1 < nit;
      if (it > 0) flush_colsums(c0 + it - 1, (it - 1) & 1);
      float *cs = cs_s + ((it & 1) * WAVES + wave) * CH;

      Frag kf[NCHK];
#pragma unroll
      for (int c = 0; c < NCHK; ++c) kf[c].q = read_key_frag<DT, D>(kb, 0, c, l32, half);
      f32x16 acc[2];
      auto chain = [&](int j) {                         // MFMA chain of block j, and the fragment hand-over
        const int k = j / TQ, q = j % TQ;
        f32x16 a;
#pragma unroll
        for (int i = 0; i < 16; ++i) a[i] = 0.f;
#pragma unroll
        for (int c = 0; c < NCHK; ++c) {
          a = mma<DT>(qf[q][c], kf[c], a);
          if (q == TQ - 1 && k + 1 < KT) kf[c].q = read_key_frag<DT, D>(kb, k + 1, c, l32, half);
        }
        acc[j & 1] = a;
      };
      chain(0);
      float colsum = 0.f, kdv[KT];
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int k = j / TQ, q = j % TQ;
        if (q == 0) {
#ifndef MIXKV_NODMA
          if (has_next) fetch_tile<DT, D, WAVES>(Kb, row_bytes, cbase + CH, k, N, kn, wave, lane);
#endif
          colsum = 0.f;
        }
        // block j is complete: its mean-key rows (0 and 1 of the spare tile, half 0) first
        if (q == kb_q) kdv[k] = acc[j & 1][0] + acc[j & 1][1];
        if (j + 1 < NB) chain(j + 1);
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
          const float4 nb = *reinterpret_cast<const float4 *>(&nb_s[(wave * TQ + q) * 32 + 8 * k4 + 4 * half]);
          const f32x16 &a = acc[j & 1];
          colsum += fast_exp2(fmaf(a[4 * k4 + 0], c2, nb.x)) + fast_exp2(fmaf(a[4 * k4 + 1], c2, nb.y)) +
                    fast_exp2(fmaf(a[4 * k4 + 2], c2, nb.z)) + fast_exp2(fmaf(a[4 * k4 + 3], c2, nb.w));
        }
        if (j + 1 < NB) {
#pragma unroll
          for (int c = 0; c < NCHK; ++c) {               // one MFMA, then its share of the vector work
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 48 / NCHK, 0);
          }
        }
        if (q == TQ - 1) {
          colsum += __shfl_xor(colsum, 32);
          if (half == 0) cs[k * 32 + l32] = colsum;
        }
      }
      if (wave == kb_wave && half == 0) {
#pragma unroll
        for (int k = 0; k < KT; ++k) kdot[cbase + k * 32 + l32] = kdv[k];
      }
    };

    for (int it = 0; it < nit; it += 2) {
      // a chunk is "free" when even its last key is visible to every row and the mean key rides
      // in a spare tile; the general path handles the rest
      const bool free_a = spare && (c0 + it + 1) * CH - 1 <= free_limit;
      if (free_a) do_chunk_fast(it, kbuf_a, kbuf_b); else do_chunk(it, kbuf_a, kbuf_b);
      if (it + 1 < nit) {
        const bool free_b = spare && (c0 + it + 2) * CH - 1 <= free_limit;
        if (free_b) do_chunk_fast(it + 1, kbuf_b, kbuf_a); else do_chunk(it + 1, kbuf_b, kbuf_a);
      }
    }
    __syncthreads();
    flush_colsums(c0 + nit - 1, (nit - 1) & 1);
    item += nit;
  }
  TFLUSH;
#ifdef MIXKV_TIMING
  if (threadIdx.x == 0) { mixkv_dbg[blockIdx.x * 16 + 5] = wall_clock64(); mixkv_dbg[blockIdx.x * 16 + 7] = __builtin_readcyclecounter(); }
#endif
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

// Grid of the two streaming kernels: enough workgroups to fill the chip once, never more than items.
int stream_grid(const Shape &s, int nunits, int num_cus) {
  int waves, tq;
  stream_config(s.QT, &waves, &tq);
  const int64_t T = (int64_t)nunits * s.nchunks;
  int64_t cap = (int64_t)num_cus * (waves == 4 ? 2 : 1);
  if (cap > kMaxStreamGrid) cap = kMaxStreamGrid;
  return (int)(T < cap ? T : cap);
}

template <int DT, int D, int WAVES, int TQ>
static hipError_t launch_stats_c(const Shape &s, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                                 int nunits, int grid, int64_t slot0, hipStream_t st) {
  auto kern = stats_kernel<DT, D, WAVES, TQ>;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES * 64), 0, st, s, in, ws, w, unit0, nunits, slot0);
  return hipGetLastError();
}

template <int DT, int D, int WAVES, int TQ>
static hipError_t launch_attn_c(const Shape &s, const LayerInTable &in, const LayerOutTable &out, char *ws,
                                const Workspace &w, int64_t unit0, int nunits, int grid, int64_t slot0, hipStream_t st) {
  auto kern = attn_kernel<DT, D, WAVES, TQ>;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES * 64), 0, st, s, in, out, ws, w, unit0, nunits, grid, slot0);
  return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_stats_t(const Shape &s, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                                 int nunits, int grid, int64_t slot0, hipStream_t st) {
  int waves, tq;
  stream_config(s.QT, &waves, &tq);
  if (waves == 4 && tq == 1) return launch_stats_c<DT, D, 4, 1>(s, in, ws, w, unit0, nunits, grid, slot0, st);
  if (waves == 4) return launch_stats_c<DT, D, 4, 2>(s, in, ws, w, unit0, nunits, grid, slot0, st);
  return launch_stats_c<DT, D, 8, 2>(s, in, ws, w, unit0, nunits, grid, slot0, st);
}

template <int DT, int D>
static hipError_t launch_attn_t(const Shape &s, const LayerInTable &in, const LayerOutTable &out, char *ws,
                                const Workspace &w, int64_t unit0, int nunits, int grid, int64_t slot0, hipStream_t st) {
  int waves, tq;
  stream_config(s.QT, &waves, &tq);
  if (waves == 4 && tq == 1) return launch_attn_c<DT, D, 4, 1>(s, in, out, ws, w, unit0, nunits, grid, slot0, st);
  if (waves == 4) return launch_attn_c<DT, D, 4, 2>(s, in, out, ws, w, unit0, nunits, grid, slot0, st);
  return launch_attn_c<DT, D, 8, 2>(s, in, out, ws, w, unit0, nunits, grid, slot0, st);
}

hipError_t launch_stats(const Shape &s, int dtype, const LayerInTable &in, char *ws, const Workspace &w, int64_t unit0,
                        int nunits, int grid, int64_t slot0, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_stats_t<MIXKV_BF16, 128>(s, in, ws, w, unit0, nunits, grid, slot0, st);
    return launch_stats_t<MIXKV_BF16, 64>(s, in, ws, w, unit0, nunits, grid, slot0, st);
  }
  if (s.D == 128) return launch_stats_t<MIXKV_F32, 128>(s, in, ws, w, unit0, nunits, grid, slot0, st);
  return launch_stats_t<MIXKV_F32, 64>(s, in, ws, w, unit0, nunits, grid, slot0, st);
}

// `grid` must be the grid stats_kernel ran with: both kernels split the same items the same way,
// and attn_kernel uses it to find the partials of its units.
hipError_t launch_attn(const Shape &s, int dtype, const LayerInTable &in, const LayerOutTable &out, char *ws,
                       const Workspace &w, int64_t unit0, int nunits, int grid, int64_t slot0, hipStream_t st) {
  if (dtype == MIXKV_BF16) {
    if (s.D == 128) return launch_attn_t<MIXKV_BF16, 128>(s, in, out, ws, w, unit0, nunits, grid, slot0, st);
    return launch_attn_t<MIXKV_BF16, 64>(s, in, out, ws, w, unit0, nunits, grid, slot0, st);
  }
  if (s.D == 128) return launch_attn_t<MIXKV_F32, 128>(s, in, out, ws, w, unit0, nunits, grid, slot0, st);
  return launch_attn_t<MIXKV_F32, 64>(s, in, out, ws, w, unit0, nunits, grid, slot0, st);
}

}  // namespace mixkv
