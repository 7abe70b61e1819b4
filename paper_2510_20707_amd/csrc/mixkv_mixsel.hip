// mixsel_kernel: score mixing and (optionally) the fixed-budget top-B' selection of one unit in a
// single workgroup, with every per-key quantity held in registers.
//
// Loading, pooling, statistics and mixing deal the candidates to the threads in groups of four,
// round-robin, so that every load is coalesced; the pooled attention needs neighbours, so the raw
// attention row is staged once in LDS.  For the selection thread t owns the EPT consecutive
// candidates [t*EPT, (t+1)*EPT) (the mixed scores change hands through the same LDS row), so the
// kept indices come out in ascending order from a plain prefix sum.  The selection is a
// most-significant-digit radix select on order-preserving integer keys kept in registers; it
// starts at the first bit in which the keys of the head differ at all, which keeps the first
// histogram from collapsing into one bin.
//
// Paper: Sec. 3.2 Eq. 2 (importance = attention + scaled value norm), Sec. 3.3 (min-max and mean
// matching of the diversity, Eq. 5 mix), Sec. 3.1 / Algorithm 1 (TopB with B' = B - W); Sec. 4.3 /
// Table 4 for the variants (key-norm intrinsic score, un-weighted and one-sided mixes, given weights).
#include <mutex>

#include "mixkv_internal.h"
#include "mixkv_wave.h"

namespace mixkv {

constexpr int kMsMaxThreads = 1024, kMsMaxWaves = kMsMaxThreads / 64;
constexpr int kDigit = 11, kBins = 1 << kDigit;     // radix-select digit

struct MsScratch {
  float f[kMsMaxWaves][8];
  float fr[8];
  uint32_t ur[2];
  int i[kMsMaxWaves + 1];
  int hist[kBins];
  int hist0[kBins];                      // the first round's histogram of a head, for a second threshold on the same keys
  int bin, krem, cut;
};

// Block-wide reduction of NS sums, NMIN minima and NMAX maxima at once; every thread gets the
// results back in place.  Fixed order: lanes in lane order inside a wave, then waves in wave order.
template <int NW, int NS, int NMIN, int NMAX>
__device__ __forceinline__ void block_reduce_mixed(float (&v)[NS + NMIN + NMAX], MsScratch &sc) {
  constexpr int NV = NS + NMIN + NMAX;
  static_assert(NV <= 8 && NW <= 16, "scratch holds eight values for sixteen waves");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < NV; ++k)
    v[k] = k < NS ? wave_reduce<WSum>(v[k], 0.f)
                  : (k < NS + NMIN ? wave_reduce<WMin>(v[k], INFINITY) : wave_reduce<WMax>(v[k], -INFINITY));
  __syncthreads();                       // scratch may still be read from a previous call
  if (lane == 0)
#pragma unroll
    for (int k = 0; k < NV; ++k) sc.f[wave][k] = v[k];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    // every wave folds the NW partials itself (one row of lanes), so no third barrier is needed
    const float id = k < NS ? 0.f : (k < NS + NMIN ? INFINITY : -INFINITY);
    float x = (lane & 15) < NW ? sc.f[lane & 15][k] : id;
    x = k < NS ? row_scan_incl<WSum>(x, id) : (k < NS + NMIN ? row_scan_incl<WMin>(x, id) : row_scan_incl<WMax>(x, id));
    v[k] = read_lane(x, 15);
  }
}

// Block-wide minimum and maximum of unsigned keys through two LDS atomics per wave (integer
// min / max do not depend on the order).  sc.ur must hold {0xffffffff, 0} from before an earlier
// barrier of the kernel.
__device__ __forceinline__ void block_minmax_u32(uint32_t &lo, uint32_t &hi, MsScratch &sc) {
  const int lane = threadIdx.x & 63;
  lo = wave_reduce<WMin>(lo, 0xffffffffu);
  hi = wave_reduce<WMax>(hi, 0u);
  if (lane == 0) { atomicMin(&sc.ur[0], lo); atomicMax(&sc.ur[1], hi); }
  __syncthreads();
  lo = sc.ur[0];
  hi = sc.ur[1];
}

// Exclusive prefix sum of one int per thread (thread order); *total receives the block sum.
__device__ __forceinline__ int read_lane_dyn(int x, int lane_uniform) {
  return __builtin_amdgcn_readlane(x, __builtin_amdgcn_readfirstlane(lane_uniform));
}

template <int NW>
__device__ __forceinline__ int block_scan_excl(int v, MsScratch &sc, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int wtot;
  const int inc = wave_scan_incl_add(v, &wtot);
  __syncthreads();
  if (lane == 0) sc.i[wave] = wtot;
  __syncthreads();
  const int x = (lane & 15) < NW ? sc.i[lane & 15] : 0;
  const int y = row_scan_incl<WSum>(x, 0);              // inclusive over the waves, in every row of lanes
  *total = read_lane(y, 15);
  const int before = wave == 0 ? 0 : read_lane_dyn(y, wave - 1);
  return before + inc - v;
}

__device__ __forceinline__ uint32_t order_key_u(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0;                          // -0 and +0 are the same score
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One count into a shared histogram bin per lane, with the lanes that share the wave's most common
// bin (as seen from its first active lane) merged into a single atomic.
__device__ __forceinline__ void hist_add(int *hist, int bin, bool on) {
  const unsigned long long act = __ballot(on);
  if (act == 0) return;
  const int first = __ffsll((long long)act) - 1;                  // wave-uniform
  const int b0 = __builtin_amdgcn_readlane(bin, first);
  const unsigned long long same = __ballot(on && bin == b0);
  const int lane = threadIdx.x & 63;
  if (lane == first) atomicAdd(&hist[b0], __popcll(same));
  if (on && bin != b0) atomicAdd(&hist[bin], 1);
}

// Threshold of the k largest of a workgroup's keys (1 <= k <= number of valid keys): every thread holds
// EPT keys, those with their bit set in `vmask` valid, and [kmin, kmax] is the range of all valid keys.  Most-significant-digit radix select from the first
// bit in which the keys differ.  Returns tau, the k-th largest key, and in krem how many of the
// keys equal to tau still belong to the k (0: all of them).  Ends behind a barrier: may be called again.
// The first round counts every valid key and does not depend on k: FIRST = 1 keeps its histogram
// aside, FIRST = 2 takes it from there (a second threshold on the same keys), 0 does neither.
template <int THREADS, int EPT, int FIRST = 0>
__device__ __forceinline__ uint32_t radix_threshold(const uint32_t (&key)[EPT], uint32_t vmask, uint32_t kmin, uint32_t kmax,
                                                    int k, MsScratch &sc, int &krem) {
  constexpr int NW = THREADS / 64;
  const int tid = threadIdx.x;
  // bits at and above `undecided` are common to all keys; digits of up to kDigit bits from there down
  int undecided = kmin == kmax ? 0 : 32 - __clz((int)(kmin ^ kmax));
  uint32_t prefix = undecided >= 32 ? 0u : (kmax >> undecided) << undecided;
  bool all_equal = false, first = true;
  while (undecided > 0) {
    const int wbits = min(kDigit, undecided), shift = undecided - wbits;
    const uint32_t himask = undecided >= 32 ? 0u : ~0u << undecided;
    const bool saved = FIRST == 2 && first;             // this round's histogram is already in hist0
    int *hist = saved ? sc.hist0 : sc.hist;
    if (!saved) {
      for (int i = tid; i < kBins; i += THREADS) sc.hist[i] = 0;
      __syncthreads();
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const bool on = ((vmask >> e) & 1u) != 0 && (key[e] & himask) == (prefix & himask);
        hist_add(sc.hist, (int)((key[e] >> shift) & ((1u << wbits) - 1u)), on);
      }
      __syncthreads();
    }
    // walk the bins from the top: thread t sums bins [kBins - (t+1)*BPT, kBins - t*BPT)
    constexpr int BPT = (kBins + THREADS - 1) / THREADS;
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
      const int bi = kBins - 1 - (tid * BPT + j);
      const int c = bi >= 0 ? hist[bi] : 0;
      if (FIRST == 1 && first && bi >= 0) sc.hist0[bi] = c;
      cnt += c;
    }
    first = false;
    int total;
    const int excl = block_scan_excl<NW>(cnt, sc, &total);
    if (excl < k && k <= excl + cnt) {
      int run = excl;
#pragma unroll
      for (int j = 0; j < BPT; ++j) {
        const int bi = kBins - 1 - (tid * BPT + j);
        const int c = bi >= 0 ? hist[bi] : 0;
        if (run < k && k <= run + c) { sc.bin = bi; sc.krem = k - run; sc.cut = c; }
        run += c;
      }
    }
    __syncthreads();
    prefix |= (uint32_t)sc.bin << shift;
    k = sc.krem;
    undecided = shift;
    const bool whole_bin = sc.cut == k && shift > 0 && prefix != 0;
    __syncthreads();
    // Every key of the bin is needed: the kept set is "all keys at or above the bin", whatever
    // the lower digits are, so the remaining rounds can be skipped.
    if (whole_bin) { prefix -= 1; all_equal = true; break; }
  }
  krem = all_equal ? 0 : k;
  return prefix;
}

// Bit 31 of a candidate-list entry: the candidate is one of its head's `floor` best.
constexpr uint32_t kFloorFlag = 0x80000000u;

// TopB' of one head: the Bp >= 1 candidates with the largest scores, ties to the smaller index, out
// of the EPT consecutive candidates base .. base + nvalid - 1 every thread holds in a[] (Sec. 3.1 /
// Algorithm 1, TopB).  The kept positions go to idx[0, Bp) in ascending order.  With ckey not null
// the list is a head's candidates for the head-adaptive split: the order keys go beside the
// positions, and the head's `floor` <= Bp best carry kFloorFlag in their position word.
// sc.ur must hold {0xffffffff, 0} from before an earlier barrier.
template <int THREADS, int EPT>
__device__ __forceinline__ void top_select(const float (&a)[EPT], int nvalid, int base, int Bp, int32_t *idx,
                                           uint32_t *ckey, int floor, MsScratch &sc) {
  constexpr int NW = THREADS / 64;
  uint32_t key[EPT];
  uint32_t kmin = 0xffffffffu, kmax = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    key[e] = order_key_u(a[e]);
    if (e < nvalid) { kmin = min(kmin, key[e]); kmax = max(kmax, key[e]); }
  }
  block_minmax_u32(kmin, kmax, sc);
  const uint32_t vmask = nvalid >= EPT ? (EPT >= 32 ? 0xffffffffu : (1u << (EPT & 31)) - 1u)
                                       : (nvalid <= 0 ? 0u : (1u << nvalid) - 1u);
  int k;                             // of the keys equal to tau, the first k (by position) are kept
  const bool flags = ckey != nullptr && floor > 0;
  int kf = 0;
  uint32_t tau, tauf = 0xffffffffu;
  if (flags) {
    tau = radix_threshold<THREADS, EPT, 1>(key, vmask, kmin, kmax, Bp, sc, k);
    tauf = radix_threshold<THREADS, EPT, 2>(key, vmask, kmin, kmax, floor, sc, kf);
  } else {
    tau = radix_threshold<THREADS, EPT>(key, vmask, kmin, kmax, Bp, sc, k);
  }
  // one scan carries both counts: keys above tau (low half) and keys equal to tau (high half)
  int ngt = 0, neq = 0, neqf = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const bool in = e < nvalid;
    ngt += (in && key[e] > tau) ? 1 : 0;
    neq += (in && key[e] == tau) ? 1 : 0;
    neqf += (in && key[e] == tauf) ? 1 : 0;
  }
  int total;
  const int packed = block_scan_excl<NW>(ngt | (neq << 16), sc, &total);
  int seen = packed >> 16;                          // equal keys at smaller indices
  int pos = (packed & 0xffff) + min(seen, k);       // kept entries at smaller indices
  int seenf = flags ? block_scan_excl<NW>(neqf, sc, &total) : 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (e < nvalid) {
      bool sel = key[e] > tau;
      if (key[e] == tau) sel = seen++ < k;
      bool inf = flags && key[e] > tauf;
      if (flags && key[e] == tauf) inf = seenf++ < kf;
      if (sel) {
        if (pos < Bp) {
          idx[pos] = (int32_t)((uint32_t)(base + e) | (inf ? kFloorFlag : 0u));
          if (ckey) ckey[pos] = key[e];
        }
        ++pos;
      }
    }
  }
}

// Rows head h of a layer keeps and its first row inside the batch item: B each, or the layer's
// row of the budget table (per-head mode), the heads packed back to back.
__device__ __forceinline__ void head_rows(const Shape &s, const int32_t *budgets, int layer, int h, int &Bh, int &row0) {
  Bh = s.B;
  row0 = h * s.B;
  if (budgets) {
    const int32_t *bl = budgets + layer * s.hkv;
    row0 = 0;
    for (int j = 0; j < h; ++j) row0 += bl[j];
    Bh = bl[h];
  }
}

// After the candidates of a head: the W window positions, the head's count and its offsets.
__device__ __forceinline__ void finish_head(const Shape &s, const LayerOut &O, int b, int h, int Bh, int row0,
                                            int32_t *idx, int threads) {
  const int tid = threadIdx.x, Bp = Bh - s.W;
  for (int wv = tid; wv < s.W; wv += threads) idx[Bp + wv] = s.Nc + wv;
  if (tid == 0) {
    O.counts[b * s.hkv + h] = Bh;
    if (O.offsets) {
      O.offsets[b * (s.hkv + 1) + h] = row0;
      if (h == s.hkv - 1) O.offsets[b * (s.hkv + 1) + s.hkv] = row0 + Bh;
    }
  }
}

template <int THREADS, int EPT, bool SELECT>
__global__ __launch_bounds__(THREADS) void mixsel_kernel(Shape s, LayerOutTable out, char *ws, Workspace w,
                                                           int64_t unit0, LayerInTable in, int gather_eb, int cand_m,
                                                           const int32_t *budgets) {
  constexpr int NW = THREADS / 64;
  extern __shared__ float a_s[];                        // [Nc] raw window attention of this head
  __shared__ MsScratch sc;
  const int tid = threadIdx.x, ul = blockIdx.x;
  const int64_t unit = unit0 + ul;
  const int layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  const LayerOut O = out.l[layer];
  const float *araw = reinterpret_cast<const float *>(ws + w.araw) + unit * s.Npad;
  const float *vnorm = reinterpret_cast<const float *>(ws + w.vnorm) + unit * s.Npad;
  const float *kdot = reinterpret_cast<const float *>(ws + w.sdiv) + unit * s.Npad;
  const float *invn = reinterpret_cast<const float *>(ws + w.invnorm) + unit * s.Npad;
  const float r = reinterpret_cast<const float *>(ws + w.rbar)[unit];
  const int Nc = s.Nc, N = s.N, base = tid * EPT;
  const bool use_v = s.intrinsic != MIXKV_INTRINSIC_NONE;      // an intrinsic score takes part (held in v[])
  const bool knorm = s.intrinsic == MIXKV_INTRINSIC_KNORM;
  const float inv_n = 1.f / (float)Nc;
  float wi, wd;
  mix_weights(s.mix, r, s.mix == MIXKV_MIX_GIVEN_R ? in.l[layer].r_given[bh] : 0.f, wi, wd);

  // ---- load.  The first phases deal the candidates to the threads in groups of four, group
  // g * THREADS + tid to thread tid: consecutive lanes read consecutive 16 bytes (the per-unit rows
  // are padded past Nc).  Only the attention stays in registers; the sums and extrema of the
  // intrinsic score and the diversity are taken as they pass, and the mix reads the two a second
  // time (from L2: the kernel before wrote them).  Three register arrays of EPT would not fit the
  // 128 registers a 1024-thread workgroup leaves each lane at EPT = 32, and runs of EPT consecutive
  // candidates per thread would touch one cache line per lane and load.  The selection does need
  // consecutive runs (ascending output from one prefix sum): s_comp reaches their owners through LDS.
  auto cidx = [&](int e) { return (((e >> 2) * THREADS + tid) << 2) + (e & 3); };
  const int nvalid = Nc - base;             // consecutive ownership: candidates of this thread inside the row
  float a[EPT];
  float st[7] = {0.f, 0.f, 0.f, INFINITY, INFINITY, -INFINITY, -INFINITY};   // sums a, v, d | min v, d | max v, d
  // intrinsic score and diversity of the four candidates from i on (zeros past the row)
  auto load_vd = [&](int i, float4 &vr, float4 &dr) {
    float4 kr = make_float4(0.f, 0.f, 0.f, 0.f), nr = kr;
    vr = kr;
    if (i < Nc) {
      if (s.kstats) {                        // else nobody wrote them: the diversity is 0 and carries weight 0
        kr = *reinterpret_cast<const float4 *>(kdot + i);
        nr = *reinterpret_cast<const float4 *>(invn + i);
      }
      if (knorm) vr = make_float4(neg_key_norm(nr.x), neg_key_norm(nr.y), neg_key_norm(nr.z), neg_key_norm(nr.w));
      else if (use_v) vr = *reinterpret_cast<const float4 *>(vnorm + i);
    }
    // s_div: a product rounded on its own.  The minimum is taken from the first reading and must
    // cancel exactly against the second, so the compiler may not fuse the product into the
    // subtraction that follows there (it may by default); the empty statements hide where it came from.
    dr = make_float4(-kr.x * nr.x, -kr.y * nr.y, -kr.z * nr.z, -kr.w * nr.w);
    asm("" : "+v"(dr.x), "+v"(dr.y), "+v"(dr.z), "+v"(dr.w));
  };
  // The raw attention row goes to LDS with one pad word per 32 so that the accesses of
  // consecutive-range owners (a thread stride of EPT words) spread over the banks.
  auto slot = [](int i) { return i + (i >> 5); };
  if (tid == 0) { sc.ur[0] = 0xffffffffu; sc.ur[1] = 0u; }   // for the key range, read after later barriers
#pragma unroll
  for (int e4 = 0; e4 < EPT; e4 += 4) {
    const int i = cidx(e4);
    float4 ar = make_float4(0.f, 0.f, 0.f, 0.f), vr, dr;
    if (i < Nc) ar = *reinterpret_cast<const float4 *>(araw + i);
    load_vd(i, vr, dr);
    const float a4[4] = {ar.x, ar.y, ar.z, ar.w};
    const float v4[4] = {vr.x, vr.y, vr.z, vr.w}, d4[4] = {dr.x, dr.y, dr.z, dr.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a[e4 + j] = a4[j];
      if (i + j < Nc) {
        a_s[slot(i + j)] = a4[j];
        st[1] += v4[j]; st[2] += d4[j];
        st[3] = fminf(st[3], v4[j]); st[4] = fminf(st[4], d4[j]);
        st[5] = fmaxf(st[5], v4[j]); st[6] = fmaxf(st[6], d4[j]);
      }
    }
  }
  __syncthreads();

  // ---- pooled attention (candidates only) and the first round of statistics
  if (s.pool != MIXKV_POOL_NONE && s.pool_k > 1) {
    const int hk = s.pool_k >> 1;
    const bool is_max = s.pool == MIXKV_POOL_MAX;
    const float fill = is_max ? -INFINITY : 0.f;        // out-of-range taps: ignored by max, zero for avg
    if (hk <= 3) {
      // sliding window in registers over each group of four: its own values plus three neighbours
      // on either side
      constexpr int RUN = 4;
#pragma unroll
      for (int e0 = 0; e0 < EPT; e0 += RUN) {
        const int i0 = cidx(e0);
        float win[RUN + 6];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
          const int il = i0 - 3 + j, ir = i0 + RUN + j;
          win[j] = (il >= 0 && il < Nc) ? a_s[slot(il)] : fill;
          win[RUN + 3 + j] = (ir < Nc) ? a_s[slot(ir)] : fill;
        }
#pragma unroll
        for (int e = 0; e < RUN; ++e) win[3 + e] = (i0 + e < Nc) ? a[e0 + e] : fill;
#pragma unroll
        for (int e = 0; e < RUN; ++e) {
          float acc = win[3 + e];
          if (is_max) {
            if (hk >= 1) acc = fmaxf(acc, fmaxf(win[2 + e], win[4 + e]));
            if (hk >= 2) acc = fmaxf(acc, fmaxf(win[1 + e], win[5 + e]));
            if (hk >= 3) acc = fmaxf(acc, fmaxf(win[e], win[6 + e]));
          } else {
            // same left-to-right order as a plain loop over the taps
            acc = 0.f;
            if (hk >= 3) acc += win[e];
            if (hk >= 2) acc += win[1 + e];
            if (hk >= 1) acc += win[2 + e];
            acc += win[3 + e];
            if (hk >= 1) acc += win[4 + e];
            if (hk >= 2) acc += win[5 + e];
            if (hk >= 3) acc += win[6 + e];
            acc = acc / (float)s.pool_k;
          }
          a[e0 + e] = acc;
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const int i = cidx(e);
        if (i < Nc) {
          const int lo = max(0, i - hk), hi = min(Nc - 1, i + hk);
          float acc = a_s[slot(lo)];
          if (is_max) {
            for (int j = lo + 1; j <= hi; ++j) acc = fmaxf(acc, a_s[slot(j)]);
          } else {
            for (int j = lo + 1; j <= hi; ++j) acc += a_s[slot(j)];
            acc = acc / (float)s.pool_k;
          }
          a[e] = acc;
        }
      }
    }
  }
  // One round of statistics over the candidates.  The means of the min-max normalised intrinsic score
  // and diversity follow from the plain sums: sum((x - min) * c) = (sum(x) - Nc * min) * c, and
  // mean(s_imp) = mean(s_ex) + f_in * mean(s_in_norm).
#pragma unroll
  for (int e = 0; e < EPT; ++e)
    if (cidx(e) < Nc) st[0] += a[e];
  block_reduce_mixed<NW, 3, 2, 2>(st, sc);
  const float mean_ex = st[0] * inv_n;
  const float vmin = st[3], dmin = st[4];
  const float rvden = 1.f / (st[5] - vmin + s.eps), rdden = 1.f / (st[6] - dmin + s.eps);
  const float mean_in = (st[1] - (float)Nc * vmin) * rvden * inv_n;     // mean of the normalised value norm
  const float mean_dn = (st[2] - (float)Nc * dmin) * rdden * inv_n;     // mean of the normalised diversity
  const float f_in = use_v ? mean_ex / (mean_in + s.eps) : 0.f;         // Sec. 3.2: scale VNorm to mean(s_ex)
  const float mean_imp = use_v ? mean_ex + f_in * mean_in : mean_ex;
  const float f_div = mean_imp / (mean_dn + s.eps);                      // Sec. 3.3: scale diversity to mean(s_imp)
  auto s_comp = [&](float ai, float vi, float di) {
    const float imp = use_v ? ai + (vi - vmin) * rvden * f_in : ai;       // Eq. 2
    return wi * imp + wd * ((di - dmin) * rdden * f_div);                 // Eq. 5
  };
  // every thread is past the reduction's barriers, so the pooling has read all it needs of the raw
  // row: s_comp replaces it in LDS and comes back dealt in consecutive runs of EPT
#pragma unroll
  for (int e4 = 0; e4 < EPT; e4 += 4) {
    const int i = cidx(e4);
    float4 vr, dr;
    load_vd(i, vr, dr);
    const float v4[4] = {vr.x, vr.y, vr.z, vr.w}, d4[4] = {dr.x, dr.y, dr.z, dr.w};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (i + j < Nc) a_s[slot(i + j)] = s_comp(a[e4 + j], v4[j], d4[j]);
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < EPT; ++e) a[e] = e < nvalid ? a_s[slot(base + e)] : 0.f;

  if (O.scores) {
    float *scores = O.scores + (int64_t)bh * N;
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if (e < nvalid) scores[base + e] = a[e];
    for (int i = Nc + tid; i < N; i += THREADS) scores[i] = INFINITY;
  }
  if constexpr (!SELECT) return;

  // ---- TopB': the B' candidates with the largest s_comp, ties to the smaller index.  In fixed
  // budget mode B' = B - W and the indices are the head's final ones; with a budget table (per-head
  // mode) B is the head's own entry and the heads of a batch item are packed back to back.  With cand_m > 0 (head-adaptive
  // mode) the head's best cand_m candidates go to the workspace with their keys instead: no head
  // can end up keeping more than that, so the budget split only has to look at those.
  const bool cand = cand_m > 0;
  const int h = bh % s.hkv, b = bh / s.hkv;
  int Bh, row0;                                        // rows this head keeps, and its first row in the batch item
  head_rows(s, budgets, layer, h, Bh, row0);
  const int64_t out_row0 = (int64_t)b * s.hkv * s.B + row0;
  int32_t *idx = cand ? reinterpret_cast<int32_t *>(ws + w.cand_idx) + unit * kMaxCandPerHead : O.indices + out_row0;
  uint32_t *ckey = reinterpret_cast<uint32_t *>(ws + w.cand_key) + unit * kMaxCandPerHead;
  const int Bp = cand ? cand_m : Bh - s.W;
  if (Bp > 0) top_select<THREADS, EPT>(a, nvalid, base, Bp, idx, cand ? ckey : nullptr, s.floor_, sc);
  if (cand) return;
  finish_head(s, O, b, h, Bh, row0, idx, THREADS);
  // ---- gather of the kept rows (Sec. 3.1, the compacted cache), if asked for: gather_eb is the
  // element size in bytes, 0 to skip.  16 bytes per thread and step; the head's indices are read
  // back after a workgroup barrier (same compute unit, so they are visible).
  if (gather_eb > 0) {
    __syncthreads();
    const LayerIn L = in.l[layer];
    const int ppr = s.D * gather_eb / 16;
    const char *Kh = reinterpret_cast<const char *>(L.K) + ((int64_t)b * L.sb + (int64_t)h * L.sh) * gather_eb;
    const char *Vh = reinterpret_cast<const char *>(L.V) + ((int64_t)b * L.sb + (int64_t)h * L.sh) * gather_eb;
    char *Ko = reinterpret_cast<char *>(O.K_out) + out_row0 * s.D * gather_eb;
    char *Vo = reinterpret_cast<char *>(O.V_out) + out_row0 * s.D * gather_eb;
    for (int p = tid; p < Bh * ppr; p += THREADS) {
      const int row = p / ppr, piece = p - row * ppr;
      const int src = min(max(idx[row], 0), N - 1);    // indices come from the selection above; the clamp only guards the load
      const int64_t so = (int64_t)src * L.sn * gather_eb + piece * 16;
      const uint4 kv = *reinterpret_cast<const uint4 *>(Kh + so);
      const uint4 vv = *reinterpret_cast<const uint4 *>(Vh + so);
      *reinterpret_cast<uint4 *>(Ko + (int64_t)p * 16) = kv;
      *reinterpret_cast<uint4 *>(Vo + (int64_t)p * 16) = vv;
    }
  }
}

// topsel_kernel: the selection half alone, on scores that are already in memory (the caller's, for
// mixkv_select).  One workgroup per unit reads the Nc candidate scores of its head once (coalesced,
// through the padded LDS row to their consecutive-range owners) and selects from registers as
// above: the head's final rows in fixed and per-head mode, or with cand_m > 0 its best cand_m
// candidates with their keys for the head-adaptive split (Sec. 3.1 / Algorithm 1, TopB).
template <int THREADS, int EPT>
__global__ __launch_bounds__(THREADS) void topsel_kernel(Shape s, LayerOutTable out, char *ws, Workspace w, int64_t unit0,
                                                           int cand_m, const int32_t *budgets) {
  extern __shared__ float a_s[];                        // [Nc] padded: the head's scores
  __shared__ MsScratch sc;
  const int tid = threadIdx.x, ul = blockIdx.x;
  const int64_t unit = unit0 + ul;
  const int layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  const LayerOut O = out.l[layer];
  const float *scores = O.scores + (int64_t)bh * s.N;
  const int Nc = s.Nc, base = tid * EPT, nvalid = Nc - base;
  auto slot = [](int i) { return i + (i >> 5); };
  if (tid == 0) { sc.ur[0] = 0xffffffffu; sc.ur[1] = 0u; }
  for (int i = tid; i < Nc; i += THREADS) a_s[slot(i)] = scores[i];
  __syncthreads();
  float a[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) a[e] = e < nvalid ? a_s[slot(base + e)] : 0.f;
  const bool cand = cand_m > 0;
  const int h = bh % s.hkv, b = bh / s.hkv;
  int Bh, row0;
  head_rows(s, budgets, layer, h, Bh, row0);
  int32_t *idx = cand ? reinterpret_cast<int32_t *>(ws + w.cand_idx) + unit * kMaxCandPerHead
                      : O.indices + (int64_t)b * s.hkv * s.B + row0;
  uint32_t *ckey = cand ? reinterpret_cast<uint32_t *>(ws + w.cand_key) + unit * kMaxCandPerHead : nullptr;
  const int Bp = cand ? cand_m : Bh - s.W;
  if (Bp > 0) top_select<THREADS, EPT>(a, nvalid, base, Bp, idx, ckey, s.floor_, sc);
  if (!cand) finish_head(s, O, b, h, Bh, row0, idx, THREADS);
}

// candsplit_kernel: head-adaptive budgets from candidate lists, one workgroup per (layer, batch
// item).  Every head brings its best M candidates (ascending positions, with keys, its f best
// marked); a head keeps its floor, i.e. its f best, and the rest of the layer's pool goes to the
// best remaining candidates of all heads together, ties to the smaller head, then the smaller
// position.  A head can keep at most f + H * (B' - f) <= M candidates, so the lists hold every
// candidate that can be kept and the result is the same as ranking all scores.  Thread t owns the
// entries [4t, 4t + 4) of the H lists laid end to end: that order is the tie order, and the kept
// entries of a head come out in ascending position from one prefix sum.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void candsplit_kernel(Shape s, LayerOutTable out, char *ws, Workspace w, int64_t unit0,
                                                              int M) {
  constexpr int NW = THREADS / 64, EPT = 4;
  __shared__ MsScratch sc;
  __shared__ int hstart[65];                           // kept entries before each head's list; [H]: all
  const int tid = threadIdx.x, lb = blockIdx.x, layer = lb / s.batch, b = lb - layer * s.batch;
  const LayerOut O = out.l[layer];
  const int Nc = s.Nc, H = s.hkv, n = H * M, rest = H * (s.Bp - s.floor_);
  const int64_t unit = unit0 + (int64_t)lb * H;        // first head of this (layer, batch item)
  const uint32_t *cidx = reinterpret_cast<const uint32_t *>(ws + w.cand_idx) + unit * kMaxCandPerHead;
  const uint32_t *ckey = reinterpret_cast<const uint32_t *>(ws + w.cand_key) + unit * kMaxCandPerHead;
  int32_t *idx = O.indices + (int64_t)b * H * s.B;
  if (tid == 0) { sc.ur[0] = 0xffffffffu; sc.ur[1] = 0u; }
  uint32_t key[EPT], pw[EPT];
  int head[EPT];
  uint32_t inmask = 0, vmask = 0;                       // entries inside the lists; of those, outside the floors
  uint32_t kmin = 0xffffffffu, kmax = 0;
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int e = tid * EPT + j;
    head[j] = e / M;
    key[j] = 0; pw[j] = 0;
    if (e < n) {
      const int at = head[j] * kMaxCandPerHead + (e - head[j] * M);
      key[j] = ckey[at];
      pw[j] = cidx[at];
      inmask |= 1u << j;
      if (!(pw[j] & kFloorFlag)) { vmask |= 1u << j; kmin = min(kmin, key[j]); kmax = max(kmax, key[j]); }
    }
  }
  __syncthreads();
  uint32_t tau = 0xffffffffu;
  int k = 0;
  if (rest > 0) {
    block_minmax_u32(kmin, kmax, sc);
    tau = radix_threshold<THREADS, EPT>(key, vmask, kmin, kmax, rest, sc, k);
  }
  int ngt = 0, neq = 0;
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const bool v = ((vmask >> j) & 1u) != 0 && rest > 0;
    ngt += (((inmask & ~vmask) >> j) & 1u) + ((v && key[j] > tau) ? 1 : 0);    // floor entries are kept as they are
    neq += (v && key[j] == tau) ? 1 : 0;
  }
  int total;
  const int packed = block_scan_excl<NW>(ngt | (neq << 16), sc, &total);
  int seen = packed >> 16;
  int pos = (packed & 0xffff) + min(seen, k);          // kept entries before this thread's
  const int kept = (total & 0xffff) + min(total >> 16, k);
  bool keep[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const bool v = ((vmask >> j) & 1u) != 0 && rest > 0;
    keep[j] = (((inmask & ~vmask) >> j) & 1u) != 0 || (v && key[j] > tau);
    if (v && key[j] == tau) keep[j] = seen++ < k;
    if (((inmask >> j) & 1u) && tid * EPT + j == head[j] * M) hstart[head[j]] = pos;   // first entry of a list
    if (keep[j]) idx[pos + head[j] * s.W] = (int32_t)(pw[j] & ~kFloorFlag);
    pos += keep[j] ? 1 : 0;
  }
  if (tid == 0) hstart[H] = kept;
  __syncthreads();
  // per head: count, offset, and the window behind the kept candidates
  for (int h = tid >> 6; h < H; h += NW) {
    const int lane = tid & 63, first = hstart[h] + h * s.W, cnt = hstart[h + 1] - hstart[h];
    for (int wv = lane; wv < s.W; wv += 64) idx[first + cnt + wv] = Nc + wv;
    if (lane == 0) {
      O.counts[b * H + h] = cnt + s.W;
      O.offsets[b * (H + 1) + h] = first;
      if (h == H - 1) O.offsets[b * (H + 1) + H] = first + cnt + s.W;
    }
  }
}

// Largest sequence the fused kernel handles: 32 candidates per thread, and the raw attention row
// must fit in LDS next to the scratch.
constexpr int kMsMaxLds = 140 * 1024;

// Raises a kernel's dynamic-LDS limit to kMsMaxLds the first time it is launched on a device.
struct LdsLimitOnce {
  static constexpr int kMaxDevices = 64;
  std::mutex mu;
  bool done[kMaxDevices] = {};
  hipError_t raise(const void *kern) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!done[dev]) {
      e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMsMaxLds);
      if (e != hipSuccess) return e;
      done[dev] = true;
    }
    return hipSuccess;
  }
};
bool mixsel_supported(const Shape &s) { return s.Nc <= kMsMaxThreads * 32 && (size_t)(s.Nc + s.Nc / 32 + 1) * 4 <= (size_t)kMsMaxLds; }

template <int THREADS, int EPT>
static hipError_t launch_mixsel_e(const Shape &s, bool select, const LayerOutTable &out, char *ws, const Workspace &w,
                                  int64_t unit0, int nunits, const LayerInTable &in, int gather_eb, int cand_m,
                                  const int32_t *budgets, hipStream_t st) {
  const size_t lds = (size_t)(s.Nc + s.Nc / 32 + 1) * 4;
  // The kernels may use more dynamic LDS than the default limit.  The limit is a property of the
  // kernel, shared by every stream and thread, so it is raised once, to the most mixsel_supported
  // admits, once per device, and never touched again (a per-launch value could be lowered by another
  // thread between this thread's call and its launch).
  if (select) {
    auto kern = mixsel_kernel<THREADS, EPT, true>;
    static LdsLimitOnce once;
    const hipError_t attr = once.raise(reinterpret_cast<const void *>(kern));
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, dim3(nunits), dim3(THREADS), lds, st, s, out, ws, w, unit0, in, gather_eb, cand_m, budgets);
  } else {
    auto kern = mixsel_kernel<THREADS, EPT, false>;
    static LdsLimitOnce once;
    const hipError_t attr = once.raise(reinterpret_cast<const void *>(kern));
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, dim3(nunits), dim3(THREADS), lds, st, s, out, ws, w, unit0, in, 0, 0, nullptr);
  }
  return hipGetLastError();
}

// Mix (and, with `select`, selection: the final fixed-budget one, or with cand_m > 0 every head's
// best cand_m candidates for the head-adaptive split; with `gather_eb` > 0 also the gather of the
// kept rows, gather_eb being the element size) for `nunits` units starting at unit0.  Few waves per
// workgroup keep the many block-wide steps cheap; long heads get more threads.
hipError_t launch_mixsel(const Shape &s, bool select, const LayerOutTable &out, char *ws, const Workspace &w,
                         int64_t unit0, int nunits, const LayerInTable &in, int gather_eb, int cand_m,
                         const int32_t *budgets, hipStream_t st) {
  const int nc = s.Nc;
  if (nc <= 256 * 8) return launch_mixsel_e<256, 8>(s, select, out, ws, w, unit0, nunits, in, gather_eb, cand_m, budgets, st);
  if (nc <= 512 * 8) return launch_mixsel_e<512, 8>(s, select, out, ws, w, unit0, nunits, in, gather_eb, cand_m, budgets, st);
  if (nc <= 1024 * 8) return launch_mixsel_e<1024, 8>(s, select, out, ws, w, unit0, nunits, in, gather_eb, cand_m, budgets, st);
  if (nc <= 1024 * 16) return launch_mixsel_e<1024, 16>(s, select, out, ws, w, unit0, nunits, in, gather_eb, cand_m, budgets, st);
  return launch_mixsel_e<1024, 32>(s, select, out, ws, w, unit0, nunits, in, gather_eb, cand_m, budgets, st);
}

template <int THREADS, int EPT>
static hipError_t launch_topsel_e(const Shape &s, const LayerOutTable &out, char *ws, const Workspace &w, int64_t unit0,
                                  int nunits, int cand_m, const int32_t *budgets, hipStream_t st) {
  const size_t lds = (size_t)(s.Nc + s.Nc / 32 + 1) * 4;
  auto kern = topsel_kernel<THREADS, EPT>;
  static LdsLimitOnce once;
  const hipError_t attr = once.raise(reinterpret_cast<const void *>(kern));
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(nunits), dim3(THREADS), lds, st, s, out, ws, w, unit0, cand_m, budgets);
  return hipGetLastError();
}

// Selection on scores in memory for `nunits` units starting at unit0 (requires mixsel_supported):
// final rows, or with cand_m > 0 every head's best cand_m candidates for the head-adaptive split.
hipError_t launch_topsel(const Shape &s, const LayerOutTable &out, char *ws, const Workspace &w, int64_t unit0, int nunits,
                         int cand_m, const int32_t *budgets, hipStream_t st) {
  const int nc = s.Nc;
  if (nc <= 256 * 8) return launch_topsel_e<256, 8>(s, out, ws, w, unit0, nunits, cand_m, budgets, st);
  if (nc <= 512 * 8) return launch_topsel_e<512, 8>(s, out, ws, w, unit0, nunits, cand_m, budgets, st);
  if (nc <= 1024 * 8) return launch_topsel_e<1024, 8>(s, out, ws, w, unit0, nunits, cand_m, budgets, st);
  if (nc <= 1024 * 16) return launch_topsel_e<1024, 16>(s, out, ws, w, unit0, nunits, cand_m, budgets, st);
  return launch_topsel_e<1024, 32>(s, out, ws, w, unit0, nunits, cand_m, budgets, st);
}

// The head-adaptive split of `nlayers` layers' candidate lists of M entries per head.
hipError_t launch_select_candidates(const Shape &s, const LayerOutTable &out, char *ws, const Workspace &w, int64_t unit0,
                                    int nlayers, int cand_m, hipStream_t st) {
  const int n = cand_m * s.hkv, grid = nlayers * s.batch;
  if (n <= 256 * 4) hipLaunchKernelGGL(candsplit_kernel<256>, dim3(grid), dim3(256), 0, st, s, out, ws, w, unit0, cand_m);
  else if (n <= 512 * 4) hipLaunchKernelGGL(candsplit_kernel<512>, dim3(grid), dim3(512), 0, st, s, out, ws, w, unit0, cand_m);
  else hipLaunchKernelGGL(candsplit_kernel<1024>, dim3(grid), dim3(1024), 0, st, s, out, ws, w, unit0, cand_m);
  return hipGetLastError();
}

}  // namespace mixkv
