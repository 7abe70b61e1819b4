// Score mixing, top-B selection and the K/V gather: everything that works on N floats per head
// instead of N*D cache elements.
#include "mixkv_internal.h"

namespace mixkv {

constexpr int kMaxAdaptiveHeads = 64;

// ------------------------------------------------------------------------------------------------
// block-wide helpers (blockDim.x == kSelectThreads, a multiple of 64)
// ------------------------------------------------------------------------------------------------
struct OpSum { __device__ static float id() { return 0.f; } __device__ static float f(float a, float b) { return a + b; } };
struct OpMin { __device__ static float id() { return INFINITY; } __device__ static float f(float a, float b) { return fminf(a, b); } };
struct OpMax { __device__ static float id() { return -INFINITY; } __device__ static float f(float a, float b) { return fmaxf(a, b); } };

template <class Op>
__device__ float block_reduce(float v, float *scratch /* [blockDim/64 + 1] */) {
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) v = Op::f(v, __shfl_xor(v, sft));
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();                       // scratch may still be read by a previous call
  if ((threadIdx.x & 63) == 0) scratch[wave] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    float a = Op::id();
    for (int i = 0; i < nw; ++i) a = Op::f(a, scratch[i]);   // fixed order
    scratch[nw] = a;
  }
  __syncthreads();
  return scratch[nw];
}

// Exclusive prefix sum of one int per thread; *total receives the block sum.
__device__ int block_exclusive_scan(int v, int *scratch /* [blockDim/64 + 1] */, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  int inc = v;
#pragma unroll
  for (int sft = 1; sft < 64; sft <<= 1) {
    int o = __shfl_up(inc, sft);
    if (lane >= sft) inc += o;
  }
  __syncthreads();
  if (lane == 63) scratch[wave] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    int a = 0;
    for (int i = 0; i < nw; ++i) { int t = scratch[i]; scratch[i] = a; a += t; }
    scratch[nw] = a;
  }
  __syncthreads();
  *total = scratch[nw];
  return scratch[wave] + inc - v;
}

// Order-preserving map float -> uint32 (larger float <=> larger key); -0 is folded onto +0 so
// that equal scores have equal keys.
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct SelectScratch {
  int hist[256];
  int iscr[kSelectThreads / 64 + 1];
  int bin, krem, cut;
};

// One count into a shared histogram bin per lane, with the lanes that share the wave's most common
// bin (as seen from its first active lane) merged into a single atomic: scores of one head often
// agree in their leading bits, and 64 atomics on one LDS word would run one after the other.
__device__ __forceinline__ void hist_add_merged(int *hist, int bin, bool on) {
  const unsigned long long act = __ballot(on);
  if (act == 0) return;
  const int first = __ffsll((long long)act) - 1;                  // wave-uniform
  const int b0 = __builtin_amdgcn_readlane(bin, first);
  const unsigned long long same = __ballot(on && bin == b0);
  if ((int)(threadIdx.x & 63) == first) atomicAdd(&hist[b0], __popcll(same));
  if (on && bin != b0) atomicAdd(&hist[bin], 1);
}

// k-th largest key among the valid elements (r, i), r in [0, rows), i in [0, n), ranked by key
// (rows exist so that a caller with several heads needs no division per element): returns the
// threshold key and how many elements equal to it are still needed (need >= 1).  Requires
// 1 <= k <= number of valid elements.  KeyFn: (int r, int i, uint32_t &key) -> bool valid.
template <class KeyFn>
__device__ void radix_select(int rows, int n, int k, KeyFn keyfn, SelectScratch &sc, uint32_t *tau, int *need) {
  uint32_t prefix = 0, mask = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = threadIdx.x; i < 256; i += blockDim.x) sc.hist[i] = 0;
    __syncthreads();
    constexpr int U = 8;                                        // loads in flight per thread
    for (int r = 0; r < rows; ++r)
      for (int i0 = 0; i0 < n; i0 += U * blockDim.x) {          // whole waves stay in the loop: the merge uses ballots
        uint32_t key[U];
        bool on[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
          const int i = i0 + j * blockDim.x + threadIdx.x;
          key[j] = 0;
          on[j] = i < n && keyfn(r, i, key[j]) && (key[j] & mask) == prefix;
        }
#pragma unroll
        for (int j = 0; j < U; ++j) hist_add_merged(sc.hist, (int)((key[j] >> shift) & 0xff), on[j]);
      }
    __syncthreads();
    // scan the bins from the top: thread t looks at bin 255 - t
    int cnt = (threadIdx.x < 256) ? sc.hist[255 - threadIdx.x] : 0;
    int total;
    int excl = block_exclusive_scan(cnt, sc.iscr, &total);
    if (threadIdx.x < 256 && excl < k && k <= excl + cnt) {
      sc.bin = 255 - threadIdx.x;
      sc.krem = k - excl;
    }
    __syncthreads();
    prefix |= (uint32_t)sc.bin << shift;
    mask |= 0xffu << shift;
    k = sc.krem;
    __syncthreads();
  }
  *tau = prefix;
  *need = k;
}

// Ownership for ordered passes over n elements: wave w owns the contiguous segment
// [w * seg, (w + 1) * seg) with seg a multiple of 64, and visits it 64 consecutive elements at a
// time (element = segment start + c * 64 + lane), so every load is one contiguous 256-byte run.
// The order of elements is (wave, c, lane) = ascending index.
struct WaveSeg {
  int lo, hi, lane, wave, nw;
  __device__ WaveSeg(int n) {
    lane = threadIdx.x & 63; wave = threadIdx.x >> 6; nw = blockDim.x >> 6;
    const int seg = ((n + nw - 1) / nw + 63) / 64 * 64;
    lo = min(n, wave * seg); hi = min(n, lo + seg);
  }
};
__device__ __forceinline__ int lanes_below(unsigned long long m) {   // set bits of m at lanes below this one
  return __popcll(m & ((1ull << (threadIdx.x & 63)) - 1ull));
}

// Exclusive prefix over the waves of one int per wave (the same value in all its lanes); *total
// receives the block sum.
__device__ int wave_totals_scan(int wtot, SelectScratch &sc, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if (lane == 0) sc.iscr[wave] = wtot;
  __syncthreads();
  int before = 0, all = 0;
  for (int i = 0; i < nw; ++i) { const int t = sc.iscr[i]; before += i < wave ? t : 0; all += t; }
  *total = all;
  return before;
}

// Position r * n + i of the `need`-th (1-based) valid element with key == tau, in (row, index)
// order.
template <class KeyFn>
__device__ int kth_equal_index(int rows, int n, uint32_t tau, int need, KeyFn keyfn, SelectScratch &sc) {
  constexpr int U = 4;
  const WaveSeg g(n);
  if (threadIdx.x == 0) sc.cut = -1;
  for (int r = 0; r < rows; ++r) {
    int wtot = 0;
    for (int c0 = g.lo; c0 < g.hi; c0 += 64 * U) {
      bool eq[U];
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const int i = c0 + j * 64 + g.lane;
        uint32_t key = 0;
        eq[j] = i < g.hi && keyfn(r, i, key) && key == tau;
      }
#pragma unroll
      for (int j = 0; j < U; ++j) wtot += __popcll(__ballot(eq[j]));
    }
    int total;
    const int before = wave_totals_scan(wtot, sc, &total);
    if (need <= total) {                               // block-uniform: the element is in this row
      if (before < need && need <= before + wtot) {    // wave-uniform: and in this wave's segment
        int seen = before;
        for (int c0 = g.lo; c0 < g.hi; c0 += 64) {
          const int i = c0 + g.lane;
          uint32_t key = 0;
          const bool eq = i < g.hi && keyfn(r, i, key) && key == tau;
          const unsigned long long m = __ballot(eq);
          if (eq && seen + lanes_below(m) + 1 == need) sc.cut = r * n + i;
          seen += __popcll(m);
          if (seen >= need) break;
        }
      }
      break;
    }
    need -= total;
  }
  __syncthreads();
  int cut = sc.cut;
  __syncthreads();
  return cut;
}

// Ordered compaction: writes the indices i in [0, n) with pred(i, scores[i]), ascending, to dst
// (at most `cap` of them, the size of the destination); returns the count.
template <class Pred>
__device__ int compact_ascending(int n, const float *scores, Pred pred, int32_t *dst, int cap, SelectScratch &sc) {
  constexpr int U = 4;
  const WaveSeg g(n);
  int wtot = 0;
  for (int c0 = g.lo; c0 < g.hi; c0 += 64 * U) {
    bool in[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const int i = c0 + j * 64 + g.lane;
      const float v = i < g.hi ? scores[i] : 0.f;
      in[j] = i < g.hi && pred(i, v);
    }
#pragma unroll
    for (int j = 0; j < U; ++j) wtot += __popcll(__ballot(in[j]));
  }
  int total;
  int pos = wave_totals_scan(wtot, sc, &total);
  for (int c0 = g.lo; c0 < g.hi; c0 += 64 * U) {
    bool in[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const int i = c0 + j * 64 + g.lane;
      const float v = i < g.hi ? scores[i] : 0.f;
      in[j] = i < g.hi && pred(i, v);
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const unsigned long long m = __ballot(in[j]);
      const int at = pos + lanes_below(m);
      if (in[j] && at < cap) dst[at] = c0 + j * 64 + g.lane;
      pos += __popcll(m);
    }
  }
  return min(total, cap);
}

// ------------------------------------------------------------------------------------------------
// mix_kernel: one workgroup per unit.  Pools the window attention (candidates only), min-max
// normalises and mean-matches the value norms and the diversity, and mixes with the head's
// redundancy (paper Sec. 3.2 Eq. 2, Sec. 3.3 Eq. 5; Algorithm 1).  All statistics are over the
// Nc candidates.  Writes s_comp to scores[0, Nc) and +inf to the window slots.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float pooled(const float *a, int i, int n, int mode, int k) {
  if (mode == MIXKV_POOL_NONE || k == 1) return a[i];
  const int half = k >> 1, lo = max(0, i - half), hi = min(n - 1, i + half);
  if (mode == MIXKV_POOL_MAX) {
    float m = a[lo];
    for (int j = lo + 1; j <= hi; ++j) m = fmaxf(m, a[j]);
    return m;
  }
  float sum = 0.f;
  for (int j = lo; j <= hi; ++j) sum += a[j];
  return sum / (float)k;
}

__global__ __launch_bounds__(kSelectThreads) void mix_kernel(Shape s, LayerOutTable out, char *ws, Workspace w,
                                                            int64_t unit0, LayerInTable in) {
  __shared__ float fscr[kSelectThreads / 64 + 1];
  const int ul = blockIdx.x, tid = threadIdx.x, NT = blockDim.x;
  const int64_t unit = unit0 + ul;
  const int layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  float *scores = out.l[layer].scores + (int64_t)bh * s.N;
  const float *araw = reinterpret_cast<const float *>(ws + w.araw) + unit * s.Npad;
  const float *vnorm = reinterpret_cast<const float *>(ws + w.vnorm) + unit * s.Npad;
  const float *kdot = reinterpret_cast<const float *>(ws + w.sdiv) + unit * s.Npad;
  const float *invn = reinterpret_cast<const float *>(ws + w.invnorm) + unit * s.Npad;
  // s_div_i = -Khat_i . Kbar: a product rounded on its own wherever it is formed.  Its minimum has to
  // cancel exactly against the same product further down, so the compiler may not fuse it into
  // the subtraction there (the empty statement hides where the value came from).
  auto sdiv_at = [&](int i) {
    if (!s.kstats) return 0.f;                 // nobody wrote the key statistics: diversity 0, weight 0
    float d = -kdot[i] * invn[i];
    asm("" : "+v"(d));
    return d;
  };
  const float r = reinterpret_cast<const float *>(ws + w.rbar)[unit];
  const int Nc = s.Nc;
  const bool use_v = s.intrinsic != MIXKV_INTRINSIC_NONE;
  const bool knorm = s.intrinsic == MIXKV_INTRINSIC_KNORM;
  auto sin_at = [&](int i) { return knorm ? neg_key_norm(invn[i]) : vnorm[i]; };   // intrinsic score (Sec. 3.2)
  const float inv_n = 1.f / (float)Nc;
  float wi, wd;
  mix_weights(s.mix, r, s.mix == MIXKV_MIX_GIVEN_R ? in.l[layer].r_given[bh] : 0.f, wi, wd);

  float sum_ex = 0.f, vmin = INFINITY, vmax = -INFINITY, dmin = INFINITY, dmax = -INFINITY;
  for (int i = tid; i < Nc; i += NT) {
    float a = pooled(araw, i, Nc, s.pool, s.pool_k);
    scores[i] = a;                          // parked here; re-read by the same thread below
    sum_ex += a;
    if (use_v) { float v = sin_at(i); vmin = fminf(vmin, v); vmax = fmaxf(vmax, v); }
    float d = sdiv_at(i);
    dmin = fminf(dmin, d);
    dmax = fmaxf(dmax, d);
  }
  const float mean_ex = block_reduce<OpSum>(sum_ex, fscr) * inv_n;
  dmin = block_reduce<OpMin>(dmin, fscr);
  dmax = block_reduce<OpMax>(dmax, fscr);
  const float dden = dmax - dmin + s.eps;
  float vden = 1.f, f_in = 0.f;
  if (use_v) {
    vmin = block_reduce<OpMin>(vmin, fscr);
    vmax = block_reduce<OpMax>(vmax, fscr);
    vden = vmax - vmin + s.eps;
  }
  float sum_in = 0.f, sum_dn = 0.f;
  for (int i = tid; i < Nc; i += NT) {
    if (use_v) sum_in += (sin_at(i) - vmin) / vden;
    sum_dn += (sdiv_at(i) - dmin) / dden;
  }
  const float mean_dn = block_reduce<OpSum>(sum_dn, fscr) * inv_n;
  if (use_v) {
    const float mean_in = block_reduce<OpSum>(sum_in, fscr) * inv_n;
    f_in = mean_ex / (mean_in + s.eps);
  }
  float sum_imp = 0.f;
  for (int i = tid; i < Nc; i += NT) {
    float imp = scores[i];
    if (use_v) imp += ((sin_at(i) - vmin) / vden) * f_in;
    scores[i] = imp;
    sum_imp += imp;
  }
  const float mean_imp = block_reduce<OpSum>(sum_imp, fscr) * inv_n;
  const float f_div = mean_imp / (mean_dn + s.eps);
  for (int i = tid; i < Nc; i += NT) {
    float dn = (sdiv_at(i) - dmin) / dden;
    scores[i] = wi * scores[i] + wd * (dn * f_div);
  }
  for (int i = Nc + tid; i < s.N; i += NT) scores[i] = INFINITY;
}

// ------------------------------------------------------------------------------------------------
// select kernels (paper Sec. 3.1 TopB; Algorithm 1 TopB step: B' = B - W candidates, window kept)
// ------------------------------------------------------------------------------------------------
// One workgroup per unit; every head keeps B rows, or with a budget table (per-head mode,
// [layers of this launch][hkv]) its own entry, the heads of a batch item packed back to back.
__global__ __launch_bounds__(kSelectThreads) void select_fixed_kernel(Shape s, LayerOutTable out, const int32_t *budgets) {
  __shared__ SelectScratch sc;
  const int ul = blockIdx.x, layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  const int h = bh % s.hkv, b = bh / s.hkv;
  const LayerOut O = out.l[layer];
  const float *scores = O.scores + (int64_t)bh * s.N;
  int Bh = s.B, row0 = h * s.B;
  if (budgets) {
    const int32_t *bl = budgets + layer * s.hkv;
    row0 = 0;
    for (int j = 0; j < h; ++j) row0 += bl[j];
    Bh = bl[h];
  }
  const int Bp = Bh - s.W;
  int32_t *idx = O.indices + (int64_t)b * s.hkv * s.B + row0;
  auto keyfn = [&](int i, uint32_t &key) { key = order_key(scores[i]); return true; };
  if (Bp > 0) {
    uint32_t tau;
    int need;
    radix_select(1, s.Nc, Bp, [&](int, int i, uint32_t &key) { return keyfn(i, key); }, sc, &tau, &need);
    const int cut = kth_equal_index(1, s.Nc, tau, need, [&](int, int i, uint32_t &key) { return keyfn(i, key); }, sc);
    compact_ascending(s.Nc, scores, [&](int i, float v) { uint32_t k = order_key(v); return k > tau || (k == tau && i <= cut); },
                      idx, Bp, sc);
  }
  for (int wv = threadIdx.x; wv < s.W; wv += blockDim.x) idx[Bp + wv] = s.Nc + wv;
  if (threadIdx.x == 0) {
    O.counts[bh] = Bh;
    if (O.offsets) {
      O.offsets[b * (s.hkv + 1) + h] = row0;
      if (h == s.hkv - 1) O.offsets[b * (s.hkv + 1) + s.hkv] = row0 + Bh;
    }
  }
}

struct IntChunk { int32_t v[512]; };
__global__ void upload_ints_kernel(IntChunk c, int n, int32_t *dst) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = c.v[i];
}
hipError_t upload_ints(const int32_t *host, int n, int32_t *dev, hipStream_t st) {
  for (int at = 0; at < n; at += 512) {
    IntChunk c;
    const int m = n - at < 512 ? n - at : 512;
    for (int i = 0; i < m; ++i) c.v[i] = host[at + i];
    hipLaunchKernelGGL(upload_ints_kernel, dim3(2), dim3(256), 0, st, c, m, dev + at);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Head-adaptive budgets: one workgroup per (layer, batch item).
__global__ __launch_bounds__(kSelectThreads) void select_adaptive_kernel(Shape s, LayerOutTable out) {
  __shared__ SelectScratch sc;
  __shared__ uint32_t tauF[kMaxAdaptiveHeads];
  __shared__ int cutF[kMaxAdaptiveHeads];
  __shared__ int offs[kMaxAdaptiveHeads + 1];
  const int lb = blockIdx.x, layer = lb / s.batch, b = lb - layer * s.batch;
  const LayerOut O = out.l[layer];
  const float *scores = O.scores + (int64_t)b * s.hkv * s.N;
  const int Nc = s.Nc, H = s.hkv, f = s.floor_;
  int32_t *idx = O.indices + (int64_t)b * H * s.B;

  // 1. every head's own top-`floor`
  for (int h = 0; h < H; ++h) {
    const float *sh = scores + (int64_t)h * s.N;
    uint32_t tau = 0xffffffffu;
    int cut = -1;
    if (f > 0) {
      auto keyfn = [&](int i, uint32_t &key) { key = order_key(sh[i]); return true; };
      int need;
      radix_select(1, Nc, f, [&](int, int i, uint32_t &key) { return keyfn(i, key); }, sc, &tau, &need);
      cut = kth_equal_index(1, Nc, tau, need, [&](int, int i, uint32_t &key) { return keyfn(i, key); }, sc);
    }
    if (threadIdx.x == 0) { tauF[h] = tau; cutF[h] = cut; }
    __syncthreads();
  }
  auto in_floor = [&](int h, int i, uint32_t key) { return f > 0 && (key > tauF[h] || (key == tauF[h] && i <= cutF[h])); };

  // 2. the rest of the layer's pool goes to the best remaining candidates of all heads together
  const int rest = H * (s.Bp - f);
  uint32_t tauR = 0xffffffffu;
  int cutR = -1;
  if (rest > 0) {
    auto keyfn = [&](int h, int i, uint32_t &key) {
      key = order_key(scores[(int64_t)h * s.N + i]);
      return !in_floor(h, i, key);
    };
    int need;
    radix_select(H, Nc, rest, keyfn, sc, &tauR, &need);
    cutR = kth_equal_index(H, Nc, tauR, need, keyfn, sc);
  }

  // 3. per head: ordered compaction of floor set + share of the pool, then the window
  int base = 0;
  for (int h = 0; h < H; ++h) {
    const float *sh = scores + (int64_t)h * s.N;
    auto pred = [&](int i, float v) {
      uint32_t key = order_key(v);
      if (in_floor(h, i, key)) return true;
      return rest > 0 && (key > tauR || (key == tauR && h * Nc + i <= cutR));
    };
    const int cnt = compact_ascending(Nc, sh, pred, idx + base, H * s.B - base - s.W * (H - h), sc);
    for (int wv = threadIdx.x; wv < s.W; wv += blockDim.x) idx[base + cnt + wv] = Nc + wv;
    if (threadIdx.x == 0) {
      O.counts[b * H + h] = cnt + s.W;
      offs[h] = base;
    }
    base += cnt + s.W;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    offs[H] = base;
    for (int h = 0; h <= H; ++h) O.offsets[b * (H + 1) + h] = offs[h];
  }
}

// ------------------------------------------------------------------------------------------------
// gather_kernel: K_out[p] = K[idx[p]], V_out[p] = V[idx[p]] for the packed kept rows p of one
// (layer, batch item); 16 bytes per lane, a row is D*EB/16 consecutive lanes (Sec. 3.1, the
// compacted cache).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_kernel(Shape s, int eb, LayerInTable in, LayerOutTable out) {
  const int lb = blockIdx.y, layer = lb / s.batch, b = lb - layer * s.batch;
  const LayerIn L = in.l[layer];
  const LayerOut O = out.l[layer];
  const int ppr = s.D * eb / 16, rows_per_block = blockDim.x / ppr;
  const int p = blockIdx.x * rows_per_block + threadIdx.x / ppr, piece = threadIdx.x % ppr;
  const int H = s.hkv, total = H * s.B;
  if (p >= total) return;
  int h;
  if (s.adaptive || s.per_head) {
    const int32_t *offs = O.offsets + b * (H + 1);
    if (p >= offs[H]) return;                          // per-head budgets may leave the tail unused
    h = 0;
    while (h + 1 < H && p >= offs[h + 1]) ++h;
  } else {
    h = p / s.B;
  }
  const int64_t prow = (int64_t)b * total + p;
  const int src = min(max(O.indices[prow], 0), s.N - 1);   // indices come from select; the clamp only guards the load
  const int64_t src_off = ((int64_t)b * L.sb + (int64_t)h * L.sh + (int64_t)src * L.sn) * eb + piece * 16;
  const int64_t dst_off = prow * s.D * eb + piece * 16;
  uint4 kv = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(L.K) + src_off);
  uint4 vv = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(L.V) + src_off);
  *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(O.K_out) + dst_off) = kv;
  *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(O.V_out) + dst_off) = vv;
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
hipError_t launch_mix(const Shape &s, const LayerInTable &in, const LayerOutTable &out, char *ws, const Workspace &w,
                      int64_t unit0, int nunits, hipStream_t st) {
  hipLaunchKernelGGL(mix_kernel, dim3(nunits), dim3(kSelectThreads), 0, st, s, out, ws, w, unit0, in);
  return hipGetLastError();
}

hipError_t launch_select(const Shape &s, const LayerOutTable &out, int nlayers, const int32_t *budgets, hipStream_t st) {
  if (s.adaptive)
    hipLaunchKernelGGL(select_adaptive_kernel, dim3(nlayers * s.batch), dim3(kSelectThreads), 0, st, s, out);
  else
    hipLaunchKernelGGL(select_fixed_kernel, dim3(nlayers * s.units_per_layer), dim3(kSelectThreads), 0, st, s, out,
                       budgets);
  return hipGetLastError();
}

hipError_t launch_gather(const Shape &s, int dtype, const LayerInTable &in, const LayerOutTable &out, int nlayers,
                         hipStream_t st) {
  const int eb = dtype == MIXKV_BF16 ? 2 : 4;
  const int ppr = s.D * eb / 16, rows_per_block = 256 / ppr;
  const int total = s.hkv * s.B;
  dim3 grid((total + rows_per_block - 1) / rows_per_block, nlayers * s.batch);
  hipLaunchKernelGGL(gather_kernel, grid, dim3(256), 0, st, s, eb, in, out);
  return hipGetLastError();
}

// Candidates a head has to hand to the budget split: its floor plus the whole shared pool; 0 if
// that does not shorten the lists enough for the small kernel.
int adaptive_candidates(const Shape &s) {
  const int64_t M = (int64_t)s.floor_ + (int64_t)s.hkv * (s.Bp - s.floor_);
  if (M < 1 || M > s.Nc || M > kMaxCandPerHead || M * s.hkv > kMaxCandPerGroup) return 0;
  return (int)M;
}

int max_adaptive_heads() { return kMaxAdaptiveHeads; }

}  // namespace mixkv
