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

// k-th largest key among the valid elements idx in [0, n): returns the threshold key and how many
// elements equal to it are still needed (need >= 1).  Requires 1 <= k <= number of valid elements.
// KeyFn: (int idx, uint32_t &key) -> bool valid.
template <class KeyFn>
__device__ void radix_select(int n, int k, KeyFn keyfn, SelectScratch &sc, uint32_t *tau, int *need) {
  uint32_t prefix = 0, mask = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = threadIdx.x; i < 256; i += blockDim.x) sc.hist[i] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      uint32_t key;
      if (keyfn(i, key) && (key & mask) == prefix) atomicAdd(&sc.hist[(key >> shift) & 0xff], 1);
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

// Index of the `need`-th (1-based) valid element with key == tau, in index order.
template <class KeyFn>
__device__ int kth_equal_index(int n, uint32_t tau, int need, KeyFn keyfn, SelectScratch &sc) {
  const int per = (n + blockDim.x - 1) / blockDim.x;
  const int lo = min(n, (int)threadIdx.x * per), hi = min(n, lo + per);
  int cnt = 0;
  for (int i = lo; i < hi; ++i) {
    uint32_t key;
    if (keyfn(i, key) && key == tau) ++cnt;
  }
  int total;
  int excl = block_exclusive_scan(cnt, sc.iscr, &total);
  if (excl < need && need <= excl + cnt) {
    int seen = excl;
    for (int i = lo; i < hi; ++i) {
      uint32_t key;
      if (keyfn(i, key) && key == tau && ++seen == need) { sc.cut = i; break; }
    }
  }
  __syncthreads();
  int cut = sc.cut;
  __syncthreads();
  return cut;
}

// Ordered compaction: writes the indices i in [0, n) with pred(i), ascending, to dst (at most `cap`
// of them, the size of the destination); returns the count.
template <class Pred>
__device__ int compact_ascending(int n, Pred pred, int32_t *dst, int cap, SelectScratch &sc) {
  const int per = (n + blockDim.x - 1) / blockDim.x;
  const int lo = min(n, (int)threadIdx.x * per), hi = min(n, lo + per);
  int cnt = 0;
  for (int i = lo; i < hi; ++i) cnt += pred(i) ? 1 : 0;
  int total;
  int pos = block_exclusive_scan(cnt, sc.iscr, &total);
  for (int i = lo; i < hi; ++i)
    if (pred(i)) {
      if (pos < cap) dst[pos] = i;
      ++pos;
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
                                                            int64_t unit0) {
  __shared__ float fscr[kSelectThreads / 64 + 1];
  const int ul = blockIdx.x, tid = threadIdx.x, NT = blockDim.x;
  const int64_t unit = unit0 + ul;
  const int layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  float *scores = out.l[layer].scores + (int64_t)bh * s.N;
  const float *araw = reinterpret_cast<const float *>(ws + w.araw) + unit * s.Npad;
  const float *vnorm = reinterpret_cast<const float *>(ws + w.vnorm) + unit * s.Npad;
  const float *kdot = reinterpret_cast<const float *>(ws + w.sdiv) + unit * s.Npad;
  const float *invn = reinterpret_cast<const float *>(ws + w.invnorm) + unit * s.Npad;
  auto sdiv_at = [&](int i) { return -kdot[i] * invn[i]; };   // s_div_i = -Khat_i . Kbar
  const float r = reinterpret_cast<const float *>(ws + w.rbar)[unit];
  const int Nc = s.Nc;
  const bool use_v = s.intrinsic == MIXKV_INTRINSIC_VNORM;
  const float inv_n = 1.f / (float)Nc;

  float sum_ex = 0.f, vmin = INFINITY, vmax = -INFINITY, dmin = INFINITY, dmax = -INFINITY;
  for (int i = tid; i < Nc; i += NT) {
    float a = pooled(araw, i, Nc, s.pool, s.pool_k);
    scores[i] = a;                          // parked here; re-read by the same thread below
    sum_ex += a;
    if (use_v) { float v = vnorm[i]; vmin = fminf(vmin, v); vmax = fmaxf(vmax, v); }
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
    if (use_v) sum_in += (vnorm[i] - vmin) / vden;
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
    if (use_v) imp += ((vnorm[i] - vmin) / vden) * f_in;
    scores[i] = imp;
    sum_imp += imp;
  }
  const float mean_imp = block_reduce<OpSum>(sum_imp, fscr) * inv_n;
  const float f_div = mean_imp / (mean_dn + s.eps);
  for (int i = tid; i < Nc; i += NT) {
    float dn = (sdiv_at(i) - dmin) / dden;
    scores[i] = (1.f - r) * scores[i] + r * (dn * f_div);
  }
  for (int i = Nc + tid; i < s.N; i += NT) scores[i] = INFINITY;
}

// ------------------------------------------------------------------------------------------------
// select kernels (paper Sec. 3.1 TopB; Algorithm 1 TopB step: B' = B - W candidates, window kept)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelectThreads) void select_fixed_kernel(Shape s, LayerOutTable out) {
  __shared__ SelectScratch sc;
  const int ul = blockIdx.x, layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  const LayerOut O = out.l[layer];
  const float *scores = O.scores + (int64_t)bh * s.N;
  int32_t *idx = O.indices + (int64_t)bh * s.B;
  auto keyfn = [&](int i, uint32_t &key) { key = order_key(scores[i]); return true; };
  if (s.Bp > 0) {
    uint32_t tau;
    int need;
    radix_select(s.Nc, s.Bp, keyfn, sc, &tau, &need);
    const int cut = kth_equal_index(s.Nc, tau, need, keyfn, sc);
    compact_ascending(s.Nc, [&](int i) { uint32_t k = order_key(scores[i]); return k > tau || (k == tau && i <= cut); },
                      idx, s.Bp, sc);
  }
  for (int wv = threadIdx.x; wv < s.W; wv += blockDim.x) idx[s.Bp + wv] = s.Nc + wv;
  if (threadIdx.x == 0) {
    const int h = bh % s.hkv, b = bh / s.hkv;
    O.counts[bh] = s.B;
    if (O.offsets) {
      O.offsets[b * (s.hkv + 1) + h] = h * s.B;
      if (h == s.hkv - 1) O.offsets[b * (s.hkv + 1) + s.hkv] = s.hkv * s.B;
    }
  }
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
      radix_select(Nc, f, keyfn, sc, &tau, &need);
      cut = kth_equal_index(Nc, tau, need, keyfn, sc);
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
    auto keyfn = [&](int fi, uint32_t &key) {
      const int h = fi / Nc, i = fi - h * Nc;
      key = order_key(scores[(int64_t)h * s.N + i]);
      return !in_floor(h, i, key);
    };
    int need;
    radix_select(H * Nc, rest, keyfn, sc, &tauR, &need);
    cutR = kth_equal_index(H * Nc, tauR, need, keyfn, sc);
  }

  // 3. per head: ordered compaction of floor set + share of the pool, then the window
  int base = 0;
  for (int h = 0; h < H; ++h) {
    const float *sh = scores + (int64_t)h * s.N;
    auto pred = [&](int i) {
      uint32_t key = order_key(sh[i]);
      if (in_floor(h, i, key)) return true;
      return rest > 0 && (key > tauR || (key == tauR && h * Nc + i <= cutR));
    };
    const int cnt = compact_ascending(Nc, pred, idx + base, H * s.B - base - s.W * (H - h), sc);
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
  if (s.adaptive) {
    const int32_t *offs = O.offsets + b * (H + 1);
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
hipError_t launch_mix(const Shape &s, const LayerOutTable &out, char *ws, const Workspace &w, int64_t unit0, int nunits,
                      hipStream_t st) {
  hipLaunchKernelGGL(mix_kernel, dim3(nunits), dim3(kSelectThreads), 0, st, s, out, ws, w, unit0);
  return hipGetLastError();
}

hipError_t launch_select(const Shape &s, const LayerOutTable &out, int nlayers, hipStream_t st) {
  if (s.adaptive)
    hipLaunchKernelGGL(select_adaptive_kernel, dim3(nlayers * s.batch), dim3(kSelectThreads), 0, st, s, out);
  else
    hipLaunchKernelGGL(select_fixed_kernel, dim3(nlayers * s.units_per_layer), dim3(kSelectThreads), 0, st, s, out);
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

int max_adaptive_heads() { return kMaxAdaptiveHeads; }

}  // namespace mixkv
