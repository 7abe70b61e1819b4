// Attention of one new token over the compacted cache (paper Sec. 3.1: the compressed K, V are
// what the attention of the decoding phase reads).  One workgroup per (layer, batch item, KV head,
// group of up to eight query heads): the head's kept rows, then the rows appended since the
// compression, are streamed once; every lane owns one 16-byte piece of a row slot and carries a
// running softmax (maximum, sum, weighted value piece) per query head, so nothing crosses lanes
// inside the loop except the dot-product reduction over the lanes of a row.  Long caches are
// split over several workgroups per head (contiguous row ranges); each leaves its running softmax
// in the workspace and decode_merge_kernel folds them in order.
//
// bf16 caches go through the matrix cores (decode_mfma_kernel): the rows travel global -> LDS in
// 32-row tiles, the scores of a tile against all query heads of the group are one chain of MFMAs
// with the keys on the output rows, and the weighted values a second product with the weights as
// they stand in the accumulators.  fp32 caches take the vector path (decode_kernel).
#include "mixkv_stream.h"

namespace mixkv {

struct DecodeLayer {
  const void *Kc, *Vc;               // compacted rows as mixkv_compress wrote them
  const int32_t *counts, *offsets;   // rows per head; first row of a head inside its batch item (packed layouts)
  const void *Kt, *Vt;               // [batch, hkv, tail_cap, D] rows appended since
  const void *Q;                     // [batch, hq, D]
  void *out;                         // [batch, hq, D]
};
struct DecodeTable { DecodeLayer l[kLayersPerLaunch]; };

struct DShape {
  int32_t batch, hq, hkv, G, B, tail_len, tail_cap, packed, units_per_layer, gchunks, nsplit;
  int32_t hpw, gt;       // query heads a workgroup serves (per group chunk), and the head stride of its partials
  float scale_log2e;
};

constexpr int kDecThreads = 512, kDecWaves = kDecThreads / 64, kDecHeads = 8;

template <int DT>
__device__ __forceinline__ void unpack16(const uint4 &q, float *x) {
  if constexpr (DT == MIXKV_BF16) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x[2 * j] = __uint_as_float(w[j] << 16);
      x[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
  } else {
    x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y);
    x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
  }
}

__device__ __forceinline__ uint16_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// GT: query heads carried per workgroup (1, 2, 4 or 8; heads past G are idle).
template <int DT, int D, int GT>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(DShape s, DecodeTable tab, float *part) {
  constexpr int EB = DT == MIXKV_BF16 ? 2 : 4, E = 16 / EB, PPR = D * EB / 16, RPL = 64 / PPR;
  __shared__ float sm[kDecWaves][GT], sl[kDecWaves][GT], so[kDecWaves][GT][D];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane / PPR, piece = lane - lr * PPR;
  const int sp = blockIdx.x % s.nsplit, ugc = blockIdx.x / s.nsplit;   // row split, (unit, query-head group)
  const int ul = ugc / s.gchunks, gc = ugc - ul * s.gchunks;
  const int layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  const int b = bh / s.hkv, h = bh - b * s.hkv;
  const DecodeLayer L = tab.l[layer];
  const int g0 = gc * kDecHeads, ng = min(GT, s.G - g0);          // query heads of this workgroup

  // rows of this head: `cnt` compacted ones, then `tail_len` appended ones
  const int cap = s.packed ? s.hkv * s.B : s.B;                   // rows the head's slot can hold at most
  int row0 = s.packed ? (L.offsets ? L.offsets[b * (s.hkv + 1) + h] : 0) : 0;
  row0 = min(max(row0, 0), cap);
  const int cnt = min(max(L.counts[bh], 0), cap - row0);          // the clamps only guard the loads
  const int n_all = cnt + s.tail_len;
  const int r_begin = (int)((int64_t)n_all * sp / s.nsplit), n = (int)((int64_t)n_all * (sp + 1) / s.nsplit);   // rows [r_begin, n)
  const int64_t slot_rows = s.packed ? (int64_t)b * s.hkv * s.B + row0 : (int64_t)bh * s.B;
  const char *Kc = reinterpret_cast<const char *>(L.Kc) + slot_rows * D * EB;
  const char *Vc = reinterpret_cast<const char *>(L.Vc) + slot_rows * D * EB;
  const char *Kt = reinterpret_cast<const char *>(L.Kt) + (int64_t)bh * s.tail_cap * D * EB;
  const char *Vt = reinterpret_cast<const char *>(L.Vt) + (int64_t)bh * s.tail_cap * D * EB;

  // this lane's piece of every query row, already times softmax_scale * log2(e)
  float q[GT][E];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const int gq = g < ng ? g0 + g : g0;
    const uint4 v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(L.Q) +
                                                     ((int64_t)(b * s.hq + h * s.G + gq) * D) * EB + piece * 16);
    unpack16<DT>(v, q[g]);
#pragma unroll
    for (int e = 0; e < E; ++e) q[g][e] *= s.scale_log2e;
  }
  float m[GT], l[GT], o[GT][E];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) o[g][e] = 0.f;
  }

  auto row_ptrs = [&](int row, const char *&kp, const char *&vp) {
    if (row < cnt) { kp = Kc + (int64_t)row * D * EB; vp = Vc + (int64_t)row * D * EB; }
    else { kp = Kt + (int64_t)(row - cnt) * D * EB; vp = Vt + (int64_t)(row - cnt) * D * EB; }
  };
  constexpr int U = 4;                                             // row groups in flight per wave
  for (int r = r_begin + wave * RPL; r < n; r += kDecWaves * RPL * U) {
    uint4 kq[U], vq[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = r + u * kDecWaves * RPL + lr;
      ok[u] = row < n;
      kq[u] = make_uint4(0u, 0u, 0u, 0u); vq[u] = kq[u];
      if (ok[u]) {
        const char *kp, *vp;
        row_ptrs(row, kp, vp);
        kq[u] = *reinterpret_cast<const uint4 *>(kp + piece * 16);
        vq[u] = *reinterpret_cast<const uint4 *>(vp + piece * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[E], v[E];
      unpack16<DT>(kq[u], x);
      unpack16<DT>(vq[u], v);
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) part = fmaf(q[g][e], x[e], part);
        const float dot = seg_sum<PPR>(part);                     // all lanes take part in the reduction
        const float sc = ok[u] ? dot : -INFINITY;
        // the running maximum moves (and the sums are rescaled) only in the steps where some row
        // slot of the wave sees a new one
        if (__builtin_amdgcn_ballot_w64(sc > m[g]) != 0) {
          const float mn = fmaxf(m[g], sc);
          const float f = __builtin_amdgcn_exp2f(m[g] - (mn == -INFINITY ? 0.f : mn));
          l[g] *= f;
#pragma unroll
          for (int e = 0; e < E; ++e) o[g][e] *= f;
          m[g] = mn;
        }
        const float p = __builtin_amdgcn_exp2f(sc - (m[g] == -INFINITY ? 0.f : m[g]));
        l[g] += p;
#pragma unroll
        for (int e = 0; e < E; ++e) o[g][e] = fmaf(p, v[e], o[g][e]);
      }
    }
  }
  // fold the row slots of the wave (lanes holding the same piece), then the waves through LDS
#pragma unroll
  for (int off = PPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const float m2 = __shfl_xor(m[g], off), l2 = __shfl_xor(l[g], off);
      const float mn = fmaxf(m[g], m2), mu = mn == -INFINITY ? 0.f : mn;
      const float f1 = __builtin_amdgcn_exp2f(m[g] - mu), f2 = __builtin_amdgcn_exp2f(m2 - mu);
      l[g] = l[g] * f1 + l2 * f2;
#pragma unroll
      for (int e = 0; e < E; ++e) o[g][e] = o[g][e] * f1 + __shfl_xor(o[g][e], off) * f2;
      m[g] = mn;
    }
  }
  if (lane < PPR) {
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      if (piece == 0) { sm[wave][g] = m[g]; sl[wave][g] = l[g]; }
#pragma unroll
      for (int e = 0; e < E; ++e) so[wave][g][piece * E + e] = o[g][e];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < ng * D; idx += kDecThreads) {
    const int g = idx / D, d = idx - g * D;
    float mn = sm[0][g];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) mn = fmaxf(mn, sm[w][g]);
    const float mu = mn == -INFINITY ? 0.f : mn;
    float acc = 0.f, tot = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {                          // waves in order
      const float f = __builtin_amdgcn_exp2f(sm[w][g] - mu);
      acc = fmaf(so[w][g][d], f, acc);
      tot = fmaf(sl[w][g], f, tot);
    }
    if (s.nsplit > 1) {                                            // partial: weighted values, then (max, sum)
      float *dst = part + ((int64_t)blockIdx.x * GT + g) * (D + 2);
      dst[d] = acc;
      if (d == 0) { dst[D] = mn; dst[D + 1] = tot; }
      continue;
    }
    const float res = tot > 0.f ? acc / tot : 0.f;
    const int64_t at = (int64_t)(b * s.hq + h * s.G + g0 + g) * D + d;
    if constexpr (DT == MIXKV_BF16) reinterpret_cast<uint16_t *>(L.out)[at] = bf16_rne(res);
    else reinterpret_cast<float *>(L.out)[at] = res;
  }
}

// ------------------------------------------------------------------------------------------------
// decode_mfma_kernel (bf16): one workgroup of D/32 waves per (layer, batch item, KV head, chunk of
// up to 32 query heads, row range).
//   * Tiles of 32 rows of K and of V go global -> LDS through the ring of mixkv_stream.h (direct
//     loads, requested kLead tiles ahead, bank-rotated images); the compacted rows and the appended
//     tail are two runs of memory, so every lane picks its row's base; rows past the range re-read
//     the last row and are masked.
//   * Scores: keys on the MFMA output rows, query heads on the columns (heads past the chunk are
//     zero columns), so lane (g = lane % 32, half) holds sixteen rows' scores of head g.  Every wave
//     forms the whole score tile and its weights: the waves agree bit for bit, and nothing crosses
//     waves inside the loop.
//   * Weights exp2(x - m_g) with an offset m_g that only moves when a head's sum leaves the range of
//     a float (see stats_kernel), split into a bf16 head and a bf16 remainder; the accumulator
//     registers of one half-wave are, in order, the contraction index of the second product, so they
//     feed it as they stand.
//   * Weighted values: wave w owns the 32 elements [32 w, 32 w + 32) of the output rows; its A
//     operand is that slice of V transposed, read from the tile image two bytes at a time (8 reads
//     per fragment), its output lane (g, half) holds head g's sixteen elements of the slice.
// Partials and outputs have the layout of decode_kernel.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(D * 2, 2) void decode_mfma_kernel(DShape s, DecodeTable tab, float *part) {
  constexpr int DT = MIXKV_BF16, EB = 2, PPR = D * EB / 16, TILE = 32 * PPR, WAVES = D / 32, RPL = 64 / PPR;
  constexpr int NCHK = D / 16;                            // MFMAs per score tile
  constexpr int KL = (TILE / 64 + WAVES - 1) / WAVES;     // requests per wave, tile and tensor
  static_assert(TILE / 64 == KL * WAVES, "every wave issues the same number of requests");
  __shared__ uint4 kring[kRing * TILE], vring[kRing * TILE];

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sp = blockIdx.x % s.nsplit, ugc = blockIdx.x / s.nsplit;   // row split, (unit, query-head chunk)
  const int ul = ugc / s.gchunks, gc = ugc - ul * s.gchunks;
  const int layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  const int b = bh / s.hkv, h = bh - b * s.hkv;
  const DecodeLayer L = tab.l[layer];
  const int g0 = gc * s.hpw, ng = min(s.hpw, s.G - g0);           // query heads of this workgroup
  const float c2 = s.scale_log2e;

  // rows of this head: `cnt` compacted ones, then `tail_len` appended ones
  const int cap = s.packed ? s.hkv * s.B : s.B;                   // rows the head's slot can hold at most
  int row0 = s.packed ? (L.offsets ? L.offsets[b * (s.hkv + 1) + h] : 0) : 0;
  row0 = min(max(row0, 0), cap);
  const int cnt = min(max(L.counts[bh], 0), cap - row0);          // the clamps only guard the loads
  const int n_all = cnt + s.tail_len;
  const int r_begin = (int)((int64_t)n_all * sp / s.nsplit), n = (int)((int64_t)n_all * (sp + 1) / s.nsplit);   // rows [r_begin, n)
  const int nt = (n - r_begin + 31) / 32;                         // tiles of the range
  const int64_t slot_rows = s.packed ? (int64_t)b * s.hkv * s.B + row0 : (int64_t)bh * s.B;
  constexpr int RB = D * EB;
  const char *Kc = reinterpret_cast<const char *>(L.Kc) + slot_rows * RB;
  const char *Vc = reinterpret_cast<const char *>(L.Vc) + slot_rows * RB;
  const char *Kt = reinterpret_cast<const char *>(L.Kt) + ((int64_t)bh * s.tail_cap - cnt) * RB;   // row r >= cnt at Kt + r * RB
  const char *Vt = reinterpret_cast<const char *>(L.Vt) + ((int64_t)bh * s.tail_cap - cnt) * RB;

  const uint32_t kring_a = lds_base_of(kring), vring_a = lds_base_of(vring);
  const int lrow = lane / PPR, lq = lane % PPR;
  // Request tile tr of the range into its ring image: load j covers slots [64 j, 64 j + 64) of the
  // image, i.e. rows [j RPL, (j + 1) RPL) of the tile; wave w issues the loads w, w + WAVES, ...
  auto request = [&](int tr) {
    const int tb = r_begin + tr * 32;
    const uint32_t off = (uint32_t)(tr & (kRing - 1)) * (TILE * 16);
#pragma unroll
    for (int jj = 0; jj < KL; ++jj) {
      const int j = jj * WAVES + wave;
      const int trow = j * RPL + lrow;
      const int row = min(tb + trow, n - 1);                       // rows past the range repeat its last row
      const int64_t at = (int64_t)row * RB + (lq ^ tile_swz<DT, D>(trow)) * 16;
      const char *kp = (row < cnt ? Kc : Kt) + at, *vp = (row < cnt ? Vc : Vt) + at;
      __builtin_amdgcn_global_load_lds((glb_void_t *)kp, (lds_void_t *)(uintptr_t)(kring_a + off + j * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((glb_void_t *)vp, (lds_void_t *)(uintptr_t)(vring_a + off + j * 1024), 16, 0, 0);
    }
  };
#pragma unroll
  for (int j = 0; j < kLead; ++j)
    if (j < nt) request(j);

  // the query heads in fragment form: lane (g, half) holds every other 16-byte piece of head g's row
  Frag qf[NCHK];
  {
    const bool live = l32 < ng;
    const char *qrow = reinterpret_cast<const char *>(L.Q) + ((int64_t)(b * s.hq + h * s.G + g0 + (live ? l32 : 0)) * D) * EB +
                       half * 16;
#pragma unroll
    for (int c = 0; c < NCHK; ++c) {
      const uint4 v = *reinterpret_cast<const uint4 *>(qrow + c * 32);
      qf[c].q = live ? v : make_uint4(0, 0, 0, 0);
    }
  }
  // nothing may be pending when the tile loop is entered: its waits count the requests issued inside it
  wait_vm<0>();

  float m = -INFINITY, l = 0.f;      // head g's offset and this half-wave's share of the sum of weights
  f32x16 o;                          // head g's sixteen output elements of this wave's slice, times 2^-m
#pragma unroll
  for (int i = 0; i < 16; ++i) o[i] = 0.f;
  // two-byte index into a V tile image of element d = 32 wave + l32 of tile row r
  const int vd = wave * 32 + l32;
  auto v_at = [&](int r) { return r * (PPR * 8) + (((vd >> 3) ^ tile_swz<DT, D>(r)) << 3) + (vd & 7); };

  auto tile_step = [&](auto slot_c, int t) {
    constexpr int SLOT = decltype(slot_c)::value;
    __builtin_amdgcn_sched_barrier(0);
    wait_tile<2 * KL>(t, nt);
    lds_barrier();
    if (t + kLead < nt) request(t + kLead);              // into the image tile t - 1 has left
    __builtin_amdgcn_sched_barrier(0);
    const uint4 *img = kring + SLOT * TILE;
    const uint16_t *vimg = reinterpret_cast<const uint16_t *>(vring + SLOT * TILE);
    const int tb = r_begin + t * 32;

    // ---- scores of the tile's 32 rows against the query heads
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    {
      Frag kf[NCHK];
#pragma unroll
      for (int c = 0; c < NCHK; ++c) kf[c].q = read_key_frag<DT, D>(img, 0, c, l32, half);
#pragma unroll
      for (int c = 0; c < NCHK; ++c) acc = mma<DT>(kf[c], qf[c], acc);
    }
    // ---- this wave's slice of V, transposed: fragment ks holds for element d the rows of the
    // accumulator registers [8 ks, 8 ks + 8) of this half-wave
    Frag vf[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        const int ra = 8 * (2 * ks + (j >> 2)) + 4 * half + (j & 3);
        vf[ks].u[j >> 1] = (uint32_t)vimg[v_at(ra)] | ((uint32_t)vimg[v_at(ra + 1)] << 16);
      }
    if (tb + 32 > n) {                                   // the range ends inside the tile: mask
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = (tb + 8 * (i >> 2) + 4 * half + (i & 3) >= n) ? -INFINITY : acc[i];
    }
    // ---- weights.  The terms are formed with the offset as it stands; only if the sum leaves the
    // range (or there is no offset yet) does the wave move the offset to the tile's maximum, rescale
    // what it has and form the terms again.  Both half-waves of a head share the offset.
    float p[16], sum[4];
    {
      const float nmu = -m;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        p[i] = fast_exp2(fmaf(acc[i], c2, nmu));
        sum[i & 3] = i < 4 ? p[i] : sum[i & 3] + p[i];
      }
    }
    float lnew = l + ((sum[0] + sum[1]) + (sum[2] + sum[3]));
    if (__builtin_amdgcn_ballot_w64(!(lnew < 1e30f)) != 0) {
      float tmax = fmaxf(acc[0], acc[1]);
#pragma unroll
      for (int i = 2; i < 16; i += 2) tmax = fmaxf(fmaxf(tmax, acc[i]), acc[i + 1]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float mn = fmaxf(m, tmax * c2);              // c2 > 0: scaling commutes with max
      const float mu = (mn == -INFINITY) ? 0.f : mn;
      const float f = fast_exp2(m - mu);                 // 0 while there is no offset yet
      float s2[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        p[i] = fast_exp2(fmaf(acc[i], c2, -mu));
        s2[i & 3] += p[i];
      }
      lnew = l * f + ((s2[0] + s2[1]) + (s2[2] + s2[3]));
#pragma unroll
      for (int i = 0; i < 16; ++i) o[i] *= f;
      m = mn;
    }
    l = lnew;
    // ---- weighted values: bf16 head and remainder of every weight
    Frag ph[2], pl[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float x = p[8 * ks + j];
        const __bf16 hi = (__bf16)x;
        ph[ks].h[j] = hi;
        pl[ks].h[j] = (__bf16)(x - (float)hi);
      }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      o = mma<DT>(vf[ks], ph[ks], o);
      o = mma<DT>(vf[ks], pl[ks], o);
    }
  };
  static_assert(kRing == 4, "unrolled four times below");
  for (int t = 0; t < nt; t += kRing) {
    tile_step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < nt) tile_step(std::integral_constant<int, 1>{}, t + 1);
    if (t + 2 < nt) tile_step(std::integral_constant<int, 2>{}, t + 2);
    if (t + 3 < nt) tile_step(std::integral_constant<int, 3>{}, t + 3);
  }

  // ---- the head's sum of weights from both half-waves (fixed order), then the outputs
  const float lo = __shfl_xor(l, 32);
  const float tot = half == 0 ? l + lo : lo + l;
  if (l32 >= ng) return;
  if (s.nsplit > 1) {                                    // partial: weighted values, then (offset, sum)
    float *dst = part + ((int64_t)blockIdx.x * s.gt + l32) * (D + 2);
#pragma unroll
    for (int i = 0; i < 16; ++i) dst[wave * 32 + 8 * (i >> 2) + 4 * half + (i & 3)] = o[i];
    if (wave == 0 && half == 0) { dst[D] = m; dst[D + 1] = tot; }
    return;
  }
  uint16_t *out = reinterpret_cast<uint16_t *>(L.out) + (int64_t)(b * s.hq + h * s.G + g0 + l32) * D + wave * 32;
#pragma unroll
  for (int i = 0; i < 16; ++i) out[8 * (i >> 2) + 4 * half + (i & 3)] = bf16_rne(tot > 0.f ? o[i] / tot : 0.f);
}

// Folds the nsplit <= 16 partial results of one (unit, query-head chunk) in split order and writes the
// output rows: one thread per output element (blockIdx.y walks the chunk's elements 256 at a time), every
// split's three values requested before the first is used.
constexpr int kDecMaxSplit = 16;
template <int DT, int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(DShape s, DecodeTable tab, const float *part) {
  const int ugc = blockIdx.x, ul = ugc / s.gchunks, gc = ugc - ul * s.gchunks;
  const int layer = ul / s.units_per_layer, bh = ul - layer * s.units_per_layer;
  const int b = bh / s.hkv, h = bh - b * s.hkv;
  const int g0 = gc * s.hpw, ng = min(s.hpw, s.G - g0);
  const int idx = blockIdx.y * 256 + threadIdx.x;
  if (idx >= ng * D) return;
  const int g = idx / D, d = idx - g * D;
  const float *src = part + ((int64_t)ugc * s.nsplit * s.gt + g) * (D + 2);
  const int64_t step = (int64_t)s.gt * (D + 2);                    // from one split to the next
  float pm[kDecMaxSplit], pa[kDecMaxSplit], pl[kDecMaxSplit];
#pragma unroll
  for (int sp = 0; sp < kDecMaxSplit; ++sp) {
    const bool on = sp < s.nsplit;
    const float *at = src + (on ? sp : 0) * step;
    pm[sp] = on ? at[D] : -INFINITY;
    pa[sp] = on ? at[d] : 0.f;
    pl[sp] = on ? at[D + 1] : 0.f;
  }
  float mn = -INFINITY;
#pragma unroll
  for (int sp = 0; sp < kDecMaxSplit; ++sp) mn = fmaxf(mn, pm[sp]);
  const float mu = mn == -INFINITY ? 0.f : mn;
  float acc = 0.f, tot = 0.f;
#pragma unroll
  for (int sp = 0; sp < kDecMaxSplit; ++sp) {                      // splits in order; absent ones add zeros
    const float f = __builtin_amdgcn_exp2f(pm[sp] - mu);
    acc = fmaf(pa[sp], f, acc);
    tot = fmaf(pl[sp], f, tot);
  }
  const float res = tot > 0.f ? acc / tot : 0.f;
  const int64_t at = (int64_t)(b * s.hq + h * s.G + g0 + g) * D + d;
  if constexpr (DT == MIXKV_BF16) reinterpret_cast<uint16_t *>(tab.l[layer].out)[at] = bf16_rne(res);
  else reinterpret_cast<float *>(tab.l[layer].out)[at] = res;
}

template <int DT, int D, int GT>
static void launch_decode_gt(const DShape &s, const DecodeTable &t, int nunits, float *part, hipStream_t st) {
  const dim3 grid((unsigned)(nunits * s.gchunks * s.nsplit)), block(kDecThreads);
  hipLaunchKernelGGL((decode_kernel<DT, D, GT>), grid, block, 0, st, s, t, part);
  if (s.nsplit > 1)
    hipLaunchKernelGGL((decode_merge_kernel<DT, D>), dim3((unsigned)(nunits * s.gchunks), (unsigned)((s.gt * D + 255) / 256)), dim3(256), 0, st, s, t,
                       part);
}

template <int DT, int D>
static void launch_decode_g(const DShape &s, const DecodeTable &t, int nunits, int gt, float *part, hipStream_t st) {
  switch (gt) {
    case 1: launch_decode_gt<DT, D, 1>(s, t, nunits, part, st); break;
    case 2: launch_decode_gt<DT, D, 2>(s, t, nunits, part, st); break;
    case 4: launch_decode_gt<DT, D, 4>(s, t, nunits, part, st); break;
    default: launch_decode_gt<DT, D, 8>(s, t, nunits, part, st); break;
  }
}

template <int D>
static void launch_decode_mfma(const DShape &s, const DecodeTable &t, int nunits, float *part, hipStream_t st) {
  const dim3 grid((unsigned)(nunits * s.gchunks * s.nsplit)), block(D * 2);
  hipLaunchKernelGGL((decode_mfma_kernel<D>), grid, block, 0, st, s, t, part);
  if (s.nsplit > 1)
    hipLaunchKernelGGL((decode_merge_kernel<MIXKV_BF16, D>), dim3((unsigned)(nunits * s.gchunks), (unsigned)((s.gt * D + 255) / 256)), dim3(256),
                       0, st, s, t, part);
}

constexpr int kDecMfmaHeads = 32;    // query heads of one group a matrix-core workgroup serves: the columns of a tile
constexpr int kDecTargetWgs = 512;   // two resident workgroups on each of 256 compute units

// Query heads served per workgroup (hpw), their stride in the partials (gt), chunks of query heads
// per group and row splits per head for a shape.  Host only; depends on nothing but the arguments.
static void decode_config(const Shape &sh, int dtype, int n_layers, int tail_len, int *hpw, int *gt, int *gchunks,
                          int *nsplit) {
  const int rows = sh.B + tail_len;                     // per head, on average in the packed layouts
  if (dtype == MIXKV_BF16) {
    // Matrix-core path.  A workgroup's fixed cost (dependent loads of counts, queries and the first
    // tiles) is a few microseconds, so rows are split only as far as it takes to put two workgroups
    // on every compute unit, and never below 256 rows a piece (short caches: no merge launch).
    *hpw = kDecMfmaHeads;
    *gt = sh.G < kDecMfmaHeads ? sh.G : kDecMfmaHeads;
    *gchunks = (sh.G + kDecMfmaHeads - 1) / kDecMfmaHeads;
    const int64_t wgs = (int64_t)n_layers * sh.units_per_layer * *gchunks;
    int ns = (int)(kDecTargetWgs / (wgs < 1 ? 1 : wgs));
    const int by_rows = rows / 256;
    if (ns > by_rows) ns = by_rows;
    *nsplit = ns < 1 ? 1 : (ns > kDecMaxSplit ? kDecMaxSplit : ns);
    return;
  }
  *hpw = kDecHeads;
  *gt = 1;
  while (*gt < sh.G && *gt < kDecHeads) *gt <<= 1;
  *gchunks = (sh.G + kDecHeads - 1) / kDecHeads;
  int ns = (rows + 383) / 384;
  *nsplit = ns < 1 ? 1 : (ns > kDecMaxSplit ? kDecMaxSplit : ns);
}
static size_t decode_part_bytes(const Shape &sh, int n_layers, int gt, int gchunks, int nsplit) {
  if (nsplit == 1) return 0;
  return (size_t)n_layers * sh.units_per_layer * gchunks * nsplit * gt * (sh.D + 2) * sizeof(float);
}

}  // namespace mixkv

extern "C" mixkv_status mixkv_decode_workspace_size(const mixkv_params *params, int32_t n_layers, int32_t tail_len,
                                                    size_t *bytes) {
  using namespace mixkv;
  Shape sh;
  mixkv_status st = make_shape(params, &sh);
  if (st != MIXKV_OK) return st;
  if (!bytes || n_layers < 1 || n_layers > MIXKV_MAX_LAYERS || tail_len < 0) return MIXKV_ERR_INVALID_ARG;
  int hpw, gt, gchunks, nsplit;
  decode_config(sh, params->dtype, n_layers, tail_len, &hpw, &gt, &gchunks, &nsplit);
  *bytes = (decode_part_bytes(sh, n_layers, gt, gchunks, nsplit) + 255) / 256 * 256;
  return MIXKV_OK;
}

extern "C" mixkv_status mixkv_decode_attention(const mixkv_params *params, const mixkv_decode_layer *layers,
                                               int32_t n_layers, int32_t tail_len, int32_t tail_capacity,
                                               void *workspace, size_t workspace_bytes, void *hip_stream) {
  using namespace mixkv;
  Shape sh;
  mixkv_status st = make_shape(params, &sh);
  if (st != MIXKV_OK) return st;
  if (!layers || n_layers < 1 || n_layers > MIXKV_MAX_LAYERS) return MIXKV_ERR_INVALID_ARG;
  if (tail_len < 0 || tail_capacity < tail_len) return MIXKV_ERR_INVALID_ARG;
  int hpw, gt, gchunks, nsplit;
  decode_config(sh, params->dtype, n_layers, tail_len, &hpw, &gt, &gchunks, &nsplit);
  const size_t need = decode_part_bytes(sh, n_layers, gt, gchunks, nsplit);
  if (need > 0) {
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return MIXKV_ERR_INVALID_ARG;
    if (workspace_bytes < need) return MIXKV_ERR_WORKSPACE_TOO_SMALL;
  }
  const bool packed = params->budget_mode != MIXKV_BUDGET_FIXED;
  auto bad16 = [](const void *p) { return !p || (reinterpret_cast<uintptr_t>(p) & 15u); };
  for (int l = 0; l < n_layers; ++l) {
    const mixkv_decode_layer &d = layers[l];
    if (bad16(d.K_cache) || bad16(d.V_cache) || bad16(d.Q) || bad16(d.out) || !d.counts) return MIXKV_ERR_INVALID_ARG;
    if (packed && !d.offsets) return MIXKV_ERR_INVALID_ARG;
    if (tail_len > 0 && (bad16(d.K_tail) || bad16(d.V_tail))) return MIXKV_ERR_INVALID_ARG;
  }
  DShape s;
  s.batch = sh.batch; s.hq = sh.hq; s.hkv = sh.hkv; s.G = sh.G; s.B = sh.B;
  s.tail_len = tail_len; s.tail_cap = tail_capacity; s.packed = packed; s.units_per_layer = sh.units_per_layer;
  s.gchunks = gchunks; s.nsplit = nsplit; s.hpw = hpw; s.gt = gt;
  s.scale_log2e = sh.scale_log2e;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  for (int l0 = 0; l0 < n_layers; l0 += kLayersPerLaunch) {
    const int nl = (n_layers - l0 < kLayersPerLaunch) ? n_layers - l0 : kLayersPerLaunch;
    DecodeTable t;
    for (int l = 0; l < kLayersPerLaunch; ++l) t.l[l] = DecodeLayer{};
    for (int l = 0; l < nl; ++l) {
      const mixkv_decode_layer &d = layers[l0 + l];
      t.l[l] = DecodeLayer{d.K_cache, d.V_cache, d.counts, d.offsets, d.K_tail, d.V_tail, d.Q, d.out};
    }
    const int nunits = nl * sh.units_per_layer;
    // this launch group's partials
    float *part = need > 0 ? reinterpret_cast<float *>(workspace) +
                                 (size_t)l0 * sh.units_per_layer * gchunks * nsplit * gt * (sh.D + 2)
                           : nullptr;
    if (params->dtype == MIXKV_BF16) {
      if (sh.D == 128) launch_decode_mfma<128>(s, t, nunits, part, stream);
      else launch_decode_mfma<64>(s, t, nunits, part, stream);
    } else {
      if (sh.D == 128) launch_decode_g<MIXKV_F32, 128>(s, t, nunits, gt, part, stream);
      else launch_decode_g<MIXKV_F32, 64>(s, t, nunits, gt, part, stream);
    }
    if (hipGetLastError() != hipSuccess) return MIXKV_ERR_HIP;
  }
  return MIXKV_OK;
}

// ------------------------------------------------------------------------------------------------
// mixkv_append: the new token's key and value rows go to row `position` of every head's tail
// (Sec. 3.1: decoding continues on the compressed cache).  16 bytes per thread; thread p of the
// launch copies piece p % PPR of (layer, batch item, head) p / PPR, once for K and once for V.
// ------------------------------------------------------------------------------------------------
namespace mixkv {
struct AppendLayer { const char *K_new, *V_new; char *K_tail, *V_tail; };
struct AppendTable { AppendLayer l[kLayersPerLaunch]; };

__global__ __launch_bounds__(256) void append_kernel(AppendTable tab, int units_per_layer, int nunits, int ppr,
                                                      int position, int tail_cap) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= nunits * ppr) return;
  const int ul = p / ppr, piece = p - ul * ppr;
  const int layer = ul / units_per_layer, bh = ul - layer * units_per_layer;
  const AppendLayer L = tab.l[layer];
  const int64_t src = ((int64_t)bh * ppr + piece) * 16;
  const int64_t dst = (((int64_t)bh * tail_cap + position) * ppr + piece) * 16;
  const uint4 k = *reinterpret_cast<const uint4 *>(L.K_new + src);
  const uint4 v = *reinterpret_cast<const uint4 *>(L.V_new + src);
  *reinterpret_cast<uint4 *>(L.K_tail + dst) = k;
  *reinterpret_cast<uint4 *>(L.V_tail + dst) = v;
}
}  // namespace mixkv

extern "C" mixkv_status mixkv_append(const mixkv_params *params, const mixkv_append_layer *layers, int32_t n_layers,
                                     int32_t position, int32_t tail_capacity, void *hip_stream) {
  using namespace mixkv;
  Shape sh;
  mixkv_status st = make_shape(params, &sh);
  if (st != MIXKV_OK) return st;
  if (!layers || n_layers < 1 || n_layers > MIXKV_MAX_LAYERS) return MIXKV_ERR_INVALID_ARG;
  if (position < 0 || position >= tail_capacity) return MIXKV_ERR_INVALID_ARG;
  const int eb = params->dtype == MIXKV_BF16 ? 2 : 4, ppr = sh.D * eb / 16;
  const size_t new_bytes = (size_t)sh.units_per_layer * sh.D * eb, tail_bytes = new_bytes * (size_t)tail_capacity;
  auto bad16 = [](const void *p) { return !p || (reinterpret_cast<uintptr_t>(p) & 15u); };
  auto overlap = [](const void *a, size_t na, const void *b, size_t nb) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
  };
  for (int l = 0; l < n_layers; ++l) {
    const mixkv_append_layer &a = layers[l];
    if (bad16(a.K_new) || bad16(a.V_new) || bad16(a.K_tail) || bad16(a.V_tail)) return MIXKV_ERR_INVALID_ARG;
    if (overlap(a.K_tail, tail_bytes, a.K_new, new_bytes) || overlap(a.K_tail, tail_bytes, a.V_new, new_bytes) ||
        overlap(a.V_tail, tail_bytes, a.K_new, new_bytes) || overlap(a.V_tail, tail_bytes, a.V_new, new_bytes) ||
        overlap(a.K_tail, tail_bytes, a.V_tail, tail_bytes))
      return MIXKV_ERR_INVALID_ARG;
  }
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  for (int l0 = 0; l0 < n_layers; l0 += kLayersPerLaunch) {
    const int nl = (n_layers - l0 < kLayersPerLaunch) ? n_layers - l0 : kLayersPerLaunch;
    AppendTable t;
    for (int l = 0; l < kLayersPerLaunch; ++l) t.l[l] = AppendLayer{nullptr, nullptr, nullptr, nullptr};
    for (int l = 0; l < nl; ++l) {
      const mixkv_append_layer &a = layers[l0 + l];
      t.l[l] = AppendLayer{static_cast<const char *>(a.K_new), static_cast<const char *>(a.V_new),
                           static_cast<char *>(a.K_tail), static_cast<char *>(a.V_tail)};
    }
    const int nunits = nl * sh.units_per_layer, threads = nunits * ppr;
    hipLaunchKernelGGL(append_kernel, dim3((threads + 255) / 256), dim3(256), 0, stream, t, sh.units_per_layer, nunits, ppr,
                       position, tail_capacity);
    if (hipGetLastError() != hipSuccess) return MIXKV_ERR_HIP;
  }
  return MIXKV_OK;
}
