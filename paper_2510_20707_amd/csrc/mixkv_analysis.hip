// Redundancy analysis of cached keys or values: the mean off-diagonal cosine similarity of one
// head's rows and the block-mean heat-map of its cosine matrix (paper: Sec. 1, the figures on
// key / value similarity inside a head and across heads; Sec. 3.3, Eq. 3-4 for the matrix and
// its off-diagonal mean).
//
// The N x N matrix is never formed.  With Xh the L2-normalised rows and S_a the sum of the rows
// of block a, the mean of the matrix over block a x block b is S_a . S_b / (n_a n_b), and the sum
// of all entries is |sum_a S_a|^2.  So one streaming pass over X produces the block sums
// (blocksum_kernel, bound by HBM); blockgram_kernel forms their Gram matrix in LDS tiles and
// redundancy_kernel folds them into the off-diagonal mean.
#include "mixkv_internal.h"
#include "mixkv_wave.h"

namespace mixkv {

struct RowsIn {
  const void *X;
  int64_t sb, sh, sn;   // strides in elements
};
struct RowsInTable { RowsIn l[kLayersPerLaunch]; };
struct SimOut {
  float *redundancy, *block_map;
};
struct SimOutTable { SimOut l[kLayersPerLaunch]; };

struct AShape {
  int32_t batch, heads, N, D, block, nb, units_per_layer;
};

// 1 / max(|x|, 1e-30) from the sum of squares, 0 for a zero row (same convention as the scoring
// path: tiny sums are scaled by 2^64 before the hardware reciprocal square root).
template <int DT>
__device__ __forceinline__ float inv_norm_a(float ss) {
  const bool tiny = ss < 1e-30f;
  const float x = tiny ? ss * 18446744073709551616.f : ss;
  float y = __builtin_amdgcn_rsqf(x);
  y = y * fmaf(-0.5f * x, y * y, 1.5f);
  y = tiny ? y * 4294967296.f : y;
  return ss > 0.f ? fminf(y, 1e30f) : 0.f;
}

// One wave per block of rows.  A row is PPR consecutive lanes of 16 bytes; a wave load covers
// 64 / PPR rows.  Each lane keeps the running sum of its piece of the normalised rows; at the end
// the lanes holding the same piece are folded and the first PPR lanes store S_a.  diag[a] gets
// sum_i |Xh_i|^2 (the number of non-zero rows up to rounding), the trace part of the matrix.
template <int DT, int D>
__global__ __launch_bounds__(256) void blocksum_kernel(AShape a, RowsInTable in, float *S, float *diag, int nunits) {
  constexpr int EB = DT == MIXKV_BF16 ? 2 : 4, E = 16 / EB, PPR = D * EB / 16, RPL = 64 / PPR, U = 8;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wgs_per_unit = (a.nb + 3) / 4;
  const int ul = blockIdx.x / wgs_per_unit, blk = (blockIdx.x - ul * wgs_per_unit) * 4 + wave;
  if (ul >= nunits || blk >= a.nb) return;             // whole waves leave; no barrier below
  const int layer = ul / a.units_per_layer, bh = ul - layer * a.units_per_layer;
  const int b = bh / a.heads, h = bh - b * a.heads;
  const RowsIn L = in.l[layer];
  const char *base = reinterpret_cast<const char *>(L.X) + ((int64_t)b * L.sb + (int64_t)h * L.sh) * EB;
  const int r0 = blk * a.block, rend = min(a.N, r0 + a.block);
  const int lr = lane / PPR, piece = lane - lr * PPR;
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  float dsum = 0.f;
  for (int r = r0; r < rend; r += RPL * U) {
    uint4 q[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = r + u * RPL + lr;
      q[u] = make_uint4(0u, 0u, 0u, 0u);
      if (row < rend) q[u] = *reinterpret_cast<const uint4 *>(base + (int64_t)row * L.sn * EB + piece * 16);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[E];
      if constexpr (DT == MIXKV_BF16) {
        const uint32_t w[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          x[2 * j] = __uint_as_float(w[j] << 16);
          x[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
        }
      } else {
        x[0] = __uint_as_float(q[u].x); x[1] = __uint_as_float(q[u].y);
        x[2] = __uint_as_float(q[u].z); x[3] = __uint_as_float(q[u].w);
      }
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) ss = fmaf(x[e], x[e], ss);
      ss = seg_sum<PPR>(ss);
      const float inv = inv_norm_a<DT>(ss);              // rows past the block are all zero: inv = 0
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] = fmaf(inv, x[e], acc[e]);
      if (piece == 0) dsum = fmaf(inv * inv, ss, dsum);
    }
  }
#pragma unroll
  for (int o = PPR; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += __shfl_xor(acc[e], o);
    dsum += __shfl_xor(dsum, o);
  }
  if (lane < PPR) {
    float *dst = S + ((int64_t)ul * a.nb + blk) * D + piece * E;
#pragma unroll
    for (int e = 0; e < E; e += 4) *reinterpret_cast<float4 *>(dst + e) = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
  }
  if (lane == 0) diag[(int64_t)ul * a.nb + blk] = dsum;
}

// Heat-map: one workgroup per (unit, 64 x 64 tile of the map).  The two sets of 64 block sums go
// through LDS in slices of 64 dimensions (rows padded by four floats, so the 16 columns a wave
// reads at once fall into different banks); every thread owns a 4 x 4 patch of the tile:
// rows ty + 16 i, columns tx + 16 j.  M[a][b] = S_a . S_b / (n_a n_b).
constexpr int kMapTile = 64, kMapSlice = 64;
template <int D>
__global__ __launch_bounds__(256) void blockgram_kernel(AShape a, SimOutTable out, const float *S) {
  __shared__ float sa[kMapTile][kMapSlice + 4], sb[kMapTile][kMapSlice + 4];
  const int tiles = (a.nb + kMapTile - 1) / kMapTile;
  const int ul = blockIdx.x / (tiles * tiles), t = blockIdx.x - ul * tiles * tiles;
  const int a0 = (t / tiles) * kMapTile, b0 = (t % tiles) * kMapTile;
  const int layer = ul / a.units_per_layer, bh = ul - layer * a.units_per_layer;
  float *map = out.l[layer].block_map;
  if (!map) return;                                     // uniform over the workgroup
  const float *Su = S + (int64_t)ul * a.nb * D;
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int d0 = 0; d0 < D; d0 += kMapSlice) {
    if (d0 > 0) __syncthreads();
    // 64 rows x 16 float4 per operand: four float4 per thread and operand, coalesced along d
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int e = tid + 256 * k, r = e >> 4, c = e & 15;
      // rows past the last block read the last one (always in bounds) and are zeroed afterwards: a
      // conditional load of either the row or a zero constant is compiled into a load from either the
      // row or a copy of the constant in scratch memory
      const int ra = min(a0 + r, a.nb - 1), rb = min(b0 + r, a.nb - 1);
      float4 va = *reinterpret_cast<const float4 *>(Su + (int64_t)ra * D + d0 + 4 * c);
      float4 vb = *reinterpret_cast<const float4 *>(Su + (int64_t)rb * D + d0 + 4 * c);
      if (a0 + r >= a.nb) va = make_float4(0.f, 0.f, 0.f, 0.f);
      if (b0 + r >= a.nb) vb = make_float4(0.f, 0.f, 0.f, 0.f);
      *reinterpret_cast<float4 *>(&sa[r][4 * c]) = va;
      *reinterpret_cast<float4 *>(&sb[r][4 * c]) = vb;
    }
    __syncthreads();
#pragma unroll 4
    for (int d = 0; d < kMapSlice; d += 4) {
      float4 x[4], y[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) x[i] = *reinterpret_cast<const float4 *>(&sa[ty + 16 * i][d]);
#pragma unroll
      for (int j = 0; j < 4; ++j) y[j] = *reinterpret_cast<const float4 *>(&sb[tx + 16 * j][d]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(x[i].x, y[j].x, acc[i][j]); acc[i][j] = fmaf(x[i].y, y[j].y, acc[i][j]);
          acc[i][j] = fmaf(x[i].z, y[j].z, acc[i][j]); acc[i][j] = fmaf(x[i].w, y[j].w, acc[i][j]);
        }
    }
  }
  auto rows_of = [&](int blk) { return min(a.N, (blk + 1) * a.block) - blk * a.block; };
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ba = a0 + ty + 16 * i;
    if (ba >= a.nb) continue;
    const float inv_na = 1.f / (float)rows_of(ba);
    float *row = map + ((int64_t)bh * a.nb + ba) * a.nb;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int bb = b0 + tx + 16 * j;
      if (bb < a.nb) row[bb] = acc[i][j] * inv_na / (float)rows_of(bb);
    }
  }
}

// Off-diagonal mean, one workgroup of 1024 threads per unit: the sum of all entries of the cosine
// matrix is |sum_a S_a|^2 and its trace sum_a diag[a].  Partial sums are taken over interleaved
// blocks and folded in a fixed order, in double.
constexpr int kRedThreads = 1024;
template <int D>
__global__ __launch_bounds__(kRedThreads) void redundancy_kernel(AShape a, SimOutTable out, const float *S, const float *diag) {
  constexpr int PARTS = kRedThreads / D;
  __shared__ double part[kRedThreads];
  const int ul = blockIdx.x, layer = ul / a.units_per_layer, bh = ul - layer * a.units_per_layer;
  float *red = out.l[layer].redundancy;
  if (!red) return;                                     // uniform over the workgroup
  const float *Su = S + (int64_t)ul * a.nb * D;
  const int tid = threadIdx.x, d = tid % D, pt = tid / D;
  double t4[4] = {0.0, 0.0, 0.0, 0.0};                 // four loads in flight; folded in a fixed order
  for (int bb = pt; bb < a.nb; bb += 4 * PARTS)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (bb + q * PARTS < a.nb) t4[q] += (double)Su[(int64_t)(bb + q * PARTS) * D + d];
  part[tid] = (t4[0] + t4[1]) + (t4[2] + t4[3]);
  __syncthreads();
  double sq = 0.0;
  if (tid < D) {
    double v = 0.0;
#pragma unroll
    for (int q = 0; q < PARTS; ++q) v += part[q * D + tid];
    sq = v * v;
  }
  double tr = 0.0;
  for (int bb = tid; bb < a.nb; bb += kRedThreads) tr += (double)diag[(int64_t)ul * a.nb + bb];
  __syncthreads();
  part[tid] = sq - tr;                                   // every thread's share of (all entries - trace)
  __syncthreads();
  // fold in two levels (32 x 32), each level in index order, so the LDS reads of a level overlap
  double g = 0.0;
  if (tid < 32) {
    double v[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = part[tid * 32 + i];
#pragma unroll
    for (int i = 0; i < 32; ++i) g += v[i];
  }
  __syncthreads();
  if (tid < 32) part[tid] = g;
  __syncthreads();
  if (tid == 0) {
    double v[32], off = 0.0;
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = part[i];
#pragma unroll
    for (int i = 0; i < 32; ++i) off += v[i];
    const double n = (double)a.N;
    red[bh] = (float)(off / (n * (n - 1.0)));
  }
}

static size_t align256(size_t x) { return (x + 255) / 256 * 256; }

static mixkv_status analysis_shape(const mixkv_params *p, int32_t block, AShape *a) {
  Shape s;
  mixkv_status st = make_shape(p, &s);
  if (st != MIXKV_OK) return st;
  if (block < 1 || block > s.N) return MIXKV_ERR_INVALID_ARG;
  a->batch = s.batch; a->heads = s.hkv; a->N = s.N; a->D = s.D; a->block = block;
  a->nb = (s.N + block - 1) / block;
  a->units_per_layer = s.units_per_layer;
  const int64_t tiles = (a->nb + kMapTile - 1) / kMapTile, per_launch = (int64_t)kLayersPerLaunch * a->units_per_layer;
  if (a->nb * per_launch > INT32_MAX || tiles * tiles * per_launch > INT32_MAX) return MIXKV_ERR_UNSUPPORTED;   // grid sizes
  return MIXKV_OK;
}

}  // namespace mixkv

extern "C" {

mixkv_status mixkv_similarity_workspace_size(const mixkv_params *params, int32_t n_layers, int32_t block, size_t *bytes) {
  mixkv::AShape a;
  mixkv_status st = mixkv::analysis_shape(params, block, &a);
  if (st != MIXKV_OK) return st;
  if (!bytes || n_layers < 1 || n_layers > MIXKV_MAX_LAYERS) return MIXKV_ERR_INVALID_ARG;
  const size_t units = (size_t)n_layers * a.units_per_layer;
  *bytes = mixkv::align256(units * a.nb * a.D * 4) + mixkv::align256(units * a.nb * 4);
  return MIXKV_OK;
}

mixkv_status mixkv_similarity(const mixkv_params *params, const mixkv_rows_in *in, const mixkv_similarity_out *out,
                              int32_t n_layers, int32_t block, void *workspace, size_t workspace_bytes,
                              void *hip_stream) {
  using namespace mixkv;
  AShape a;
  mixkv_status st = analysis_shape(params, block, &a);
  if (st != MIXKV_OK) return st;
  if (!in || !out || n_layers < 1 || n_layers > MIXKV_MAX_LAYERS) return MIXKV_ERR_INVALID_ARG;
  size_t need = 0;
  st = mixkv_similarity_workspace_size(params, n_layers, block, &need);
  if (st != MIXKV_OK) return st;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return MIXKV_ERR_INVALID_ARG;
  if (workspace_bytes < need) return MIXKV_ERR_WORKSPACE_TOO_SMALL;
  const int eb = params->dtype == MIXKV_BF16 ? 2 : 4;
  for (int l = 0; l < n_layers; ++l) {
    const mixkv_rows_in &li = in[l];
    if (!li.X || (reinterpret_cast<uintptr_t>(li.X) & 15u)) return MIXKV_ERR_INVALID_ARG;
    if (li.stride_n < a.D || li.stride_h < 0 || li.stride_b < 0) return MIXKV_ERR_INVALID_ARG;
    if ((li.stride_n * eb) % 16 || (li.stride_h * eb) % 16 || (li.stride_b * eb) % 16) return MIXKV_ERR_INVALID_ARG;
    if (!out[l].redundancy && !out[l].block_map) return MIXKV_ERR_INVALID_ARG;
  }
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t units = (size_t)n_layers * a.units_per_layer;
  float *S = reinterpret_cast<float *>(workspace);
  float *diag = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + align256(units * a.nb * a.D * 4));
  for (int l0 = 0; l0 < n_layers; l0 += kLayersPerLaunch) {
    const int nl = (n_layers - l0 < kLayersPerLaunch) ? n_layers - l0 : kLayersPerLaunch;
    RowsInTable ti;
    SimOutTable to;
    for (int l = 0; l < kLayersPerLaunch; ++l) {
      ti.l[l] = RowsIn{nullptr, 0, 0, 0};
      to.l[l] = SimOut{nullptr, nullptr};
    }
    for (int l = 0; l < nl; ++l) {
      ti.l[l] = RowsIn{in[l0 + l].X, in[l0 + l].stride_b, in[l0 + l].stride_h, in[l0 + l].stride_n};
      to.l[l] = SimOut{out[l0 + l].redundancy, out[l0 + l].block_map};
    }
    const int nunits = nl * a.units_per_layer;
    const size_t unit0 = (size_t)l0 * a.units_per_layer;
    float *Sg = S + unit0 * a.nb * a.D, *dg = diag + unit0 * a.nb;
    const int tiles = (a.nb + kMapTile - 1) / kMapTile;
    const dim3 grid_a((unsigned)(nunits * ((a.nb + 3) / 4))), grid_b((unsigned)(nunits * tiles * tiles)), grid_r(nunits);
    const bool bf = params->dtype == MIXKV_BF16;
    if (a.D == 128) {
      if (bf) hipLaunchKernelGGL((blocksum_kernel<MIXKV_BF16, 128>), grid_a, dim3(256), 0, stream, a, ti, Sg, dg, nunits);
      else hipLaunchKernelGGL((blocksum_kernel<MIXKV_F32, 128>), grid_a, dim3(256), 0, stream, a, ti, Sg, dg, nunits);
      hipLaunchKernelGGL(blockgram_kernel<128>, grid_b, dim3(256), 0, stream, a, to, Sg);
      hipLaunchKernelGGL(redundancy_kernel<128>, grid_r, dim3(kRedThreads), 0, stream, a, to, Sg, dg);
    } else {
      if (bf) hipLaunchKernelGGL((blocksum_kernel<MIXKV_BF16, 64>), grid_a, dim3(256), 0, stream, a, ti, Sg, dg, nunits);
      else hipLaunchKernelGGL((blocksum_kernel<MIXKV_F32, 64>), grid_a, dim3(256), 0, stream, a, ti, Sg, dg, nunits);
      hipLaunchKernelGGL(blockgram_kernel<64>, grid_b, dim3(256), 0, stream, a, to, Sg);
      hipLaunchKernelGGL(redundancy_kernel<64>, grid_r, dim3(kRedThreads), 0, stream, a, to, Sg, dg);
    }
    if (hipGetLastError() != hipSuccess) return MIXKV_ERR_HIP;
  }
  return MIXKV_OK;
}

}  // extern "C"
