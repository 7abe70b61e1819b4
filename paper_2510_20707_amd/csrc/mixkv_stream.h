// Device helpers shared by the kernels that stream the cache through the matrix cores: MFMA
// fragments, the bank-rotated LDS image of a 32-row tile and its direct global->LDS loads, counted
// waits, norms and the merge of running softmax statistics.
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
#pragma once
#include <type_traits>
#include "mixkv_internal.h"
#include "mixkv_wave.h"

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
    // the four floats are taken out of the 16-byte member the loads wrote: reading them through the
    // union's float array instead sends whole fragment arrays through scratch memory
    const uint32_t au[4] = {a.q.x, a.q.y, a.q.z, a.q.w}, bu[4] = {b.q.x, b.q.y, b.q.z, b.q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(au[i]), __uint_as_float(bu[i]), acc, 0, 0, 0);
    return acc;
  }
}

template <int DT>
__device__ __forceinline__ float frag_elem(const Frag &f, int j) {
  if constexpr (DT == MIXKV_BF16) {
    uint32_t u = f.u[j >> 1];
    return __uint_as_float((j & 1) ? (u & 0xffff0000u) : (u << 16));
  } else {
    const uint32_t u[4] = {f.q.x, f.q.y, f.q.z, f.q.w};
    return __uint_as_float(u[j]);
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Sum of squares of the elements of one 16-byte piece (bf16: four two-element dot products).
template <int DT>
__device__ __forceinline__ float piece_sumsq(const Frag &f) {
  float ss = 0.f;
  if constexpr (DT == MIXKV_BF16) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bf16x2 v = __builtin_bit_cast(bf16x2, f.u[j]);
      ss = __builtin_amdgcn_fdot2_f32_bf16(v, v, ss, false);
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float x = frag_elem<DT>(f, j);
      ss = fmaf(x, x, ss);
    }
  }
  return ss;
}

// 1 / max(sqrt(ss), 1e-30) without a branch: the hardware reciprocal square root (one Newton step
// on top for f32 inputs); sums of squares too small for it are scaled by 2^64 first, and a zero
// key gets 0 (its normalised key is the zero vector either way).
template <int DT>
__device__ __forceinline__ float inv_norm(float ss) {
  const bool tiny = ss < 1e-30f;
  const float x = tiny ? ss * 18446744073709551616.f : ss;
  float y = __builtin_amdgcn_rsqf(x);
  if constexpr (DT == MIXKV_F32) y = y * fmaf(-0.5f * x, y * y, 1.5f);
  y = tiny ? y * 4294967296.f : y;
  return ss > 0.f ? fminf(y, 1e30f) : 0.f;
}

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

// Key tiles per chunk.  A chunk is the unit of the work split between workgroups and of the
// column-sum hand-over in attn_kernel; wide f32 tiles get one tile per chunk.
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

// Issue the direct-to-LDS loads of the 32-row tile that starts at row tb (keys or values) into the
// tile image at LDS byte address `img`.  Load j covers slots [64j, 64j+64) of the image; lane i
// fetches the piece that belongs in slot 64j + i.  Waves take loads round-robin and every wave
// issues the same number (with fewer loads than waves some are issued twice), so a wave can count
// its requests in flight.  The address is a wave-uniform 64-bit base plus a 32-bit lane offset.
// In the last tile of a sequence, rows past N-1 re-read row N-1 (their results are masked or
// discarded).
//
// `img` is an integer on purpose: the destination of the load then carries no object identity, and
// the compiler does not make later reads of the ring wait for every load in flight - the waits are
// placed by hand (wait_vm) where the data is needed.
//
// `tile` points at row tb of the tensor (the callers keep it as a running scalar pointer, so the
// common path is that pointer plus loop-invariant scalar and lane offsets and needs no vector
// arithmetic).  fetch_tile_clamped is the last tile of a sequence, kept out of line.
template <int DT, int D, int WAVES>
__device__ __attribute__((noinline)) void fetch_tile_clamped(const char *tile, int64_t row_bytes, int tb, int N, uint32_t img,
                                                             int wave, int lane) {
  constexpr int PPR = D * Tr<DT>::EB / 16, LOADS = 32 * PPR / 64, RPL = 64 / PPR;
  const int lrow = lane / PPR, lq = lane % PPR;
#pragma unroll
  for (int jj = 0; jj < (LOADS + WAVES - 1) / WAVES; ++jj) {
    const int j = (jj * WAVES + wave) % LOADS;
    const int row = j * RPL + lrow;
    const int krow = min(row, N - 1 - tb);                     // rows past the last one repeat it
    const char *src = tile + (int64_t)krow * row_bytes + (lq ^ tile_swz<DT, D>(row)) * 16;
    __builtin_amdgcn_global_load_lds((glb_void_t *)src, (lds_void_t *)(uintptr_t)(img + j * 1024), 16, 0, 0);
  }
}

template <int DT, int D, int WAVES>
__device__ __forceinline__ void fetch_tile(const char *tile, int64_t row_bytes, int tb, int N, uint32_t img, int wave,
                                           int lane) {
  constexpr int PPR = D * Tr<DT>::EB / 16, LOADS = 32 * PPR / 64;      // loads per tile
  constexpr int RPL = 64 / PPR;                                         // rows per load
  static_assert(PPR <= 64 && 64 % PPR == 0, "row pieces must divide a load");
  if (tb + 32 <= N) {
    const int lrow = lane / PPR, lq = lane % PPR;
    const uint32_t rb = (uint32_t)row_bytes;
#pragma unroll
    for (int jj = 0; jj < (LOADS + WAVES - 1) / WAVES; ++jj) {
      const int j = (jj * WAVES + wave) % LOADS;
      const char *base = tile + (int64_t)(j * RPL) * row_bytes;                  // wave-uniform
      const uint32_t off = (uint32_t)lrow * rb + (uint32_t)((lq ^ tile_swz<DT, D>(j * RPL + lrow)) * 16);   // loop-invariant
      __builtin_amdgcn_global_load_lds((glb_void_t *)(base + off), (lds_void_t *)(uintptr_t)(img + j * 1024), 16, 0, 0);
    }
  } else {
    fetch_tile_clamped<DT, D, WAVES>(tile, row_bytes, tb, N, img, wave, lane);
  }
}

// LDS byte address of a __shared__ object, laundered through a register so that nothing derived
// from it is tied to the object (see fetch_tile).
__device__ __forceinline__ uint32_t lds_base_of(const void *p) {
  uint32_t a = (uint32_t)(uintptr_t)(lds_void_t *)p;
  asm volatile("" : "+s"(a));
  return a;
}

// Fragment c of key tile k for lane (row l32, half): piece 2c + half of row l32.
template <int DT, int D>
__device__ __forceinline__ uint4 read_key_frag(const uint4 *kb, int k, int c, int l32, int half) {
  constexpr int PPR = D * Tr<DT>::EB / 16;
  return kb[(k * 32 + l32) * PPR + ((2 * c + half) ^ tile_swz<DT, D>(l32))];
}

// ------------------------------------------------------------------------------------------------
// The tile ring.  Tiles of 32 rows travel global -> LDS through a ring of kRing tile images.  Every
// request is issued kLead tile steps before its data is used, in every wave, for keys and values
// alike: the memory counter of a wave retires in order, so a uniform lead means that waiting for
// the oldest request never waits for a younger one.  One tile step is
//     wait until this wave's share of tile t has landed; barrier; request tile t + kLead (into the
//     image of tile t - 1, which every wave has left behind by passing the barrier); work on t.
// ------------------------------------------------------------------------------------------------
constexpr int kRing = 4, kLead = 3;
static_assert((kRing & (kRing - 1)) == 0 && kLead < kRing, "ring slots are taken modulo a power of two");

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also drain the memory
// counter, i.e. wait for every tile in flight and throw the lead away.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// s_waitcnt vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt and lgkmcnt left open)
template <int NOUT>
__device__ __forceinline__ void wait_vm() {
  static_assert(NOUT >= 0 && NOUT < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((NOUT & 15) | ((NOUT >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Wait for this wave's requests of tile t.  Younger than those are the requests of the kLead - 1
// tiles after it (PER_TILE each, and any store since) as long as the run still had tiles to
// request; near the end of a run everything is awaited.
template <int PER_TILE>
__device__ __forceinline__ void wait_tile(int t, int nt) {
  if (t + kLead <= nt) wait_vm<(kLead - 1) * PER_TILE>(); else wait_vm<0>();
}

}  // namespace mixkv
