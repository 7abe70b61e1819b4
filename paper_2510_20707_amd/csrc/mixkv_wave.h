// Wave-level primitives on data-parallel-primitive (DPP) row shifts: cross-lane steps that run in
// the vector ALU instead of going through the LDS crossbar.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mixkv {

struct WSum { template <class T> __device__ static T f(T a, T b) { return a + b; } };
struct WMin { template <class T> __device__ static T f(T a, T b) { return a < b ? a : b; } };
struct WMax { template <class T> __device__ static T f(T a, T b) { return a > b ? a : b; } };

template <int CTRL>
__device__ __forceinline__ int dpp_or_old(int old, int src) {
  // lanes whose source lies outside their row of 16 keep `old`
  return __builtin_amdgcn_update_dpp(old, src, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ int as_bits(int x) { return x; }
__device__ __forceinline__ int as_bits(uint32_t x) { return (int)x; }
__device__ __forceinline__ int as_bits(float x) { return __float_as_int(x); }
__device__ __forceinline__ void from_bits(int b, int &x) { x = b; }
__device__ __forceinline__ void from_bits(int b, uint32_t &x) { x = (uint32_t)b; }
__device__ __forceinline__ void from_bits(int b, float &x) { x = __int_as_float(b); }

// Inclusive scan inside each row of 16 lanes (lane order); `id` is the identity of Op.
template <class Op, class T>
__device__ __forceinline__ T row_scan_incl(T x, T id) {
  T t;
  from_bits(dpp_or_old<0x111>(as_bits(id), as_bits(x)), t); x = Op::f(x, t);   // row_shr:1
  from_bits(dpp_or_old<0x112>(as_bits(id), as_bits(x)), t); x = Op::f(x, t);   // row_shr:2
  from_bits(dpp_or_old<0x114>(as_bits(id), as_bits(x)), t); x = Op::f(x, t);   // row_shr:4
  from_bits(dpp_or_old<0x118>(as_bits(id), as_bits(x)), t); x = Op::f(x, t);   // row_shr:8
  return x;
}

template <class T> __device__ __forceinline__ T read_lane(T x, int lane) {
  T r;
  from_bits(__builtin_amdgcn_readlane(as_bits(x), lane), r);
  return r;
}

// Reduction over the 64 lanes of a wave, rows folded in lane order; the result is wave-uniform.
template <class Op, class T>
__device__ __forceinline__ T wave_reduce(T x, T id) {
  x = row_scan_incl<Op>(x, id);
  const T r0 = read_lane(x, 15), r1 = read_lane(x, 31), r2 = read_lane(x, 47), r3 = read_lane(x, 63);
  return Op::f(Op::f(r0, r1), Op::f(r2, r3));
}

// Reduction over each row of 16 lanes; the row's total is valid in its lane 15.
template <class Op, class T>
__device__ __forceinline__ T row_reduce_to_lane15(T x, T id) { return row_scan_incl<Op>(x, id); }

// Sum over aligned segments of SEG consecutive lanes (SEG = 8, 16 or 32); every lane of a
// segment receives its total.  Butterfly of DPP lane permutations, so the order is fixed.
template <int SEG>
__device__ __forceinline__ float seg_sum(float x) {
  static_assert(SEG == 8 || SEG == 16 || SEG == 32, "segment width");
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, true));   // row_half_mirror
  if (SEG >= 16) x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, true));  // row_mirror
  if (SEG >= 32) x += __shfl_xor(x, 16);
  return x;
}

// Inclusive prefix sum over the 64 lanes of a wave; *total receives the wave sum.
__device__ __forceinline__ int wave_scan_incl_add(int x, int *total) {
  x = row_scan_incl<WSum>(x, 0);
  const int r0 = read_lane(x, 15), r1 = read_lane(x, 31), r2 = read_lane(x, 47), r3 = read_lane(x, 63);
  const int row = (threadIdx.x & 63) >> 4;
  x += row == 0 ? 0 : (row == 1 ? r0 : (row == 2 ? r0 + r1 : r0 + r1 + r2));
  *total = r0 + r1 + r2 + r3;
  return x;
}

}  // namespace mixkv
