// Wave64 reductions built on DPP lane permutes (no LDS round trips).
//
// quad_perm and row_ror permute lanes inside a row of 16 and never read an
// inactive or out-of-range lane, so no identity element is needed.  After the
// four steps every lane holds its row's result; the four row results are then
// combined from lanes 0, 16, 32 and 48 in a fixed order.  All 64 lanes must be
// active at the call.
#pragma once
#include <hip/hip_runtime.h>

namespace smoe {

constexpr int kDppQuadSwap1 = 0xB1;   // quad_perm:[1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;   // quad_perm:[2,3,0,1]
constexpr int kDppRowRor4 = 0x124;    // row_ror:4
constexpr int kDppRowRor8 = 0x128;    // row_ror:8

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ float lane_f(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Sum over the 64 lanes; the result is uniform.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<kDppQuadSwap1>(v);
  v += dpp_f<kDppQuadSwap2>(v);
  v += dpp_f<kDppRowRor4>(v);
  v += dpp_f<kDppRowRor8>(v);
  return (lane_f(v, 0) + lane_f(v, 16)) + (lane_f(v, 32) + lane_f(v, 48));
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<kDppQuadSwap1>(v));
  v = fmaxf(v, dpp_f<kDppQuadSwap2>(v));
  v = fmaxf(v, dpp_f<kDppRowRor4>(v));
  v = fmaxf(v, dpp_f<kDppRowRor8>(v));
  return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}

// (value, index) pair ordering: larger value first, lower index on equal values.
__device__ __forceinline__ void take_better(float& val, int& idx, float ov, int oi) {
  if (ov > val || (ov == val && oi < idx)) { val = ov; idx = oi; }
}

// Lane holding the largest value among lanes with `valid` set; lower lane wins
// ties; -1 when no lane is valid.  Uniform result.
__device__ __forceinline__ int wave_argmax(float v, bool valid, int lane) {
  float val = valid ? v : -INFINITY;
  int idx = valid ? lane : 64;
  take_better(val, idx, dpp_f<kDppQuadSwap1>(val), dpp_i<kDppQuadSwap1>(idx));
  take_better(val, idx, dpp_f<kDppQuadSwap2>(val), dpp_i<kDppQuadSwap2>(idx));
  take_better(val, idx, dpp_f<kDppRowRor4>(val), dpp_i<kDppRowRor4>(idx));
  take_better(val, idx, dpp_f<kDppRowRor8>(val), dpp_i<kDppRowRor8>(idx));
  float bv = lane_f(val, 0);
  int bi = __builtin_amdgcn_readlane(idx, 0);
  take_better(bv, bi, lane_f(val, 16), __builtin_amdgcn_readlane(idx, 16));
  take_better(bv, bi, lane_f(val, 32), __builtin_amdgcn_readlane(idx, 32));
  take_better(bv, bi, lane_f(val, 48), __builtin_amdgcn_readlane(idx, 48));
  return bi == 64 ? -1 : bi;
}

}  // namespace smoe
