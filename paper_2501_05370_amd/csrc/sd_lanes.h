// Cross-lane exchanges of a 64-wide wavefront that stay in the vector ALU (gfx950).
//
// lane_xor<MASK>(v) returns v of lane (lane ^ MASK).  The generic shuffle goes through the LDS crossbar
// (an address computation, a queue slot and its round trip per 32-bit word); a butterfly reduction is a chain
// of such exchanges, each waiting for the one before, so in kernels that run two wavefronts per SIMD the
// round trips are not hidden.  Here the masks inside a row of 16 lanes use DPP controls and the two across
// rows use the row-swap instructions:
//   1, 2   quad_perm
//   4      row_shl:4 into lane groups 0 and 2 of each row, row_shr:4 into groups 1 and 3 (bank masks)
//   8      row_ror:8
//   16     v_permlane16_swap: odd rows of the first operand trade places with even rows of the second
//   32     v_permlane32_swap: upper half of the first operand trades places with the lower half of the second
// Both partners of an exchange read each other's value, so a butterfly sum built from these is bit-identical
// on all lanes (floating-point addition commutes), which the accept tests rely on.
#pragma once
#include <hip/hip_runtime.h>

namespace sdlane {

typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

template <int MASK>
__device__ __forceinline__ int lane_xor(int v) {
  static_assert(MASK == 1 || MASK == 2 || MASK == 4 || MASK == 8 || MASK == 16 || MASK == 32, "one bit");
  if constexpr (MASK == 1) {
    return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);          // quad_perm:[1,0,3,2]
  } else if constexpr (MASK == 2) {
    return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);          // quad_perm:[2,3,0,1]
  } else if constexpr (MASK == 4) {
    const int up = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xF, 0x5, false);  // row_shl:4 -> lanes 0-3, 8-11
    return __builtin_amdgcn_update_dpp(up, v, 0x114, 0xF, 0xA, false);         // row_shr:4 -> lanes 4-7, 12-15
  } else if constexpr (MASK == 8) {
    return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, false);          // row_ror:8
  } else if constexpr (MASK == 16) {
    const uint2v r = __builtin_amdgcn_permlane16_swap(static_cast<unsigned>(v), static_cast<unsigned>(v), false, false);
    return static_cast<int>((__lane_id() & 16) ? r[0] : r[1]);
  } else {
    const uint2v r = __builtin_amdgcn_permlane32_swap(static_cast<unsigned>(v), static_cast<unsigned>(v), false, false);
    return static_cast<int>((__lane_id() & 32) ? r[0] : r[1]);
  }
}

template <int MASK>
__device__ __forceinline__ double lane_xor(double v) {
  const long long bits = __double_as_longlong(v);
  const int lo = lane_xor<MASK>(static_cast<int>(bits));
  const int hi = lane_xor<MASK>(static_cast<int>(bits >> 32));
  return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned int>(lo));
}

// v + (v of lane ^ MASK) for the two row-swap masks: after the swap the two results hold the two addends in
// the same order on both partners, so no select is needed and the sum has the same bits on both.
template <int MASK>
__device__ __forceinline__ double pair_sum_rows(double v) {
  static_assert(MASK == 16 || MASK == 32, "row-swap masks");
  const long long bits = __double_as_longlong(v);
  const unsigned lo = static_cast<unsigned>(bits), hi = static_cast<unsigned>(bits >> 32);
  uint2v rl, rh;
  if constexpr (MASK == 16) {
    rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
  } else {
    rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
  }
  const double a = __longlong_as_double((static_cast<long long>(rh[0]) << 32) | rl[0]);
  const double b = __longlong_as_double((static_cast<long long>(rh[1]) << 32) | rl[1]);
  return a + b;
}

// Halving step of a transposed reduction at distance MASK: a lane whose bit MASK is clear keeps `lower`, a
// lane whose bit is set keeps `upper`, and each adds its partner's copy of the value it keeps.  For the two
// row-swap masks one swap per 32-bit half delivers exactly that with no select; for 4 the two shifted moves
// are written under bank masks so the operand needs no select either.
template <int MASK>
__device__ __forceinline__ double halving_add(double lower, double upper) {
  const long long lb = __double_as_longlong(lower), ub = __double_as_longlong(upper);
  const unsigned l0 = static_cast<unsigned>(lb), l1 = static_cast<unsigned>(lb >> 32);
  const unsigned u0 = static_cast<unsigned>(ub), u1 = static_cast<unsigned>(ub >> 32);
  if constexpr (MASK == 16 || MASK == 32) {
    uint2v r0, r1;
    if constexpr (MASK == 16) {
      r0 = __builtin_amdgcn_permlane16_swap(l0, u0, false, false);
      r1 = __builtin_amdgcn_permlane16_swap(l1, u1, false, false);
    } else {
      r0 = __builtin_amdgcn_permlane32_swap(l0, u0, false, false);
      r1 = __builtin_amdgcn_permlane32_swap(l1, u1, false, false);
    }
    const double a = __longlong_as_double((static_cast<long long>(r1[0]) << 32) | r0[0]);
    const double b = __longlong_as_double((static_cast<long long>(r1[1]) << 32) | r0[1]);
    return a + b;
  } else {
    const bool up = __lane_id() & MASK;
    const double keep = up ? upper : lower;
    if constexpr (MASK == 4) {
      int g0 = __builtin_amdgcn_update_dpp(0, static_cast<int>(l0), 0x104, 0xF, 0x5, false);
      g0 = __builtin_amdgcn_update_dpp(g0, static_cast<int>(u0), 0x114, 0xF, 0xA, false);
      int g1 = __builtin_amdgcn_update_dpp(0, static_cast<int>(l1), 0x104, 0xF, 0x5, false);
      g1 = __builtin_amdgcn_update_dpp(g1, static_cast<int>(u1), 0x114, 0xF, 0xA, false);
      return keep + __longlong_as_double((static_cast<long long>(g1) << 32) | static_cast<unsigned>(g0));
    } else {
      const double send = up ? lower : upper;
      return keep + lane_xor<MASK>(send);
    }
  }
}

// Sum over the wavefront, the same bits on every lane.
__device__ __forceinline__ double wave_sum(double v) {
  v += lane_xor<1>(v);
  v += lane_xor<2>(v);
  v += lane_xor<4>(v);
  v += lane_xor<8>(v);
  v = pair_sum_rows<16>(v);
  return pair_sum_rows<32>(v);
}

}  // namespace sdlane
