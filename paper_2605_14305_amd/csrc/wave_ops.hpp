// Wavefront-wide (64 lanes) reductions and scans built on DPP, the cross-lane datapath of the
// VALU: row_shr inside rows of 16 lanes, then row_bcast15 / row_bcast31 to carry row totals into
// the following rows.  Fixed association order, hence bit-reproducible; no LDS round trips.
#pragma once
#include <hip/hip_runtime.h>

namespace fef {

// v_mov_b32 with DPP control CTRL; lanes whose source lane is outside the row, or whose row is
// masked off by ROW_MASK, keep `old`.
template <int CTRL, int ROW_MASK>
__device__ inline int dpp_mov(int old, int src) {
  return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xf, false);
}

constexpr int kDppRowShr = 0x110;  // + n: shift right by n lanes inside a row of 16
constexpr int kDppBcast15 = 0x142; // lane 15 of each row to every lane of the next row
constexpr int kDppBcast31 = 0x143; // lane 31 to every lane of rows 2 and 3

// Inclusive scan over the 64 lanes with a binary operation given as a functor on int bit
// patterns; `ident` is the bit pattern of the identity.
template <class Op>
__device__ inline int wave_scan_bits(int x, int ident, Op op) {
  x = op(x, dpp_mov<kDppRowShr + 1, 0xf>(ident, x));
  x = op(x, dpp_mov<kDppRowShr + 2, 0xf>(ident, x));
  x = op(x, dpp_mov<kDppRowShr + 4, 0xf>(ident, x));
  x = op(x, dpp_mov<kDppRowShr + 8, 0xf>(ident, x));
  x = op(x, dpp_mov<kDppBcast15, 0xa>(ident, x));
  x = op(x, dpp_mov<kDppBcast31, 0xc>(ident, x));
  return x;
}

__device__ inline float wave_scan_add(float x) {  // inclusive prefix sums in lane order
  return __builtin_bit_cast(float, wave_scan_bits(__builtin_bit_cast(int, x), 0, [](int a, int b) {
    return __builtin_bit_cast(int, __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b));
  }));
}
__device__ inline float wave_sum(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_scan_add(x)), 63));
}
__device__ inline float wave_max(float x) {
  const int r = wave_scan_bits(__builtin_bit_cast(int, x), (int)0xff800000, [](int a, int b) {
    return __builtin_bit_cast(int, fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b)));
  });
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(r, 63));
}
__device__ inline int wave_min_int(int x) {
  return __builtin_amdgcn_readlane(wave_scan_bits(x, 0x7fffffff, [](int a, int b) { return a < b ? a : b; }), 63);
}
__device__ inline int wave_max_int(int x) {
  return __builtin_amdgcn_readlane(wave_scan_bits(x, (int)0x80000000, [](int a, int b) { return a > b ? a : b; }), 63);
}

}  // namespace fef
