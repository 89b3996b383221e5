// Internal helpers shared by the vocabulary-head kernels.
#pragma once
#include <hip/hip_ext.h>
#include <math.h>

#include "fef_device.hpp"

// Launch a head kernel; the dispatch-timestamp events need the extended launch call, every other
// launch uses the plain one (which a capturing stream records like any kernel node).
#define FEF_LAUNCH_HEAD(kernel, grid, block, a, ...)                                              \
  do {                                                                                            \
    if ((a).ev_begin || (a).ev_end)                                                               \
      hipExtLaunchKernelGGL(kernel, grid, block, 0, (a).stream, (a).ev_begin, (a).ev_end, 0, __VA_ARGS__); \
    else                                                                                          \
      hipLaunchKernelGGL(kernel, grid, block, 0, (a).stream, __VA_ARGS__);                        \
  } while (0)

namespace fef {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// Workgroup barrier that waits for this wavefront's LDS traffic only.  __syncthreads() would
// also drain the vector-memory counter and with it the W tiles prefetched for later steps.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Row r of this launch (0 <= r < nrows) is row row0 + r of the stacked [draft; target] matrix.
__device__ inline const __bf16* h_row(const HeadArgs& a, int r) {
  const int g = a.row0 + r;
  return g < a.BK ? (const __bf16*)a.h_draft + (size_t)g * a.d
                  : (const __bf16*)a.h_target + (size_t)(g - a.BK) * a.d;
}

// LDS tiles of bf16 are [rows][64 k] = 128 B per row.  The LDS has 64 four-byte banks, so two
// consecutive rows cover all banks once; the eight 16-byte chunks of a row are stored at
// chunk ^ ((row >> 1) & 7) so that 16-byte reads of one k-chunk over 16 consecutive rows
// touch every bank exactly once.
#ifndef FEF_SWZ_SHIFT
#define FEF_SWZ_SHIFT 1
#endif
__device__ inline int swz(int row, int chunk) { return row * 8 + (chunk ^ ((row >> FEF_SWZ_SHIFT) & 7)); }

// DPP within rows of 16 lanes: rotate right by N lanes (row_ror:N).
template <int N>
__device__ inline float row_ror(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x120 + N, 0xf, 0xf, false));
}
// All-reduce over the 16 lanes of a DPP row.
__device__ inline float row16_max(float x) {
  x = fmaxf(x, row_ror<8>(x)); x = fmaxf(x, row_ror<4>(x));
  x = fmaxf(x, row_ror<2>(x)); x = fmaxf(x, row_ror<1>(x));
  return x;
}
// Value of lane l ^ 16 (the other 16-lane row of the same 32-lane half): ds_swizzle in bit mode,
// and_mask 0x1f, or_mask 0, xor_mask 0x10.  Uses the LDS crossbar, no LDS memory.
__device__ inline float swap16(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, x), 0x401F));
}
__device__ inline float row16_sum(float x) {
  x += row_ror<8>(x); x += row_ror<4>(x); x += row_ror<2>(x); x += row_ror<1>(x);
  return x;
}

}  // namespace fef
