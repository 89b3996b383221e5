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

// ---------------------------------------------------------------------------------------------
// Pieces shared by the LDS-tiled MFMA kernels (32-wide k-steps, v_mfma_f32_32x32x16_bf16).
// ---------------------------------------------------------------------------------------------

// LDS tiles of [rows][32 k] bf16 = 64 B per row = four 16-byte chunks.  The LDS has 64 four-byte
// banks, i.e. four such rows per sweep, so chunk c of row r is kept at position c ^ ((r >> 2) & 3):
// the 16-byte fragment reads of 16 consecutive rows then touch every bank once.
__device__ inline int swz4(int row, int chunk) { return row * 4 + (chunk ^ ((row >> 2) & 3)); }

// global_load_lds_dwordx4: lane l copies 16 bytes from its global address to LDS offset
// lds_off + 16 l (lds_off wavefront-uniform, carried in M0).  Written as inline assembly so
// that the compiler's wait-count pass does not tie the fragment reads of one stage to the
// loads still in flight for the others (it would drain them all once per ring cycle);
// completion is tracked by hand with vmcnt before the workgroup barrier.
__device__ inline void load_to_lds_16(const void* gptr, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(gptr), "s"(lds_off) : "memory");
}
// Wait until at most N of this wavefront's vector-memory operations are outstanding.
template <int N>
__device__ inline void wait_newer() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
__device__ inline uint32_t lds_offset(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)p);
}
// x_k = max(x_k, x_k rotated right by N lanes inside its row of 16), for G registers that do not depend on one
// another, in one statement: the two wait states a DPP read needs after a vector write of its source are paid once
// in front, not once per instruction.
template <int N>
__device__ inline void max_ror_x8(float* x) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8, "rotation inside a row of 16 lanes");
  asm("s_nop 1\n\t"
      "v_max_f32_dpp %0, %0, %0 row_ror:%8 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %1, %1, %1 row_ror:%8 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %2, %2, %2 row_ror:%8 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %3, %3, %3 row_ror:%8 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %4, %4, %4 row_ror:%8 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %5, %5, %5 row_ror:%8 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %6, %6, %6 row_ror:%8 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %7, %7, %7 row_ror:%8 row_mask:0xf bank_mask:0xf"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
      : "n"(N));
}
template <int N>
__device__ inline void max_ror_x4(float* x) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8, "rotation inside a row of 16 lanes");
  asm("s_nop 1\n\t"
      "v_max_f32_dpp %0, %0, %0 row_ror:%4 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %1, %1, %1 row_ror:%4 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %2, %2, %2 row_ror:%4 row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %3, %3, %3 row_ror:%4 row_mask:0xf bank_mask:0xf"
      : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3])
      : "n"(N));
}
// RB registers, RB a multiple of 4
template <int N, int RB>
__device__ inline void max_ror_all(float* x) {
  static_assert(RB % 4 == 0, "groups of eight and four");
#pragma unroll
  for (int q = 0; q + 8 <= RB; q += 8) max_ror_x8<N>(x + q);
  if constexpr (RB % 8 == 4) max_ror_x4<N>(x + RB - 4);
}
// max of numbers that are not NaN in one instruction (fmaxf also quiets signalling NaNs, which costs a second one)
__device__ inline float vmax(float x, float y) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
  return r;
}
__device__ inline float vmax3(float x, float y, float z) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(y), "v"(z));
  return r;
}

// Epilogue of a wavefront that holds NI x 2 accumulator tiles of 32 x 32: rows mw .. mw + 32 NI - 1,
// tokens vbase .. vbase + 63.  Writes the scaled logits and one (max, sum exp) partial per row.
// D layout of the 32x32 MFMA: lane holds D[8 (r/4) + 4 h + r%4][j32], r = 0..15, so for a fixed r
// the 32 lanes of a half-wavefront hold 32 consecutive tokens of one row: a dword store writes two
// full 128-byte lines, and the (max, sum exp) over the 64 tokens is a reduction over those 32
// lanes (four DPP steps inside rows of 16 lanes and one swap of the two rows).  No LDS, and no
// branch in the interior tiles, so the 16 NI independent (row tile, r) chains interleave freely.
//
// CE = true is the cross-entropy use of the head: nothing is written but the partials and, for
// the lane that holds a row's label token, that token's scaled logit.
//
// The partials do not go to memory but to LDS, lds_part[row of the workgroup tile][4 token groups of 64], for the
// caller to merge into one partial per (row, workgroup tile); mw_local is the wavefront's first row inside the
// workgroup tile and lcol its token group.  A wavefront whose tokens all lie past V leaves (-inf, 0).  (The pointer
// is typed as LDS: through a generic pointer the writes would be FLAT instructions, which count in the
// vector-memory counter too and complete out of its order, and the kernels that call this with loads in flight
// wait by count.)
template <int NI, bool CE = false, int RB = 16>
__device__ __forceinline__ void store_logits_and_partials(const HeadArgs& a, floatx16 (&acc)[NI][2], int mw, int vbase,
                                                 int M, int lane, float2* lds_part, int mw_local, int lcol) {
  static_assert(RB == 4 || RB == 8 || RB == 16, "accumulator indices per batch");
  constexpr float kLog2e = 1.4426950408889634f;
  const int j32 = lane & 31, h = lane >> 5;
  const float sc = a.inv_tau;
  const int v0 = vbase + j32, v1 = v0 + 32;
  float* lbase = CE ? nullptr : a.logits + (size_t)(mw + 4 * h) * a.ldl + v0;
  typedef float floatx2 __attribute__((ext_vector_type(2)));  // float2's layout, assignable in any address space
  typedef __attribute__((address_space(3))) floatx2 lds_floatx2;
  lds_floatx2* pbase = (lds_floatx2*)lds_part + (mw_local + 4 * h) * 4 + lcol;
  constexpr int pstride = 4;
  if (vbase >= a.V) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (j32 == 0) pbase[(i * 32 + 8 * (r >> 2) + (r & 3)) * pstride] = floatx2{-INFINITY, 0.f};
    return;
  }
  if constexpr (CE) {
    // The label token's logit of a row lies in exactly one lane of one wavefront.  Most calls hold none (64 of V
    // tokens, 32 NI rows): every lane looks up one or two of the rows' labels, and a label that falls among this
    // call's tokens is fetched in a loop over the hits with wavefront-uniform indices (the 32 x 32 accumulator tile
    // and the element inside it by comparison of scalars; the lane that holds it stores it).  Going through all of a
    // lane's elements with a label lookup each is a chain of load latencies per hit, and the workgroup that pays it
    // falls out of step with those it shares operand tiles with through L2.
#pragma unroll
    for (int q = 0; q < (32 * NI + kWave - 1) / kWave; ++q) {
      const int rl = q * kWave + lane;
      const int lab = rl < 32 * NI && mw + rl < M ? a.labels[mw + rl] : -1;
      unsigned long long hits = __builtin_amdgcn_ballot_w64((unsigned)(lab - vbase) < 64u && lab < a.V);
      while (hits != 0) {  // wavefront-uniform
        const int src = __builtin_ctzll(hits);
        hits &= hits - 1;
        const int rowl = q * kWave + src;                                 // row inside this call's rows
        const int col = __builtin_amdgcn_readlane(lab, src) - vbase;      // token inside its 64
        const int ti = rowl >> 5, x = rowl & 31, th = (x >> 2) & 1, tr = ((x >> 3) << 2) | (x & 3);
        const int tc = col >> 5, tj = col & 31;
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
          for (int c = 0; c < 2; ++c)
            if (i == ti && c == tc) {  // wavefront-uniform: one of the accumulator tiles
              v = acc[i][c][0];
#pragma unroll
              for (int r = 1; r < 16; ++r) v = r == tr ? acc[i][c][r] : v;
            }
        if (lane == tj + 32 * th) a.label_logit[mw + rowl] = v * sc;
      }
    }
  }
  if (mw + 32 * NI <= M && vbase + 64 <= a.V) {  // interior: wavefront-uniform
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      // phase by phase over RB accumulator indices at a time, so that the RB reduction chains
      // are independent neighbours in program order (RB = 16 where the epilogue's arithmetic is
      // on the critical path, less where registers are short)
#pragma unroll
      for (int rb = 0; rb < 16; rb += RB) {
        float mx[RB], e[RB];
#pragma unroll
        for (int q = 0; q < RB; ++q) {
          const int r = rb + q;
          const int mr = i * 32 + 8 * (r >> 2) + (r & 3);
          const float l0 = acc[i][0][r] * sc, l1 = acc[i][1][r] * sc;
          acc[i][0][r] = l0;
          acc[i][1][r] = l1;
          if constexpr (!CE) {
            float* dst = lbase + (size_t)mr * a.ldl;
            // non-temporal: the logits are read next by another kernel, and as ordinary stores they
            // sit dirty in L2 and push out the W and H lines the neighbouring workgroups are about
            // to ask for (measured: 6 % of the kernel's time at M = 128 and 256, 0.5 % at M >= 1024)
            __builtin_nontemporal_store(l0, dst);
            __builtin_nontemporal_store(l1, dst + 32);
          }
          mx[q] = vmax(l0, l1);
        }
        max_ror_all<8, RB>(mx);
        max_ror_all<4, RB>(mx);
        max_ror_all<2, RB>(mx);
        max_ror_all<1, RB>(mx);
#pragma unroll
        for (int q = 0; q < RB; ++q) e[q] = swap16(mx[q]);
#pragma unroll
        for (int q = 0; q < RB; ++q) mx[q] = vmax(mx[q], e[q]);
#pragma unroll
        for (int q = 0; q < RB; ++q) {
          const float mb = mx[q] * kLog2e;
          e[q] = __builtin_amdgcn_exp2f(fmaf(acc[i][0][rb + q], kLog2e, -mb)) +
                 __builtin_amdgcn_exp2f(fmaf(acc[i][1][rb + q], kLog2e, -mb));
        }
#pragma unroll
        for (int q = 0; q < RB; ++q) e[q] += row_ror<8>(e[q]);
#pragma unroll
        for (int q = 0; q < RB; ++q) e[q] += row_ror<4>(e[q]);
#pragma unroll
        for (int q = 0; q < RB; ++q) e[q] += row_ror<2>(e[q]);
#pragma unroll
        for (int q = 0; q < RB; ++q) e[q] += row_ror<1>(e[q]);
        float t[RB];
#pragma unroll
        for (int q = 0; q < RB; ++q) t[q] = swap16(e[q]);
        // every lane of a half-wavefront holds its row's pair and writes it to the same address
#pragma unroll
        for (int q = 0; q < RB; ++q) {
          const int r = rb + q;
          const int mr = i * 32 + 8 * (r >> 2) + (r & 3);
          pbase[mr * pstride] = floatx2{mx[q], e[q] + t[q]};
        }
      }
    }
  } else if (vbase < a.V) {  // edge tiles: rows past M and tokens past V are masked
    const bool ok0 = v0 < a.V, ok1 = v1 < a.V;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int mr = i * 32 + 8 * (r >> 2) + (r & 3);
        const bool row_ok = mw + 4 * h + mr < M;
        const float l0 = acc[i][0][r] * sc, l1 = acc[i][1][r] * sc;
        if constexpr (!CE) {
          float* dst = lbase + (size_t)mr * a.ldl;
          if (row_ok && ok0) dst[0] = l0;
          if (row_ok && ok1) dst[32] = l1;
        }
        float mx = row16_max(fmaxf(ok0 ? l0 : -INFINITY, ok1 ? l1 : -INFINITY));
        mx = fmaxf(mx, swap16(mx));  // finite: token vbase itself is valid
        const float mb = mx * kLog2e;
        float e = (ok0 ? exp2f(fmaf(l0, kLog2e, -mb)) : 0.f) + (ok1 ? exp2f(fmaf(l1, kLog2e, -mb)) : 0.f);
        e = row16_sum(e);
        e += swap16(e);
        if (j32 == 0) pbase[mr * pstride] = floatx2{row_ok ? mx : -INFINITY, row_ok ? e : 0.f};
      }
    }
  }
}

// One (max, sum exp) partial per (row, workgroup tile of 256 tokens): the four partials of a row that the epilogue
// left in LDS ([row of the tile][4 slots], each over a quarter of the tile's tokens; which quarter is the epilogue's
// business), merged in a fixed order by the thread that owns the row.  A quarter of the partials for the kernels
// that read them next.  rows: rows of the workgroup tile; m0: its first row; nt: its 256-token tile.
__device__ inline void merge_tile_partials(const HeadArgs& a, const float2* lp, int rows, int m0, int nt, int M, int tid) {
  constexpr float kLog2e = 1.4426950408889634f;
  if (tid < rows && m0 + tid < M) {
    float2 p[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) p[c] = lp[tid * 4 + c];
    const float mx = fmaxf(fmaxf(p[0].x, p[1].x), fmaxf(p[2].x, p[3].x));  // finite: the tile's first token exists
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) sum += p[c].y * exp2f((p[c].x - mx) * kLog2e);
    a.partials[(size_t)(m0 + tid) * a.nT + nt] = make_float2(mx, sum);
  }
}

}  // namespace fef
