// Finish of the cross-entropy use of the vocabulary head (Algorithm 1, token-level loss):
// CE_m = log sum_v exp(L[m, v]) - L[m, label_m], loss = sum_m CE_m.  The head kernels have left
// per (row, vocabulary tile) partials (max, sum exp) and the label token's logit per row; no
// logits exist in memory.  Fixed reduction trees: the results are reproducible bit for bit.
#include <math.h>

#include "fef_device.hpp"
#include "wave_ops.hpp"

namespace fef {
namespace {

constexpr int NT = 256, NW = NT / kWave;

// label logits start as NaN, so that a label no head kernel meets (>= V) shows in the result
__global__ __launch_bounds__(NT) void ce_init_kernel(float* label_logit, int R) {
  const int r = blockIdx.x * NT + threadIdx.x;
  if (r < R) label_logit[r] = __builtin_nanf("");
}

// one wavefront per row
__global__ __launch_bounds__(NT) void ce_row_kernel(CeArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x * NW + wave;
  if (r >= a.R) return;
  const int lab = a.labels[r];
  float ce = 0.f;
  if (lab >= 0) {  // wavefront-uniform
    const float2* P = a.partials + (size_t)r * a.nT;
    // One pass: each lane merges its partials eight at a time (eight independent loads in
    // flight), carrying a running (max, sum exp); the lanes' pairs are merged after the loop.
    float mx = -INFINITY, sm = 0.f;
    for (int t0 = lane; t0 < a.nT; t0 += 8 * kWave) {
      float2 p[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int t = t0 + j * kWave;
        p[j] = t < a.nT ? P[t] : make_float2(-INFINITY, 0.f);
      }
      float m8 = mx;
#pragma unroll
      for (int j = 0; j < 8; ++j) m8 = fmaxf(m8, p[j].x);
      float s8 = sm > 0.f ? sm * expf(mx - m8) : 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) s8 += p[j].y > 0.f ? p[j].y * expf(p[j].x - m8) : 0.f;
      mx = m8;
      sm = s8;
    }
    const float wmx = wave_max(mx);
    sm = sm > 0.f ? sm * expf(mx - wmx) : 0.f;
    mx = wmx;
    sm = wave_sum(sm);
    ce = mx + logf(sm) - a.label_logit[r];
  }
  if (lane == 0) a.out_ce[r] = ce;
}

// one workgroup: thread t sums rows t, t + 256, ... in order, then a fixed tree over the threads
__global__ __launch_bounds__(NT) void ce_sum_kernel(CeArgs a) {
  __shared__ float part[NW];
  float s = 0.f;
  for (int r = threadIdx.x; r < a.R; r += NT) s += a.out_ce[r];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < NW; ++w) t += part[w];
    a.out_loss[0] = t;
  }
}

}  // namespace

hipError_t launch_ce_init(float* label_logit, int R, hipStream_t stream) {
  hipLaunchKernelGGL(ce_init_kernel, dim3((R + NT - 1) / NT), dim3(NT), 0, stream, label_logit, R);
  return hipGetLastError();
}

hipError_t launch_ce_finish(const CeArgs& a) {
  hipLaunchKernelGGL(ce_row_kernel, dim3((a.R + NW - 1) / NW), dim3(NT), 0, a.stream, a);
  if (a.out_loss) hipLaunchKernelGGL(ce_sum_kernel, dim3(1), dim3(NT), 0, a.stream, a);
  return hipGetLastError();
}

}  // namespace fef
