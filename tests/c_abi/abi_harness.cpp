// Calls the library through its C header alone: plain hipMalloc'd buffers, no Python, no torch.
// What it checks needs no second implementation: with identical draft and target hidden states the
// two laws coincide, so every acceptance ratio is 1 and Algorithm 2 accepts the whole window
// (accept_len = K, the committed tokens are the drafts, exactly those K positions leave the mask);
// a repeated call gives the same bits; a workspace that is too small is refused.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

#include "fef.h"

#define HIP_OK(x)                                                                  \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      return 2;                                                                    \
    }                                                                              \
  } while (0)
#define CHECK(c)                                                     \
  do {                                                               \
    if (!(c)) {                                                      \
      std::printf("FAILED line %d: %s\n", __LINE__, #c);             \
      return 1;                                                      \
    }                                                                \
  } while (0)

static uint16_t to_bf16(float f) {  // round to nearest even
  uint32_t u;
  std::memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static int run_case(int B, int K, int block, int d, int V) {
  std::printf("case B=%d K=%d block=%d d=%d V=%d\n", B, K, block, d, V);
  std::fflush(stdout);
  std::mt19937 rng(1234u + (unsigned)(B * 131 + K * 17 + V));
  std::normal_distribution<float> nd(0.f, 1.f);
  std::vector<uint16_t> W((size_t)V * d), H((size_t)B * K * d);
  const float sigma_h = 3.f / (0.02f * std::sqrt((float)d));
  for (auto& w : W) w = to_bf16(0.02f * nd(rng));
  for (auto& h : H) h = to_bf16(sigma_h * nd(rng));

  void *dW, *dH, *ws;
  int32_t *tok, *acc, *drafts;
  uint8_t* rem;
  HIP_OK(hipMalloc(&dW, W.size() * 2));
  HIP_OK(hipMalloc(&dH, H.size() * 2));
  HIP_OK(hipMalloc((void**)&tok, (size_t)B * K * 4));
  HIP_OK(hipMalloc((void**)&drafts, (size_t)B * K * 4));
  HIP_OK(hipMalloc((void**)&acc, (size_t)B * 4));
  HIP_OK(hipMalloc((void**)&rem, (size_t)B * block));
  HIP_OK(hipMemcpy(dW, W.data(), W.size() * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dH, H.data(), H.size() * 2, hipMemcpyHostToDevice));

  fef_params p;
  std::memset(&p, 0, sizeof p);
  p.struct_size = sizeof p;
  p.B = B; p.d = d; p.V = V;
  p.dtype = FEF_BF16;
  p.temperature = 1.f;
  p.step = 3;
  p.n_rm = -1;
  p.final_pass = 1;
  p.recorrupt_prob = 1.f;
  p.diag_draft_tokens = drafts;
  const size_t need = fef_workspace_bytes(&p, K, block);
  CHECK(need > 0);
  HIP_OK(hipMalloc(&ws, need));
  p.workspace = ws;

  // a workspace that is one byte short is refused and nothing runs
  p.workspace_bytes = need - 1;
  CHECK(fef_verify_step(&p, dH, dH, dW, K, block, 42, tok, acc, rem) == FEF_ERR_WORKSPACE);
  p.workspace_bytes = need;

  std::vector<int32_t> t1((size_t)B * K), t2(t1.size()), dr(t1.size()), a1(B), a2(B);
  std::vector<uint8_t> r1((size_t)B * block), r2(r1.size());
  for (int rep = 0; rep < 2; ++rep) {
    const fef_status s = fef_verify_step(&p, dH, dH, dW, K, block, 42, tok, acc, rem);
    if (s != FEF_OK) {
      std::printf("fef_verify_step: %s (%s)\n", fef_status_string(s), fef_last_error());
      return 1;
    }
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(rep ? t2.data() : t1.data(), tok, t1.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(rep ? a2.data() : a1.data(), acc, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(rep ? r2.data() : r1.data(), rem, r1.size(), hipMemcpyDeviceToHost));
  }
  HIP_OK(hipMemcpy(dr.data(), drafts, dr.size() * 4, hipMemcpyDeviceToHost));
  CHECK(t1 == t2 && a1 == a2 && r1 == r2);  // same inputs and seed, same bits
  for (int b = 0; b < B; ++b) {
    CHECK(a1[b] == K);  // identical laws: every draft accepted
    for (int m = 0; m < K; ++m) {
      const int32_t x = t1[(size_t)b * K + m];
      CHECK(x >= 0 && x < V && x == dr[(size_t)b * K + m]);
    }
    // a fresh block: the window is its first K positions; they are resolved, the rest is not
    for (int i = 0; i < block; ++i) CHECK(r1[(size_t)b * block + i] == (i < K ? 0 : 1));
  }
  HIP_OK(hipFree(ws)); HIP_OK(hipFree(rem)); HIP_OK(hipFree(acc)); HIP_OK(hipFree(drafts));
  HIP_OK(hipFree(tok)); HIP_OK(hipFree(dH)); HIP_OK(hipFree(dW));
  return 0;
}

int main() {
  std::printf("fef ABI version %d\n", fef_abi_version());
  if (fef_abi_version() != FEF_ABI_VERSION) {
    std::printf("library and header disagree\n");
    return 1;
  }
  // one shape per head kernel the selection rule can pick: skinny, streaming (both heights), 256 x 256
  const int cases[][5] = {{1, 8, 32, 512, 3000}, {4, 8, 16, 256, 1500}, {8, 8, 16, 256, 700}, {20, 8, 16, 128, 1000}};
  for (const auto& c : cases) {
    const int rc = run_case(c[0], c[1], c[2], c[3], c[4]);
    if (rc) return rc;
  }
  std::printf("OK\n");
  return 0;
}
