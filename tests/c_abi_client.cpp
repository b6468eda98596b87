// A client of include/zz.h that uses nothing but the C ABI and the HIP runtime (no Python, no
// torch): it allocates the arena, the workspace and the tensors with hipMalloc, appends a cache,
// runs prefill, decode and the fused decode step on a retrieval and a streaming layer, and checks
// the outputs against closed forms.  With q = 0 every visible key gets the same weight, so with
// V[j][d] = j the output is the mean of the attended positions (Sections 1 and 3.3: all j <= i
// for a retrieval head; the S sink positions and the W newest for a streaming head).
// Built by __graft_entry__.build(); run by tests/test_c_abi_client.py on the GPU.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "zz.h"

#define HIP_OK(x)                                                                  \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      std::printf("FAIL: %s -> %s\n", #x, hipGetErrorString(e_));                  \
      return 2;                                                                    \
    }                                                                              \
  } while (0)
#define ZZ_OK_(x)                                                                  \
  do {                                                                             \
    int rc_ = (x);                                                                 \
    if (rc_ != ZZ_OK) {                                                            \
      std::printf("FAIL: %s -> %s %s\n", #x, zz_strerror(rc_), zz_last_error_detail()); \
      return 3;                                                                    \
    }                                                                              \
  } while (0)

static uint16_t to_bf16(float f) {  // exact for the small integers used here
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}
static float from_bf16(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// mean of the positions query i attends to
static double mean_attended(int i, bool streaming, int S, int W) {
  double sum = 0;
  int n = 0;
  for (int j = 0; j <= i; ++j)
    if (!streaming || j < S || i - j < W) {
      sum += j;
      ++n;
    }
  return sum / n;
}

int main() {
  const int L = 2, Hq = 8, Hkv = 2, D = 128, B = 2, S = 4, W = 24, T = 200, CHUNK = 96;
  const uint8_t layer_mask[L] = {0, 1};
  zz_config cfg;
  std::memset(&cfg, 0, sizeof(cfg));
  cfg.n_layers = L; cfg.n_q_heads = Hq; cfg.n_kv_heads = Hkv; cfg.head_dim = D; cfg.batch = B; cfg.max_ctx = T + 8;
  cfg.sink = S; cfg.window = W; cfg.max_chunk = CHUNK; cfg.layout = ZZ_ZIGZAG; cfg.layer_is_streaming = layer_mask;
  const size_t arena_bytes = zz_arena_bytes(&cfg), ws_bytes = zz_workspace_bytes(&cfg);
  if (!arena_bytes || !ws_bytes) { std::printf("FAIL: sizes\n"); return 1; }
  void *arena = nullptr, *ws = nullptr;
  HIP_OK(hipMalloc(&arena, arena_bytes));
  HIP_OK(hipMalloc(&ws, ws_bytes));
  HIP_OK(hipMemset(arena, 0xFF, arena_bytes));   // NaN patterns: an unwritten slot that leaks shows up
  zz_ctx *ctx = nullptr;
  ZZ_OK_(zz_create(&cfg, arena, arena_bytes, ws, ws_bytes, &ctx));

  // host tensors: q = 0, k arbitrary small integers, v[j][d] = j   (j < 256: exact in bf16)
  const size_t kv_elems = (size_t)B * T * Hkv * D, q_elems = (size_t)B * T * Hq * D;
  std::vector<uint16_t> hk(kv_elems), hv(kv_elems), hq(q_elems, to_bf16(0.f)), ho(q_elems);
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < T; ++j)
      for (int g = 0; g < Hkv; ++g)
        for (int d = 0; d < D; ++d) {
          const size_t at = (((size_t)b * T + j) * Hkv + g) * D + d;
          hk[at] = to_bf16((float)((j * 7 + d * 3 + g) % 5 - 2));
          hv[at] = to_bf16((float)j);
        }
  uint16_t *dq, *dout;
  HIP_OK(hipMalloc((void **)&dq, q_elems * 2));
  HIP_OK(hipMalloc((void **)&dout, q_elems * 2));
  HIP_OK(hipMemcpy(dq, hq.data(), q_elems * 2, hipMemcpyHostToDevice));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  int failures = 0;
  auto expect = [&](const char *what, int layer, int i, float got) {
    const double want = mean_attended(i, layer_mask[layer] != 0, S, W);
    if (!(std::fabs(got - want) <= 0.01 * (1.0 + want))) {   // bf16 output: 8 bits of mantissa
      if (failures < 10) std::printf("FAIL: %s layer %d position %d: got %g, want %g\n", what, layer, i, got, want);
      ++failures;
    }
  };
  // per sequence the chunk [a, e) is contiguous inside [B, T, ...] only for B == 1: stage chunk tensors
  std::vector<uint16_t> ck, cv;
  uint16_t *dck, *dcv;
  HIP_OK(hipMalloc((void **)&dck, (size_t)B * CHUNK * Hkv * D * 2));
  HIP_OK(hipMalloc((void **)&dcv, (size_t)B * CHUNK * Hkv * D * 2));
  for (int layer = 0; layer < L; ++layer) {
    const int n_prefill = T - 8;
    for (int a = 0; a < n_prefill; a += CHUNK) {
      const int n = (a + CHUNK < n_prefill ? CHUNK : n_prefill - a);
      ck.assign((size_t)B * n * Hkv * D, 0);
      cv.assign((size_t)B * n * Hkv * D, 0);
      for (int b = 0; b < B; ++b) {
        std::memcpy(&ck[(size_t)b * n * Hkv * D], &hk[((size_t)b * T + a) * Hkv * D], (size_t)n * Hkv * D * 2);
        std::memcpy(&cv[(size_t)b * n * Hkv * D], &hv[((size_t)b * T + a) * Hkv * D], (size_t)n * Hkv * D * 2);
      }
      HIP_OK(hipMemcpy(dck, ck.data(), ck.size() * 2, hipMemcpyHostToDevice));
      HIP_OK(hipMemcpy(dcv, cv.data(), cv.size() * 2, hipMemcpyHostToDevice));
      ZZ_OK_(zz_attn_prefill(ctx, layer, dq, dck, dcv, n, dout, stream));   // q is all zeros: any rows do
      ZZ_OK_(zz_kv_append(ctx, layer, dck, dcv, n, stream));
      HIP_OK(hipStreamSynchronize(stream));
      HIP_OK(hipMemcpy(ho.data(), dout, (size_t)B * n * Hq * D * 2, hipMemcpyDeviceToHost));
      for (int b = 0; b < B; ++b)
        for (int i = 0; i < n; i += 7)
          for (int h = 0; h < Hq; h += 3)
            expect("prefill", layer, a + i, from_bf16(ho[(((size_t)b * n + i) * Hq + h) * D + (i + h) % D]));
    }
    if (zz_layer_len(ctx, layer) != n_prefill) { std::printf("FAIL: length\n"); return 1; }
    // decode: four steps as append + attention, four as the fused step
    for (int t = n_prefill; t < T; ++t) {
      ck.assign((size_t)B * Hkv * D, 0);
      cv.assign((size_t)B * Hkv * D, 0);
      for (int b = 0; b < B; ++b) {
        std::memcpy(&ck[(size_t)b * Hkv * D], &hk[((size_t)b * T + t) * Hkv * D], (size_t)Hkv * D * 2);
        std::memcpy(&cv[(size_t)b * Hkv * D], &hv[((size_t)b * T + t) * Hkv * D], (size_t)Hkv * D * 2);
      }
      HIP_OK(hipMemcpy(dck, ck.data(), ck.size() * 2, hipMemcpyHostToDevice));
      HIP_OK(hipMemcpy(dcv, cv.data(), cv.size() * 2, hipMemcpyHostToDevice));
      if (t < n_prefill + 4) {
        ZZ_OK_(zz_kv_append(ctx, layer, dck, dcv, 1, stream));
        ZZ_OK_(zz_attn_decode(ctx, layer, dq, dout, stream));
      } else {
        ZZ_OK_(zz_decode_step(ctx, layer, dq, dck, dcv, dout, stream));
      }
      HIP_OK(hipStreamSynchronize(stream));
      HIP_OK(hipMemcpy(ho.data(), dout, (size_t)B * Hq * D * 2, hipMemcpyDeviceToHost));
      for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) expect("decode", layer, t, from_bf16(ho[((size_t)b * Hq + h) * D + (t + h) % D]));
    }
    if (zz_layer_len(ctx, layer) != T) { std::printf("FAIL: length after decode\n"); return 1; }
  }
  if (zz_attn_decode(ctx, 5, dq, dout, stream) != ZZ_ERANGE) { std::printf("FAIL: error path\n"); return 1; }
  ZZ_OK_(zz_destroy(ctx));
  HIP_OK(hipStreamDestroy(stream));
  hipFree(dq); hipFree(dout); hipFree(dck); hipFree(dcv); hipFree(arena); hipFree(ws);
  if (failures) { std::printf("FAIL: %d mismatches\n", failures); return 1; }
  std::printf("PASS\n");
  return 0;
}
