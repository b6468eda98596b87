// Host-side check of the runtime behind include/zz.h under AddressSanitizer and
// UndefinedBehaviorSanitizer, without a GPU: zz_api.cpp and zz_transport.cpp are compiled
// with the host compiler, the kernel launchers are replaced by recorders that validate what
// the host hands to a launch (grid within limits, every sequence's split range inside the
// partials the workspace holds, prefix sums consistent with the grid).  Built and run by
// tests/test_host_sanitized.py.
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "zz_internal.h"

static int g_launches = 0, g_fail = 0;

#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::fprintf(stderr, "%s:%d: EXPECT(%s) failed\n", __FILE__, __LINE__, #cond); \
      ++g_fail;                                                             \
    }                                                                       \
  } while (0)

// ---- recorders standing in for the launchers of zz_kernels.hip ----
const char *hipGetErrorString(hipError_t) { return "stub"; }
int zz_query_num_cu() { return 256; }
hipError_t zz_static_scratch(char **out) {
  *out = (char *)0x40000000;
  return hipSuccess;
}
static bool g_capturing = false;
bool zz_stream_is_capturing(hipStream_t) { return g_capturing; }

static int g_append_launches = 0, g_prefill_launches = 0;
hipError_t zz_launch_append(const zz_append_params &p, const zz_seq_lens &lens, hipStream_t) {
  ++g_launches;
  ++g_append_launches;
  EXPECT(!lens.ragged || p.batch <= ZZ_MAX_RAGGED_BATCH);
  EXPECT(p.n_new > 0 && p.batch > 0 && p.len >= 0);
  for (int g = 0; g < p.n_kv_heads; ++g) EXPECT(p.head_index[g] < p.grp[p.head_group[g]].n_heads);
  return hipSuccess;
}
static int g_stage_launches = 0;
hipError_t zz_launch_stage(const zz_stage_params &p, const zz_seq_lens &, hipStream_t) {
  ++g_launches;
  ++g_stage_launches;
  EXPECT(p.n_new > 0 && (p.n_new + 31) / 32 <= p.stage_tiles);
  return hipSuccess;
}
hipError_t zz_launch_prefill(const zz_prefill_params &p, const zz_seq_lens &lens, int, hipStream_t) {
  ++g_launches;
  ++g_prefill_launches;
  EXPECT(!lens.ragged || p.batch <= ZZ_MAX_RAGGED_BATCH);
  if (lens.ragged)
    for (int b = 0; b < p.batch; ++b) EXPECT(((int64_t)lens.len[b] + 31) / 32 <= p.grp.n_tiles || p.grp.streaming);
  EXPECT(p.n_new > 0 && p.n_past >= 0 && p.batch > 0 && p.grp.n_heads > 0);
  EXPECT(((int64_t)p.n_past + 31) / 32 <= p.grp.n_tiles || p.grp.streaming);
  return hipSuccess;
}
static int g_skewed_launches = 0;
hipError_t zz_launch_decode(const zz_decode_params &p, hipStream_t) {
  ++g_launches;
  EXPECT(p.n_splits >= 1 && p.n_splits <= ZZ_MAX_SPLITS && p.tiles_per_split >= 1);
  EXPECT(p.n_tiles_valid == (p.n_valid + 31) / 32 && p.n_tiles_valid <= p.grp.n_tiles);
  EXPECT((int64_t)(p.n_splits - 1) * p.tiles_per_split < p.n_tiles_valid);   // no empty split
  EXPECT((int64_t)p.n_splits * p.tiles_per_split >= p.n_tiles_valid);        // every tile covered
  EXPECT(p.new_slot < p.n_valid);
  EXPECT(p.batch <= 65535 && p.grp.n_heads <= 65535);
  // the ranges the kernel will derive tile the cache exactly once, whichever parity a unit starts on
  EXPECT(p.tile_skew >= 0 && p.tile_skew < p.tiles_per_split);
  for (int parity = 0; parity < 2; ++parity) {
    int next = 0;
    for (int s = 0; s < p.n_splits; ++s) {
      int t0, t1;
      zz_split_range(s, p.n_splits, p.tiles_per_split, p.tile_skew, parity, p.n_tiles_valid, &t0, &t1);
      EXPECT(t0 == next && t1 > t0);
      next = t1;
    }
    EXPECT(next == p.n_tiles_valid);
  }
  if (p.tile_skew > 0) ++g_skewed_launches;
  return hipSuccess;
}
hipError_t zz_launch_decode_ragged(const zz_decode_ragged_params &p, int total_wg, hipStream_t) {
  ++g_launches;
  const int B = p.u.batch;
  EXPECT(B <= ZZ_MAX_RAGGED_BATCH && p.first_wg[0] == 0 && p.first_wg[B] == total_wg && total_wg >= B);
  EXPECT(p.u.tiles_per_split >= 1);
  for (int b = 0; b < B; ++b) {
    const int64_t len = p.seq_len[b];
    const int64_t n_valid = p.u.grp.streaming ? (len < p.sink + p.window ? len : p.sink + p.window) : len;
    const int64_t tiles = (n_valid + 31) / 32;
    const int splits = p.first_wg[b + 1] - p.first_wg[b];
    EXPECT(len >= 1 && tiles <= p.u.grp.n_tiles);
    EXPECT(splits >= 1 && splits <= ZZ_MAX_SPLITS);
    EXPECT((int64_t)(splits - 1) * p.u.tiles_per_split < tiles);
    EXPECT((int64_t)splits * p.u.tiles_per_split >= tiles);
  }
  return hipSuccess;
}
static int g_zero_launches = 0;
hipError_t zz_launch_zero(int *, int n, hipStream_t) {
  ++g_launches;
  ++g_zero_launches;
  EXPECT(n > 0);
  return hipSuccess;
}
hipError_t zz_launch_probe_read(const void *, size_t bytes, int, int n_wg, void *, hipStream_t) {
  ++g_launches;
  EXPECT(bytes >= 16384 && n_wg > 0);
  return hipSuccess;
}

// ---- the scenarios ----
static zz_ctx *make(int L, int Hq, int Hkv, int D, int B, int max_ctx, int S, int W, int chunk, int layout,
                    const std::vector<uint8_t> &lmask, const std::vector<uint8_t> &hmask) {
  zz_config c;
  std::memset(&c, 0, sizeof(c));
  c.n_layers = L; c.n_q_heads = Hq; c.n_kv_heads = Hkv; c.head_dim = D; c.batch = B; c.max_ctx = max_ctx;
  c.sink = S; c.window = W; c.max_chunk = chunk; c.layout = layout;
  c.layer_is_streaming = lmask.empty() ? nullptr : lmask.data();
  c.kvhead_is_streaming = hmask.empty() ? nullptr : hmask.data();
  zz_ctx *ctx = nullptr;
  const int rc = zz_create(&c, (void *)0x10000000, zz_arena_bytes(&c), (void *)0x20000000, zz_workspace_bytes(&c), &ctx);
  EXPECT(rc == ZZ_OK && ctx);
  return ctx;
}

static unsigned rng_state = 12345;
static unsigned rnd() { return rng_state = rng_state * 1664525u + 1013904223u; }

// Host time of one zz_decode_step call (argument checks, launch plan, argument block), with the
// recorders in place of the launches: what the library itself adds to a decode step per layer.
static int time_decode_calls() {
  void *T = (void *)0x30000000;
  struct Case { const char *name; int B; bool unequal; } cases[] = {
      {"batch 1, 32k, equal lengths", 1, false}, {"batch 4, 128k, equal lengths", 4, false},
      {"batch 8, unequal lengths", 8, true}, {"batch 256, unequal lengths", 256, true}};
  for (const Case &cs : cases) {
    zz_ctx *ctx = make(2, 32, 8, 128, cs.B, 131072 + 8, 64, 256, 0, ZZ_ZIGZAG, {0, 1}, {});
    const int reps = 200000;
    double ns[2] = {0, 0};
    for (int layer = 0; layer < 2; ++layer) {
      const auto t0 = std::chrono::steady_clock::now();
      for (int r = 0; r < reps; ++r) {
        if ((r & 7) == 0)   // stay inside max_ctx; amortised over eight calls
          for (int b = 0; b < cs.B; ++b) zz_set_seq_len(ctx, layer, b, cs.unequal ? 1000 + 500 * (b % 200) : (cs.B == 1 ? 32767 : 131071));
        if (zz_decode_step(ctx, layer, T, T, T, T, nullptr) != ZZ_OK) return 1;
      }
      ns[layer] = std::chrono::duration<double, std::nano>(std::chrono::steady_clock::now() - t0).count() / reps;
    }
    std::printf("zz_decode_step host time, %s: retrieval layer %.0f ns, streaming layer %.0f ns per call\n", cs.name, ns[0], ns[1]);
    zz_destroy(ctx);
  }
  return 0;
}

int main(int argc, char **argv) {
  if (argc > 1 && std::strcmp(argv[1], "--time") == 0) return time_decode_calls();
  void *T = (void *)0x30000000;  // fake, aligned tensor address: the recorders never touch it
  // 0. the split ranges on their own: every (tiles per split, split count, length of the last split, skew,
  // parity) up to 12 tiles per split and 9 splits, under the conditions the host promises the kernel
  for (int tps = 1; tps <= 12; ++tps)
    for (int ns = 1; ns <= 9; ++ns)
      for (int last = 1; last <= tps; ++last)
        for (int skew = 0; skew < last && skew < tps; ++skew)
          for (int parity = 0; parity < 2; ++parity) {
            const int n_tiles = (ns - 1) * tps + last;
            int next = 0;
            for (int s = 0; s < ns; ++s) {
              int t0, t1;
              zz_split_range(s, ns, tps, skew, parity, n_tiles, &t0, &t1);
              EXPECT(t0 == next && t1 > t0);
              if (skew == 0) EXPECT(t0 == s * tps);
              next = t1;
            }
            EXPECT(next == n_tiles);
          }
  // 0b. decode calls with explicit skews, split counts and lengths: the launch recorder checks each plan
  {
    zz_ctx *ctx = make(2, 32, 8, 128, 3, 40000, 64, 256, 0, ZZ_ZIGZAG, {0, 1}, {});
    for (int skew : {0, 50, 200})
      for (int splits : {0, 2, 3, 7, 8, 33, 128})
        for (int64_t n : {1, 100, 1023, 1024, 3333, 20000, 39998}) {
          EXPECT(zz_tune(ctx, ZZ_TUNE_DECODE_XCD_SKEW, skew) == ZZ_OK);
          EXPECT(zz_tune(ctx, ZZ_TUNE_DECODE_SPLITS, splits) == ZZ_OK);
          EXPECT(zz_set_layer_len(ctx, 0, n) == ZZ_OK);
          EXPECT(zz_decode_step(ctx, 0, T, T, T, T, nullptr) == ZZ_OK);
          EXPECT(zz_attn_decode(ctx, 0, T, T, nullptr) == ZZ_OK);
        }
    EXPECT(g_skewed_launches > 20);
    EXPECT(zz_tune(ctx, ZZ_TUNE_DECODE_XCD_SKEW, 201) == ZZ_ERANGE);
    zz_destroy(ctx);
  }
  // 1. zigzag stack, equal lengths: append / prefill / decode at many lengths and split settings
  {
    zz_ctx *ctx = make(4, 32, 8, 128, 4, 131072, 64, 256, 4096, ZZ_ZIGZAG, {0, 1, 0, 1}, {});
    const int64_t lens[] = {0, 1, 31, 32, 33, 319, 320, 321, 511, 513, 4095, 4096, 65537, 131071};
    for (int64_t n : lens)
      for (int splits : {0, 1, 7, 128})
        for (int layer = 0; layer < 4; ++layer) {
          EXPECT(zz_tune(ctx, ZZ_TUNE_DECODE_SPLITS, splits) == ZZ_OK);
          EXPECT(zz_set_layer_len(ctx, layer, n) == ZZ_OK);
          EXPECT(zz_decode_step(ctx, layer, T, T, T, T, nullptr) == ZZ_OK);
          EXPECT(zz_layer_len(ctx, layer) == n + 1);
          EXPECT(zz_attn_decode(ctx, layer, T, T, nullptr) == ZZ_OK);
          EXPECT(zz_set_layer_len(ctx, layer, n) == ZZ_OK);
          const int n_new = n + 4096 <= 131072 ? 4096 : (int)(131072 - n);
          EXPECT(zz_attn_prefill(ctx, layer, T, T, T, n_new, T, nullptr) == ZZ_OK);
          EXPECT(zz_kv_append(ctx, layer, T, T, n_new, nullptr) == ZZ_OK);
          int64_t v = 0, c = 0;
          EXPECT(zz_set_layer_len(ctx, layer, n) == ZZ_OK);
          EXPECT(zz_prefill_tile_counts(ctx, layer, n_new, &v, &c) == ZZ_OK && v > 0 && v <= c);
        }
    EXPECT(zz_destroy(ctx) == ZZ_OK);
  }
  // 1b. the split counters are cleared ahead of every decode call until one clear has been issued
  //     outside a stream capture (a clear recorded into a graph runs only on replay)
  {
    zz_ctx *ctx = make(1, 32, 8, 128, 1, 4096, 64, 256, 0, ZZ_ZIGZAG, {0}, {});
    EXPECT(zz_set_layer_len(ctx, 0, 1000) == ZZ_OK);
    g_zero_launches = 0;
    g_capturing = true;
    EXPECT(zz_attn_decode(ctx, 0, T, T, nullptr) == ZZ_OK);
    EXPECT(zz_attn_decode(ctx, 0, T, T, nullptr) == ZZ_OK);
    EXPECT(g_zero_launches == 2);
    g_capturing = false;
    EXPECT(zz_attn_decode(ctx, 0, T, T, nullptr) == ZZ_OK);
    EXPECT(g_zero_launches == 3);
    EXPECT(zz_attn_decode(ctx, 0, T, T, nullptr) == ZZ_OK);
    g_capturing = true;
    EXPECT(zz_attn_decode(ctx, 0, T, T, nullptr) == ZZ_OK);
    EXPECT(g_zero_launches == 3);
    g_capturing = false;
    EXPECT(zz_destroy(ctx) == ZZ_OK);
  }
  // 2. unequal lengths, random, zigzag and mixed, up to the largest batch
  for (int layout : {ZZ_ZIGZAG, ZZ_MIXED})
    for (int B : {2, 5, 64, ZZ_MAX_RAGGED_BATCH}) {
      std::vector<uint8_t> hm(2 * 8);
      for (auto &x : hm) x = rnd() & 1;
      zz_ctx *ctx = layout == ZZ_ZIGZAG ? make(2, 32, 8, 128, B, 40000, 64, 256, 512, layout, {0, 1}, {})
                                        : make(2, 32, 8, 128, B, 40000, 64, 256, 512, layout, {}, hm);
      for (int round = 0; round < 40; ++round) {
        EXPECT(zz_tune(ctx, ZZ_TUNE_DECODE_SPLITS, round % 4 == 3 ? 1 + (int)(rnd() % 128) : 0) == ZZ_OK);
        EXPECT(zz_tune(ctx, ZZ_TUNE_NUM_CU, round % 5 == 4 ? 1 + (int)(rnd() % 512) : 256) == ZZ_OK);
        for (int layer = 0; layer < 2; ++layer) {
          for (int b = 0; b < B; ++b) {
            const unsigned r = rnd();
            const int64_t n = (r & 3) == 0 ? 1 + (r >> 8) % 40 : (r & 3) == 1 ? 1 + (r >> 8) % 2000 : 1 + (r >> 8) % 39000;
            EXPECT(zz_set_seq_len(ctx, layer, b, n) == ZZ_OK);
          }
          std::vector<int64_t> before(B);
          for (int b = 0; b < B; ++b) before[b] = zz_seq_len(ctx, layer, b);
          EXPECT(zz_attn_decode(ctx, layer, T, T, nullptr) == ZZ_OK);
          EXPECT(zz_decode_step(ctx, layer, T, T, T, T, nullptr) == ZZ_OK);
          for (int b = 0; b < B; ++b) EXPECT(zz_seq_len(ctx, layer, b) == before[b] + 1);
          int ns = 0, tps = 0;
          for (int grp = 0; grp < 2; ++grp) EXPECT(zz_decode_plan(ctx, layer, grp, &ns, &tps) == ZZ_OK);
          // unequal lengths or not: one attention launch per head kind behind one staging launch, and
          // one append launch (two for a layer of both kinds when the tile-wise kernel takes the retrieval heads)
          const int kinds = zz_layer_launches(ctx, layer);
          g_stage_launches = g_prefill_launches = 0;
          EXPECT(zz_attn_prefill(ctx, layer, T, T, T, 100, T, nullptr) == ZZ_OK);
          EXPECT(g_prefill_launches == kinds && g_stage_launches == 1);
          g_append_launches = 0;
          EXPECT(zz_kv_append(ctx, layer, T, T, 100, nullptr) == ZZ_OK);
          EXPECT(g_append_launches == 1);
          g_append_launches = 0;
          EXPECT(zz_kv_append(ctx, layer, T, T, 1, nullptr) == ZZ_OK);
          EXPECT(g_append_launches == 1);
          for (int b = 0; b < B; ++b) EXPECT(zz_set_seq_len(ctx, layer, b, zz_seq_len(ctx, layer, b) - 1) == ZZ_OK);
          const int b = (int)(rnd() % B);
          EXPECT(zz_attn_prefill_seq(ctx, layer, b, T, T, T, 512, T, nullptr) == ZZ_OK);
          EXPECT(zz_kv_append_seq(ctx, layer, b, T, T, 512, nullptr) == ZZ_OK);
          EXPECT(zz_seq_len(ctx, layer, b) == before[b] + 1 + 100 + 512);
          int64_t v = 0, c = 0;
          EXPECT(zz_prefill_tile_counts(ctx, layer, 512, &v, &c) == ZZ_OK && v > 0 && v <= c);
        }
      }
      EXPECT(zz_reset(ctx) == ZZ_OK);
      EXPECT(zz_destroy(ctx) == ZZ_OK);
    }
  // 3. offsets and slots at the edges of a large arena
  {
    zz_ctx *ctx = make(3, 16, 16, 64, 7, 1 << 20, 0, 1, 0, ZZ_MIXED, {}, std::vector<uint8_t>(3 * 16, 1));
    EXPECT(zz_kv_elem_offset(ctx, 2, 1, 6, 15, 0, 63) >= 0);
    EXPECT(zz_kv_elem_offset(ctx, 2, 1, 6, 15, 1, 0) == ZZ_ERANGE);   // S + W = 1 slot
    EXPECT(zz_destroy(ctx) == ZZ_OK);
    zz_config c;
    std::memset(&c, 0, sizeof(c));
    std::vector<uint8_t> lm = {0, 1};
    c.n_layers = 2; c.n_q_heads = 64; c.n_kv_heads = 64; c.head_dim = 128; c.batch = 65535; c.max_ctx = 1 << 30;
    c.sink = 1 << 29; c.window = 1 << 29; c.layout = ZZ_ZIGZAG; c.layer_is_streaming = lm.data();
    EXPECT(zz_arena_bytes(&c) > 0 && zz_workspace_bytes(&c) > 0);     // sizes computed in 64 bits
    EXPECT(zz_slot_of(&c, 1, 0, ((int64_t)1 << 30) - 1) == ((int64_t)1 << 29) + (((int64_t)1 << 29) - 1) % ((int64_t)1 << 29));
  }
  // 4. transport selection on random importances, all sparsities that give whole layer counts
  for (int L : {1, 2, 8, 32})
    for (int H : {1, 8}) {
      std::vector<float> alpha((size_t)L * H);
      for (auto &a : alpha) a = (rnd() >> 8) / 16777216.0f;
      std::vector<uint8_t> mask(L);
      for (int p = 0; p <= L; ++p) {
        double loss = 0;
        EXPECT(zz_transport_select(alpha.data(), L, H, (float)p / L, 0.1f, mask.data(), &loss) == ZZ_OK);
        int cnt = 0;
        for (auto m : mask) cnt += m;
        EXPECT(cnt == p);
      }
    }
  std::printf("launches recorded: %d, failures: %d\n", g_launches, g_fail);
  return g_fail ? 1 : 0;
}
