// Host runtime behind the C ABI in include/zz.h: config validation, arena layout,
// per-layer length tracking, slot arithmetic and launch planning.  Everything here
// is integer host code and runs without a GPU; only the zz_launch_* calls touch HIP.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "zz_internal.h"

namespace {

struct Group {
  int n_heads = 0;
  uint8_t heads[ZZ_MAX_KV_HEADS] = {0};
  int64_t capacity = 0;  // slots per (batch, head)
  int n_tiles = 0;       // ceil(capacity / 32)
  size_t base = 0;       // byte offset of the region in the arena
  bool streaming = false;
};

struct Layer {
  Group grp[2];  // 0: retrieval heads, 1: streaming heads
  uint8_t head_group[ZZ_MAX_KV_HEADS] = {0};
  uint8_t head_index[ZZ_MAX_KV_HEADS] = {0};
  std::vector<int64_t> len;  // tokens appended so far, per sequence

  bool uniform() const {
    for (int64_t v : len)
      if (v != len[0]) return false;
    return true;
  }
  int64_t longest() const {
    int64_t m = 0;
    for (int64_t v : len) m = v > m ? v : m;
    return m;
  }
};

struct Layout {
  std::vector<Layer> layers;
  size_t arena_bytes = 0;
  size_t ws_part_o = 0, ws_part_ml = 0, ws_counters = 0, ws_debug = 0, ws_stage = 0, ws_bytes = 0;
  int stage_tiles = 0;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t kv_tile_bytes(int D) { return (size_t)2 * ZZ_TILE_SLOTS * D * 2; }

int validate(const zz_config *c) {
  if (!c) return ZZ_EINVAL;
  if (c->n_layers < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->batch < 1 || c->max_ctx < 1) return ZZ_EINVAL;
  if (c->sink < 0 || c->window < 1 || c->max_chunk < 0) return ZZ_EINVAL;
  if (c->layout != ZZ_ZIGZAG && c->layout != ZZ_MIXED) return ZZ_EINVAL;
  if (!(c->softmax_scale >= 0.0f) || !std::isfinite(c->softmax_scale)) return ZZ_EINVAL;
  if (c->head_dim != 64 && c->head_dim != 128) return ZZ_EUNSUPPORTED;
  if (c->n_kv_heads > ZZ_MAX_KV_HEADS) return ZZ_EUNSUPPORTED;
  if (c->batch > 65535) return ZZ_EUNSUPPORTED;  // the batch index is a grid dimension
  if (c->n_q_heads % c->n_kv_heads != 0) return ZZ_EINVAL;
  if (c->n_q_heads / c->n_kv_heads > 16) return ZZ_EUNSUPPORTED;
  if ((int64_t)c->sink + c->window > (int64_t)1 << 30 || c->max_ctx > (1 << 30)) return ZZ_EUNSUPPORTED;
  if (c->layout == ZZ_ZIGZAG && !c->layer_is_streaming) return ZZ_ESTATE;
  if (c->layout == ZZ_MIXED && !c->kvhead_is_streaming) return ZZ_ESTATE;
  return ZZ_OK;
}

bool head_streams(const zz_config *c, int layer, int g) {
  if (c->layout == ZZ_ZIGZAG) return c->layer_is_streaming[layer] != 0;
  return c->kvhead_is_streaming[(size_t)layer * c->n_kv_heads + g] != 0;
}

// Lays out every layer's regions; assumes validate() passed.
void build_layout(const zz_config *c, Layout *lo) {
  const size_t tile = kv_tile_bytes(c->head_dim);
  lo->layers.assign(c->n_layers, Layer());
  size_t off = 0;
  for (int l = 0; l < c->n_layers; ++l) {
    Layer &L = lo->layers[l];
    L.len.assign(c->batch, 0);
    L.grp[0].streaming = false;
    L.grp[1].streaming = true;
    for (int g = 0; g < c->n_kv_heads; ++g) {
      Group &G = L.grp[head_streams(c, l, g) ? 1 : 0];
      L.head_group[g] = head_streams(c, l, g) ? 1 : 0;
      L.head_index[g] = (uint8_t)G.n_heads;
      G.heads[G.n_heads++] = (uint8_t)g;
    }
    for (int k = 0; k < 2; ++k) {
      Group &G = L.grp[k];
      G.capacity = k ? (int64_t)c->sink + c->window : (int64_t)c->max_ctx;
      G.n_tiles = (int)ceil_div(G.capacity, ZZ_TILE_SLOTS);
      G.base = off;
      off += (size_t)c->batch * G.n_heads * G.n_tiles * tile;
      off = align_up(off, 256);
    }
  }
  lo->arena_bytes = off;
  size_t w = 0;
  lo->ws_part_o = w;
  w += align_up((size_t)c->batch * c->n_q_heads * ZZ_MAX_SPLITS * c->head_dim * sizeof(float), 256);
  lo->ws_part_ml = w;
  w += align_up((size_t)c->batch * c->n_q_heads * ZZ_MAX_SPLITS * 2 * sizeof(float), 256);
  lo->ws_counters = w;
  w += align_up((size_t)c->batch * c->n_kv_heads * sizeof(int), 256);
  lo->ws_debug = w;   // one word, written only by a bounds-checking debug build
  w += 256;
  lo->ws_stage = w;
  lo->stage_tiles = (int)ceil_div(c->max_chunk, ZZ_TILE_SLOTS);
  // (two more tiles behind the last head's area: the prefill kernel requests tiles a fixed distance ahead
  // and its last requests, which nobody reads, may run that far past a head's staged chunk)
  w += align_up(((size_t)c->batch * c->n_kv_heads * lo->stage_tiles + 2) * tile, 256);
  lo->ws_bytes = w;
}

inline int64_t slot_rule(bool streaming, int64_t pos, int64_t S, int64_t W) {
  if (!streaming || pos < S) return pos;
  return S + (pos - S) % W;
}

}  // namespace

struct zz_ctx {
  zz_config cfg;
  std::vector<uint8_t> layer_mask, head_mask;
  Layout lo;
  char *arena = nullptr;
  char *ws = nullptr;
  float scale = 0.f;
  int num_cu = 0;          // 0: not queried yet
  // One workgroup (four waves, two 16 KiB tiles in flight each) per compute unit already
  // saturates HBM; more resident workgroups only lengthen the memory queues, and with
  // them the latency every workgroup pays for its first tile and for its merge.
  int tune_wg_per_cu = 1;
  int tune_splits = 0;
  int tune_prefill_pairing = 1;
  int tune_xcd_skew_permille = 50;   // measured best at 128k, batch 4 (0.870 -> 0.887 of the HBM peak)
  int tune_xcd_skew_min_tiles = 128; // shorter splits gain nothing (64 tiles) or lose (32)
  // The split counters live in caller memory that the library has never seen: every decode call
  // enqueues a small clear ahead of its attention launch until one such clear has been issued on
  // a stream that is not being captured (a clear recorded into a graph only runs when the graph
  // is replayed, so it does not count).  The merge re-arms a counter it has used.
  bool counters_zeroed = false;
  std::vector<int64_t> seen, tiles;  // per-sequence scratch of the decode call (sized at create: no heap work per call)
  const float *rope_cos = nullptr, *rope_sin = nullptr;   // caller's tables [rope_rows][D/2], or null: K is stored as given
  int64_t rope_rows = 0;
};

namespace {

// The group's region as the kernels see it, starting at sequence b0.
zz_group_dev dev_group(const zz_ctx *ctx, const Group &G, int b0 = 0) {
  zz_group_dev d;
  d.base = ctx->arena + G.base + (size_t)b0 * G.n_heads * G.n_tiles * kv_tile_bytes(ctx->cfg.head_dim);
  d.n_heads = G.n_heads;
  d.n_tiles = G.n_tiles;
  d.streaming = G.streaming ? 1 : 0;
  d.capacity = (int32_t)G.capacity;
  return d;
}

thread_local char g_detail[256] = "";

// Records what the HIP runtime said about a rejected launch and maps it to ZZ_EHIP.
int hip_failed(const char *what, hipError_t e) {
  std::snprintf(g_detail, sizeof(g_detail), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
  return ZZ_EHIP;
}

inline bool misaligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

int check_layer(const zz_ctx *ctx, int layer) {
  if (!ctx) return ZZ_EINVAL;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return ZZ_ERANGE;
  return ZZ_OK;
}

int64_t occupied(const zz_ctx *ctx, const Group &G, int64_t len) {
  return G.streaming ? (len < G.capacity ? len : G.capacity) : len;
}

int num_cu(zz_ctx *ctx) {
  if (ctx->num_cu <= 0) {
    int n = zz_query_num_cu();
    ctx->num_cu = n > 0 ? n : 256;
  }
  return ctx->num_cu;
}

// Split-K plan for one group: enough workgroups to fill the chip, at least one
// tile per wave of a workgroup, never more partials than the workspace holds.
// Tiles by which the ranges of two neighbouring splits differ (see decode_body): the configured fraction of
// a split, only for splits long enough for whole tiles to express it, and only if the last split, which may
// be shorter than the others, keeps at least one tile when it is the one that gives.
int decode_tile_skew(const zz_ctx *ctx, int n_tiles, int n_splits, int tps) {
  if (n_splits < 2 || ctx->tune_xcd_skew_permille <= 0 || tps < ctx->tune_xcd_skew_min_tiles) return 0;
  const int skew = (int)(((int64_t)tps * ctx->tune_xcd_skew_permille + 500) / 1000);
  const int last = n_tiles - (n_splits - 1) * tps;
  return (skew > 0 && last > skew) ? skew : 0;
}

void plan_decode(const zz_ctx *ctx, int cu, const Group &G, int64_t len, int *n_splits, int *tiles_per_split) {
  const int64_t n_valid = occupied(ctx, G, len);
  const int64_t n_tiles = ceil_div(n_valid, ZZ_TILE_SLOTS);
  if (G.n_heads == 0 || n_tiles == 0) {
    *n_splits = 0;
    *tiles_per_split = 0;
    return;
  }
  const int64_t units = (int64_t)ctx->cfg.batch * G.n_heads;
  int64_t splits = ctx->tune_splits > 0 ? ctx->tune_splits : ceil_div((int64_t)cu * ctx->tune_wg_per_cu, units);
  if (splits < 1) splits = 1;
  int64_t tps = ceil_div(n_tiles, splits);
  // A short cache (a streaming head's S+W slots) is latency-bound either way: one workgroup
  // per unit needs no cross-workgroup merge, which costs more than a few extra tiles per wave.
  if (n_tiles <= 4 * ZZ_WAVES_PER_WG && ctx->tune_splits <= 0) tps = n_tiles;
  if (tps < ZZ_WAVES_PER_WG && ctx->tune_splits <= 0) tps = ZZ_WAVES_PER_WG;
  if (tps > n_tiles) tps = n_tiles;
  splits = ceil_div(n_tiles, tps);
  if (splits > ZZ_MAX_SPLITS) {
    tps = ceil_div(n_tiles, ZZ_MAX_SPLITS);
    splits = ceil_div(n_tiles, tps);
  }
  *n_splits = (int)splits;
  *tiles_per_split = (int)tps;
}

// Split-K plan for sequences of different lengths (len[b]: tokens the attention of sequence
// b sees).  One tiles-per-split value for the whole launch; sequence b gets
// ceil(tiles_b / tps) workgroups per head.  The kernel runs one workgroup per compute unit,
// so a launch with more workgroups than the chip holds would pay a second round for a few
// stragglers: tps is the smallest value whose workgroups fit in one round (if the batch
// allows it at all), which also equalises the work per workgroup as far as whole tiles can.
// Returns the workgroups per head; first_wg[0..B] are the prefix sums.
int plan_decode_ragged(const zz_ctx *ctx, int cu, const Group &G, const int64_t *len, int64_t *tiles, uint16_t *first_wg,
                       int *tiles_per_split) {
  const int B = ctx->cfg.batch;
  int64_t total = 0, longest = 0;
  for (int b = 0; b < B; ++b) {
    tiles[b] = ceil_div(occupied(ctx, G, len[b]), ZZ_TILE_SLOTS);
    total += tiles[b];
    longest = tiles[b] > longest ? tiles[b] : longest;
  }
  auto wgs = [&](int64_t tps) {
    int64_t n = 0;
    for (int b = 0; b < B; ++b) n += ceil_div(tiles[b], tps);
    return n;
  };
  int64_t tps;
  if (ctx->tune_splits > 0) {
    tps = ceil_div(longest, ctx->tune_splits);
  } else {
    int64_t room = (int64_t)cu * ctx->tune_wg_per_cu / G.n_heads;  // workgroups per head in one round
    if (room < B) room = B;                                         // every sequence needs one anyway
    int64_t lo = ceil_div(total, room), hi = longest;               // wgs(hi) == B <= room
    if (lo < 4 * ZZ_WAVES_PER_WG) lo = 4 * ZZ_WAVES_PER_WG;         // short caches stay unsplit, as in plan_decode
    if (hi < lo) hi = lo;
    while (lo < hi) {
      const int64_t mid = (lo + hi) / 2;
      if (wgs(mid) <= room) hi = mid; else lo = mid + 1;
    }
    tps = lo;
  }
  if (tps < 1) tps = 1;
  if (ceil_div(longest, tps) > ZZ_MAX_SPLITS) tps = ceil_div(longest, ZZ_MAX_SPLITS);
  first_wg[0] = 0;
  for (int b = 0; b < B; ++b) first_wg[b + 1] = (uint16_t)(first_wg[b] + ceil_div(tiles[b], tps));
  *tiles_per_split = (int)tps;
  return first_wg[B];
}

}  // namespace

extern "C" {

size_t zz_arena_bytes(const zz_config *cfg) {
  if (validate(cfg) != ZZ_OK) return 0;
  Layout lo;
  build_layout(cfg, &lo);
  return lo.arena_bytes;
}

size_t zz_workspace_bytes(const zz_config *cfg) {
  if (validate(cfg) != ZZ_OK) return 0;
  Layout lo;
  build_layout(cfg, &lo);
  return lo.ws_bytes;
}

int zz_create(const zz_config *cfg, void *kv_arena, size_t arena_bytes, void *workspace, size_t workspace_bytes,
              zz_ctx **out) {
  if (!out) return ZZ_EINVAL;
  *out = nullptr;
  int rc = validate(cfg);
  if (rc != ZZ_OK) return rc;
  if (!kv_arena || !workspace) return ZZ_EINVAL;
  if (misaligned(kv_arena, 256) || misaligned(workspace, 256)) return ZZ_EALIGN;
  zz_ctx *ctx = new (std::nothrow) zz_ctx();
  if (!ctx) return ZZ_ENOSPC;
  ctx->cfg = *cfg;
  if (cfg->layout == ZZ_ZIGZAG) {
    ctx->layer_mask.assign(cfg->layer_is_streaming, cfg->layer_is_streaming + cfg->n_layers);
    ctx->cfg.layer_is_streaming = ctx->layer_mask.data();
    ctx->cfg.kvhead_is_streaming = nullptr;
  } else {
    ctx->head_mask.assign(cfg->kvhead_is_streaming,
                          cfg->kvhead_is_streaming + (size_t)cfg->n_layers * cfg->n_kv_heads);
    ctx->cfg.kvhead_is_streaming = ctx->head_mask.data();
    ctx->cfg.layer_is_streaming = nullptr;
  }
  build_layout(&ctx->cfg, &ctx->lo);
  if (arena_bytes < ctx->lo.arena_bytes || workspace_bytes < ctx->lo.ws_bytes) {
    delete ctx;
    return ZZ_ENOSPC;
  }
  ctx->arena = (char *)kv_arena;
  ctx->ws = (char *)workspace;
  ctx->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  ctx->seen.assign(cfg->batch, 0);
  ctx->tiles.assign(cfg->batch, 0);
  *out = ctx;
  return ZZ_OK;
}

int zz_destroy(zz_ctx *ctx) {
  if (!ctx) return ZZ_EINVAL;
  delete ctx;
  return ZZ_OK;
}

int zz_reset(zz_ctx *ctx) {
  if (!ctx) return ZZ_EINVAL;
  for (auto &L : ctx->lo.layers) L.len.assign(ctx->cfg.batch, 0);
  return ZZ_OK;
}

int64_t zz_layer_len(const zz_ctx *ctx, int layer) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  return ctx->lo.layers[layer].longest();
}

int zz_set_layer_len(zz_ctx *ctx, int layer, int64_t len) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  if (len < 0 || len > ctx->cfg.max_ctx) return ZZ_ERANGE;
  ctx->lo.layers[layer].len.assign(ctx->cfg.batch, len);
  return ZZ_OK;
}

int64_t zz_seq_len(const zz_ctx *ctx, int layer, int b) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  if (b < 0 || b >= ctx->cfg.batch) return ZZ_ERANGE;
  return ctx->lo.layers[layer].len[b];
}

int zz_set_seq_len(zz_ctx *ctx, int layer, int b, int64_t len) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  if (b < 0 || b >= ctx->cfg.batch || len < 0 || len > ctx->cfg.max_ctx) return ZZ_ERANGE;
  ctx->lo.layers[layer].len[b] = len;
  return ZZ_OK;
}

int zz_set_rope_tables(zz_ctx *ctx, const float *cos_table, const float *sin_table, int64_t rows) {
  if (!ctx) return ZZ_EINVAL;
  if (!cos_table && !sin_table && rows == 0) {
    ctx->rope_cos = ctx->rope_sin = nullptr;
    ctx->rope_rows = 0;
    return ZZ_OK;
  }
  if (!cos_table || !sin_table || rows < 1) return ZZ_EINVAL;
  if (misaligned(cos_table, 16) || misaligned(sin_table, 16)) return ZZ_EALIGN;
  ctx->rope_cos = cos_table;
  ctx->rope_sin = sin_table;
  ctx->rope_rows = rows;
  return ZZ_OK;
}

int zz_layer_launches(const zz_ctx *ctx, int layer) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  const Layer &L = ctx->lo.layers[layer];
  return (L.grp[0].n_heads > 0) + (L.grp[1].n_heads > 0);
}

int64_t zz_slot_of(const zz_config *cfg, int layer, int kv_head, int64_t pos) {
  int rc = validate(cfg);
  if (rc != ZZ_OK) return rc;
  if (layer < 0 || layer >= cfg->n_layers || kv_head < 0 || kv_head >= cfg->n_kv_heads || pos < 0) return ZZ_ERANGE;
  const bool st = head_streams(cfg, layer, kv_head);
  if (!st && pos >= cfg->max_ctx) return ZZ_ERANGE;
  return slot_rule(st, pos, cfg->sink, cfg->window);
}

int64_t zz_kv_elem_offset(const zz_ctx *ctx, int layer, int which, int b, int kv_head, int64_t slot, int d) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  const zz_config &c = ctx->cfg;
  if (which < 0 || which > 1) return ZZ_EINVAL;
  if (b < 0 || b >= c.batch || kv_head < 0 || kv_head >= c.n_kv_heads || d < 0 || d >= c.head_dim) return ZZ_ERANGE;
  const Layer &L = ctx->lo.layers[layer];
  const Group &G = L.grp[L.head_group[kv_head]];
  if (slot < 0 || slot >= G.capacity) return ZZ_ERANGE;
  const int64_t D = c.head_dim;
  const int64_t tile = slot / ZZ_TILE_SLOTS, t = slot % ZZ_TILE_SLOTS;
  int64_t elem;
  if (which == 0)
    elem = (((t / 16) * (D / 8) + d / 8) * 16 + t % 16) * 8 + d % 8;
  else
    elem = ((((int64_t)(d / 16) * 4 + (t % 16) / 4) * 16 + d % 16) * 8 + 4 * (t / 16) + t % 4) + 32 * D;
  const int64_t tile_index = ((int64_t)b * G.n_heads + L.head_index[kv_head]) * G.n_tiles + tile;
  return (int64_t)G.base + tile_index * (int64_t)kv_tile_bytes(c.head_dim) + elem * 2;
}

size_t zz_debug_word_offset(const zz_config *cfg) {
  if (validate(cfg) != ZZ_OK) return 0;
  Layout lo;
  build_layout(cfg, &lo);
  return lo.ws_debug;
}

int zz_is_debug_build(void) {
#ifdef ZZ_DEBUG_BOUNDS
  return 1;
#else
  return 0;
#endif
}

int zz_tune(zz_ctx *ctx, int key, int value) {
  if (!ctx) return ZZ_EINVAL;
  switch (key) {
    case ZZ_TUNE_DECODE_WG_PER_CU:
      if (value < 1 || value > 64) return ZZ_ERANGE;
      ctx->tune_wg_per_cu = value;
      return ZZ_OK;
    case ZZ_TUNE_DECODE_SPLITS:
      if (value < 0 || value > ZZ_MAX_SPLITS) return ZZ_ERANGE;
      ctx->tune_splits = value;
      return ZZ_OK;
    case ZZ_TUNE_NUM_CU:
      if (value < 1 || value > 4096) return ZZ_ERANGE;
      ctx->num_cu = value;
      return ZZ_OK;
    case ZZ_TUNE_DECODE_XCD_SKEW:
      if (value < 0 || value > 200) return ZZ_ERANGE;
      ctx->tune_xcd_skew_permille = value;
      ctx->tune_xcd_skew_min_tiles = 1;   // an explicit setting applies to splits of any length
      return ZZ_OK;
    case ZZ_TUNE_PREFILL_PAIRING:
      if (value < 0 || value > 2) return ZZ_ERANGE;
      ctx->tune_prefill_pairing = value;
      return ZZ_OK;
    default:
      return ZZ_EINVAL;
  }
}

int zz_decode_plan(const zz_ctx *ctx, int layer, int group, int *n_splits, int *tiles_per_split) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  if (group < 0 || group > 1 || !n_splits || !tiles_per_split) return ZZ_EINVAL;
  const Layer &L = ctx->lo.layers[layer];
  const int cu = num_cu(const_cast<zz_ctx *>(ctx));
  if (L.uniform()) {
    plan_decode(ctx, cu, L.grp[group], L.len[0], n_splits, tiles_per_split);
    return ZZ_OK;
  }
  *n_splits = *tiles_per_split = 0;
  if (L.grp[group].n_heads == 0) return ZZ_OK;
  if (ctx->cfg.batch > ZZ_MAX_RAGGED_BATCH) return ZZ_EUNSUPPORTED;
  uint16_t first_wg[ZZ_MAX_RAGGED_BATCH + 1];
  std::vector<int64_t> tiles(ctx->cfg.batch);
  plan_decode_ragged(ctx, cu, L.grp[group], L.len.data(), tiles.data(), first_wg, tiles_per_split);
  for (int b = 0; b < ctx->cfg.batch; ++b)
    if (first_wg[b + 1] - first_wg[b] > *n_splits) *n_splits = first_wg[b + 1] - first_wg[b];
  return ZZ_OK;
}

namespace {

// The lengths of sequences [b0, b0 + nb) of a layer as a launch takes them: one common value,
// or the per-sequence table (at most ZZ_MAX_RAGGED_BATCH sequences).
void fill_lens(const Layer &L, int b0, int nb, bool ragged, zz_seq_lens *out) {
  out->ragged = ragged ? 1u : 0u;
  if (ragged)
    for (int b = 0; b < nb; ++b) out->len[b] = (uint32_t)L.len[b0 + b];
}

// Appends n_new tokens to sequences [b0, b0 + nb) of the layer, which share the length
// `len` (ragged: each at its own length, one launch all the same); k_new, v_new point at the
// rows of sequence b0.
int append_run(zz_ctx *ctx, Layer &L, int b0, int nb, int64_t len, const void *k_new, const void *v_new, int n_new,
               void *stream, bool ragged = false) {
  const zz_config &c = ctx->cfg;
  zz_append_params p;
  std::memset(&p, 0, sizeof(p));
  p.k_new = k_new;
  p.v_new = v_new;
  p.grp[0] = dev_group(ctx, L.grp[0], b0);
  p.grp[1] = dev_group(ctx, L.grp[1], b0);
  std::memcpy(p.head_group, L.head_group, sizeof(p.head_group));
  std::memcpy(p.head_index, L.head_index, sizeof(p.head_index));
  p.len = len;
  p.n_new = n_new;
  p.batch = nb;
  p.n_kv_heads = c.n_kv_heads;
  p.head_dim = c.head_dim;
  p.sink = c.sink;
  p.window = c.window;
  p.only_group = -1;
  p.debug_word = (uint32_t *)(ctx->ws + ctx->lo.ws_debug);
  p.rope_cos = ctx->rope_cos;
  p.rope_sin = ctx->rope_sin;
  zz_seq_lens lens;
  fill_lens(L, b0, nb, ragged, &lens);
  if (hipError_t e = zz_launch_append(p, lens, (hipStream_t)stream)) return hip_failed("append kernel", e);
  return ZZ_OK;
}

// Attention of n_new new positions for sequences [b0, b0 + nb), which share the length
// n_past (ragged: each at its own length); all four tensors point at the rows of sequence b0.
int prefill_run(zz_ctx *ctx, const Layer &L, int b0, int nb, int64_t n_past, const void *q, const void *k_new,
                const void *v_new, int n_new, void *out, void *stream, bool ragged = false) {
  const zz_config &c = ctx->cfg;
  zz_stage_params sp;
  std::memset(&sp, 0, sizeof(sp));
  sp.k_new = k_new;
  sp.v_new = v_new;
  sp.stage_tiles = ctx->lo.stage_tiles;
  sp.stage = ctx->ws + ctx->lo.ws_stage + (size_t)b0 * c.n_kv_heads * sp.stage_tiles * kv_tile_bytes(c.head_dim);
  sp.n_new = n_new;
  sp.batch = nb;
  sp.n_kv_heads = c.n_kv_heads;
  sp.head_dim = c.head_dim;
  sp.debug_word = (uint32_t *)(ctx->ws + ctx->lo.ws_debug);
  sp.rope_cos = ctx->rope_cos;
  sp.rope_sin = ctx->rope_sin;
  sp.n_past = n_past;
  zz_seq_lens lens;
  fill_lens(L, b0, nb, ragged, &lens);
  if (hipError_t e = zz_launch_stage(sp, lens, (hipStream_t)stream)) return hip_failed("staging kernel", e);
  for (int k = 0; k < 2; ++k) {
    const Group &G = L.grp[k];
    if (G.n_heads == 0) continue;
    zz_prefill_params p;
    std::memset(&p, 0, sizeof(p));
    p.grp = dev_group(ctx, G, b0);
    std::memcpy(p.heads, G.heads, sizeof(p.heads));
    p.q = q;
    p.out = out;
    p.stage = sp.stage;
    p.stage_tiles = sp.stage_tiles;
    p.n_past = (int)n_past;
    p.n_new = n_new;
    p.batch = nb;
    p.n_q_heads = c.n_q_heads;
    p.n_kv_heads = c.n_kv_heads;
    p.head_dim = c.head_dim;
    p.group_size = c.n_q_heads / c.n_kv_heads;
    p.sink = c.sink;
    p.window = c.window;
    p.scale_log2e = ctx->scale * 1.4426950408889634f;
    if (hipError_t e = zz_launch_prefill(p, lens, ctx->tune_prefill_pairing == 0 ? -1 : ctx->tune_prefill_pairing == 2 ? 0 : num_cu(ctx), (hipStream_t)stream)) return hip_failed("prefill kernel", e);
  }
  return ZZ_OK;
}

inline const void *rows_of(const void *base, int b, int n_new, int heads, int D) {
  return base ? (const char *)base + (size_t)b * n_new * heads * D * 2 : nullptr;
}

int check_chunk(const zz_ctx *ctx, int layer, const void *k_new, const void *v_new, int n_new) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  if (n_new < 0) return ZZ_ERANGE;
  if (n_new == 0) return ZZ_OK;
  if (!k_new || !v_new) return ZZ_EINVAL;
  if (misaligned(k_new, 16) || misaligned(v_new, 16)) return ZZ_EALIGN;
  return ZZ_OK;
}

}  // namespace

int zz_kv_append(zz_ctx *ctx, int layer, const void *k_new, const void *v_new, int n_new, void *stream) {
  int rc = check_chunk(ctx, layer, k_new, v_new, n_new);
  if (rc != ZZ_OK || n_new == 0) return rc;
  Layer &L = ctx->lo.layers[layer];
  const zz_config &c = ctx->cfg;
  if (L.longest() + n_new > c.max_ctx) return ZZ_ENOSPC;  // the length counter itself is bounded by max_ctx
  if (ctx->rope_cos && L.longest() + n_new > ctx->rope_rows) return ZZ_ERANGE;
  if (L.uniform()) {
    rc = append_run(ctx, L, 0, c.batch, L.len[0], k_new, v_new, n_new, stream);
    if (rc != ZZ_OK) return rc;
  } else if (c.batch <= ZZ_MAX_RAGGED_BATCH) {
    rc = append_run(ctx, L, 0, c.batch, 0, k_new, v_new, n_new, stream, true);   // one launch, lengths in its arguments
    if (rc != ZZ_OK) return rc;
  } else {
    for (int b = 0; b < c.batch; ++b) {
      rc = append_run(ctx, L, b, 1, L.len[b], rows_of(k_new, b, n_new, c.n_kv_heads, c.head_dim),
                      rows_of(v_new, b, n_new, c.n_kv_heads, c.head_dim), n_new, stream);
      if (rc != ZZ_OK) return rc;  // launches already issued only wrote slots past the unchanged lengths
    }
  }
  for (auto &v : L.len) v += n_new;
  return ZZ_OK;
}

int zz_kv_append_seq(zz_ctx *ctx, int layer, int b, const void *k_new, const void *v_new, int n_new, void *stream) {
  int rc = check_chunk(ctx, layer, k_new, v_new, n_new);
  if (rc != ZZ_OK) return rc;
  if (b < 0 || b >= ctx->cfg.batch) return ZZ_ERANGE;
  if (n_new == 0) return ZZ_OK;
  Layer &L = ctx->lo.layers[layer];
  if (L.len[b] + n_new > ctx->cfg.max_ctx) return ZZ_ENOSPC;
  if (ctx->rope_cos && L.len[b] + n_new > ctx->rope_rows) return ZZ_ERANGE;
  rc = append_run(ctx, L, b, 1, L.len[b], k_new, v_new, n_new, stream);
  if (rc != ZZ_OK) return rc;
  L.len[b] += n_new;
  return ZZ_OK;
}

// Shared by zz_attn_decode (k_new == nullptr: the newest token is already cached) and
// zz_decode_step (the newest token is appended by the attention launch itself).
static int decode_impl(zz_ctx *ctx, int layer, const void *q, const void *k_new, const void *v_new, void *out,
                       void *stream, bool static_scratch = false) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  const bool fused = k_new != nullptr || v_new != nullptr;
  if (!q || !out || (fused && (!k_new || !v_new))) return ZZ_EINVAL;
  if (misaligned(q, 16) || misaligned(out, 16) || misaligned(k_new, 16) || misaligned(v_new, 16)) return ZZ_EALIGN;
  Layer &L = ctx->lo.layers[layer];
  const zz_config &c = ctx->cfg;
  const int64_t add = fused ? 1 : 0;
  // one pass over the lengths: equal or not, longest, shortest
  const int64_t len0 = L.len[0];
  int64_t longest = len0, shortest = len0;
  for (int b = 1; b < c.batch; ++b) {
    const int64_t v = L.len[b];
    longest = v > longest ? v : longest;
    shortest = v < shortest ? v : shortest;
  }
  const bool uniform = longest == shortest;
  if (fused && longest + 1 > c.max_ctx) return ZZ_ENOSPC;
  if (fused && ctx->rope_cos && longest + 1 > ctx->rope_rows) return ZZ_ERANGE;
  if (shortest + add <= 0) return ZZ_ESTATE;
  if (!uniform && c.batch > ZZ_MAX_RAGGED_BATCH) return ZZ_EUNSUPPORTED;
  const int cu = num_cu(ctx);
  int *counters = (int *)(ctx->ws + ctx->lo.ws_counters);
  float *part_ml = (float *)(ctx->ws + ctx->lo.ws_part_ml), *part_o = (float *)(ctx->ws + ctx->lo.ws_part_o);
  if (static_scratch) {
    // the library's own array instead of the workspace: [counters | (max, sum) pairs | partial outputs]
    const int64_t units = (int64_t)c.batch * c.n_kv_heads, elems = (int64_t)c.batch * c.n_q_heads * c.head_dim;
    if (units > ZZ_STATIC_MAX_UNITS || elems > ZZ_STATIC_MAX_ROW_ELEMS) {
      std::snprintf(g_detail, sizeof(g_detail),
                    "zz_attn_decode_static: batch*n_kv_heads = %lld (limit %d), batch*n_q_heads*head_dim = %lld (limit %d)",
                    (long long)units, ZZ_STATIC_MAX_UNITS, (long long)elems, ZZ_STATIC_MAX_ROW_ELEMS);
      return ZZ_ENOSPC;
    }
    char *base = nullptr;
    if (hipError_t e = zz_static_scratch(&base)) return hip_failed("address of the static scratch array", e);
    constexpr size_t counters_bytes = (size_t)ZZ_STATIC_MAX_UNITS * sizeof(int);
    constexpr size_t ml_bytes = (size_t)(ZZ_STATIC_MAX_ROW_ELEMS / 64) * ZZ_MAX_SPLITS * 2 * sizeof(float);  // head_dim >= 64
    constexpr size_t o_bytes = (size_t)ZZ_STATIC_MAX_ROW_ELEMS * ZZ_MAX_SPLITS * sizeof(float);
    static_assert(counters_bytes + ml_bytes + o_bytes == ZZ_STATIC_SCRATCH_BYTES, "regions fill the static array exactly");
    counters = (int *)base;
    part_ml = (float *)(base + counters_bytes);
    part_o = (float *)(base + counters_bytes + ml_bytes);
    // shared by every context and call on this GPU: cleared every time
    if (hipError_t e = zz_launch_zero(counters, c.batch * c.n_kv_heads, (hipStream_t)stream))
      return hip_failed("counter clear kernel", e);
  } else if (!ctx->counters_zeroed) {
    const bool capturing = zz_stream_is_capturing((hipStream_t)stream);
    if (hipError_t e = zz_launch_zero(counters, c.batch * c.n_kv_heads, (hipStream_t)stream))
      return hip_failed("counter clear kernel", e);
    ctx->counters_zeroed = !capturing;
  }
  for (int k = 0; k < 2; ++k) {
    const Group &G = L.grp[k];
    if (G.n_heads == 0) continue;
    // everything both launch forms share; the per-sequence form embeds it
    auto fill = [&](zz_decode_params &p) {
      p.tile_skew = 0;
      p.grp = dev_group(ctx, G);
      std::memcpy(p.heads, G.heads, sizeof(p.heads));
      p.q = q;
      p.out = out;
      p.part_o = part_o;
      p.part_ml = part_ml;
      p.counters = counters;
      p.k_new = k_new;
      p.v_new = v_new;
      p.batch = c.batch;
      p.n_q_heads = c.n_q_heads;
      p.n_kv_heads = c.n_kv_heads;
      p.head_dim = c.head_dim;
      p.group_size = c.n_q_heads / c.n_kv_heads;
      p.scale_log2e = ctx->scale * 1.4426950408889634f;
      p.debug_word = (uint32_t *)(ctx->ws + ctx->lo.ws_debug);
      p.rope_cos = fused ? ctx->rope_cos : nullptr;
      p.rope_sin = fused ? ctx->rope_sin : nullptr;
      p.new_pos = 0;
    };
    if (uniform) {
      zz_decode_params p;
      fill(p);
      const int64_t len = len0 + add;
      p.new_slot = fused ? (int32_t)slot_rule(G.streaming, len - 1, c.sink, c.window) : -1;
      p.new_pos = (int32_t)(len - 1);
      p.n_valid = (int)occupied(ctx, G, len);
      p.n_tiles_valid = (int)ceil_div(p.n_valid, ZZ_TILE_SLOTS);
      plan_decode(ctx, cu, G, len, &p.n_splits, &p.tiles_per_split);
      p.tile_skew = decode_tile_skew(ctx, p.n_tiles_valid, p.n_splits, p.tiles_per_split);
      if (hipError_t e = zz_launch_decode(p, (hipStream_t)stream)) return hip_failed("decode kernel", e);
    } else {
      zz_decode_ragged_params rp;
      fill(rp.u);
      zz_decode_params &p = rp.u;
      p.new_slot = fused ? 0 : -1;  // only the sign is read: each sequence's slot follows from its length
      p.n_valid = p.n_tiles_valid = p.n_splits = 0;
      rp.sink = c.sink;
      rp.window = c.window;
      for (int b = 0; b < c.batch; ++b) {
        ctx->seen[b] = L.len[b] + add;
        rp.seq_len[b] = (uint32_t)ctx->seen[b];
      }
      const int total_wg =
          plan_decode_ragged(ctx, cu, G, ctx->seen.data(), ctx->tiles.data(), rp.first_wg, &p.tiles_per_split);
      if (hipError_t e = zz_launch_decode_ragged(rp, total_wg, (hipStream_t)stream))
        return hip_failed("decode kernel (per-sequence lengths)", e);
    }
  }
  if (fused)
    for (auto &v : L.len) v += 1;
  return ZZ_OK;
}

int zz_attn_decode(zz_ctx *ctx, int layer, const void *q, void *out, void *stream) {
  return decode_impl(ctx, layer, q, nullptr, nullptr, out, stream);
}

int zz_attn_decode_static(zz_ctx *ctx, int layer, const void *q, void *out, void *stream) {
  return decode_impl(ctx, layer, q, nullptr, nullptr, out, stream, true);
}

int zz_decode_step(zz_ctx *ctx, int layer, const void *q, const void *k_new, const void *v_new, void *out,
                   void *stream) {
  if (!k_new || !v_new) return ZZ_EINVAL;
  return decode_impl(ctx, layer, q, k_new, v_new, out, stream);
}

static int check_prefill(const zz_ctx *ctx, int layer, const void *q, const void *k_new, const void *v_new, int n_new,
                         const void *out) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  if (n_new < 0) return ZZ_ERANGE;
  if (n_new == 0) return ZZ_OK;
  if (!q || !k_new || !v_new || !out) return ZZ_EINVAL;
  if (misaligned(q, 16) || misaligned(k_new, 16) || misaligned(v_new, 16) || misaligned(out, 16)) return ZZ_EALIGN;
  if (n_new > ctx->cfg.max_chunk) return ZZ_ERANGE;
  return ZZ_OK;
}

int zz_attn_prefill(zz_ctx *ctx, int layer, const void *q, const void *k_new, const void *v_new, int n_new,
                    void *out, void *stream) {
  int rc = check_prefill(ctx, layer, q, k_new, v_new, n_new, out);
  if (rc != ZZ_OK || n_new == 0) return rc;
  const zz_config &c = ctx->cfg;
  const Layer &L = ctx->lo.layers[layer];
  if (L.longest() + n_new > c.max_ctx) return ZZ_ENOSPC;
  if (ctx->rope_cos && L.longest() + n_new > ctx->rope_rows) return ZZ_ERANGE;
  if (L.uniform()) return prefill_run(ctx, L, 0, c.batch, L.len[0], q, k_new, v_new, n_new, out, stream);
  if (c.batch <= ZZ_MAX_RAGGED_BATCH) return prefill_run(ctx, L, 0, c.batch, 0, q, k_new, v_new, n_new, out, stream, true);
  for (int b = 0; b < c.batch; ++b) {
    rc = prefill_run(ctx, L, b, 1, L.len[b], rows_of(q, b, n_new, c.n_q_heads, c.head_dim),
                     rows_of(k_new, b, n_new, c.n_kv_heads, c.head_dim),
                     rows_of(v_new, b, n_new, c.n_kv_heads, c.head_dim), n_new,
                     (void *)rows_of(out, b, n_new, c.n_q_heads, c.head_dim), stream);
    if (rc != ZZ_OK) return rc;
  }
  return ZZ_OK;
}

int zz_attn_prefill_seq(zz_ctx *ctx, int layer, int b, const void *q, const void *k_new, const void *v_new, int n_new,
                        void *out, void *stream) {
  int rc = check_prefill(ctx, layer, q, k_new, v_new, n_new, out);
  if (rc != ZZ_OK) return rc;
  if (b < 0 || b >= ctx->cfg.batch) return ZZ_ERANGE;
  if (n_new == 0) return ZZ_OK;
  const Layer &L = ctx->lo.layers[layer];
  if (L.len[b] + n_new > ctx->cfg.max_ctx) return ZZ_ENOSPC;
  if (ctx->rope_cos && L.len[b] + n_new > ctx->rope_rows) return ZZ_ERANGE;
  return prefill_run(ctx, L, b, 1, L.len[b], q, k_new, v_new, n_new, out, stream);
}

int zz_prefill_tile_counts(const zz_ctx *ctx, int layer, int n_new, int64_t *visited, int64_t *causal) {
  int rc = check_layer(ctx, layer);
  if (rc != ZZ_OK) return rc;
  if (!visited || !causal) return ZZ_EINVAL;
  const zz_config &c = ctx->cfg;
  if (n_new < 1 || n_new > c.max_chunk) return ZZ_ERANGE;
  const Layer &L = ctx->lo.layers[layer];
  const int64_t S = c.sink, W = c.window;
  const int G = c.n_q_heads / c.n_kv_heads;
  const int Gc = zz_prefill_heads_per_wave(G);
  const int QB = ZZ_WAVES_PER_WG * 16 * (ZZ_PREFILL_NB / Gc);  // query positions per workgroup, as the launcher chooses
  int64_t vis = 0, cau = 0;
  for (int b = 0; b < c.batch; ++b) {
    const int64_t n_past = L.len[b];
    for (int k = 0; k < 2; ++k) {
      const Group &Gr = L.grp[k];
      if (Gr.n_heads == 0) continue;
      const int64_t wgs_per_range = (int64_t)Gr.n_heads * (G / Gc);
      const int64_t n_ct = ceil_div(occupied(ctx, Gr, n_past), ZZ_TILE_SLOTS);  // every occupied cached tile is read
      for (int64_t iq0 = 0; iq0 < n_new; iq0 += QB) {
        const int64_t iq_last = (iq0 + QB < n_new ? iq0 + QB : n_new) - 1;
        const int64_t I_lo = n_past + iq0, k_hi = iq_last / ZZ_TILE_SLOTS;
        // the causal lower triangle at this granularity: every cached position plus staged tiles up to the diagonal
        const int64_t all = ceil_div(n_past, ZZ_TILE_SLOTS) + k_hi + 1;
        int64_t ks_end = 0, kw_begin = 0;
        if (Gr.streaming) {
          if (n_past < S) {
            const int64_t e = (S - 1 - n_past) / ZZ_TILE_SLOTS;
            ks_end = (e < k_hi ? e : k_hi) + 1;
          }
          const int64_t first_win = I_lo - W + 1 - n_past;
          kw_begin = first_win > 0 ? first_win / ZZ_TILE_SLOTS : 0;
          if (kw_begin < ks_end) kw_begin = ks_end;
        }
        const int64_t v = n_ct + ks_end + (k_hi >= kw_begin ? k_hi - kw_begin + 1 : 0);
        vis += v * wgs_per_range;
        cau += all * wgs_per_range;
      }
    }
  }
  *visited = vis;
  *causal = cau;
  return ZZ_OK;
}

int zz_probe_read(zz_ctx *ctx, const void *buf, size_t bytes, int nontemporal, void *stream) {
  if (!ctx || !buf) return ZZ_EINVAL;
  if (misaligned(buf, 16)) return ZZ_EALIGN;
  if (bytes < 16 * 1024) return ZZ_ERANGE;
  // the 4 KiB the kernel may (never, in practice) write to is the start of the split-K partials
  if (hipError_t e = zz_launch_probe_read(buf, bytes, nontemporal, num_cu(ctx), ctx->ws + ctx->lo.ws_part_o,
                                          (hipStream_t)stream))
    return hip_failed("read probe kernel", e);
  return ZZ_OK;
}

const char *zz_last_error_detail(void) { return g_detail; }

const char *zz_strerror(int code) {
  switch (code) {
    case ZZ_OK: return "ok";
    case ZZ_EINVAL: return "invalid argument (null pointer, non-positive size or unknown enum)";
    case ZZ_ERANGE: return "layer, head, position or token count out of range";
    case ZZ_ENOSPC: return "no space: append past max_ctx, arena/workspace too small, or shape beyond the static scratch";
    case ZZ_EALIGN: return "pointer not aligned (tensors 16 bytes, arena and workspace 256 bytes)";
    case ZZ_ESTATE: return "wrong state: empty layer, or the mask for the chosen layout is missing";
    case ZZ_EUNSUPPORTED: return "unsupported shape (head_dim must be 64 or 128, Hq/Hkv <= 16, Hkv <= 64)";
    case ZZ_EHIP: return "the HIP runtime rejected a kernel launch";
    default: return "unknown error code";
  }
}

}  // extern "C"
