// Internal interface between the host runtime (zz_api.cpp) and the gfx950 kernels
// (zz_kernels.hip).  Plain structs passed by value as kernel arguments: the library
// owns no device memory, so per-launch tables (head lists) travel in the argument
// buffer instead.
#ifndef ZZ_INTERNAL_H
#define ZZ_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "zz.h"

#define ZZ_WAVES_PER_WG 4

// Prefill tiling, shared by the launcher and by the host-side tile counter: a wave owns
// ZZ_PREFILL_NB column blocks of 16 query positions, spread over Gc heads of the KV group.
#define ZZ_PREFILL_NB 2
#define ZZ_PREFILL_WG_PER_CU 2
static inline int zz_prefill_heads_per_wave(int group_size) {
  int gc = ZZ_PREFILL_NB;
  while (gc > 1 && group_size % gc != 0) gc >>= 1;
  return gc;
}

// One head group of a layer: the heads of one kind (retrieval or streaming).
struct zz_group_dev {
  char *base;          // arena address of the group's region: [B][n_heads][n_tiles] KV tiles
  int32_t n_heads;     // KV heads in the group
  int32_t n_tiles;     // tiles per (batch, head) = ceil(capacity / 32)
  int32_t streaming;   // 1: sink + ring slots; 0: slot == position
  int32_t capacity;    // slots per (batch, head): max_ctx or S + W (n_tiles is that, rounded up to whole tiles)
};

// Per-sequence lengths of a launch over sequences that differ in length (append, prefill): with
// ragged != 0 sequence b of the launch has len[b] tokens cached, and the single length in the
// launch's own parameters (zz_append_params::len, zz_prefill_params::n_past) is not used.
struct zz_seq_lens {
  uint32_t ragged;
  uint32_t len[ZZ_MAX_RAGGED_BATCH];
};

struct zz_append_params {
  const void *k_new, *v_new;      // [B, n_new, Hkv, D] bf16
  zz_group_dev grp[2];
  uint8_t head_group[ZZ_MAX_KV_HEADS];  // kv head -> group (0/1)
  uint8_t head_index[ZZ_MAX_KV_HEADS];  // kv head -> index inside its group
  int64_t len;                    // tokens already in the layer
  int32_t n_new, batch, n_kv_heads, head_dim;
  int32_t sink, window;
  int32_t only_group;             // -1: every head; 0/1: only the heads of that group (the rest belongs to another launch)
  uint32_t *debug_word;           // a build with ZZ_DEBUG_BOUNDS counts here the slot writes it refused; otherwise unused
  const float *rope_cos, *rope_sin;  // [rows][D/2] fp32 tables, or null: K rows are rotated by their position's angles
  int32_t stage;                  // 1: the chunk goes to slots 0.. of an empty area (prefill staging); positions still count from len
};

struct zz_decode_params {
  zz_group_dev grp;
  uint8_t heads[ZZ_MAX_KV_HEADS]; // kv head ids of the group, ascending
  const void *q;                  // [B, Hq, D] bf16
  void *out;                      // [B, Hq, D] bf16
  float *part_o;                  // [B, Hq, ZZ_MAX_SPLITS, D]
  float *part_ml;                 // [B, Hq, ZZ_MAX_SPLITS, 2]  (max in log2 units, sum)
  int *counters;                  // [B, Hkv] workgroups of the unit that have finished; 0 between launches
  const void *k_new, *v_new;      // fused append: [B, 1, Hkv, D] rows of the newest token (or null)
  int32_t new_slot;               // slot the newest token goes to, -1 if it is already in the cache
  int32_t n_valid;                // occupied slots (prefix of the cache)
  int32_t n_tiles_valid;          // ceil(n_valid / 32)
  int32_t tiles_per_split, n_splits;
  int32_t tile_skew;              // tiles a split on an even XCD takes more, its odd neighbour fewer (0: even ranges)
  int32_t batch, n_q_heads, n_kv_heads, head_dim, group_size;
  float scale_log2e;              // softmax scale * log2(e)
  uint32_t *debug_word;           // as in zz_append_params (the fused append writes a slot too)
  const float *rope_cos, *rope_sin;  // as in zz_append_params: rotation of the newest token's K row
  int32_t new_pos;                // position of the newest token (its row of the tables)
};

// The range of tiles [t0, t1) of split `split` of a unit with n_tiles tiles in n_splits splits of
// tiles_per_split.  With tile_skew > 0 the two splits of a pair (2k, 2k+1) share their 2 * tiles_per_split
// tiles unevenly: the one whose workgroup has an even linear index (first_parity: parity of the index of the
// workgroup with split 0) takes tile_skew more, the other as many fewer; an unpaired last split keeps its
// plain range.  The ranges of splits 0 .. n_splits-1 tile [0, n_tiles) exactly once, none empty, provided
// (n_splits-1) * tiles_per_split < n_tiles <= n_splits * tiles_per_split and the last split's plain length
// exceeds tile_skew: what the host guarantees (plan_decode, decode_tile_skew) and its test harness checks
// for every launch and, on its own, over all small cases.  Used by the kernel and by the host's checks.
#if defined(__HIPCC__) || defined(__CUDACC__)
#define ZZ_HOST_DEVICE __host__ __device__
#else
#define ZZ_HOST_DEVICE
#endif
ZZ_HOST_DEVICE inline void zz_split_range(int split, int n_splits, int tiles_per_split, int tile_skew, int first_parity,
                                          int n_tiles, int *t0, int *t1) {
  int a = split * tiles_per_split, b = a + tiles_per_split;
  if (tile_skew > 0) {
    const int base = (split & ~1) * tiles_per_split;
    const int first_len = tiles_per_split + ((first_parity & 1) == 0 ? tile_skew : -tile_skew);
    if (split & 1) {
      a = base + first_len;
      b = base + 2 * tiles_per_split;
    } else if (split + 1 < n_splits) {
      a = base;
      b = base + first_len;
    }
  }
  *t0 = a;
  *t1 = b < n_tiles ? b : n_tiles;
}

// Decode over sequences of different lengths: the workgroups of all sequences form one
// flat grid dimension, sequence b owning workgroups [first_wg[b], first_wg[b+1]); every
// per-sequence quantity (occupied slots, slot of the newest token) follows from seq_len[b].
// The fields of `u` that describe one common length (n_valid, n_tiles_valid, n_splits,
// new_slot) are unused except new_slot's sign: >= 0 means the step appends.
struct zz_decode_ragged_params {
  zz_decode_params u;
  int32_t sink, window;
  uint32_t seq_len[ZZ_MAX_RAGGED_BATCH];        // tokens the attention of sequence b sees
  uint16_t first_wg[ZZ_MAX_RAGGED_BATCH + 1];   // prefix sums of the per-sequence split counts
};

// Where the keys of a prefill call come from: cached tiles, then the staged chunk.
struct zz_prefill_params {
  zz_group_dev grp;
  uint8_t heads[ZZ_MAX_KV_HEADS];
  const void *q;                  // [B, n_new, Hq, D]
  void *out;                      // [B, n_new, Hq, D]
  const char *stage;              // staged chunk: [B][Hkv][stage_tiles] KV tiles, token idx -> slot idx
  int32_t stage_tiles;            // tiles per (batch, kv head) in the staging area (stride)
  int32_t n_past;                 // tokens already cached (query positions start here)
  int32_t n_new;
  int32_t batch, n_q_heads, n_kv_heads, head_dim, group_size;
  int32_t sink, window;
  float scale_log2e;
};

struct zz_stage_params {
  const void *k_new, *v_new;      // [B, n_new, Hkv, D]
  char *stage;
  int32_t stage_tiles, n_new, batch, n_kv_heads, head_dim;
  uint32_t *debug_word;
  const float *rope_cos, *rope_sin;
  int64_t n_past;                 // position of the chunk's first token (equal lengths)
};

hipError_t zz_launch_append(const zz_append_params &p, const zz_seq_lens &lens, hipStream_t s);
hipError_t zz_launch_decode(const zz_decode_params &p, hipStream_t s);
hipError_t zz_launch_decode_ragged(const zz_decode_ragged_params &p, int total_wg, hipStream_t s);
hipError_t zz_launch_zero(int *p, int n, hipStream_t s);
hipError_t zz_launch_stage(const zz_stage_params &p, const zz_seq_lens &lens, hipStream_t s);
// pair_min_wg: the eight-wave form (two head chunks of a KV head per workgroup) is used where the shape permits
// it and the launch then has at least that many workgroups; negative: never
hipError_t zz_launch_prefill(const zz_prefill_params &p, const zz_seq_lens &lens, int pair_min_wg, hipStream_t s);
hipError_t zz_launch_probe_read(const void *buf, size_t bytes, int nontemporal, int n_wg, void *sink, hipStream_t s);
int zz_query_num_cu();  // compute units of the current device, or 0 if none is usable
// Device address, on the current device, of the library's own static scratch array
// (ZZ_STATIC_SCRATCH_BYTES bytes): resolved once per device, then kept.
hipError_t zz_static_scratch(char **out);
bool zz_stream_is_capturing(hipStream_t s);  // true while launches on `s` are recorded into a graph instead of run

#endif
