/*
 * zz.h - C ABI of the ZigzagAttention inference hot path for AMD MI355X (gfx950).
 *
 * What the library computes (arXiv 2508.12407):
 *   - Section 2.2: every transformer layer is either all-retrieval or all-streaming
 *     (p of L layers streaming), so a layer needs exactly one attention launch.
 *   - Sections 1 and 2.1: a retrieval head runs full causal attention over every
 *     cached token; a streaming head keeps only the attention-sink tokens and a
 *     recent window and waives the rest of its KV cache.
 *   - Section 3.3: sink size S and window length W parameterise streaming attention.
 *   - Section 2.1 (last paragraph): the DuoAttention layout mixes both kinds of
 *     head inside one layer and pays two attention launches per layer; it is
 *     available here as ZZ_MIXED, the comparison baseline.
 *
 * Readings where the paper is silent: the window is the W newest positions
 * including the query's own (a streaming head sees at most S+W tokens); the kind
 * is a property of a KV head (all Hq/Hkv query heads of its group follow it);
 * keys arrive already position-encoded; softmax scale defaults to 1/sqrt(head_dim).
 *
 * Conventions for every entry point
 *   - All tensors are bf16 (16-bit brain float), contiguous, 16-byte aligned DEVICE
 *     memory owned by the caller.  The KV arena and the workspace are caller-owned
 *     DEVICE memory too.  `zz_config` and the two mask arrays are HOST memory and are
 *     copied by zz_create.  `zz_ctx` is host memory owned by the library.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue kernels: the library never allocates device memory, never
 *     synchronises and never copies the arena.
 *   - Return value: 0 (ZZ_OK) or a negative ZZ_E* code.  All argument checks run on
 *     the host before anything is launched; a call that fails one has launched nothing
 *     and changed no length.  ZZ_EHIP (the runtime refused a launch) changes no length
 *     either, but a call made of several launches (two head kinds, one launch per
 *     sequence) does not recall those already issued.  n_new == 0 is a successful no-op.
 *   - Every sequence of the batch has its own length per layer.  The batched calls
 *     advance all B sequences by the same number of tokens, each from its own length;
 *     the *_seq calls advance one sequence, which is how prompts of different lengths
 *     enter a batch.  A batched call is one launch per head kind whether the lengths of the
 *     layer are equal or not (unequal: the per-sequence lengths travel in the launch's
 *     arguments), for batches of at most ZZ_MAX_RAGGED_BATCH sequences; larger batches of
 *     unequal lengths are served one sequence at a time by zz_kv_append and zz_attn_prefill
 *     and refused (ZZ_EUNSUPPORTED) by zz_attn_decode and zz_decode_step.
 *   - A context must not be used from two host threads at once.
 *   - HIP-graph capture.  Every call may be made on a stream that is being captured: the
 *     launches are recorded instead of run.  The host-side bookkeeping (sequence lengths)
 *     advances once, at the call; a replay repeats the recorded kernels with the recorded
 *     arguments (the same slot is written again, the same number of tokens is attended) and
 *     changes no length.  To decode further tokens by replay, the caller captures one graph per
 *     step or re-records.  The split counters in the workspace are cleared by a small kernel
 *     ahead of the attention launch of every zz_attn_decode / zz_decode_step call until one such
 *     call has been made on a stream that was not being captured; that clear, when recorded,
 *     stays in the graph and is harmless on replay (counters are zero between launches).
 */
#ifndef ZZ_H
#define ZZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZZ_TILE_SLOTS 32   /* cache slots per KV tile                                   */
#define ZZ_MAX_KV_HEADS 64 /* upper bound on n_kv_heads                                  */
#define ZZ_MAX_SPLITS 128  /* upper bound on split-K partials per (batch, query head)    */
#define ZZ_MAX_RAGGED_BATCH 256 /* largest batch whose sequences may differ in length at decode */
/* Static split-K scratch of zz_attn_decode_static, held once per GPU: 64 KiB of counters,
 * 512 KiB of (max, sum) pairs, 16 MiB of partial outputs. */
#define ZZ_STATIC_MAX_UNITS 16384          /* batch * n_kv_heads                          */
#define ZZ_STATIC_MAX_ROW_ELEMS 32768      /* batch * n_q_heads * head_dim                */
#define ZZ_STATIC_SCRATCH_BYTES (64 * 1024 + 512 * 1024 + 16 * 1024 * 1024)

enum {
  ZZ_OK = 0,
  ZZ_EINVAL = -1,       /* null pointer, non-positive size, bad enum                      */
  ZZ_ERANGE = -2,       /* layer / head / n_new out of range                              */
  ZZ_ENOSPC = -3,       /* append past max_ctx; arena or workspace too small              */
  ZZ_EALIGN = -4,       /* a device pointer is not 16-byte (arena: 256-byte) aligned      */
  ZZ_ESTATE = -5,       /* decode on an empty layer; mask missing for the chosen layout   */
  ZZ_EUNSUPPORTED = -6, /* head_dim, group size or head count outside what is built       */
  ZZ_EHIP = -7          /* a kernel launch was rejected by the HIP runtime                */
};

enum { ZZ_ZIGZAG = 0, ZZ_MIXED = 1 };

typedef struct zz_ctx zz_ctx;

typedef struct zz_config {
  int32_t n_layers;   /* L >= 1                                                           */
  int32_t n_q_heads;  /* Hq, multiple of n_kv_heads, Hq / Hkv <= 16                       */
  int32_t n_kv_heads; /* Hkv <= ZZ_MAX_KV_HEADS                                           */
  int32_t head_dim;   /* D: 64 or 128                                                     */
  int32_t batch;      /* 1 <= B <= 65535                                                  */
  int32_t max_ctx;    /* capacity of a retrieval cache, tokens                            */
  int32_t sink;       /* S >= 0  (Section 3.3)                                            */
  int32_t window;     /* W >= 1  (Section 3.3), includes the query's own position         */
  int32_t max_chunk;  /* largest n_new accepted by zz_attn_prefill (0: prefill unused)    */
  int32_t layout;     /* ZZ_ZIGZAG or ZZ_MIXED                                            */
  float softmax_scale;                /* 0 => 1/sqrt(head_dim)                            */
  const uint8_t *layer_is_streaming;  /* HOST [n_layers]; required for ZZ_ZIGZAG          */
  const uint8_t *kvhead_is_streaming; /* HOST [n_layers*n_kv_heads]; required for ZZ_MIXED */
} zz_config;

/* Bytes of DEVICE memory the caller must provide; 0 if the config is invalid.  Pure host
 * arithmetic.  The arena holds the KV cache of every layer: max_ctx slots per retrieval head
 * (Section 1: the cache grows linearly with the context) and S + W slots per streaming head
 * (Sections 1 and 3.3: the rest is waived), in whole 32-slot tiles; layout under
 * zz_kv_elem_offset.  The workspace holds the split-K partials and counters of one decode
 * launch and the staged chunk of one prefill call (build conventions, not from the paper). */
size_t zz_arena_bytes(const zz_config *cfg);
size_t zz_workspace_bytes(const zz_config *cfg);

/* Validate `cfg`, lay the per-layer caches out inside `kv_arena` (256-byte aligned DEVICE
 * memory) and create a context (HOST memory, freed by zz_destroy) with every layer empty.
 * The per-layer kind comes from layer_is_streaming (Section 2.2: p of the L layers stream)
 * or, for the comparison layout, from kvhead_is_streaming (Section 2.1).  Neither the arena
 * nor the workspace is touched.  ZZ_ENOSPC if either is smaller than zz_*_bytes says,
 * ZZ_EALIGN if misaligned, ZZ_ESTATE if the mask of the chosen layout is NULL. */
int zz_create(const zz_config *cfg, void *kv_arena, size_t arena_bytes, void *workspace,
              size_t workspace_bytes, zz_ctx **out);
int zz_destroy(zz_ctx *ctx);
int zz_reset(zz_ctx *ctx); /* all layer lengths := 0 */

/* Append n_new tokens to layer `layer` (Sections 1 and 3.3: a retrieval head keeps
 * every token, a streaming head keeps the S sink tokens plus the W newest ones).
 * k_new, v_new: DEVICE [B, n_new, Hkv, D].  A token at position pos goes to slot
 * zz_slot_of(pos); a streaming ring slot is overwritten by the token W positions
 * later, which is the eviction.  The result equals n_new single-token appends.
 * ZZ_ENOSPC if the layer's length would exceed max_ctx (lengths of all layers, also
 * all-streaming ones, are bounded by max_ctx). */
int zz_kv_append(zz_ctx *ctx, int layer, const void *k_new, const void *v_new, int n_new, void *stream);
/* The same for sequence b alone: k_new, v_new: DEVICE [1, n_new, Hkv, D]; only that
 * sequence's length changes.  ZZ_ERANGE if b is not in [0, B). */
int zz_kv_append_seq(zz_ctx *ctx, int layer, int b, const void *k_new, const void *v_new, int n_new, void *stream);

/* Attention for n_new new query positions [len, len + n_new) of layer `layer`, where
 * len = zz_layer_len(layer), over the cached tokens followed by (k_new, v_new)
 * (Section 1: prefilling phase; masks as above, each query at its own position).
 * q, out: DEVICE [B, n_new, Hq, D]; k_new, v_new: DEVICE [B, n_new, Hkv, D].
 * Does not change the cache: call zz_kv_append with the same k_new, v_new afterwards.
 * 1 <= n_new <= max_chunk.  Uses the workspace; calls on one context must be stream-ordered. */
int zz_attn_prefill(zz_ctx *ctx, int layer, const void *q, const void *k_new, const void *v_new,
                    int n_new, void *out, void *stream);
/* The same for sequence b alone (query positions [zz_seq_len(b), zz_seq_len(b) + n_new)):
 * q, out: DEVICE [1, n_new, Hq, D]; k_new, v_new: DEVICE [1, n_new, Hkv, D].  Follow it with
 * zz_kv_append_seq.  ZZ_ERANGE if b is not in [0, B). */
int zz_attn_prefill_seq(zz_ctx *ctx, int layer, int b, const void *q, const void *k_new, const void *v_new,
                        int n_new, void *out, void *stream);

/* Attention for the newest cached position of layer `layer` (Section 1: decoding
 * phase): call after zz_kv_append(..., 1).  q, out: DEVICE [B, Hq, D].
 * ZZ_ESTATE if a sequence of the layer is empty.  Uses the workspace. */
int zz_attn_decode(zz_ctx *ctx, int layer, const void *q, void *out, void *stream);

/* zz_attn_decode for callers that cannot allocate device memory or hand a workspace over at
 * the time of the call (code under HIP-graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the same launches with the same result, but the split-K partials and
 * counters go to a static array inside the library (ZZ_STATIC_SCRATCH_BYTES per GPU, resolved
 * on the call's first use on a device and held until the process ends) instead of the
 * context's workspace.  The call allocates nothing.  q, out: DEVICE [B, Hq, D], as above.
 * Limits: batch * n_kv_heads <= ZZ_STATIC_MAX_UNITS and batch * n_q_heads * head_dim <=
 * ZZ_STATIC_MAX_ROW_ELEMS (128k / batch 4 and 32k / batch 8 at 32 heads of 128 fit), else
 * ZZ_ENOSPC with nothing launched (zz_last_error_detail says which limit).  Every call on a GPU,
 * from any context, uses that GPU's one array: the counters are cleared by a small kernel
 * ahead of the attention launch, the rest is overwritten before it is read; calls that
 * overlap in time on one GPU (different streams or contexts) race and must be ordered by the
 * caller. */
int zz_attn_decode_static(zz_ctx *ctx, int layer, const void *q, void *out, void *stream);

/* One decode step of a layer in a single launch per head kind: appends the newest
 * token's rows (k_new, v_new: DEVICE [B, 1, Hkv, D]) and attends from it (q, out:
 * DEVICE [B, Hq, D]).  Same result, same cache contents and same length afterwards as
 * zz_kv_append(ctx, layer, k_new, v_new, 1, stream) followed by
 * zz_attn_decode(ctx, layer, q, out, stream); it removes the separate append launch,
 * the remaining per-layer overhead next to the one attention of Section 2.2.
 * ZZ_ENOSPC if the layer is full; other errors as for the two calls. */
int zz_decode_step(zz_ctx *ctx, int layer, const void *q, const void *k_new, const void *v_new, void *out,
                   void *stream);

/* Rotary position encoding at append (not in the paper, whose model, Section 3.1, uses it; a step
 * next to the hot path fused in, in the spirit of Section 1's concern with per-layer overhead).
 * cos_table, sin_table: DEVICE fp32 [rows][D/2], 16-byte aligned, caller-owned, alive while set.
 * Once set, every K row that enters the context - zz_kv_append, the chunk of zz_attn_prefill,
 * the newest token of zz_decode_step - is rotated before it is stored or attended: element i
 * with element i + D/2 by the angle of row p of the tables, p the token's absolute position in
 * its sequence (streaming caches keep the positions the tokens had: no re-indexing), computed
 * in fp32 as x cos - y sin / x cos + y sin and rounded to bf16.  V and q are taken as given: the
 * caller rotates q.  A call that would need a row >= rows returns ZZ_ERANGE and launches nothing.
 * (NULL, NULL, 0) switches it off again; the default. */
int zz_set_rope_tables(zz_ctx *ctx, const float *cos_table, const float *sin_table, int64_t rows);

/* Tokens appended to the layer so far (of its longest sequence, if they differ), or a
 * negative error code.  Host bookkeeping only (build convention): a streaming layer counts
 * every token it has seen, not the S + W it still holds, because the slot of the next token
 * and the positions of the cached ones follow from that count. */
int64_t zz_layer_len(const zz_ctx *ctx, int layer);
/* Overwrite the length of every sequence of a layer (restoring a snapshot of the arena).
 * 0 <= len <= max_ctx. */
int zz_set_layer_len(zz_ctx *ctx, int layer, int64_t len);
/* The same per sequence.  ZZ_ERANGE if b is not in [0, B). */
int64_t zz_seq_len(const zz_ctx *ctx, int layer, int b);
int zz_set_seq_len(zz_ctx *ctx, int layer, int b, int64_t len);

/* Attention launches zz_attn_decode issues for this layer: 1 for a zigzag layer
 * (Section 2.2), 2 for a mixed layer holding both kinds of head (Section 2.1). */
int zz_layer_launches(const zz_ctx *ctx, int layer);

/* Pure host arithmetic: the cache slot a token at position `pos` of (layer, kv_head)
 * is written to.  Retrieval: pos.  Streaming, with S the sink size and W the window length of
 * Section 3.3: pos if pos < S, else S + (pos - S) mod W.  The paper only names the two
 * parameters; that sink tokens sit in S fixed slots outside the ring and that the ring has
 * exactly W slots (the window includes the query's own position) is this build's reading.
 * Negative error code on bad arguments (ZZ_ERANGE if pos >= max_ctx on a retrieval head). */
int64_t zz_slot_of(const zz_config *cfg, int layer, int kv_head, int64_t pos);

/* Pure host arithmetic: byte offset inside the arena of element d of slot `slot`
 * of (layer, batch b, kv_head); which = 0 for K, 1 for V.  Negative on bad arguments.
 *
 * Arena layout.  Layers in order; inside a layer first the retrieval heads' region,
 * then the streaming heads' region (one of the two is empty in a zigzag layer).  A
 * region is [B][heads of that kind, ascending][n_tiles] KV tiles with
 * n_tiles = ceil(capacity / 32), capacity = max_ctx or S + W.  A KV tile holds 32
 * consecutive slots: 64*D bytes of K followed by 64*D bytes of V, each stored in the
 * register image of the 16x16x32 bf16 MFMA operand it feeds, so a wavefront streams
 * a tile with sixteen (D = 128) fully coalesced 1 KiB loads and no shuffling.
 * For slot-in-tile t (0..31) and element d (0..D-1):
 *   K: element index ((( (t/16)*(D/8) + d/8 )*16 + t%16 )*8 + d%8)
 *   V: element index ((( (d/16)*4 + (t%16)/4 )*16 + d%16 )*8 + 4*(t/16) + t%4) + 32*D
 * (element index * 2 = byte offset inside the tile). */
int64_t zz_kv_elem_offset(const zz_ctx *ctx, int layer, int which, int b, int kv_head, int64_t slot, int d);

/* Pure host arithmetic: how many (group of four waves, 32-key tile) visits the next
 * zz_attn_prefill(layer, n_new) performs, and how many a kernel that skipped
 * nothing below the causal diagonal would perform at the same granularity
 * (four waves - a workgroup, or half of an eight-wave one - cover 64 consecutive query
 * positions for even group sizes and 128 for odd ones).  1 - visited/causal is the skipped-tile
 * fraction that the sink + window mask of streaming heads allows (Section 3.3). */
int zz_prefill_tile_counts(const zz_ctx *ctx, int layer, int n_new, int64_t *visited, int64_t *causal);

/* Transport optimisation (Section 2.2, Eq. 5), host only: from converged head importances
 * alpha (HOST, [n_layers*n_heads], each in [0,1]) choose the p = sparsity*n_layers
 * layers that become all-streaming.  Heads are first classified as the paper's starting
 * point does (the p*H heads of smallest alpha are streaming heads); turning a
 * retrieval head into a streaming one costs +alpha, the reverse costs -omega*alpha, keeping a
 * head costs 0; the set of p layers minimising the summed cost is returned in
 * layer_is_streaming (HOST, [n_layers], 0/1; ties go to the lower layer index) and the
 * minimum in *loss (may be NULL).  The cost of a candidate differs from a constant only by
 * the sum over its layers of (alpha of the layer's retrieval heads + omega * alpha of its
 * streaming heads), so sorting the layers by that key gives the same optimum as examining
 * all C(L,p) candidates one by one, in O(L*H + L log L).  0 <= omega <= 1; 0 <= sparsity <= 1
 * and sparsity*n_layers must be a whole number (p/L = s), else ZZ_ERANGE. */
int zz_transport_select(const float *alpha, int n_layers, int n_heads, float sparsity, float omega,
                        uint8_t *layer_is_streaming, double *loss);

const char *zz_strerror(int code);
/* What the HIP runtime reported for the calling thread's most recent ZZ_EHIP
 * (which kernel, hipGetErrorString text); "" if there was none. */
const char *zz_last_error_detail(void);


/* ------------------------------------------------------------------------------------------
 * Measurement and tuning.  Nothing below is part of the method or needed to use it: these
 * calls exist for the benchmark and the tests (forcing split counts, reading the launch plan,
 * timing the memory system).
 * ------------------------------------------------------------------------------------------ */

/* Tuning knobs, for measurement.  key: */
enum {
  ZZ_TUNE_DECODE_WG_PER_CU = 1,  /* target decode workgroups per compute unit (default 1)  */
  ZZ_TUNE_DECODE_SPLITS = 2,     /* force the split count (0 = automatic)                  */
  ZZ_TUNE_NUM_CU = 3,            /* override the detected compute-unit count               */
  ZZ_TUNE_DECODE_XCD_SKEW = 5,   /* in 1/1000 of a split: how much longer the range of a decode split
                                    that lands on an even XCD is, and its odd neighbour's shorter
                                    (default 50, applied to splits of 128 tiles or more; a value
                                    set here applies to splits of any length; 0: even ranges) */
  ZZ_TUNE_PREFILL_PAIRING = 4    /* 1 (default): prefill runs two head chunks of a KV head in
                                    one eight-wave workgroup where the shape allows, for retrieval
                                    heads, if the launch keeps a workgroup per compute unit and the
                                    cache already holds at least a chunk; 0: never; 2: wherever
                                    the shape allows */
};
int zz_tune(zz_ctx *ctx, int key, int value);

/* Split count and tiles per split the next zz_attn_decode would use for group
 * `group` (0 retrieval, 1 streaming) of the layer; 0 splits if the group is empty.
 * With unequal sequence lengths one tiles-per-split value serves the whole launch,
 * sequence b takes ceil(its tiles / tiles_per_split) workgroups per head, and *n_splits
 * is the largest of those counts. */
int zz_decode_plan(const zz_ctx *ctx, int layer, int group, int *n_splits, int *tiles_per_split);

/* Debug build.  A library compiled with -DZZ_DEBUG_BOUNDS (libzz_debug.so, built next to the
 * regular one) checks every cache-slot write of the append kernels and of the fused append
 * against the slot capacity and the byte range of the head's region before it stores; a write
 * that fails the check is dropped and counted in one 32-bit word of the workspace, at the
 * byte offset zz_debug_word_offset returns (0 for an invalid config).  The caller zeroes the
 * word and reads it back; the regular build never touches it.  zz_is_debug_build: 1 or 0. */
size_t zz_debug_word_offset(const zz_config *cfg);
int zz_is_debug_build(void);

/* Measurement aid, not part of the method: streams `bytes` (rounded down to 16 KiB) of DEVICE
 * memory `buf` through one workgroup per compute unit with the decode kernel's access pattern
 * and discards them; nontemporal != 0 uses the same non-temporal loads as the decode kernel.
 * Timed by the caller, it gives the read bandwidth the memory system delivers to that
 * pattern: the practical ceiling beside the published peak. */
int zz_probe_read(zz_ctx *ctx, const void *buf, size_t bytes, int nontemporal, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ZZ_H */
