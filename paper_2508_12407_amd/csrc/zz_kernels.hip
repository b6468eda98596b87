// gfx950 (CDNA4, MI355X) kernels of the ZigzagAttention hot path.
//
// Data layout.  The KV cache is stored in "KV tiles" of 32 slots: 64*D bytes of K
// then 64*D bytes of V, each laid out as the register image of the operand it
// feeds to v_mfma_f32_16x16x32_bf16, so lane L's i-th 16-byte load of a tile is at
// byte i*1024 + L*16 and a wavefront streams a tile as 1 KiB contiguous loads with
// no LDS staging and no shuffles.
//
// MFMA operand convention used throughout (16x16x32, A: MxK, B: KxN, C: MxN):
//   lane L supplies A[m = L%16][k = 8*(L/16) .. +7] and B[k = 8*(L/16) .. +7][n = L%16],
//   and receives C[m = 4*(L/16) + r][n = L%16], r = 0..3.
// Scores:  S^T[token][column] = K[token][:] . Q[column][:]   (A = K tile, B = Q)
// Output:  O^T[d][column]    = sum_token V[token][d] P[token][column]  (A = V tile, B = P)
// A "column" is one of up to 16 query rows sharing the KV head: the G query heads
// of the group in decode, 16 query positions of one head in prefill.  The lane that
// holds score rows 4*kg+r of token blocks 0 and 1 is exactly the lane that must
// supply P for k = 8*kg .. +7, once the V tile orders its tokens that way, so the
// probabilities never move between lanes.
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

#include "zz_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define ZZ_NEG_INF (-__builtin_inff())

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// K/V of the cache are read once per launch and never again: a non-temporal load
// keeps the stream from displacing anything in L2 / the memory-side cache and is
// measurably faster on MI355X than a default-policy load for pure streaming.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Split-K partials cross workgroups that may sit on different XCDs, whose L2s are not
// coherent with each other for ordinary accesses.  Device-scope relaxed atomics go
// straight to the device-coherent level (sc1), so neither side needs an L2-wide
// write-back / invalidate fence (which costs far more than the whole merge).
__device__ __forceinline__ void store_device_coherent(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device_coherent(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint4 pick(bool c, uint4 a, uint4 b) {
  return make_uint4(c ? a.x : b.x, c ? a.y : b.y, c ? a.z : b.z, c ? a.w : b.w);
}

__device__ __forceinline__ float xor_lanes(float v, int mask) { return __shfl_xor(v, mask, 64); }

// Debug build (-DZZ_DEBUG_BOUNDS): every cache-slot write is checked against the head's slot
// capacity and tile count first; a write that fails is dropped and counted, never issued.
#ifdef ZZ_DEBUG_BOUNDS
#define ZZ_SLOT_WRITE_OK(ok, word) ((ok) ? true : ((word) ? (atomicAdd((word), 1u), false) : false))
#else
#define ZZ_SLOT_WRITE_OK(ok, word) true
#endif

// Rotary position encoding of eight consecutive elements of a K row: `own` (elements d .. d+7) turned
// together with `partner` (the elements D/2 away) by the angles of the row's position,
//     lower half:  x cos - y sin        upper half:  x cos + y sin        (y: the partner element)
// in fp32 from the bf16 inputs and the caller's fp32 tables, rounded to bf16 (nearest even).
// cs, sn: the eight table entries of the pair indices d mod D/2 .. +7.
__device__ __forceinline__ uint4 rope_chunk(uint4 own, uint4 partner, const float *cs, const float *sn, bool upper) {
  const float4 c0 = *(const float4 *)cs, c1 = *(const float4 *)(cs + 4);
  const float4 s0 = *(const float4 *)sn, s1 = *(const float4 *)(sn + 4);
  const float c[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
  const float sg[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
  const unsigned xo[4] = {own.x, own.y, own.z, own.w}, yo[4] = {partner.x, partner.y, partner.z, partner.w};
  unsigned r[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    unsigned packed = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int j = 2 * w + h;
      const float x = __builtin_bit_cast(float, h ? (xo[w] & 0xffff0000u) : (xo[w] << 16));
      const float y = __builtin_bit_cast(float, h ? (yo[w] & 0xffff0000u) : (yo[w] << 16));
      const float v = fmaf(upper ? y : -y, sg[j], x * c[j]);
      const __bf16 vb = (__bf16)v;
      packed |= (unsigned)__builtin_bit_cast(unsigned short, vb) << (16 * h);
    }
    r[w] = packed;
  }
  return make_uint4(r[0], r[1], r[2], r[3]);
}

// --------------------------------------------------------------------------
// Append / evict: scatter new K, V rows into their tiles.
// One thread per (batch, new token, kv head, 8-element chunk of the head vector).
// --------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void zz_append_kernel(zz_append_params p, zz_seq_lens sl) {
  constexpr int CH = D / 8;
  const int64_t total = (int64_t)p.batch * p.n_new * p.n_kv_heads * CH;
  int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const int c = (int)(tid % CH);
  tid /= CH;
  const int g = (int)(tid % p.n_kv_heads);
  tid /= p.n_kv_heads;
  const int idx = (int)(tid % p.n_new);
  const int b = (int)(tid / p.n_new);

  if (p.only_group >= 0 && p.head_group[g] != p.only_group) return;
  const zz_group_dev &G = p.grp[p.head_group[g]];
  const int64_t len = sl.ragged ? (int64_t)sl.len[b] : p.len;   // tokens the sequence holds already
  const int64_t pos = (p.stage ? 0 : len) + idx;                 // where the token goes (staging: an empty area)
  int64_t slot = pos;
  if (G.streaming && pos >= p.sink) {
    // a ring token that a later token of this same call overwrites is never written,
    // so the result does not depend on the order threads run in
    if (pos + p.window <= len + p.n_new - 1) return;   // (never a staging launch: its heads do not evict)
    slot = p.sink + (pos - p.sink) % p.window;
  }
  const int64_t src = ((((int64_t)b * p.n_new + idx) * p.n_kv_heads + g) * D) / 8 + c;
  uint4 kv = ((const uint4 *)p.k_new)[src];
  const uint4 vv = ((const uint4 *)p.v_new)[src];
  if (p.rope_cos) {
    const bool upper = c >= CH / 2;
    const uint4 partner = ((const uint4 *)p.k_new)[upper ? src - CH / 2 : src + CH / 2];
    const int64_t row = (len + idx) * (D / 2) + 8 * (c % (CH / 2));
    kv = rope_chunk(kv, partner, p.rope_cos + row, p.rope_sin + row, upper);
  }

  const int64_t tile = slot / ZZ_TILE_SLOTS;
  const int t = (int)(slot % ZZ_TILE_SLOTS);
  if (!ZZ_SLOT_WRITE_OK(slot >= 0 && slot < G.capacity && tile < G.n_tiles && p.head_index[g] < G.n_heads, p.debug_word)) return;
  char *tb = G.base + (((int64_t)b * G.n_heads + p.head_index[g]) * G.n_tiles + tile) * (int64_t)(128 * D);
  // K: 16-byte chunk c of the row -> [t/16][c][t%16]
  ((uint4 *)tb)[((t >> 4) * CH + c) * 16 + (t & 15)] = kv;
  // V: element d -> [d/16][(t%16)/4][d%16][4*(t/16) + t%4], after the 64*D bytes of K
  unsigned short *vt = (unsigned short *)tb + 32 * D;
  const unsigned int w[4] = {vv.x, vv.y, vv.z, vv.w};
  const int e = 4 * (t >> 4) + (t & 3);
  const int kgv = (t & 15) >> 2;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int d = 8 * c + i;
    const unsigned short val = (unsigned short)((i & 1) ? (w[i >> 1] >> 16) : (w[i >> 1] & 0xffffu));
    vt[((((d >> 4) * 4 + kgv) * 16 + (d & 15)) << 3) + e] = val;
  }
}

// Bulk append into never-evicting heads (retrieval caches, the prefill staging area): one
// workgroup per (tile, head, sequence).  K rows go out as 16-byte pieces as above; the V rows
// of the tile are transposed through LDS so that a full tile is written as 16-byte pieces
// too (the per-token kernel scatters V in 2-byte pieces, which more than doubles the bytes
// HBM has to write).  A tile only partly covered by the call keeps the 2-byte stores, so
// slots that already hold older tokens are not touched.
// grid (most tiles any sequence touches, heads of group 0, B): with sequences of different
// lengths each starts at its own tile, and a workgroup past its sequence's last tile has nothing to do.
template <int D>
__global__ __launch_bounds__(256) void zz_append_bulk_kernel(zz_append_params p, zz_seq_lens sl) {
  constexpr int CH = D / 8;
  __shared__ unsigned short sv[32][D + 2];
  const zz_group_dev &G = p.grp[0];
  const int hi = blockIdx.y, b = blockIdx.z;
  int g = 0;
  for (int j = 0; j < p.n_kv_heads; ++j)
    if (p.head_group[j] == 0 && p.head_index[j] == hi) g = j;
  const int64_t held = sl.ragged ? (int64_t)sl.len[b] : p.len;   // tokens the sequence holds: position of the chunk's first token
  const int64_t len = p.stage ? 0 : held;                         // slot of the chunk's first token (staging: an empty area)
  const int64_t tile = len / ZZ_TILE_SLOTS + blockIdx.x;
  if (tile * 32 >= len + p.n_new) return;   // (the whole workgroup)
  const int64_t s_lo = max(tile * 32, len), s_hi = min(tile * 32 + 32, len + (int64_t)p.n_new);  // slots == positions (+ held - len)
  if (!ZZ_SLOT_WRITE_OK(s_lo >= 0 && s_hi <= G.capacity && tile < G.n_tiles && hi < G.n_heads, threadIdx.x == 0 ? p.debug_word : nullptr))
    return;   // (the whole workgroup: the condition is the same for all its threads)
  char *tb = G.base + (((int64_t)b * G.n_heads + hi) * G.n_tiles + tile) * (int64_t)(128 * D);
  for (int idx = threadIdx.x; idx < 32 * CH; idx += 256) {
    const int t = idx / CH, c = idx % CH;
    const int64_t slot = tile * 32 + t;
    if (slot < s_lo || slot >= s_hi) continue;
    const int64_t src = ((((int64_t)b * p.n_new + (slot - len)) * p.n_kv_heads + g) * D) / 8 + c;
    uint4 kv = ((const uint4 *)p.k_new)[src];
    if (p.rope_cos) {
      const bool upper = c >= CH / 2;
      const uint4 partner = ((const uint4 *)p.k_new)[upper ? src - CH / 2 : src + CH / 2];
      const int64_t row = (held + (slot - len)) * (D / 2) + 8 * (c % (CH / 2));
      kv = rope_chunk(kv, partner, p.rope_cos + row, p.rope_sin + row, upper);
    }
    ((uint4 *)tb)[((t >> 4) * CH + c) * 16 + (t & 15)] = kv;
    const uint4 vv = ((const uint4 *)p.v_new)[src];
    const unsigned w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) sv[t][8 * c + i] = (unsigned short)((i & 1) ? (w[i >> 1] >> 16) : (w[i >> 1] & 0xffffu));
  }
  __syncthreads();
  const bool full = s_lo == tile * 32 && s_hi == tile * 32 + 32;
  unsigned short *vt = (unsigned short *)tb + 32 * D;
  for (int o = threadIdx.x; o < 4 * D; o += 256) {   // o = (d/16 * 4 + key group) * 16 + d%16: one 16-byte piece of the V image
    const int dd = o & 15, kgv = (o >> 4) & 3, nb = o >> 6;
    const int d = 16 * nb + dd;
    unsigned short e8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) e8[e] = sv[(e < 4 ? 0 : 16) + 4 * kgv + (e & 3)][d];
    if (full) {
      ((uint4 *)vt)[o] = make_uint4(e8[0] | ((unsigned)e8[1] << 16), e8[2] | ((unsigned)e8[3] << 16),
                                    e8[4] | ((unsigned)e8[5] << 16), e8[6] | ((unsigned)e8[7] << 16));
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int64_t slot = tile * 32 + (e < 4 ? 0 : 16) + 4 * kgv + (e & 3);
        if (slot >= s_lo && slot < s_hi) vt[(o << 3) + e] = e8[e];
      }
    }
  }
}

// --------------------------------------------------------------------------
// Shared tile arithmetic: scores of one 32-slot tile for one column block, and
// the online-softmax step that turns them into the bf16 P operand.
// --------------------------------------------------------------------------

// x[0..3]: tokens 4*kg+r of block 0, x[4..7]: tokens 16+4*kg+r (already scaled to
// log2 units and masked with -inf).  Updates (m, l), returns P and the factor the
// running output must be multiplied by.
__device__ __forceinline__ bf16x8 softmax_step(const float (&x)[8], float &m, float &l, float &alpha) {
  float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
  mx = fmaxf(mx, xor_lanes(mx, 16));
  mx = fmaxf(mx, xor_lanes(mx, 32));
  const float m_new = fmaxf(m, mx);
  const float m_safe = (m_new == ZZ_NEG_INF) ? 0.f : m_new;  // a column with nothing visible yet
  alpha = fast_exp2(m - m_safe);
  bf16x8 P;
  float sum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const __bf16 pb = (__bf16)fast_exp2(x[e] - m_safe);
    P[e] = pb;
    sum += (float)pb;  // normalise by what is actually multiplied into V
  }
  l = l * alpha + sum;
  m = m_new;
  return P;
}

// --------------------------------------------------------------------------
// Decode: split-K over the occupied slots of one (batch, kv head).
// grid (n_splits, heads of the group, B), 4 waves per workgroup; wave w takes tiles
// t0+w, t0+w+4, ... of the workgroup's range, double-buffered in registers.  The
// workgroup of a unit that finishes last merges the unit's partials, so a layer's
// attention is one launch.
// --------------------------------------------------------------------------
template <int D, int WAVES>
__device__ __forceinline__ void decode_body(const zz_decode_params &p, const int split, const int b, const int n_valid,
                                            const int n_tiles_valid, const int n_splits, const int new_slot,
                                            const int new_pos) {
  constexpr int KS = D / 32;      // MFMA k-steps over the head dimension
  constexpr int NL = D / 16;      // 1 KiB loads in the K part (= 2*KS) and in the V part
  constexpr int TILE_U4 = 8 * D;  // uint4 per KV tile
  constexpr int OP = D + 4;       // padded row of the cross-wave reduction buffer
  constexpr int NT = 64 * WAVES;  // threads per workgroup
  constexpr int COLS = WAVES == 4 ? 16 : 8;  // columns the reduction buffer holds (group size limit of the launch)

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, kg = lane >> 4;
  const int hg = blockIdx.y;
  const int G = p.group_size;
  const int g = p.heads[hg];

  bf16x8 qop[KS];
  {
    const uint4 *qp = (const uint4 *)p.q + ((int64_t)b * p.n_q_heads + g * G + (col < G ? col : 0)) * (D / 8) + kg;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      uint4 v = qp[4 * s];
      if (col >= G) v = make_uint4(0, 0, 0, 0);
      qop[s] = as_bf16x8(v);
    }
  }

  const uint4 *tiles = (const uint4 *)p.grp.base + ((int64_t)b * p.grp.n_heads + hg) * p.grp.n_tiles * TILE_U4 + lane;
  // The split's range of tiles.  With a skew, consecutive splits share their two ranges unevenly: workgroups
  // go to the eight XCDs round robin by their linear index, and the XCDs of even index stream from HBM about
  // 6 % faster than the odd ones (measured; the launch ends with its slowest workgroup), so the split that
  // lands on an even XCD takes tile_skew tiles more and its neighbour as many fewer.  A wrong guess of the
  // placement costs time, never correctness: the ranges still tile the cache exactly once.
  int t0, t1;
  zz_split_range(split, n_splits, p.tiles_per_split, p.tile_skew,
                 (int)(gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z)) & 1, n_tiles_valid, &t0, &t1);
  const int last_tile = n_tiles_valid - 1;
  const bool partial_tail = (n_valid & 31) != 0;

  f32x4 acc[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = ZZ_NEG_INF, l = 0.f;

  auto load_tile = [&](uint4(&kv)[2 * NL], int t) __attribute__((always_inline)) {
    const uint4 *src = tiles + (int64_t)t * TILE_U4;
#pragma unroll
    for (int i = 0; i < 2 * NL; ++i) kv[i] = load_stream(src + i * 64);
  };

  // ---- fused append (decode step): the newest token's K, V rows ----
  // Exactly one wave of the grid reads the tile the new token belongs to.  That wave
  // overwrites, in the registers it has just loaded, the lanes' pieces of the new
  // token's slot with the new rows, and stores the same pieces to the cache for the
  // steps to come; nobody else reads that slot in this launch, and what it held (the
  // token evicted from a ring, or nothing) is replaced in registers whatever the load saw.
  const int tile_new = new_slot >> 5;  // new_slot < 0: nothing to append
  const bool owner = new_slot >= 0 && tile_new >= t0 + wave && tile_new < t1 && ((tile_new - t0 - wave) & (WAVES - 1)) == 0;
  uint4 knew[KS];
  unsigned short vnew[NL];
  if (owner) {
    const uint4 *kp = (const uint4 *)p.k_new + ((int64_t)b * p.n_kv_heads + g) * (D / 8) + kg;
    const unsigned short *vp = (const unsigned short *)p.v_new + ((int64_t)b * p.n_kv_heads + g) * D + col;
#pragma unroll
    for (int s = 0; s < KS; ++s) knew[s] = kp[4 * s];
    if (p.rope_cos) {
      // chunk 4s + kg of the row pairs with the chunk D/16 further on or back: the same lane's s +- KS/2
      uint4 turned[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const bool upper = s >= KS / 2;
        const int64_t row = (int64_t)new_pos * (D / 2) + 8 * ((4 * s + kg) % (D / 16));
        turned[s] = rope_chunk(knew[s], knew[upper ? s - KS / 2 : s + KS / 2], p.rope_cos + row, p.rope_sin + row, upper);
      }
#pragma unroll
      for (int s = 0; s < KS; ++s) knew[s] = turned[s];
    }
#pragma unroll
    for (int i = 0; i < NL; ++i) vnew[i] = vp[16 * i];
  }
  auto patch_new_token = [&](uint4(&kv)[2 * NL]) __attribute__((always_inline)) {
    if (!ZZ_SLOT_WRITE_OK(new_slot < p.grp.capacity && tile_new < p.grp.n_tiles, lane == 0 ? p.debug_word : nullptr)) return;
    const int tn = new_slot & 31, jn = tn & 15, kgn = jn >> 2;
    const int en = 4 * (tn >> 4) + (tn & 3);  // which of the lane's 8 V tokens
    uint4 *tile = const_cast<uint4 *>(tiles) - lane + (int64_t)tile_new * TILE_U4;
    // (value selects with constant register indices: a conditional store into kv[] would
    // turn into an indexed one and push the tile buffers out of registers)
    const bool in_lo = col == jn && tn < 16, in_hi = col == jn && tn >= 16;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      kv[s] = pick(in_lo, knew[s], kv[s]);
      kv[KS + s] = pick(in_hi, knew[s], kv[KS + s]);
      if (col == jn) tile[((tn >> 4) * (D / 8) + 4 * s + kg) * 16 + jn] = knew[s];
    }
    if (kg == kgn) {
      unsigned short *vt = (unsigned short *)tile + 32 * D;
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        unsigned w[4] = {kv[NL + i].x, kv[NL + i].y, kv[NL + i].z, kv[NL + i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const unsigned lo = (en == 2 * j) ? (unsigned)vnew[i] : (w[j] & 0xffffu);
          const unsigned hi = (en == 2 * j + 1) ? ((unsigned)vnew[i] << 16) : (w[j] & 0xffff0000u);
          w[j] = lo | hi;
        }
        kv[NL + i] = make_uint4(w[0], w[1], w[2], w[3]);
        vt[(((i * 4 + kgn) * 16 + col) << 3) + en] = vnew[i];
      }
    }
  };

  auto compute = [&](uint4(&kv)[2 * NL], int t) __attribute__((always_inline)) {
    if (owner && t == tile_new) patch_new_token(kv);
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kv[s]), qop[s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kv[KS + s]), qop[s], s1, 0, 0, 0);
    }
    float x[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      x[r] = s0[r] * p.scale_log2e;
      x[4 + r] = s1[r] * p.scale_log2e;
    }
    if (partial_tail && t == last_tile) {
      // slots past n_valid were never written: no score, and their V bits (possibly
      // NaN patterns) must not reach the accumulating MFMA
      const int base = t * 32 + 4 * kg;
      unsigned int keep[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (base + r >= n_valid) x[r] = ZZ_NEG_INF;
        if (base + 16 + r >= n_valid) x[4 + r] = ZZ_NEG_INF;
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int s_lo = base + (w >= 2 ? 16 : 0) + 2 * (w & 1);
        keep[w] = (s_lo < n_valid ? 0x0000ffffu : 0u) | (s_lo + 1 < n_valid ? 0xffff0000u : 0u);
      }
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        kv[NL + i].x &= keep[0];
        kv[NL + i].y &= keep[1];
        kv[NL + i].z &= keep[2];
        kv[NL + i].w &= keep[3];
      }
    }
    float alpha;
    const bf16x8 P = softmax_step(x, m, l, alpha);
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int i = 0; i < NL; ++i) acc[i] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < NL; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kv[NL + i]), P, acc[i], 0, 0, 0);
  };

  if constexpr (WAVES == 8) {
    // at most two tiles per wave (the launcher guarantees t1 - t0 <= 16): both requested at once
    uint4 bufA[2 * NL], bufB[2 * NL];
    const int ta = t0 + wave, tb = ta + WAVES;
    if (ta < t1) load_tile(bufA, ta);
    if (tb < t1) load_tile(bufB, tb);
    if (ta < t1) compute(bufA, ta);
    if (tb < t1) compute(bufB, tb);
  } else {
    uint4 bufA[2 * NL], bufB[2 * NL];
    int t = t0 + wave;
    if (t < t1) load_tile(bufA, t);
    for (; t < t1; t += 2 * WAVES) {
      const int tn = t + WAVES;
      if (tn < t1) load_tile(bufB, tn);
      compute(bufA, t);
      if (tn < t1) {
        if (tn + WAVES < t1) load_tile(bufA, tn + WAVES);
        compute(bufB, tn);
      }
    }
  }

  // ---- combine the four waves of the workgroup through LDS ----
  __shared__ float s_o[WAVES][COLS][OP];
  __shared__ float s_m[WAVES][COLS];
  __shared__ float s_l[WAVES][COLS];
  float l_tot = l + xor_lanes(l, 16);
  l_tot += xor_lanes(l_tot, 32);
  if (col < G) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) s_o[wave][col][16 * i + 4 * kg + r] = acc[i][r];
    if (kg == 0) {
      s_m[wave][col] = m;
      s_l[wave][col] = l_tot;
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += NT) {
    const int c = idx / D, d = idx % D;
    float M = ZZ_NEG_INF;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) M = fmaxf(M, s_m[w][c]);
    const float Ms = (M == ZZ_NEG_INF) ? 0.f : M;
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float f = fast_exp2(s_m[w][c] - Ms);
      L += s_l[w][c] * f;
      O += s_o[w][c][d] * f;
    }
    const int h = g * G + c;
    if (n_splits == 1) {
      ((__bf16 *)p.out)[((int64_t)b * p.n_q_heads + h) * D + d] = (__bf16)(O / L);
    } else {
      const int64_t row = ((int64_t)b * p.n_q_heads + h) * ZZ_MAX_SPLITS + split;
      store_device_coherent(p.part_o + row * D + d, O);
      if (d == 0) {
        store_device_coherent(p.part_ml + row * 2, M);
        store_device_coherent(p.part_ml + row * 2 + 1, L);
      }
    }
  }
  if (n_splits == 1) return;

  // ---- cross-split log-sum-exp combine by whichever workgroup of the unit ends last ----
  // The partial stores above are device-coherent; each wave waits until its own have
  // completed (vmcnt reaches 0 only when the stores are acknowledged), the barrier
  // collects the four waves, then one thread counts the workgroup in.  The
  // workgroup that completes the count reads every partial of the unit back with
  // device-coherent loads, writes the output and re-arms the counter.
  // What this leans on, all of it gfx950 behaviour rather than the language's memory model: a store
  // with the device-coherent policy is acknowledged (vmcnt drops) only once it is visible to
  // every compute unit of the device; the counter is a device-scope atomic executed in order after
  // that wait; the merging workgroup's loads carry the same policy and so never hit a line an L2 of
  // another XCD kept.  The signal fences keep the compiler from moving the stores, the wait, the
  // increment and the loads across one another (the asm statement's memory clobber does the same).
  __shared__ int s_is_last;
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int *counter = p.counters + b * p.n_kv_heads + g;
  if (threadIdx.x == 0)
    s_is_last = (__hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_splits - 1);
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __syncthreads();
  if (!s_is_last) return;
  // Three short phases instead of one thread walking all splits (each device-coherent
  // load is a full memory round trip): (1) all (max, sum) pairs of the unit into LDS, one
  // per thread; (2) one wave per column turns them into normalised weights 2^(m_s-M)/L
  // with lane-parallel reductions; (3) each output element is a weighted sum of its
  // partials, loads issued eight at a time.  The cross-wave buffer is free by now.
  float *s_ms = &s_o[0][0][0];                   // [COLS][ZZ_MAX_SPLITS] maxima, then weights
  float *s_ls = s_ms + COLS * ZZ_MAX_SPLITS;     // [COLS][ZZ_MAX_SPLITS] sums
  static_assert(sizeof(s_o) >= 2 * COLS * ZZ_MAX_SPLITS * sizeof(float), "merge scratch fits the reduction buffer");
  const int ns = n_splits;
  for (int idx = threadIdx.x; idx < G * ns; idx += NT) {
    const int c = idx / ns, s = idx - c * ns;
    const int64_t row = ((int64_t)b * p.n_q_heads + g * G + c) * ZZ_MAX_SPLITS + s;
    s_ms[c * ZZ_MAX_SPLITS + s] = load_device_coherent(p.part_ml + row * 2);
    s_ls[c * ZZ_MAX_SPLITS + s] = load_device_coherent(p.part_ml + row * 2 + 1);
  }
  __syncthreads();
  for (int c = wave; c < G; c += WAVES) {
    float m0 = lane < ns ? s_ms[c * ZZ_MAX_SPLITS + lane] : ZZ_NEG_INF;
    float m1 = lane + 64 < ns ? s_ms[c * ZZ_MAX_SPLITS + lane + 64] : ZZ_NEG_INF;
    float M = fmaxf(m0, m1);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, xor_lanes(M, o));
    const float f0 = lane < ns ? fast_exp2(m0 - M) : 0.f;        // every split saw at least one key: M is finite
    const float f1 = lane + 64 < ns ? fast_exp2(m1 - M) : 0.f;
    float L = (lane < ns ? s_ls[c * ZZ_MAX_SPLITS + lane] * f0 : 0.f) +
              (lane + 64 < ns ? s_ls[c * ZZ_MAX_SPLITS + lane + 64] * f1 : 0.f);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) L += xor_lanes(L, o);
    const float inv = 1.0f / L;
    if (lane < ns) s_ms[c * ZZ_MAX_SPLITS + lane] = f0 * inv;
    if (lane + 64 < ns) s_ms[c * ZZ_MAX_SPLITS + lane + 64] = f1 * inv;
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += NT) {
    const int c = idx / D, d = idx % D;
    const int h = g * G + c;
    const float *po = p.part_o + ((int64_t)b * p.n_q_heads + h) * ZZ_MAX_SPLITS * D + d;
    const float *wt = s_ms + c * ZZ_MAX_SPLITS;
    float O = 0.f;
    int s = 0;
    for (; s + 8 <= ns; s += 8) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = load_device_coherent(po + (int64_t)(s + j) * D);
#pragma unroll
      for (int j = 0; j < 8; ++j) O = fmaf(v[j], wt[s + j], O);
    }
    if (s < ns) {
      // the last, incomplete group also goes out as eight loads at once (indices past the last split
      // repeat it with weight zero): single loads would each wait out a whole round trip
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = load_device_coherent(po + (int64_t)min(s + j, ns - 1) * D);
#pragma unroll
      for (int j = 0; j < 8; ++j) O = fmaf(v[j], s + j < ns ? wt[s + j] : 0.f, O);
    }
    ((__bf16 *)p.out)[((int64_t)b * p.n_q_heads + h) * D + d] = (__bf16)O;
  }
  if (threadIdx.x == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D>
__global__ __launch_bounds__(256) void zz_decode_kernel(zz_decode_params p) {
  decode_body<D, 4>(p, blockIdx.x, blockIdx.z, p.n_valid, p.n_tiles_valid, p.n_splits, p.new_slot, p.new_pos);
}

// Short caches (one workgroup per unit, at most 16 tiles: a streaming head's sink + window):
// eight waves, so that every wave has at most two tiles and requests both at once.  The launch
// is a chain of latencies (dispatch, one memory round trip, two tiles of arithmetic, the merge
// through LDS) instead of two or three round trips in a row.  Group sizes up to 8.
template <int D>
__global__ __launch_bounds__(512) void zz_decode_short_kernel(zz_decode_params p) {
  decode_body<D, 8>(p, blockIdx.x, blockIdx.z, p.n_valid, p.n_tiles_valid, p.n_splits, p.new_slot, p.new_pos);
}

// Sequences of different lengths: grid (all workgroups of all sequences, heads of the group).
// A workgroup finds its sequence in the prefix sums of the per-sequence split counts (a scan
// over scalar kernel arguments) and derives that sequence's occupied slots and the slot of
// its newest token from its length; the rest is the kernel above.
template <int D, int WAVES>
__device__ __forceinline__ void decode_ragged_body(const zz_decode_ragged_params &p) {
  const int wg = blockIdx.x;
  int b = 0;
  while (b + 1 < p.u.batch && p.first_wg[b + 1] <= wg) ++b;
  const int split = wg - p.first_wg[b];
  const int n_splits = p.first_wg[b + 1] - p.first_wg[b];
  const int len = (int)p.seq_len[b];
  const bool streaming = p.u.grp.streaming != 0;
  const int n_valid = streaming ? min(len, p.sink + p.window) : len;
  const int newest = len - 1;
  const int slot = (!streaming || newest < p.sink) ? newest : p.sink + (newest - p.sink) % p.window;
  decode_body<D, WAVES>(p.u, split, b, n_valid, (n_valid + 31) >> 5, n_splits, p.u.new_slot >= 0 ? slot : -1, newest);
}

template <int D>
__global__ __launch_bounds__(256) void zz_decode_ragged_kernel(zz_decode_ragged_params p) {
  decode_ragged_body<D, 4>(p);
}
// every sequence's cache is short (one workgroup each, at most 16 tiles): eight waves, as above
template <int D>
__global__ __launch_bounds__(512) void zz_decode_ragged_short_kernel(zz_decode_ragged_params p) {
  decode_ragged_body<D, 8>(p);
}

// Zeroes the split counters once per context (the library never memsets caller memory).
__global__ void zz_zero_kernel(int *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// --------------------------------------------------------------------------
// Prefill: flash-style over KV tiles, columns = 16 query positions of one head.
// A workgroup owns 4*QW consecutive query positions of one KV head; wave w owns
// QW = 16*NB/Gc of them as NB column blocks (Gc heads x NB/Gc blocks of 16
// positions), so every K/V operand it reads from LDS feeds NB MFMAs.
//
// K/V tiles travel HBM/L2 -> LDS once per workgroup with direct-to-LDS loads
// (global_load_lds_dwordx4: each wave deposits 1 KiB chunks, lane L at byte L*16,
// i.e. the operand image unchanged) into two rings of four half-tiles (K parts,
// V parts); every wave reads operands back with conflict-free ds_read_b128.
//
// The loop is software-pipelined over three tiles, so that the three stages of an
// iteration are independent of each other:
//     iteration n:   S(n+1) = K(n+1) Q^T        (MFMA)
//                    O     += V(n-1)^T P(n-1)   (MFMA)
//                    P(n)   = softmax step on S(n)   (VALU)
// Two workgroups are resident per compute unit, i.e. two waves per SIMD: while one runs
// its block of MFMAs the other runs its softmax on the vector ALU.
// The running reference maximum is only raised when a column's scores exceed it by
// more than 2^8 (exact in fp32/bf16, P stays <= 256), so the accumulators are
// rescaled a handful of times per query, not whenever a new maximum appears.
//
// Keys come from the cached tiles (positions < n_past), then from the staged chunk
// (position = n_past + index).  Staged tiles no query of the workgroup can see
// (above the diagonal; for streaming heads also between sink and window) are never
// loaded.  grid (query blocks, heads of the group * head chunks, B), 4 waves.
// --------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void lds_void;

// N consecutive 1 KiB chunks, global -> LDS, without passing through registers: lane L's
// 16 bytes at src_lane + j*1024 land at LDS byte lds_base + j*1024 + L*16.  Written as
// asm so that the compiler's wait-count insertion does not tie every later LDS read to
// these loads (it would wait for all of them, prefetches included); the loop below
// waits with an explicit vmcnt for exactly the tiles it is about to read.
template <int N>
__device__ __forceinline__ void dma_to_lds(const void *tile_base, unsigned lane_byte_off, unsigned lds_base) {
  // tile_base and lds_base are wave-uniform (scalar registers); only the lane offset is a vector.
  // The compiler does not look inside an asm statement when it inserts wait states: the
  // s_nop 4 covers both a scalar register written by v_readfirstlane just before (five wait
  // states before a memory instruction may read it) and the write of M0 (one).
  static_assert(N == 1 || N == 2, "chunks per wave");
  // (the builtin returns a signed int: both halves go through unsigned before they are joined)
  const unsigned long long a = (unsigned long long)tile_base;
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)a);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32));
  const unsigned long long sbase = ((unsigned long long)hi << 32) | (unsigned long long)lo;
  if constexpr (N == 2)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\t"
                 "global_load_lds_dwordx4 %0, %1\n\t"
                 "global_load_lds_dwordx4 %0, %1 offset:1024" ::"v"(lane_byte_off), "s"(sbase), "s"(lds_base)
                 : "memory", "m0");
  if constexpr (N == 1)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 4\n\t"
                 "global_load_lds_dwordx4 %0, %1" ::"v"(lane_byte_off), "s"(sbase), "s"(lds_base)
                 : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Maximum over the four key groups of a column: lanes L, L^16, L^32, L^48.
// v_permlane16_swap exchanges the odd 16-lane rows of its first register with the even rows of
// its second, v_permlane32_swap the upper half of the first with the lower half of the second;
// started from two copies of a value, each step leaves every lane with its own value in one
// register and its partner's in the other.  Written as asm: through the builtin this compiler
// reads both results from the first register, so the maximum of the pair degenerates to a
// broadcast of key group 0.  (s_nop: the compiler does not insert the wait states a VALU write
// needs before a lane-permuting read inside an asm statement.)
__device__ __forceinline__ float max_over_kg(float v) {
  float a = v, b = v;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\tv_max_f32 %0, %0, %1" : "+v"(a), "+v"(b));
  b = a;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_max_f32 %0, %0, %1" : "+v"(a), "+v"(b));
  return a;
}

#define ZZ_RESCALE_THRESHOLD 8.0f  // in log2 units

// PAIRED: two such groups of four waves in one workgroup, on two head chunks of the same KV head and the
// same query positions.  They share the K/V ring (each tile is requested once for both) and, in the
// pipelined loop, run half an iteration apart: every SIMD holds one wave of each group, and while one
// group is in its matrix stage the other is in its softmax stage, held there by workgroup barriers
// between the stages.  (Two independent workgroups per compute unit fall into step with each other
// instead: both in the matrix stage, then both in the softmax stage, with the matrix pipe idle.)
template <int D, int NB, bool PAIRED>
__global__ __launch_bounds__(PAIRED ? 512 : 256, PAIRED ? 1 : ZZ_PREFILL_WG_PER_CU) void zz_prefill_kernel(zz_prefill_params p, zz_seq_lens sl, int Gc) {
  constexpr int KS = D / 32, NL = D / 16, HALF_U4 = 4 * D, TILE_U4 = 8 * D;
  constexpr int RING_WAVES = PAIRED ? 2 * ZZ_WAVES_PER_WG : ZZ_WAVES_PER_WG;   // waves that fill the ring together
  constexpr int CPW = NL / RING_WAVES;  // 1 KiB chunks of a K part (or V part) each wave brings in
  static_assert(CPW >= 1 && CPW * RING_WAVES == NL, "a part's chunks divide evenly over the waves");
  constexpr int RING = 4;  // power of two: the slot of tile n is n & 3
  __shared__ uint4 s_k[RING][HALF_U4];
  __shared__ uint4 s_v[RING][HALF_U4];

  const int lane = threadIdx.x & 63;
  const int ring_wave = threadIdx.x >> 6;             // the wave's place among those that fill the ring
  const int wave = ring_wave & (ZZ_WAVES_PER_WG - 1);   // ... among the four that share its query block
  const int pair_group = ring_wave / ZZ_WAVES_PER_WG;   // 0, or 1 for the second group of a paired workgroup
  const int col = lane & 15, kg = lane >> 4;
  const int G = p.group_size;
  const int n_hchunks = G / Gc;
  const int ny = PAIRED ? n_hchunks / 2 : n_hchunks;    // workgroups per KV head along y
  const int hg = blockIdx.y / ny, hc = PAIRED ? 2 * (blockIdx.y % ny) + pair_group : blockIdx.y % ny;
  const int b = blockIdx.z;
  const int n_past = sl.ragged ? (int)sl.len[b] : p.n_past;   // tokens this sequence holds already
  const int g = p.heads[hg];
  const int QW = 16 * (NB / Gc);
  // later query blocks see more staged keys: they are dispatched first, so the launch does not end
  // on its longest workgroups
  const int iq_wg = (gridDim.x - 1 - blockIdx.x) * ZZ_WAVES_PER_WG * QW;  // first query index of the workgroup
  const int iq0 = iq_wg + wave * QW;                    // ... of the wave (may lie past n_new: an idle wave
                                                        // computes on masked columns and stores nothing)
  const int i_lo = n_past + iq0;                      // the wave's first query position
  const int I_lo = n_past + iq_wg;                    // the workgroup's range of query positions
  const int I_hi = n_past + min(iq_wg + ZZ_WAVES_PER_WG * QW, p.n_new) - 1;
  const bool streaming = p.grp.streaming != 0;
  const int S = p.sink, W = p.window;
  const float c = p.scale_log2e;

  // ---- the workgroup's tile sequence ----
  // Cached tiles come before staged tiles, except that tiles which are "plain" for all
  // four waves (every slot occupied, every key visible to every query: full cached tiles
  // of a retrieval head and staged tiles wholly before the workgroup's first query) are
  // taken first, by the pipelined loop without any mask arithmetic; softmax does not care
  // about the order of keys.  The rest (ragged last cached tile, diagonal and tail tiles,
  // everything of a streaming head) goes through the masked loop.
  const int occ = streaming ? min(n_past, S + W) : n_past;
  const int n_ct = (occ + 31) >> 5;
  const int k_hi = (I_hi - n_past) >> 5;
  int ks_end = 0, kw_begin = 0;
  if (streaming) {
    if (n_past < S) ks_end = min(k_hi, (S - 1 - n_past) >> 5) + 1;  // sink tokens arriving with this chunk
    const int first_win = I_lo - W + 1 - n_past;                      // oldest window token, as a chunk index
    kw_begin = max(ks_end, first_win > 0 ? first_win >> 5 : 0);
  }
  const int n_tiles = n_ct + ks_end + max(0, k_hi - kw_begin + 1);
  const int nc_full = streaming ? 0 : occ >> 5;        // plain cached tiles
  const int ns_plain = streaming ? 0 : iq_wg >> 5;     // plain staged tiles (iq_wg is a multiple of 64)
  int n_fast = nc_full + ns_plain;
  if (!(n_fast & 1)) n_fast = max(n_fast - 1, 0);      // the pipelined loop takes 1 + 2k tiles
  const uint4 *ctiles = (const uint4 *)p.grp.base + ((int64_t)b * p.grp.n_heads + hg) * p.grp.n_tiles * TILE_U4;
  const uint4 *stiles = (const uint4 *)p.stage + ((int64_t)b * p.n_kv_heads + g) * p.stage_tiles * TILE_U4;

  // n-th tile of the sequence -> (pointer, cache tile index or -1, staged tile index or -1)
  auto tile_src = [&](int n, int &ct, int &sk) -> const uint4 * {
    ct = sk = -1;
    if (streaming) {
      if (n < n_ct) {
        ct = n;
      } else {
        const int m = n - n_ct;
        sk = m < ks_end ? m : kw_begin + (m - ks_end);
      }
    } else if (n < nc_full) {
      ct = n;
    } else if (n < nc_full + ns_plain) {
      sk = n - nc_full;
    } else if (n < n_ct + ns_plain) {
      ct = nc_full;  // the ragged last cached tile
    } else {
      sk = n - n_ct;
    }
    return ct >= 0 ? ctiles + (int64_t)ct * TILE_U4 : stiles + (int64_t)sk * TILE_U4;
  };
  // Requests for the K part / V part of the n-th tile of the sequence into ring slot n & 3.
  // Each wave brings CPW KiB-chunks of the part; the tile address stays in scalar registers.
  const unsigned lane_off = (unsigned)(ring_wave * CPW * 64 + lane) * 16u;
  const unsigned lds_k0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void *)&s_k[0][ring_wave * CPW * 64]);
  const unsigned lds_v0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void *)&s_v[0][ring_wave * CPW * 64]);
  auto issue_k = [&](int n) {
    int ct, sk;
    const uint4 *src = tile_src(n, ct, sk);
    dma_to_lds<CPW>(src, lane_off, lds_k0 + (unsigned)(n & (RING - 1)) * (HALF_U4 * 16));
  };
  auto issue_v = [&](int n) {
    int ct, sk;
    const uint4 *src = tile_src(n, ct, sk) + HALF_U4;
    dma_to_lds<CPW>(src, lane_off, lds_v0 + (unsigned)(n & (RING - 1)) * (HALF_U4 * 16));
  };
  // ---- per column block: head, query position, Q operand ----
  int qpos[NB];
  bf16x8 qop[NB][KS];
#pragma unroll
  for (int cb = 0; cb < NB; ++cb) {
    const int h = g * G + hc * Gc + cb % Gc;
    const int iq = iq0 + (cb / Gc) * 16 + col;
    const bool ok = iq < p.n_new;
    qpos[cb] = ok ? n_past + iq : -1;  // -1: sees nothing, output not stored
    const uint4 *qp = (const uint4 *)p.q + (((int64_t)b * p.n_new + (ok ? iq : 0)) * p.n_q_heads + h) * (D / 8) + kg;
#pragma unroll
    for (int s = 0; s < KS; ++s) qop[cb][s] = as_bf16x8(qp[4 * s]);
  }
  // Make the Q loads land here.  Otherwise their waits sit at their first use inside the
  // loop, and since the DMA loads are invisible to the compiler's counting, those waits
  // would also drain every K/V prefetch, in every iteration.
#pragma unroll
  for (int cb = 0; cb < NB; ++cb)
#pragma unroll
    for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qop[cb][s]));

  f32x4 acc[NB][NL];
  f32x4 lsum[NB];       // row sums of P, produced by an MFMA against an all-ones operand
  float mc[NB];         // reference maxima, in log2 units (score * scale * log2 e); -inf: nothing seen yet
  float nref[NB];       // what the fast path adds to score * c: minus the reference (0 while it is -inf)
  float thr[NB];        // exponent above which the reference must be raised: -inf until a key has been seen
  float alpha_pend[NB]; // factor the accumulators still have to be multiplied by
  bool pend = false;
#pragma unroll
  for (int cb = 0; cb < NB; ++cb) {
    mc[cb] = ZZ_NEG_INF;
    nref[cb] = 0.f;
    thr[cb] = ZZ_NEG_INF;
    alpha_pend[cb] = 1.f;
    lsum[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NL; ++i) acc[cb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  // ---- the three stages ----
  // LDS -> registers: the K operands of tile n (token block 0 then 1, per k-step) ...
  auto read_k = [&](int n, uint4(&kop)[2 * KS]) {
    const uint4 *kt = &s_k[n & (RING - 1)][0] + lane;
#pragma unroll
    for (int i = 0; i < 2 * KS; ++i) kop[i] = kt[i * 64];
  };
  // ... and V operands [k0, k1) of tile n (one per 16 head dimensions)
  auto read_v = [&](int n, uint4(&vop)[NL], int k0, int k1) {
    const uint4 *vt = &s_v[n & (RING - 1)][0] + lane;
#pragma unroll
    for (int k = 0; k < NL; ++k)
      if (k >= k0 && k < k1) vop[k] = vt[k * 64];
  };
  auto qk_mfma = [&](const uint4(&kop)[2 * KS], f32x4(&s0)[NB], f32x4(&s1)[NB]) {
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) s0[cb] = s1[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) {
        s0[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kop[s]), qop[cb][s], s0[cb], 0, 0, 0);
        s1[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kop[KS + s]), qop[cb][s], s1[cb], 0, 0, 0);
      }
    }
  };
  auto qk = [&](int n, f32x4(&s0)[NB], f32x4(&s1)[NB]) {
    uint4 kop[2 * KS];
    read_k(n, kop);
    qk_mfma(kop, s0, s1);
  };
  // masks of tile n: -inf into the scores of keys a query may not see, and which of the
  // lane's 8 V tokens exist at all (empty slots may hold NaN bit patterns)
  auto mask_tile = [&](int n, f32x4(&s0)[NB], f32x4(&s1)[NB], unsigned(&keep)[4]) {
    int ct, sk;
    (void)tile_src(n, ct, sk);
    bool plain;  // every key of the tile exists and is visible to every query of the wave
    if (ct >= 0)
      plain = !streaming && ct * 32 + 32 <= occ;
    else
      plain = !streaming && sk * 32 + 32 <= p.n_new && n_past + sk * 32 + 31 <= i_lo && iq0 + QW <= p.n_new;
    if (plain) {
      keep[0] = keep[1] = keep[2] = keep[3] = 0xffffffffu;
      return;
    }
    int pos[8];
    const int newest = n_past - 1 - S;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int t = (e < 4 ? 0 : 16) + 4 * kg + (e & 3);
      int ps = -1;
      if (ct >= 0) {
        const int slot = ct * 32 + t;
        if (slot < occ) ps = (!streaming || slot < S) ? slot : slot + W * ((newest - (slot - S)) / W);
      } else {
        const int idx = sk * 32 + t;
        if (idx < p.n_new) ps = n_past + idx;
      }
      pos[e] = ps;
    }
#pragma unroll
    for (int w = 0; w < 4; ++w)
      keep[w] = (pos[2 * w] >= 0 ? 0x0000ffffu : 0u) | (pos[2 * w + 1] >= 0 ? 0xffff0000u : 0u);
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
      const int i = qpos[cb];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int j = pos[e];
        const bool vis = (j >= 0) && (j <= i) && (!streaming || j < S || i - j < W);
        if (!vis) {
          if (e < 4)
            s0[cb][e & 3] = ZZ_NEG_INF;
          else
            s1[cb][e & 3] = ZZ_NEG_INF;
        }
      }
    }
  };
  // Softmax step of one tile.  Fast path: x = score * c - reference (one fma per score, computed
  // anyway), the lane's largest x, one compare per column block: a reference is only raised when
  // some score of the column exceeds it by 2^8, and no lane can see that without its own x
  // exceeding the threshold, so while no lane of the wave does, nothing else happens and
  // P = 2^x.  (The maxima are taken over fma results, which the compiler knows to be
  // canonical: v_max3 without the quieting v_max x, x in front of every input that it puts
  // before maxima of raw MFMA results.)  Otherwise, a few times per query: raise().
  auto exponents = [&](const f32x4(&s0)[NB], const f32x4(&s1)[NB], float(&x)[NB][8]) {
#pragma unroll
    for (int cb = 0; cb < NB; ++cb)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        x[cb][r] = fmaf(s0[cb][r], c, nref[cb]);
        x[cb][4 + r] = fmaf(s1[cb][r], c, nref[cb]);
      }
  };
  // lm[cb]: the lane's largest exponent against the current reference.  New reference of a
  // column whose largest score exceeds the old one by more than the threshold (always, for the
  // first key a column sees): that largest score, over all four key groups.
  auto raise = [&](const float(&lm)[NB]) {
    bool grew = false;
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
      const float mxc = max_over_kg(lm[cb]) - nref[cb];     // back to score * c (nref is 0 or -reference)
      const float old = mc[cb];
      const bool grow = mxc > old + ZZ_RESCALE_THRESHOLD;   // also true for the first visible key (old = -inf)
      const float ref = grow ? mxc : old;
      const bool seen = ref != ZZ_NEG_INF;
      alpha_pend[cb] = grow ? alpha_pend[cb] * fast_exp2(old - ref) : alpha_pend[cb];   // old = -inf: 0 times an empty sum
      mc[cb] = ref;
      nref[cb] = seen ? -ref : 0.f;
      thr[cb] = seen ? ZZ_RESCALE_THRESHOLD : ZZ_NEG_INF;
      grew |= grow;
    }
    pend |= grew;
  };
  auto softmax = [&](const f32x4(&s0)[NB], const f32x4(&s1)[NB], bf16x8(&P)[NB]) {
    float x[NB][8], lm[NB];
    exponents(s0, s1, x);
    bool trig = false;
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
      lm[cb] = fmaxf(fmaxf(fmaxf(x[cb][0], x[cb][1]), fmaxf(x[cb][2], x[cb][3])),
                     fmaxf(fmaxf(x[cb][4], x[cb][5]), fmaxf(x[cb][6], x[cb][7])));
      trig |= lm[cb] > thr[cb];
    }
    if (__any(trig)) {
      raise(lm);
      exponents(s0, s1, x);
    }
#pragma unroll
    for (int cb = 0; cb < NB; ++cb)
#pragma unroll
      for (int e = 0; e < 8; ++e) P[cb][e] = (__bf16)fast_exp2(x[cb][e]);
  };
  auto rescale = [&]() {
    if (__any(pend)) {
#pragma unroll
      for (int cb = 0; cb < NB; ++cb) {
        lsum[cb] *= alpha_pend[cb];
#pragma unroll
        for (int k = 0; k < NL; ++k) acc[cb][k] *= alpha_pend[cb];
        alpha_pend[cb] = 1.f;
      }
      pend = false;
    }
  };
  auto pv_mfma = [&](const uint4(&vop)[NL], const bf16x8(&P)[NB], const unsigned *keep) {
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      uint4 vraw = vop[k];
      if (keep) {
        vraw.x &= keep[0];
        vraw.y &= keep[1];
        vraw.z &= keep[2];
        vraw.w &= keep[3];
      }
      const bf16x8 vk = as_bf16x8(vraw);
#pragma unroll
      for (int cb = 0; cb < NB; ++cb)
        acc[cb][k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vk, P[cb], acc[cb][k], 0, 0, 0);
    }
#pragma unroll
    for (int cb = 0; cb < NB; ++cb)
      lsum[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, P[cb], lsum[cb], 0, 0, 0);
  };
  auto pv = [&](int n, const bf16x8(&P)[NB], const unsigned *keep) {
    uint4 vop[NL];
    read_v(n, vop, 0, NL);
    pv_mfma(vop, P, keep);
  };

  // The values a stage hands to the next iteration are pinned where they are produced:
  // being pure register arithmetic, the compiler would otherwise sink the whole softmax
  // step down to the first use of P, one barrier later, and undo the overlap.
  auto pin_p = [&](bf16x8(&P)[NB]) {
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) asm volatile("" : "+v"(P[cb]));
  };
  auto pin = [&](f32x4(&s0)[NB], f32x4(&s1)[NB], bf16x8(&P)[NB]) {
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) asm volatile("" : "+v"(s0[cb]), "+v"(s1[cb]), "+v"(P[cb]));
  };
  // Issue order inside one iteration: the 34 MFMAs of the two matrix stages as one block at raised
  // wave priority, then the softmax arithmetic as one block.  The two waves that share a SIMD
  // (one from each resident workgroup) then fall into opposite phases, one feeding the matrix pipe
  // while the other runs on the vector ALU; left to interleave the stages instruction by
  // instruction, both waves compete for both pipes all the time (measured 4 to 7 % slower).
  auto mfma_phase_begin = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
  };
  auto mfma_phase_end = [&]() {
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- software pipeline over the plain tiles [0, n_fast) ----
  // Iteration n computes scores of tile n+1 and P V of tile n-1, then softmax of tile n; the loop body
  // is two iterations (registers alternate between the A and B sets) behind one barrier.
  // Ring slot of tile t is t & 3, for K parts and V parts alike.
  // Every instruction of the loop costs its wave an issue slot, scalar ones and waits included, and
  // the two waves of a SIMD hardly issue side by side: the body is kept short.  Tile requests walk the
  // sequence with a running pointer each (K requests run ahead of V requests), the body is written
  // for a constant ring slot (two copies: tiles 1,2 mod 4 and 3,0 mod 4), all operands of a matrix
  // stage are requested before the softmax next to it and waited for once.
  // kq / vq (masked loop): next tile whose K part / V part has not been requested yet.
  int kq = 0, vq = 0;
  if (n_fast > 0) {
    f32x4 sA0[NB], sA1[NB], sB0[NB], sB1[NB];
    bf16x8 PA[NB], PB[NB];
    // The fast sequence is the full cached tiles, then staged tiles; requests past its end (the loop
    // requests a fixed distance ahead) go on into staged tiles nobody reads: valid memory (the staging
    // area is padded for them), landing in ring slots the loop is done with.
    const char *const cached_end = (const char *)(ctiles + (int64_t)nc_full * TILE_U4);
    const char *pk = nc_full > 0 ? (const char *)ctiles : (const char *)stiles;
    const char *pvv = pk;
    auto next_tile = [&](const char *&ptr) -> const char * {
      const char *cur = ptr;
      ptr += TILE_U4 * 16;
      ptr = ptr == cached_end ? (const char *)stiles : ptr;
      return cur;
    };
    auto request_k = [&](int slot) { dma_to_lds<CPW>(next_tile(pk), lane_off, lds_k0 + (unsigned)slot * (HALF_U4 * 16)); };
    auto request_v = [&](int slot) {
      dma_to_lds<CPW>(next_tile(pvv) + HALF_U4 * 16, lane_off, lds_v0 + (unsigned)slot * (HALF_U4 * 16));
    };
    if constexpr (PAIRED) {
      // Both groups in step through the first two tiles.  Requests go out in the order the loop continues them
      // (per tile n: V(n+1), then K(n+4)):  K(0) K(1) K(2) V(0) K(3) V(1), then K(4) once K(0) has been read.
      auto wg_barrier = [&]() { asm volatile("s_barrier" ::: "memory"); };
      request_k(0);
      request_k(1);
      request_k(2);
      request_v(0);
      request_k(3);
      request_v(1);
      wait_vmcnt<5 * CPW>();  // K(0)
      wg_barrier();
      qk(0, sA0, sA1);
      wait_vmcnt<4 * CPW>();  // K(1)
      wg_barrier();           // ... and every wave has read K(0)
      request_k(0);           // K(4)
      qk(1, sB0, sB1);
      softmax(sA0, sA1, PA);
      rescale();
      pin(sB0, sB1, PA);
      wait_vmcnt<3 * CPW>();  // K(2), V(0)
      wg_barrier();
      if (pair_group == 1) wg_barrier();   // the second group runs one stage behind the first from here on
      // One tile n of a group.  [softmax stage] V(n+1) and K(n+4) requested, the K operands of tile n+1 read
      // from LDS while the softmax of tile n runs; wait for them and for this wave's share of K(n+2), which
      // everyone reads two stages on; barrier.  [matrix stage] the V operands of tile n-1 read from LDS while
      // the scores of tile n+1 are computed, then P V of tile n-1; wait for this wave's share of V(n), which
      // everyone reads in the matrix stage after next; barrier.  With the first group in stage 2n and the
      // second in 2n+1 for the softmax of tile n: K(j) is last read in stage 2j-1 and its slot refilled (by
      // K(j+4)) from stage 2j on; V(j) is last read in stage 2j+4 and its slot refilled (by V(j+4)) from
      // stage 2j+6 on.
      auto half = [&](auto slot_k, auto slot_v, const f32x4(&sc0)[NB], const f32x4(&sc1)[NB], bf16x8(&Pc)[NB],
                      f32x4(&sn0)[NB], f32x4(&sn1)[NB], const bf16x8(&Pp)[NB], auto dma_k_slot, auto dma_v_slot) {
        uint4 kop[2 * KS], vop[NL];
        request_v(decltype(dma_v_slot)::value);
        request_k(decltype(dma_k_slot)::value);
        read_k(decltype(slot_k)::value, kop);
        __builtin_amdgcn_sched_barrier(0);
        softmax(sc0, sc1, Pc);
        pin_p(Pc);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): the K operands are in registers
        wait_vmcnt<4 * CPW>();                // K(n+2); later: V(n), K(n+3), V(n+1), K(n+4)
        wg_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_v(decltype(slot_v)::value, vop, 0, NL);
        __builtin_amdgcn_sched_barrier(0);
        qk_mfma(kop, sn0, sn1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0xC07F);   // the V operands are in registers
        pv_mfma(vop, Pp, nullptr);
        __builtin_amdgcn_sched_barrier(0);
        rescale();
        wait_vmcnt<3 * CPW>();                // V(n); later: K(n+3), V(n+1), K(n+4)
        wg_barrier();
        __builtin_amdgcn_sched_barrier(0);
      };
      auto pair = [&](auto s) {
        constexpr int S0 = decltype(s)::value;
        using std::integral_constant;
        // odd n = S0 (mod 4): current scores in B, previous P in A; K(n+4) goes to slot n, V(n+1) to slot n+1
        half(integral_constant<int, (S0 + 1) & 3>{}, integral_constant<int, (S0 + 3) & 3>{}, sB0, sB1, PB, sA0, sA1, PA,
             integral_constant<int, S0 & 3>{}, integral_constant<int, (S0 + 1) & 3>{});
        // even n+1
        half(integral_constant<int, (S0 + 2) & 3>{}, integral_constant<int, S0 & 3>{}, sA0, sA1, PA, sB0, sB1, PB,
             integral_constant<int, (S0 + 1) & 3>{}, integral_constant<int, (S0 + 2) & 3>{});
      };
      int n = 1;
      for (; n + 2 < n_fast; n += 4) {
        pair(std::integral_constant<int, 1>{});
        pair(std::integral_constant<int, 3>{});
      }
      if (n < n_fast) pair(std::integral_constant<int, 1>{});
      if (pair_group == 0) wg_barrier();   // the first group waits for the second group's last stage
    } else {
    request_k(0);
    request_k(1);
    wait_vmcnt<CPW>();  // K(0)
    __syncthreads();
    request_k(2);
    request_v(0);
    qk(0, sA0, sA1);
    // n = 0: no P V yet
    wait_vmcnt<2 * CPW>();
    __syncthreads();
    request_k(3);
    request_v(1);
    qk(1, sB0, sB1);
    softmax(sA0, sA1, PA);
    rescale();   // the first reference: the factor it brings belongs to the (still empty) sums before tile 0
    pin(sB0, sB1, PA);
    // One half: the matrix stage's operands (K of tile slot_k, V of tile slot_v) requested from LDS, the
    // softmax of the current tile on the vector ALU while they arrive, one wait, then the matrix stage
    // (scores of the next tile, P V of the previous one) with the wave's share of two tile requests inside.
    auto half = [&](auto slot_k, auto slot_v, const f32x4(&sc0)[NB], const f32x4(&sc1)[NB], bf16x8(&Pc)[NB],
                    f32x4(&sn0)[NB], f32x4(&sn1)[NB], const bf16x8(&Pp)[NB], auto dma_k_slot, auto dma_v_slot) {
      uint4 kop[2 * KS], vop[NL];
      read_k(decltype(slot_k)::value, kop);
      read_v(decltype(slot_v)::value, vop, 0, NL);
      __builtin_amdgcn_sched_barrier(0);
      softmax(sc0, sc1, Pc);
      pin_p(Pc);
      mfma_phase_begin();
      __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): every operand is in, no further waits among the MFMAs
      request_k(decltype(dma_k_slot)::value);
      __builtin_amdgcn_sched_barrier(0);
      qk_mfma(kop, sn0, sn1);
      request_v(decltype(dma_v_slot)::value);
      __builtin_amdgcn_sched_barrier(0);
      pv_mfma(vop, Pp, nullptr);
      mfma_phase_end();
      rescale();
      __builtin_amdgcn_sched_barrier(0);
    };
    // A pair of tiles n, n+1 with n = s (mod 4), s = 1 or 3.  At the barrier K(n+1), K(n+2), V(n-1), V(n)
    // have landed (everything requested one pair ago) and every wave is done with the previous pair,
    // whose four ring slots the requests of this pair refill: K(n+3), V(n+1), K(n+4), V(n+2).
    auto pair = [&](auto s) {
      constexpr int S0 = decltype(s)::value;
      using std::integral_constant;
      wait_vmcnt<0>();
      __syncthreads();
      // odd n: current scores in B, previous P in A
      half(integral_constant<int, (S0 + 1) & 3>{}, integral_constant<int, (S0 + 3) & 3>{}, sB0, sB1, PB, sA0, sA1, PA,
           integral_constant<int, (S0 + 3) & 3>{}, integral_constant<int, (S0 + 1) & 3>{});
      // even n+1: current scores in A, previous P in B (for the last pair the scores computed here are
      // those of tile n_fast, which the masked loop redoes)
      half(integral_constant<int, (S0 + 2) & 3>{}, integral_constant<int, S0 & 3>{}, sA0, sA1, PA, sB0, sB1, PB,
           integral_constant<int, S0 & 3>{}, integral_constant<int, (S0 + 2) & 3>{});
    };
    int n = 1;
    for (; n + 2 < n_fast; n += 4) {
      pair(std::integral_constant<int, 1>{});
      pair(std::integral_constant<int, 3>{});
    }
    if (n < n_fast) pair(std::integral_constant<int, 1>{});
    }
    // drain: the last P is in A
    wait_vmcnt<0>();
    __syncthreads();
    rescale();
    pv(n_fast - 1, PA, nullptr);
    wait_vmcnt<0>();  // the surplus requests still write LDS; the masked loop's own come after them
    kq = vq = n_fast;
  }

  // ---- masked loop over the remaining tiles, one tile per iteration ----
  for (int n = n_fast; n < n_tiles; ++n) {
    if (kq <= n) {  // only when nothing has been requested yet
      issue_k(n);
      kq = n + 1;
    }
    if (vq <= n) {
      issue_v(n);
      vq = n + 1;
    }
    wait_vmcnt<0>();
    __syncthreads();  // tile n is in; everyone is done with tile n-1
    if (kq <= n + 1 && n + 1 < n_tiles) {
      issue_k(n + 1);
      kq = n + 2;
    }
    if (vq <= n + 1 && n + 1 < n_tiles) {
      issue_v(n + 1);
      vq = n + 2;
    }
    f32x4 s0[NB], s1[NB];
    bf16x8 P[NB];
    unsigned keep[4];
    qk(n, s0, s1);
    mask_tile(n, s0, s1, keep);
    softmax(s0, s1, P);
    rescale();
    pv(n, P, keep);
  }
  wait_vmcnt<0>();  // nothing may still be writing LDS when the workgroup ends

  // ---- normalise and store ----
#pragma unroll
  for (int cb = 0; cb < NB; ++cb) {
    if (qpos[cb] < 0) continue;
    const float inv = 1.0f / lsum[cb][0];  // all 16 rows of the ones-product equal the column's sum
    const int h = g * G + hc * Gc + cb % Gc;
    const int iq = qpos[cb] - n_past;
    __bf16 *op = (__bf16 *)p.out + (((int64_t)b * p.n_new + iq) * p.n_q_heads + h) * D + 4 * kg;
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
      bf16x4 o;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[r] = (__bf16)(acc[cb][k][r] * inv);
      *(bf16x4 *)(op + 16 * k) = o;
    }
  }
}

// --------------------------------------------------------------------------
// Measurement aid: a pure streaming read of a buffer, with the decode kernel's access
// pattern (one workgroup per compute unit, each wave 16 KiB at a time, 1 KiB per load) and
// nothing else: what the memory system delivers to this pattern is the practical ceiling
// the decode kernel is compared with, next to the published peak.
// --------------------------------------------------------------------------
template <bool NT>
__global__ __launch_bounds__(256) void zz_probe_read_kernel(const uint4 *p, size_t n_blocks, uint4 *sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t per = (n_blocks + gridDim.x - 1) / gridDim.x;
  const size_t b1 = min((size_t)(blockIdx.x + 1) * per, n_blocks);
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t blk = (size_t)blockIdx.x * per + wave; blk < b1; blk += ZZ_WAVES_PER_WG) {
    const uint4 *src = p + blk * (16 * 64) + lane;
    uint4 v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = NT ? load_stream(src + i * 64) : src[i * 64];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      acc.x ^= v[i].x;
      acc.y ^= v[i].y;
      acc.z ^= v[i].z;
      acc.w ^= v[i].w;
    }
  }
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u) sink[threadIdx.x] = acc;  // keeps the loads alive
}

// --------------------------------------------------------------------------
// Launchers
// --------------------------------------------------------------------------

// The launch's own status: hipGetLastError() would also report errors other runtime
// calls of the caller (an event query that is not ready yet) left behind.
template <typename P, typename... Extra>
static hipError_t launch(void (*kernel)(P, Extra...), dim3 grid, dim3 block, hipStream_t s, P p, Extra... extra) {
  void *args[] = {(void *)&p, (void *)&extra...};
  return hipLaunchKernel((const void *)kernel, grid, block, args, 0, s);
}

int zz_query_num_cu() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return n;
}

// Split-K scratch of zz_attn_decode_static, for callers that may not allocate: one array per
// GPU, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and clears get the address that call returns, looked up once
// per device with that device current.
static __device__ __align__(256) unsigned char scratch[ZZ_STATIC_SCRATCH_BYTES];

hipError_t zz_static_scratch(char **out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static char *ptr[MAX_DEVICES] = {nullptr};
  *out = nullptr;
  int dev = 0;
  if (hipError_t e = hipGetDevice(&dev)) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void *p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr[dev] = (char *)p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

bool zz_stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return st != hipStreamCaptureStatusNone;
}

hipError_t zz_launch_append(const zz_append_params &p0, const zz_seq_lens &lens, hipStream_t s) {
  zz_append_params p = p0;
  // many tokens into never-evicting heads: the tile-wise kernel; streaming heads (at most S+W
  // surviving tokens) and short appends: the per-token kernel
  if (p.n_new >= ZZ_TILE_SLOTS && p.grp[0].n_heads > 0 && p.only_group < 0) {
    // tiles touched by the sequence that straddles the most of them
    int64_t most = 0;
    for (int b = 0; b < (lens.ragged && !p.stage ? p.batch : 1); ++b) {
      const int64_t len = p.stage ? 0 : lens.ragged ? (int64_t)lens.len[b] : p.len;
      const int64_t tiles = (len + p.n_new - 1) / ZZ_TILE_SLOTS - len / ZZ_TILE_SLOTS + 1;
      most = tiles > most ? tiles : most;
    }
    const dim3 grid((unsigned)most, p.grp[0].n_heads, p.batch);
    hipError_t e = p.head_dim == 128 ? launch(zz_append_bulk_kernel<128>, grid, dim3(256), s, p, lens)
                                     : launch(zz_append_bulk_kernel<64>, grid, dim3(256), s, p, lens);
    if (e != hipSuccess || p.grp[1].n_heads == 0) return e;
    p.only_group = 1;
  }
  const int64_t total = (int64_t)p.batch * p.n_new * p.n_kv_heads * (p.head_dim / 8);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (p.head_dim == 128) return launch(zz_append_kernel<128>, dim3(blocks), dim3(256), s, p, lens);
  return launch(zz_append_kernel<64>, dim3(blocks), dim3(256), s, p, lens);
}

hipError_t zz_launch_stage(const zz_stage_params &sp, const zz_seq_lens &lens, hipStream_t s) {
  // staging is an append of the chunk into an empty, never-evicting cache of its own; the sequences'
  // lengths only matter as positions (rotation angles)
  zz_append_params p = {};
  p.k_new = sp.k_new;
  p.v_new = sp.v_new;
  p.grp[0].base = sp.stage;
  p.grp[0].n_heads = sp.n_kv_heads;
  p.grp[0].n_tiles = sp.stage_tiles;
  p.grp[0].capacity = sp.stage_tiles * ZZ_TILE_SLOTS;
  p.grp[0].streaming = 0;
  p.debug_word = sp.debug_word;
  for (int g = 0; g < sp.n_kv_heads; ++g) {
    p.head_group[g] = 0;
    p.head_index[g] = (uint8_t)g;
  }
  p.len = sp.n_past;
  p.stage = 1;
  p.rope_cos = sp.rope_cos;
  p.rope_sin = sp.rope_sin;
  p.n_new = sp.n_new;
  p.batch = sp.batch;
  p.n_kv_heads = sp.n_kv_heads;
  p.head_dim = sp.head_dim;
  p.sink = 0;
  p.window = 1;
  p.only_group = -1;
  return zz_launch_append(p, lens, s);
}

hipError_t zz_launch_decode(const zz_decode_params &p, hipStream_t s) {
  const dim3 grid(p.n_splits, p.grp.n_heads, p.batch);
  if (p.n_splits == 1 && p.n_tiles_valid > 4 && p.n_tiles_valid <= 16 && p.group_size <= 8)
    return p.head_dim == 128 ? launch(zz_decode_short_kernel<128>, grid, dim3(512), s, p)
                             : launch(zz_decode_short_kernel<64>, grid, dim3(512), s, p);
  hipError_t e = p.head_dim == 128 ? launch(zz_decode_kernel<128>, grid, dim3(256), s, p)
                                   : launch(zz_decode_kernel<64>, grid, dim3(256), s, p);
  return e;
}

hipError_t zz_launch_decode_ragged(const zz_decode_ragged_params &p, int total_wg, hipStream_t s) {
  const dim3 grid(total_wg, p.u.grp.n_heads, 1);
  int64_t longest = 0;
  for (int b = 0; b < p.u.batch; ++b) longest = p.seq_len[b] > longest ? p.seq_len[b] : longest;
  if (p.u.grp.streaming && longest > p.sink + p.window) longest = p.sink + p.window;
  const int64_t most_tiles = (longest + ZZ_TILE_SLOTS - 1) / ZZ_TILE_SLOTS;
  if (total_wg == p.u.batch && most_tiles > 4 && most_tiles <= 16 && p.u.group_size <= 8)
    return p.u.head_dim == 128 ? launch(zz_decode_ragged_short_kernel<128>, grid, dim3(512), s, p)
                               : launch(zz_decode_ragged_short_kernel<64>, grid, dim3(512), s, p);
  return p.u.head_dim == 128 ? launch(zz_decode_ragged_kernel<128>, grid, dim3(256), s, p)
                             : launch(zz_decode_ragged_kernel<64>, grid, dim3(256), s, p);
}

hipError_t zz_launch_zero(int *p, int n, hipStream_t s) {
  return launch(zz_zero_kernel, dim3((n + 255) / 256), dim3(256), s, p, n);
}

hipError_t zz_launch_probe_read(const void *buf, size_t bytes, int nontemporal, int n_wg, void *sink, hipStream_t s) {
  const size_t n_blocks = bytes / (16 * 1024);
  if (nontemporal) return launch(zz_probe_read_kernel<true>, dim3(n_wg), dim3(256), s, (const uint4 *)buf, n_blocks, (uint4 *)sink);
  return launch(zz_probe_read_kernel<false>, dim3(n_wg), dim3(256), s, (const uint4 *)buf, n_blocks, (uint4 *)sink);
}

hipError_t zz_launch_prefill(const zz_prefill_params &p, const zz_seq_lens &lens, int pair_min_wg, hipStream_t s) {
  constexpr int NB = ZZ_PREFILL_NB;
  const int G = p.group_size;
  const int Gc = zz_prefill_heads_per_wave(G);  // heads per wave, divides NB
  const int qw = 16 * (NB / Gc) * ZZ_WAVES_PER_WG;        // query positions per workgroup
  const int n_hchunks = G / Gc;
  const dim3 grid((p.n_new + qw - 1) / qw, p.grp.n_heads * n_hchunks, p.batch);
  // Two head chunks of a KV head in one workgroup of eight waves where the head count allows it and the
  // launch still has a workgroup for every compute unit that way (a 1k-token chunk at batch 1 has not: the
  // four-wave form then spreads over twice as many units and is the faster one).  pair_min_wg = 0: always.
  // (Nor does it pay on a chunk with little behind it, where most tiles are diagonal ones outside the
  // pipelined loop: 4 % slower on the first 4096-token chunk of a prompt, equal on the second, faster after.)
  const int64_t paired_wgs = (int64_t)grid.x * (grid.y / 2) * grid.z;
  int64_t longest_past = p.n_past;
  if (lens.ragged)
    for (int b = 0; b < p.batch; ++b) longest_past = lens.len[b] > longest_past ? (int64_t)lens.len[b] : longest_past;
  // (And not on a streaming head: its few tiles all go through the masked loop, which the eight waves run
  // in step; 124 us against 71 us for a 4096-token chunk.)
  const bool worth = pair_min_wg == 0 || (paired_wgs >= pair_min_wg && longest_past >= p.n_new && !p.grp.streaming);
  if (pair_min_wg >= 0 && p.head_dim == 128 && n_hchunks % 2 == 0 && worth)
    return launch(zz_prefill_kernel<128, NB, true>, dim3(grid.x, grid.y / 2, grid.z), dim3(512), s, p, lens, Gc);
  if (p.head_dim == 128) return launch(zz_prefill_kernel<128, NB, false>, grid, dim3(256), s, p, lens, Gc);
  return launch(zz_prefill_kernel<64, NB, false>, grid, dim3(256), s, p, lens, Gc);
}
