// Paged attention of a bf16 model on the matrix cores. Queries, the K/V cache and the probabilities are half precision
// (what the engine computes and stores itself is half precision; only the weights are bf16 values), fp32 accumulation.
//
// Data layout (per layer):  K cache [block][kv head][16 tokens][hd]   (token-major: a tile is the A operand of QK^T)
//                           V cache [block][kv head][hd][16 tokens]   (dimension-major: a tile is the B operand of PV)
//                           q       [token][q head][hd] half, already rotated and scaled by 1/sqrt(hd)
// One KV block (16 tokens of one kv head) is one contiguous 2-4 KB tile that a wave loads with 16-byte (K) and
// 8-byte (V) lane loads. Scores are computed as S[token][column] = K_tile . q_column (v_mfma_f32_16x16x32_f16),
// where a column is a q head of the GQA group (decode) or a query position of one head (prefill). The
// accumulator layout of S (column = lane%16, tokens = 4*(lane/16)+i) is exactly the A-operand layout of
// v_mfma_f32_16x16x16_f16, so the probabilities feed O[column][dim] += P . V without leaving registers.
// Softmax is the online form (running maximum and sum per column), all in fp32.
#pragma once
#include "blink_device.h"
#include "mfma_gemm.h"

typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f16x8_t ld_tile(const f16_t* p) {   // one lane's 16 bytes of a half-precision tile (K cache, queries)
  const uint4 v = *(const uint4*)p;
  return *(const f16x8_t*)&v;
}

template <int HD, int CT>
struct AttnAcc {
  floatx4_t o[CT][HD / 16];   // rows = columns of S (4*(lane/16)+i), column = dim d*16 + lane%16
  float m[CT], l[CT];         // running max / sum of this lane's column (lane%16)
};

template <int HD, int CT>
__device__ __forceinline__ void attn_init(AttnAcc<HD, CT>& a) {
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    a.m[c] = -INFINITY;
    a.l[c] = 0.f;
#pragma unroll
    for (int d = 0; d < HD / 16; ++d) a.o[c][d] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  }
}

// One KV block. Kt/Vt: the block's tiles for this kv head. j0: position of the block's first token.
// lim[c]: number of visible keys (position + 1) for this lane's column of column-tile c.
template <int HD>
struct KVTile {
  f16x8_t ka[HD / 32];
  f16x4_t vb[HD / 16];
};

template <int HD>
__device__ __forceinline__ void kv_load(const f16_t* Kt, const f16_t* Vt, KVTile<HD>& r) {
  const u32 lane = threadIdx.x & 63, lg = lane >> 4, lc = lane & 15;
#pragma unroll
  for (int s = 0; s < HD / 32; ++s) r.ka[s] = ld_tile(Kt + lc * HD + s * 32 + lg * 8);
#pragma unroll
  for (int d = 0; d < HD / 16; ++d) {
    const uint2 v = *(const uint2*)(Vt + (d * 16 + lc) * 16 + lg * 4);
    r.vb[d] = *(const f16x4_t*)&v;
  }
}

// max / sum over the four lanes l, l^16, l^32, l^48 with the lane-swap instructions of gfx950 (vector ALU; a shuffle
// goes through the LDS crossbar). With both operands equal, v_permlane16_swap returns (x[l & ~16], x[l | 16]) and
// v_permlane32_swap (x[l & ~32], x[l | 32]) in every lane: the pair a lane and its partner hold.
__device__ __forceinline__ float quad_max(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_sum(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <int HD, int CT>
__device__ __forceinline__ void attn_block(const KVTile<HD>& kv, const f16x8_t (&q)[CT][HD / 32], u32 j0,
                                           const u32 (&lim)[CT], AttnAcc<HD, CT>& a) {
  const u32 lane = threadIdx.x & 63, lg = lane >> 4;
  const f16x8_t (&ka)[HD / 32] = kv.ka;
  const f16x4_t (&vb)[HD / 16] = kv.vb;
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    // two independent accumulation chains (a product waits for the one before it in its chain)
    floatx4_t s4 = floatx4_t{0.f, 0.f, 0.f, 0.f}, s4b = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < HD / 32; s += 2) {
      s4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[s], q[c][s], s4, 0, 0, 0);
      s4b = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[s + 1], q[c][s + 1], s4b, 0, 0, 0);
    }
    s4 += s4b;
    float bm = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (j0 + lg * 4 + i >= lim[c]) s4[i] = -INFINITY;
      bm = fmaxf(bm, s4[i]);
    }
    bm = quad_max(bm);
    const float mn = fmaxf(a.m[c], bm);
    // A column that has seen no visible key yet (a prompt chunk that starts inside a KV block: the tile's early queries
    // do not see its second block) keeps m = -inf; the exponentials then take 0 as their reference, so that they give 0
    // instead of exp(-inf + inf)
    const float mref = mn == -INFINITY ? 0.f : mn;
    float p[4], ps = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = __expf(s4[i] - mref);    // exp(-inf) = 0 for masked keys
      ps += p[i];
    }
    ps = quad_sum(ps);
    const float corr = __expf(a.m[c] - mref);
    a.l[c] = a.l[c] * corr + ps;
    a.m[c] = mn;
    float c4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) c4[i] = __shfl(corr, lg * 4 + i);
    // probabilities (in [0, 1]) to half precision, round to nearest even
    const f16x4_t pa = {(_Float16)p[0], (_Float16)p[1], (_Float16)p[2], (_Float16)p[3]};
#pragma unroll
    for (int d = 0; d < HD / 16; ++d) {
#pragma unroll
      for (int i = 0; i < 4; ++i) a.o[c][d][i] *= c4[i];
      a.o[c][d] = __builtin_amdgcn_mfma_f32_16x16x16f16(pa, vb[d], a.o[c][d], 0, 0, 0);
    }
  }
}

#define ATTN_CHUNK_BLOCKS (ATTN_CHUNK_TOKENS / 16)   // KV blocks per decode work item
#define ATTN_WAVES 8          // waves per workgroup of the attention kernel (512 threads: at most 256 registers per lane)
#define ATTN_META_MAX 512     // sequences whose batch metadata the decode kernel keeps in LDS
struct AttnMfmaShared {
  float m[ATTN_WAVES][16], l[ATTN_WAVES][16];
  float o[ATTN_WAVES][16][128];  // [wave][q head of the group (decode) or query of the tile (prefill)][dim]
  u32 cu_chunks[ATTN_META_MAX + 1], tok[ATTN_META_MAX], ctx[ATTN_META_MAX], bslot[ATTN_META_MAX], pos0[ATTN_META_MAX];
  u32 next_item;   // decode items taken through the work counter: the item after the next one
};

// ---- decode: one workgroup per (sequence, kv head); its waves take the KV blocks round-robin ----------------------
template <int HD>
__device__ __forceinline__ void attn_decode(const DevCtx& c, u32 layer, AttnMfmaShared& sh, u32 wg, u32 nwg) {
  const u32 B = c.meta->n_seqs, G = c.nq / c.nkv;
  const u32 lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lg = lane >> 4, lc = lane & 15;   // w as a scalar: block-table reads become scalar loads
  const f16_t* Kc = (const f16_t*)c.kv + (u64)layer * c.kv_layer_stride;
  const f16_t* Vc = Kc + c.kv_kv_stride;
  const u64 tile = (u64)16 * HD;
  // Work item: (chunk of ATTN_CHUNK_TOKENS of one sequence's context, kv head). Chunks balance the load between short and long
  // contexts and give the chip enough items at small batch. A context of one chunk is finished here; longer ones
  // leave per-chunk partial results that attn_decode_combine (the next kernel) merges in chunk order.
  // The batch metadata an item needs is copied into LDS once: finding an item's sequence is a binary search, and every
  // step of it in global memory would be a dependent load in front of the item's first KV load.
  // (the library admits at most ATTN_META_MAX batch slots for a bf16 model)
  for (u32 i = threadIdx.x; i <= B; i += blockDim.x) {
    sh.cu_chunks[i] = c.cu_chunks[i];
    if (i < B) { sh.tok[i] = c.cu_seqlens[i]; sh.ctx[i] = c.seq_len[i]; sh.bslot[i] = c.seq_bslot[i]; }
  }
  __syncthreads();
  auto cu = [&](u32 i) { return sh.cu_chunks[i]; };
  const u32 total_chunks = cu(B);
  // Every wave takes blocks w, w + 8, w + 16, w + 24 of the item's chunk and keeps all four tiles in flight. The loads
  // are unconditional and the block ids are fetched first, in one batch: a load inside a branch, or an id fetched
  // between two tiles, makes the wave wait for everything in flight (loads complete in order). A slot past the
  // chunk's end repeats one of the chunk's blocks (a cache hit) and its tile is not used.
  static_assert(ATTN_CHUNK_BLOCKS == 4 * ATTN_WAVES, "four KV tiles per wave");
  constexpr u32 nw = ATTN_WAVES;
  const u32 total_items = total_chunks * c.nkv;
  struct Item { u32 ci, g, nch, t, ctx, b_lo, nb; };
  f16x8_t q[1][HD / 32];
  KVTile<HD> t0, t1, t2, t3;
  // describes the item and requests its queries and tiles (into q and t0..t3, which the previous item no longer needs)
  auto start = [&](u32 item) {
    Item it;
    it.ci = item / c.nkv; it.g = item % c.nkv;
    u32 lo = 0, hi = B;                       // sequence of chunk ci: last s with cu_chunks[s] <= ci
    while (hi - lo > 1) {
      const u32 mid = (lo + hi) / 2;
      if (cu(mid) <= it.ci) lo = mid; else hi = mid;
    }
    const u32 s = lo, ch = it.ci - cu(s);
    it.nch = cu(s + 1) - cu(s);
    it.t = sh.tok[s];              // the sequence's single token of this iteration
    it.ctx = sh.ctx[s];
    // the block table row through the constant address space and a wave-uniform address: scalar loads, which do not
    // queue behind the tile loads still in flight (the builtin returns int: each half goes through u32)
    typedef const __attribute__((address_space(4))) u32 const_u32;
    const u64 bta = (u64)(c.block_tables + (u64)sh.bslot[s] * c.max_blocks_per_seq);
    const u32 bt_hi = (u32)__builtin_amdgcn_readfirstlane((u32)(bta >> 32)), bt_lo = (u32)__builtin_amdgcn_readfirstlane((u32)bta);
    const_u32* bt = (const_u32*)(((u64)bt_hi << 32) | (u64)bt_lo);
    it.b_lo = ch * ATTN_CHUNK_BLOCKS;
    it.nb = min((it.ctx + 15) / 16, it.b_lo + ATTN_CHUNK_BLOCKS) - it.b_lo;   // 1..32 blocks: up to four per wave
    const u32 wfirst = w < it.nb ? w : 0u;
#define BLOCK_ID(j) bt[__builtin_amdgcn_readfirstlane(it.b_lo + ((w + (j) * nw < it.nb) ? w + (j) * nw : wfirst))]
    const u32 id0 = BLOCK_ID(0), id1 = BLOCK_ID(1), id2 = BLOCK_ID(2), id3 = BLOCK_ID(3);
#undef BLOCK_ID
    // (columns past the group's heads repeat its last head: an unconditional load; their results are never stored)
#pragma unroll
    for (int st = 0; st < HD / 32; ++st)
      q[0][st] = ld_tile(c.qbuf + ((u64)it.t * c.nq + it.g * G + min(lc, G - 1)) * HD + st * 32 + lg * 8);
    const u64 b0 = ((u64)id0 * c.nkv + it.g) * tile, b1 = ((u64)id1 * c.nkv + it.g) * tile;
    const u64 b2 = ((u64)id2 * c.nkv + it.g) * tile, b3 = ((u64)id3 * c.nkv + it.g) * tile;
    kv_load<HD>(Kc + b0, Vc + b0, t0); kv_load<HD>(Kc + b1, Vc + b1, t1);
    kv_load<HD>(Kc + b2, Vc + b2, t2); kv_load<HD>(Kc + b3, Vc + b3, t3);
    return it;
  };
  u32 item = wg;
  if (item >= total_items) return;
  Item cur = start(item);
  for (;;) {
    AttnAcc<HD, 1> acc;
    attn_init(acc);
    const u32 lim[1] = {cur.ctx};
    auto us = [&](const KVTile<HD>& tl, u32 j) { const u32 i = w + j * nw; if (i < cur.nb) attn_block<HD, 1>(tl, q, (cur.b_lo + i) * 16, lim, acc); };
    us(t0, 0); us(t1, 1); us(t2, 2); us(t3, 3);
    // the next item's tiles are requested before this item's partial results are merged: the waves wait for each
    // other in the merge, and without loads in flight the memory pipe of the compute unit would idle meanwhile
    const u32 nitem = item + nwg;
    const bool more = nitem < total_items;
    Item nxt = cur;
    if (more) nxt = start(nitem);
    __syncthreads();   // the previous item's combine has finished reading LDS
    if (lg == 0) { sh.m[w][lc] = acc.m[0]; sh.l[w][lc] = acc.l[0]; }
#pragma unroll
    for (int d = 0; d < HD / 16; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (lg * 4 + i < G) sh.o[w][lg * 4 + i][d * 16 + lc] = acc.o[0][d][i];
    __syncthreads();
    float* po = c.attn_part_o + ((u64)cur.ci * c.nkv + cur.g) * G * HD;
    float* pml = c.attn_part_ml + ((u64)cur.ci * c.nkv + cur.g) * G * 2;
    for (u32 idx = threadIdx.x; idx < G * HD; idx += blockDim.x) {
      const u32 h = idx / HD, dim = idx % HD;
      float M = -INFINITY;
      for (u32 ww = 0; ww < nw; ++ww) M = fmaxf(M, sh.m[ww][h]);
      float L = 0.f, O = 0.f;
      for (u32 ww = 0; ww < nw; ++ww) {      // fixed order; a wave without blocks has m = -inf and contributes 0
        const float f = __expf(sh.m[ww][h] - M);
        L += sh.l[ww][h] * f;
        O += sh.o[ww][h][dim] * f;
      }
      if (cur.nch == 1) {
        c.aq[packed_off(cur.t, (cur.g * G + h) * HD + dim, c.TBS)] = f32_to_f16(O / L);
      } else {
        po[(u64)h * HD + dim] = O;
        if (dim == 0) { pml[h * 2] = M; pml[h * 2 + 1] = L; }
      }
    }
    if (!more) break;
    cur = nxt;
    item = nitem;
  }
}

// The decode items taken from the scheduler's work list through a counter. What a launch loses against a plain
// stream of the same tiles is fixed cost, not bandwidth (measured: a launch took 26 us + 11.1 us per full item and
// compute unit, and 11.1 us per 256 KB item is what a load-only kernel reaches): a second generation of workgroups
// that starts, stages the batch metadata and waits for its first tiles when the first generation ends (only one
// eight-wave workgroup with 256 registers per lane fits a compute unit), and the uneven ends of workgroups whose items
// are dealt round-robin whatever their size. Here one workgroup per compute unit runs; its first two items are fixed
// (workgroup id, then id + workgroups), every further one is the next of the list (one relaxed atomic add on the
// launch's counter, issued while the item before it is still running; the counters are zeroed by the scheduler step);
// the list has the large items first, so the small ones fill the ends; and an item's description is one 32-byte scalar
// load instead of a search in metadata staged through LDS. An item is a run of KV blocks of one sequence and one kv head,
// walked in rounds of 32 blocks (four tile slots per wave) with the running maxima, sums and outputs kept in registers
// from round to round, and merged across the waves once, at its end: one chunk of a context (its partial result is
// merged with the other chunks' by the combine kernel) or, when the scheduler has many sequences to hand out, a whole
// context (no partial results). A wave refills each tile slot with the tile of the next round (of the same item or of
// the next one) as soon as it has consumed the slot; the next round's description and queries are fetched first (loads
// complete in order, so the queries must not queue behind the refills); the workgroup's last round runs without the
// fetching ahead. Results do not depend on which workgroup takes an item.
template <int HD>
__device__ __forceinline__ void attn_decode_dyn(const DevCtx& c, u32 layer, AttnMfmaShared& sh, u32 wg, u32 nwg) {
  const u32 nwg_eff = max(1u, nwg / 2);          // the launch has two workgroups per compute unit, of which one is resident
  if (wg >= nwg_eff) return;
  const u32 G = c.nq / c.nkv;
  const u32 lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lg = lane >> 4, lc = lane & 15;
  const f16_t* Kc = (const f16_t*)c.kv + (u64)layer * c.kv_layer_stride;
  const f16_t* Vc = Kc + c.kv_kv_stride;
  const u64 tile = (u64)16 * HD;
  static_assert(ATTN_CHUNK_BLOCKS == 4 * ATTN_WAVES, "four KV tiles per wave");
  constexpr u32 nw = ATTN_WAVES;
  const u32 n_full = c.meta->n_full_chunks, total_items = c.meta->n_chunks * c.nkv;
  typedef const __attribute__((address_space(4))) u32 const_u32;
  // a wave-uniform pointer for scalar loads (the builtin returns int: each half goes through u32 before it is widened)
  auto scalar_ptr = [&](const void* p) {
    const u64 a = (u64)p;
    const u32 hi = (u32)__builtin_amdgcn_readfirstlane((u32)(a >> 32)), lo = (u32)__builtin_amdgcn_readfirstlane((u32)a);
    return (const_u32*)(((u64)hi << 32) | (u64)lo);
  };
  // one round of an item: blocks b_lo .. b_lo + nb of the item's run (which ends at b_end), this wave's four block ids
  struct Round { u32 ci, g, nch, t, ctx, bslot, b_lo, b_end, nb, id[4]; };
  auto block_ids = [&](Round& r) {       // (slots past the round's end repeat its first block)
    const_u32* bt = scalar_ptr(c.block_tables + (u64)r.bslot * c.max_blocks_per_seq);
    r.nb = min(r.b_end, r.b_lo + ATTN_CHUNK_BLOCKS) - r.b_lo;   // 1..32 blocks: up to four per wave
    const u32 wfirst = w < r.nb ? w : 0u;
#pragma unroll
    for (u32 j = 0; j < 4; ++j) r.id[j] = bt[__builtin_amdgcn_readfirstlane(r.b_lo + ((w + j * nw < r.nb) ? w + j * nw : wfirst))];
  };
  auto first_round = [&](u32 item) {
    Round r;
    const u32 ord = item / c.nkv;
    r.g = item % c.nkv;
    const_u32* rec = scalar_ptr(c.chunk_rec + (ord < n_full ? ord : c.chunk_cap + (ord - n_full)));
    r.t = rec[0]; r.ctx = rec[1]; r.bslot = rec[2];
    r.b_lo = rec[3] * ATTN_CHUNK_BLOCKS;
    r.ci = rec[4]; r.nch = rec[5]; r.b_end = rec[6];
    block_ids(r);
    return r;
  };
  auto load_q = [&](const Round& r, f16x8_t (&qq)[1][HD / 32]) {
    // (columns past the group's heads repeat its last head: an unconditional load; their results are never stored)
#pragma unroll
    for (int st = 0; st < HD / 32; ++st)
      qq[0][st] = ld_tile(c.qbuf + ((u64)r.t * c.nq + r.g * G + min(lc, G - 1)) * HD + st * 32 + lg * 8);
  };
  auto load_tile = [&](u32 id, u32 g, KVTile<HD>& tl) {
    const u64 b0 = ((u64)id * c.nkv + g) * tile;
    kv_load<HD>(Kc + b0, Vc + b0, tl);
  };
  u32 nitem = wg + nwg_eff;
  if (wg >= total_items) return;
  f16x8_t q[1][HD / 32];
  KVTile<HD> t0, t1, t2, t3;
  Round cur = first_round(wg);
  load_q(cur, q);
  load_tile(cur.id[0], cur.g, t0); load_tile(cur.id[1], cur.g, t1); load_tile(cur.id[2], cur.g, t2); load_tile(cur.id[3], cur.g, t3);
  // merges the eight waves' partial results of the item of round `it` through LDS (fixed order) and stores the item's result
  auto finish = [&](const Round& it, const AttnAcc<HD, 1>& acc, u32 fetched) {
    __syncthreads();   // the previous item's merge has finished reading LDS (and every wave has read the previous next_item)
    if (threadIdx.x == 0) sh.next_item = fetched;
    if (lg == 0) { sh.m[w][lc] = acc.m[0]; sh.l[w][lc] = acc.l[0]; }
#pragma unroll
    for (int d = 0; d < HD / 16; ++d)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (lg * 4 + i < G) sh.o[w][lg * 4 + i][d * 16 + lc] = acc.o[0][d][i];
    __syncthreads();
    float* po = c.attn_part_o + ((u64)it.ci * c.nkv + it.g) * G * HD;
    float* pml = c.attn_part_ml + ((u64)it.ci * c.nkv + it.g) * G * 2;
    for (u32 idx = threadIdx.x; idx < G * HD; idx += blockDim.x) {
      const u32 h = idx / HD, dim = idx % HD;
      float M = -INFINITY;
      for (u32 ww = 0; ww < nw; ++ww) M = fmaxf(M, sh.m[ww][h]);
      float L = 0.f, O = 0.f;
      for (u32 ww = 0; ww < nw; ++ww) {      // a wave without blocks has m = -inf and contributes 0
        const float f = __expf(sh.m[ww][h] - M);
        L += sh.l[ww][h] * f;
        O += sh.o[ww][h][dim] * f;
      }
      if (it.nch == 1) {
        c.aq[packed_off(it.t, (it.g * G + h) * HD + dim, c.TBS)] = f32_to_f16(O / L);
      } else {
        po[(u64)h * HD + dim] = O;
        if (dim == 0) { pml[h * 2] = M; pml[h * 2 + 1] = L; }
      }
    }
  };
  AttnAcc<HD, 1> acc;
  attn_init(acc);
  for (;;) {
    const bool last_round = cur.b_lo + ATTN_CHUNK_BLOCKS >= cur.b_end;     // of the item
    if (last_round && nitem >= total_items) break;                          // and of the workgroup
    // the next round: of the same item, or the first of the next item (then the item after that one is asked for now
    // and handed to the other waves through LDS at the merge)
    u32 fetched = ~0u;
    Round nxt;
    if (last_round) {
      if (threadIdx.x == 0) fetched = 2 * nwg_eff + atomicAdd(c.attn_ctr + layer, 1u);
      nxt = first_round(nitem);
    } else {
      nxt = cur;
      nxt.b_lo = cur.b_lo + ATTN_CHUNK_BLOCKS;
      block_ids(nxt);
    }
    f16x8_t qn[1][HD / 32];
    load_q(nxt, qn);
    const u32 lim[1] = {cur.ctx};
    auto us = [&](const KVTile<HD>& tl, u32 j) { const u32 i = w + j * nw; if (i < cur.nb) attn_block<HD, 1>(tl, q, (cur.b_lo + i) * 16, lim, acc); };
    us(t0, 0); load_tile(nxt.id[0], nxt.g, t0);
    us(t1, 1); load_tile(nxt.id[1], nxt.g, t1);
    us(t2, 2); load_tile(nxt.id[2], nxt.g, t2);
    us(t3, 3); load_tile(nxt.id[3], nxt.g, t3);
    if (last_round) {
      finish(cur, acc, fetched);
      nitem = __builtin_amdgcn_readfirstlane(sh.next_item);     // written between the merge's barriers, rewritten only behind the next merge's first one
      attn_init(acc);
    }
#pragma unroll
    for (int st = 0; st < HD / 32; ++st) q[0][st] = qn[0][st];
    cur = nxt;
  }
  {   // the workgroup's last round: nothing to fetch ahead
    const u32 lim[1] = {cur.ctx};
    auto us = [&](const KVTile<HD>& tl, u32 j) { const u32 i = w + j * nw; if (i < cur.nb) attn_block<HD, 1>(tl, q, (cur.b_lo + i) * 16, lim, acc); };
    us(t0, 0); us(t1, 1); us(t2, 2); us(t3, 3);
    finish(cur, acc, ~0u);
  }
}

// Merges the per-chunk partial results of contexts longer than one chunk, in chunk order. One wave per (sequence, kv
// head); a lane takes E output elements at a time and has the partial results of all their chunks in flight together
// (the kernel is a chain of dependent loads: how many of them wait at once is what its duration depends on).
template <u32 MAXC, u32 E>
__device__ __forceinline__ void attn_combine_pair(const DevCtx& c, u32 c0, u32 nch, u32 t, u32 g, u32 G, u32 HD) {
  const u32 lane = threadIdx.x & 63, n = G * HD;
  for (u32 i0 = lane; i0 < n; i0 += 64 * E) {
    float2 ml[E][MAXC];
    float ov[E][MAXC];
#pragma unroll
    for (u32 e = 0; e < E; ++e) {
      const u32 idx = min(i0 + 64 * e, n - 1), h = idx / HD, dim = idx % HD;
#pragma unroll
      for (u32 p = 0; p < MAXC; ++p) {
        const u64 base = ((u64)(c0 + min(p, nch - 1)) * c.nkv + g) * G;
        ml[e][p] = *(const float2*)(c.attn_part_ml + (base + h) * 2);
        ov[e][p] = c.attn_part_o[(base + h) * HD + dim];
      }
    }
#pragma unroll
    for (u32 e = 0; e < E; ++e) {
      const u32 idx = i0 + 64 * e;
      float M = -INFINITY, L = 0.f, O = 0.f;
#pragma unroll
      for (u32 p = 0; p < MAXC; ++p)
        if (p < nch) M = fmaxf(M, ml[e][p].x);
#pragma unroll
      for (u32 p = 0; p < MAXC; ++p)
        if (p < nch) {
          const float f = __expf(ml[e][p].x - M);
          L += ml[e][p].y * f;
          O += ov[e][p] * f;
        }
      if (idx < n) c.aq[packed_off(t, g * n + idx, c.TBS)] = f32_to_f16(O / L);
    }
  }
}

__device__ __forceinline__ void attn_decode_combine(const DevCtx& c, u32 wg, u32 nwg) {
  const u32 B = c.meta->n_seqs, G = c.nq / c.nkv, HD = c.hd, lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if (c.cu_chunks[B] == 0) return;     // no sequence decodes in this iteration
  for (u32 pair = wg * nw + w; pair < B * c.nkv; pair += nwg * nw) {
    const u32 s = pair / c.nkv, g = pair % c.nkv;
    const u32 c0 = c.cu_chunks[s], nch = c.cu_chunks[s + 1] - c0;
    if (nch < 2) continue;
    const u32 t = c.cu_seqlens[s];
    if (nch <= 4) attn_combine_pair<4, 4>(c, c0, nch, t, g, G, HD);
    else if (nch <= 12) attn_combine_pair<12, 1>(c, c0, nch, t, g, G, HD);
    else {
      for (u32 idx = lane; idx < G * HD; idx += 64) {
        const u32 h = idx / HD, dim = idx % HD;
        float M = -INFINITY, L = 0.f, O = 0.f;
        for (u32 p = 0; p < nch; ++p) M = fmaxf(M, c.attn_part_ml[(((u64)(c0 + p) * c.nkv + g) * G + h) * 2]);
        for (u32 p = 0; p < nch; ++p) {
          const u64 base = ((u64)(c0 + p) * c.nkv + g) * G;
          const float f = __expf(c.attn_part_ml[(base + h) * 2] - M);
          L += c.attn_part_ml[(base + h) * 2 + 1] * f;
          O += c.attn_part_o[(base + h) * HD + dim] * f;
        }
        c.aq[packed_off(t, (g * G + h) * HD + dim, c.TBS)] = f32_to_f16(O / L);
      }
    }
  }
}

// ---- prefill: WPI waves per (sequence, kv head, head group of CT q heads, tile of 16 query positions) -------------
// The waves of an item take its KV blocks round-robin and merge their partial results through LDS (one pass per q
// head of the group). WPI (1, 2, 4 or 8, the same for the whole launch) trades the length of the longest chain of
// blocks a wave walks - the causal mask makes the last tile of a long prompt walk all of it - against merge work.
template <int HD, int CT>
__device__ __forceinline__ void attn_prefill(const DevCtx& c, u32 layer, AttnMfmaShared& sh, u32 wg, u32 nwg) {
  const u32 B = c.meta->n_seqs, G = c.nq / c.nkv, groups = G / CT;
  const u32 lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lg = lane >> 4, lc = lane & 15;   // w as a scalar: block-table reads become scalar loads
  const f16_t* Kc = (const f16_t*)c.kv + (u64)layer * c.kv_layer_stride;
  const f16_t* Vc = Kc + c.kv_kv_stride;
  const u64 tile = (u64)16 * HD;
  const u32 per_tile = c.nkv * groups;
  const u32 nw = blockDim.x >> 6;
  // batch metadata in LDS (the item lookup is a binary search; see the decode kernel)
  for (u32 i = threadIdx.x; i <= B; i += blockDim.x) {
    sh.cu_chunks[i] = c.cu_qtiles[i];
    if (i < B) {
      sh.tok[i] = c.cu_seqlens[i]; sh.ctx[i] = c.cu_seqlens[i + 1] - c.cu_seqlens[i]; sh.bslot[i] = c.seq_bslot[i];
      sh.pos0[i] = c.seq_pos0[i];     // position of the sequence's first token of this iteration (a later chunk of a prompt starts beyond 0)
    }
  }
  __syncthreads();
  auto cuq = [&](u32 i) { return sh.cu_chunks[i]; };
  const u64 total = (u64)cuq(B) * per_tile;
  // waves per item: doubled while the longest chain (blocks of the longest prompt / WPI) is long and the items, each
  // now taking WPI wave slots, still fit the waves that run at once
  u32 WPI = 1;
  {
    const u32 chain = (c.meta->max_pref_ctx + 15) / 16;
    const u64 slots = (u64)(nwg / 2) * nw;
    while (WPI < nw && WPI < 8 && chain > 12 * WPI && total * WPI <= slots) WPI *= 2;
    const u32 forced = (c.tune_nw >> 16) & 15u;      // bits 16-19 of the tuning word: 1, 2, 4, 8 force it (tests)
    if (forced == 1 || forced == 2 || forced == 4 || forced == 8) WPI = min(forced, nw);
  }
  const u32 gpw = nw / WPI, grp = w / WPI, wi = w % WPI;
  for (u64 base = (u64)wg * gpw; base < total; base += (u64)nwg * gpw) {
    const u64 item = base + grp;
    const bool valid = item < total;
    u32 g = 0, hg = 0, p0 = 0, t0 = 0, P = 1, last = 0, a0 = 0;   // p0: first query of the tile within the sequence's tokens of this iteration; a0: its position
    const u32* bt = c.block_tables;
    if (valid) {
      // query tiles in descending order: the causal mask makes the later tiles of a prompt walk more blocks, and the
      // workgroups that start first should take the longest chains (the short ones then fill the gaps)
      const u32 qi = cuq(B) - 1 - (u32)(item / per_tile), rem = (u32)(item % per_tile);
      g = rem / groups; hg = rem % groups;
      u32 lo = 0, hi = B;                       // sequence of query tile qi: last s with cu_qtiles[s] <= qi
      while (hi - lo > 1) {
        const u32 mid = (lo + hi) / 2;
        if (cuq(mid) <= qi) lo = mid; else hi = mid;
      }
      const u32 s = lo;
      p0 = (qi - cuq(s)) * 16;
      t0 = sh.tok[s];
      P = sh.ctx[s];
      a0 = sh.pos0[s] + p0;
      bt = c.block_tables + (u64)sh.bslot[s] * c.max_blocks_per_seq;
      last = (a0 + min(15u, P - 1 - p0)) / 16;
    }
    const bool colv = valid && p0 + lc < P;
    // queries of the tile (columns past the prompt's end repeat its last token: an unconditional load; they are
    // masked down to key 0 and never stored)
    f16x8_t q[CT][HD / 32];
    u32 lim[CT];
    const u32 qrow = t0 + min(p0 + lc, P - 1);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      lim[ct] = colv ? a0 + lc + 1 : 1;
#pragma unroll
      for (int st = 0; st < HD / 32; ++st)
        q[ct][st] = ld_tile(c.qbuf + ((u64)qrow * c.nq + g * G + hg * CT + ct) * HD + st * 32 + lg * 8);
    }
    AttnAcc<HD, CT> acc;
    attn_init(acc);
    // This wave's blocks: wi, wi + WPI, ...; two tiles in flight, alternating by code position (a register copy would
    // wait for the loads). The block ids come through scalar loads (the table is read through the constant address
    // space with a wave-uniform address), which do not queue behind the tile loads, and the tile loads are
    // unconditional: past the last block they repeat it (a cache hit) and the tile is not used.
    {
      typedef const __attribute__((address_space(4))) u32 const_u32;
      const u64 bta = (u64)bt;
      // (the builtin returns int: each half goes through u32 before it is widened, or the low half is sign-extended)
      const u32 bt_hi = (u32)__builtin_amdgcn_readfirstlane((u32)(bta >> 32)), bt_lo = (u32)__builtin_amdgcn_readfirstlane((u32)bta);
      const_u32* btc = (const_u32*)(((u64)bt_hi << 32) | (u64)bt_lo);
      const u32 lastu = __builtin_amdgcn_readfirstlane(last), gu = __builtin_amdgcn_readfirstlane(g);
      KVTile<HD> k0, k1;
      auto ld = [&](KVTile<HD>& tl, u32 jb) {
        const u64 bs = ((u64)btc[min(jb, lastu)] * c.nkv + gu) * tile;
        kv_load<HD>(Kc + bs, Vc + bs, tl);
      };
      auto us = [&](const KVTile<HD>& tl, u32 jb) { if (jb <= lastu) attn_block<HD, CT>(tl, q, jb * 16, lim, acc); };
      if (valid) {
        ld(k0, wi); ld(k1, wi + WPI);
        for (u32 jb = wi; jb <= lastu; jb += 2 * WPI) {
          us(k0, jb); ld(k0, jb + 2 * WPI);
          us(k1, jb + WPI); ld(k1, jb + 3 * WPI);
        }
      }
    }
    if (WPI == 1) {
      if (valid) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          float inv[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) inv[i] = 1.0f / __shfl(acc.l[ct], lg * 4 + i);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const u32 r = lg * 4 + i;
            if (p0 + r < P) {
#pragma unroll
              for (int d = 0; d < HD / 16; ++d)
                c.aq[packed_off(t0 + p0 + r, (g * G + hg * CT + ct) * HD + d * 16 + lc, c.TBS)] = f32_to_f16(acc.o[ct][d][i] * inv[i]);
            }
          }
        }
      }
    } else {
      // merge the WPI partial results of the item, one q head of the group per pass (fixed order of the waves)
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        __syncthreads();   // the previous pass has been read
        if (lg == 0) { sh.m[w][lc] = acc.m[ct]; sh.l[w][lc] = acc.l[ct]; }
#pragma unroll
        for (int d = 0; d < HD / 16; ++d)
#pragma unroll
          for (int i = 0; i < 4; ++i) sh.o[w][lg * 4 + i][d * 16 + lc] = acc.o[ct][d][i];
        __syncthreads();
        if (valid) {
          const u32 w0 = grp * WPI;
          for (u32 idx = wi * 64 + lane; idx < 16 * HD; idx += WPI * 64) {
            const u32 r = idx / HD, dim = idx % HD;
            if (p0 + r >= P) continue;
            float M = -INFINITY;
            for (u32 ww = 0; ww < WPI; ++ww) M = fmaxf(M, sh.m[w0 + ww][r]);
            float L = 0.f, O = 0.f;
            for (u32 ww = 0; ww < WPI; ++ww) {   // a wave without blocks has m = -inf and contributes 0
              const float f = __expf(sh.m[w0 + ww][r] - M);
              L += sh.l[w0 + ww][r] * f;
              O += sh.o[w0 + ww][r][dim] * f;
            }
            c.aq[packed_off(t0 + p0 + r, (g * G + hg * CT + ct) * HD + dim, c.TBS)] = f32_to_f16(O / L);
          }
        }
      }
    }
  }
}

template <int HD>
__device__ __forceinline__ void attn_prefill_hd(const DevCtx& c, u32 layer, AttnMfmaShared& sh, u32 wg, u32 nwg) {
  const u32 G = c.nq / c.nkv;
  switch (G) {
    case 1: attn_prefill<HD, 1>(c, layer, sh, wg, nwg); break;
    case 2: attn_prefill<HD, 2>(c, layer, sh, wg, nwg); break;
    case 3: attn_prefill<HD, 3>(c, layer, sh, wg, nwg); break;
    case 4: attn_prefill<HD, 2>(c, layer, sh, wg, nwg); break;   // two q heads per pass keep the accumulators in registers
    case 6: attn_prefill<HD, 3>(c, layer, sh, wg, nwg); break;
    case 8: attn_prefill<HD, 2>(c, layer, sh, wg, nwg); break;
    default: break;   // rejected at init
  }
}

// The sequences of an iteration that decode (one token, work items = chunks of their context) and those that process
// prompt tokens (work items = tiles of 16 queries) each have their kernel part; a mixed iteration (chunked prefill) runs
// both in the one launch, every workgroup first its share of the decode items, then of the query tiles.
__device__ __forceinline__ void phase_attention_mfma(const DevCtx& c, u32 layer, AttnMfmaShared& sh, u32 wg, u32 nwg) {
  const u32 B = c.meta->n_seqs;
  const bool dec = c.cu_chunks[B] != 0, pre = c.cu_qtiles[B] != 0;
  // In a mixed iteration every other workgroup takes its query tiles first: the decode items stream the KV cache from
  // HBM while the query tiles mostly wait on L2 and the softmax, so the two parts are spread over the launch instead
  // of all workgroups hitting HBM first and L2 afterwards.
  const bool pre_first = dec && pre && (wg & 1u) && !(c.tune_nw & 0x40000000u);   // bit 30 of the tuning word: decode part first everywhere (A/B)
  if (pre_first) {
    if (c.hd == 64) attn_prefill_hd<64>(c, layer, sh, wg, nwg); else attn_prefill_hd<128>(c, layer, sh, wg, nwg);
    __syncthreads();
  }
  if (dec) {
    // bit 23 of the tuning word (A/B): static items, one batch of loads per item, instead of the items taken through the work counter
    if (c.tune_nw & 0x800000u) {
      if (c.hd == 64) attn_decode<64>(c, layer, sh, wg, nwg); else attn_decode<128>(c, layer, sh, wg, nwg);
    } else {
      if (c.hd == 64) attn_decode_dyn<64>(c, layer, sh, wg, nwg); else attn_decode_dyn<128>(c, layer, sh, wg, nwg);
    }
  }
  if (dec && pre && !pre_first) __syncthreads();   // the batch metadata in LDS is staged again for the other part
  if (pre && !pre_first) {
    if (c.hd == 64) attn_prefill_hd<64>(c, layer, sh, wg, nwg); else attn_prefill_hd<128>(c, layer, sh, wg, nwg);
  }
}
