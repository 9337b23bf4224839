// GEMMs of the forward pass of a bf16 model on the CDNA4 matrix cores, the only dense contractions of the serving
// step. The weights are stored in bf16 (8 significant bits); for the matrix cores they are re-encoded once, at init,
// as IEEE half precision scaled by 2^8 (exact for every bf16 value of magnitude 2^-25 .. 255: a half holds 11
// significant bits), and the activation operands between the GEMMs are carried in half precision too
// (v_mfma_f32_16x16x32_f16, fp32 accumulation; same rate and the same bytes as the bf16 instruction). With bf16
// activation operands the roundings between the GEMMs (unit roundoff 2^-8, about eight per layer) add up to 3e-2 of
// the largest logit over 32 layers; half precision cuts each of them by eight. Activations saturate at the largest
// finite half instead of overflowing. Both operands live in HBM already in MFMA operand order, so that every
// wave-wide load is one contiguous kilobyte:
//
//   weights      Wp[n/16][k/32][lane][8]      lane = n%16 + 16*((k%32)/8), element = k%8   (packed once at init)
//   activations  Xp[k/32][t/16][lane][8]      lane = t%16 + 16*((k%32)/8), element = k%8   (written packed by the
//                                                                                  producing kernel's epilogue)
//
// out[t][n] = sum_k X[t][k] * W[n][k]. Three schedules, chosen per launch from the token count T of the iteration:
//   stream (T <= 64, decode at small batch): a workgroup owns 1, 2 or 4 16-row weight tiles and all token blocks; its
//     4 or 8 waves split K and keep two batches of 1 KB operand loads in flight each; weight loads are non-temporal;
//     partial sums are reduced through LDS in a fixed order. HBM bound: the weight matrix once.
//   stream over a 2-D grid (64 < T <= 256, projections with few rows): the same kernel with items of 4 weight tiles x
//     64 tokens, dealt to the XCDs in runs so that the token groups of a row block share one L2.
//   tiles through LDS (T > 64 otherwise): 128 rows x 64..256 tokens per workgroup, operand tiles fetched once per
//     workgroup and k-step into one of two LDS buffers; the token width is chosen per launch (gemm_tile_pick).
// Epilogues fuse what follows the GEMM in the model: RMSNorm scale of the *input* (a per-token scalar,
// applied to the accumulator), residual add, SiLU-gating, rotary embedding and the KV-cache write, and re-packing of
// the result as the next GEMM's activation operand together with the partial sums of squares the next RMSNorm needs.
#pragma once
#include "blink_device.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

#define W_SCALE 256.0f            // packed weights hold W * 2^8 (keeps small weights in the normal range of a half)
#define W_SCALE_INV (1.0f / 256.0f)

#define EPI_SCALED_STORE 0   // out[t][n] = rstd[t] * acc                      (QKV projection, LM head)
#define EPI_RESIDUAL 1       // x[t][n] += acc; emit packed half(x * g_next) and sum-of-squares partials
#define EPI_SILU_GATE 2      // rows interleaved (gate_j, up_j): emit packed half(silu(r*g) * (r*u))
#define EPI_QKV_ROPE 3       // rows of every head interleaved (dim p, dim p+hd/2): rotary embedding, then q to the query
                             // buffer, k and v straight into the paged cache through the slot mapping

struct MfmaGemmArgs {
  const f16_t* Wp;         // packed weights (half precision, scaled by W_SCALE)
  const f16_t* Xp;         // packed activations (half precision; K = inner dimension)
  u32 N, K;                // logical output rows and inner dimension (K % 32 == 0)
  u32 T;                   // tokens (columns)
  u32 TBS;                 // token-block stride of the packed activation buffers (the operand Xp and, unless TBS_out is set, the outputs)
  u32 TBS_out;             // 0, or the token-block stride of the packed output Hp when it differs from the operand's
  u32 col0;                // output column of token 0 (EPI_SCALED_STORE row of `out`, EPI_SILU_GATE column of Hp): a grouped
                           // GEMM writes each group's columns behind the previous group's
  const u32* tok_index;    // optional indirection: column t reads token tok_index[t] of Xp / ssq_in (LM head)
  const float* ssq_in;     // [token][K/16] partial sums of squares of the un-normalised input (null: no scaling)
  float eps;
  // EPI_SCALED_STORE
  float* out; u32 ldo;
  // EPI_RESIDUAL
  float* x; u32 ldx;       // residual stream, updated in place
  const float* g_next;     // gain of the RMSNorm that consumes x next
  f16_t* Xp_next;          // packed half(x * g_next), inner dimension N
  float* ssq_out;          // [token][N/16]
  // EPI_SILU_GATE
  f16_t* Hp;               // packed activations with inner dimension N/2
  // EPI_QKV_ROPE
  const i32* positions;
  const i32* slot_mapping;
  const float2* rope_tab;
  f16_t* qbuf;
  f16_t* Kc;               // this layer's K cache and V cache (half precision)
  f16_t* Vc;
  u32 nq, nkv, hd, bs;
  // K split across workgroups (decode iterations of 65..256 tokens in the projections with few rows): the tile kernel
  // leaves fp32 partial sums per K slice here, gemm_splitk_reduce adds them in slice order and runs the epilogue
  float* part;             // [slice][row tile][token block of 16][lane][4]; null: never split
  u64 part_cap;            // floats
  u32 tune_nw;             // tests and tuning. Low three bits: 0 automatic choice of weight tiles per workgroup, 1/2/4 forced.
                           // Bit 5 (launcher): never the kernel chain without the decode attention's merge kernels, bit 7: always.
                           // Bit 9: tile schedule with direct loads instead of LDS staging (bit 8: its 256-token
                           // workgroup tile in eight-wave kernels). Bit 10: no split of K between workgroup halves.
                           // Bit 11: no 64 x 64 streaming items for 64 < T <= 256. Bits 12-14: 2, 3, 4 or 6 force the
                           // token tiles per wave of the LDS-staged tile schedule, 7 its 256-token tile. Bit 20: eight-wave kernels never
                           // take the pair of tiles with shared weight tiles. Bit 21: no tiles wider than 128 tokens.
                           // Bit 15 (scheduler): the decode attention's work items are always chunks, bit 22: always whole
                           // contexts; bit 23: the decode attention kernel with static items. Bits 16-19: waves per item of the
                           // prefill attention. Bit 30: mixed launches run their decode part first in every workgroup.
                           // Bits 24-27: K slices of the split across workgroups (1: never split; 0: automatic).
                           // (Bits 28-29 are read at init: 2 builds the kernel chain with the reduce kernels; only it splits K.)
};

#define GEMM_MAX_WAVES 8
#define GEMM_TILE_LDS 16384   // one k-step of a 128 x 128 workgroup tile: eight 1 KB weight tiles, then eight activation tiles
struct MfmaShared {
  union {
    float red[GEMM_MAX_WAVES][4][64][4];       // [wave][token block][lane][4]  (stream schedule; scratch of the norm scales)
    unsigned char tile[2][2 * GEMM_TILE_LDS];  // [four-wave half of the workgroup][k-step parity]  (tile schedule)
  };
  float rstd[384];   // norm scales of the tokens of a workgroup tile (or pair of tiles)
};

__device__ __forceinline__ u64 packed_off(u32 t, u32 k, u32 TBS) {
  return ((u64)((k >> 5) * TBS + (t >> 4)) * 64 + (t & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

__device__ __forceinline__ f16x8_t as_f16x8(uint4 v) { return *(const f16x8_t*)&v; }
__device__ __forceinline__ f16x8_t ld_op(const f16_t* p) {   // one lane's 16 bytes of a packed tile
  return as_f16x8(*(const uint4*)p);
}

// rstd (times the inverse of the weight scale) of `count` (<= 256) tokens starting at column t0 into
// sh.rstd[off .. off + count). Sixteen lanes share a token:
// each reads every sixteenth 16-byte piece of the token's partial sums (256 contiguous bytes per token and load), up to
// sixteen tokens' loads are in flight per lane, and a butterfly over the sixteen lanes finishes the sum.
__device__ __forceinline__ void compute_rstd(const MfmaGemmArgs& a, u32 t0, u32 count, MfmaShared& sh, u32 off = 0) {
  const u32 tid = threadIdx.x;
  __syncthreads();   // the previous readers of sh.rstd are done
  if (a.ssq_in == nullptr) {
    if (tid < count) sh.rstd[off + tid] = W_SCALE_INV;
  } else if (tid < BLK_THREADS) {   // threads beyond the first 256 (8-wave launches) only join the barriers
    const u32 np = a.K / 16, l16 = tid & 15, grp = tid >> 4;
    const float* pp[16];
    float s[16];
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const u32 t = min(t0 + min(grp + 16 * it, count - 1), a.T - 1);   // clamped: results of padding tokens are dropped
      pp[it] = a.ssq_in + (u64)(a.tok_index ? a.tok_index[t] : t) * np;
      s[it] = 0.f;
    }
    const u32 passes = (count + 15) / 16;
    if ((np & 3u) == 0) {
      for (u32 q = l16 * 4; q < np; q += 64) {
#pragma unroll
        for (int it = 0; it < 16; ++it)
          if ((u32)it < passes) {
            const float4 v = *(const float4*)(pp[it] + q);
            s[it] += (v.x + v.y) + (v.z + v.w);
          }
      }
    } else {
      for (u32 q = l16; q < np; q += 16) {
#pragma unroll
        for (int it = 0; it < 16; ++it)
          if ((u32)it < passes) s[it] += pp[it][q];
      }
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      float v = s[it];
      v += __shfl_xor(v, 1); v += __shfl_xor(v, 2); v += __shfl_xor(v, 4); v += __shfl_xor(v, 8);
      const u32 tl = grp + 16 * it;
      if (l16 == 0 && tl < count) sh.rstd[off + tl] = W_SCALE_INV / sqrtf(v / (float)a.K + a.eps);
    }
  }
  __syncthreads();
}

// Epilogue of one 16(n) x 16(t) accumulator tile held by one wave. rl: index of the tile's first token in sh.rstd.
template <int EPI>
__device__ __forceinline__ void epilogue_tile(const MfmaGemmArgs& a, floatx4_t acc, u32 nt, u32 t_base, const float* rstd16) {
  const u32 lane = threadIdx.x & 63;
  const u32 t = t_base + (lane & 15);
  const u32 n0 = nt * 16 + (lane >> 4) * 4;
  const bool tv = t < a.T;
  if (EPI == EPI_SCALED_STORE) {
    if (!tv) return;
    const float r = rstd16[lane & 15];
    float* o = a.out + (u64)(t + a.col0) * a.ldo + n0;
    if (n0 + 3 < a.N && (a.ldo & 3) == 0) {
      *(float4*)o = make_float4(acc[0] * r, acc[1] * r, acc[2] * r, acc[3] * r);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (n0 + i < a.N) o[i] = acc[i] * r;
    }
  } else if (EPI == EPI_RESIDUAL) {
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (tv) {
      float* xp = a.x + (u64)t * a.ldx + n0;
      const float4 old = *(const float4*)xp;
      v[0] = old.x + acc[0] * W_SCALE_INV; v[1] = old.y + acc[1] * W_SCALE_INV;
      v[2] = old.z + acc[2] * W_SCALE_INV; v[3] = old.w + acc[3] * W_SCALE_INV;
      *(float4*)xp = make_float4(v[0], v[1], v[2], v[3]);
      const float4 g = *(const float4*)(a.g_next + n0);
      *(uint2*)(a.Xp_next + packed_off(t, n0, a.TBS)) = make_uint2(pack_f16x2(v[0] * g.x, v[1] * g.y), pack_f16x2(v[2] * g.z, v[3] * g.w));
    }
    float s = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    if (lane < 16 && tv) a.ssq_out[(u64)t * (a.N / 16) + nt] = s;
  } else if (EPI == EPI_QKV_ROPE) {
    if (!tv) return;
    const float r = rstd16[lane & 15];
    const u32 hd = a.hd, half = hd / 2, head = n0 / hd, p = (n0 % hd) >> 1;   // rows: (p, p+half, p+1, p+1+half)
    float lo0 = acc[0] * r, hi0 = acc[1] * r, lo1 = acc[2] * r, hi1 = acc[3] * r;
    if (head < a.nq + a.nkv) {
      const float4 cs = *(const float4*)(a.rope_tab + (u64)a.positions[t] * half + p);   // (cos,sin) of pairs p, p+1
      const float a0 = lo0 * cs.x - hi0 * cs.y, b0 = hi0 * cs.x + lo0 * cs.y;
      const float a1 = lo1 * cs.z - hi1 * cs.w, b1 = hi1 * cs.z + lo1 * cs.w;
      lo0 = a0; hi0 = b0; lo1 = a1; hi1 = b1;
    }
    if (head < a.nq) {
      const float sc = 1.0f / sqrtf((float)hd);
      f16_t* q = a.qbuf + ((u64)t * a.nq + head) * hd;
      *(u32*)(q + p) = pack_f16x2(lo0 * sc, lo1 * sc);
      *(u32*)(q + half + p) = pack_f16x2(hi0 * sc, hi1 * sc);
    } else {
      const u32 slot = (u32)a.slot_mapping[t];
      if (head < a.nq + a.nkv) {
        f16_t* k = a.Kc + (((u64)(slot / a.bs) * a.nkv + (head - a.nq)) * a.bs + slot % a.bs) * hd;
        *(u32*)(k + p) = pack_f16x2(lo0, lo1);
        *(u32*)(k + half + p) = pack_f16x2(hi0, hi1);
      } else {   // V is kept dimension-major inside a block: [hd][16 tokens]
        f16_t* v = a.Vc + ((u64)(slot / a.bs) * a.nkv + (head - a.nq - a.nkv)) * a.bs * hd + slot % a.bs;
        v[(u64)p * a.bs] = f32_to_f16(lo0);
        v[(u64)(p + 1) * a.bs] = f32_to_f16(lo1);
        v[(u64)(half + p) * a.bs] = f32_to_f16(hi0);
        v[(u64)(half + p + 1) * a.bs] = f32_to_f16(hi1);
      }
    }
  } else {  // EPI_SILU_GATE
    if (!tv) return;
    const float r = rstd16[lane & 15];
    const float g0 = acc[0] * r, u0 = acc[1] * r, g1 = acc[2] * r, u1 = acc[3] * r;
    const float h0 = g0 / (1.f + __expf(-g0)) * u0, h1 = g1 / (1.f + __expf(-g1)) * u1;
    const u32 j = n0 >> 1;   // pair index = inner index of the next GEMM
    *(u32*)(a.Hp + packed_off(t + a.col0, j, a.TBS_out ? a.TBS_out : a.TBS)) = pack_f16x2(h0, h1);
  }
}

// EPI_QKV_ROPE of one tile with its operands already loaded: `r` = the token's norm scale, `slot` = its place in the paged
// cache, `cs` = (cos, sin) of the two rotary pairs of this lane's rows at the token's position (unused for V rows).
__device__ __forceinline__ void rope_finish(const MfmaGemmArgs& a, floatx4_t acc, u32 nt, u32 t, float r, u32 slot, float4 cs) {
  if (t >= a.T) return;
  const u32 lane = threadIdx.x & 63, n0 = nt * 16 + (lane >> 4) * 4;
  const u32 hd = a.hd, half = hd / 2, head = n0 / hd, p = (n0 % hd) >> 1;   // rows: (p, p+half, p+1, p+1+half)
  float lo0 = acc[0] * r, hi0 = acc[1] * r, lo1 = acc[2] * r, hi1 = acc[3] * r;
  if (head < a.nq + a.nkv) {
    const float a0 = lo0 * cs.x - hi0 * cs.y, b0 = hi0 * cs.x + lo0 * cs.y;
    const float a1 = lo1 * cs.z - hi1 * cs.w, b1 = hi1 * cs.z + lo1 * cs.w;
    lo0 = a0; hi0 = b0; lo1 = a1; hi1 = b1;
  }
  if (head < a.nq) {
    const float sc = 1.0f / sqrtf((float)hd);
    f16_t* q = a.qbuf + ((u64)t * a.nq + head) * hd;
    *(u32*)(q + p) = pack_f16x2(lo0 * sc, lo1 * sc);
    *(u32*)(q + half + p) = pack_f16x2(hi0 * sc, hi1 * sc);
  } else if (head < a.nq + a.nkv) {
    f16_t* k = a.Kc + (((u64)(slot / a.bs) * a.nkv + (head - a.nq)) * a.bs + slot % a.bs) * hd;
    *(u32*)(k + p) = pack_f16x2(lo0, lo1);
    *(u32*)(k + half + p) = pack_f16x2(hi0, hi1);
  } else {   // V is kept dimension-major inside a block: [hd][16 tokens]
    f16_t* v = a.Vc + ((u64)(slot / a.bs) * a.nkv + (head - a.nq - a.nkv)) * a.bs * hd + slot % a.bs;
    v[(u64)p * a.bs] = f32_to_f16(lo0);
    v[(u64)(p + 1) * a.bs] = f32_to_f16(lo1);
    v[(u64)(half + p) * a.bs] = f32_to_f16(hi0);
    v[(u64)(half + p + 1) * a.bs] = f32_to_f16(hi1);
  }
}

// EPI_RESIDUAL of one tile with its operands already loaded: `old` = this lane's four residual values of token
// min(t, T - 1) (the caller's unconditional load), `g` = the next norm's gains of its four rows.
__device__ __forceinline__ void residual_finish(const MfmaGemmArgs& a, floatx4_t acc, u32 nt, u32 t, float4 old, float4 g) {
  const u32 lane = threadIdx.x & 63, n0 = nt * 16 + (lane >> 4) * 4;
  const bool tv = t < a.T;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  if (tv) {
    v[0] = old.x + acc[0] * W_SCALE_INV; v[1] = old.y + acc[1] * W_SCALE_INV;
    v[2] = old.z + acc[2] * W_SCALE_INV; v[3] = old.w + acc[3] * W_SCALE_INV;
    *(float4*)(a.x + (u64)t * a.ldx + n0) = make_float4(v[0], v[1], v[2], v[3]);
    *(uint2*)(a.Xp_next + packed_off(t, n0, a.TBS)) = make_uint2(pack_f16x2(v[0] * g.x, v[1] * g.y), pack_f16x2(v[2] * g.z, v[3] * g.w));
  }
  float s = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  s += __shfl_xor(s, 16);
  s += __shfl_xor(s, 32);
  if (lane < 16 && tv) a.ssq_out[(u64)t * (a.N / 16) + nt] = s;
}

// Epilogue of the TJ accumulator tiles a wave holds for one row tile (tokens t_base + 16 j + lane % 16). The epilogues that
// read memory (the residual stream, the positions and the rotary table) request the operands of all TJ tiles first and
// then compute and store tile by tile: written one tile after the other, every tile's loads would wait behind the
// previous tile's stores (the compiler has to assume that they may alias), a chain of TJ memory latencies per row tile.
// Tokens behind the last one read the last token's operands (an unconditional load) and store nothing.
// (Bit 6 of the tuning word: tile by tile, for comparison.)
template <int EPI, int TJ>
__device__ __forceinline__ void epilogue_row(const MfmaGemmArgs& a, const floatx4_t (&acc)[TJ], u32 nt, u32 t_base, const float* rstd) {
  if ((EPI != EPI_RESIDUAL && EPI != EPI_QKV_ROPE) || (a.tune_nw & 0x40u)) {
#pragma unroll
    for (int j = 0; j < TJ; ++j) epilogue_tile<EPI>(a, acc[j], nt, t_base + j * 16, rstd + j * 16);
    return;
  }
  const u32 lane = threadIdx.x & 63;
  const u32 n0 = nt * 16 + (lane >> 4) * 4;
  u32 t[TJ], tc[TJ];
#pragma unroll
  for (int j = 0; j < TJ; ++j) { t[j] = t_base + j * 16 + (lane & 15); tc[j] = min(t[j], a.T - 1); }
  if (EPI == EPI_RESIDUAL) {
    float4 old[TJ];
#pragma unroll
    for (int j = 0; j < TJ; ++j) old[j] = *(const float4*)(a.x + (u64)tc[j] * a.ldx + n0);
    const float4 g = *(const float4*)(a.g_next + n0);
#pragma unroll
    for (int j = 0; j < TJ; ++j) residual_finish(a, acc[j], nt, t[j], old[j], g);
  } else {   // EPI_QKV_ROPE
    const u32 hd = a.hd, half = hd / 2, head = n0 / hd, p = (n0 % hd) >> 1;   // rows: (p, p+half, p+1, p+1+half)
    const bool rot = head < a.nq + a.nkv;
    i32 pos[TJ];
    u32 slot[TJ];
#pragma unroll
    for (int j = 0; j < TJ; ++j) { pos[j] = a.positions[tc[j]]; slot[j] = (u32)a.slot_mapping[tc[j]]; }
    float4 cs[TJ];
#pragma unroll
    for (int j = 0; j < TJ; ++j) cs[j] = *(const float4*)(a.rope_tab + (u64)(rot ? pos[j] : 0) * half + (rot ? p : 0u));   // (cos,sin) of pairs p, p+1
#pragma unroll
    for (int j = 0; j < TJ; ++j) rope_finish(a, acc[j], nt, t[j], rstd[j * 16 + (lane & 15)], slot[j], cs[j]);
  }
}

// ---- stream schedule: T <= 64 ------------------------------------------------------------------------------------
// Weight loads bypass temporal caching: every weight byte is used once per launch, while the activation operand
// is re-read by every workgroup and should stay in L2.
__device__ __forceinline__ f16x8_t ld_op_stream(const f16_t* p) {
  typedef u32 u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
  return *(const f16x8_t*)&v;
}

// Work item of a workgroup in the round that starts at item `base`. Workgroups are dealt to the eight XCDs round-robin
// (workgroup id modulo 8), and each XCD has its own L2: the workgroups of one XCD take consecutive items, so that the
// operand blocks those items share are fetched into that L2 once. Returns ~0u when the round has no item for `wg`.
__device__ __forceinline__ u32 xcd_item(u32 base, u32 total, u32 wg, u32 nwg) {
  const u32 cnt = min(nwg, total - base);
  if (nwg & 7u) return wg < cnt ? base + wg : ~0u;
  const u32 q = (cnt + 7) / 8, x = wg & 7u, l = wg >> 3, off = x * q + l;
  return (l < q && off < cnt) ? base + off : ~0u;
}

template <int U, int NW, int TW>
struct StreamBuf {
  f16x8_t w[U][NW];
  f16x8_t x[U][TW];
};

// NW consecutive 16-row weight tiles per workgroup: every activation tile a wave loads is used for NW MFMAs, which
// divides the L2 traffic of the activation operand by NW (it is TW/NW times the weight bytes).
// k-tiles per batch of loads (two batches are in flight per wave). Measured on MI355X under the budget of 256 registers
// per lane that lets two four-wave workgroups share a compute unit: the widest variants keep fewer k-tiles per batch.
constexpr int stream_batch(int NW, int TW) {
  return NW == 1 ? (TW == 1 ? 8 : (TW == 2 ? 6 : 4))
       : NW == 4 ? (TW >= 3 ? 1 : 3)
       : ((NW * TW >= 8) ? 2 : (NW + TW >= 5 ? 3 : 4));
}
// GRID2D (64 < T <= 256, four token blocks per item): the work items are (tile group, group of 64 tokens) pairs, the
// token group varying fastest so that the workgroups running together share weight rows in L2; the weight loads are
// ordinary (cached) ones then.
template <int EPI, int NW, int TW, int U = stream_batch(NW, TW), bool GRID2D = false>
__device__ __forceinline__ void gemm_stream(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg) {
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const u32 NT = (a.N + 15) / 16, KT = a.K / 32;
  const u32 TG = GRID2D ? (a.T + 63) / 64 : 1u;            // groups of 64 tokens
  const u32 NG = ((NT + NW - 1) / NW) * TG;                // work items: groups of NW tiles x token groups
  const u32 KS = blockDim.x >> 6;                          // waves of the workgroup: each takes a slice of K
  const u32 kb = (u32)((u64)KT * w / KS), ke = (u32)((u64)KT * (w + 1) / KS);
  const u32 nbatch = (KT / KS + (KT % KS ? 1 : 0) + U - 1) / U;   // same count in every wave (loads past `ke` are zeros)
  // GRID2D: the items of one round go to the XCDs in runs (the token groups of a tile group share the weight rows in
  // one L2); otherwise item = workgroup + round * workgroups
  u32 round = 0;
  auto item_of = [&](u32 r) -> u32 {
    const u32 base = r * nwg;
    if (base >= NG) return ~0u;
    return GRID2D ? xcd_item(base, NG, wg, nwg) : (base + wg < NG ? base + wg : ~0u);
  };
  if (item_of(0) == ~0u) return;
  // per-lane offsets (in elements) of this lane's 16 bytes inside the token blocks of one k-tile
  u32 xoff[TW];
#pragma unroll
  for (int tw = 0; tw < TW; ++tw) {
    u32 tok = tw * 16 + (lane & 15);
    if (a.tok_index) tok = tok < a.T ? a.tok_index[tok] : 0;
    xoff[tw] = ((tok >> 4) * 64 + (tok & 15) + 16 * (lane >> 4)) * 8;
  }
  const u64 xk_stride = (u64)a.TBS * 512;
  const f16x8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
  auto issue = [&](StreamBuf<U, NW, TW>& b, u32 item, u32 kt0) {
    const u32 ng = item / TG;
    const bf16_t* xg = a.Xp + (u64)(item % TG) * (TW * 512);   // the item's token group: TW consecutive token blocks
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u32 kt = kt0 + u;
      const bool ok = kt < ke;
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        const u32 nt = min(ng * NW + i, NT - 1);           // a tile past the end is computed and dropped
        const bf16_t* wp = a.Wp + ((u64)nt * KT + kt) * 512 + lane * 8;
        b.w[u][i] = ok ? (GRID2D ? ld_op(wp) : ld_op_stream(wp)) : zero;
      }
#pragma unroll
      for (int tw = 0; tw < TW; ++tw) b.x[u][tw] = ok ? ld_op(xg + (u64)kt * xk_stride + xoff[tw]) : zero;
    }
  };
  // Software pipeline over the flat sequence of (tile group, batch) steps of this workgroup: while one buffer is
  // consumed by the MFMAs, the loads of the following step (possibly the first batch of the next group) fill the
  // other. The two buffers swap roles by code position (no register copies, which would wait for loads in flight).
  StreamBuf<U, NW, TW> bufA, bufB;
  u32 ng = item_of(0), b = 0;
  floatx4_t acc[NW][TW];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int tw = 0; tw < TW; ++tw) acc[i][tw] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  issue(bufA, ng, kb);               // the first loads are in flight while the norm scales are computed
  compute_rstd(a, 0, min(64 * TG, 256u), sh);
  auto step = [&](StreamBuf<U, NW, TW>& use, StreamBuf<U, NW, TW>& fill) -> bool {
    const bool last = b + 1 >= nbatch;
    const u32 nng = last ? item_of(round + 1) : ng;
    if (nng < NG) issue(fill, nng, last ? kb : kb + (b + 1) * U);
    {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < NW; ++i)
#pragma unroll
          for (int tw = 0; tw < TW; ++tw)
            acc[i][tw] = __builtin_amdgcn_mfma_f32_16x16x32_f16(use.w[u][i], use.x[u][tw], acc[i][tw], 0, 0, 0);
    }
    if (!last) { ++b; return true; }
    // the residual values and gains the epilogue of this wave's tiles will need: requested before the reduction, not behind it
    float4 pre_old[NW], pre_g[NW];
    if (EPI == EPI_RESIDUAL && w < TW && !(a.tune_nw & 0x40u)) {
      const u32 tq = min((ng % TG) * 64 + w * 16 + (lane & 15), a.T - 1);
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        const u32 n0 = min((ng / TG) * NW + i, NT - 1) * 16 + (lane >> 4) * 4;
        pre_old[i] = *(const float4*)(a.x + (u64)tq * a.ldx + n0);
        pre_g[i] = *(const float4*)(a.g_next + n0);
      }
    }
    float4 pre_cs[NW];
    u32 pre_slot = 0;
    if (EPI == EPI_QKV_ROPE && w < TW && !(a.tune_nw & 0x40u)) {     // likewise the position, the cache slot and the rotary table entries
      const u32 tq = min((ng % TG) * 64 + w * 16 + (lane & 15), a.T - 1), half = a.hd / 2;
      const u32 pos = (u32)a.positions[tq];
      pre_slot = (u32)a.slot_mapping[tq];
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        const u32 n0 = min((ng / TG) * NW + i, NT - 1) * 16 + (lane >> 4) * 4;
        const bool rot = n0 / a.hd < a.nq + a.nkv;
        pre_cs[i] = *(const float4*)(a.rope_tab + (u64)(rot ? pos : 0u) * half + (rot ? (n0 % a.hd) >> 1 : 0u));
      }
    }
    // reduce the four K-quarters through LDS, one weight tile of the group at a time
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      __syncthreads();   // the previous reduction has been read
#pragma unroll
      for (int tw = 0; tw < TW; ++tw) *(floatx4_t*)&sh.red[w][tw][lane][0] = acc[i][tw];
      __syncthreads();
      const u32 nt = (ng / TG) * NW + i, tg = ng % TG;
      if (w < TW && nt < NT) {               // wave w finishes token block w: fixed summation order
        floatx4_t s = (*(floatx4_t*)&sh.red[0][w][lane][0] + *(floatx4_t*)&sh.red[1][w][lane][0]) +
                      (*(floatx4_t*)&sh.red[2][w][lane][0] + *(floatx4_t*)&sh.red[3][w][lane][0]);
        if (KS == 8)
          s += (*(floatx4_t*)&sh.red[4][w][lane][0] + *(floatx4_t*)&sh.red[5][w][lane][0]) +
               (*(floatx4_t*)&sh.red[6][w][lane][0] + *(floatx4_t*)&sh.red[7][w][lane][0]);
        if (EPI == EPI_RESIDUAL && !(a.tune_nw & 0x40u)) residual_finish(a, s, nt, tg * 64 + w * 16 + (lane & 15), pre_old[i], pre_g[i]);
        else if (EPI == EPI_QKV_ROPE && !(a.tune_nw & 0x40u))
          rope_finish(a, s, nt, tg * 64 + w * 16 + (lane & 15), sh.rstd[tg * 64 + w * 16 + (lane & 15)], pre_slot, pre_cs[i]);
        else epilogue_tile<EPI>(a, s, nt, tg * 64 + w * 16, &sh.rstd[tg * 64 + w * 16]);
      }
#pragma unroll
      for (int tw = 0; tw < TW; ++tw) acc[i][tw] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    }
    ng = nng;
    b = 0;
    ++round;
    return ng < NG;
  };
  for (;;) {
    if (!step(bufA, bufB)) break;
    if (!step(bufB, bufA)) break;
  }
}

// ---- tile schedule: T > 64 -----------------------------------------------------------------------------------------
template <int EPI>
__device__ __forceinline__ void gemm_tile(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg) {
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const u32 NT = (a.N + 15) / 16, KT = a.K / 32;
  // workgroup tile: 128 rows x 128 tokens with four waves (2 x 2). An eight-wave launch takes 128 rows x 256 tokens
  // (2 x 4 waves) when that still leaves enough tiles for the chip; otherwise its waves 4..7 only join the barriers.
  const u32 nblocks = (NT + 7) / 8;
  const bool eight = blockDim.x == 512 && (nblocks * ((a.T + 255) / 256) >= 384 || (a.tune_nw & 0x100u));
  const u32 BT = eight ? 256u : 128u;
  const u32 tblocks = (a.T + BT - 1) / BT;
  const bool spare = !eight && w >= 4;
  const u32 wn = w & 1, wt = eight ? (w >> 1) : ((w >> 1) & 1);
  const u64 xk_stride = (u64)a.TBS * 512;
  for (u32 item = wg; item < nblocks * tblocks; item += nwg) {
    // token blocks vary fastest: the workgroups running together share a few weight row blocks (each read from HBM once
    // and then from L2) and sweep all token blocks, whose operand is small enough to stay in L2 / the memory-side cache
    const u32 tb = item % tblocks, nb = item / tblocks;
    compute_rstd(a, tb * BT, BT, sh);
    if (spare) continue;
    const u32 nt0 = nb * 8 + wn * 4;
    u32 xoff[4];
#pragma unroll
    for (int tw = 0; tw < 4; ++tw) {
      u32 tok = tb * BT + wt * 64 + tw * 16 + (lane & 15);
      if (a.tok_index) tok = tok < a.T ? a.tok_index[tok] : 0;
      else tok = min(tok, a.TBS * 16 - 1);                 // stay inside the operand buffer past the last token block
      xoff[tw] = ((tok >> 4) * 64 + (tok & 15) + 16 * (lane >> 4)) * 8;
    }
    const bf16_t* wp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) wp[i] = a.Wp + ((u64)min(nt0 + i, NT - 1) * KT) * 512 + lane * 8;
    floatx4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    // three k-steps of operand tiles in flight; the buffers rotate by code position (no register copies)
    struct Step { f16x8_t w[4], x[4]; };
    Step s0, s1, s2;
    auto ld = [&](Step& st, u32 kt) {
      if (kt < KT) {
#pragma unroll
        for (int i = 0; i < 4; ++i) st.w[i] = ld_op(wp[i] + (u64)kt * 512);
#pragma unroll
        for (int j = 0; j < 4; ++j) st.x[j] = ld_op(a.Xp + (u64)kt * xk_stride + xoff[j]);
      }
    };
    auto mm = [&](const Step& st, u32 kt) {
      if (kt < KT) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(st.w[i], st.x[j], acc[i][j], 0, 0, 0);
      }
    };
    ld(s0, 0); ld(s1, 1); ld(s2, 2);
    for (u32 kt = 0; kt < KT; kt += 3) {
      mm(s0, kt); ld(s0, kt + 3);
      mm(s1, kt + 1); ld(s1, kt + 4);
      mm(s2, kt + 2); ld(s2, kt + 5);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (nt0 + i < NT) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          epilogue_tile<EPI>(a, acc[i][j], nt0 + i, tb * BT + wt * 64 + j * 16, &sh.rstd[wt * 64 + j * 16]);
      }
  }
}

// Tile order of the tile schedule: token blocks in groups of eight; inside a group the row blocks follow each other and
// the token block varies fastest, so 64 consecutive tiles are 8 row blocks x 8 token blocks (16 operand blocks in all).
__device__ __forceinline__ void tile_coords(u32 i, u32 nblocks, u32 tblocks, u32& nb, u32& tb) {
  const u32 gsz = nblocks * 8, g = min(i / gsz, tblocks / 8), rem = i - g * gsz;
  const u32 width = min(8u, tblocks - g * 8);
  nb = rem / width;
  tb = g * 8 + rem % width;
}

// ---- K split across workgroups ---------------------------------------------------------------------------------------
// With 65..256 tokens a projection of 4096..6144 rows has only 64..96 tiles of 128 x 128, a quarter of the tile slots of
// the chip (two four-wave tiles per compute unit). Splitting K into S slices gives every slot an item; the partial sums
// (fp32, in the accumulators' own layout: 1 KB per 16 x 16 tile and slice, written and read with 16-byte lane accesses)
// stay in the L2s and the memory-side cache, and a second kernel adds them in slice order (fixed: the result does not
// depend on timing) and runs the epilogue. Returns the number of slices for this launch, 0 for "not split"; the GEMM
// kernel and its reduce kernel are launched with the same grid and derive the same number.
__device__ __forceinline__ u32 splitk_slices(const MfmaGemmArgs& a, u32 nwg, u32 gemm_threads) {
  if (a.part == nullptr || a.T <= 64 || a.T > 256 || a.tok_index != nullptr || gemm_threads != 512) return 0;
  const u32 KT = a.K / 32, nblocks = ((a.N + 15) / 16 + 7) / 8, tblocks = (a.T + 127) / 128, tiles = nblocks * tblocks;
  const u32 forced = (a.tune_nw >> 24) & 15u;
  u32 S = forced ? forced : min(8u, max(1u, nwg / tiles));   // tile slots resident at once: one eight-wave workgroup per CU, nwg = 2 per CU
  // both halves of a workgroup run the same number of k-steps (they share the barriers): slices of equal length, or an
  // even number of tiles (then the two halves' items always lie in one slice); at least eight k-steps per slice
  while (S > 1 && (KT / S < 8 || ((tiles & 1u) && KT % S) || (u64)S * nblocks * 8 * tblocks * 8 * 256 > a.part_cap)) --S;
  return S > 1 ? S : 0u;
}

// ---- tile schedule through LDS: T > 64 ---------------------------------------------------------------------------
// 128 rows x 128 tokens per four waves (64 x 64 per wave). Every k-step, the four waves fetch the step's eight weight
// tiles and eight activation tiles from global memory once (two steps ahead, in registers), store them into one of two
// LDS buffers, and read their own four + four operand tiles of the *next* step from the other buffer into a second
// register set while the MFMAs of the current step run: one barrier per k-step, global traffic half of what four
// waves loading their operands directly would request. An eight-wave workgroup runs two such tiles side by side
// (separate LDS buffers, common barriers).
// TJ (2, 3 or 4): token tiles per wave; the workgroup tile is 128 rows x 32 TJ tokens. Narrower tiles cost more operand
// traffic per flop but cut the tile grid finer: gemm_tile_pick takes the width whose rounds of workgroups finish first.
// PART: K is split into `slices` slices across work items (splitk_slices); an item accumulates one slice of one tile and
// stores the raw sums to a.part instead of running the epilogue.
template <int EPI, int TJ, bool PART = false>
__device__ __forceinline__ void gemm_tile_lds(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg, u32 slices = 1) {
  constexpr u32 BT = 32 * TJ, XT = 2 * TJ;        // tokens and activation tiles of a workgroup tile
  // bytes of one LDS buffer; the 192-token tile (TJ = 6, 20 KB per buffer) takes both halves' space and so runs in
  // four-wave workgroups only
  constexpr u32 TLB = TJ > 4 ? (8 + XT) * 1024 : GEMM_TILE_LDS;
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const u32 halves = blockDim.x >> 8, half = w >> 2, wl = w & 3, wn = wl & 1, wt = wl >> 1;
  const u32 NT = (a.N + 15) / 16, KT = a.K / 32;
  const u32 nblocks = (NT + 7) / 8, tblocks = (a.T + BT - 1) / BT, total = nblocks * tblocks;
  const u64 xk_stride = (u64)a.TBS * 512, w_stride = (u64)KT * 512;
  // LDS buffer of one k-step: weight tiles 0..7, then activation tiles 0..XT-1 (1 KB each). This wave stores weight
  // tiles 2 wl, 2 wl + 1 and activation tiles wl, wl + 4 and wl + 8 (the latter two only if the tile has that many)
  const bool x2 = TJ >= 4 || wl + 4 < XT;     // known at compile time for full-width tiles: no branch around the load
  constexpr bool x3 = TJ > 4;
  unsigned char* const Lww = sh.tile[half] + (wl * 2) * 1024 + lane * 16;
  unsigned char* const Lwx = sh.tile[half] + 8192 + wl * 1024 + lane * 16;
  const unsigned char* const Lrw = sh.tile[half] + (wn * 4) * 1024 + lane * 16;
  const unsigned char* const Lrx = sh.tile[half] + 8192 + (wt * TJ) * 1024 + lane * 16;
  // When that takes fewer rounds of eight-wave workgroups (one runs per CU, two are launched per CU), the two
  // halves of a workgroup share one tile: each accumulates half of K, and the second half's sums are added to the
  // first's through LDS before the epilogue (fixed order, so the result does not depend on timing).
  // (rounds of workgroups, one per CU: a tile takes a workgroup half as long when its halves share it)
  const u32 ncu = nwg / 2, rounds_split = (total + ncu - 1) / ncu, rounds_pair = ((total + 1) / 2 + ncu - 1) / ncu;
  const bool splitk = !PART && TJ <= 4 && halves == 2 && (KT & 1u) == 0 && rounds_split < 2 * rounds_pair && !(a.tune_nw & 0x400u);   // bit 10: never (tests)
  const u32 per_item = splitk ? 1u : halves;
  const u32 S = PART ? slices : 1u, all_items = total * S;      // items in slice-major order: tile = item % total
  const u32 nitems = (all_items + per_item - 1) / per_item;
  for (u32 base = 0; base < nitems; base += nwg) {
    const u32 it = xcd_item(base, nitems, wg, nwg);
    if (it == ~0u) continue;
    const u32 item = splitk ? it : it * halves + half;
    const bool valid = item < all_items;        // the spare half of the last pair computes a duplicate and drops it
    const u32 ks = min(item, all_items - 1) / total;   // (the spare half walks its partner's slice: same number of k-steps)
    const u32 k0 = PART ? (u32)((u64)KT * ks / S) : ((splitk && half) ? KT / 2 : 0u);
    const u32 kn = PART ? (u32)((u64)KT * (ks + 1) / S) - k0 : (splitk ? KT / 2 : KT), klast = k0 + kn - 1;
    u32 tb = 0, nb = 0;
    if (valid) tile_coords(item % total, nblocks, tblocks, nb, tb);
    const u32 nt0 = nb * 8 + wn * 4;
    const bf16_t* const gw0 = a.Wp + (u64)min(nb * 8 + wl * 2, NT - 1) * w_stride + lane * 8;
    const bf16_t* const gw1 = a.Wp + (u64)min(nb * 8 + wl * 2 + 1, NT - 1) * w_stride + lane * 8;
    // this lane's 16 bytes of the two activation tiles its wave fetches; through the token indirection (LM head) the
    // sixteen tokens of a tile come from arbitrary columns of the operand. A tile past the operand's last token block
    // (only in the last workgroup tile) is clamped: its columns are dropped by the epilogue.
    const bf16_t *gx0, *gx1, *gx2;
    if (a.tok_index) {
      const u32 ta = tb * BT + wl * 16 + (lane & 15);
      const u32 s0 = a.tok_index[min(ta, a.T - 1)], s1 = a.tok_index[min(ta + 64, a.T - 1)], s2 = a.tok_index[min(ta + 128, a.T - 1)];
      gx0 = a.Xp + ((u64)(s0 >> 4) * 64 + (s0 & 15) + 16 * (lane >> 4)) * 8;
      gx1 = a.Xp + ((u64)(s1 >> 4) * 64 + (s1 & 15) + 16 * (lane >> 4)) * 8;
      gx2 = a.Xp + ((u64)(s2 >> 4) * 64 + (s2 & 15) + 16 * (lane >> 4)) * 8;
    } else {
      gx0 = a.Xp + (u64)min(tb * XT + wl, a.TBS - 1) * 512 + lane * 8;
      gx1 = a.Xp + (u64)min(tb * XT + wl + 4, a.TBS - 1) * 512 + lane * 8;
      gx2 = a.Xp + (u64)min(tb * XT + wl + 8, a.TBS - 1) * 512 + lane * 8;
    }
    floatx4_t acc[4][TJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    // staging registers as separate variables (arrays or structs of them may end up in scratch memory)
    uint4 ga0, ga1, ga2, ga3, ga4, gb0, gb1, gb2, gb3, gb4;
    ga3 = gb3 = ga4 = gb4 = make_uint4(0, 0, 0, 0);
#define TL_GLOAD(g, kt) { const u32 kc_ = min(k0 + (u32)(kt), klast);                                                      \
      g##0 = *(const uint4*)(gw0 + (u64)kc_ * 512); g##1 = *(const uint4*)(gw1 + (u64)kc_ * 512);                          \
      g##2 = *(const uint4*)(gx0 + (u64)kc_ * xk_stride); if (x2) g##3 = *(const uint4*)(gx1 + (u64)kc_ * xk_stride);         \
      if (x3) g##4 = *(const uint4*)(gx2 + (u64)kc_ * xk_stride); }
#define TL_STORE(g, buf) { *(uint4*)(Lww + (buf) * TLB) = g##0; *(uint4*)(Lww + (buf) * TLB + 1024) = g##1;                      \
      *(uint4*)(Lwx + (buf) * TLB) = g##2; if (x2) *(uint4*)(Lwx + (buf) * TLB + 4096) = g##3;                             \
      if (x3) *(uint4*)(Lwx + (buf) * TLB + 8192) = g##4; }
#define TL_RW(buf, i) as_f16x8(*(const uint4*)(Lrw + (buf) * TLB + (i) * 1024))
#define TL_RX(buf, j) as_f16x8(*(const uint4*)(Lrx + (buf) * TLB + ((j) < TJ ? (j) : 0) * 1024))
#define TL_MM(A, W, X) A = __builtin_amdgcn_mfma_f32_16x16x32_f16(W, X, A, 0, 0, 0);
#define TL_ROW(i, o) TL_MM(acc[i][0], o.w##i, o.x0) TL_MM(acc[i][1], o.w##i, o.x1)                                         \
      if (TJ > 2) { TL_MM(acc[i][TJ > 2 ? 2 : 0], o.w##i, o.x2) } if (TJ > 3) { TL_MM(acc[i][TJ > 3 ? 3 : 0], o.w##i, o.x3) }            \
      if (TJ > 4) { TL_MM(acc[i][TJ > 4 ? 4 : 0], o.w##i, o.x4) TL_MM(acc[i][TJ > 4 ? 5 : 0], o.w##i, o.x5) }
#define TL_SB __builtin_amdgcn_sched_barrier(0);
    // step k with its operands in `o`: reads the operands of step k+1 from LDS buffer rb into `n`, stores the staged data
    // of step k+2 (in g) into LDS buffer wb and requests step k+4 into g
#define TL_STEP(o, n, g, k, rb, wb)                                                                                       \
    n.x0 = TL_RX(rb, 0); n.w0 = TL_RW(rb, 0); n.x1 = TL_RX(rb, 1); n.w1 = TL_RW(rb, 1); TL_STORE(g, wb)                   \
    TL_SB TL_ROW(0, o) TL_ROW(1, o) TL_SB                                                                                 \
    if (TJ > 2) n.x2 = TL_RX(rb, 2);                                                                                      \
    n.w2 = TL_RW(rb, 2); if (TJ > 3) n.x3 = TL_RX(rb, 3);                                                                  \
    if (TJ > 4) { n.x4 = TL_RX(rb, 4); n.x5 = TL_RX(rb, 5); }                                                             \
    n.w3 = TL_RW(rb, 3); TL_GLOAD(g, (k) + 4)                                                                             \
    TL_SB TL_ROW(2, o) TL_ROW(3, o) TL_SB                                                                                 \
    __syncthreads();
    struct Ops { f16x8_t w0, w1, w2, w3, x0, x1, x2, x3, x4, x5; };
    Ops oa, ob;
    TL_GLOAD(ga, 0) TL_GLOAD(gb, 1)             // in flight while the norm scales are computed
    if (PART) __syncthreads();                  // the previous item's last reads of the LDS tiles are done (the norm scales belong to the reduce kernel)
    else
      for (u32 h = 0; h < per_item; ++h) {
        const u32 ih = it * per_item + h;
        u32 tbh = 0, nbh = 0;
        if (ih < total) tile_coords(ih, nblocks, tblocks, nbh, tbh);
        compute_rstd(a, tbh * BT, BT, sh, h * 128);   // its barriers: the LDS tiles are free
      }
    TL_STORE(ga, 0) TL_STORE(gb, 1) TL_GLOAD(ga, 2) TL_GLOAD(gb, 3)
    __syncthreads();
    oa.w0 = TL_RW(0, 0); oa.w1 = TL_RW(0, 1); oa.w2 = TL_RW(0, 2); oa.w3 = TL_RW(0, 3);
    oa.x0 = TL_RX(0, 0); oa.x1 = TL_RX(0, 1); oa.x2 = TL_RX(0, 2); oa.x3 = TL_RX(0, 3); oa.x4 = TL_RX(0, 4); oa.x5 = TL_RX(0, 5);
    __syncthreads();   // step 0 overwrites buffer 0, which every wave has just read (later steps read a buffer one step ahead)
    for (u32 k = 0; k < kn; k += 2) {
      TL_STEP(oa, ob, ga, k, 1, 0)
      if (k + 1 < kn) { TL_STEP(ob, oa, gb, k + 1, 0, 1) }
    }
#undef TL_GLOAD
#undef TL_STORE
#undef TL_RW
#undef TL_RX
#undef TL_MM
#undef TL_ROW
#undef TL_SB
#undef TL_STEP
    if (splitk) {   // the last barrier of the k loop has passed: the LDS tiles (64 KB in all) are free
      float* red = (float*)&sh.tile[0][0] + ((u64)wl * 16 * 64 + lane) * 4;
      if (half == 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < TJ; ++j) *(floatx4_t*)(red + (i * 4 + (j & 3)) * 256) = acc[i][j];   // (never taken with TJ > 4)
      }
      __syncthreads();
      if (half == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < TJ; ++j) acc[i][j] += *(const floatx4_t*)(red + (i * 4 + (j & 3)) * 256);
      }
    }
    if (PART) {
      if (valid) {
        const u32 NTp = nblocks * 8, TBp = tblocks * (BT / 16);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < TJ; ++j)
            *(floatx4_t*)(a.part + ((((u64)ks * NTp + nt0 + i) * TBp + tb * (BT / 16) + wt * TJ + j) * 64 + lane) * 4) = acc[i][j];
      }
      continue;
    }
    const u32 rstd_off = splitk ? 0u : half * 128;
    if (valid && !(splitk && half)) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (nt0 + i < NT) {
          epilogue_row<EPI, TJ>(a, acc[i], nt0 + i, tb * BT + wt * TJ * 16, &sh.rstd[rstd_off + wt * TJ * 16]);
        }
    }
  }
}

// Second kernel of a GEMM whose K was split across workgroups: adds the slices' partial sums in slice order and runs the
// epilogue. Work item: (block of 16 tokens, group of row tiles); every wave takes two row tiles of the group and has
// all their slices' loads in flight together. Launched with four waves per workgroup and the grid of the GEMM kernel.
template <int EPI>
__device__ __forceinline__ void gemm_splitk_reduce(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg, u32 gemm_threads) {
  const u32 S = splitk_slices(a, nwg, gemm_threads);   // gemm_threads: block size of the GEMM kernel (this kernel runs four waves)
  if (S == 0) return;
  const u32 NT = (a.N + 15) / 16, nblocks = (NT + 7) / 8, tblocks = (a.T + 127) / 128;
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const u32 NTp = nblocks * 8, TBp = tblocks * 8, TB16 = (a.T + 15) / 16;
  constexpr u32 RPW = 2;
  const u32 groups = (NT + nw * RPW - 1) / (nw * RPW);
  for (u32 item = wg; item < TB16 * groups; item += nwg) {
    const u32 tb = item % TB16, g = item / TB16;
    floatx4_t v[RPW][8];
#pragma unroll
    for (u32 r = 0; r < RPW; ++r) {
      const u32 nt = min((g * nw + w) * RPW + r, NT - 1);
#pragma unroll
      for (u32 s = 0; s < 8; ++s)
        v[r][s] = *(const floatx4_t*)(a.part + ((((u64)min(s, S - 1) * NTp + nt) * TBp + tb) * 64 + lane) * 4);
    }
    compute_rstd(a, tb * 16, 16, sh);       // (its barriers also separate the items' uses of sh.rstd)
#pragma unroll
    for (u32 r = 0; r < RPW; ++r) {
      const u32 nt = (g * nw + w) * RPW + r;
      floatx4_t sum = v[r][0];
#pragma unroll
      for (u32 s = 1; s < 8; ++s)
        if (s < S) sum += v[r][s];
      if (nt < NT) epilogue_tile<EPI>(a, sum, nt, tb * 16, &sh.rstd[0]);
    }
  }
}

// Eight waves on a pair of tiles that are neighbours along the tokens: 128 rows x (2 x 32 TJ) tokens. The halves of the
// workgroup (four waves each, a tile each) share the eight weight tiles of every k-step in LDS, so the workgroup
// fetches 8 + 2 XT operand tiles per step instead of 2 x (8 + XT): a quarter less traffic between L2 and the compute
// unit, which is what bounds the tile schedule. Same pipeline as gemm_tile_lds.
template <int EPI, int TJ>
__device__ __forceinline__ void gemm_tile_lds_pair(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg) {
  constexpr u32 BT = 32 * TJ, XT = 2 * TJ, LB = 2 * GEMM_TILE_LDS;   // one LDS buffer: 8 weight tiles + 2 XT activation tiles <= 32 KB
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6;           // eight waves
  const u32 half = w >> 2, wl = w & 3, wn = wl & 1, wt = wl >> 1;
  const u32 NT = (a.N + 15) / 16, KT = a.K / 32;
  const u32 nblocks = (NT + 7) / 8, tblocks = (a.T + BT - 1) / BT, tpairs = (tblocks + 1) / 2, total = nblocks * tpairs;
  const u64 xk_stride = (u64)a.TBS * 512, w_stride = (u64)KT * 512;
  // wave w stores weight tile w and activation tiles w, w + 8 and w + 16 of the pair's 2 XT (those that exist)
  const bool x2 = TJ >= 4 || w + 8 < 2 * XT;
  constexpr bool x3 = TJ > 4;
  unsigned char* const L0 = &sh.tile[0][0];
  unsigned char* const Lww = L0 + w * 1024 + lane * 16;
  unsigned char* const Lwx = L0 + 8192 + w * 1024 + lane * 16;
  const unsigned char* const Lrw = L0 + (wn * 4) * 1024 + lane * 16;
  const unsigned char* const Lrx = L0 + 8192 + (half * XT + wt * TJ) * 1024 + lane * 16;
  for (u32 base = 0; base < total; base += nwg) {
    const u32 it = xcd_item(base, total, wg, nwg);
    if (it == ~0u) continue;
    u32 tp = 0, nb = 0;
    tile_coords(it, nblocks, tpairs, nb, tp);
    const u32 tb = tp * 2 + half;
    const bool valid = tb < tblocks;            // an odd number of token blocks leaves the last pair's second half idle
    const u32 nt0 = nb * 8 + wn * 4;
    const bf16_t* const gw = a.Wp + (u64)min(nb * 8 + w, NT - 1) * w_stride + lane * 8;
    // activation tile t of the pair (0 .. 2 XT - 1) is tile t of the 2 XT consecutive ones that start at tp * 2 XT
    const bf16_t* const gx0 = a.Xp + (u64)min(tp * 2 * XT + w, a.TBS - 1) * 512 + lane * 8;
    const bf16_t* const gx1 = a.Xp + (u64)min(tp * 2 * XT + w + 8, a.TBS - 1) * 512 + lane * 8;
    const bf16_t* const gx2 = a.Xp + (u64)min(tp * 2 * XT + w + 16, a.TBS - 1) * 512 + lane * 8;
    floatx4_t acc[4][TJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    uint4 ga0, ga1, ga2, ga3, gb0, gb1, gb2, gb3;
    ga2 = gb2 = ga3 = gb3 = make_uint4(0, 0, 0, 0);
#define TL_GLOAD(g, kt) { const u32 kc_ = min((u32)(kt), KT - 1);                                                         \
      g##0 = *(const uint4*)(gw + (u64)kc_ * 512); g##1 = *(const uint4*)(gx0 + (u64)kc_ * xk_stride);                     \
      if (x2) g##2 = *(const uint4*)(gx1 + (u64)kc_ * xk_stride); if (x3) g##3 = *(const uint4*)(gx2 + (u64)kc_ * xk_stride); }
#define TL_STORE(g, buf) { *(uint4*)(Lww + (buf) * LB) = g##0; *(uint4*)(Lwx + (buf) * LB) = g##1;                          \
      if (x2) *(uint4*)(Lwx + (buf) * LB + 8192) = g##2; if (x3) *(uint4*)(Lwx + (buf) * LB + 16384) = g##3; }
#define TL_RW(buf, i) as_f16x8(*(const uint4*)(Lrw + (buf) * LB + (i) * 1024))
#define TL_RX(buf, j) as_f16x8(*(const uint4*)(Lrx + (buf) * LB + ((j) < TJ ? (j) : 0) * 1024))
#define TL_MM(A, W, X) A = __builtin_amdgcn_mfma_f32_16x16x32_f16(W, X, A, 0, 0, 0);
#define TL_ROW(i, o) TL_MM(acc[i][0], o.w##i, o.x0) TL_MM(acc[i][1], o.w##i, o.x1)                                         \
      if (TJ > 2) { TL_MM(acc[i][TJ > 2 ? 2 : 0], o.w##i, o.x2) } if (TJ > 3) { TL_MM(acc[i][TJ > 3 ? 3 : 0], o.w##i, o.x3) }            \
      if (TJ > 4) { TL_MM(acc[i][TJ > 4 ? 4 : 0], o.w##i, o.x4) TL_MM(acc[i][TJ > 4 ? 5 : 0], o.w##i, o.x5) }
#define TL_SB __builtin_amdgcn_sched_barrier(0);
#define TL_STEP(o, n, g, k, rb, wb)                                                                                       \
    n.x0 = TL_RX(rb, 0); n.w0 = TL_RW(rb, 0); n.x1 = TL_RX(rb, 1); n.w1 = TL_RW(rb, 1); TL_STORE(g, wb)                   \
    TL_SB TL_ROW(0, o) TL_ROW(1, o) TL_SB                                                                                 \
    if (TJ > 2) n.x2 = TL_RX(rb, 2);                                                                                      \
    n.w2 = TL_RW(rb, 2); if (TJ > 3) n.x3 = TL_RX(rb, 3);                                                                  \
    if (TJ > 4) { n.x4 = TL_RX(rb, 4); n.x5 = TL_RX(rb, 5); }                                                             \
    n.w3 = TL_RW(rb, 3); TL_GLOAD(g, (k) + 4)                                                                             \
    TL_SB TL_ROW(2, o) TL_ROW(3, o) TL_SB                                                                                 \
    __syncthreads();
    struct Ops { f16x8_t w0, w1, w2, w3, x0, x1, x2, x3, x4, x5; };
    Ops oa, ob;
    TL_GLOAD(ga, 0) TL_GLOAD(gb, 1)             // in flight while the norm scales are computed
    // both tiles' tokens (at most 256 per call); its barriers: the LDS tiles are free
    if (2 * BT <= 256) compute_rstd(a, min(tp * 2 * BT, a.T - 1), 2 * BT, sh, 0);
    else { compute_rstd(a, min(tp * 2 * BT, a.T - 1), BT, sh, 0); compute_rstd(a, min(tp * 2 * BT + BT, a.T - 1), BT, sh, BT); }
    TL_STORE(ga, 0) TL_STORE(gb, 1) TL_GLOAD(ga, 2) TL_GLOAD(gb, 3)
    __syncthreads();
    oa.w0 = TL_RW(0, 0); oa.w1 = TL_RW(0, 1); oa.w2 = TL_RW(0, 2); oa.w3 = TL_RW(0, 3);
    oa.x0 = TL_RX(0, 0); oa.x1 = TL_RX(0, 1); oa.x2 = TL_RX(0, 2); oa.x3 = TL_RX(0, 3); oa.x4 = TL_RX(0, 4); oa.x5 = TL_RX(0, 5);
    __syncthreads();   // step 0 overwrites buffer 0, which every wave has just read (later steps read a buffer one step ahead)
    for (u32 k = 0; k < KT; k += 2) {
      TL_STEP(oa, ob, ga, k, 1, 0)
      if (k + 1 < KT) { TL_STEP(ob, oa, gb, k + 1, 0, 1) }
    }
#undef TL_GLOAD
#undef TL_STORE
#undef TL_RW
#undef TL_RX
#undef TL_MM
#undef TL_ROW
#undef TL_SB
#undef TL_STEP
    if (valid) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (nt0 + i < NT) {
          epilogue_row<EPI, TJ>(a, acc[i], nt0 + i, tb * BT + wt * TJ * 16, &sh.rstd[half * BT + wt * TJ * 16]);
        }
    }
  }
}

// Four waves on 128 rows x 256 tokens (64 x 128 per wave: 128 accumulator registers). The registers leave room for one
// set of operands only, so a wave reads its 4 + 8 operand tiles of a k-step from LDS at the start of the step and
// begins its 32 MFMAs as they arrive; the global data of the following steps are staged as in gemm_tile_lds (two
// register sets, two steps ahead, one barrier per step, two LDS buffers of 24 KB). Per MFMA it moves a quarter less
// through LDS and out of L2 than the 128-token tile.
template <int EPI>
__device__ __forceinline__ void gemm_tile_lds_wide(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg) {
  constexpr u32 TJ = 8, BT = 32 * TJ, XT = 2 * TJ, LB = (8 + XT) * 1024;
  const u32 lane = threadIdx.x & 63, w = (threadIdx.x >> 6) & 3, wn = w & 1, wt = w >> 1;
  const u32 NT = (a.N + 15) / 16, KT = a.K / 32;
  const u32 nblocks = (NT + 7) / 8, tblocks = (a.T + BT - 1) / BT, total = nblocks * tblocks;
  const u64 xk_stride = (u64)a.TBS * 512, w_stride = (u64)KT * 512;
  // LDS buffer of one k-step: weight tiles 0..7, then activation tiles 0..15. This wave stores weight tiles 2 w, 2 w + 1
  // and activation tiles w, w + 4, w + 8, w + 12
  unsigned char* const L0 = &sh.tile[0][0];
  unsigned char* const Lww = L0 + (w * 2) * 1024 + lane * 16;
  unsigned char* const Lwx = L0 + 8192 + w * 1024 + lane * 16;
  const unsigned char* const Lrw = L0 + (wn * 4) * 1024 + lane * 16;
  const unsigned char* const Lrx = L0 + 8192 + (wt * TJ) * 1024 + lane * 16;
  for (u32 base = 0; base < total; base += nwg) {
    const u32 it = xcd_item(base, total, wg, nwg);
    if (it == ~0u) continue;
    u32 tb = 0, nb = 0;
    tile_coords(it, nblocks, tblocks, nb, tb);
    const u32 nt0 = nb * 8 + wn * 4;
    const bf16_t* const gw0 = a.Wp + (u64)min(nb * 8 + w * 2, NT - 1) * w_stride + lane * 8;
    const bf16_t* const gw1 = a.Wp + (u64)min(nb * 8 + w * 2 + 1, NT - 1) * w_stride + lane * 8;
    // this lane's 16 bytes of the four activation tiles its wave fetches (see gemm_tile_lds: token indirection, clamping)
    const bf16_t *gx0, *gx1, *gx2, *gx3;
    if (a.tok_index) {
      const u32 ta = tb * BT + w * 16 + (lane & 15);
      const u32 s0 = a.tok_index[min(ta, a.T - 1)], s1 = a.tok_index[min(ta + 64, a.T - 1)];
      const u32 s2 = a.tok_index[min(ta + 128, a.T - 1)], s3 = a.tok_index[min(ta + 192, a.T - 1)];
      gx0 = a.Xp + ((u64)(s0 >> 4) * 64 + (s0 & 15) + 16 * (lane >> 4)) * 8;
      gx1 = a.Xp + ((u64)(s1 >> 4) * 64 + (s1 & 15) + 16 * (lane >> 4)) * 8;
      gx2 = a.Xp + ((u64)(s2 >> 4) * 64 + (s2 & 15) + 16 * (lane >> 4)) * 8;
      gx3 = a.Xp + ((u64)(s3 >> 4) * 64 + (s3 & 15) + 16 * (lane >> 4)) * 8;
    } else {
      gx0 = a.Xp + (u64)min(tb * XT + w, a.TBS - 1) * 512 + lane * 8;
      gx1 = a.Xp + (u64)min(tb * XT + w + 4, a.TBS - 1) * 512 + lane * 8;
      gx2 = a.Xp + (u64)min(tb * XT + w + 8, a.TBS - 1) * 512 + lane * 8;
      gx3 = a.Xp + (u64)min(tb * XT + w + 12, a.TBS - 1) * 512 + lane * 8;
    }
    floatx4_t acc[4][TJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    uint4 ga0, ga1, ga2, ga3, ga4, ga5, gb0, gb1, gb2, gb3, gb4, gb5;   // separate variables, see gemm_tile_lds
#define TW_GLOAD(g, kt) { const u32 kc_ = min((u32)(kt), KT - 1);                                                          \
      g##0 = *(const uint4*)(gw0 + (u64)kc_ * 512); g##1 = *(const uint4*)(gw1 + (u64)kc_ * 512);                          \
      g##2 = *(const uint4*)(gx0 + (u64)kc_ * xk_stride); g##3 = *(const uint4*)(gx1 + (u64)kc_ * xk_stride);              \
      g##4 = *(const uint4*)(gx2 + (u64)kc_ * xk_stride); g##5 = *(const uint4*)(gx3 + (u64)kc_ * xk_stride); }
#define TW_STORE(g, buf) { *(uint4*)(Lww + (buf) * LB) = g##0; *(uint4*)(Lww + (buf) * LB + 1024) = g##1;                   \
      *(uint4*)(Lwx + (buf) * LB) = g##2; *(uint4*)(Lwx + (buf) * LB + 4096) = g##3;                                       \
      *(uint4*)(Lwx + (buf) * LB + 8192) = g##4; *(uint4*)(Lwx + (buf) * LB + 12288) = g##5; }
#define TW_RW(buf, i) as_f16x8(*(const uint4*)(Lrw + (buf) * LB + (i) * 1024))
#define TW_RX(buf, j) as_f16x8(*(const uint4*)(Lrx + (buf) * LB + (j) * 1024))
#define TW_MM(A, W, X) A = __builtin_amdgcn_mfma_f32_16x16x32_f16(W, X, A, 0, 0, 0);
#define TW_COL(j, xx) TW_MM(acc[0][j], w0_, xx) TW_MM(acc[1][j], w1_, xx) TW_MM(acc[2][j], w2_, xx) TW_MM(acc[3][j], w3_, xx)
    // step k: operands from buffer rb; the staged data of step k+1 (in g) go to buffer wb; g then requests step k+3
#define TW_STEP(g, k, rb, wb) {                                                                                         \
      const f16x8_t w0_ = TW_RW(rb, 0), w1_ = TW_RW(rb, 1), w2_ = TW_RW(rb, 2), w3_ = TW_RW(rb, 3);                       \
      const f16x8_t x0_ = TW_RX(rb, 0), x1_ = TW_RX(rb, 1), x2_ = TW_RX(rb, 2), x3_ = TW_RX(rb, 3);                       \
      const f16x8_t x4_ = TW_RX(rb, 4), x5_ = TW_RX(rb, 5), x6_ = TW_RX(rb, 6), x7_ = TW_RX(rb, 7);                       \
      TW_STORE(g, wb) TW_GLOAD(g, (k) + 3)                                                                               \
      TW_COL(0, x0_) TW_COL(1, x1_) TW_COL(2, x2_) TW_COL(3, x3_) TW_COL(4, x4_) TW_COL(5, x5_) TW_COL(6, x6_) TW_COL(7, x7_) \
      __syncthreads(); }
    TW_GLOAD(ga, 0)                              // in flight while the norm scales are computed
    compute_rstd(a, tb * BT, BT, sh, 0);         // its barriers: the LDS tiles are free
    TW_STORE(ga, 0) TW_GLOAD(gb, 1) TW_GLOAD(ga, 2)
    __syncthreads();
    for (u32 k = 0; k < KT; k += 2) {
      TW_STEP(gb, k, 0, 1)
      if (k + 1 < KT) { TW_STEP(ga, k + 1, 1, 0) }
    }
#undef TW_GLOAD
#undef TW_STORE
#undef TW_RW
#undef TW_RX
#undef TW_MM
#undef TW_COL
#undef TW_STEP
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (nt0 + i < NT) {
        epilogue_row<EPI, TJ>(a, acc[i], nt0 + i, tb * BT + wt * TJ * 16, &sh.rstd[wt * TJ * 16]);
      }
  }
}

// Token width of the workgroup tiles (256, 192, 128, 96 or 64) for this GEMM: the one whose rounds of workgroups take
// the least time. A round of a narrower tile is shorter in proportion to its width, at a measured cost for the extra
// operand traffic per flop (relative to 128 tokens: 256 tokens 12 % less, 192 tokens 6 % less; 96 / 64 tokens 12 % /
// 24 % more in the four-wave kernels, 24 % / 50 % more in the eight-wave ones). Eight waves take 192 tokens only as a
// shared-weight pair (its two LDS buffers fill the 64 KB; two separate tiles of that width would not fit) and never
// the 256-token tile (their pair of 128-token tiles already shares the weights of 256 tokens).
template <int EPI>
__device__ __forceinline__ void gemm_tile_pick(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg) {
  const u32 nblocks = ((a.N + 15) / 16 + 7) / 8, halves = blockDim.x >> 8, ncu = nwg / 2;
  const u32 forced = (a.tune_nw >> 12) & 7u;       // bits 12-14 of the tuning word: 2, 3, 4, 6 force the width, 7 the 256-token tile (tests)
  const bool pair_ok = halves == 2 && !a.tok_index && !(a.tune_nw & 0x100000u);   // bit 20: never the shared pair (tests)
  const bool wide_ok = halves == 1 || pair_ok;
  u32 best = 4, best_cost = ~0u;
  for (u32 tj = 8; tj >= 2; --tj) {
    if (tj == 5 || tj == 7 || (tj == 8 && (halves != 1 || (a.tune_nw & 0x200000u))) ||
        (tj == 6 && (!wide_ok || (a.tune_nw & 0x200000u)))) continue;   // bit 21: never wider than 128 tokens (tests)
    const u32 total = nblocks * ((a.T + 32 * tj - 1) / (32 * tj));
    u32 rounds2;                                     // eight waves: in half rounds of a workgroup
    if (halves == 2) {
      const u32 r_pair = 2 * (((total + 1) / 2 + ncu - 1) / ncu), r_split = (a.K & 32u) ? ~0u : (total + ncu - 1) / ncu;
      rounds2 = tj == 6 ? r_pair : min(r_pair, r_split);
    } else {
      // four waves: two workgroups share a compute unit (workgroups w and w + ncu, by the order of dispatch). With b
      // tiles on the less loaded of the two and a on the other, the unit works 2 b tile times at the shared rate and
      // a - b (0 or 1) alone, where a tile takes 1.25 to 1.5 of its shared time (measured: a single round of 256-token
      // tiles on half of the slots against a full round of 128-token tiles; small matrices sit at the upper end, and
      // 1.5 is what the count uses). In quarters of a tile time:
      const u32 n_lo = total / nwg, extra = total % nwg, hi = n_lo + (extra > 0 ? 1u : 0u), lo = n_lo + (extra > ncu ? 1u : 0u);
      rounds2 = 8 * lo + 6 * (hi - lo);
    }
    const u32 pen = tj == 8 ? 88u : tj == 6 ? 94u : tj == 4 ? 100u : (halves == 2 ? (tj == 3 ? 124u : 150u) : (tj == 3 ? 112u : 124u));
    const u32 cost = rounds2 * tj * pen;
    if (cost < best_cost) { best_cost = cost; best = tj; }
  }
  if (forced >= 2 && forced <= 4) best = forced;
  if (forced == 6 && wide_ok) best = 6;
  if (forced == 7 && halves == 1) best = 8;
  // eight waves: a pair of tiles with shared weight tiles unless splitting K between the halves takes fewer rounds
  // (the same rule as inside gemm_tile_lds)
  bool pair = false;
  if (pair_ok) {
    const u32 tblocks = (a.T + 32 * best - 1) / (32 * best), total = nblocks * tblocks;
    const u32 rounds_split = (total + ncu - 1) / ncu, rounds_pair = ((total + 1) / 2 + ncu - 1) / ncu;
    const bool splitk = (a.K & 32u) == 0 && rounds_split < 2 * rounds_pair && !(a.tune_nw & 0x400u);
    pair = best == 6 || !splitk;
  }
  if (pair) {
    if (best == 6) gemm_tile_lds_pair<EPI, 6>(a, sh, wg, nwg);
    else if (best == 4) gemm_tile_lds_pair<EPI, 4>(a, sh, wg, nwg);
    else if (best == 3) gemm_tile_lds_pair<EPI, 3>(a, sh, wg, nwg);
    else gemm_tile_lds_pair<EPI, 2>(a, sh, wg, nwg);
  } else if (best == 8) gemm_tile_lds_wide<EPI>(a, sh, wg, nwg);
  else if (best == 6) gemm_tile_lds<EPI, 6>(a, sh, wg, nwg);
  else if (best == 4) gemm_tile_lds<EPI, 4>(a, sh, wg, nwg);
  else if (best == 3) gemm_tile_lds<EPI, 3>(a, sh, wg, nwg);
  else gemm_tile_lds<EPI, 2>(a, sh, wg, nwg);
}

// WIDE: the kernel runs eight waves per workgroup (the projections with few output rows); it never takes four weight
// tiles per workgroup, and keeping that variant out of it keeps it within the 256 registers per lane it may use.
template <int EPI, int TW, bool WIDE>
__device__ __forceinline__ void gemm_stream_nw(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg) {
  // enough tile groups to occupy the chip (one workgroup per group, >= 1.5 per CU) decides the group size
  const u32 NT = (a.N + 15) / 16;
  const u32 forced = a.tune_nw & 0x07u;
  if (forced == 1) gemm_stream<EPI, 1, TW>(a, sh, wg, nwg);
  else if (forced == 2) gemm_stream<EPI, 2, TW>(a, sh, wg, nwg);
  else if (forced == 4 && !WIDE) gemm_stream<EPI, 4, TW>(a, sh, wg, nwg);
  // measured on MI355X (llama3_8b shapes): the eight-wave kernels gain from two tiles only with >= 320 row tiles
  // (QKV), the four-wave kernels with one token block only for very tall matrices (LM head), and with several token
  // blocks the activation re-reads make two and four tiles pay off from 768 and 1536 row tiles
  else if (WIDE) {
    if (NT >= 320) gemm_stream<EPI, 2, TW>(a, sh, wg, nwg); else gemm_stream<EPI, 1, TW>(a, sh, wg, nwg);
  } else if (TW == 1) {
    if (NT >= 4096) gemm_stream<EPI, 2, TW>(a, sh, wg, nwg); else gemm_stream<EPI, 1, TW>(a, sh, wg, nwg);
  } else if (NT >= 1536) gemm_stream<EPI, 4, TW>(a, sh, wg, nwg);
  else if (NT >= 768) gemm_stream<EPI, 2, TW>(a, sh, wg, nwg);
  else gemm_stream<EPI, 1, TW>(a, sh, wg, nwg);
}

template <int EPI, bool WIDE>
__device__ __forceinline__ void gemm_mfma(const MfmaGemmArgs& a, MfmaShared& sh, u32 wg, u32 nwg) {
  if (a.T == 0) return;
  if (WIDE) {
    const u32 S = splitk_slices(a, nwg, blockDim.x);
    if (S) { gemm_tile_lds<EPI, 4, true>(a, sh, wg, nwg, S); return; }
  }
  if (a.T <= 16) gemm_stream_nw<EPI, 1, WIDE>(a, sh, wg, nwg);
  else if (a.T <= 32) gemm_stream_nw<EPI, 2, WIDE>(a, sh, wg, nwg);
  else if (a.T <= 48) gemm_stream_nw<EPI, 3, WIDE>(a, sh, wg, nwg);
  else if (a.T <= 64) gemm_stream_nw<EPI, 4, WIDE>(a, sh, wg, nwg);
  else if (WIDE && !a.tok_index && a.T <= 256 && !(a.tune_nw & 0x800u) &&
           ((a.N + 127) / 128) * ((a.T + 127) / 128) * 8 <= nwg)       // few 128 x 128 tiles: 64 x 64 items fill the chip
    gemm_stream<EPI, 4, 4, 1, true>(a, sh, wg, nwg);                      // (bit 11 of the tuning word: never)
  else if (a.tune_nw & 0x200u) gemm_tile<EPI>(a, sh, wg, nwg);   // bit 9: direct-load tiles (tests and tuning)
  else gemm_tile_pick<EPI>(a, sh, wg, nwg);
}

// ---- packing -----------------------------------------------------------------------------------------------------
// Weights [N][K] row-major bf16 -> packed tiles of half precision, scaled by W_SCALE. pair_rows > 0: the source holds
// `pair_rows` gate rows followed by `pair_rows` up rows, and packed row 2j is gate_j, row 2j+1 is up_j. perm_hd > 0:
// rows are heads of perm_hd dimensions each, re-ordered so that the two dimensions a rotary embedding pairs up are
// adjacent rows.
__device__ __forceinline__ void pack_weights(const bf16_t* src, f16_t* dst, u32 N, u32 K, u32 pair_rows, u32 perm_hd, u64 gtid,
                                             u64 gthreads) {
  const u32 NT = (N + 15) / 16, KT = K / 32;
  const u64 chunks = (u64)NT * KT * 64;
  for (u64 i = gtid; i < chunks; i += gthreads) {
    const u32 lane = (u32)(i & 63);
    const u64 tile = i >> 6;
    const u32 kt = (u32)(tile % KT), nt = (u32)(tile / KT);
    const u32 n = nt * 16 + (lane & 15), k = kt * 32 + (lane >> 4) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) {
      u32 row = pair_rows ? ((n & 1) ? pair_rows + (n >> 1) : (n >> 1)) : n;
      if (perm_hd) {   // packed row 2p of a head is its dimension p, row 2p+1 its dimension p + hd/2
        const u32 pi = n % perm_hd;
        row = n - pi + ((pi & 1) ? perm_hd / 2 + (pi >> 1) : (pi >> 1));
      }
      const uint4 b = *(const uint4*)(src + (u64)row * K + k);
      const u32 w[4] = {b.x, b.y, b.z, b.w};
      u32 o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        o[j] = pack_f16x2(__uint_as_float(w[j] << 16) * W_SCALE, __uint_as_float(w[j] & 0xFFFF0000u) * W_SCALE);
      v = make_uint4(o[0], o[1], o[2], o[3]);
    }
    *(uint4*)(dst + i * 8) = v;
  }
}
