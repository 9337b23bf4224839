// Mixture-of-experts FFN of a bf16 model (the second workload of the paper's evaluation, section 6, is such a model):
// router GEMM -> per-token selection of the n_active largest router logits (ties to the lower expert id) and softmax over
// them -> one list of tokens per expert -> the normalised inputs of all (token, expert) pairs gathered into columns grouped
// by expert -> grouped gate/up and down GEMMs (an expert's columns as independent wave items or as one GEMM of the tile
// schedules) -> weighted sum of a token's expert outputs in selection order + residual + next norm's operand.
// The expert lists are filled with atomic counters: the order of the tokens inside a list depends on timing, but a
// token's result does not depend on its place in the list (every GEMM column is accumulated on its own, in an order fixed
// by the schedule), and the per-token sum over its experts runs in selection order, so results are reproducible.
#pragma once
#include "blink_device.h"
#include "mfma_gemm.h"
#include "sampler.h"

#define MOE_MAX_EXPERTS 256
#define MOE_MAX_ACTIVE 8

#define MOE_WAVE_MAX_TOKENS 64   // experts with at most this many tokens are run by independent waves (see moe_wave_item)

struct MoeShared {
  MfmaShared mfma;
  u32 cnt[MOE_MAX_EXPERTS];
  u32 off[MOE_MAX_EXPERTS + 1];   // first column of every expert's group: counts padded to whole 16-token blocks
  u32 small_e[MOE_MAX_EXPERTS];   // experts with 1..MOE_WAVE_MAX_TOKENS tokens, and the first wave item of each
  u32 small_base[MOE_MAX_EXPERTS + 1];
  u32 big_e[MOE_MAX_EXPERTS];     // experts with more tokens: one GEMM of the workgroup schedules each
  u32 big_start[MOE_MAX_EXPERTS]; // workgroup that takes the first tile of that GEMM: the tiles of all such GEMMs go round the grid
  u32 n_small, n_big;
  float wrstd[4][64];             // per wave: norm scales of the tokens of its current item
};

// counts -> LDS, offsets by a serial prefix sum (at most 256 terms); every workgroup of the grouped kernels does this.
// NT > 0 (row tiles of an expert's matrix): also the split of the experts into those run by independent waves, with their
// wave items (moe_wave_rows row tiles each), and the rest.
__device__ __forceinline__ u32 moe_wave_rows(u32 n_tokens) { return n_tokens <= 32 ? 4u : 2u; }

__device__ __forceinline__ void moe_offsets(const DevCtx& c, MoeShared& sh, u32 NT = 0, u32 nwg = 1) {
  for (u32 e = threadIdx.x; e < c.n_experts; e += blockDim.x) sh.cnt[e] = c.moe_count[e];
  __syncthreads();
  if (threadIdx.x == 0) {
    u32 o = 0, ns = 0, nb = 0, base = 0, tiles = 0;
    for (u32 e = 0; e < c.n_experts; ++e) {
      const u32 n = sh.cnt[e];
      sh.off[e] = o;
      o += (n + 15u) & ~15u;
      if (NT && n) {
        if (n <= MOE_WAVE_MAX_TOKENS) {
          const u32 nw = moe_wave_rows(n);
          sh.small_e[ns] = e; sh.small_base[ns] = base; base += (NT + nw - 1) / nw; ++ns;
        }
        else {
          // workgroup tiles of the expert's GEMM at the tile width moe_grouped forces: 128 rows x (all tokens up to 192, else 256)
          sh.big_e[nb] = e;
          sh.big_start[nb++] = tiles % nwg;
          tiles += ((NT + 7) / 8) * (n <= 192 ? 1u : (n + 255) / 256);
        }
      }
    }
    sh.off[c.n_experts] = o;
    sh.small_base[ns] = base;
    sh.n_small = ns; sh.n_big = nb;
  }
  __syncthreads();
}

// ---- selection: one wave per token --------------------------------------------------------------------------------
__device__ __forceinline__ void moe_route(const DevCtx& c, u32 layer, u32 wg, u32 nwg) {
  const u32 T = c.meta->n_tokens, E = c.n_experts, k = c.n_active;
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (u32 t = wg * nw + w; t < T; t += nwg * nw) {
    {   // the norm scale of the token, applied when the experts' operand is gathered
      const u32 np = c.d / 16;
      float v = 0.f;
      for (u32 q = lane; q < np; q += 64) v += c.ssq[(u64)t * np + q];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (lane == 0) c.moe_rstd[t] = 1.0f / sqrtf(v / (float)c.d + c.eps);
    }
    const float* r = c.moe_logits + (u64)t * E;
    unsigned long long key[MOE_MAX_EXPERTS / 64];
#pragma unroll
    for (u32 i = 0; i < MOE_MAX_EXPERTS / 64; ++i) {
      const u32 e = lane + 64 * i;
      key[i] = e < E ? (((unsigned long long)order_key(r[e]) << 32) | (u32)~e) : 0ull;   // larger logit first, then lower id
    }
    float sel_logit = 0.f, first_logit = 0.f, denom = 0.f;
    u32 sel_e = 0;
    for (u32 j = 0; j < k; ++j) {
      unsigned long long best = key[0];
#pragma unroll
      for (u32 i = 1; i < MOE_MAX_EXPERTS / 64; ++i) best = key[i] > best ? key[i] : best;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long x = __shfl_xor(best, o);
        best = x > best ? x : best;
      }
      const u32 e = ~(u32)best;
      const float l = key_to_float((u32)(best >> 32));
#pragma unroll
      for (u32 i = 0; i < MOE_MAX_EXPERTS / 64; ++i)
        if (lane + 64 * i == e) key[i] = 0ull;       // taken
      if (j == 0) first_logit = l;
      denom += __expf(l - first_logit);
      if (lane == j) { sel_e = e; sel_logit = l; }
    }
    if (lane < k) {
      const u32 q = t * k + lane;
      const u32 pos = atomicAdd(&c.moe_count[sel_e], 1u);
      c.moe_list[(u64)sel_e * c.maxT + pos] = t;
      c.moe_sel[(u64)layer * c.maxT * k + q] = sel_e;
      c.moe_pos[q] = pos;
      c.moe_w[q] = __expf(sel_logit - first_logit) / denom;
    }
  }
}

// ---- the experts' operand: the normalised FFN input of every (token, expert) pair, columns grouped by expert ----------
// A wave writes one packed 16-column x 32-k tile (1 KB, contiguous) at a time: lane (c, kg) reads eight consecutive
// fp32 values of the residual stream of column c's token, applies the norm's gain and scale and rounds once to half
// precision. Gathering the tokens here, once, lets the grouped GEMMs read whole operand tiles instead of sixteen-byte
// pieces of sixteen different tokens per load. Columns past an expert's count (its group is padded to 16) get zeros.
__device__ __forceinline__ void moe_permute(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  moe_offsets(c, sh);
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6, E = c.n_experts;
  const u32 nblk = sh.off[E] / 16, KT = c.d / 32, lc = lane & 15, kg = lane >> 4;
  const float* g = c.layers[layer].g2;
  const u32 KQ = (KT + 3) / 4;                   // a wave item: one column block x a quarter of the k-tiles
  for (u32 item = wg * nw + w; item < nblk * 4; item += nwg * nw) {
    const u32 cb = item >> 2, k_lo = (item & 3u) * KQ, k_hi = min(KT, k_lo + KQ);
    u32 lo = 0, hi = E;                        // the expert of column block cb: last e with off[e] / 16 <= cb
    while (hi - lo > 1) {
      const u32 mid = (lo + hi) >> 1;
      if (sh.off[mid] / 16 <= cb) lo = mid; else hi = mid;
    }
    const u32 e = lo, pos = (cb - sh.off[e] / 16) * 16 + lc;
    const bool live = pos < sh.cnt[e];
    const u32 tok = live ? c.moe_list[(u64)e * c.maxT + pos] : 0u;
    const float r = live ? c.moe_rstd[tok] : 0.f;
    const float* xr = c.x + (u64)tok * c.d + kg * 8;
    f16_t* dst = c.xq_moe + ((u64)cb * 64 + lane) * 8;
    const u64 kstride = (u64)c.moe_TBS * 512;
    for (u32 k0 = k_lo; k0 < k_hi; k0 += 4) {
      float4 a[4], b[4], ga[4], gb[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {              // four k-tiles of loads in flight (the last ones of a ragged quarter repeat its last tile)
        const u32 kt = min(k0 + u, k_hi - 1);
        a[u] = *(const float4*)(xr + kt * 32); b[u] = *(const float4*)(xr + kt * 32 + 4);
        ga[u] = *(const float4*)(g + kt * 32 + kg * 8); gb[u] = *(const float4*)(g + kt * 32 + kg * 8 + 4);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (k0 + u < k_hi)
          *(uint4*)(dst + (k0 + u) * kstride) =
              make_uint4(pack_f16x2(a[u].x * ga[u].x * r, a[u].y * ga[u].y * r), pack_f16x2(a[u].z * ga[u].z * r, a[u].w * ga[u].w * r),
                         pack_f16x2(b[u].x * gb[u].x * r, b[u].y * gb[u].y * r), pack_f16x2(b[u].z * gb[u].z * r, b[u].w * gb[u].w * r));
    }
  }
}

// ---- grouped GEMMs -----------------------------------------------------------------------------------------------------
// An expert with at most MOE_WAVE_MAX_TOKENS tokens (every expert of a decode iteration, as a rule) is bound by the
// bytes of its matrices. Its GEMM is cut into wave items of four (two, beyond 32 tokens) 16-row weight tiles x all its
// tokens x the whole of K;
// the waves of the grid take the items of all such experts round-robin and run them on their own: no barrier, no
// shared memory traffic, the loads of two batches of k-tiles in flight per wave. A wave streams its rows of tiles
// (contiguous in the packed layout) with loads that bypass temporal caching and reads the tokens' operand tiles, which
// the neighbouring waves (same expert, next rows) read too, through the caches.
template <bool GATEUP, int TW>
__device__ __forceinline__ void moe_wave_item(const DevCtx& c, const LayerWP* P, MoeShared& sh, u32 e, u32 g) {
  constexpr int NW = TW <= 2 ? 4 : 2, U = 2;
  constexpr int EPI = GATEUP ? EPI_SILU_GATE : EPI_SCALED_STORE;
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const u32 cnt = sh.cnt[e], col0 = sh.off[e];
  const u32 K = GATEUP ? c.d : c.F, N = GATEUP ? 2 * c.F : c.d, KT = K / 32, NT = N / 16;
  const f16_t* Wp = GATEUP ? P->wgu + (u64)e * (2 * c.F) * c.d : P->wd + (u64)e * c.d * c.F;
  const f16_t* wp[NW];
#pragma unroll
  for (int i = 0; i < NW; ++i) wp[i] = Wp + (u64)min(g * NW + i, NT - 1) * KT * 512 + lane * 8;
  const f16_t* xp[TW];
  const u64 xk_stride = (u64)c.moe_TBS * 512;
#pragma unroll
  for (int tw = 0; tw < TW; ++tw) xp[tw] = (GATEUP ? c.xq_moe : c.hq_moe) + (u64)(col0 / 16 + tw) * 512 + lane * 8;
  struct Buf { f16x8_t w[U][NW], x[U][TW]; };
  const f16x8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
  auto issue = [&](Buf& b, u32 kt0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const u32 kt = kt0 + u;
      const bool ok = kt < KT;
#pragma unroll
      for (int i = 0; i < NW; ++i) b.w[u][i] = ok ? ld_op_stream(wp[i] + (u64)kt * 512) : zero;
#pragma unroll
      for (int tw = 0; tw < TW; ++tw) b.x[u][tw] = ok ? ld_op(xp[tw] + (u64)kt * xk_stride) : zero;
    }
  };
  floatx4_t acc[NW][TW];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int tw = 0; tw < TW; ++tw) acc[i][tw] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  auto mm = [&](const Buf& b) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < NW; ++i)
#pragma unroll
        for (int tw = 0; tw < TW; ++tw) acc[i][tw] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b.w[u][i], b.x[u][tw], acc[i][tw], 0, 0, 0);
  };
  Buf bufA, bufB;
  issue(bufA, 0);
  for (u32 kt0 = 0; kt0 < KT; kt0 += 2 * U) {
    issue(bufB, kt0 + U);
    mm(bufA);
    issue(bufA, kt0 + 2 * U);
    mm(bufB);
  }
  MfmaGemmArgs a{};
  a.T = cnt; a.N = N; a.col0 = col0; a.TBS = c.TBS;
  if (GATEUP) { a.Hp = c.hq_moe; a.TBS_out = c.moe_TBS; }
  else { a.out = c.y_moe; a.ldo = c.d; }
#pragma unroll
  for (int i = 0; i < NW; ++i)
    if (g * NW + i < NT) {
#pragma unroll
      for (int tw = 0; tw < TW; ++tw) epilogue_tile<EPI>(a, acc[i][tw], g * NW + i, tw * 16, &sh.wrstd[w][tw * 16]);
    }
}

// Experts with more tokens run as one GEMM of the workgroup schedules each (shared operand tiles in LDS); every GEMM
// starts at the workgroup behind the previous one's last tile, so the tiles of all of them go round the grid evenly.
template <bool GATEUP>
__device__ __forceinline__ void moe_grouped(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  const LayerWP* P = c.players + layer;
  const u32 Fe = c.F, N = GATEUP ? 2 * Fe : c.d;
  moe_offsets(c, sh, N / 16, nwg);
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  sh.wrstd[w][lane] = W_SCALE_INV;                   // the operands are normalised already; each wave reads only its own row
  const u32 total = sh.small_base[sh.n_small];
  for (u32 i = wg * nw + w; i < total; i += nwg * nw) {
    u32 lo = 0, hi = sh.n_small;                     // the expert of item i: last s with small_base[s] <= i
    while (hi - lo > 1) {
      const u32 mid = (lo + hi) >> 1;
      if (sh.small_base[mid] <= i) lo = mid; else hi = mid;
    }
    const u32 e = sh.small_e[lo], g = i - sh.small_base[lo];
    switch ((sh.cnt[e] + 15) / 16) {
      case 1: moe_wave_item<GATEUP, 1>(c, P, sh, e, g); break;
      case 2: moe_wave_item<GATEUP, 2>(c, P, sh, e, g); break;
      case 3: moe_wave_item<GATEUP, 3>(c, P, sh, e, g); break;
      default: moe_wave_item<GATEUP, 4>(c, P, sh, e, g); break;
    }
  }
  for (u32 b = 0; b < sh.n_big; ++b) {
    const u32 e = sh.big_e[b];
    MfmaGemmArgs a{};
    a.T = sh.cnt[e]; a.eps = c.eps; a.tune_nw = c.tune_nw; a.col0 = sh.off[e];
    // the other experts' GEMMs fill the chip: take the widest tile the expert's tokens fill instead of a narrower one
    // that would spread this one GEMM over more workgroups (bits 12-14 of the tuning word, unless the caller forces them)
    if (((a.tune_nw >> 12) & 7u) == 0)
      a.tune_nw |= (a.T <= 64 ? 2u : a.T <= 96 ? 3u : a.T <= 128 ? 4u : a.T <= 192 ? 6u : 7u) << 12;
    if (GATEUP) {
      a.TBS = c.moe_TBS; a.Wp = P->wgu + (u64)e * (2 * Fe) * c.d; a.Xp = c.xq_moe + (u64)(sh.off[e] / 16) * 512; a.N = 2 * Fe; a.K = c.d;
      a.Hp = c.hq_moe;
      gemm_mfma<EPI_SILU_GATE, false>(a, sh.mfma, (wg + nwg - sh.big_start[b]) % nwg, nwg);
    } else {
      a.TBS = c.moe_TBS; a.Wp = P->wd + (u64)e * c.d * Fe; a.Xp = c.hq_moe + (u64)(sh.off[e] / 16) * 512; a.N = c.d; a.K = Fe;
      a.out = c.y_moe; a.ldo = c.d;
      gemm_mfma<EPI_SCALED_STORE, false>(a, sh.mfma, (wg + nwg - sh.big_start[b]) % nwg, nwg);
    }
  }
}

__device__ __forceinline__ void moe_gateup(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  moe_grouped<true>(c, layer, sh, wg, nwg);
}
__device__ __forceinline__ void moe_down(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  moe_grouped<false>(c, layer, sh, wg, nwg);
}

// ---- x[t] += sum_j w_j * y[column of (t, j)], in selection order; packed operand and norm partials of the next GEMM ----
__device__ __forceinline__ void moe_combine(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  moe_offsets(c, sh);
  const u32 T = c.meta->n_tokens, d = c.d, per_row = d / 16, k = c.n_active;
  const float* g = layer + 1 < c.n_layers ? c.layers[layer + 1].g1 : c.gf;
  for (u64 i = (u64)wg * blockDim.x + threadIdx.x; i < (u64)T * per_row; i += (u64)nwg * blockDim.x) {
    const u32 t = (u32)(i / per_row), nt = (u32)(i % per_row), k0 = nt * 16;
    float* xp = c.x + (u64)t * d + k0;
    float v[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 o = *(const float4*)(xp + 4 * q);
      v[4 * q] = o.x; v[4 * q + 1] = o.y; v[4 * q + 2] = o.z; v[4 * q + 3] = o.w;
    }
    for (u32 j = 0; j < k; ++j) {
      const u32 q = t * k + j;
      const u32 col = sh.off[c.moe_sel[(u64)layer * c.maxT * k + q]] + c.moe_pos[q];
      const float wj = c.moe_w[q];
      const float* y = c.y_moe + (u64)col * d + k0;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float4 o = *(const float4*)(y + 4 * u);
        v[4 * u] += wj * o.x; v[4 * u + 1] += wj * o.y; v[4 * u + 2] += wj * o.z; v[4 * u + 3] += wj * o.w;
      }
    }
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) *(float4*)(xp + 4 * q) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      u32 wv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a = v[8 * h + 2 * j], b = v[8 * h + 2 * j + 1];
        ss += a * a + b * b;
        wv[j] = pack_f16x2(a * g[k0 + 8 * h + 2 * j], b * g[k0 + 8 * h + 2 * j + 1]);
      }
      *(uint4*)(c.xq + packed_off(t, k0 + 8 * h, c.TBS)) = make_uint4(wv[0], wv[1], wv[2], wv[3]);
    }
    c.ssq[(u64)t * per_row + nt] = ss;
  }
}
