// Mixture-of-experts FFN of a bf16 model (the second workload of the paper's evaluation, section 6, is such a model):
// router GEMM -> per-token selection of the n_active largest router logits (ties to the lower expert id) and softmax over
// them -> one list of tokens per expert -> grouped gate/up and down GEMMs, every expert's tokens as one GEMM of the
// existing schedules -> weighted sum of a token's expert outputs in selection order + residual + next norm's operand.
// The expert lists are filled with atomic counters: the order of the tokens inside a list depends on timing, but a
// token's result does not depend on its place in the list (every GEMM column is accumulated on its own, in an order fixed
// by the schedule), and the per-token sum over its experts runs in selection order, so results are reproducible.
#pragma once
#include "blink_device.h"
#include "mfma_gemm.h"
#include "sampler.h"

#define MOE_MAX_EXPERTS 256
#define MOE_MAX_ACTIVE 8

struct MoeShared {
  MfmaShared mfma;
  u32 cnt[MOE_MAX_EXPERTS];
  u32 off[MOE_MAX_EXPERTS + 1];   // first column of every expert's group: counts padded to whole 16-token blocks
};

// counts -> LDS, offsets by a serial prefix sum (at most 256 terms); every workgroup of the grouped kernels does this
__device__ __forceinline__ void moe_offsets(const DevCtx& c, u32* cnt, u32* off) {
  for (u32 e = threadIdx.x; e < c.n_experts; e += blockDim.x) cnt[e] = c.moe_count[e];
  __syncthreads();
  if (threadIdx.x == 0) {
    u32 o = 0;
    for (u32 e = 0; e < c.n_experts; ++e) { off[e] = o; o += (cnt[e] + 15u) & ~15u; }
    off[c.n_experts] = o;
  }
  __syncthreads();
}

// ---- selection: one wave per token --------------------------------------------------------------------------------
__device__ __forceinline__ void moe_route(const DevCtx& c, u32 layer, u32 wg, u32 nwg) {
  const u32 T = c.meta->n_tokens, E = c.n_experts, k = c.n_active;
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (u32 t = wg * nw + w; t < T; t += nwg * nw) {
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

// ---- grouped GEMMs: every expert's token list is one GEMM of the existing schedules; the workgroups start each expert's
// items at a different place so that the experts' items interleave over the grid ---------------------------------------
__device__ __forceinline__ void moe_gateup(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  moe_offsets(c, sh.cnt, sh.off);
  const LayerWP* P = c.players + layer;
  const u32 Fe = c.F;
  for (u32 e = 0; e < c.n_experts; ++e) {
    if (sh.cnt[e] == 0) continue;
    MfmaGemmArgs a{};
    a.T = sh.cnt[e]; a.TBS = c.TBS; a.eps = c.eps; a.tune_nw = c.tune_nw;
    a.Wp = P->wgu + (u64)e * (2 * Fe) * c.d; a.Xp = c.xq; a.N = 2 * Fe; a.K = c.d; a.ssq_in = c.ssq;
    a.tok_index = c.moe_list + (u64)e * c.maxT;
    a.Hp = c.hq_moe; a.TBS_out = c.moe_TBS; a.col0 = sh.off[e];
    gemm_mfma<EPI_SILU_GATE, false>(a, sh.mfma, (wg + nwg - (e * 97u) % nwg) % nwg, nwg);
  }
}

__device__ __forceinline__ void moe_down(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  moe_offsets(c, sh.cnt, sh.off);
  const LayerWP* P = c.players + layer;
  const u32 Fe = c.F;
  for (u32 e = 0; e < c.n_experts; ++e) {
    if (sh.cnt[e] == 0) continue;
    MfmaGemmArgs a{};
    a.T = sh.cnt[e]; a.TBS = c.moe_TBS; a.eps = c.eps; a.tune_nw = c.tune_nw;
    a.Wp = P->wd + (u64)e * c.d * Fe; a.Xp = c.hq_moe + (u64)(sh.off[e] / 16) * 512; a.N = c.d; a.K = Fe;
    a.out = c.y_moe; a.ldo = c.d; a.col0 = sh.off[e];
    gemm_mfma<EPI_SCALED_STORE, false>(a, sh.mfma, (wg + nwg - (e * 61u) % nwg) % nwg, nwg);
  }
}

// ---- x[t] += sum_j w_j * y[column of (t, j)], in selection order; packed operand and norm partials of the next GEMM ----
__device__ __forceinline__ void moe_combine(const DevCtx& c, u32 layer, MoeShared& sh, u32 wg, u32 nwg) {
  moe_offsets(c, sh.cnt, sh.off);
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
