// The ordered list of phases of one loop iteration and their dispatch. A phase is a grid-wide step that
// must be complete before the next begins (a kernel boundary in host-enqueued mode, a grid barrier in
// the resident loop). Shapes are read from the device metadata written by the scheduler step.
#pragma once
#include "blink_device.h"
#include "sched.h"
#include "forward.h"
#include "mfma_gemm.h"
#include "attention_mfma.h"
#include "sampler.h"
#include "moe.h"

enum {
  PH_EMBED = 0,
  PH_NORM1, PH_QKV, PH_ROPE, PH_ATTN, PH_OPROJ, PH_NORM2, PH_GATEUP, PH_DOWN,   // per layer
  PH_FINAL_NORM, PH_LM_HEAD, PH_SAMPLE,
  PH_ATTN_COMBINE,  // bf16 path only, directly after PH_ATTN of the same layer
  PH_QKV_RED, PH_OPROJ_RED, PH_DOWN_RED,  // bf16 path, chains with K split across workgroups: second kernel of that GEMM
  PH_ROUTER, PH_ROUTE, PH_MOE_GATEUP, PH_MOE_DOWN, PH_MOE_COMBINE,  // mixture of experts: in place of PH_GATEUP and PH_DOWN
  PH_MOE_PERMUTE                                                    // (runs between PH_ROUTE and PH_MOE_GATEUP)
};
#define PH_LAYER_FIRST PH_NORM1
#define PH_LAYER_LAST PH_DOWN

// LDS of a phase kernel: the union of what the fp32 and the bf16 variant of that phase need (kept per phase so
// that the GEMM kernels are not charged the attention kernels' LDS and keep their occupancy)
union PhaseShared {
  GemmShared gemm;
  AttnShared attn;
  MfmaShared mfma;
  AttnMfmaShared attn_mfma;
  SamplerShared sampler;
  float red[8];
};
union GemmPhaseShared { GemmShared gemm; MfmaShared mfma; };
union AttnPhaseShared { AttnShared attn; AttnMfmaShared attn_mfma; };
union SmallPhaseShared { float red[8]; };
template <int PH> struct PhaseSharedOf { typedef GemmPhaseShared type; };
template <> struct PhaseSharedOf<PH_ATTN> { typedef AttnPhaseShared type; };
template <> struct PhaseSharedOf<PH_SAMPLE> { typedef SamplerShared type; };
template <> struct PhaseSharedOf<PH_EMBED> { typedef SmallPhaseShared type; };
template <> struct PhaseSharedOf<PH_NORM1> { typedef SmallPhaseShared type; };
template <> struct PhaseSharedOf<PH_NORM2> { typedef SmallPhaseShared type; };
template <> struct PhaseSharedOf<PH_FINAL_NORM> { typedef SmallPhaseShared type; };
template <> struct PhaseSharedOf<PH_ROPE> { typedef SmallPhaseShared type; };
template <> struct PhaseSharedOf<PH_ATTN_COMBINE> { typedef SmallPhaseShared type; };
template <> struct PhaseSharedOf<PH_ROUTE> { typedef SmallPhaseShared type; };
template <> struct PhaseSharedOf<PH_MOE_GATEUP> { typedef MoeShared type; };
template <> struct PhaseSharedOf<PH_MOE_DOWN> { typedef MoeShared type; };
template <> struct PhaseSharedOf<PH_MOE_COMBINE> { typedef MoeShared type; };
template <> struct PhaseSharedOf<PH_MOE_PERMUTE> { typedef MoeShared type; };

template <typename WT>
__device__ __forceinline__ void run_phase_t(const DevCtx& c, int ph, u32 layer, void* shp, u32 wg, u32 nwg) {
  PhaseShared& sh = *(PhaseShared*)shp;   // only the member that belongs to phase `ph` is touched
  const IterMeta* m = c.meta;
  const u32 T = m->n_tokens, B = m->n_samples;     // B: the sequences that sample in this iteration (rows of the logits)
  const LayerW* L = c.layers + layer;
  switch (ph) {
    case PH_EMBED: phase_embed<WT>(c, wg, nwg); break;
    case PH_NORM1: phase_rmsnorm(c, c.x, L->g1, c.h, nullptr, sh.red, wg, nwg); break;
    case PH_QKV:
      phase_gemm<WT, GA_PLAIN, GE_STORE>(c.h, c.d, (const WT*)L->wqkv, c.qkv, c.qkv_n, T, c.qkv_n, c.d, sh.gemm, wg, nwg);
      break;
    case PH_ROPE: phase_rope_kvwrite<WT>(c, layer, wg, nwg); break;
    case PH_ATTN: phase_attention<WT, false>(c, layer, sh.attn, wg, nwg); break;
    case PH_OPROJ:
      phase_gemm<WT, GA_PLAIN, GE_ADD>(c.attn, c.nq * c.hd, (const WT*)L->wo, c.x, c.d, T, c.d, c.nq * c.hd, sh.gemm, wg, nwg);
      break;
    case PH_NORM2: phase_rmsnorm(c, c.x, L->g2, c.h, nullptr, sh.red, wg, nwg); break;
    case PH_GATEUP:
      phase_gemm<WT, GA_PLAIN, GE_STORE>(c.h, c.d, (const WT*)L->wgu, c.gu, 2 * c.F, T, 2 * c.F, c.d, sh.gemm, wg, nwg);
      break;
    case PH_DOWN:
      phase_gemm<WT, GA_SILU_MUL, GE_ADD>(c.gu, 2 * c.F, (const WT*)L->wd, c.x, c.d, T, c.d, c.F, sh.gemm, wg, nwg);
      break;
    case PH_FINAL_NORM: phase_rmsnorm(c, c.x, c.gf, c.hlast, c.last_idx, sh.red, wg, nwg); break;
    case PH_LM_HEAD:
      phase_gemm<WT, GA_PLAIN, GE_STORE>(c.hlast, c.d, (const WT*)c.lm, c.logits, c.V, B, c.V, c.d, sh.gemm, wg, nwg);
      break;
    case PH_SAMPLE:
      if (c.spec_k) phase_sample_publish_spec(c, *(SamplerShared*)shp, wg, nwg);
      else phase_sample_publish(c, *(SamplerShared*)shp, wg, nwg);
      break;
  }
}

// bf16 path: MFMA GEMMs on packed operands with the norms, the residual adds and the SiLU gate fused into their
// epilogues; the separate norm phases do not exist here.
__device__ __forceinline__ void run_phase_bf16(const DevCtx& c, int ph, u32 layer, void* shp, u32 wg, u32 nwg) {
  PhaseShared& sh = *(PhaseShared*)shp;
  const IterMeta* m = c.meta;
  const LayerWP* P = c.players + layer;
  MfmaGemmArgs a{};
  a.T = m->n_tokens;
  a.TBS = c.TBS;
  a.eps = c.eps;
  a.tune_nw = c.tune_nw;
  a.part = c.splitk_ok ? c.gemm_part : nullptr;
  a.part_cap = c.gemm_part_cap;
  if (ph == PH_QKV_RED || ph == PH_OPROJ_RED || ph == PH_DOWN_RED) {
    if (a.part == nullptr || a.T <= 64 || a.T > 256) return;    // this iteration's GEMMs did not split K
  }
  switch (ph) {
    case PH_EMBED: phase_embed_packed(c, wg, nwg); break;
    case PH_QKV:
    case PH_QKV_RED:
      a.Wp = P->wqkv; a.Xp = c.xq; a.N = c.qkv_n; a.K = c.d; a.ssq_in = c.ssq;
      a.positions = c.positions; a.slot_mapping = c.slot_mapping; a.rope_tab = c.rope_tab; a.qbuf = c.qbuf;
      a.Kc = (f16_t*)c.kv + (u64)layer * c.kv_layer_stride; a.Vc = a.Kc + c.kv_kv_stride;
      a.nq = c.nq; a.nkv = c.nkv; a.hd = c.hd; a.bs = c.bs;
      if (ph == PH_QKV) gemm_mfma<EPI_QKV_ROPE, true>(a, sh.mfma, wg, nwg);
      else gemm_splitk_reduce<EPI_QKV_ROPE>(a, sh.mfma, wg, nwg, 512);
      break;
    case PH_ATTN: phase_attention_mfma(c, layer, sh.attn_mfma, wg, nwg); break;
    case PH_ATTN_COMBINE: attn_decode_combine(c, wg, nwg); break;
    case PH_ROUTER:     // router logits of every token; its first workgroup also clears the experts' counters for this layer
      if (wg == 0)
        for (u32 e = threadIdx.x; e < c.n_experts; e += blockDim.x) c.moe_count[e] = 0;
      a.Wp = P->wr; a.Xp = c.xq; a.N = c.n_experts; a.K = c.d; a.ssq_in = c.ssq; a.out = c.moe_logits; a.ldo = c.n_experts;
      // few rows: with 65..256 tokens the (row tile, 64 tokens) items of the streaming schedule spread the matrix over
      // more workgroups than its single 128-row block of the tiled schedules would
      if (a.T > 64 && a.T <= 256) gemm_stream<EPI_SCALED_STORE, 1, 4, stream_batch(1, 4), true>(a, sh.mfma, wg, nwg);
      else gemm_mfma<EPI_SCALED_STORE, false>(a, sh.mfma, wg, nwg);
      break;
    case PH_ROUTE: moe_route(c, layer, wg, nwg); break;
    case PH_MOE_PERMUTE: moe_permute(c, layer, *(MoeShared*)shp, wg, nwg); break;
    case PH_MOE_GATEUP: moe_gateup(c, layer, *(MoeShared*)shp, wg, nwg); break;
    case PH_MOE_DOWN: moe_down(c, layer, *(MoeShared*)shp, wg, nwg); break;
    case PH_MOE_COMBINE: moe_combine(c, layer, *(MoeShared*)shp, wg, nwg); break;
    case PH_OPROJ:
    case PH_OPROJ_RED:
      a.Wp = P->wo; a.Xp = c.aq; a.N = c.d; a.K = c.nq * c.hd; a.x = c.x; a.ldx = c.d; a.g_next = c.layers[layer].g2;
      a.Xp_next = c.xq; a.ssq_out = c.ssq;
      if (ph == PH_OPROJ) gemm_mfma<EPI_RESIDUAL, true>(a, sh.mfma, wg, nwg);
      else gemm_splitk_reduce<EPI_RESIDUAL>(a, sh.mfma, wg, nwg, 512);
      break;
    case PH_GATEUP:
      a.Wp = P->wgu; a.Xp = c.xq; a.N = 2 * c.F; a.K = c.d; a.ssq_in = c.ssq; a.Hp = c.hq;
      gemm_mfma<EPI_SILU_GATE, false>(a, sh.mfma, wg, nwg);
      break;
    case PH_DOWN:
    case PH_DOWN_RED:
      a.Wp = P->wd; a.Xp = c.hq; a.N = c.d; a.K = c.F; a.x = c.x; a.ldx = c.d;
      a.g_next = layer + 1 < c.n_layers ? c.layers[layer + 1].g1 : c.gf;
      a.Xp_next = c.xq; a.ssq_out = c.ssq;
      if (ph == PH_DOWN) gemm_mfma<EPI_RESIDUAL, true>(a, sh.mfma, wg, nwg);
      else gemm_splitk_reduce<EPI_RESIDUAL>(a, sh.mfma, wg, nwg, 512);
      break;
    case PH_LM_HEAD:
      a.Wp = c.lm_p; a.Xp = c.xq; a.N = c.V; a.K = c.d; a.T = m->n_samples; a.tok_index = c.last_idx; a.ssq_in = c.ssq;
      a.out = c.logits; a.ldo = c.V;
      gemm_mfma<EPI_SCALED_STORE, false>(a, sh.mfma, wg, nwg);
      break;
    case PH_SAMPLE:
      if (c.spec_k) phase_sample_publish_spec(c, *(SamplerShared*)shp, wg, nwg);
      else phase_sample_publish(c, *(SamplerShared*)shp, wg, nwg);
      break;
    default: break;   // the norms and the rotary / KV-write step are fused into the GEMMs
  }
}

__device__ __forceinline__ void run_phase(const DevCtx& c, int ph, u32 layer, void* sh, u32 wg, u32 nwg) {
  if (c.meta->skip || c.meta->kind == KIND_IDLE) return;
  if (c.dtype == 1) run_phase_bf16(c, ph, layer, sh, wg, nwg);
  else run_phase_t<float>(c, ph, layer, sh, wg, nwg);
}
