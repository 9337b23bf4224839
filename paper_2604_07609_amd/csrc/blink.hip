// libblink: host side of the C ABI (provisioning, ring producer, token reader, loop launcher) and the
// kernel entry points. See include/blink.h for the contract of every exported function.
#include "../../include/blink.h"
#include "blink_device.h"
#include "phases.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

// ================================================================================================
// kernels
// ================================================================================================
__global__ void __launch_bounds__(BLK_THREADS) k_sched(DevCtx c) {
  __shared__ SchedShared sh;
  sched_step(c, sh);
}

// speculative decoding: the drafts of the running greedy requests, ahead of the scheduler step that feeds them
__global__ void __launch_bounds__(BLK_THREADS) k_spec_draft(DevCtx c) { spec_draft(c, blockIdx.x, gridDim.x); }

// one named kernel per phase so that profiles attribute time to the step of the forward pass. Two workgroups per
// compute unit (at most 256 registers per lane): the start and the end of one workgroup overlap the other's streaming.
#define PHASE_KERNEL(name, PH)                                                   \
  __global__ void __launch_bounds__(BLK_THREADS, 2) name(DevCtx c, u32 layer) {  \
    __shared__ PhaseSharedOf<PH>::type sh;                                       \
    run_phase(c, PH, layer, &sh, blockIdx.x, gridDim.x);                         \
  }
PHASE_KERNEL(k_embed, PH_EMBED)
PHASE_KERNEL(k_norm1, PH_NORM1)
// The projections with few output rows (QKV, attention output, FFN down) run eight waves per workgroup on the bf16
// path so that K is split eight ways and enough weight bytes are in flight; the fp32 path keeps four.
#define PHASE_KERNEL8(name, PH)                                                  \
  __global__ void __launch_bounds__(512) name(DevCtx c, u32 layer) {             \
    __shared__ PhaseSharedOf<PH>::type sh;                                       \
    run_phase(c, PH, layer, &sh, blockIdx.x, gridDim.x);                         \
  }
PHASE_KERNEL8(k_qkv, PH_QKV)
PHASE_KERNEL(k_rope_kvwrite, PH_ROPE)
PHASE_KERNEL8(k_attention, PH_ATTN)
PHASE_KERNEL8(k_oproj, PH_OPROJ)
PHASE_KERNEL(k_norm2, PH_NORM2)
PHASE_KERNEL(k_gateup, PH_GATEUP)
PHASE_KERNEL8(k_down, PH_DOWN)
PHASE_KERNEL(k_final_norm, PH_FINAL_NORM)
PHASE_KERNEL(k_lm_head, PH_LM_HEAD)
PHASE_KERNEL(k_sample_publish, PH_SAMPLE)
PHASE_KERNEL(k_attention_combine, PH_ATTN_COMBINE)
PHASE_KERNEL(k_qkv_reduce, PH_QKV_RED)
PHASE_KERNEL(k_oproj_reduce, PH_OPROJ_RED)
PHASE_KERNEL(k_down_reduce, PH_DOWN_RED)
PHASE_KERNEL(k_moe_router, PH_ROUTER)
PHASE_KERNEL(k_moe_route, PH_ROUTE)
PHASE_KERNEL(k_moe_gateup, PH_MOE_GATEUP)
PHASE_KERNEL(k_moe_down, PH_MOE_DOWN)
PHASE_KERNEL(k_moe_combine, PH_MOE_COMBINE)
PHASE_KERNEL(k_moe_permute, PH_MOE_PERMUTE)

typedef void (*phase_kernel_t)(DevCtx, u32);
static phase_kernel_t phase_kernel(int ph) {
  switch (ph) {
    case PH_EMBED: return k_embed;
    case PH_NORM1: return k_norm1;
    case PH_QKV: return k_qkv;
    case PH_ROPE: return k_rope_kvwrite;
    case PH_ATTN: return k_attention;
    case PH_OPROJ: return k_oproj;
    case PH_NORM2: return k_norm2;
    case PH_GATEUP: return k_gateup;
    case PH_DOWN: return k_down;
    case PH_FINAL_NORM: return k_final_norm;
    case PH_LM_HEAD: return k_lm_head;
    case PH_ATTN_COMBINE: return k_attention_combine;
    case PH_QKV_RED: return k_qkv_reduce;
    case PH_OPROJ_RED: return k_oproj_reduce;
    case PH_DOWN_RED: return k_down_reduce;
    case PH_ROUTER: return k_moe_router;
    case PH_ROUTE: return k_moe_route;
    case PH_MOE_GATEUP: return k_moe_gateup;
    case PH_MOE_DOWN: return k_moe_down;
    case PH_MOE_COMBINE: return k_moe_combine;
    case PH_MOE_PERMUTE: return k_moe_permute;
    default: return k_sample_publish;
  }
}

// (cos, sin) of pos * theta^(-2i/hd), evaluated in fp64 and rounded once
__global__ void k_rope_table(float2* tab, u32 max_pos, u32 half, double theta) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (u64)max_pos * half) return;
  const u32 p = (u32)(i / half), j = (u32)(i % half);
  const double ang = (double)p * pow(theta, -2.0 * (double)j / (double)(2 * half));
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}

__global__ void __launch_bounds__(BLK_THREADS) k_pack_weights(const bf16_t* src, f16_t* dst, u32 N, u32 K, u32 pair_rows, u32 perm_hd) {
  pack_weights(src, dst, N, K, pair_rows, perm_hd, (u64)blockIdx.x * blockDim.x + threadIdx.x, (u64)gridDim.x * blockDim.x);
}

// plain copy of `n16` 16-byte words: the known-size kernel that calibrates the HBM traffic counters
__global__ void __launch_bounds__(BLK_THREADS) k_copy_calibration(const uint4* src, uint4* dst, u64 n16) {
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (u64)gridDim.x * blockDim.x) dst[i] = src[i];
}

// plain read of `n16` 16-byte words, eight non-temporal loads in flight per lane: what a kernel that only reads (the decode
// attention's KV stream, a decode GEMM's weight stream) can reach. The sum is written only if it equals a value it never takes.
__global__ void __launch_bounds__(BLK_THREADS) k_read_calibration(const uint4* src, u32* dst, u64 n16) {
  typedef u32 u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t* p = (const u32x4_t*)src;
  const u64 stride = (u64)gridDim.x * blockDim.x;
  u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  u32 acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u32x4_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  for (; i < n16; i += stride) { const u32x4_t v = p[i]; acc ^= v[0] ^ v[1] ^ v[2] ^ v[3]; }
  if (acc == 0x9E3779B9u) dst[(u64)blockIdx.x * blockDim.x + threadIdx.x] = acc;     // (the buffer holds zeros)
}

// register-only MFMA loop (sixteen independent 16x16x32 bf16 products per round and wave): the rate the matrix cores
// sustain on this chip at its clocks, beside which the GEMM kernels' rates are read
__global__ void __launch_bounds__(BLK_THREADS) k_mfma_calibration(float* dst, u32 rounds) {
  const u32 lane = threadIdx.x & 63;
  bf16x8_t x, y;
#pragma unroll
  for (int i = 0; i < 8; ++i) { x[i] = (__bf16)(0.001f * (float)((lane + i) & 7)); y[i] = (__bf16)(0.002f * (float)((lane * 3 + i) & 7)); }
  floatx4_t acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  for (u32 r = 0; r < rounds; ++r) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, acc[i], 0, 0, 0);
  }
  floatx4_t s = acc[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) s += acc[i];
  dst[(u64)blockIdx.x * blockDim.x + threadIdx.x] = s[0] + s[1] + s[2] + s[3];
}

__global__ void __launch_bounds__(BLK_THREADS) k_sample_rows(const float* logits, u32 n_rows, u32 V, const SampleRowParams* params,
                                                             const u32* token_index, i32* tokens) {
  __shared__ SamplerShared sh;
  sample_rows(logits, n_rows, V, params, token_index, tokens, sh);
}

// the device clock, written to pinned host memory (blink_clock_sync)
__global__ void k_clock_probe(HostMirror* m) {
  __hip_atomic_store(&m->clock_probe, dev_now_ns(), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ void k_open_window(SchedState* ss, u64 iter_limit) {
  ss->stopped = 0;
  ss->iter_limit = iter_limit;
}

// ================================================================================================
// host
// ================================================================================================
static thread_local std::string g_err;
static int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
#define HIPCHK(x)                                                                                   \
  do {                                                                                              \
    hipError_t e_ = (x);                                                                            \
    if (e_ != hipSuccess) return fail(BLINK_ERR_DEVICE, "%s: %s (%s:%d)", #x, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

struct blink_engine {
  blink_config cfg{};
  DevCtx ctx{};
  int n_cu = 256;
  u32 grid = 512;
  hipStream_t compute = nullptr, s_in = nullptr, s_out = nullptr;
  std::vector<void*> dev_allocs;
  std::vector<void*> host_allocs;
  HostCtrl* hctrl = nullptr;
  HostMirror* hmirror = nullptr;
  // producer side
  u64 next_ticket = 0;
  char* stage_in = nullptr;       // pinned: descriptor + status + prompt
  // reader side
  std::vector<std::atomic<u32>> shadow_state;   // host view: 0 empty, 1 in flight
  std::vector<u32> delivered;
  std::vector<u64> slot_ticket;
  SlotStatus* stage_status = nullptr;  // pinned [ring_slots]
  OutRec* stage_out = nullptr;         // pinned
  u64 stage_out_cap = 0;
  SlotStatus* stage_empty = nullptr;   // pinned zero status
  // loop
  std::thread launcher;
  hipGraphExec_t iter_graph = nullptr;        // the kernel chain of one iteration
  hipGraphExec_t iter_graph_whole = nullptr;  // the chain without the merge kernels of the decode attention (whole_chain_ok)
  bool whole_chain_ok = false;                // the shorter chain exists for this engine
  char *host_step_h = nullptr, *host_step_d = nullptr;   // BLINK_FLAG_HOST_STEP: pinned and device ends of the per-step copies
  u64 host_step_bytes = 0;
  int timed_phase = -1;                 // phase whose launches are bracketed by HIP events (-1: none)
  std::vector<hipEvent_t> phase_ev;     // [depth][n_layers][2]
  std::vector<float> phase_ms;          // per enqueued iteration of the current window: summed duration
  std::vector<hipEvent_t> events;
  std::atomic<bool> loop_active{false};
  std::atomic<int> loop_rc{0};
  std::atomic<u32> windows{0};
  bool shut = false;
  char *calib_src = nullptr, *calib_dst = nullptr;   // buffers of blink_calibration_copy
  u64 calib_bytes = 64ull << 20;
  u64 weight_bytes = 0, kv_bytes = 0, ring_bytes = 0;
  std::mutex dev_mu;   // serialises hipSetDevice-dependent host calls that allocate nothing

  explicit blink_engine(u32 slots) : shadow_state(slots) {}
};

template <typename T>
static int dalloc(blink_engine* e, T** p, u64 count, bool zero = true) {
  void* q = nullptr;
  const u64 bytes = count * sizeof(T) > 0 ? count * sizeof(T) : 16;
  HIPCHK(hipMalloc(&q, bytes));
  e->dev_allocs.push_back(q);
  if (zero) HIPCHK(hipMemset(q, 0, bytes));
  *p = (T*)q;
  return 0;
}
template <typename T>
static int halloc(blink_engine* e, T** p, u64 count) {
  void* q = nullptr;
  HIPCHK(hipHostMalloc(&q, count * sizeof(T) > 0 ? count * sizeof(T) : 16, hipHostMallocMapped));
  memset(q, 0, count * sizeof(T));
  e->host_allocs.push_back(q);
  *p = (T*)q;
  return 0;
}

static u64 expected_weight_bytes(const blink_config* c) {
  const u64 es = c->dtype == 1 ? 2 : 4;
  const u64 d = c->d_model, hd = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, F = c->d_ffn, V = c->vocab;
  const u64 E = c->n_experts;
  const u64 ffn = E ? E * d + E * 3 * F * d : 3 * F * d;   // router and E experts, or the one dense FFN
  const u64 per_layer = 4 * d + 4 * d + es * ((nq + 2 * nkv) * hd * d + d * nq * hd + ffn);
  return es * V * d * 2 + c->n_layers * per_layer + 4 * d;
}

static void free_all(blink_engine* e) {
  if (e->iter_graph) (void)hipGraphExecDestroy(e->iter_graph);
  if (e->iter_graph_whole) (void)hipGraphExecDestroy(e->iter_graph_whole);
  for (hipEvent_t ev : e->events) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : e->phase_ev) (void)hipEventDestroy(ev);
  for (void* p : e->dev_allocs) (void)hipFree(p);
  for (void* p : e->host_allocs) (void)hipHostFree(p);
  if (e->compute) (void)hipStreamDestroy(e->compute);
  if (e->s_in) (void)hipStreamDestroy(e->s_in);
  if (e->s_out) (void)hipStreamDestroy(e->s_out);
  delete e;
}

static int build_graph(blink_engine* e);

static int init_impl(const blink_config* cfg, blink_engine* e) {
  HIPCHK(hipSetDevice(cfg->device));
  hipDeviceProp_t prop;
  HIPCHK(hipGetDeviceProperties(&prop, cfg->device));
  e->n_cu = prop.multiProcessorCount;
  e->ctx.n_cu = (u32)e->n_cu;
  e->grid = (u32)e->n_cu * 2;
  HIPCHK(hipStreamCreateWithFlags(&e->compute, hipStreamNonBlocking));
  HIPCHK(hipStreamCreateWithFlags(&e->s_in, hipStreamNonBlocking));
  HIPCHK(hipStreamCreateWithFlags(&e->s_out, hipStreamNonBlocking));
  DevCtx& c = e->ctx;
  c.n_layers = cfg->n_layers; c.d = cfg->d_model; c.nq = cfg->n_q_heads; c.nkv = cfg->n_kv_heads; c.hd = cfg->head_dim;
  c.F = cfg->d_ffn; c.V = cfg->vocab; c.dtype = cfg->dtype; c.eps = cfg->rms_eps; c.theta = cfg->rope_theta;
  c.bs = cfg->kv_block_size; c.n_blocks = cfg->kv_num_blocks; c.max_batch = cfg->max_batch; c.max_seq_len = cfg->max_seq_len;
  c.max_prefill_tokens = cfg->max_prefill_tokens; c.ring_slots = cfg->ring_slots;
  c.max_blocks_per_seq = (cfg->max_seq_len + cfg->kv_block_size - 1) / cfg->kv_block_size;
  // a prefill iteration holds at most max_prefill_tokens, except that its first request is exempt
  c.maxT = std::max(std::max(cfg->max_prefill_tokens, cfg->max_seq_len), cfg->max_batch);
  c.eos = cfg->eos_token_id; c.flags = cfg->flags; c.trace_cap = cfg->trace_capacity ? cfg->trace_capacity : 65536u;
  c.qkv_n = (c.nq + 2 * c.nkv) * c.hd;
  c.n_experts = cfg->n_experts; c.n_active = cfg->n_experts ? cfg->n_active : 0;
  // speculative decoding: a decoding sequence feeds up to 1 + spec_k tokens and has a logits row for each of them
  c.spec_k = (cfg->flags & BLINK_FLAG_SPECULATIVE) ? cfg->spec_tokens : 0u;
  const u64 rows_cap = (u64)c.max_batch * (c.spec_k + 1);
  c.maxT = std::max<u32>(c.maxT, (u32)rows_cap);
  const u64 es = c.dtype == 1 ? 2 : 4;

  // ---- ring ----
  SlotStatus* status; SlotDesc* desc; i32* in_arena; OutRec* out_arena;
  if (int rc = dalloc(e, &status, c.ring_slots)) return rc;
  if (int rc = dalloc(e, &desc, c.ring_slots)) return rc;
  if (int rc = dalloc(e, &in_arena, (u64)c.ring_slots * c.max_seq_len, false)) return rc;
  if (int rc = dalloc(e, &out_arena, (u64)c.ring_slots * c.max_seq_len, false)) return rc;
  c.status = status; c.desc = desc; c.in_arena = in_arena; c.out_arena = out_arena;
  e->ring_bytes = (u64)c.ring_slots * (sizeof(SlotStatus) + sizeof(SlotDesc) + (u64)c.max_seq_len * (4 + sizeof(OutRec)));
  if (int rc = halloc(e, &e->hctrl, 1)) return rc;
  if (int rc = halloc(e, &e->hmirror, 1)) return rc;
  c.hctrl = e->hctrl; c.hmirror = e->hmirror;
  if (int rc = halloc(e, &e->stage_in, sizeof(SlotDesc) + sizeof(SlotStatus) + (u64)c.max_seq_len * 4)) return rc;
  if (int rc = halloc(e, &e->stage_status, c.ring_slots)) return rc;
  e->stage_out_cap = 1u << 16;
  if (int rc = halloc(e, &e->stage_out, e->stage_out_cap)) return rc;
  if (int rc = halloc(e, &e->stage_empty, 1)) return rc;
  e->delivered.assign(c.ring_slots, 0);
  e->slot_ticket.assign(c.ring_slots, 0);
  for (auto& s : e->shadow_state) s.store(0);

  // ---- scheduler state ----
  if (int rc = dalloc(e, &c.ss, 1)) return rc;
  if (int rc = dalloc(e, &c.run, c.max_batch)) return rc;
  if (int rc = dalloc(e, &c.preq, c.max_batch)) return rc;
  if (int rc = dalloc(e, &c.block_tables, (u64)c.max_batch * c.max_blocks_per_seq)) return rc;
  {
    u32 cap = 1;
    while (cap < c.n_blocks) cap <<= 1;
    c.fs_mask = cap - 1;
    if (int rc = dalloc(e, &c.free_stack, cap)) return rc;
    if (cfg->flags & BLINK_FLAG_PREFIX_CACHE) {
      c.pc_bmask = 2 * cap - 1;
      if (int rc = dalloc(e, &c.pc_ref, c.n_blocks)) return rc;
      if (int rc = dalloc(e, &c.pc_key, c.n_blocks)) return rc;
      if (int rc = dalloc(e, &c.pc_flags, c.n_blocks)) return rc;
      if (int rc = dalloc(e, &c.pc_next, c.n_blocks)) return rc;
      if (int rc = dalloc(e, &c.pc_pos, c.n_blocks)) return rc;
      if (int rc = dalloc(e, &c.pc_bucket, 2ull * cap, false)) return rc;
      HIPCHK(hipMemset(c.pc_bucket, 0xFF, 2ull * cap * 4));     // ~0u: empty chain
    }
  }
  if (int rc = dalloc(e, &c.meta, 1)) return rc;
  if (int rc = dalloc(e, &c.seq_bslot, c.max_batch)) return rc;
  if (int rc = dalloc(e, &c.seq_len, c.max_batch)) return rc;
  if (int rc = dalloc(e, &c.cu_seqlens, c.max_batch + 1)) return rc;
  if (int rc = dalloc(e, &c.last_idx, rows_cap)) return rc;
  if (c.spec_k) {
    if (int rc = dalloc(e, &c.spec_len, c.max_batch)) return rc;
    if (int rc = dalloc(e, &c.spec_tok, (u64)c.max_batch * SPEC_MAX_DRAFTS)) return rc;
    if (int rc = dalloc(e, &c.sample_row0, c.max_batch)) return rc;
    if (int rc = dalloc(e, &c.sample_nrow, c.max_batch)) return rc;
    if (int rc = dalloc(e, &c.sample_tok0, c.max_batch)) return rc;
  }
  if (int rc = dalloc(e, &c.sample_bslot, c.max_batch)) return rc;
  if (int rc = dalloc(e, &c.seq_pos0, c.max_batch)) return rc;
  if (int rc = dalloc(e, &c.seq_ring, c.max_batch)) return rc;
  if (int rc = dalloc(e, &c.cu_qtiles, c.max_batch + 1)) return rc;
  if (int rc = dalloc(e, &c.cu_chunks, c.max_batch + 1)) return rc;
  if (int rc = dalloc(e, &c.input_ids, c.maxT)) return rc;
  if (int rc = dalloc(e, &c.positions, c.maxT)) return rc;
  if (int rc = dalloc(e, &c.slot_mapping, c.maxT)) return rc;
  if (int rc = dalloc(e, &c.tok_seq, c.maxT)) return rc;
  if (int rc = dalloc(e, &c.trace, c.trace_cap)) return rc;
  {
    std::vector<u32> fs(c.n_blocks);
    for (u32 i = 0; i < c.n_blocks; ++i) fs[i] = c.n_blocks - 1 - i;   // first pops return 0, 1, 2, ...
    HIPCHK(hipMemcpy(c.free_stack, fs.data(), (u64)c.n_blocks * 4, hipMemcpyHostToDevice));
    SchedState s0{};
    s0.free_top = c.n_blocks;
    s0.stopped = 1;
    HIPCHK(hipMemcpy(c.ss, &s0, sizeof s0, hipMemcpyHostToDevice));
  }

  // ---- weights ----
  // fp32 model: the blob is uploaded as is and the matrices are used in their [out][in] layout.
  // bf16 model: the embedding table and the gains are kept as they come; every other matrix goes through a staging
  // buffer into its packed form (MFMA operand order) and the row-major copy is not kept.
  c.tune_nw = cfg->tune;
  {
    std::vector<LayerW> lw(c.n_layers);
    const u64 d = c.d, hd = c.hd, nq = c.nq, nkv = c.nkv, F = c.F, V = c.V;
    const char* hsrc = (const char*)cfg->weights;
    u64 off = 0;
    if (c.dtype == 0) {
      char* wdev;
      if (int rc = dalloc(e, &wdev, cfg->weights_bytes, false)) return rc;
      HIPCHK(hipMemcpy(wdev, hsrc, cfg->weights_bytes, hipMemcpyHostToDevice));
      e->weight_bytes = cfg->weights_bytes;
      c.embed = wdev + off; off += es * V * d;
      for (u32 l = 0; l < c.n_layers; ++l) {
        lw[l].g1 = (const float*)(wdev + off); off += 4 * d;
        lw[l].wqkv = wdev + off; off += es * (nq + 2 * nkv) * hd * d;
        lw[l].wo = wdev + off; off += es * d * nq * hd;
        lw[l].g2 = (const float*)(wdev + off); off += 4 * d;
        lw[l].wgu = wdev + off; off += es * 2 * F * d;
        lw[l].wd = wdev + off; off += es * d * F;
      }
      c.gf = (const float*)(wdev + off); off += 4 * d;
      c.lm = wdev + off; off += es * V * d;
    } else {
      std::vector<LayerWP> lp(c.n_layers);
      const u64 stage_bytes = 2 * std::max(std::max(std::max(V * d, 2 * F * d), (u64)c.n_experts * d), std::max((nq + 2 * nkv) * hd * d, d * nq * hd));
      char *stage = nullptr, *embed = nullptr;
      float* gains = nullptr;
      HIPCHK(hipMalloc((void**)&stage, stage_bytes));     // freed at the end of this block, on every path
      // src_off2 != 0: the second half of the rows is stored there (an expert's up matrix lies apart from its gate matrix)
      auto pack_to = [&](f16_t* p, u64 src_off, u64 src_off2, u32 N, u32 K, u32 pair_rows, u32 perm_hd) -> int {
        if (src_off2) {
          HIPCHK(hipMemcpy(stage, hsrc + src_off, (u64)N * K, hipMemcpyHostToDevice));
          HIPCHK(hipMemcpy(stage + (u64)N * K, hsrc + src_off2, (u64)N * K, hipMemcpyHostToDevice));
        } else {
          HIPCHK(hipMemcpy(stage, hsrc + src_off, (u64)N * K * 2, hipMemcpyHostToDevice));
        }
        hipLaunchKernelGGL(k_pack_weights, dim3(2048), dim3(BLK_THREADS), 0, e->compute, (const bf16_t*)stage, p, N, K, pair_rows, perm_hd);
        HIPCHK(hipGetLastError());
        HIPCHK(hipStreamSynchronize(e->compute));          // the staging buffer is reused by the next matrix
        return 0;
      };
      auto pack = [&](u64 src_off, u32 N, u32 K, u32 pair_rows, u32 perm_hd, const f16_t** dst) -> int {
        f16_t* p;
        const u64 elems = (u64)((N + 15) / 16) * 16 * K;
        if (int rc = dalloc(e, &p, elems, false)) return rc;
        if (int rc = pack_to(p, src_off, 0, N, K, pair_rows, perm_hd)) return rc;
        *dst = p;
        e->weight_bytes += elems * 2;
        return 0;
      };
      // the experts of one layer: packed one after the other (2F x d gate/up pairs, then d x F down matrices)
      auto pack_experts = [&](u64 off_g, u64 off_u, u64 off_d, LayerWP& lp_l) -> int {
        const u64 E = c.n_experts;
        f16_t *pgu, *pd;
        if (int rc = dalloc(e, &pgu, E * 2 * F * d, false)) return rc;
        if (int rc = dalloc(e, &pd, E * d * F, false)) return rc;
        for (u64 x = 0; x < E; ++x) {
          if (int rc = pack_to(pgu + x * 2 * F * d, off_g + x * 2 * F * d, off_u + x * 2 * F * d, 2 * c.F, c.d, c.F, 0)) return rc;
          if (int rc = pack_to(pd + x * d * F, off_d + x * 2 * d * F, 0, c.d, c.F, 0, 0)) return rc;
        }
        lp_l.wgu = pgu; lp_l.wd = pd;
        e->weight_bytes += E * 3 * F * d * 2;
        return 0;
      };
      auto all = [&]() -> int {
        if (int rc = dalloc(e, &embed, 2 * V * d, false)) return rc;
        if (int rc = dalloc(e, &gains, (2 * (u64)c.n_layers + 1) * d, false)) return rc;
        HIPCHK(hipMemcpy(embed, hsrc + off, 2 * V * d, hipMemcpyHostToDevice));
        c.embed = embed; off += 2 * V * d;
        e->weight_bytes = 2 * V * d + (2 * (u64)c.n_layers + 1) * d * 4;
        for (u32 l = 0; l < c.n_layers; ++l) {
          float* g1 = gains + (2 * (u64)l) * d;
          float* g2 = g1 + d;
          HIPCHK(hipMemcpy(g1, hsrc + off, 4 * d, hipMemcpyHostToDevice)); off += 4 * d;
          if (int rc = pack(off, c.qkv_n, c.d, 0, c.hd, &lp[l].wqkv)) return rc;
          off += 2 * (nq + 2 * nkv) * hd * d;
          if (int rc = pack(off, c.d, c.nq * c.hd, 0, 0, &lp[l].wo)) return rc;
          off += 2 * d * nq * hd;
          HIPCHK(hipMemcpy(g2, hsrc + off, 4 * d, hipMemcpyHostToDevice)); off += 4 * d;
          if (c.n_experts) {
            const u64 E = c.n_experts;
            if (int rc = pack(off, c.n_experts, c.d, 0, 0, &lp[l].wr)) return rc;
            off += 2 * E * d;
            if (int rc = pack_experts(off, off + 2 * E * F * d, off + 4 * E * F * d, lp[l])) return rc;
            off += 2 * 3 * E * F * d;
          } else {
            if (int rc = pack(off, 2 * c.F, c.d, c.F, 0, &lp[l].wgu)) return rc;
            off += 2 * 2 * F * d;
            if (int rc = pack(off, c.d, c.F, 0, 0, &lp[l].wd)) return rc;
            off += 2 * d * F;
          }
          lw[l].g1 = g1; lw[l].g2 = g2; lw[l].wqkv = lw[l].wo = lw[l].wgu = lw[l].wd = nullptr;
        }
        float* gf = gains + 2 * (u64)c.n_layers * d;
        HIPCHK(hipMemcpy(gf, hsrc + off, 4 * d, hipMemcpyHostToDevice)); off += 4 * d;
        c.gf = gf;
        if (int rc = pack(off, c.V, c.d, 0, 0, &c.lm_p)) return rc;
        off += 2 * V * d;
        c.lm = nullptr;
        return 0;
      };
      const int rc = all();
      const std::string keep = g_err;
      (void)hipFree(stage);
      g_err = keep;
      if (rc) return rc;
      LayerWP* dp;
      if (int rc2 = dalloc(e, &dp, c.n_layers)) return rc2;
      HIPCHK(hipMemcpy(dp, lp.data(), sizeof(LayerWP) * c.n_layers, hipMemcpyHostToDevice));
      c.players = dp;
    }
    if (off != cfg->weights_bytes) return fail(BLINK_ERR_INVAL, "internal: weight layout %llu != %llu", (unsigned long long)off, (unsigned long long)cfg->weights_bytes);
    LayerW* dl;
    if (int rc = dalloc(e, &dl, c.n_layers)) return rc;
    HIPCHK(hipMemcpy(dl, lw.data(), sizeof(LayerW) * c.n_layers, hipMemcpyHostToDevice));
    c.layers = dl;
  }
  {
    float2* tab;
    if (int rc = dalloc(e, &tab, (u64)c.max_seq_len * (c.hd / 2), false)) return rc;
    const u64 n = (u64)c.max_seq_len * (c.hd / 2);
    hipLaunchKernelGGL(k_rope_table, dim3((u32)((n + 255) / 256)), dim3(256), 0, e->compute, tab, c.max_seq_len, c.hd / 2, (double)c.theta);
    HIPCHK(hipGetLastError());
    c.rope_tab = tab;
  }
  // ---- bf16 model: packed activation operands between the GEMMs, decode attention partials ----
  c.TBS = ((c.maxT + 255) / 256) * 16;   // whole 256-token workgroup tiles
  if (c.dtype == 1) {
    const u64 tile_tokens = (u64)c.TBS * 16;
    if (int rc = dalloc(e, &c.xq, tile_tokens * c.d)) return rc;
    if (int rc = dalloc(e, &c.aq, tile_tokens * c.nq * c.hd)) return rc;
    if (c.n_experts) {
      // every (token, selected expert) pair is a column of the grouped GEMMs; the columns of one expert start at a
      // multiple of 16, and a workgroup tile may read up to 255 columns past the last one
      const u64 cols = (u64)c.maxT * c.n_active + 16ull * c.n_experts + 256 + 16;
      c.moe_TBS = (u32)((cols + 15) / 16);
      if (int rc = dalloc(e, &c.hq_moe, (u64)c.moe_TBS * 16 * c.F)) return rc;
      if (int rc = dalloc(e, &c.xq_moe, (u64)c.moe_TBS * 16 * c.d)) return rc;
      if (int rc = dalloc(e, &c.y_moe, (u64)c.moe_TBS * 16 * c.d, false)) return rc;
      if (int rc = dalloc(e, &c.moe_logits, (u64)c.maxT * c.n_experts, false)) return rc;
      if (int rc = dalloc(e, &c.moe_count, c.n_experts)) return rc;
      if (int rc = dalloc(e, &c.moe_list, (u64)c.n_experts * c.maxT)) return rc;
      if (int rc = dalloc(e, &c.moe_sel, (u64)c.n_layers * c.maxT * c.n_active)) return rc;
      if (int rc = dalloc(e, &c.moe_pos, (u64)c.maxT * c.n_active)) return rc;
      if (int rc = dalloc(e, &c.moe_w, (u64)c.maxT * c.n_active)) return rc;
      if (int rc = dalloc(e, &c.moe_rstd, c.maxT)) return rc;
    } else if (int rc = dalloc(e, &c.hq, tile_tokens * c.F)) return rc;
    if (int rc = dalloc(e, &c.ssq, tile_tokens * (c.d / 16))) return rc;
    if (int rc = dalloc(e, &c.qbuf, (u64)c.maxT * c.nq * c.hd)) return rc;
    if (c.max_batch > 64 && ((cfg->tune >> 28) & 3u) == 2u) {   // the chain with K split across workgroups: up to eight K slices of the widest split GEMM at 256 tokens
      c.splitk_ok = 1;
      const u64 rows = ((std::max<u64>(c.qkv_n, c.d) + 127) / 128) * 128;
      c.gemm_part_cap = 8ull * rows * 256;
      if (int rc = dalloc(e, &c.gemm_part, c.gemm_part_cap, false)) return rc;
    }
    {
      c.chunk_cap = c.max_batch * ((c.max_seq_len + ATTN_CHUNK_TOKENS - 1) / ATTN_CHUNK_TOKENS);
      if (int rc = dalloc(e, &c.chunk_rec, 2ull * c.chunk_cap)) return rc;
      if (int rc = dalloc(e, &c.attn_ctr, c.n_layers)) return rc;
    }
    {
      const u64 chunks = (u64)c.max_batch * ((c.max_seq_len + ATTN_CHUNK_TOKENS - 1) / ATTN_CHUNK_TOKENS), G = c.nq / c.nkv;
      if (int rc = dalloc(e, &c.attn_part_o, chunks * c.nkv * G * c.hd)) return rc;
      if (int rc = dalloc(e, &c.attn_part_ml, chunks * c.nkv * G * 2)) return rc;
    }
  }
  if (int rc = dalloc(e, &e->calib_src, e->calib_bytes)) return rc;
  if (int rc = dalloc(e, &e->calib_dst, e->calib_bytes)) return rc;
  // ---- KV pool ----
  c.kv_kv_stride = (u64)c.n_blocks * c.nkv * c.bs * c.hd;
  c.kv_layer_stride = 2 * c.kv_kv_stride;
  e->kv_bytes = (u64)c.n_layers * c.kv_layer_stride * es;
  char* kv;
  if (int rc = dalloc(e, &kv, e->kv_bytes, true)) return rc;   // zeroed: masked keys multiply cached values by 0
  c.kv = kv;
  // ---- activations ----
  if (int rc = dalloc(e, &c.x, (u64)c.maxT * c.d)) return rc;
  if (c.dtype == 0) {
    if (int rc = dalloc(e, &c.h, (u64)c.maxT * c.d)) return rc;
    if (int rc = dalloc(e, &c.qkv, (u64)c.maxT * c.qkv_n)) return rc;
    if (int rc = dalloc(e, &c.attn, (u64)c.maxT * c.nq * c.hd)) return rc;
    if (int rc = dalloc(e, &c.gu, (u64)c.maxT * 2 * c.F)) return rc;
    if (int rc = dalloc(e, &c.hlast, rows_cap * c.d)) return rc;
  }
  if (int rc = dalloc(e, &c.logits, rows_cap * c.V)) return rc;
  HIPCHK(hipStreamSynchronize(e->compute));
  HIPCHK(hipDeviceSynchronize());
  c.idle_poll_ns = 1000ull * (cfg->idle_poll_us ? cfg->idle_poll_us : 2000u);
  e->hctrl->exit_when_idle = (cfg->flags & BLINK_FLAG_EXIT_WHEN_IDLE) ? 1u : 0u;
  {
    u32 depth = cfg->pump_depth ? cfg->pump_depth : 8u;
    if (depth > 1024) depth = 1024;
    if (cfg->flags & BLINK_FLAG_HOST_STEP) {
      depth = 1;
      e->host_step_bytes = 32ull * c.max_batch;
      if (int rc = halloc(e, &e->host_step_h, e->host_step_bytes)) return rc;
      if (int rc = dalloc(e, &e->host_step_d, e->host_step_bytes)) return rc;
    }
    e->events.resize(depth);
    for (u32 i = 0; i < depth; ++i) HIPCHK(hipEventCreateWithFlags(&e->events[i], hipEventDisableTiming));
    e->phase_ev.resize((u64)depth * c.n_layers * 2);
    for (auto& ev : e->phase_ev) HIPCHK(hipEventCreate(&ev));
  }
  if (int rc = build_graph(e)) return rc;
  return 0;
}

extern "C" int blink_init(const blink_config* cfg, blink_engine** out) {
  g_err.clear();
  if (!cfg || !out) return fail(BLINK_ERR_INVAL, "null argument");
  *out = nullptr;
  if (!cfg->weights) return fail(BLINK_ERR_INVAL, "weights is null");
  if (cfg->dtype > 1) return fail(BLINK_ERR_INVAL, "dtype must be 0 (fp32) or 1 (bf16)");
  if (!cfg->n_layers || !cfg->d_model || !cfg->n_q_heads || !cfg->n_kv_heads || !cfg->d_ffn || !cfg->vocab)
    return fail(BLINK_ERR_INVAL, "zero model dimension");
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return fail(BLINK_ERR_INVAL, "head_dim must be 64 or 128");
  if (cfg->n_q_heads % cfg->n_kv_heads || cfg->n_q_heads / cfg->n_kv_heads > ATT_MAX_G)
    return fail(BLINK_ERR_INVAL, "n_q_heads must be a multiple (at most %d) of n_kv_heads", ATT_MAX_G);
  if (cfg->d_model % 32 || cfg->d_ffn % 32 || (cfg->n_q_heads * cfg->head_dim) % 32)
    return fail(BLINK_ERR_INVAL, "d_model, d_ffn and n_q_heads*head_dim must be multiples of 32");
  if (cfg->dtype == 1) {
    const u32 G = cfg->n_q_heads / cfg->n_kv_heads;
    if (!(G == 1 || G == 2 || G == 3 || G == 4 || G == 6 || G == 8))
      return fail(BLINK_ERR_INVAL, "bf16 path: n_q_heads / n_kv_heads must be 1, 2, 3, 4, 6 or 8");
  }
  if (cfg->n_experts) {
    if (cfg->dtype != 1) return fail(BLINK_ERR_INVAL, "mixture-of-experts models are built for dtype 1 (bf16 weights) only");
    if (cfg->n_experts > MOE_MAX_EXPERTS || !cfg->n_active || cfg->n_active > MOE_MAX_ACTIVE || cfg->n_active > cfg->n_experts)
      return fail(BLINK_ERR_INVAL, "n_experts must be at most %d and n_active in [1, min(%d, n_experts)]", MOE_MAX_EXPERTS, MOE_MAX_ACTIVE);
  }
  if (cfg->vocab >= (1u << 24)) return fail(BLINK_ERR_INVAL, "vocab must be below 2^24");
  if (cfg->kv_block_size != 16) return fail(BLINK_ERR_INVAL, "kv_block_size must be 16");
  if (!cfg->kv_num_blocks || !cfg->max_batch || cfg->max_batch > SCHED_MAX_BATCH)
    return fail(BLINK_ERR_INVAL, "kv_num_blocks must be positive and max_batch in [1, %d]", SCHED_MAX_BATCH);
  if (cfg->dtype == 1 && cfg->max_batch > ATTN_META_MAX)
    return fail(BLINK_ERR_INVAL, "bf16 models take at most %d batch slots (attention keeps the batch metadata in LDS)", ATTN_META_MAX);
  if (!cfg->max_seq_len || !cfg->max_prefill_tokens) return fail(BLINK_ERR_INVAL, "max_seq_len and max_prefill_tokens must be positive");
  if (cfg->max_seq_len >= (1u << 22)) return fail(BLINK_ERR_INVAL, "max_seq_len must be below 2^22 (the scheduler sorts contexts by a 32-bit key)");
  if ((cfg->flags & BLINK_FLAG_CHUNKED_PREFILL) && (cfg->flags & BLINK_FLAG_PREEMPTION))
    return fail(BLINK_ERR_INVAL, "preemption is built for the plain (pause-and-resume) mode, not together with chunked prefill");
  if ((cfg->flags & BLINK_FLAG_PREFIX_CACHE) && (cfg->flags & (BLINK_FLAG_CHUNKED_PREFILL | BLINK_FLAG_PREEMPTION)))
    return fail(BLINK_ERR_INVAL, "prefix caching is built for the plain mode, not together with chunked prefill or preemption");
  if ((cfg->flags & BLINK_FLAG_CHUNKED_PREFILL) && cfg->max_prefill_tokens <= cfg->max_batch)
    return fail(BLINK_ERR_INVAL, "chunked prefill: max_prefill_tokens (the token budget of an iteration) must exceed max_batch");
  if (cfg->flags & BLINK_FLAG_SPECULATIVE) {
    if (cfg->flags & (BLINK_FLAG_CHUNKED_PREFILL | BLINK_FLAG_PREEMPTION | BLINK_FLAG_PREFIX_CACHE))
      return fail(BLINK_ERR_INVAL, "speculative decoding is built for the plain mode, not together with chunked prefill, preemption or prefix caching");
    if (cfg->spec_tokens < 1 || cfg->spec_tokens >= SPEC_MAX_DRAFTS)
      return fail(BLINK_ERR_INVAL, "speculative decoding: spec_tokens must be in [1, %u]", SPEC_MAX_DRAFTS - 1);
  }
  if (!cfg->ring_slots || (cfg->ring_slots & (cfg->ring_slots - 1))) return fail(BLINK_ERR_INVAL, "ring_slots must be a power of two");
  if (cfg->weights_bytes != expected_weight_bytes(cfg))
    return fail(BLINK_ERR_INVAL, "weights_bytes is %llu, the model needs %llu", (unsigned long long)cfg->weights_bytes,
                (unsigned long long)expected_weight_bytes(cfg));
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev <= 0) return fail(BLINK_ERR_DEVICE, "no HIP device available");
  if (cfg->device < 0 || cfg->device >= n_dev) return fail(BLINK_ERR_INVAL, "device %d out of range", cfg->device);
  blink_engine* e = new blink_engine(cfg->ring_slots);
  e->cfg = *cfg;
  e->cfg.weights = nullptr;
  const int rc = init_impl(cfg, e);
  if (rc) {
    const std::string keep = g_err;
    free_all(e);
    g_err = keep;
    return rc;
  }
  *out = e;
  return BLINK_OK;
}

extern "C" int blink_submit(blink_engine* e, const int32_t* prompt, uint32_t n_prompt, uint32_t max_new_tokens,
                            const blink_sampling* sp, uint64_t* request_id_out) {
  g_err.clear();
  if (!e || !prompt || !sp) return fail(BLINK_ERR_INVAL, "null argument");
  if (e->shut) return fail(BLINK_ERR_STATE, "engine is shut down");
  const DevCtx& c = e->ctx;
  if (n_prompt == 0 || max_new_tokens == 0) return fail(BLINK_ERR_INVAL, "empty prompt or max_new_tokens == 0");
  if (!(sp->temperature >= 0.f) || !(sp->top_p > 0.f && sp->top_p <= 1.f)) return fail(BLINK_ERR_INVAL, "temperature must be >= 0 and top_p in (0,1]");
  if (sp->temperature > 0.f && (sp->top_k == 0 || sp->top_k > SAMPLER_MAX_K) && c.V > SAMPLER_MAX_K)
    return fail(BLINK_ERR_INVAL, "sampling needs top_k in [1, %d] when vocab exceeds %d", SAMPLER_MAX_K, SAMPLER_MAX_K);
  if ((u64)n_prompt + max_new_tokens > c.max_seq_len) return fail(BLINK_ERR_TOO_LARGE, "prompt + max_new_tokens exceeds max_seq_len");
  const u64 need = std::max<u64>(1, ((u64)n_prompt + max_new_tokens - 1 + c.bs - 1) / c.bs);
  if (need > c.n_blocks) return fail(BLINK_ERR_TOO_LARGE, "KV reservation of %llu blocks exceeds the pool", (unsigned long long)need);
  for (u32 i = 0; i < n_prompt; ++i)
    if (prompt[i] < 0 || (u32)prompt[i] >= c.V) return fail(BLINK_ERR_INVAL, "token id %d at %u outside the vocabulary", prompt[i], i);
  const u64 t = e->next_ticket;
  const u32 slot = (u32)(t & (c.ring_slots - 1));
  if (e->shadow_state[slot].load(std::memory_order_acquire) != 0) return fail(BLINK_ERR_FULL, "ring slot %u still in use", slot);
  HIPCHK(hipSetDevice(e->cfg.device));
  // payload first: prompt tokens and descriptor; then the state word (section 4.4 "RDMA datapath")
  SlotDesc* d = (SlotDesc*)e->stage_in;
  SlotStatus* st = (SlotStatus*)(e->stage_in + sizeof(SlotDesc));
  i32* ptoks = (i32*)(e->stage_in + sizeof(SlotDesc) + sizeof(SlotStatus));
  memset(d, 0, sizeof *d);
  d->ticket = t; d->n_prompt = n_prompt; d->max_new = max_new_tokens; d->temperature = sp->temperature; d->top_k = sp->top_k;
  d->top_p = sp->top_p; d->seed = sp->seed;
  memcpy(ptoks, prompt, (u64)n_prompt * 4);
  st->state = BLINK_SLOT_PREFILL_PENDING; st->gen_count = 0; st->ticket_lo = (u32)t; st->flags = 0;
  HIPCHK(hipMemcpyAsync(c.in_arena + (u64)slot * c.max_seq_len, ptoks, (u64)n_prompt * 4, hipMemcpyHostToDevice, e->s_in));
  HIPCHK(hipMemcpyAsync(c.desc + slot, d, sizeof *d, hipMemcpyHostToDevice, e->s_in));
  HIPCHK(hipStreamSynchronize(e->s_in));
  e->slot_ticket[slot] = t;
  e->delivered[slot] = 0;
  e->shadow_state[slot].store(1, std::memory_order_release);
  HIPCHK(hipMemcpyAsync(c.status + slot, st, sizeof *st, hipMemcpyHostToDevice, e->s_in));
  HIPCHK(hipStreamSynchronize(e->s_in));
  e->next_ticket = t + 1;
  if (request_id_out) *request_id_out = t;
  return BLINK_OK;
}

// ---- loop launcher -----------------------------------------------------------------------------------------
// The host thread is a pump: it enqueues the fixed kernel chain of one iteration, several iterations ahead,
// and never reads a result the device waits for. Every decision (what runs, on which shapes, when the window
// ends) is taken on the device; an iteration enqueued after the window has ended costs a few empty kernels.
static bool has_split_chain(const blink_engine* e) { return e->ctx.dtype == 1 && e->ctx.splitk_ok != 0; }

static bool phase_per_layer(int ph) { return (ph >= PH_LAYER_FIRST && ph <= PH_LAYER_LAST) || ph >= PH_ATTN_COMBINE; }

static int launch_phase(blink_engine* e, const DevCtx& ctx, hipStream_t st, int ph, u32 layer, u64 enq_index) {
  if (e->ctx.dtype == 1 && (ph == PH_NORM1 || ph == PH_NORM2 || ph == PH_FINAL_NORM || ph == PH_ROPE)) return 0;   // fused into the GEMMs
  const bool timed = e->timed_phase == ph && enq_index != ~0ull;
  hipEvent_t a = nullptr, b = nullptr;
  if (timed) {
    const u64 slot = (enq_index % e->events.size()) * e->ctx.n_layers + (phase_per_layer(ph) ? layer : 0);
    a = e->phase_ev[2 * slot];
    b = e->phase_ev[2 * slot + 1];
    HIPCHK(hipEventRecord(a, st));
  }
  // (bit 31 of the tuning word: the narrow projections run four waves per workgroup like the other GEMMs)
  const bool wide = ph == PH_ATTN || ((ph == PH_QKV || ph == PH_OPROJ || ph == PH_DOWN) && !(e->cfg.tune & 0x80000000u));
  const u32 threads = (wide && e->ctx.dtype == 1) ? 512u : (u32)BLK_THREADS;
  hipLaunchKernelGGL(phase_kernel(ph), dim3(e->grid), dim3(threads), 0, st, ctx, layer);
  if (timed) HIPCHK(hipEventRecord(b, st));
  return 0;
}

// The kernel chain of one iteration. An engine made with bits 28-29 of blink_config.tune = 2 runs the chain that lets
// the narrow GEMMs split K across workgroups when the iteration has 65..256 tokens; it carries a reduce kernel behind
// each of them (three more launches per layer, which do nothing in other iterations). Measured on the llama3_8b shape at
// 256 tokens, the second kernel costs what the split saves (QKV 60 -> 32 + 21 us, attention output 32 -> 26 + 14 us,
// down 69 -> 54 + 14 us), so the default chain does not split.
// whole_chain: the chain for iterations whose decode attention takes whole contexts as its items. The scheduler step
// of this chain is told to make them so whatever the batch (bit 22 of its tuning word), no item leaves a partial
// result, and the merge kernel behind every attention launch is left out: 32 launches less per iteration on a
// 32-layer model (an empty kernel costs 4-5 us here, the gap before the next one 2-3 us).
static int enqueue_iteration_kernels(blink_engine* e, hipStream_t st, u64 enq_index, bool whole_chain) {
  const bool split = has_split_chain(e);
  DevCtx c = e->ctx;
  if (whole_chain) c.tune_nw |= 0x400000u;
  if (c.spec_k) hipLaunchKernelGGL(k_spec_draft, dim3((c.max_batch + 3) / 4), dim3(BLK_THREADS), 0, st, c);
  hipLaunchKernelGGL(k_sched, dim3(1), dim3(BLK_THREADS), 0, st, c);
  if (int rc = launch_phase(e, c, st, PH_EMBED, 0, enq_index)) return rc;
  for (u32 l = 0; l < c.n_layers; ++l)
    for (int ph = PH_LAYER_FIRST; ph <= PH_LAYER_LAST; ++ph) {
      if (c.n_experts && (ph == PH_GATEUP || ph == PH_DOWN)) {    // mixture of experts: six kernels in place of the two
        if (ph == PH_DOWN) continue;
        static const int moe_chain[] = {PH_ROUTER, PH_ROUTE, PH_MOE_PERMUTE, PH_MOE_GATEUP, PH_MOE_DOWN, PH_MOE_COMBINE};
        for (int mp : moe_chain)
          if (int rc = launch_phase(e, c, st, mp, l, enq_index)) return rc;
        continue;
      }
      if (int rc = launch_phase(e, c, st, ph, l, enq_index)) return rc;
      const int after = ph == PH_ATTN ? PH_ATTN_COMBINE : ph == PH_QKV ? PH_QKV_RED : ph == PH_OPROJ ? PH_OPROJ_RED : ph == PH_DOWN ? PH_DOWN_RED : -1;
      if (c.dtype == 1 && after >= 0 && (after == PH_ATTN_COMBINE ? !whole_chain : split))
        if (int rc = launch_phase(e, c, st, after, l, enq_index)) return rc;
    }
  if (int rc = launch_phase(e, c, st, PH_FINAL_NORM, 0, enq_index)) return rc;
  if (int rc = launch_phase(e, c, st, PH_LM_HEAD, 0, enq_index)) return rc;
  if (int rc = launch_phase(e, c, st, PH_SAMPLE, 0, enq_index)) return rc;
  HIPCHK(hipGetLastError());
  return 0;
}

static int capture_chain(blink_engine* e, bool whole_chain, hipGraphExec_t* out) {
  hipGraph_t g = nullptr;
  HIPCHK(hipStreamBeginCapture(e->compute, hipStreamCaptureModeThreadLocal));
  const int rc = enqueue_iteration_kernels(e, e->compute, ~0ull, whole_chain);
  hipError_t er = hipStreamEndCapture(e->compute, &g);
  if (rc) return rc;
  HIPCHK(er);
  HIPCHK(hipGraphInstantiate(out, g, nullptr, nullptr, 0));
  HIPCHK(hipGraphDestroy(g));
  return 0;
}

static int build_graph(blink_engine* e) {
  // The shorter chain exists where the scheduler can make whole contexts the items of every decode iteration: bf16
  // models in the plain mode, unless the tuning word forces chunk items or the static kernel (bits 15, 23) or rules
  // the chain out (bit 5).
  const u32 ext = BLINK_FLAG_CHUNKED_PREFILL | BLINK_FLAG_PREEMPTION | BLINK_FLAG_PREFIX_CACHE | BLINK_FLAG_SPECULATIVE;
  e->whole_chain_ok = e->ctx.dtype == 1 && e->ctx.chunk_rec && !(e->cfg.flags & ext) && !(e->cfg.tune & 0x808020u);
  if (e->cfg.flags & BLINK_FLAG_NO_GRAPH) return 0;
  if (int rc = capture_chain(e, false, &e->iter_graph)) return rc;
  if (e->whole_chain_ok)
    if (int rc = capture_chain(e, true, &e->iter_graph_whole)) return rc;
  return 0;
}

// Which chain the next iteration runs is the launcher's choice, and the only one it makes: from the number of running
// sequences the scheduler step last mirrored to the host (a plain read of pinned memory, several iterations old, a hint
// and nothing more) it takes the shorter chain when the device would make whole contexts the items anyway (the same
// threshold). Either chain is correct for any iteration; a stale hint costs a few iterations with the other item shape.
static bool pick_whole_chain(const blink_engine* e) {
  if (!e->whole_chain_ok) return false;
  if (e->cfg.tune & 0x80u) return true;          // bit 7 of the tuning word: always (tests)
  const u32 nrun = *(volatile const u32*)&e->hmirror->n_running;
  return (u64)nrun * e->ctx.nkv >= WHOLE_CONTEXT_PAIRS_PER_CU * (u64)e->ctx.n_cu;
}

static int enqueue_iteration(blink_engine* e, u64 enq_index) {
  const bool whole = pick_whole_chain(e);
  if (e->iter_graph && e->timed_phase < 0) {
    HIPCHK(hipGraphLaunch(whole ? e->iter_graph_whole : e->iter_graph, e->compute));
    return 0;
  }
  return enqueue_iteration_kernels(e, e->compute, enq_index, whole);
}

// durations of the timed phase for the iteration enqueued at enq_index (its events have completed)
static void harvest_phase_times(blink_engine* e, u64 enq_index) {
  if (e->timed_phase < 0) return;
  const bool per_layer = phase_per_layer(e->timed_phase);
  const u32 n = per_layer ? e->ctx.n_layers : 1;
  float sum = 0.f;
  for (u32 l = 0; l < n; ++l) {
    const u64 slot = (enq_index % e->events.size()) * e->ctx.n_layers + l;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e->phase_ev[2 * slot], e->phase_ev[2 * slot + 1]) == hipSuccess) sum += ms;
  }
  e->phase_ms.push_back(sum);
}

static void pump_loop(blink_engine* e) {
  int rc = 0;
  if (hipSetDevice(e->cfg.device) != hipSuccess) rc = BLINK_ERR_DEVICE;
  const u32 depth = (u32)e->events.size();
  u64 enq = 0;
  while (rc == 0) {
    if (enq >= depth) {   // wait for the iteration enqueued `depth` ago: bounds the work in flight
      if (hipEventSynchronize(e->events[enq % depth]) != hipSuccess) { rc = BLINK_ERR_DEVICE; break; }
      harvest_phase_times(e, enq - depth);
      if (e->hmirror->error) { rc = BLINK_ERR_DEVICE; break; }
      if (__atomic_load_n(&e->hmirror->stopped, __ATOMIC_ACQUIRE)) break;
      if (e->host_step_bytes) {   // the previous iteration has ended: its tokens to the host, a batch description back
        const u64 tok_bytes = sizeof(i32) * (u64)e->ctx.max_batch;
        if (hipMemcpyAsync(e->host_step_h, e->ctx.input_ids, tok_bytes, hipMemcpyDeviceToHost, e->compute) != hipSuccess ||
            hipStreamSynchronize(e->compute) != hipSuccess ||
            hipMemcpyAsync(e->host_step_d, e->host_step_h, e->host_step_bytes, hipMemcpyHostToDevice, e->compute) != hipSuccess) {
          rc = BLINK_ERR_DEVICE;
          break;
        }
      }
    }
    rc = enqueue_iteration(e, enq);
    if (rc == 0 && hipEventRecord(e->events[enq % depth], e->compute) != hipSuccess) rc = BLINK_ERR_DEVICE;
    ++enq;
  }
  if (hipStreamSynchronize(e->compute) != hipSuccess && rc == 0) rc = BLINK_ERR_DEVICE;
  if (rc == 0) for (u64 i = enq > depth ? enq - depth : 0; i < enq; ++i) harvest_phase_times(e, i);
  if (rc == 0 && e->hmirror->error) rc = BLINK_ERR_DEVICE;
  e->loop_rc.store(rc);
  e->loop_active.store(false, std::memory_order_release);
}

extern "C" int blink_run(blink_engine* e, uint64_t max_iterations) {
  g_err.clear();
  if (!e) return fail(BLINK_ERR_INVAL, "null engine");
  if (e->shut) return fail(BLINK_ERR_STATE, "engine is shut down");
  if (e->loop_active.load(std::memory_order_acquire)) return fail(BLINK_ERR_STATE, "the loop is already running");
  if (e->launcher.joinable()) e->launcher.join();
  HIPCHK(hipSetDevice(e->cfg.device));
  if (e->hmirror->error) return fail(BLINK_ERR_DEVICE, "device loop error %u", e->hmirror->error);
  const u64 iter_limit = max_iterations ? e->hmirror->iteration + max_iterations : 0;
  e->hmirror->stopped = 0;
  hipLaunchKernelGGL(k_open_window, dim3(1), dim3(1), 0, e->compute, e->ctx.ss, iter_limit);
  HIPCHK(hipGetLastError());
  e->loop_active.store(true, std::memory_order_release);
  e->loop_rc.store(0);
  e->windows.fetch_add(1);
  e->phase_ms.clear();
  e->launcher = std::thread(pump_loop, e);
  return BLINK_OK;
}

extern "C" int blink_set_exit_when_idle(blink_engine* e, uint32_t on) {
  g_err.clear();
  if (!e) return fail(BLINK_ERR_INVAL, "null engine");
  if (e->shut) return fail(BLINK_ERR_STATE, "engine is shut down");
  if (e->loop_active.load(std::memory_order_acquire)) return fail(BLINK_ERR_STATE, "stop the loop first");
  __atomic_store_n(&e->hctrl->exit_when_idle, on ? 1u : 0u, __ATOMIC_RELEASE);
  return BLINK_OK;
}

extern "C" int blink_wait(blink_engine* e) {
  g_err.clear();
  if (!e) return fail(BLINK_ERR_INVAL, "null engine");
  if (e->launcher.joinable()) e->launcher.join();
  const int rc = e->loop_rc.load();
  if (rc) return fail(rc, "the loop ended with an error (device error %u)", e->hmirror ? e->hmirror->error : 0u);
  return BLINK_OK;
}

extern "C" int blink_poll_outputs(blink_engine* e, blink_event* buf, uint32_t cap, uint32_t* n_out) {
  g_err.clear();
  if (!e || !n_out || (!buf && cap)) return fail(BLINK_ERR_INVAL, "null argument");
  *n_out = 0;
  if (e->shut) return fail(BLINK_ERR_STATE, "engine is shut down");
  const DevCtx& c = e->ctx;
  HIPCHK(hipSetDevice(e->cfg.device));
  // one bulk read of the slot metadata (section 4.4 "Token reader")
  HIPCHK(hipMemcpyAsync(e->stage_status, c.status, sizeof(SlotStatus) * c.ring_slots, hipMemcpyDeviceToHost, e->s_out));
  HIPCHK(hipStreamSynchronize(e->s_out));
  struct Pick { u32 slot, from, n, stage_off; bool completed; };
  std::vector<Pick> picks;
  u64 staged = 0;
  u32 budget = cap;
  for (u32 slot = 0; slot < c.ring_slots && budget > 0; ++slot) {
    if (e->shadow_state[slot].load(std::memory_order_acquire) == 0) continue;
    const SlotStatus& st = e->stage_status[slot];
    if (st.ticket_lo != (u32)e->slot_ticket[slot]) continue;
    const u32 gen = st.gen_count, have = e->delivered[slot];
    if (gen <= have) continue;
    u32 n = std::min(gen - have, budget);
    if (staged + n > e->stage_out_cap) n = (u32)(e->stage_out_cap - staged);
    if (n == 0) break;
    picks.push_back({slot, have, n, (u32)staged, st.state == BLINK_SLOT_DECODE_COMPLETED && have + n == gen});
    HIPCHK(hipMemcpyAsync(e->stage_out + staged, c.out_arena + (u64)slot * c.max_seq_len + have, sizeof(OutRec) * n,
                          hipMemcpyDeviceToHost, e->s_out));
    staged += n;
    budget -= n;
  }
  if (picks.empty()) return BLINK_OK;
  HIPCHK(hipStreamSynchronize(e->s_out));
  // events across requests ordered by (iteration, ring slot); per request by index
  u32 w = 0;
  for (const Pick& p : picks)
    for (u32 i = 0; i < p.n; ++i) {
      const OutRec& r = e->stage_out[p.stage_off + i];
      blink_event& ev = buf[w++];
      ev.request_id = e->slot_ticket[p.slot];
      ev.index = p.from + i;
      ev.token = r.token;
      ev.flags = (ev.index == 0 ? BLINK_EVENT_FIRST : 0u) | ((p.completed && i + 1 == p.n) ? BLINK_EVENT_LAST : 0u);
      ev.iteration = r.iteration;
      ev.device_ns = r.device_ns;
    }
  // completed slots go back to EMPTY (the frontend's edge of the life cycle), then become reusable
  bool any_done = false;
  for (const Pick& p : picks) {
    e->delivered[p.slot] = p.from + p.n;
    if (p.completed) {
      HIPCHK(hipMemcpyAsync(c.status + p.slot, e->stage_empty, sizeof(SlotStatus), hipMemcpyHostToDevice, e->s_out));
      any_done = true;
    }
  }
  if (any_done) {
    HIPCHK(hipStreamSynchronize(e->s_out));
    for (const Pick& p : picks)
      if (p.completed) e->shadow_state[p.slot].store(0, std::memory_order_release);
  }
  *n_out = w;
  return BLINK_OK;
}

extern "C" int blink_stop(blink_engine* e) {
  g_err.clear();
  if (!e) return fail(BLINK_ERR_INVAL, "null engine");
  if (e->shut) return fail(BLINK_ERR_STATE, "engine is shut down");
  __atomic_store_n(&e->hctrl->stop, 1u, __ATOMIC_RELEASE);
  if (e->launcher.joinable()) e->launcher.join();
  __atomic_store_n(&e->hctrl->stop, 0u, __ATOMIC_RELEASE);
  const int rc = e->loop_rc.load();
  if (rc) return fail(rc, "the loop ended with an error (device error %u)", e->hmirror->error);
  return BLINK_OK;
}

extern "C" int blink_shutdown(blink_engine* e) {
  g_err.clear();
  if (!e) return fail(BLINK_ERR_INVAL, "null engine");
  (void)hipSetDevice(e->cfg.device);
  e->shut = true;
  if (e->hctrl) __atomic_store_n(&e->hctrl->stop, 1u, __ATOMIC_RELEASE);
  if (e->launcher.joinable()) e->launcher.join();
  (void)hipDeviceSynchronize();
  free_all(e);
  return BLINK_OK;
}

// the most recent min(cap_records, records kept) trace records, oldest of them first
extern "C" int blink_get_trace(blink_engine* e, blink_trace_record* buf, uint64_t cap_records, uint64_t* n_out) {
  g_err.clear();
  if (!e || !n_out || (!buf && cap_records)) return fail(BLINK_ERR_INVAL, "null argument");
  static_assert(sizeof(blink_trace_record) == sizeof(TraceRec), "trace record layout");
  if (e->loop_active.load()) return fail(BLINK_ERR_STATE, "stop the loop before reading the trace");
  HIPCHK(hipSetDevice(e->cfg.device));
  const u64 iters = e->hmirror->iteration;
  const u64 have = std::min<u64>(iters, e->ctx.trace_cap);
  const u64 n = std::min<u64>(have, cap_records);
  const u64 first = iters - n;
  for (u64 i = 0; i < n; ++i) {
    const u64 idx = (first + i) % e->ctx.trace_cap;
    const u64 run = std::min<u64>(n - i, e->ctx.trace_cap - idx);
    HIPCHK(hipMemcpy(buf + i, e->ctx.trace + idx, run * sizeof(TraceRec), hipMemcpyDeviceToHost));
    i += run - 1;
  }
  *n_out = n;
  return BLINK_OK;
}

extern "C" int blink_get_stats(blink_engine* e, blink_stats* out) {
  g_err.clear();
  if (!e || !out) return fail(BLINK_ERR_INVAL, "null argument");
  memset(out, 0, sizeof *out);
  out->running = e->loop_active.load() ? 1u : 0u;
  out->windows = e->windows.load();
  out->kv_bytes = e->kv_bytes; out->weight_bytes = e->weight_bytes; out->ring_bytes = e->ring_bytes;
  if (out->running) {   // only the host mirror is read while the loop is active
    out->iterations = e->hmirror->iteration;
    out->tokens_out = e->hmirror->tokens_out;
    out->n_running = e->hmirror->n_running;
    out->device_error = e->hmirror->error;
    return BLINK_OK;
  }
  HIPCHK(hipSetDevice(e->cfg.device));
  SchedState s;
  HIPCHK(hipMemcpy(&s, e->ctx.ss, sizeof s, hipMemcpyDeviceToHost));
  out->iterations = s.iteration; out->prefill_iterations = s.prefill_iterations; out->tokens_out = s.tokens_out;
  out->tokens_prefilled = s.tokens_prefilled; out->next_ticket = s.next_ticket; out->n_running = s.n_running;
  out->free_blocks = s.free_top - s.free_lo; out->committed_blocks = s.committed; out->device_error = s.error;
  out->prefix_hit_blocks = s.cache_hits; out->prefix_evictions = s.evictions; out->pinned_blocks = s.pinned; out->pad1 = 0;
  out->spec_drafted = s.drafted; out->spec_accepted = s.accepted;
  return BLINK_OK;
}

extern "C" int blink_debug_read(blink_engine* e, uint32_t what, void* buf, uint64_t cap_bytes, uint64_t* n_bytes) {
  g_err.clear();
  if (!e || !buf || !n_bytes) return fail(BLINK_ERR_INVAL, "null argument");
  if (e->loop_active.load()) return fail(BLINK_ERR_STATE, "stop the loop before reading device state");
  HIPCHK(hipSetDevice(e->cfg.device));
  const DevCtx& c = e->ctx;
  IterMeta m;
  SchedState s;
  HIPCHK(hipMemcpy(&m, c.meta, sizeof m, hipMemcpyDeviceToHost));
  HIPCHK(hipMemcpy(&s, c.ss, sizeof s, hipMemcpyDeviceToHost));
  const void* src = nullptr;
  u64 n = 0;
  switch (what) {
    case BLINK_DBG_LOGITS: src = c.logits; n = (u64)m.n_samples * c.V * 4; break;
    case BLINK_DBG_FREE_STACK: {
      const u32 count = s.free_top - s.free_lo;
      n = 4 + (u64)count * 4;
      if (n > cap_bytes) return fail(BLINK_ERR_INVAL, "buffer too small: need %llu bytes", (unsigned long long)n);
      memcpy(buf, &count, 4);
      std::vector<u32> ring((u64)c.fs_mask + 1);
      HIPCHK(hipMemcpy(ring.data(), c.free_stack, ring.size() * 4, hipMemcpyDeviceToHost));
      for (u32 i = 0; i < count; ++i) ((u32*)buf)[1 + i] = ring[(s.free_lo + i) & c.fs_mask];
      *n_bytes = n;
      return BLINK_OK;
    }
    case BLINK_DBG_INPUT_IDS: src = c.input_ids; n = (u64)m.n_tokens * 4; break;
    case BLINK_DBG_POSITIONS: src = c.positions; n = (u64)m.n_tokens * 4; break;
    case BLINK_DBG_SLOT_MAPPING: src = c.slot_mapping; n = (u64)m.n_tokens * 4; break;
    case BLINK_DBG_SEQ_BATCH_SLOT: src = c.seq_bslot; n = (u64)m.n_seqs * 4; break;
    case BLINK_DBG_BLOCK_TABLES: src = c.block_tables; n = (u64)c.max_batch * c.max_blocks_per_seq * 4; break;
    case BLINK_DBG_SEQ_LENS: src = c.seq_len; n = (u64)m.n_seqs * 4; break;
    case BLINK_DBG_CU_SEQLENS: src = c.cu_seqlens; n = ((u64)m.n_seqs + 1) * 4; break;
    case BLINK_DBG_SLOT_STATES: {
      n = (u64)c.ring_slots * 4;
      if (n > cap_bytes) return fail(BLINK_ERR_INVAL, "buffer too small: need %llu bytes", (unsigned long long)n);
      std::vector<SlotStatus> st(c.ring_slots);
      HIPCHK(hipMemcpy(st.data(), c.status, sizeof(SlotStatus) * c.ring_slots, hipMemcpyDeviceToHost));
      for (u32 i = 0; i < c.ring_slots; ++i) ((u32*)buf)[i] = st[i].state;
      *n_bytes = n;
      return BLINK_OK;
    }
    case BLINK_DBG_HIDDEN: src = c.x; n = (u64)m.n_tokens * c.d * 4; break;
    case BLINK_DBG_ROUTING: {
      if (!c.n_experts) return fail(BLINK_ERR_INVAL, "not a mixture-of-experts model");
      const u64 row = (u64)m.n_tokens * c.n_active * 4;
      n = row * c.n_layers;
      if (n > cap_bytes) return fail(BLINK_ERR_INVAL, "buffer too small: need %llu bytes", (unsigned long long)n);
      for (u32 l = 0; l < c.n_layers && row; ++l)
        HIPCHK(hipMemcpy((char*)buf + l * row, c.moe_sel + (u64)l * c.maxT * c.n_active, row, hipMemcpyDeviceToHost));
      *n_bytes = n;
      return BLINK_OK;
    }
    case BLINK_DBG_ATTN_ITEMS: {
      if (!c.chunk_rec) return fail(BLINK_ERR_INVAL, "not a bf16 model");
      static_assert(sizeof(ChunkRec) == 32, "work list record layout");
      n = (u64)m.n_chunks * sizeof(ChunkRec);
      if (n > cap_bytes) return fail(BLINK_ERR_INVAL, "buffer too small: need %llu bytes", (unsigned long long)n);
      const u64 n_first = (u64)m.n_full_chunks * sizeof(ChunkRec);
      if (n_first) HIPCHK(hipMemcpy(buf, c.chunk_rec, n_first, hipMemcpyDeviceToHost));
      if (n > n_first) HIPCHK(hipMemcpy((char*)buf + n_first, c.chunk_rec + c.chunk_cap, n - n_first, hipMemcpyDeviceToHost));
      *n_bytes = n;
      return BLINK_OK;
    }
    default: return fail(BLINK_ERR_INVAL, "unknown selector %u", what);
  }
  if (n > cap_bytes) return fail(BLINK_ERR_INVAL, "buffer too small: need %llu bytes", (unsigned long long)n);
  if (n) HIPCHK(hipMemcpy(buf, src, n, hipMemcpyDeviceToHost));
  *n_bytes = n;
  return BLINK_OK;
}

extern "C" int blink_time_phase(blink_engine* e, int32_t phase) {
  g_err.clear();
  if (!e) return fail(BLINK_ERR_INVAL, "null engine");
  if (e->loop_active.load()) return fail(BLINK_ERR_STATE, "stop the loop first");
  if (phase < -1 || phase > PH_MOE_PERMUTE) return fail(BLINK_ERR_INVAL, "phase out of range");
  e->timed_phase = phase;
  return BLINK_OK;
}

extern "C" int blink_get_phase_times(blink_engine* e, float* ms_per_iteration, uint64_t cap, uint64_t* n_out) {
  g_err.clear();
  if (!e || !n_out || (!ms_per_iteration && cap)) return fail(BLINK_ERR_INVAL, "null argument");
  if (e->loop_active.load()) return fail(BLINK_ERR_STATE, "stop the loop first");
  const u64 n = std::min<u64>(cap, e->phase_ms.size());
  for (u64 i = 0; i < n; ++i) ms_per_iteration[i] = e->phase_ms[i];
  *n_out = n;
  return BLINK_OK;
}

extern "C" int blink_calibration_copy(blink_engine* e, uint64_t bytes) {
  g_err.clear();
  if (!e) return fail(BLINK_ERR_INVAL, "null engine");
  if (e->loop_active.load()) return fail(BLINK_ERR_STATE, "stop the loop first");
  void* src = e->calib_src;
  void* dst = e->calib_dst;
  const u64 cap = e->calib_bytes;
  if (bytes == 0 || bytes > cap || (bytes & 15)) return fail(BLINK_ERR_INVAL, "bytes must be a multiple of 16 in (0, %llu]", (unsigned long long)cap);
  HIPCHK(hipSetDevice(e->cfg.device));
  hipLaunchKernelGGL(k_copy_calibration, dim3(e->grid * 4), dim3(BLK_THREADS), 0, e->compute, (const uint4*)src, (uint4*)dst, bytes / 16);
  HIPCHK(hipGetLastError());
  HIPCHK(hipStreamSynchronize(e->compute));
  return BLINK_OK;
}

extern "C" int blink_calibration_rates(blink_engine* e, double* copy_gbs, double* mfma_bf16_tflops, double* read_gbs) {
  g_err.clear();
  if (!e || !copy_gbs || !mfma_bf16_tflops || !read_gbs) return fail(BLINK_ERR_INVAL, "null argument");
  if (e->loop_active.load()) return fail(BLINK_ERR_STATE, "stop the loop first");
  HIPCHK(hipSetDevice(e->cfg.device));
  hipEvent_t t0, t1;
  HIPCHK(hipEventCreate(&t0));
  HIPCHK(hipEventCreate(&t1));
  // copy buffers of 1 GiB each, held only during this call: far larger than the 256 MB last-level cache, so the rate is HBM's
  const u64 copy_bytes = 1ull << 30, n16 = copy_bytes / 16;
  char *src = nullptr, *dst = nullptr;
  if (hipMalloc((void**)&src, copy_bytes) != hipSuccess || hipMalloc((void**)&dst, copy_bytes) != hipSuccess) {
    if (src) (void)hipFree(src);
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    (void)hipGetLastError();
    return fail(BLINK_ERR_DEVICE, "no room for the two 1 GiB copy buffers");
  }
  const u32 rounds = 4096, wgs = e->grid * 2;        // the MFMA loop writes one float per lane: 1 MiB of the 64 MiB buffer
  float best_copy = 0.f, best_mfma = 0.f, best_read = 0.f;
  int rc = hipMemsetAsync(src, 0, copy_bytes, e->compute) == hipSuccess ? BLINK_OK : BLINK_ERR_DEVICE;
  for (int rep = 0; rep < 4 && rc == BLINK_OK; ++rep) {   // the first repetition warms up; the best of the rest counts
    float ms = 0.f;
    if (hipEventRecord(t0, e->compute) != hipSuccess) { rc = BLINK_ERR_DEVICE; break; }
    hipLaunchKernelGGL(k_copy_calibration, dim3(e->grid * 4), dim3(BLK_THREADS), 0, e->compute, (const uint4*)src, (uint4*)dst, n16);
    if (hipEventRecord(t1, e->compute) != hipSuccess || hipEventSynchronize(t1) != hipSuccess || hipEventElapsedTime(&ms, t0, t1) != hipSuccess) { rc = BLINK_ERR_DEVICE; break; }
    if (rep && (best_copy == 0.f || ms < best_copy)) best_copy = ms;
    if (hipEventRecord(t0, e->compute) != hipSuccess) { rc = BLINK_ERR_DEVICE; break; }
    hipLaunchKernelGGL(k_mfma_calibration, dim3(wgs), dim3(BLK_THREADS), 0, e->compute, (float*)e->calib_dst, rounds);
    if (hipEventRecord(t1, e->compute) != hipSuccess || hipEventSynchronize(t1) != hipSuccess || hipEventElapsedTime(&ms, t0, t1) != hipSuccess) { rc = BLINK_ERR_DEVICE; break; }
    if (rep && (best_mfma == 0.f || ms < best_mfma)) best_mfma = ms;
    if (hipEventRecord(t0, e->compute) != hipSuccess) { rc = BLINK_ERR_DEVICE; break; }
    hipLaunchKernelGGL(k_read_calibration, dim3(e->grid), dim3(BLK_THREADS), 0, e->compute, (const uint4*)src, (u32*)e->calib_dst, n16);
    if (hipEventRecord(t1, e->compute) != hipSuccess || hipEventSynchronize(t1) != hipSuccess || hipEventElapsedTime(&ms, t0, t1) != hipSuccess) { rc = BLINK_ERR_DEVICE; break; }
    if (rep && (best_read == 0.f || ms < best_read)) best_read = ms;
  }
  (void)hipStreamSynchronize(e->compute);
  (void)hipFree(src);
  (void)hipFree(dst);
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
  if (rc != BLINK_OK || hipGetLastError() != hipSuccess) return fail(BLINK_ERR_DEVICE, "calibration kernels failed");
  *copy_gbs = 2.0 * (double)(n16 * 16) / ((double)best_copy * 1e-3) / 1e9;   // bytes read + bytes written
  *read_gbs = (double)(n16 * 16) / ((double)best_read * 1e-3) / 1e9;
  *mfma_bf16_tflops = (double)wgs * (BLK_THREADS / 64) * rounds * 16.0 * (2.0 * 16 * 16 * 32) / ((double)best_mfma * 1e-3) / 1e12;
  return BLINK_OK;
}

static u64 host_now_ns() {
  return (u64)std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

extern "C" int blink_clock_sync(blink_engine* e, uint64_t* device_ns, uint64_t* host_ns, uint64_t* uncertainty_ns) {
  g_err.clear();
  if (!e || !device_ns || !host_ns || !uncertainty_ns) return fail(BLINK_ERR_INVAL, "null argument");
  if (e->shut) return fail(BLINK_ERR_STATE, "engine is shut down");
  std::lock_guard<std::mutex> lk(e->dev_mu);
  HIPCHK(hipSetDevice(e->cfg.device));
  u64 best_span = ~0ull;
  for (int rep = 0; rep < 8; ++rep) {
    __atomic_store_n(&e->hmirror->clock_probe, 0ull, __ATOMIC_RELEASE);
    const u64 h0 = host_now_ns();
    hipLaunchKernelGGL(k_clock_probe, dim3(1), dim3(1), 0, e->s_in, e->hmirror);   // not the compute stream: the loop may be running there
    HIPCHK(hipGetLastError());
    u64 dv = 0, h1 = h0;
    while ((dv = __atomic_load_n(&e->hmirror->clock_probe, __ATOMIC_ACQUIRE)) == 0) {
      h1 = host_now_ns();
      if (h1 - h0 > 2000000000ull) return fail(BLINK_ERR_DEVICE, "the clock probe kernel did not run within 2 s");
    }
    h1 = host_now_ns();
    HIPCHK(hipStreamSynchronize(e->s_in));
    // the device read its clock somewhere between h0 and h1; the launch takes most of that span, so the read is
    // placed at its end, and the whole span is reported as the uncertainty
    if (h1 - h0 < best_span) { best_span = h1 - h0; *device_ns = dv; *host_ns = h1; *uncertainty_ns = h1 - h0; }
  }
  return BLINK_OK;
}

// ---- stand-alone sampler ------------------------------------------------------------------------------------
static int sample_rows_check(const float* logits, uint32_t n_rows, uint32_t vocab, const blink_sampling* params,
                             const uint32_t* token_index, int32_t* tokens_out) {
  if (!logits || !params || !token_index || !tokens_out) return fail(BLINK_ERR_INVAL, "null argument");
  if (n_rows == 0 || vocab == 0 || vocab >= (1u << 24)) return fail(BLINK_ERR_INVAL, "n_rows must be positive and vocab in [1, 2^24)");
  for (u32 r = 0; r < n_rows; ++r) {
    const blink_sampling& sp = params[r];
    if (!(sp.temperature >= 0.f) || !(sp.top_p > 0.f && sp.top_p <= 1.f)) return fail(BLINK_ERR_INVAL, "row %u: temperature must be >= 0 and top_p in (0,1]", r);
    if (sp.temperature > 0.f && (sp.top_k == 0 || sp.top_k > SAMPLER_MAX_K) && vocab > SAMPLER_MAX_K)
      return fail(BLINK_ERR_INVAL, "row %u: sampling needs top_k in [1, %d] when vocab exceeds %d", r, SAMPLER_MAX_K, SAMPLER_MAX_K);
  }
  return BLINK_OK;
}

// Device staging of one call, 256-byte aligned parts: logits rows, parameters, output indices, tokens.
struct SampleStaging { u64 params, index, tokens, total; };
static SampleStaging sample_staging(uint32_t n_rows, uint32_t vocab) {
  auto pad = [](u64 b) { return (b + 255) & ~255ull; };
  SampleStaging s;
  s.params = pad((u64)n_rows * vocab * 4);
  s.index = s.params + pad((u64)n_rows * sizeof(blink_sampling));
  s.tokens = s.index + pad((u64)n_rows * 4);
  s.total = s.tokens + pad((u64)n_rows * 4);
  return s;
}

// copies the rows and their parameters into the staging memory at `dev`, samples, copies the tokens back
static int sample_rows_on(char* dev, hipStream_t st, const float* logits, uint32_t n_rows, uint32_t vocab, const blink_sampling* params,
                          const uint32_t* token_index, int32_t* tokens_out) {
  static_assert(sizeof(blink_sampling) == sizeof(SampleRowParams), "the kernel reads blink_sampling as it is");
  const SampleStaging s = sample_staging(n_rows, vocab);
  HIPCHK(hipMemcpyAsync(dev, logits, (u64)n_rows * vocab * 4, hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(dev + s.params, params, (u64)n_rows * sizeof(blink_sampling), hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(dev + s.index, token_index, (u64)n_rows * 4, hipMemcpyHostToDevice, st));
  hipLaunchKernelGGL(k_sample_rows, dim3(std::min<u32>(n_rows, 1024u)), dim3(BLK_THREADS), 0, st, (const float*)dev, n_rows, vocab,
                     (const SampleRowParams*)(dev + s.params), (const u32*)(dev + s.index), (i32*)(dev + s.tokens));
  HIPCHK(hipGetLastError());
  HIPCHK(hipMemcpyAsync(tokens_out, dev + s.tokens, (u64)n_rows * 4, hipMemcpyDeviceToHost, st));
  HIPCHK(hipStreamSynchronize(st));
  return BLINK_OK;
}

extern "C" int blink_sample_rows(int32_t device, const float* logits, uint32_t n_rows, uint32_t vocab, const blink_sampling* params,
                                 const uint32_t* token_index, int32_t* tokens_out) {
  g_err.clear();
  if (int rc = sample_rows_check(logits, n_rows, vocab, params, token_index, tokens_out)) return rc;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev <= 0) return fail(BLINK_ERR_DEVICE, "no HIP device available");
  if (device < 0 || device >= n_dev) return fail(BLINK_ERR_INVAL, "device %d out of range", device);
  HIPCHK(hipSetDevice(device));
  char* dev = nullptr;
  HIPCHK(hipMalloc((void**)&dev, sample_staging(n_rows, vocab).total));
  const int rc = sample_rows_on(dev, nullptr, logits, n_rows, vocab, params, token_index, tokens_out);
  const std::string keep = g_err;
  (void)hipFree(dev);
  g_err = keep;
  return rc;
}

// ---- the same without any allocation: the staging lives in a static device array ------------------------------------
#define SAMPLE_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[SAMPLE_SCRATCH_BYTES];
#define SAMPLE_MAX_DEVICES 64
static std::mutex g_scratch_mu;                          // one call at a time per process: the calls share the array
static char* g_scratch_ptr[SAMPLE_MAX_DEVICES] = {};     // device address of `scratch` on every device used so far

extern "C" int blink_sample_rows_static(int32_t device, const float* logits, uint32_t n_rows, uint32_t vocab, const blink_sampling* params,
                                        const uint32_t* token_index, int32_t* tokens_out) {
  g_err.clear();
  if (int rc = sample_rows_check(logits, n_rows, vocab, params, token_index, tokens_out)) return rc;
  const u64 need = sample_staging(n_rows, vocab).total;
  if (need > SAMPLE_SCRATCH_BYTES)
    return fail(BLINK_ERR_TOO_LARGE, "%u rows of %u logits need %llu bytes of staging, the static buffer holds %u", n_rows, vocab,
                (unsigned long long)need, (unsigned)SAMPLE_SCRATCH_BYTES);
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev <= 0) return fail(BLINK_ERR_DEVICE, "no HIP device available");
  if (device < 0 || device >= n_dev || device >= SAMPLE_MAX_DEVICES) return fail(BLINK_ERR_INVAL, "device %d out of range", device);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  HIPCHK(hipSetDevice(device));
  if (!g_scratch_ptr[device]) {   // every device holds its own copy of the array at its own address
    char* p = nullptr;
    HIPCHK(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(BLINK_ERR_DEVICE, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[device] = p;
  }
  return sample_rows_on(g_scratch_ptr[device], nullptr, logits, n_rows, vocab, params, token_index, tokens_out);
}

extern "C" const char* blink_last_error(void) { return g_err.c_str(); }
