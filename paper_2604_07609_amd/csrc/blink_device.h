// Device-resident data structures of the serving loop (ring, scheduler state, batch metadata).
// Included by the host library and by every kernel file; plain structs only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;
typedef int32_t i32;
typedef uint16_t bf16_t;  // bf16 bit pattern
typedef uint16_t f16_t;   // IEEE half-precision bit pattern

#define BLK_THREADS 256
#define ATTN_CHUNK_TOKENS 512    // context tokens per decode-attention work item (32 KV blocks)
#define WAVE 64

// ---- ring (section 4.2 "Ring buffer"): slots + input/output token arenas --------------------------
struct SlotStatus {   // 16 B per slot: the metadata block the token reader fetches in one copy (section 4.4)
  u32 state;          // BLINK_SLOT_*
  u32 gen_count;      // tokens published so far
  u32 ticket_lo;      // low 32 bits of the owning ticket
  u32 flags;          // bit0: finished
};

struct SlotDesc {     // 64 B per slot, written by the producer before the state word
  u64 ticket;
  u32 n_prompt;
  u32 max_new;
  float temperature;
  u32 top_k;
  float top_p;
  u32 pad0;
  u64 seed;
  u64 pad1[3];
};

struct OutRec {       // 16 B per generated token in the output arena
  i32 token;
  u32 iteration;
  u64 device_ns;
};

// ---- scheduler state: everything survives the end of a loop window --------------------------------
struct RunEntry {     // one batch slot
  u32 valid;
  u32 ring_slot;
  u64 ticket;
  u32 P;              // prompt length
  u32 max_new;
  u32 gen;            // tokens generated
  u32 ctx_len;        // tokens whose K/V are in the cache
  u32 reserved;       // worst-case block reservation
  u32 n_blocks;       // blocks held
  u32 finished;
  i32 last_token;
  float temperature;
  u32 top_k;
  float top_p;
  u32 in_iter;        // 1 when admitted in the current iteration
  u32 paused;         // 1 while its slot state is DECODE_PAUSED
  u32 prefilled;      // prompt tokens whose K/V are in the cache (== P once the request decodes)
  u32 chunk;          // tokens the admitting (or resuming) iteration processes: the prompt, its first chunk (chunked prefill), the
                      // part of it behind the cached prefix (prefix caching), or prompt + outputs so far (a resumed request)
  u32 n_matched;      // prefix caching: leading blocks of the block table that were found in the table
  u64 seed;
  u64 h_end;          // prefix caching: key of the last matched block (the chain continues from it)
};

struct SchedState {
  u64 next_ticket;
  u64 iteration;        // non-idle iterations so far
  u64 prefill_iterations;
  u64 tokens_out;
  u64 tokens_prefilled;
  u64 idle_since_ns;    // device clock when the loop last turned idle (0: not idle)
  u32 free_top;         // entries in the free stack
  u32 committed;        // sum of reservations
  u32 n_running;
  u32 stopped;          // set by the scheduler when the window ends; cleared by the host at blink_run
  u32 error;
  u32 pad;
  u64 iter_limit;       // the window ends once `iteration` reaches this (0: no limit); set at blink_run
  u32 n_preempted;      // preempted requests waiting to be resumed (entries of DevCtx::preq)
  u32 free_lo;          // prefix caching: the free list is a double-ended queue, free_lo .. free_top (free-running counters,
                        // reduced modulo the queue's capacity); otherwise 0 and free_top is the number of free blocks
  u64 chains;           // scheduler kernels run so far (iterations, idle polls and launches past the end of a window)
  u32 pinned;           // prefix caching: cached blocks that running requests hold
  u32 pad3;
  u64 cache_hits;       // blocks matched so far
  u64 evictions;        // idle cached blocks reused so far
  u64 drafted;          // speculative decoding: draft tokens fed / confirmed so far
  u64 accepted;
};

// batch metadata of the current iteration (what the scheduler populates before the forward pass)
struct IterMeta {
  u32 kind;             // 0 idle, 1 prefill, 2 decode
  u32 n_seqs;
  u32 n_tokens;
  u32 iteration;
  u32 max_q_len;        // longest token run of one sequence in this iteration
  u32 max_ctx;          // longest context after this iteration
  u32 trace_idx;
  u32 skip;             // 1: the window has ended, phases do nothing (the rest describes the last real iteration)
  u32 n_samples;        // sequences that sample a token in this iteration (all of them unless a prompt chunk leaves its prompt incomplete)
  u32 max_pref_ctx;     // longest context after this iteration among the sequences that process prompt tokens
  u32 n_sample_seqs;    // sequences that sample (n_samples counts logits rows: more than one per sequence with speculative decoding)
  u32 n_full_chunks;    // decode attention work: chunks of ATTN_CHUNK_TOKENS context tokens that are full, listed first ...
  u32 n_chunks;         // ... and all chunks (the others are the last, partly filled chunk of a context)
  u32 pad;
};

// (sequence, kv head) pairs per compute unit from which the decode attention's work items are whole contexts; the
// launcher takes the kernel chain without the merge kernels from the same count (read from the host mirror)
#define WHOLE_CONTEXT_PAIRS_PER_CU 4ull

// One work item of the decode attention (times the kv heads), as the kernel takes it from the scheduler (32 bytes: one
// scalar load of a wave): a run of KV blocks of one decoding sequence that one workgroup walks, ATTN_CHUNK_TOKENS at a
// time, into one result. With few sequences an item is one chunk of a context (so that the chip has enough items; the
// chunks' partial results are merged by the combine kernel): full chunks are listed first (DevCtx::chunk_rec[0 ..
// n_full_chunks)), the partly filled ones behind them from DevCtx::chunk_rec[chunk_cap]. With many sequences an item is
// a whole context (no partial results, fewer merges), listed longest first. The workgroups take the list in order.
struct ChunkRec {
  u32 tok;              // index of the sequence's token of this iteration
  u32 ctx;              // context length after this iteration
  u32 bslot;            // batch slot (row of the block table)
  u32 ch;               // first chunk of the run inside the context
  u32 ci;               // chunk id of the result: cu_chunks[sequence] + ch (where a partial result goes)
  u32 nch;              // results of this context (1: the item's result is final)
  u32 b_end;            // KV block behind the run's last one
  u32 pad1;
};

struct TraceRec {       // mirrors blink_trace_record
  u32 iteration, kind;
  u64 tail;
  u32 n_admitted, n_seqs, n_tokens, free_blocks;
  u64 first_admitted;
  u64 t_sched_begin, t_sched_end, t_forward_end, t_publish_end;
  u64 ctx_tokens;
  u64 chain;
  u32 n_resumed, n_preempted;
};

// host-visible mirror in pinned host memory, written by the scheduler with system-scope stores
struct HostMirror {
  u64 iteration;
  u64 tokens_out;
  u32 stopped;
  u32 error;
  u32 n_running;
  u32 idle;
  u64 clock_probe;      // device clock written by the clock probe kernel
};

// host -> device control words (pinned host memory, read by the scheduler with system-scope loads)
struct HostCtrl {
  u32 stop;             // blink_stop / blink_shutdown
  u32 exit_when_idle;   // the window ends by itself once nothing is running and nothing is pending (and idle polling is off)
};

struct LayerW {
  const float* g1;
  const void* wqkv;     // [ (nq+2nkv)*hd ][d]
  const void* wo;       // [d][nq*hd]
  const float* g2;
  const void* wgu;      // [2F][d]: gate rows then up rows
  const void* wd;       // [d][F]
};

struct LayerWP {        // weights of a bf16 model re-tiled into MFMA operand order and re-encoded as scaled halves (see mfma_gemm.h)
  const f16_t* wqkv;    // N = (nq+2nkv)*hd, K = d
  const f16_t* wo;      // N = d, K = nq*hd
  const f16_t* wgu;     // N = 2F (gate_j, up_j interleaved), K = d; mixture of experts: the experts' matrices one after the other
  const f16_t* wd;      // N = d, K = F; mixture of experts: one per expert, one after the other
  const f16_t* wr;      // mixture of experts: router, N = n_experts, K = d
};

struct DevCtx {
  // model
  u32 n_layers, d, nq, nkv, hd, F, V, dtype;
  u32 n_experts, n_active;   // mixture of experts (0: dense FFN); F is then the width of one expert
  float eps, theta;
  // engine
  u32 bs, n_blocks, max_batch, max_seq_len, max_prefill_tokens, ring_slots, max_blocks_per_seq, maxT;
  i32 eos;
  u32 flags, trace_cap, qkv_n;
  u32 n_cu;             // compute units of the device
  u64 idle_poll_ns;     // how long the scheduler step of an empty engine polls the ring before it reports an idle iteration
  // ring
  SlotStatus* status;
  SlotDesc* desc;
  i32* in_arena;        // [ring_slots][max_seq_len]
  OutRec* out_arena;    // [ring_slots][max_seq_len]
  HostCtrl* hctrl;
  HostMirror* hmirror;
  // scheduler
  SchedState* ss;
  RunEntry* run;
  RunEntry* preq;       // [max_batch] preemption mode: the preempted requests (no blocks, no batch slot), unordered
  u32* block_tables;    // [max_batch][max_blocks_per_seq]
  // speculative decoding: drafts per batch slot (written by the draft kernel ahead of the scheduler), and per sampling
  // sequence its first logits row, number of rows and the token index of its first row
  u32 spec_k;
  u32* spec_len;        // [max_batch]
  i32* spec_tok;        // [max_batch][8]
  u32* sample_row0;     // [max_batch]
  u32* sample_nrow;     // [max_batch]
  u32* sample_tok0;     // [max_batch]
  u32* free_stack;      // [fs_mask + 1 >= n_blocks] (a ring when prefix caching pushes at its bottom)
  u32 fs_mask;
  // prefix caching: per block, reference count, key, flags (PC_CACHED: in the table; PC_LINKED: a node of a bucket's chain,
  // possibly stale), next node of the chain, position in the free queue while idle; the heads of the buckets' chains
  u32* pc_ref;
  u64* pc_key;
  u32* pc_flags;
  u32* pc_next;
  u32* pc_pos;
  u32* pc_bucket;
  u32 pc_bmask;
  IterMeta* meta;
  u32* seq_bslot;       // [max_batch]
  u32* seq_len;         // [max_batch]
  u32* cu_seqlens;      // [max_batch+1]
  u32* last_idx;        // [max_batch * (spec_k + 1)] token index of every logits row (one per sampling sequence: its last token; with
                        // speculative decoding one per token a decoding sequence processes)
  u32* sample_bslot;    // [max_batch] batch slot of every sampling sequence
  u32* seq_pos0;        // [max_batch] position of the first token every sequence processes in this iteration
  u32* seq_ring;        // [max_batch] ring slot of a sequence that processes prompt tokens, ~0 for a decoding one
  u32* cu_qtiles;       // [max_batch+1] prefix sum of ceil(tokens/16) per sequence of the iteration
  ChunkRec* chunk_rec;  // [2 * chunk_cap] (bf16 models; null otherwise)
  u32 chunk_cap;        // max_batch * chunks of the longest context
  u32* attn_ctr;        // [n_layers] work counters of the decode attention launches, zeroed by the scheduler step
  u32* cu_chunks;       // [max_batch+1] prefix sum of ceil(context/ATTN_CHUNK_TOKENS) per sequence (decode attention work items)
  i32* input_ids;       // [maxT]
  i32* positions;       // [maxT]
  i32* slot_mapping;    // [maxT]
  u32* tok_seq;         // [maxT]
  TraceRec* trace;
  // weights
  const void* embed;
  const LayerW* layers;
  const float* gf;
  const void* lm;
  const float2* rope_tab;  // [max_seq_len][hd/2] (cos, sin)
  // KV pool: [layer][2][n_blocks][nkv][bs][hd]
  void* kv;
  u64 kv_layer_stride;  // elements
  u64 kv_kv_stride;     // elements between the K and the V half of a layer
  // activations
  float* x;             // [maxT][d] residual stream
  float* h;             // [maxT][d] normalised input of a GEMM
  float* qkv;           // [maxT][qkv_n]
  float* attn;          // [maxT][nq*hd]
  float* gu;            // [maxT][2F]
  float* hlast;         // [max_batch][d]
  float* logits;        // [max_batch][V]
  // bf16 path: packed weights and packed activation operands
  const LayerWP* players;
  const f16_t* lm_p;
  f16_t* xq;            // packed half(x * gain of the next RMSNorm), inner dimension d
  f16_t* aq;            // packed attention output (half), inner dimension nq*hd
  f16_t* qbuf;          // [maxT][nq][hd] rotated queries scaled by 1/sqrt(hd), half precision like the KV cache they meet
  f16_t* hq;            // packed half(silu(gate)*up), inner dimension F
  float* ssq;           // [token][d/16] partial sums of squares of the residual stream
  u32 TBS;              // token-block stride of the packed activation buffers
  u32 tune_nw;          // tuning knob of the streaming GEMM (0: automatic)
  // mixture of experts
  float* moe_logits;    // [maxT][n_experts] router logits
  u32* moe_count;       // [n_experts] tokens routed to every expert in the current layer
  u32* moe_list;        // [n_experts][maxT] their token indices (order inside a list depends on timing, results do not)
  u32* moe_sel;         // [n_layers][maxT * n_active] selected expert of every (token, slot), kept per layer for tests
  u32* moe_pos;         // [maxT * n_active] place of the pair in its expert's list
  float* moe_w;         // [maxT * n_active] softmax weight of the pair
  float* moe_rstd;      // [maxT] norm scale of the token's FFN input
  f16_t* xq_moe;        // packed normalised FFN input of all pairs, columns grouped by expert, inner dimension d
  f16_t* hq_moe;        // packed silu(gate)*up of all pairs, columns grouped by expert (groups padded to 16), inner dimension F
  float* y_moe;         // [columns][d] expert outputs of all pairs
  u32 moe_TBS;          // token-block stride of hq_moe
  // GEMMs with K split across workgroups (decode iterations of 65..256 tokens): the slices' fp32 partial sums
  float* gemm_part;
  u64 gemm_part_cap;    // floats
  u32 splitk_ok;        // 1: the engine's kernel chain carries the reduce kernels (a chain without them never splits)
  // decode attention: partial (max, sum, output) of every chunk of a context longer than one chunk
  float* attn_part_o;   // [chunk][kv head][G][hd]
  float* attn_part_ml;  // [chunk][kv head][G][2]
};

__device__ __forceinline__ u64 dev_now_ns() { return wall_clock64() * 10ull; }  // 100 MHz constant clock

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((u32)b) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even; inputs are finite
  u32 u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// two floats to half precision (round to nearest even), saturating at the largest finite half; low half = a
__device__ __forceinline__ u32 pack_f16x2(float a, float b) {
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  const half2_t h = {(_Float16)__builtin_fminf(__builtin_fmaxf(a, -65504.f), 65504.f),
                     (_Float16)__builtin_fminf(__builtin_fmaxf(b, -65504.f), 65504.f)};
  return *(const u32*)&h;
}
__device__ __forceinline__ f16_t f32_to_f16(float a) { return (f16_t)(pack_f16x2(a, 0.f) & 0xFFFFu); }
