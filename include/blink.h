/*
 * blink.h - C ABI of the on-GPU serving step of Blink (CPU-free LLM serving).
 *
 * The library implements the backend of section 4.2 of the paper ("Backend: GPU-resident
 * inference engine") for one AMD MI355X: a request ring in HBM, an on-GPU scheduler step
 * (ring poll, FCFS continuous batching with inline prefill, paged-KV block accounting,
 * batch metadata), the prefill/decode forward pass of a Llama-style decoder over paged KV,
 * on-device sampling and token publication. Every decision of an iteration is taken on the
 * device from device state; the loop itself is a fixed kernel chain (one HIP graph per
 * iteration) that a host thread only enqueues, a few iterations ahead, without reading any
 * result the device waits for (HIP has no device-side launch, which the paper's persistent
 * scheduler kernel relies on). While nothing is running the scheduler kernel polls the ring
 * on the device for a bounded time, so a request that reaches an idle engine is claimed
 * within microseconds. The host side of this ABI stands in for the paper's
 * SmartNIC frontend (section 4.4): blink_submit plays the RDMA datapath (payload first,
 * then the slot state), blink_poll_outputs plays the token reader (one bulk read of the
 * slot metadata, compare generation counts, fetch new tokens).
 *
 * All functions return 0 on success or a negative BLINK_ERR_* code. Nothing throws.
 * All pointers are HOST pointers. The engine owns every byte of device memory; the caller
 * owns `weights`, `prompt` and event buffers, which are copied before the call returns.
 * Threads: one thread may call blink_submit while another calls blink_poll_outputs and the
 * device loop runs; all other calls are made from one control thread.
 */
#ifndef BLINK_H
#define BLINK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BLINK_OK 0
#define BLINK_ERR_INVAL (-1)     /* null pointer, empty prompt, token id outside [0, vocab), bad sampling parameter */
#define BLINK_ERR_TOO_LARGE (-2) /* prompt + max_new_tokens exceeds max_seq_len, or its KV reservation exceeds the pool */
#define BLINK_ERR_FULL (-3)      /* the ring slot of the next ticket is not empty yet: back-pressure, retry later */
#define BLINK_ERR_DEVICE (-4)    /* a HIP call failed, or the device loop reported an internal error */
#define BLINK_ERR_STATE (-5)     /* call not allowed now: run while running, submit after shutdown, ... */

/* blink_config.flags */
#define BLINK_FLAG_TRACE 1u          /* record one trace record per iteration (blink_get_trace) */
#define BLINK_FLAG_EXIT_WHEN_IDLE 2u /* the loop stops by itself once nothing is running and nothing is pending (initial
                                        setting; blink_set_exit_when_idle changes it between windows) */
#define BLINK_FLAG_KEEP_LOGITS 8u    /* keep the logits of the last iteration readable via blink_debug_read */
#define BLINK_FLAG_NO_GRAPH 16u      /* enqueue the kernels of an iteration one by one instead of as one HIP graph */
#define BLINK_FLAG_CHUNKED_PREFILL 32u /* mixed iterations (section 7 of the paper, "chunked prefill"): every iteration runs all
                                        decoding requests (one token each, never paused) and fills the rest of its token
                                        budget, max_prefill_tokens, with prompt tokens in ticket order; a prompt longer than
                                        what is left continues in the next iteration, and a request samples its first token
                                        in the iteration that processes the last token of its prompt. Without the flag an
                                        admission makes a prefill-only iteration and running decodes pause (section 4.2) */

#define BLINK_FLAG_PREEMPTION 64u    /* on-demand KV growth (section 4.2: the DECODE_PAUSED state exists "to support preemption"):
                                        no worst-case reservation; a request is admitted when the blocks of its prompt are free,
                                        decoding requests take blocks as their contexts grow, and when a decode iteration needs
                                        more blocks than are free the most recently submitted running requests are preempted
                                        (blocks back to the free list, DECODE_PAUSED) and later resumed, before any new
                                        admission and lowest ticket first, by recomputing prompt + tokens generated so far.
                                        Not together with BLINK_FLAG_CHUNKED_PREFILL */

#define BLINK_FLAG_PREFIX_CACHE 128u /* prefix caching (section 7: a hash table inside the scheduler maps token prefixes to KV blocks):
                                        a new request whose prompt starts with full blocks of tokens that an earlier prompt
                                        started with shares those blocks and computes only the rest. Keys are chained 64-bit
                                        hashes of the prefix; cached blocks are reference-counted; unreferenced ones stay
                                        in the table at the bottom of the free queue until their block is reused. Plain mode
                                        only (not with CHUNKED_PREFILL or PREEMPTION) */

#define BLINK_FLAG_SPECULATIVE 256u  /* speculative decoding (section 7: draft generation, target verification, only accepted tokens
                                        are published) without a second model: a greedy request's drafts are the up to
                                        blink_config.spec_tokens tokens that followed the most recent earlier occurrence of its
                                        last two tokens in its own prompt and outputs (within the last 1024 positions); a decode
                                        iteration feeds them behind the last token, computes logits at every fed position, and
                                        emits row by row while the row's token confirms the next draft: exactly the tokens
                                        one-token-per-iteration decoding emits. Sampled requests never speculate. Plain mode only */

#define BLINK_FLAG_HOST_STEP 512u     /* measurement only (section 4.2, the comparison of the two scheduler placements on one engine):
                                        the launcher thread keeps nothing enqueued ahead. It waits for every iteration to end,
                                        copies a token array of the batch's size to host memory and a batch description
                                        (32 bytes per batch slot) back to the device, and only then enqueues the next
                                        iteration: the per-step synchronisation and PCIe round trip of a host-resident
                                        scheduler. The scheduling itself is still done by the device, so what this
                                        measures is a lower bound of such a scheduler's cost. Results are unchanged */

/* slot life cycle of the ring (section 4.2, "Ring buffer") */
enum {
  BLINK_SLOT_EMPTY = 0,
  BLINK_SLOT_PREFILL_PENDING = 1,
  BLINK_SLOT_PREFILL_PROCESSING = 2,
  BLINK_SLOT_DECODE_PROCESSING = 3,
  BLINK_SLOT_DECODE_COMPLETED = 4,
  BLINK_SLOT_DECODE_PAUSED = 5
};

typedef struct blink_engine blink_engine;

typedef struct {
  /* model: Llama-style decoder, no biases, untied LM head */
  uint32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  uint32_t dtype;              /* 0: fp32 weights, activations and KV cache. 1: bf16 weights; what the engine computes and
                                  stores itself (activations between the GEMMs, queries, KV cache, probabilities) is
                                  IEEE half precision, 2 bytes like bf16 but with 11 significant bits, so that the logits
                                  of a 32-layer model stay within 2e-2 of an exact evaluation; fp32 accumulation */
  float rms_eps;
  float rope_theta;
  const void* weights;         /* blob: embed[V][d]; per layer g1[d] wq[nq*hd][d] wk[nkv*hd][d] wv[nkv*hd][d]
                                  wo[d][nq*hd] g2[d] wg[F][d] wu[F][d] wd[d][F]; gf[d]; lm[V][d]. Matrices
                                  row-major [out][in] in `dtype`; the gains g1,g2,gf always fp32 */
  uint64_t weights_bytes;      /* must equal the size implied by the fields above */
  /* KV pool and scheduler */
  uint32_t kv_block_size;      /* tokens per KV block; 16 */
  uint32_t kv_num_blocks;      /* blocks in the pool */
  uint32_t max_batch;          /* batch slots (running sequences), <= 1024 (fp32 model) or <= 512 (bf16 model) */
  uint32_t max_seq_len;        /* prompt + generated tokens of one request */
  uint32_t max_prefill_tokens; /* prompt tokens per prefill iteration (the first admitted request is exempt); with
                                  BLINK_FLAG_CHUNKED_PREFILL: tokens per iteration, decodes included (must exceed max_batch) */
  uint32_t ring_slots;         /* power of two */
  int32_t eos_token_id;        /* -1: none */
  int32_t device;              /* HIP device ordinal */
  uint32_t flags;              /* BLINK_FLAG_* */
  uint32_t trace_capacity;     /* trace records kept (0: 65536); older records are overwritten */
  uint32_t idle_poll_us;       /* how long the scheduler kernel of an idle iteration keeps polling the ring on the
                                  device before it gives the iteration up (0: 2000). A request that arrives meanwhile
                                  is admitted by that same kernel */
  uint32_t pump_depth;         /* iterations the launcher thread keeps enqueued ahead of the device (0: 8; at most 1024) */
  uint32_t tune;               /* tests and tuning: forces variants of the GEMM and attention kernels (0: automatic
                                  choice; the bits are listed in csrc/mfma_gemm.h) */
  /* mixture-of-experts FFN (the second model of the paper's evaluation, section 6, is of this kind); bf16 models only */
  uint32_t n_experts;          /* 0: dense FFN. E > 0 (at most 256): every layer has a router wr[E][d] and E experts of
                                  width d_ffn; the blob then holds, in place of wg wu wd: wr[E][d] wg[E][F][d] wu[E][F][d]
                                  wd[E][d][F] */
  uint32_t n_active;           /* experts per token (1 .. min(8, n_experts)): the n_active largest router logits, ties to
                                  the lower expert id; their outputs are weighted by the softmax over those logits */
  uint32_t spec_tokens;        /* BLINK_FLAG_SPECULATIVE: most drafts per request and iteration, 1 .. 7 */
} blink_config;

typedef struct {
  float temperature;           /* 0: greedy (largest logit, ties to the lowest id) */
  uint32_t top_k;              /* 0: no top-k filter */
  float top_p;                 /* in (0, 1] */
  uint64_t seed;               /* Philox4x32-10 key; the counter is the index of the output token */
} blink_sampling;

#define BLINK_EVENT_FIRST 1u
#define BLINK_EVENT_LAST 2u

typedef struct {
  uint64_t request_id;         /* ticket returned by blink_submit */
  uint32_t index;              /* 0-based index of this token in the request's output */
  int32_t token;
  uint32_t flags;              /* BLINK_EVENT_* */
  uint32_t iteration;          /* loop iteration that produced the token */
  uint64_t device_ns;          /* device wall clock when the token was published */
} blink_event;

/* one record per iteration (section 4.2 loop: scan, claim, batch, launch, publish) */
typedef struct {
  uint32_t iteration;
  uint32_t kind;               /* 1 prefill (the iteration processes prompt tokens), 2 decode */
  uint64_t tail;               /* tickets below this were visible to the poll of this iteration */
  uint32_t n_admitted;
  uint32_t n_seqs;
  uint32_t n_tokens;
  uint32_t free_blocks;        /* after allocation */
  uint64_t first_admitted;     /* ticket, valid when n_admitted > 0 */
  uint64_t t_sched_begin_ns, t_sched_end_ns, t_forward_end_ns, t_publish_end_ns; /* device wall clock */
  uint64_t ctx_tokens;         /* sum over the batch of the context lengths its attention reads (KV tokens) */
  uint64_t chain;              /* ordinal of the scheduler kernel launch that ran this iteration, counted since init over
                                  all launches (idle polls and launches past the end of a window included): lines a
                                  profiler's list of dispatches up with the iterations */
  uint32_t n_resumed;          /* preempted requests resumed in this iteration (they prefill before the admitted ones) */
  uint32_t n_preempted;        /* requests preempted in this iteration */
} blink_trace_record;

typedef struct {
  uint64_t iterations;         /* non-idle iterations executed since init */
  uint64_t prefill_iterations;
  uint64_t tokens_out;         /* output tokens published */
  uint64_t tokens_prefilled;   /* prompt tokens processed */
  uint64_t next_ticket;        /* first ticket not yet admitted */
  uint32_t n_running;
  uint32_t free_blocks;
  uint32_t committed_blocks;
  uint32_t device_error;       /* non-zero: the loop stopped on an internal error */
  uint32_t running;            /* 1 while the loop is active */
  uint32_t windows;            /* blink_run calls so far */
  uint64_t kv_bytes, weight_bytes, ring_bytes;
  uint64_t prefix_hit_blocks;  /* prefix caching: prompt blocks found in the table so far */
  uint64_t prefix_evictions;   /* idle cached blocks whose memory was reused so far */
  uint32_t pinned_blocks;      /* cached blocks held by running requests */
  uint32_t pad1;
  uint64_t spec_drafted;       /* speculative decoding: draft tokens fed so far */
  uint64_t spec_accepted;      /* draft tokens confirmed so far */
} blink_stats;

/* blink_debug_read selectors (tests only; call while the loop is stopped) */
enum {
  BLINK_DBG_LOGITS = 1,        /* float[sampling sequences][vocab] of the last iteration, in batch-slot order (needs
                                  BLINK_FLAG_KEEP_LOGITS); every sequence samples unless a prompt chunk leaves its prompt incomplete */
  BLINK_DBG_FREE_STACK = 2,    /* uint32 free_top, then uint32[free_top] block ids, bottom first */
  BLINK_DBG_INPUT_IDS = 3,     /* int32[n_tokens] of the last iteration */
  BLINK_DBG_POSITIONS = 4,     /* int32[n_tokens] */
  BLINK_DBG_SLOT_MAPPING = 5,  /* int32[n_tokens] */
  BLINK_DBG_SEQ_BATCH_SLOT = 6,/* uint32[n_seqs] */
  BLINK_DBG_BLOCK_TABLES = 7,  /* uint32[max_batch][max_blocks_per_seq], rows by batch slot */
  BLINK_DBG_SEQ_LENS = 8,      /* uint32[n_seqs] */
  BLINK_DBG_CU_SEQLENS = 9,    /* uint32[n_seqs + 1] */
  BLINK_DBG_SLOT_STATES = 10,  /* uint32[ring_slots] */
  BLINK_DBG_HIDDEN = 11,       /* float[n_tokens][d_model]: residual stream after the last layer */
  BLINK_DBG_ROUTING = 12,      /* mixture of experts: uint32[n_layers][n_tokens][n_active], the experts every token of the
                                  last iteration was routed to, in selection order */
  BLINK_DBG_ATTN_ITEMS = 13    /* bf16 models: the work list the scheduler step handed to the decode attention of the last
                                  iteration, in the order the workgroups take it: uint32[items][8] = token index, context
                                  length, batch slot, first 512-token chunk of the item, chunk id of its result, results
                                  of its context, KV block behind its last one, 0 */
};

/* Provisioning (section 4.1): allocates all device memory, uploads and re-tiles the weights, builds the
 * ring, the free list and the scheduler state. The serving path (submit, run, poll) allocates nothing
 * afterwards; of the measurement helpers only blink_calibration_rates allocates (and frees) buffers of its own. */
int blink_init(const blink_config* cfg, blink_engine** out);

/* Ring write (section 4.4 "RDMA datapath"): copies the descriptor and the prompt into the slot of the next
 * ticket, then sets the slot state to PREFILL_PENDING. request_id_out receives the ticket (0,1,2,.. in
 * submission order, which is the FCFS order). BLINK_ERR_FULL when that slot has not been emptied yet. */
int blink_submit(blink_engine* e, const int32_t* prompt, uint32_t n_prompt, uint32_t max_new_tokens,
                 const blink_sampling* sampling, uint64_t* request_id_out);

/* Starts the serving loop (section 4.2 "Persistent scheduler") and returns at once. The loop ends after
 * max_iterations forward passes (0: unbounded), on blink_shutdown, or when idle if BLINK_FLAG_EXIT_WHEN_IDLE.
 * All state lives in device memory and survives the end of the loop: calling blink_run again continues
 * from the same logical point. BLINK_ERR_STATE if the loop is still active. Host work per iteration: one graph
 * launch and one event record by the launcher thread, nothing else. (bf16 engines in the plain mode hold two
 * captured chains, with and without the kernels that merge partial results of the decode attention; the launcher
 * picks one from the number of running sequences the device last mirrored to host memory, a hint that no result
 * depends on.) */
int blink_run(blink_engine* e, uint64_t max_iterations);

/* Whether the loop ends by itself when it finds nothing running and nothing pending (on), or keeps polling the ring
 * until blink_stop (off). Takes effect from the next blink_run; BLINK_ERR_STATE while the loop is active. */
int blink_set_exit_when_idle(blink_engine* e, uint32_t on);

/* Blocks until the loop started by blink_run has ended. Returns BLINK_ERR_DEVICE if it ended on an error. */
int blink_wait(blink_engine* e);

/* Token reader (section 4.4): non-blocking. Reads the slot metadata in one copy, compares generation counts
 * with the host's shadow, fetches the new tokens and writes up to cap events: per request in index order.
 * A slot returns to EMPTY once its LAST event has been delivered. */
int blink_poll_outputs(blink_engine* e, blink_event* buf, uint32_t cap, uint32_t* n_out);

/* Ends the current window: sets the device stop flag, waits for the loop to end, clears the flag. All state
 * stays in device memory; blink_run continues from the same point. */
int blink_stop(blink_engine* e);

/* Sets the device stop flag, waits for the loop to end, frees everything. The handle is invalid afterwards. */
int blink_shutdown(blink_engine* e);

/* Measurement and test helpers. */
/* The most recent min(cap_records, records kept) trace records, oldest of them first (needs BLINK_FLAG_TRACE; the loop
 * must be stopped). */
int blink_get_trace(blink_engine* e, blink_trace_record* buf, uint64_t cap_records, uint64_t* n_out);
int blink_get_stats(blink_engine* e, blink_stats* out);
int blink_debug_read(blink_engine* e, uint32_t what, void* buf, uint64_t cap_bytes, uint64_t* n_bytes);
/* Kernel timing for the roofline report. blink_time_phase selects one phase of the forward pass (0 embedding;
 * per layer: 1 norm, 2 QKV GEMM, 3 rotary + KV write, 4 attention, 5 output GEMM, 6 norm, 7 gate/up GEMM,
 * 8 down GEMM; 9 final norm, 10 LM head, 11 sample + publish; bf16 models also 12 merge of the decode attention's
 * chunks, 13 / 14 / 15 second kernel of the QKV / output / down GEMM when K is split across workgroups; a
 * mixture-of-experts model runs, in place of 7 and 8: 16 router GEMM, 17 expert selection, 18 grouped gate/up GEMMs,
 * 19 grouped down GEMMs, 20 weighted sum + residual, and 21 (between 17 and 18) the experts' operand gathered by
 * expert; -1 none). A
 * bf16 model has no kernels for phases 1, 3, 6 and 9 (fused into the GEMMs). While a phase is selected, the loop
 * brackets every launch of that phase's kernel with HIP events on the compute stream. After the loop has
 * stopped, blink_get_phase_times returns, per iteration enqueued in the last window and in enqueue order, the
 * summed duration in milliseconds of that kernel's launches (one per layer for per-layer phases). */
int blink_time_phase(blink_engine* e, int32_t phase);
int blink_get_phase_times(blink_engine* e, float* ms_per_iteration, uint64_t cap, uint64_t* n_out);
/* Launches one plain device-to-device copy kernel of `bytes` bytes (a multiple of 16, at most
 * 64 MiB, between two buffers set aside at init) on the compute stream and waits for it: a kernel of known traffic
 * against which hardware HBM counters are scaled. The loop must be stopped. */
int blink_calibration_copy(blink_engine* e, uint64_t bytes);
/* Measures, with HIP events on the compute stream, what three plain kernels sustain on this device: a device-to-device
 * copy of 1 GiB between two buffers this call allocates and frees (bytes read plus bytes written per second, in GB/s), a
 * register-only loop of 16x16x32 bf16 MFMA products on every compute unit (TFLOP/s), and a read of the same 1 GiB with
 * eight 16-byte loads in flight per lane (bytes read per second, in GB/s). All are written to host memory; the best of
 * three timed runs counts. Context for the roofline report: what the GEMM and attention kernels could reach at most.
 * The loop must be stopped. */
int blink_calibration_rates(blink_engine* e, double* copy_gbs, double* mfma_bf16_tflops, double* read_gbs);
/* Relates the device clock of blink_event.device_ns and of the trace to the host's monotonic clock (CLOCK_MONOTONIC,
 * nanoseconds): a one-thread kernel on a side stream writes the device clock to pinned host memory while the host
 * reads its own clock before the launch and after the value arrives. Of eight such probes the one with the shortest
 * span is returned: device_ns was read no later than host_ns and no earlier than host_ns - uncertainty_ns. May be
 * called while the loop runs. */
int blink_clock_sync(blink_engine* e, uint64_t* device_ns, uint64_t* host_ns, uint64_t* uncertainty_ns);
/* The sampler of the serving step on its own (section 4.2: temperature / top-k / top-p sampling inside the step), for
 * tests and for callers that bring their own logits: row r of logits[n_rows][vocab] (host memory, fp32) is sampled with
 * params[r]; token_index[r] is the index of the output token (the Philox counter). tokens_out[n_rows] (host). Needs no
 * engine: allocates device staging for the rows on `device`, runs the sampler kernel of the loop on the default
 * stream, copies the tokens back and frees the staging. BLINK_ERR_INVAL on a bad parameter (as blink_submit). */
int blink_sample_rows(int32_t device, const float* logits, uint32_t n_rows, uint32_t vocab, const blink_sampling* params,
                      const uint32_t* token_index, int32_t* tokens_out);
/* blink_sample_rows for callers that cannot allocate (code under HIP graph capture nearby, tight serving loops, harnesses
 * that forbid hipMalloc): the same arguments, the same kernel and the same result, but the device staging is a static
 * device array of 16 MiB that every GPU the library runs on holds until the process ends, so the call allocates and
 * frees nothing. BLINK_ERR_TOO_LARGE when the rows, their parameters and the tokens (each part padded to 256 bytes)
 * exceed 16 MiB (e.g. more than 32 rows of 128256 logits). Every call on a GPU uses that GPU's one array and overwrites
 * the part it needs (nothing has to start at zero): calls from one process are serialised by the library; calls that
 * overlap on one GPU from different processes do not share the array (each process has its own copy). */
int blink_sample_rows_static(int32_t device, const float* logits, uint32_t n_rows, uint32_t vocab, const blink_sampling* params,
                             const uint32_t* token_index, int32_t* tokens_out);
/* Message of the last error on the calling thread ("" if none). The pointer stays valid until the next call. */
const char* blink_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
