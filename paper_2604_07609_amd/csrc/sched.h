// The scheduler step of the serving loop: one workgroup of 256 threads, the first kernel of every iteration's
// chain (section 4.2 of the paper: "Persistent scheduler", "Parallel slot scanning", "Continuous batching with
// inline prefill"; the paper's scheduler is one resident kernel that launches graphs from the device, here it is
// a kernel per iteration that a host thread enqueues ahead of time).
// Per iteration: retire finished requests, poll the ring for the contiguous run of pending tickets,
// admit FCFS under the batch-slot / block-reservation / prefill-token limits, allocate KV blocks from
// the free stack by prefix-sum offsets (deterministic block ids), and build the batch metadata.
// With nothing running and nothing pending it keeps polling the ring on the device for a bounded time.
// Integer work only; all decisions are functions of device state, never of the host.
//
// Prefix caching (flag 128; the paper's section 7 names a hash table inside the scheduler that maps token prefixes to
// blocks): full blocks of prompt tokens are entered into a table under a chained 64-bit hash of the whole prefix. A new
// request walks its prompt's keys until the first miss; the blocks found head its block table and its prefill starts
// behind them. Cached blocks carry reference counts; a block whose count drops to zero stays in the table and goes to
// the BOTTOM of the free list (a double-ended queue then), so private blocks are reused first and idle cached blocks
// oldest first; a pop of an idle cached block evicts it. The table is a set of chains through the blocks
// (pc_bucket / pc_next); an evicted block's node stays in its chain, marked stale, until the block is entered again.
#pragma once
#include "blink_device.h"

#define SLOT_EMPTY 0u
#define SLOT_PREFILL_PENDING 1u
#define SLOT_PREFILL_PROCESSING 2u
#define SLOT_DECODE_PROCESSING 3u
#define SLOT_DECODE_COMPLETED 4u
#define SLOT_DECODE_PAUSED 5u

#define KIND_IDLE 0u
#define KIND_PREFILL 1u
#define KIND_DECODE 2u

#define SCHED_MAX_BATCH 1024

#define PC_CACHED 1u
#define PC_LINKED 2u
#define PC_H0 0x243F6A8885A308D3ull
#define FS(i) c.free_stack[(i) & c.fs_mask]

struct SchedShared {
  u32 wave_part[8];
  u32 wave_part2[8];
  u32 free_list[SCHED_MAX_BATCH];
  u32 seq_tok0[SCHED_MAX_BATCH];     // prefill metadata: first token, batch slot and ring slot of every sequence
  u32 seq_bslot[SCHED_MAX_BATCH];
  u32 seq_ring[SCHED_MAX_BATCH];
  u32 seq_pos0[SCHED_MAX_BATCH];
  u32 seq_P[SCHED_MAX_BATCH];        // prompt length: positions beyond it take the request's own output tokens (a resumed request)
  alignas(16) u32 dec_key[SCHED_MAX_BATCH];   // per batch slot: sort key of a decoding sequence (0: none), its chunk id ...
  u32 dec_si[SCHED_MAX_BATCH];
  u32 dec_tok[SCHED_MAX_BATCH];      // ... and the index of its token
  u32 flag;
  u32 exit_idle;
  u64 chain;
  u64 part64[8];
  u64 pc_g[BLK_THREADS];             // prefix caching: hashes of a strip of blocks
};

// The output function of splitmix64, and the hash of one block of 16 token ids: a polynomial in (id + 1) modulo 2^64 with
// that generator's increment as multiplier, mixed once.
__device__ __forceinline__ u64 pc_mix64(u64 z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__device__ __forceinline__ u64 pc_block_hash(const i32* toks) {
  u64 a = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i)
    a = a * 0x9E3779B97F4A7C15ull + (u64)(u32)__hip_atomic_load(toks + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) + 1ull;
  return pc_mix64(a);
}
// the cached block with key h, or ~0u (stale nodes of evicted blocks are passed over; the walk is bounded)
__device__ __forceinline__ u32 pc_lookup(const DevCtx& c, u64 h) {
  u32 n = c.pc_bucket[(u32)h & c.pc_bmask];
  for (u32 steps = 0; n != ~0u && steps < c.n_blocks; ++steps) {
    if ((c.pc_flags[n] & PC_CACHED) && c.pc_key[n] == h) return n;
    n = c.pc_next[n];
  }
  return ~0u;
}
// Enters block blk under key h (one thread). A stale node of the block is taken out of its old chain first. Returns
// false, and leaves the block private, when the key is in the table already.
__device__ __forceinline__ bool pc_insert(const DevCtx& c, u32 blk, u64 h) {
  if (c.pc_flags[blk] & PC_LINKED) {
    const u32 ob = (u32)c.pc_key[blk] & c.pc_bmask;
    u32 n = c.pc_bucket[ob];
    if (n == blk) c.pc_bucket[ob] = c.pc_next[blk];
    else {
      u32 steps = 0;
      while (n != ~0u && c.pc_next[n] != blk && steps < c.n_blocks) { n = c.pc_next[n]; ++steps; }
      if (n != ~0u && c.pc_next[n] == blk) c.pc_next[n] = c.pc_next[blk];
      else c.ss->error = 4;            // cannot happen: a linked block is in the chain of its key
    }
    c.pc_flags[blk] = 0;
  }
  if (pc_lookup(c, h) != ~0u) return false;
  const u32 bi = (u32)h & c.pc_bmask;
  c.pc_next[blk] = c.pc_bucket[bi];
  c.pc_bucket[bi] = blk;
  c.pc_key[blk] = h;
  c.pc_flags[blk] = PC_CACHED | PC_LINKED;
  c.pc_ref[blk] = 1;
  return true;
}

// ---- speculative decoding: the drafts of every running greedy request, one wave per batch slot ------------------------
// Token i of a request: its prompt, then its outputs.
#define SPEC_LOOKBACK 1024u
#define SPEC_MAX_DRAFTS 8u
__device__ __forceinline__ i32 spec_token_at(const DevCtx& c, const RunEntry& r, u32 i) {
  const u64 base = (u64)r.ring_slot * c.max_seq_len;
  if (i < r.P) return __hip_atomic_load(c.in_arena + base + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  return c.out_arena[base + (i - r.P)].token;
}
// With n tokens so far: the most recent i <= n - 3 (not below n - 2 - SPEC_LOOKBACK) with tokens i, i + 1 equal to tokens
// n - 2, n - 1; the tokens from i + 2 on, at most spec_k, are the drafts. The lanes test 64 places at a time, from the
// most recent backwards. Runs ahead of the scheduler kernel, which cuts the count to what the request may still emit.
__device__ __forceinline__ void spec_draft(const DevCtx& c, u32 wg, u32 nwg) {
  const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (u32 b = wg * nw + w; b < c.max_batch; b += nwg * nw) {
    const RunEntry r = c.run[b];
    u32 len = 0;
    if (r.valid && !r.finished && r.temperature == 0.f && r.gen >= 1 && r.P + r.gen >= 3) {
      const i32 n = (i32)(r.P + r.gen);
      const i32 t1 = spec_token_at(c, r, (u32)n - 2), t2 = spec_token_at(c, r, (u32)n - 1);
      const i32 lowest = max(0, n - 2 - (i32)SPEC_LOOKBACK);
      i32 found = -1;
      for (i32 hi = n - 3; hi >= lowest && found < 0; hi -= 64) {
        const i32 i = hi - (i32)lane;
        const bool hit = i >= lowest && spec_token_at(c, r, (u32)i) == t1 && spec_token_at(c, r, (u32)i + 1) == t2;
        const unsigned long long bal = __ballot(hit);
        if (bal) found = hi - (i32)(__ffsll((long long)bal) - 1);      // the lowest lane that hit tested the most recent place
      }
      if (found >= 0) {
        len = min(c.spec_k, (u32)(n - (found + 2)));
        if (lane < len) c.spec_tok[(u64)b * SPEC_MAX_DRAFTS + lane] = spec_token_at(c, r, (u32)found + 2 + lane);
      }
    }
    if (lane == 0) c.spec_len[b] = len;
  }
}

// Exclusive prefix sum over the 256 threads of the workgroup; total returned in `total`.
__device__ __forceinline__ u32 block_excl_scan(u32 v, u32& total, u32* part) {
  const u32 lane = threadIdx.x & 63u, w = threadIdx.x >> 6;
  u32 inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    u32 t = __shfl_up(inc, o);
    if (lane >= (u32)o) inc += t;
  }
  __syncthreads();
  if (lane == 63u) part[w] = inc;
  __syncthreads();
  u32 base = 0, tot = 0;
#pragma unroll
  for (u32 i = 0; i < BLK_THREADS / WAVE; ++i) {
    u32 s = part[i];
    if (i < w) base += s;
    tot += s;
  }
  total = tot;
  return base + inc - v;
}

// Two exclusive prefix sums at once (one pair of barriers): the values travel as the halves of a 64-bit word.
__device__ __forceinline__ void block_excl_scan2(u32 a, u32 b, u32& off_a, u32& off_b, u32& tot_a, u32& tot_b, u64* part) {
  const u32 lane = threadIdx.x & 63u, w = threadIdx.x >> 6;
  const u64 v = (u64)a | ((u64)b << 32);
  u64 inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const u32 lo = __shfl_up((u32)inc, o), hi = __shfl_up((u32)(inc >> 32), o);
    if (lane >= (u32)o) inc += (u64)lo | ((u64)hi << 32);
  }
  __syncthreads();
  if (lane == 63u) part[w] = inc;
  __syncthreads();
  u64 base = 0, tot = 0;
#pragma unroll
  for (u32 i = 0; i < BLK_THREADS / WAVE; ++i) {
    const u64 s = part[i];
    if (i < w) base += s;
    tot += s;
  }
  const u64 ex = base + inc - v;
  off_a = (u32)ex; off_b = (u32)(ex >> 32);
  tot_a = (u32)tot; tot_b = (u32)(tot >> 32);
}

__device__ __forceinline__ u32 block_max(u32 v, u32* part) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, (u32)__shfl_xor((int)v, o));
  __syncthreads();
  if ((threadIdx.x & 63u) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  u32 m = 0;
#pragma unroll
  for (u32 i = 0; i < BLK_THREADS / WAVE; ++i) m = max(m, part[i]);
  return m;
}

// Maximum of a 64-bit key over the 256 threads of the workgroup (part: 8 x u64 of LDS).
__device__ __forceinline__ u64 block_max64(u64 v, u64* part) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const u64 t = __shfl_xor(v, o);
    v = t > v ? t : v;
  }
  __syncthreads();
  if ((threadIdx.x & 63u) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  u64 m = part[0];
#pragma unroll
  for (u32 i = 1; i < BLK_THREADS / WAVE; ++i) m = part[i] > m ? part[i] : m;
  return m;
}

// Number of leading threads (thread 0 upwards) whose predicate holds.
__device__ __forceinline__ u32 block_prefix_count(bool pred, u32* part) {
  const u32 w = threadIdx.x >> 6;
  unsigned long long b = __ballot(pred);
  u32 cnt = (~b == 0ull) ? 64u : (u32)(__ffsll((long long)~b) - 1);
  __syncthreads();
  if ((threadIdx.x & 63u) == 0) part[w] = cnt;
  __syncthreads();
  u32 tot = 0;
#pragma unroll
  for (u32 i = 0; i < BLK_THREADS / WAVE; ++i) {
    u32 s = part[i];
    tot += s;
    if (s < 64u) break;
  }
  return tot;
}

__device__ __forceinline__ void set_slot_state(SlotStatus* st, u32 state) {
  __hip_atomic_store(&st->state, state, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// One scheduler step. Must be called by all 256 threads of exactly one workgroup.
__device__ void sched_step(const DevCtx& c, SchedShared& sh) {
  const u32 tid = threadIdx.x;
  SchedState* ss = c.ss;

  // ---- window gate -----------------------------------------------------------------------------------
  if (tid == 0) {
    const u64 chain = ss->chains;
    ss->chains = chain + 1;
    sh.chain = chain;
    u32 stop = ss->stopped | ss->error;
    const u64 iter_limit = ss->iter_limit;
    if (iter_limit != 0 && ss->iteration >= iter_limit) stop = 1;
    if (__hip_atomic_load(&c.hctrl->stop, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM)) stop = 1;
    // ---- idle poll: nothing is running, so only a new arrival can give this iteration work. One thread watches the
    // slot of the next ticket (and the stop word) until the slot turns pending or the time allowed has passed; the
    // wait is bounded by the device clock, so the kernel always ends.
    const u32 exit_idle = __hip_atomic_load(&c.hctrl->exit_when_idle, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    sh.exit_idle = exit_idle;
    if (!stop && ss->n_running == 0 && !exit_idle) {
      const u64 t0 = dev_now_ns(), next = ss->next_ticket;
      const u32 slot = (u32)(next & (u64)(c.ring_slots - 1));
      for (;;) {
        if (__hip_atomic_load(&c.status[slot].state, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM) == SLOT_PREFILL_PENDING &&
            __hip_atomic_load(&c.desc[slot].ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == next) break;
        if (__hip_atomic_load(&c.hctrl->stop, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM)) { stop = 1; break; }
        if (dev_now_ns() - t0 >= c.idle_poll_ns) break;
        __builtin_amdgcn_s_sleep(16);
      }
    }
    sh.flag = stop;
  }
  __syncthreads();
  const u64 t_begin = dev_now_ns();   // the scheduling time of the iteration is counted from the end of the idle poll
  if (sh.flag) {
    if (tid == 0) {
      ss->stopped = 1;
      c.meta->skip = 1;
      c.hmirror->iteration = ss->iteration;
      c.hmirror->tokens_out = ss->tokens_out;
      c.hmirror->n_running = ss->n_running;
      c.hmirror->error = ss->error;
      __hip_atomic_store(&c.hmirror->stopped, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    return;
  }

  u32 top = ss->free_top, committed = ss->committed, nrun = ss->n_running;
  const u64 next0 = ss->next_ticket;
  const u32 mbs = c.max_blocks_per_seq;
  const bool pcache = (c.flags & 128u) != 0;
  u32 lo = ss->free_lo, pinned = ss->pinned, hits = 0;
  __syncthreads();

  // ---- (1) retire, batch slot ascending; blocks go back in block-table order ------------------------------
  if (pcache) {
    // prefix caching: the finished requests one at a time (their shared blocks' counts and the order at the bottom of the
    // queue depend on it), the threads over a request's blocks. A private block goes on top; a cached block loses a
    // reference, and one whose count reaches zero goes to the bottom, the request's idle blocks in table order upwards.
    u32 n_fin = 0;
    for (u32 base = 0; base < c.max_batch; base += BLK_THREADS) {
      const u32 b = base + tid;
      const bool fin = b < c.max_batch && c.run[b].valid && c.run[b].finished;
      u32 tot;
      const u32 off = block_excl_scan(fin ? 1u : 0u, tot, sh.wave_part);
      if (fin) sh.seq_bslot[n_fin + off] = b;
      n_fin += tot;
    }
    __syncthreads();
    for (u32 i = 0; i < n_fin; ++i) {
      const u32 b = sh.seq_bslot[i], nb = c.run[b].n_blocks, resv = c.run[b].reserved;
      const u32* bt = c.block_tables + (u64)b * mbs;
      u32 n_idle = 0;
      for (u32 jb = 0; jb < nb; jb += BLK_THREADS) {
        const u32 j = jb + tid;
        const bool v = j < nb;
        const u32 blk = v ? bt[j] : 0u;
        const bool cached = v && (c.pc_flags[blk] & PC_CACHED);
        bool idle = false;
        if (cached) {
          const u32 left = c.pc_ref[blk] - 1;
          c.pc_ref[blk] = left;
          idle = left == 0;
        }
        u32 totp, toti;
        const u32 offp = block_excl_scan((v && !cached) ? 1u : 0u, totp, sh.wave_part);
        const u32 offi = block_excl_scan(idle ? 1u : 0u, toti, sh.wave_part2);
        if (v && !cached) FS(top + offp) = blk;
        if (idle) c.pc_pos[blk] = n_idle + offi;         // its rank among the request's idle blocks, for the second pass
        top += totp;
        n_idle += toti;
      }
      __syncthreads();
      // a cached block of this request's table with no reference left is one this request has just brought to zero (it
      // held a reference until now): its pc_pos holds its rank among them
      for (u32 j = tid; j < nb; j += BLK_THREADS) {
        const u32 blk = bt[j];
        if ((c.pc_flags[blk] & PC_CACHED) && c.pc_ref[blk] == 0) {
          const u32 p = lo - n_idle + c.pc_pos[blk];
          FS(p) = blk;
          c.pc_pos[blk] = p;
        }
      }
      if (tid == 0) c.run[b].valid = 0;
      lo -= n_idle;
      pinned -= n_idle;
      committed -= resv;
      nrun -= 1;
      __syncthreads();
    }
  } else
  for (u32 base = 0; base < c.max_batch; base += BLK_THREADS) {
    const u32 b = base + tid;
    const bool fin = b < c.max_batch && c.run[b].valid && c.run[b].finished;
    const u32 nb = fin ? c.run[b].n_blocks : 0u;
    u32 tot, tot_resv, tot_fin;
    const u32 off = block_excl_scan(nb, tot, sh.wave_part);
    block_excl_scan(fin ? c.run[b].reserved : 0u, tot_resv, sh.wave_part2);
    block_excl_scan(fin ? 1u : 0u, tot_fin, sh.wave_part);
    for (u32 j = 0; j < nb; ++j) FS(top + off + j) = c.block_tables[(u64)b * mbs + j];
    if (fin) c.run[b].valid = 0;
    top += tot;
    committed -= tot_resv;
    nrun -= tot_fin;
  }
  __syncthreads();

  // ---- free batch slots, ascending -----------------------------------------------------------------------
  u32 n_free = 0;
  for (u32 base = 0; base < c.max_batch; base += BLK_THREADS) {
    const u32 b = base + tid;
    const bool fr = b < c.max_batch && !c.run[b].valid;
    u32 tot;
    const u32 off = block_excl_scan(fr ? 1u : 0u, tot, sh.wave_part);
    if (fr) sh.free_list[n_free + off] = b;
    n_free += tot;
  }
  __syncthreads();

  // ---- chunked prefill: the token budget of the iteration goes first to the running requests (one token per decoding
  // request, then the one request that may be part-way through its prompt); admissions take what is left ----------
  const bool chunked = (c.flags & 32u) != 0;
  const u32 budget = c.max_prefill_tokens;
  u32 used = 0, chunk_part = 0;
  if (chunked) {
    u32 n_dec = 0, part_rem = 0;
    for (u32 base = 0; base < c.max_batch; base += BLK_THREADS) {
      const u32 b = base + tid;
      const bool v = b < c.max_batch && c.run[b].valid;
      const u32 rem = v ? c.run[b].P - c.run[b].prefilled : 0u;
      u32 td, tr;
      block_excl_scan(v && rem == 0 ? 1u : 0u, td, sh.wave_part);
      block_excl_scan(rem, tr, sh.wave_part2);       // at most one running request has prompt tokens left
      n_dec += td;
      part_rem += tr;
    }
    chunk_part = min(part_rem, budget - min(budget, n_dec));
    used = n_dec + chunk_part;
    __syncthreads();
  }

  // ---- preemption mode: the preempted requests come back first, lowest ticket first, one at a time (a rare path); the
  // first that does not fit stops every admission behind it. A request fits when a batch slot is free and the blocks of
  // the tokens it prefills (its prompt and what it has generated so far) are free beside those promised before it.
  const bool preempt = (c.flags & 64u) != 0;
  u32 resumed = 0, promised = 0, tokens_admitted = 0, n_pre = preempt ? ss->n_preempted : 0u;
  bool blocked = false;
  while (n_pre > 0 && !blocked) {
    u64 key = 0;                                   // smallest ticket = largest inverted ticket; low bits: the entry's index
    for (u32 i = tid; i < n_pre; i += BLK_THREADS) {
      const u64 k = ((~c.preq[i].ticket) << 12) | i;
      key = k > key ? k : key;
    }
    key = block_max64(key, sh.part64);
    const u32 idx = (u32)(key & 0xFFFu);
    const RunEntry cand = c.preq[idx];
    const u32 ntok = cand.P + cand.gen, need = (ntok + c.bs - 1) / c.bs;
    __syncthreads();                               // everyone has read the entry before it is overwritten below
    if (resumed >= n_free || promised + need > top || (resumed > 0 && (u64)tokens_admitted + ntok > (u64)c.max_prefill_tokens)) {
      blocked = true;
      break;
    }
    if (tid == 0) {
      RunEntry& r = c.run[sh.free_list[resumed]];
      r = cand;
      r.valid = 1;
      r.ctx_len = 0;
      r.n_blocks = 0;
      r.reserved = 0;
      r.in_iter = 1;
      r.prefilled = ntok;
      r.chunk = ntok;
      c.preq[idx] = c.preq[n_pre - 1];             // the last entry fills the hole
    }
    __syncthreads();
    promised += need;
    tokens_admitted += ntok;
    ++resumed;
    --n_pre;
  }

  // ---- (2) poll the ring + (3) admit FCFS, 256 candidate tickets at a time ----------------------------------
  u32 admitted = 0, charged_idle = 0;
  u64 tail = next0;
  u64 first_admitted = 0;
  for (;;) {
    if (blocked) break;                            // a preempted request waits: nobody overtakes it
    const u64 t = next0 + admitted + tid;
    const u32 slot = (u32)(t & (u64)(c.ring_slots - 1));
    bool pend = false;
    u32 P = 0, max_new = 0;
    if (tid < c.ring_slots) {
      const u32 st = __hip_atomic_load(&c.status[slot].state, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
      if (st == SLOT_PREFILL_PENDING) {
        const u64 tk = __hip_atomic_load(&c.desc[slot].ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        pend = tk == t;
      }
    }
    const u32 vis = block_prefix_count(pend, sh.wave_part);
    tail = next0 + admitted + vis;
    const bool cand = tid < vis;
    if (cand) {
      P = __hip_atomic_load(&c.desc[slot].n_prompt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      max_new = __hip_atomic_load(&c.desc[slot].max_new, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    const u32 ord = resumed + admitted + tid;                              // admission order within the iteration
    u32 need = 0;
    if (cand) {
      need = preempt ? (P + c.bs - 1) / c.bs : (P + max_new - 1 + c.bs - 1) / c.bs;   // blocks of the prompt now, or the worst-case reservation
      if (need == 0) need = 1;
    }
    // prefix caching: the candidate walks the keys of its prompt's leading blocks (never the block of the last prompt token)
    // until the first miss; the blocks found go straight into the block table of the batch slot it would take. The table
    // and the reference counts do not change before every admission of the iteration is decided.
    u32 n_match = 0, n_idle_match = 0;
    u64 h_end = PC_H0;
    if (pcache && cand && ord < n_free) {
      u32* bt = c.block_tables + (u64)sh.free_list[ord] * mbs;
      const i32* toks = c.in_arena + (u64)slot * c.max_seq_len;
      for (u32 j = 0; j < (P - 1) / c.bs; ++j) {
        const u64 hj = pc_mix64(h_end ^ pc_block_hash(toks + (u64)j * 16));
        const u32 blk = pc_lookup(c, hj);
        if (blk == ~0u) break;
        bt[j] = blk;
        n_idle_match += c.pc_ref[blk] == 0 ? 1u : 0u;
        h_end = hj;
        ++n_match;
      }
      need -= n_match;                  // its private reservation: the matched blocks are the table's
    }
    const u32 charge = need + n_idle_match;          // a matched block that is idle now becomes a block in use
    const u32 P_new = cand ? P - n_match * c.bs : 0u;  // tokens it computes
    u32 totn, totp, totr;
    const u32 sn = block_excl_scan(charge, totn, sh.wave_part) + charge;     // inclusive
    const u32 sp = block_excl_scan(P_new, totp, sh.wave_part2) + P_new;
    const u32 sr = pcache ? block_excl_scan(need, totr, sh.wave_part) + need : sn;
    // tokens of the budget already spoken for when this candidate's turn comes (chunked mode)
    const u64 before = (u64)used + tokens_admitted + (sp - P_new);
    const bool ok = cand && ord < n_free &&
                    (preempt ? (u64)promised + sn <= (u64)top : (u64)committed + pinned + charged_idle + sn <= (u64)c.n_blocks) &&
                    (chunked ? before < (u64)budget : (ord == 0 || (u64)tokens_admitted + sp <= (u64)c.max_prefill_tokens));
    const u32 adm = block_prefix_count(ok, sh.wave_part);
    if (tid < adm) {
      const u32 b = sh.free_list[ord];
      RunEntry& r = c.run[b];
      r.valid = 1;
      r.ring_slot = slot;
      r.ticket = t;
      r.P = P;
      r.max_new = max_new;
      r.gen = 0;
      r.ctx_len = 0;
      r.reserved = preempt ? 0u : need;
      r.n_blocks = n_match;
      r.n_matched = n_match;
      r.h_end = h_end;
      r.finished = 0;
      r.last_token = -1;
      r.temperature = c.desc[slot].temperature;
      r.top_k = c.desc[slot].top_k;
      r.top_p = c.desc[slot].top_p;
      r.seed = c.desc[slot].seed;
      r.in_iter = 1;
      r.paused = 0;
      r.prefilled = chunked ? 0u : P;       // without chunking the whole prompt is processed in this iteration
      r.chunk = chunked ? (u32)min((u64)P, (u64)budget - before) : P_new;
      // claim by compare-and-swap (section 4.2 "Ring buffer")
      u32 expect = SLOT_PREFILL_PENDING;
      if (!__hip_atomic_compare_exchange_strong(&c.status[slot].state, &expect, SLOT_PREFILL_PROCESSING, __ATOMIC_ACQ_REL,
                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM))
        ss->error = 2;
    }
    // totals of the admitted prefix: broadcast sn/sp of thread adm-1
    __syncthreads();
    if (adm > 0 && tid == adm - 1) {
      sh.wave_part2[0] = sn;
      sh.wave_part2[1] = sp;
      sh.wave_part2[2] = sr;
    }
    __syncthreads();
    if (adm > 0) {
      if (preempt) promised += sh.wave_part2[0];
      else {
        committed += sh.wave_part2[2];                            // the private reservations
        charged_idle += sh.wave_part2[0] - sh.wave_part2[2];      // idle blocks the admitted take into use (counted per candidate)
      }
      tokens_admitted += sh.wave_part2[1];
      if (admitted == 0) first_admitted = next0;
    }
    admitted += adm;
    __syncthreads();
    if (adm < BLK_THREADS) break;   // stopped inside this chunk (nothing pending, or a limit was hit)
  }
  nrun += admitted + resumed;

  // ---- prefix caching: the admitted requests take their matched blocks, in admission order. The threads raise the counts
  // of one request's blocks; a block that was idle leaves the free queue, the queue's top element taking its place (one
  // thread, in block-table order: the arrangement of the queue depends on the order) -------------------------------
  if (pcache) {
    for (u32 i = 0; i < admitted; ++i) {
      const u32 b = sh.free_list[i], m = c.run[b].n_matched;
      const u32* bt = c.block_tables + (u64)b * mbs;
      for (u32 jb = 0; jb < m; jb += BLK_THREADS) {
        const u32 j = jb + tid;
        const bool v = j < m;
        const u32 blk = v ? bt[j] : 0u;
        bool was_idle = false;
        if (v) {
          const u32 r0 = c.pc_ref[blk];
          c.pc_ref[blk] = r0 + 1;
          was_idle = r0 == 0;
        }
        u32 tot;
        const u32 off = block_excl_scan(was_idle ? 1u : 0u, tot, sh.wave_part);
        if (was_idle) sh.seq_tok0[off] = blk;
        __syncthreads();
        if (tid == 0) {
          u32 t = top;
          for (u32 q = 0; q < tot; ++q) {
            const u32 p = c.pc_pos[sh.seq_tok0[q]];
            --t;
            const u32 moved = FS(t);
            FS(p) = moved;
            if (c.pc_flags[moved] & PC_CACHED) c.pc_pos[moved] = p;
          }
        }
        top -= tot;
        pinned += tot;
        __syncthreads();
      }
      hits += m;
    }
  }

  // ---- (4) kind: an iteration with prompt tokens in it counts as a prefill iteration ---------------------------
  const u32 kind = (admitted + resumed > 0 || chunk_part > 0) ? KIND_PREFILL : (nrun > 0 ? KIND_DECODE : KIND_IDLE);
  __syncthreads();

  // ---- preemption mode, decode iteration: when the sequences whose context has filled their blocks need more blocks
  // than are free, the most recently submitted running request (highest ticket) gives up its blocks (back to the stack
  // in block-table order), its batch slot and its place (DECODE_PAUSED), one request at a time until the rest fits ---
  u32 n_preempted_now = 0;
  if (preempt && kind == KIND_DECODE) {
    u32 need_total = 0;
    for (u32 base = 0; base < c.max_batch; base += BLK_THREADS) {
      const u32 b = base + tid;
      u32 tn;
      block_excl_scan((b < c.max_batch && c.run[b].valid && c.run[b].ctx_len == c.run[b].n_blocks * c.bs) ? 1u : 0u, tn, sh.wave_part);
      need_total += tn;
    }
    while (need_total > top && nrun > 1) {
      u64 key = 0;
      for (u32 b = tid; b < c.max_batch; b += BLK_THREADS)
        if (c.run[b].valid) {
          const u64 k = ((c.run[b].ticket + 1) << 12) | b;
          key = k > key ? k : key;
        }
      key = block_max64(key, sh.part64);
      const u32 b = (u32)(key & 0xFFFu);
      const RunEntry v = c.run[b];
      __syncthreads();
      for (u32 j = tid; j < v.n_blocks; j += BLK_THREADS) FS(top + j) = c.block_tables[(u64)b * mbs + j];
      if (tid == 0) {
        RunEntry& q = c.preq[n_pre];
        q = v;
        q.valid = 0;
        q.n_blocks = 0;
        q.ctx_len = 0;
        q.paused = 1;
        c.run[b].valid = 0;
        if (!v.paused) set_slot_state(&c.status[v.ring_slot], SLOT_DECODE_PAUSED);
      }
      __syncthreads();
      top += v.n_blocks;
      need_total -= (v.ctx_len == v.n_blocks * c.bs) ? 1u : 0u;
      ++n_pre;
      --nrun;
      ++n_preempted_now;
    }
    if (need_total > top && tid == 0) ss->error = 3;     // cannot happen: a request that does not fit the pool alone is refused at submission
  }

  // ---- (5) allocate + (6) metadata, batch slot ascending ----------------------------------------------------
  // Sequences of the iteration: without chunking the newly admitted (prefill iteration) or all running (decode
  // iteration); with chunking all running, each with its share of the token budget. A sequence samples a token
  // unless its prompt is still incomplete after this iteration.
  u32 n_seqs = 0, n_tok = 0, n_alloc = 0, n_qt = 0, n_ch = 0, n_smp = 0, n_rows = 0, n_dec_seq = 0, max_q = 0, max_ctx = 0, max_pref = 0;
  u32 n_full = 0, n_part = 0;     // full and partly filled chunks of the decoding sequences so far
  // Work items of the decode attention: chunks of the contexts, or, with at least four sequence x kv-head pairs per
  // compute unit, whole contexts (bit 22 of the tuning word: always; bit 15, or bit 23, the kernel with static items: never).
  // Measured on the llama3_8b shape (8 kv heads, 256 compute units), decode iteration with chunks / whole contexts: 96
  // sequences 10.04 / 10.23 ms, 128: 11.12 / 11.11, 192: 13.62 / 13.22, 256: 14.94 / 14.44 (with few items per compute unit
  // whole contexts of 1 to 10 rounds do not balance; with many, the saved merges and partial results win). From the same
  // count on the launcher runs the kernel chain without the merge kernels, which takes a further 0.1 ms off the whole
  // contexts' side (96 sequences 10.10 / 10.22, 128: 11.22 / 11.12, 144: 12.56 / 12.23).
  const bool group = c.chunk_rec && !(c.tune_nw & 0x808000u) && ((c.tune_nw & 0x400000u) || (u64)nrun * c.nkv >= WHOLE_CONTEXT_PAIRS_PER_CU * (u64)c.n_cu);
  const u32 spec_k = (c.flags & 256u) ? c.spec_k : 0u;
  u64 n_ctx = 0;
  if (kind != KIND_IDLE) {
    for (u32 base = 0; base < c.max_batch; base += BLK_THREADS) {
      const u32 b = base + tid;
      bool in = false, pref = false, smp = false, multi = false;   // multi: several tokens of one sequence attend like a prompt chunk
      u32 nalloc = 0, ntok = 0, pos0 = 0, nb = 0, nrow = 0;
      if (b < c.max_batch && c.run[b].valid) {
        RunEntry& r = c.run[b];
        nb = r.n_blocks;
        if (chunked) {
          in = true;
          pref = r.prefilled < r.P;
          ntok = pref ? (r.in_iter ? r.chunk : chunk_part) : 1u;
          pos0 = pref ? r.prefilled : r.ctx_len;
          smp = !pref || r.prefilled + ntok == r.P;
        } else if (kind == KIND_PREFILL) {
          in = pref = smp = r.in_iter != 0;
          ntok = r.chunk;                     // the prompt; behind a cached prefix, its rest; a resumed request's prompt and outputs
          pos0 = r.P + r.gen - r.chunk;
          if (!in && !r.paused) {
            set_slot_state(&c.status[r.ring_slot], SLOT_DECODE_PAUSED);   // running decodes wait for the prefill
            r.paused = 1;
          }
        } else {
          in = smp = true;
          ntok = 1;
          pos0 = r.ctx_len;
          // speculative decoding: a greedy request also processes its drafts, as many as it may still emit minus one
          if (spec_k && r.temperature == 0.f) ntok += min(c.spec_len[b], r.max_new - r.gen - 1);
        }
        multi = pref || ntok > 1;
        // (a request whose drafts were rejected may already hold the block its next tokens go to)
        if (in) nalloc = max((pos0 + ntok + c.bs - 1) / c.bs, nb) - nb;
        else ntok = 0;
        nrow = smp ? ((spec_k && !pref) ? ntok : 1u) : 0u;    // logits rows: the last token; every token of a decoding sequence when drafts are verified
      }
      u32 tots, tota, tott, totq, totc, totm, totx, totf, totp, totr, totd;
      const u32 ctx_after = in ? pos0 + ntok : 0u;
      const bool dec_seq = in && !multi;
      const u32 nch = !dec_seq ? 0u : group ? 1u : (ctx_after + ATTN_CHUNK_TOKENS - 1) / ATTN_CHUNK_TOKENS;
      const u32 nfull = (!dec_seq || group) ? 0u : ctx_after / ATTN_CHUNK_TOKENS;
      u32 foff, poff, coff, qoff, si, mi, aoff, toff, ri, doff;
      block_excl_scan2(nfull, nch - nfull, foff, poff, totf, totp, sh.part64);
      block_excl_scan2(nch, multi ? (ntok + 15) / 16 : 0u, coff, qoff, totc, totq, sh.part64);
      block_excl_scan2(in ? 1u : 0u, smp ? 1u : 0u, si, mi, tots, totm, sh.part64);
      block_excl_scan2(nalloc, ntok, aoff, toff, tota, tott, sh.part64);
      block_excl_scan2(nrow, (in && !pref) ? 1u : 0u, ri, doff, totr, totd, sh.part64);
      block_excl_scan(ctx_after, totx, sh.wave_part);     // context tokens the attention of this iteration reads
      foff += n_full; poff += n_part; coff += n_ch; qoff += n_qt; si += n_seqs; mi += n_smp; aoff += n_alloc; toff += n_tok; ri += n_rows;
      n_dec_seq += totd;
      if (in) {
        RunEntry& r = c.run[b];
        u32* bt = c.block_tables + (u64)b * mbs;
        for (u32 j = 0; j < nalloc; ++j) {
          const u32 blk = FS(top - 1 - (aoff + j));
          bt[nb + j] = blk;
          if (pcache && (c.pc_flags[blk] & PC_CACHED)) {      // an idle cached block is reused: out of the table (its node goes stale)
            c.pc_flags[blk] = PC_LINKED;
            atomicAdd((unsigned long long*)&ss->evictions, 1ull);
          }
        }
        r.n_blocks = nb + nalloc;
        c.seq_bslot[si] = b;
        c.cu_seqlens[si] = toff;
        c.cu_qtiles[si] = qoff;
        c.cu_chunks[si] = coff;
        c.seq_pos0[si] = pos0;
        c.seq_ring[si] = pref ? r.ring_slot : ~0u;
        c.seq_len[si] = ctx_after;
        if (c.chunk_rec && !group) {      // the decode attention's work list: full chunks first, the partly filled ones behind them
          for (u32 j = 0; j < nch; ++j) {
            ChunkRec rec;
            rec.tok = toff; rec.ctx = ctx_after; rec.bslot = b; rec.ch = j; rec.ci = coff + j; rec.nch = nch;
            rec.b_end = min((ctx_after + 15) / 16, (j + 1) * (u32)(ATTN_CHUNK_TOKENS / 16)); rec.pad1 = 0;
            c.chunk_rec[j < nfull ? foff + j : c.chunk_cap + poff] = rec;
          }
        }
        if (smp) {
          for (u32 j = 0; j < nrow; ++j) c.last_idx[ri + j] = toff + ntok - nrow + j;
          c.sample_bslot[mi] = b;
          if (spec_k) { c.sample_row0[mi] = ri; c.sample_nrow[mi] = nrow; c.sample_tok0[mi] = toff + ntok - nrow; }
        }
        if (!pref) {
          c.input_ids[toff] = r.last_token;
          c.positions[toff] = (i32)pos0;
          c.slot_mapping[toff] = (i32)(bt[pos0 / c.bs] * c.bs + pos0 % c.bs);
          c.tok_seq[toff] = si;
          for (u32 j = 1; j < ntok; ++j) {          // the drafts behind the last token, at the next positions
            const u32 p = pos0 + j;
            c.input_ids[toff + j] = c.spec_tok[(u64)b * SPEC_MAX_DRAFTS + j - 1];
            c.positions[toff + j] = (i32)p;
            c.slot_mapping[toff + j] = (i32)(bt[p / c.bs] * c.bs + p % c.bs);
            c.tok_seq[toff + j] = si;
          }
          if (r.paused) {
            set_slot_state(&c.status[r.ring_slot], SLOT_DECODE_PROCESSING);
            r.paused = 0;
          }
        } else {
          r.prefilled = pos0 + ntok;
          r.in_iter = 0;
        }
        r.ctx_len = ctx_after;
      }
      // (sort key of a decoding sequence: context length, then the lower batch slot first; unique, 0 for no sequence)
      if (group && b < SCHED_MAX_BATCH) { sh.dec_key[b] = (b < c.max_batch && dec_seq) ? (ctx_after << 10) | (1023u - b) : 0u; sh.dec_si[b] = coff; sh.dec_tok[b] = toff; }
      max_q = max(max_q, block_max(ntok, sh.wave_part2));
      max_ctx = max(max_ctx, block_max(ctx_after, sh.wave_part));
      max_pref = max(max_pref, block_max(multi ? ctx_after : 0u, sh.wave_part2));
      n_ctx += totx;
      n_seqs += tots;
      n_alloc += tota;
      n_tok += tott;
      n_qt += totq;
      n_ch += totc;
      n_full += totf;
      n_part += totp;
      n_smp += totm;
      n_rows += totr;
    }
    top -= n_alloc;
    __syncthreads();
    if (group) {
      // whole contexts, longest first: a sequence's place in the list is the number of decoding sequences with a larger
      // key (a longer context, or an equal one in a lower batch slot); sixteen keys per step, read as four 16-byte words
      const u32 strips = (c.max_batch + BLK_THREADS - 1) / BLK_THREADS * BLK_THREADS;      // (keys behind max_batch up to here are 0)
      for (u32 base = 0; base < c.max_batch; base += BLK_THREADS) {
        const u32 b = base + tid;
        const u32 key = b < c.max_batch ? sh.dec_key[b] : 0u;
        if (key) {
          u32 rank = 0;
          for (u32 b2 = 0; b2 < strips; b2 += 16) {
            const uint4 k0 = *(const uint4*)&sh.dec_key[b2], k1 = *(const uint4*)&sh.dec_key[b2 + 4];
            const uint4 k2 = *(const uint4*)&sh.dec_key[b2 + 8], k3 = *(const uint4*)&sh.dec_key[b2 + 12];
            rank += (k0.x > key) + (k0.y > key) + (k0.z > key) + (k0.w > key) + (k1.x > key) + (k1.y > key) + (k1.z > key) + (k1.w > key) +
                    (k2.x > key) + (k2.y > key) + (k2.z > key) + (k2.w > key) + (k3.x > key) + (k3.y > key) + (k3.z > key) + (k3.w > key);
          }
          ChunkRec rec;
          rec.tok = sh.dec_tok[b]; rec.ctx = key >> 10; rec.bslot = b; rec.ch = 0; rec.ci = sh.dec_si[b]; rec.nch = 1;
          rec.b_end = ((key >> 10) + 15) / 16; rec.pad1 = 0;
          c.chunk_rec[rank] = rec;
        }
      }
      n_full = n_ch;      // one item per decoding sequence, all in the first list
      n_part = 0;
    }
    if (tid == 0) {
      c.cu_seqlens[n_seqs] = n_tok;
      c.cu_qtiles[n_seqs] = n_qt;
      c.cu_chunks[n_seqs] = n_ch;
    }
    if (kind == KIND_PREFILL) {
      // token-level metadata of the prompts, threads over all tokens of the iteration: the per-sequence values a token
      // needs are staged in LDS once, a token finds its sequence by binary search there, and four tokens per thread
      // have their loads in flight together
      for (u32 s = tid; s < n_seqs; s += BLK_THREADS) {
        const u32 b = c.seq_bslot[s];
        sh.seq_tok0[s] = c.cu_seqlens[s];
        sh.seq_bslot[s] = b;
        sh.seq_ring[s] = c.seq_ring[s];      // ~0u for a decoding sequence: its one token is already written
        sh.seq_pos0[s] = c.seq_pos0[s];
        sh.seq_P[s] = c.run[b].P;
      }
      __syncthreads();
      for (u32 base = 0; base < n_tok; base += 4 * BLK_THREADS) {
        u32 sq[4], pp[4], blk[4];
        i32 id[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const u32 tk = min(base + u * BLK_THREADS + tid, n_tok - 1);
          u32 lo = 0, hi = n_seqs;              // last s with seq_tok0[s] <= tk
          while (hi - lo > 1) {
            const u32 mid = (lo + hi) / 2;
            if (sh.seq_tok0[mid] <= tk) lo = mid; else hi = mid;
          }
          sq[u] = lo;
          pp[u] = sh.seq_pos0[lo] + (tk - sh.seq_tok0[lo]);       // position in the prompt = in the context
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const u32 ring = sh.seq_ring[sq[u]];
          blk[u] = c.block_tables[(u64)sh.seq_bslot[sq[u]] * mbs + pp[u] / c.bs];
          const u32 rs = ring == ~0u ? 0u : ring, P = sh.seq_P[sq[u]];
          if (ring != ~0u && pp[u] >= P) id[u] = c.out_arena[(u64)rs * c.max_seq_len + (pp[u] - P)].token;
          else id[u] = __hip_atomic_load(c.in_arena + (u64)rs * c.max_seq_len + (ring == ~0u ? 0u : pp[u]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const u32 tk = base + u * BLK_THREADS + tid;
          if (tk < n_tok && sh.seq_ring[sq[u]] != ~0u) {
            c.input_ids[tk] = id[u];
            c.positions[tk] = (i32)pp[u];
            c.slot_mapping[tk] = (i32)(blk[u] * c.bs + pp[u] % c.bs);
            c.tok_seq[tk] = sq[u];
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- prefix caching: the admitted requests enter their own full prompt blocks behind the matched ones into the table,
  // batch slot ascending (a key that is there already, from an earlier request of this very iteration too, leaves the
  // block private). The threads hash a strip of blocks; one thread chains the keys and links the blocks ------------
  if (pcache && kind == KIND_PREFILL) {
    for (u32 s = 0; s < n_seqs; ++s) {
      const u32 b = c.seq_bslot[s];
      const u32 m = c.run[b].n_matched, nfull = c.run[b].P / c.bs;
      const i32* toks = c.in_arena + (u64)c.run[b].ring_slot * c.max_seq_len;
      const u32* bt = c.block_tables + (u64)b * mbs;
      u64 h = c.run[b].h_end;
      for (u32 jb = m; jb < nfull; jb += BLK_THREADS) {
        const u32 cnt = min((u32)BLK_THREADS, nfull - jb);
        if (tid < cnt) sh.pc_g[tid] = pc_block_hash(toks + (u64)(jb + tid) * 16);
        __syncthreads();
        if (tid == 0) {
          u32 n_ins = 0;
          for (u32 q = 0; q < cnt; ++q) {
            h = pc_mix64(h ^ sh.pc_g[q]);
            if (pc_insert(c, bt[jb + q], h)) ++n_ins;
          }
          c.run[b].reserved -= n_ins;
          sh.wave_part[0] = n_ins;
          sh.part64[0] = h;
        }
        __syncthreads();
        committed -= sh.wave_part[0];
        pinned += sh.wave_part[0];
        h = sh.part64[0];
        __syncthreads();
      }
    }
  }

  // ---- write back ------------------------------------------------------------------------------------------
  if (c.attn_ctr)
    for (u32 l = tid; l < c.n_layers; l += BLK_THREADS) c.attn_ctr[l] = 0;     // work counters of this iteration's decode attention launches
  if (tid == 0) {
    const u64 now = dev_now_ns();
    ss->free_top = top;
    ss->free_lo = lo;
    ss->pinned = pinned;
    ss->cache_hits += hits;
    ss->committed = committed;
    ss->n_running = nrun;
    ss->next_ticket = next0 + admitted;
    if (preempt) ss->n_preempted = n_pre;
    IterMeta* m = c.meta;
    m->kind = kind;
    m->skip = 0;
    m->n_seqs = n_seqs;
    m->n_samples = n_rows;
    m->n_sample_seqs = n_smp;
    m->n_full_chunks = n_full;
    m->n_chunks = n_full + n_part;
    m->n_tokens = n_tok;
    m->max_q_len = max_q;
    m->max_ctx = max_ctx;
    m->max_pref_ctx = max_pref;
    u32 stopped = 0;
    if (kind != KIND_IDLE) {
      const u64 it = ss->iteration;
      m->iteration = (u32)it;
      ss->iteration = it + 1;
      if (!spec_k) ss->tokens_out += n_smp;      // (with speculative decoding the sampler counts what it emits)
      ss->idle_since_ns = 0;
      if (kind == KIND_PREFILL) {
        ss->prefill_iterations += 1;
        ss->tokens_prefilled += n_tok - n_dec_seq;
      }
      const u32 ti = (u32)(it % c.trace_cap);
      m->trace_idx = ti;
      if (c.flags & 1u) {
        TraceRec& tr = c.trace[ti];
        tr.iteration = (u32)it;
        tr.kind = kind;
        tr.tail = tail;
        tr.n_admitted = admitted;
        tr.n_seqs = n_seqs;
        tr.n_tokens = n_tok;
        tr.free_blocks = top - lo;
        tr.first_admitted = first_admitted;
        tr.t_sched_begin = t_begin;
        tr.t_sched_end = now;
        tr.t_forward_end = 0;
        tr.t_publish_end = 0;
        tr.ctx_tokens = n_ctx;
        tr.chain = sh.chain;
        tr.n_resumed = resumed;
        tr.n_preempted = n_preempted_now;
      }
    } else {
      if (ss->idle_since_ns == 0) ss->idle_since_ns = now;
      if (sh.exit_idle) {            // exit when idle: nothing running, nothing pending
        ss->stopped = 1;
        stopped = 1;
      }
    }
    c.hmirror->iteration = ss->iteration;
    c.hmirror->tokens_out = ss->tokens_out;
    c.hmirror->n_running = nrun;
    c.hmirror->error = ss->error;
    c.hmirror->idle = kind == KIND_IDLE;
    __hip_atomic_store(&c.hmirror->stopped, stopped, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}
