// On-device sampling and token publication: one workgroup per sequence (section 4.2 of the paper:
// sampling runs inside the step, the scheduler publishes tokens and status to the ring).
// Greedy: largest logit, ties to the lowest id. Otherwise temperature -> top-k -> top-p -> inverse-CDF
// draw with one Philox4x32-10 uniform per output token (key = request seed, counter = output index).
// Candidates are ordered by (logit descending, id ascending) through a composite 64-bit key, selected
// with a radix select over the logits row and sorted in LDS.
#pragma once
#include "blink_device.h"
#include "sched.h"

#define SAMPLER_MAX_K 1024

struct SamplerShared {
  u32 hist[256];
  unsigned long long cand[SAMPLER_MAX_K];
  float cum[SAMPLER_MAX_K];
  unsigned long long red64[4];
  float redf[8];
  u32 misc[8];
};

__device__ __forceinline__ u32 order_key(float f) {   // monotone map float -> u32
  const u32 u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(u32 k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// Visits every element of a logits row once, each thread in ascending index order: f(value, index). 16-byte loads in
// batches of eight per thread; the loads of the next batch are in flight while the current one is consumed (two
// register sets that swap roles by code position).
#define SCAN_LOAD(v, c)                                                                                  \
  _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                                        \
    const u32 idx = (c) + u * (BLK_THREADS * 4) + tid * 4;                                               \
    v[u] = idx < V ? *(const float4*)(row + idx) : make_float4(0.f, 0.f, 0.f, 0.f);                       \
  }
#define SCAN_USE(v, c)                                                                                   \
  _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                                        \
    const u32 idx = (c) + u * (BLK_THREADS * 4) + tid * 4;                                               \
    if (idx < V) { f(v[u].x, idx); f(v[u].y, idx + 1); f(v[u].z, idx + 2); f(v[u].w, idx + 3); }          \
  }
template <typename F>
__device__ __forceinline__ void scan_row(const float* row, u32 V, F f) {
  const u32 tid = threadIdx.x;
  if ((V & 3u) == 0 && ((size_t)row & 15u) == 0) {
    constexpr u32 STEP = BLK_THREADS * 32;
    float4 va[8], vb[8];
    SCAN_LOAD(va, 0u)
    for (u32 c0 = 0; c0 < V; c0 += 2 * STEP) {
      SCAN_LOAD(vb, c0 + STEP)          // past the end of the row every load is switched off
      SCAN_USE(va, c0)
      SCAN_LOAD(va, c0 + 2 * STEP)
      SCAN_USE(vb, c0 + STEP)
    }
  } else {
    for (u32 i = tid; i < V; i += BLK_THREADS) f(row[i], i);
  }
}
#undef SCAN_LOAD
#undef SCAN_USE

// Philox4x32-10 (Salmon et al., SC'11): returns the first output word.
__device__ __forceinline__ u32 philox4x32_10_first(u32 c0, u32 c1, u32 c2, u32 c3, u32 k0, u32 k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const u64 p0 = (u64)0xD2511F53u * c0, p1 = (u64)0xCD9E8D57u * c2;
    const u32 n0 = (u32)(p1 >> 32) ^ c1 ^ k0, n1 = (u32)p1, n2 = (u32)(p0 >> 32) ^ c3 ^ k1, n3 = (u32)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  return c0;
}

__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long t = __shfl_xor(v, o);
    v = t > v ? t : v;
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long m = red[0];
#pragma unroll
  for (int i = 1; i < 4; ++i) m = red[i] > m ? red[i] : m;
  return m;
}

// One radix-select digit: among the items whose composite key matches `prefix` on the bits above
// `shift + 8`, find the digit (8 bits at `shift`) that holds the k_rem-th largest; updates prefix, k_rem.
// Composite key = (order_key(logit) << 32) | ~id.
__device__ __forceinline__ void radix_digit(const float* row, u32 V, int shift, unsigned long long& prefix, u32& k_rem,
                                            SamplerShared& sh) {
  const u32 tid = threadIdx.x;
  __syncthreads();
  sh.hist[tid] = 0;
  __syncthreads();
  const unsigned long long himask = shift + 8 >= 64 ? 0ull : (~0ull << (shift + 8));
  scan_row(row, V, [&](float val, u32 i) {
    const unsigned long long key = ((unsigned long long)order_key(val) << 32) | (u32)~i;
    if ((key & himask) == (prefix & himask)) atomicAdd(&sh.hist[(u32)(key >> shift) & 255u], 1u);
  });
  __syncthreads();
  if (tid == 0) {
    u32 rem = k_rem, digit = 0;
    for (int b = 255; b >= 0; --b) {
      const u32 cnt = sh.hist[b];
      if (cnt >= rem) { digit = (u32)b; break; }
      rem -= cnt;
    }
    sh.misc[0] = digit;
    sh.misc[1] = rem;
  }
  __syncthreads();
  prefix |= (unsigned long long)sh.misc[0] << shift;
  k_rem = sh.misc[1];
}

// Bitonic sort of n (a power of two) 64-bit keys in LDS, descending; all 256 threads.
__device__ __forceinline__ void bitonic_sort_desc(unsigned long long* v, u32 n) {
  const u32 tid = threadIdx.x;
  for (u32 size = 2; size <= n; size <<= 1) {
    for (u32 stride = size >> 1; stride > 0; stride >>= 1) {
      for (u32 i = tid; i < n / 2; i += BLK_THREADS) {
        const u32 lo = (i / stride) * stride * 2 + (i % stride), hi = lo + stride;
        const bool desc = ((lo & size) == 0);
        const unsigned long long a = v[lo], b = v[hi];
        if ((a < b) == desc) { v[lo] = b; v[hi] = a; }
      }
      __syncthreads();
    }
  }
}

// Leaves the k largest composite keys (order_key(logit) << 32 | ~id) of the row in sh.cand[0..k), descending, the
// rest of sh.cand[0..npow) holding smaller keys or zero padding. Returns npow (a power of two >= k).
__device__ __forceinline__ u32 select_top_k(const float* row, u32 V, u32 k, SamplerShared& sh) {
  const u32 tid = threadIdx.x;
  // (1) One pass: every thread keeps the four largest keys among the elements it visits and the largest logit it
  // dropped. The 1024 kept keys are sorted; their k-th largest is the exact threshold unless some thread dropped
  // a logit at or above its logit (a tie with the threshold's logit goes to the exact stages below).
  if (k <= 256) {
    // Sorted by (logit descending, id ascending): a thread meets its ids in ascending order, so among equal logits the
    // one it holds already comes first, and a strict comparison of the 32-bit logit keys decides every insertion. No
    // branches: key and id move down the four places through selects.
    u32 q0 = 0, q1 = 0, q2 = 0, q3 = 0, i0 = 0, i1 = 0, i2 = 0, i3 = 0, dropped = 0;
    scan_row(row, V, [&](float val, u32 i) {
      u32 xk = order_key(val), xi = i;
#define TOPK_PLACE(q, id) { const bool c = xk > q; const u32 hk = c ? xk : q, hi = c ? xi : id; xk = c ? q : xk; xi = c ? id : xi; q = hk; id = hi; }
      TOPK_PLACE(q0, i0) TOPK_PLACE(q1, i1) TOPK_PLACE(q2, i2) TOPK_PLACE(q3, i3)
#undef TOPK_PLACE
      dropped = max(dropped, xk);      // the logit key of whatever fell out at the bottom
    });
    __syncthreads();
    sh.cand[tid * 4] = q0 ? ((unsigned long long)q0 << 32) | (u32)~i0 : 0ull;
    sh.cand[tid * 4 + 1] = q1 ? ((unsigned long long)q1 << 32) | (u32)~i1 : 0ull;
    sh.cand[tid * 4 + 2] = q2 ? ((unsigned long long)q2 << 32) | (u32)~i2 : 0ull;
    sh.cand[tid * 4 + 3] = q3 ? ((unsigned long long)q3 << 32) | (u32)~i3 : 0ull;
    __syncthreads();
    bitonic_sort_desc(sh.cand, SAMPLER_MAX_K);
    const u32 thr = (u32)(sh.cand[k - 1] >> 32);
    const u32 worst = block_max(dropped, sh.misc);
    if (worst < thr) return SAMPLER_MAX_K;      // every dropped logit lies strictly below the k-th kept one
  }
  // (2) Counting search for a key `lo` with k <= f(lo) <= SAMPLER_MAX_K, f(p) = #{key >= p} (non-increasing in p):
  // start at the row maximum, double the distance below it until k keys are covered, bisect if too many are.
  u32 kmax = 0;
  scan_row(row, V, [&](float val, u32) { kmax = max(kmax, order_key(val)); });
  kmax = block_max(kmax, sh.misc);
  u32 lo = 0, cnt = 0;
  bool found = false;
  {
    u32 few = kmax, many = 0, step = 1u << 18;   // `few`: a probe with f < k; `many`: one with f > SAMPLER_MAX_K
    bool have_many = false, few_is_open = true;
    for (int pass = 0; pass < 64 && !found; ++pass) {
      u32 probe;
      if (pass == 0) probe = kmax;
      else if (!have_many) { probe = few > step ? few - step : 0u; step = step < (1u << 30) ? step << 1 : step; }
      else { if (few - many <= 1) break; probe = many + (few - many) / 2; }
      u32 local = 0;
      scan_row(row, V, [&](float val, u32) { local += order_key(val) >= probe ? 1u : 0u; });
      u32 total;
      block_excl_scan(local, total, sh.misc);
      if (total < k) { few = probe; few_is_open = false; if (probe == 0) break; }
      else if (total <= SAMPLER_MAX_K) { lo = probe; cnt = total; found = true; }
      else { many = probe; have_many = true; if (few_is_open) break; }
    }
  }
  unsigned long long prefix;
  if (found) {
    prefix = (unsigned long long)lo << 32;      // every (key, id) with key >= lo is a candidate
  } else {                                      // (3) massive ties: exact radix select on the composite key
    prefix = 0;
    u32 k_rem = k;
    for (int shift = 56; shift >= 32; shift -= 8) radix_digit(row, V, shift, prefix, k_rem, sh);
    prefix |= 0xFF000000ull;                    // ids are below 2^24: the top byte of ~id is 0xFF for every item
    for (int shift = 16; shift >= 0; shift -= 8) radix_digit(row, V, shift, prefix, k_rem, sh);
    cnt = k;
  }
  __syncthreads();
  if (tid == 0) sh.misc[2] = 0;
  __syncthreads();
  scan_row(row, V, [&](float val, u32 i) {
    const unsigned long long key = ((unsigned long long)order_key(val) << 32) | (u32)~i;
    if (key >= prefix) {
      const u32 p = atomicAdd(&sh.misc[2], 1u);
      if (p < SAMPLER_MAX_K) sh.cand[p] = key;
    }
  });
  __syncthreads();
  u32 npow = 1;
  while (npow < cnt) npow <<= 1;
  for (u32 i = cnt + tid; i < npow; i += BLK_THREADS) sh.cand[i] = 0ull;   // padding sorts to the end
  __syncthreads();
  bitonic_sort_desc(sh.cand, npow);
  return npow;
}

// Next token of one logits row; all 256 threads of the workgroup take part and all return the token.
// gen: index of the output token being sampled (the Philox counter).
__device__ __forceinline__ i32 sample_row(const float* row, u32 V, float temperature, u32 top_k, float top_p, u64 seed, u32 gen,
                                          SamplerShared& sh) {
  const u32 tid = threadIdx.x;
  if (temperature == 0.f) {
    unsigned long long best = 0;
    scan_row(row, V, [&](float val, u32 i) {
      const unsigned long long key = ((unsigned long long)order_key(val) << 32) | (u32)~i;
      best = key > best ? key : best;
    });
    best = block_max_u64(best, sh.red64);
    return (i32)(~(u32)best);
  }
  u32 k = top_k == 0 || top_k > V ? V : top_k;
  if (k > SAMPLER_MAX_K) k = SAMPLER_MAX_K;   // the entry points reject what does not fit; defensive clamp
  const u32 npow = select_top_k(row, V, k, sh);   // sh.cand[0..k) = the k largest (logit, then lower id) in order
  // softmax numerators of the kept candidates at temperature T, cumulative sums in candidate order
  const float invT = 1.0f / temperature;
  const float zmax = key_to_float((u32)(sh.cand[0] >> 32)) * invT;
  const u32 per = (npow + BLK_THREADS - 1) / BLK_THREADS;   // consecutive candidates per thread
  float local[SAMPLER_MAX_K / BLK_THREADS];
  float run_sum = 0.f;
#pragma unroll
  for (u32 j = 0; j < SAMPLER_MAX_K / BLK_THREADS; ++j) {
    const u32 i = tid * per + j;
    float p = 0.f;
    if (j < per && i < k) p = __expf(key_to_float((u32)(sh.cand[i] >> 32)) * invT - zmax);
    run_sum += p;
    local[j] = run_sum;
  }
  // exclusive scan of the per-thread sums (fixed order)
  float inc = run_sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float t = __shfl_up(inc, o);
    if ((tid & 63u) >= (u32)o) inc += t;
  }
  __syncthreads();
  if ((tid & 63u) == 63u) sh.redf[tid >> 6] = inc;
  __syncthreads();
  float base = inc - run_sum;
  for (u32 w = 0; w < (tid >> 6); ++w) base += sh.redf[w];
#pragma unroll
  for (u32 j = 0; j < SAMPLER_MAX_K / BLK_THREADS; ++j) {
    const u32 i = tid * per + j;
    if (j < per && i < npow) sh.cum[i] = base + local[j];
  }
  __syncthreads();
  if (tid == 0) {
    const float total = sh.cum[k - 1];
    const float thr = top_p * total;
    // shortest prefix reaching top_p: binary search for the first cum >= thr
    u32 lo = 0, hi = k - 1;
    while (lo < hi) {
      const u32 mid = (lo + hi) / 2;
      if (sh.cum[mid] >= thr) hi = mid; else lo = mid + 1;
    }
    const u32 n_keep = lo + 1;
    const u32 x0 = philox4x32_10_first(gen, 0u, 0u, 0u, (u32)seed, (u32)(seed >> 32));
    const float u = (float)(x0 >> 8) * (1.0f / 16777216.0f);
    const float target = u * sh.cum[n_keep - 1];
    lo = 0; hi = n_keep - 1;
    while (lo < hi) {   // first cum > target
      const u32 mid = (lo + hi) / 2;
      if (sh.cum[mid] > target) hi = mid; else lo = mid + 1;
    }
    sh.misc[3] = ~(u32)sh.cand[lo];
  }
  __syncthreads();
  const i32 token = (i32)sh.misc[3];
  __syncthreads();   // sh.misc is free for the next row
  return token;
}

__device__ __forceinline__ void phase_sample_publish(const DevCtx& c, SamplerShared& sh, u32 wg, u32 nwg) {
  const IterMeta* meta = c.meta;
  const u32 n_seqs = meta->n_samples, V = c.V, tid = threadIdx.x;      // the sequences that sample in this iteration
  if (wg == 0 && tid == 0 && (c.flags & 1u)) c.trace[meta->trace_idx].t_forward_end = dev_now_ns();
  for (u32 s = wg; s < n_seqs; s += nwg) {
    const u32 b = c.sample_bslot[s];
    RunEntry& r = c.run[b];
    const i32 token = sample_row(c.logits + (u64)s * V, V, r.temperature, r.top_k, r.top_p, r.seed, r.gen, sh);
    // ---- publish (section 4.2: tokens and status go back to the ring) ------------------------------------
    if (tid == 0) {
      const u32 idx = r.gen;
      const u32 slot = r.ring_slot;
      OutRec* o = c.out_arena + (u64)slot * c.max_seq_len + idx;
      o->token = token;
      o->iteration = meta->iteration;
      o->device_ns = dev_now_ns();
      r.gen = idx + 1;
      r.last_token = token;
      r.paused = 0;             // the status word written below says PROCESSING or COMPLETED (a resumed request was PAUSED until now)
      const bool done = (idx + 1 == r.max_new) || (token == c.eos);
      u32 state = SLOT_DECODE_PROCESSING;
      if (done) {
        r.finished = 1;
        state = SLOT_DECODE_COMPLETED;
      }
      __threadfence_system();
      // state and generation count are published together as one 64-bit word
      const u64 word = (u64)state | ((u64)(idx + 1) << 32);
      __hip_atomic_store((u64*)&c.status[slot], word, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    __syncthreads();
  }
  if (wg == 0 && tid == 0 && (c.flags & 1u)) c.trace[meta->trace_idx].t_publish_end = dev_now_ns();
}

// Speculative decoding: a sequence has one logits row per token it was fed (its last token, then its drafts). One workgroup
// walks the rows of a sequence in order: row j gives the token of output index gen + j, which is emitted; the walk goes on
// only while the token equals the draft fed at the next position and the request has not finished. What is emitted is what
// one-token-per-iteration decoding emits; the cache entries of rejected drafts lie beyond the context length afterwards.
__device__ __forceinline__ void phase_sample_publish_spec(const DevCtx& c, SamplerShared& sh, u32 wg, u32 nwg) {
  const IterMeta* meta = c.meta;
  const u32 V = c.V, tid = threadIdx.x;
  if (wg == 0 && tid == 0 && (c.flags & 1u)) c.trace[meta->trace_idx].t_forward_end = dev_now_ns();
  for (u32 s = wg; s < meta->n_sample_seqs; s += nwg) {
    const u32 b = c.sample_bslot[s], row0 = c.sample_row0[s], nrow = c.sample_nrow[s], tok0 = c.sample_tok0[s];
    RunEntry& r = c.run[b];
    const u32 idx0 = r.gen, slot = r.ring_slot, max_new = r.max_new;
    const float temperature = r.temperature, top_p = r.top_p;
    const u32 top_k = r.top_k;
    const u64 seed = r.seed;
    u32 emitted = 0;
    i32 last = -1;
    bool done = false;
    for (u32 j = 0; j < nrow; ++j) {
      const i32 token = sample_row(c.logits + (u64)(row0 + j) * V, V, temperature, top_k, top_p, seed, idx0 + j, sh);
      if (tid == 0) {
        OutRec* o = c.out_arena + (u64)slot * c.max_seq_len + idx0 + j;
        o->token = token;
        o->iteration = meta->iteration;
        o->device_ns = dev_now_ns();
      }
      ++emitted;
      last = token;
      done = (idx0 + emitted == max_new) || (token == c.eos);
      if (done || j + 1 == nrow || token != c.input_ids[tok0 + j + 1]) break;
    }
    if (tid == 0) {
      r.gen = idx0 + emitted;
      r.last_token = last;
      r.paused = 0;
      r.ctx_len -= nrow - emitted;            // the scheduler counted every fed token; the rejected drafts' entries are dead
      u32 state = SLOT_DECODE_PROCESSING;
      if (done) {
        r.finished = 1;
        state = SLOT_DECODE_COMPLETED;
      }
      atomicAdd((unsigned long long*)&c.ss->tokens_out, (unsigned long long)emitted);
      if (nrow > 1) {
        atomicAdd((unsigned long long*)&c.ss->drafted, (unsigned long long)(nrow - 1));
        atomicAdd((unsigned long long*)&c.ss->accepted, (unsigned long long)(emitted - 1));
      }
      __threadfence_system();
      const u64 word = (u64)state | ((u64)(idx0 + emitted) << 32);
      __hip_atomic_store((u64*)&c.status[slot], word, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    __syncthreads();
  }
  if (wg == 0 && tid == 0 && (c.flags & 1u)) c.trace[meta->trace_idx].t_publish_end = dev_now_ns();
}

// Stand-alone sampling of a batch of logits rows (no engine): one workgroup per row, grid-stride.
struct SampleRowParams {   // the layout of blink_sampling (24 bytes)
  float temperature;
  u32 top_k;
  float top_p;
  u32 pad;
  u64 seed;
};
__device__ __forceinline__ void sample_rows(const float* logits, u32 n_rows, u32 V, const SampleRowParams* params, const u32* token_index,
                                            i32* tokens, SamplerShared& sh) {
  for (u32 r = blockIdx.x; r < n_rows; r += gridDim.x) {
    const SampleRowParams p = params[r];
    const i32 token = sample_row(logits + (u64)r * V, V, p.temperature, p.top_k, p.top_p, p.seed, token_index[r], sh);
    if (threadIdx.x == 0) tokens[r] = token;
  }
}
