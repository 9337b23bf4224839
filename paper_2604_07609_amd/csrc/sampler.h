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
  for (u32 i = tid; i < V; i += BLK_THREADS) {
    const unsigned long long key = ((unsigned long long)order_key(row[i]) << 32) | (u32)~i;
    if ((key & himask) == (prefix & himask)) atomicAdd(&sh.hist[(u32)(key >> shift) & 255u], 1u);
  }
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

__device__ void phase_sample_publish(const DevCtx& c, SamplerShared& sh, u32 wg, u32 nwg) {
  const IterMeta* meta = c.meta;
  const u32 n_seqs = meta->n_seqs, V = c.V, tid = threadIdx.x;
  if (wg == 0 && tid == 0 && (c.flags & 1u)) c.trace[meta->trace_idx].t_forward_end = dev_now_ns();
  for (u32 s = wg; s < n_seqs; s += nwg) {
    const u32 b = c.seq_bslot[s];
    RunEntry& r = c.run[b];
    const float* row = c.logits + (u64)s * V;
    i32 token;
    if (r.temperature == 0.f) {
      unsigned long long best = 0;
      for (u32 i = tid; i < V; i += BLK_THREADS) {
        const unsigned long long key = ((unsigned long long)order_key(row[i]) << 32) | (u32)~i;
        best = key > best ? key : best;
      }
      best = block_max_u64(best, sh.red64);
      token = (i32)(~(u32)best);
    } else {
      u32 k = r.top_k == 0 || r.top_k > V ? V : r.top_k;
      if (k > SAMPLER_MAX_K) k = SAMPLER_MAX_K;   // submit rejects what does not fit; defensive clamp
      // threshold composite key of the k-th largest candidate
      unsigned long long prefix = 0;
      u32 k_rem = k;
      for (int shift = 56; shift >= 32; shift -= 8) radix_digit(row, V, shift, prefix, k_rem, sh);
      // ids below 2^24: the low word is ~id, its top byte is 0xFF for every item
      prefix |= 0xFF000000ull;
      for (int shift = 16; shift >= 0; shift -= 8) radix_digit(row, V, shift, prefix, k_rem, sh);
      // gather the k items with composite key >= threshold
      __syncthreads();
      if (tid == 0) sh.misc[2] = 0;
      __syncthreads();
      for (u32 i = tid; i < V; i += BLK_THREADS) {
        const unsigned long long key = ((unsigned long long)order_key(row[i]) << 32) | (u32)~i;
        if (key >= prefix) {
          const u32 p = atomicAdd(&sh.misc[2], 1u);
          if (p < SAMPLER_MAX_K) sh.cand[p] = key;
        }
      }
      __syncthreads();
      u32 npow = 1;
      while (npow < k) npow <<= 1;
      for (u32 i = k + tid; i < npow; i += BLK_THREADS) sh.cand[i] = 0ull;   // pads sort to the end
      __syncthreads();
      // bitonic sort, descending
      for (u32 size = 2; size <= npow; size <<= 1) {
        for (u32 stride = size >> 1; stride > 0; stride >>= 1) {
          for (u32 i = tid; i < npow / 2; i += BLK_THREADS) {
            const u32 lo = (i / stride) * stride * 2 + (i % stride), hi = lo + stride;
            const bool desc = ((lo & size) == 0);
            const unsigned long long a = sh.cand[lo], bb = sh.cand[hi];
            if ((a < bb) == desc) { sh.cand[lo] = bb; sh.cand[hi] = a; }
          }
          __syncthreads();
        }
      }
      // softmax numerators of the kept candidates at temperature T, cumulative sums in candidate order
      const float invT = 1.0f / r.temperature;
      const float zmax = key_to_float((u32)(sh.cand[0] >> 32)) * invT;
      const u32 per = (npow + BLK_THREADS - 1) / BLK_THREADS;   // consecutive candidates per thread
      float local[SAMPLER_MAX_K / BLK_THREADS];
      float run_sum = 0.f;
      for (u32 j = 0; j < per; ++j) {
        const u32 i = tid * per + j;
        float p = 0.f;
        if (i < k) p = __expf(key_to_float((u32)(sh.cand[i] >> 32)) * invT - zmax);
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
      for (u32 j = 0; j < per; ++j) {
        const u32 i = tid * per + j;
        if (i < npow) sh.cum[i] = base + local[j];
      }
      __syncthreads();
      if (tid == 0) {
        const float total = sh.cum[k - 1];
        const float thr = r.top_p * total;
        // shortest prefix reaching top_p: binary search for the first cum >= thr
        u32 lo = 0, hi = k - 1;
        while (lo < hi) {
          const u32 mid = (lo + hi) / 2;
          if (sh.cum[mid] >= thr) hi = mid; else lo = mid + 1;
        }
        const u32 n_keep = lo + 1;
        const u32 x0 = philox4x32_10_first(r.gen, 0u, 0u, 0u, (u32)r.seed, (u32)(r.seed >> 32));
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
      token = (i32)sh.misc[3];
    }
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
