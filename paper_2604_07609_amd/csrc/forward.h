// Forward pass of the Llama-style decoder over paged KV: generic phases (fp32 weights, and the
// reference-quality path for bf16 weights). Each phase is a device function that loops over its work
// items with a workgroup stride, reading the batch shape from the device-resident metadata, so the
// same code runs from a host-enqueued kernel sequence and from the resident loop kernel. The model is
// the decoder that the paper's engine treats as opaque (section 4.3); shapes come from the workloads.
#pragma once
#include "blink_device.h"

template <typename WT> struct WLoad;
template <> struct WLoad<float> {
  static __device__ __forceinline__ float get(const float* p, u64 i) { return p[i]; }
  static __device__ __forceinline__ void load8(const float* p, float* o) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
  static __device__ __forceinline__ void put(float* p, u64 i, float v) { p[i] = v; }
};
template <> struct WLoad<bf16_t> {
  static __device__ __forceinline__ float get(const bf16_t* p, u64 i) { return bf16_to_f32(p[i]); }
  static __device__ __forceinline__ void load8(const bf16_t* p, float* o) {
    const uint4 a = *(const uint4*)p;
    const u32 w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void put(bf16_t* p, u64 i, float v) { p[i] = f32_to_bf16(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
// Sum over the workgroup in a fixed order (waves 0..3); red: 4 floats of LDS.
__device__ __forceinline__ float block_sum_f(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}
__device__ __forceinline__ float block_max_f(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__device__ __forceinline__ u64 packed_act_off(u32 t, u32 k, u32 TBS) {   // same layout as mfma_gemm.h
  return ((u64)((k >> 5) * TBS + (t >> 4)) * 64 + (t & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

// ---- embedding gather: x[t] = E[input_ids[t]] ---------------------------------------------------------------
template <typename WT>
__device__ __forceinline__ void phase_embed(const DevCtx& c, u32 wg, u32 nwg) {
  const u32 T = c.meta->n_tokens, d = c.d;
  const WT* E = (const WT*)c.embed;
  const u32 per_row = d / 8;
  for (u64 i = (u64)wg * BLK_THREADS + threadIdx.x; i < (u64)T * per_row; i += (u64)nwg * BLK_THREADS) {
    const u32 t = (u32)(i / per_row), j = (u32)(i % per_row) * 8;
    float v[8];
    WLoad<WT>::load8(E + (u64)c.input_ids[t] * d + j, v);
    float* o = c.x + (u64)t * d + j;
    *(float4*)o = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
}

// ---- embedding gather of the bf16 path: residual stream, packed operand of the first GEMM (x * g1 of layer 0)
// and the partial sums of squares its RMSNorm needs; one thread per (token, 16 columns) --------------------------
__device__ __forceinline__ void phase_embed_packed(const DevCtx& c, u32 wg, u32 nwg) {
  const u32 T = c.meta->n_tokens, d = c.d, per_row = d / 16;
  const bf16_t* E = (const bf16_t*)c.embed;
  const float* g = c.layers[0].g1;
  for (u64 i = (u64)wg * BLK_THREADS + threadIdx.x; i < (u64)T * per_row; i += (u64)nwg * BLK_THREADS) {
    const u32 t = (u32)(i / per_row), nt = (u32)(i % per_row), k0 = nt * 16;
    float v[16];
    WLoad<bf16_t>::load8(E + (u64)c.input_ids[t] * d + k0, v);
    WLoad<bf16_t>::load8(E + (u64)c.input_ids[t] * d + k0 + 8, v + 8);
    float* o = c.x + (u64)t * d + k0;
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) *(float4*)(o + 4 * j) = make_float4(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      u32 w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a = v[8 * h + 2 * j], b = v[8 * h + 2 * j + 1];
        ss += a * a + b * b;
        w[j] = pack_f16x2(a * g[k0 + 8 * h + 2 * j], b * g[k0 + 8 * h + 2 * j + 1]);
      }
      *(uint4*)(c.xq + packed_act_off(t, k0 + 8 * h, c.TBS)) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    c.ssq[(u64)t * per_row + nt] = ss;
  }
}

// ---- RMSNorm: out[r] = in[row(r)] * g / sqrt(mean(in^2) + eps); one workgroup per row -------------------------
// rows == nullptr: row(r) = r, n_rows = n_tokens; else row(r) = rows[r], n_rows = sampling sequences (their last positions).
__device__ __forceinline__ void phase_rmsnorm(const DevCtx& c, const float* in, const float* g, float* out, const u32* rows, float* red,
                              u32 wg, u32 nwg) {
  const u32 n = rows ? c.meta->n_samples : c.meta->n_tokens, d = c.d;
  for (u32 r = wg; r < n; r += nwg) {
    const float* x = in + (u64)(rows ? rows[r] : r) * d;
    float ss = 0.f;
    for (u32 j = threadIdx.x; j < d; j += BLK_THREADS) ss += x[j] * x[j];
    ss = block_sum_f(ss, red);
    const float rstd = 1.0f / sqrtf(ss / (float)d + c.eps);
    for (u32 j = threadIdx.x; j < d; j += BLK_THREADS) out[(u64)r * d + j] = x[j] * rstd * g[j];
  }
}

// ---- generic GEMM: out[t][n] (+)= sum_k a(t,k) * W[n][k] ---------------------------------------------------------
// 32 x 64 output tile per workgroup, K in steps of 32 through LDS, 2 x 4 outputs per thread, fp32 FMA.
#define GA_PLAIN 0
#define GA_SILU_MUL 1   // a(t,k) = silu(A[t][k]) * A[t][K + k]   (A has 2K columns: gate | up)
#define GE_STORE 0
#define GE_ADD 1        // out += result (residual connection, in place)
#define G_BM 32
#define G_BN 64
#define G_BK 32
struct GemmShared {
  float As[G_BK][G_BM + 1];
  float Ws[G_BK][G_BN + 4];
};

template <typename WT, int AMODE, int EMODE>
__device__ __forceinline__ void phase_gemm(const float* A, u32 lda, const WT* W, float* out, u32 ldo, u32 T, u32 N, u32 K, GemmShared& sh,
                           u32 wg, u32 nwg) {
  const u32 tid = threadIdx.x;
  const u32 mt = (T + G_BM - 1) / G_BM, nt = (N + G_BN - 1) / G_BN;
  const u32 tm = tid / 16, tn = tid % 16;
  for (u32 tile = wg; tile < mt * nt; tile += nwg) {
    const u32 t0 = (tile % mt) * G_BM, n0 = (tile / mt) * G_BN;
    float acc[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    for (u32 k0 = 0; k0 < K; k0 += G_BK) {
      {  // A tile: thread -> row tid/8, 4 consecutive k
        const u32 r = tid / 8, kk = (tid % 8) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (t0 + r < T) {
          const float* ap = A + (u64)(t0 + r) * lda + k0 + kk;
          v = *(const float4*)ap;
          if (AMODE == GA_SILU_MUL) {
            const float4 u = *(const float4*)(ap + K);
            v.x = v.x / (1.f + __expf(-v.x)) * u.x;
            v.y = v.y / (1.f + __expf(-v.y)) * u.y;
            v.z = v.z / (1.f + __expf(-v.z)) * u.z;
            v.w = v.w / (1.f + __expf(-v.w)) * u.w;
          }
        }
        sh.As[kk][r] = v.x; sh.As[kk + 1][r] = v.y; sh.As[kk + 2][r] = v.z; sh.As[kk + 3][r] = v.w;
      }
      {  // W tile: thread -> row tid/4, 8 consecutive k
        const u32 r = tid / 4, kk = (tid % 4) * 8;
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (n0 + r < N) WLoad<WT>::load8(W + (u64)(n0 + r) * K + k0 + kk, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) sh.Ws[kk + i][r] = v[i];
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < G_BK; ++k) {
        const float a0 = sh.As[k][tm * 2], a1 = sh.As[k][tm * 2 + 1];
        const float4 w = *(const float4*)&sh.Ws[k][tn * 4];
        acc[0][0] += a0 * w.x; acc[0][1] += a0 * w.y; acc[0][2] += a0 * w.z; acc[0][3] += a0 * w.w;
        acc[1][0] += a1 * w.x; acc[1][1] += a1 * w.y; acc[1][2] += a1 * w.z; acc[1][3] += a1 * w.w;
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const u32 t = t0 + tm * 2 + i;
      if (t >= T) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32 n = n0 + tn * 4 + j;
        if (n >= N) continue;
        float* o = out + (u64)t * ldo + n;
        if (EMODE == GE_ADD) *o += acc[i][j]; else *o = acc[i][j];
      }
    }
  }
}

// ---- rotary embedding on q and k (rotate-half pairing), K/V write through the slot mapping --------------------
template <typename WT>
__device__ __forceinline__ void phase_rope_kvwrite(const DevCtx& c, u32 layer, u32 wg, u32 nwg) {
  const u32 T = c.meta->n_tokens, hd = c.hd, half = hd / 2, nh = c.nq + 2 * c.nkv;
  WT* Kc = (WT*)c.kv + (u64)layer * c.kv_layer_stride;
  WT* Vc = Kc + c.kv_kv_stride;
  const u64 total = (u64)T * nh * half;
  for (u64 i = (u64)wg * BLK_THREADS + threadIdx.x; i < total; i += (u64)nwg * BLK_THREADS) {
    const u32 p = (u32)(i % half), hh = (u32)((i / half) % nh), t = (u32)(i / ((u64)half * nh));
    float* q = c.qkv + (u64)t * c.qkv_n + (u64)hh * hd;
    const float a = q[p], b = q[p + half];
    if (hh < c.nq + c.nkv) {
      const float2 cs = c.rope_tab[(u64)c.positions[t] * half + p];
      const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
      if (hh < c.nq) {
        q[p] = ra;
        q[p + half] = rb;
      } else {
        const u32 slot = (u32)c.slot_mapping[t], g = hh - c.nq;
        const u64 o = (((u64)(slot / c.bs) * c.nkv + g) * c.bs + slot % c.bs) * hd;
        WLoad<WT>::put(Kc, o + p, ra);
        WLoad<WT>::put(Kc, o + p + half, rb);
      }
    } else {
      const u32 slot = (u32)c.slot_mapping[t], g = hh - c.nq - c.nkv;
      const u64 o = (((u64)(slot / c.bs) * c.nkv + g) * c.bs + slot % c.bs) * hd;
      WLoad<WT>::put(Vc, o + p, a);
      WLoad<WT>::put(Vc, o + p + half, b);
    }
  }
}

// ---- generic paged attention: one workgroup per (token, kv head); online softmax over chunks of 256 keys ------
#define ATT_MAX_G 8
struct AttnShared {
  float q[ATT_MAX_G][128];
  float p[ATT_MAX_G][BLK_THREADS];
  float red[8];
  float accred[4][ATT_MAX_G][64];
};

template <typename WT, bool PACKED_OUT>
__device__ __forceinline__ void phase_attention(const DevCtx& c, u32 layer, AttnShared& sh, u32 wg, u32 nwg) {
  const u32 T = c.meta->n_tokens, hd = c.hd, G = c.nq / c.nkv, tid = threadIdx.x;
  const WT* Kc = (const WT*)c.kv + (u64)layer * c.kv_layer_stride;
  const WT* Vc = Kc + c.kv_kv_stride;
  const float scale = 1.0f / sqrtf((float)hd);
  const u32 nparts = BLK_THREADS / hd, dd = tid % hd, part = tid / hd;
  for (u32 item = wg; item < T * c.nkv; item += nwg) {
    const u32 t = item / c.nkv, g = item % c.nkv;
    const u32 n = (u32)c.positions[t] + 1;
    const u32* bt = c.block_tables + (u64)c.seq_bslot[c.tok_seq[t]] * c.max_blocks_per_seq;
    __syncthreads();
    for (u32 i = tid; i < G * hd; i += BLK_THREADS)
      sh.q[i / hd][i % hd] = c.qkv[(u64)t * c.qkv_n + (u64)(g * G) * hd + i] * scale;
    __syncthreads();
    float m[ATT_MAX_G], l[ATT_MAX_G], acc[ATT_MAX_G];
#pragma unroll
    for (int h = 0; h < ATT_MAX_G; ++h) { m[h] = -INFINITY; l[h] = 0.f; acc[h] = 0.f; }
    for (u32 c0 = 0; c0 < n; c0 += BLK_THREADS) {
      const u32 j = c0 + tid;
      const bool valid = j < n;
      float s[ATT_MAX_G];
#pragma unroll
      for (int h = 0; h < ATT_MAX_G; ++h) s[h] = 0.f;
      if (valid) {
        const WT* kp = Kc + (((u64)bt[j / c.bs] * c.nkv + g) * c.bs + j % c.bs) * hd;
        for (u32 d0 = 0; d0 < hd; d0 += 8) {
          float kv[8];
          WLoad<WT>::load8(kp + d0, kv);
#pragma unroll
          for (int h = 0; h < ATT_MAX_G; ++h)
            if ((u32)h < G) {
#pragma unroll
              for (int i = 0; i < 8; ++i) s[h] += sh.q[h][d0 + i] * kv[i];
            }
        }
      }
#pragma unroll
      for (int h = 0; h < ATT_MAX_G; ++h) {
        if ((u32)h >= G) break;
        const float cm = block_max_f(valid ? s[h] : -INFINITY, sh.red);
        const float mn = fmaxf(m[h], cm);
        const float p = valid ? __expf(s[h] - mn) : 0.f;
        sh.p[h][tid] = p;
        const float cs = block_sum_f(p, sh.red + 4);
        const float corr = __expf(m[h] - mn);     // exp(-inf) = 0 on the first chunk
        l[h] = l[h] * corr + cs;
        acc[h] *= corr;
        m[h] = mn;
      }
      __syncthreads();
      const u32 cn = min((u32)BLK_THREADS, n - c0);
      for (u32 jj = part; jj < cn; jj += nparts) {
        const u32 jg = c0 + jj;
        const float v = WLoad<WT>::get(Vc, (((u64)bt[jg / c.bs] * c.nkv + g) * c.bs + jg % c.bs) * hd + dd);
#pragma unroll
        for (int h = 0; h < ATT_MAX_G; ++h)
          if ((u32)h < G) acc[h] += sh.p[h][jj] * v;
      }
      __syncthreads();
    }
    // combine the key-partitions (fixed order), normalise, write
    const u32 slot64 = dd % 64;
    for (u32 d0 = 0; d0 < hd; d0 += 64) {   // accred holds 64 dims at a time
      __syncthreads();
      if (dd >= d0 && dd < d0 + 64) {
#pragma unroll
        for (int h = 0; h < ATT_MAX_G; ++h)
          if ((u32)h < G) sh.accred[part][h][slot64] = acc[h];
      }
      __syncthreads();
      if (part == 0 && dd >= d0 && dd < d0 + 64) {
#pragma unroll
        for (int h = 0; h < ATT_MAX_G; ++h)
          if ((u32)h < G) {
            float a = 0.f;
            for (u32 pp = 0; pp < nparts; ++pp) a += sh.accred[pp][h][slot64];
            if (PACKED_OUT) c.aq[packed_act_off(t, (g * G + h) * hd + dd, c.TBS)] = f32_to_f16(a / l[h]);
            else c.attn[(u64)t * (c.nq * hd) + (u64)(g * G + h) * hd + dd] = a / l[h];
          }
      }
    }
  }
}
