// Batch-1 decode kernels for gfx950: bandwidth-bound GEMVs with fused
// prologues/epilogues, split-K attention over the KV cache, greedy sampling.
//
// One decoding step (the loop body of the paper's Alg. 1) is, per layer:
//   [RMSNorm + QKV GEMV + RoPE + KV-cache write] -> [split-K attention + combine]
//   -> [O GEMV + residual] -> [RMSNorm + gate/up GEMV + SwiGLU] -> [down GEMV + residual]
// then [final RMSNorm + LM-head GEMV + block argmax] -> [argmax + state advance].
// Batch 1 gives one multiply-add per weight byte pair, so none of this is a
// dense contraction: no MFMA, only 128-bit coalesced weight streams, fp32
// accumulation and DPP reductions.
#pragma once
#include "ll_device.h"

enum GemvMode { GM_QKV = 0, GM_ORES = 1, GM_GATEUP = 2, GM_DOWN = 3, GM_LMHEAD = 4 };

struct GemvArgs {
  const half_t* w0;    // QKV: Wq | O/down/LM head: the matrix | gate/up: W_gate
  const half_t* w1;    // QKV: Wk | gate/up: W_up
  const half_t* w2;    // QKV: Wv
  const float* xin;    // input vector [K], fp32
  const half_t* gain;  // RMSNorm gain [K] for the fused-norm modes
  float* out;          // QKV: rotated q [d] | O/down: residual stream x (+=) | gate/up: m [F] | LM head: logits
  int N;               // output rows per matrix
  int K;               // input length (multiple of 8)
  float eps;
  // QKV epilogue
  half_t* kcache;      // this layer's keys   [head][max_seq][head_dim]
  half_t* vcache;      // this layer's values [head][max_seq][head_dim]
  const float2* rope;  // [max_seq][head_dim/2] (cos, sin)
  const DevState* st;
  int head_dim, max_seq;
  // LM-head epilogue
  float* amax_val;     // [gridDim.x] best logit seen by each workgroup
  int* amax_idx;
  int x_row_from_prompt;  // 1: input vector is row (st->n_prompt - 1) of a [rows][K] matrix
};

// The input vector is staged in LDS as fp32 in a lane-major layout: for the
// 512-element chunk c, lane l owns elements c*512 + l*8 .. +7, stored as two
// float4 at c*512 + l*4 and c*512 + 256 + l*4, so a wave reads it with two
// conflict-free 128-bit LDS loads per chunk.  Padding up to a multiple of U
// chunks is zero, which lets the weight loads clamp their address instead of
// branching at a ragged tail.
//
// Each wave owns pairs of weight rows (two accumulators share every LDS read):
//   QKV     rows (j, j + head_dim/2) of one head, so RoPE is applied in registers
//   gate/up row r of W_gate with row r of W_up, so SwiGLU is applied in registers
//   others  rows (2p, 2p+1)
// RMSNorm is folded in as y = (W (x*g)) * rsqrt(mean(x^2)+eps): the scalar
// factor multiplies the accumulator, so the weight stream never waits for it.
template <int MODE, int U>
__global__ __launch_bounds__(LL_WG) void gemv_kernel(GemvArgs a) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.K;
  const int nch = (K + 511) >> 9;
  const int nchp = ((nch + U - 1) / U) * U;
  float* red = lds + nchp * 512;
  constexpr bool NORM = (MODE == GM_QKV || MODE == GM_GATEUP || MODE == GM_LMHEAD);

  const int d_half = a.N >> 1;
  int P;
  if (MODE == GM_QKV) P = 3 * d_half;
  else if (MODE == GM_GATEUP) P = a.N;
  else P = (a.N + 1) >> 1;

  // row pair p -> the two weight rows this wave streams
  const half_t *pa = a.w0, *pb = a.w0;
  int sec = 0, rowA = 0, rowB = 0;
  auto select_rows = [&](int p) {
    if (MODE == GM_QKV) {
      sec = p / d_half;
      const int pp = p - sec * d_half;
      const half_t* base = sec == 0 ? a.w0 : (sec == 1 ? a.w1 : a.w2);
      if (sec < 2) {
        const int hh = a.head_dim >> 1;
        const int head = pp / hh, j = pp - head * hh;
        rowA = head * a.head_dim + j;
        rowB = rowA + hh;
      } else {
        rowA = 2 * pp;
        rowB = rowA + 1;
      }
      pa = base + (size_t)rowA * K;
      pb = base + (size_t)rowB * K;
    } else if (MODE == GM_GATEUP) {
      rowA = rowB = p;
      pa = a.w0 + (size_t)p * K;
      pb = a.w1 + (size_t)p * K;
    } else {
      rowA = 2 * p;
      rowB = min(rowA + 1, a.N - 1);
      pa = a.w0 + (size_t)rowA * K;
      pb = a.w0 + (size_t)rowB * K;
    }
  };
  h8 wa[U], wb[U];
  auto load_group = [&](int c0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = min((c0 + u) * 512 + lane * 8, K - 8);
      wa[u] = load_stream(pa + k);
      wb[u] = load_stream(pb + k);
    }
  };

  // The weight stream does not depend on the input vector: put the first
  // loads of this wave's first row pair in flight before staging x, so HBM is
  // already busy while the prologue runs.
  const int gw = blockIdx.x * (LL_WG / 64) + wave, GW = gridDim.x * (LL_WG / 64);
  if (gw < P) {
    select_rows(gw);
    load_group(0);
  }

  const float* xin = a.xin;
  if (MODE == GM_LMHEAD && a.x_row_from_prompt) xin += (size_t)(a.st->n_prompt - 1) * K;

  float ss = 0.f;
  for (int i = tid; i < nchp * 128; i += LL_WG) {
    const int k = i * 4;
    f4 v = {0.f, 0.f, 0.f, 0.f};
    if (k < K) {
      v = *reinterpret_cast<const f4*>(xin + k);
      if (NORM) {
        ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
        h4 g = *reinterpret_cast<const h4*>(a.gain + k);
        v[0] *= (float)g[0]; v[1] *= (float)g[1]; v[2] *= (float)g[2]; v[3] *= (float)g[3];
      }
    }
    const int c = k >> 9, r = k & 511;
    *reinterpret_cast<f4*>(lds + c * 512 + ((r >> 2) & 1) * 256 + (r >> 3) * 4) = v;
  }
  if (NORM) {
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
  }
  __syncthreads();
  float inv = 1.f;
  if (NORM) inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)K + a.eps);

  float best_v = -INFINITY;
  int best_i = 0x7fffffff;

  for (int p = gw; p < P; p += GW) {
    if (p != gw) select_rows(p);
    float accA = 0.f, accB = 0.f;
    for (int c0 = 0; c0 < nch; c0 += U) {
      if (p != gw || c0 != 0) load_group(c0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float* xp = lds + (c0 + u) * 512 + lane * 4;
        const f4 x0 = *reinterpret_cast<const f4*>(xp);
        const f4 x1 = *reinterpret_cast<const f4*>(xp + 256);
        accA = dot8(wa[u], x0, x1, accA);
        accB = dot8(wb[u], x0, x1, accB);
      }
    }
    accA = wave_sum(accA) * inv;
    accB = wave_sum(accB) * inv;

    if (MODE == GM_QKV) {
      const int pos = a.st->pos;
      if (sec < 2) {
        const int hh = a.head_dim >> 1;
        const int head = rowA / a.head_dim, j = rowA - head * a.head_dim;
        const float2 cs = a.rope[(size_t)pos * hh + j];
        const float ra = accA * cs.x - accB * cs.y;
        const float rb = accB * cs.x + accA * cs.y;
        if (lane == 0) {
          if (sec == 0) {
            a.out[rowA] = ra;
            a.out[rowB] = rb;
          } else {
            half_t* kr = a.kcache + ((size_t)head * a.max_seq + pos) * a.head_dim;
            kr[j] = (half_t)ra;
            kr[j + hh] = (half_t)rb;
          }
        }
      } else if (lane == 0) {
        const int head = rowA / a.head_dim, e = rowA - head * a.head_dim;
        half_t* vr = a.vcache + ((size_t)head * a.max_seq + pos) * a.head_dim;
        vr[e] = (half_t)accA;
        vr[e + 1] = (half_t)accB;
      }
    } else if (MODE == GM_GATEUP) {
      if (lane == 0) a.out[p] = accA / (1.0f + expf(-accA)) * accB;
    } else if (MODE == GM_ORES || MODE == GM_DOWN) {
      if (lane == 0) {
        a.out[rowA] += accA;
        if (rowB != rowA) a.out[rowB] += accB;
      }
    } else {  // GM_LMHEAD
      if (lane == 0) {
        a.out[rowA] = accA;
        if (rowB != rowA) a.out[rowB] = accB;
      }
      if (accA > best_v) { best_v = accA; best_i = rowA; }   // rows ascend within a wave:
      if (rowB != rowA && accB > best_v) { best_v = accB; best_i = rowB; }  // '>' keeps the lowest index
    }
  }

  if (MODE == GM_LMHEAD) {
    __syncthreads();  // everyone is done reading red[] as the norm factor
    int* redi = reinterpret_cast<int*>(red + 4);
    if (lane == 0) { red[wave] = best_v; redi[wave] = best_i; }
    __syncthreads();
    if (tid == 0) {
      float bv = red[0];
      int bi = redi[0];
      for (int w = 1; w < LL_WG / 64; ++w)
        if (red[w] > bv || (red[w] == bv && redi[w] < bi)) { bv = red[w]; bi = redi[w]; }
      a.amax_val[blockIdx.x] = bv;
      a.amax_idx[blockIdx.x] = bi;
    }
  }
}

// x = float(E[next_token])
__global__ __launch_bounds__(LL_WG) void embed_kernel(const half_t* __restrict__ emb,
                                                      const DevState* __restrict__ st,
                                                      float* __restrict__ x, int d) {
  const int tok = st->next_token;
  const int i = (blockIdx.x * LL_WG + threadIdx.x) * 8;
  if (i < d) {
    const h8 e = *reinterpret_cast<const h8*>(emb + (size_t)tok * d + i);
#pragma unroll
    for (int j = 0; j < 8; ++j) x[i + j] = (float)e[j];
  }
}

// Split-K attention of the one new query against keys 0..pos of one head.
//
// grid = (heads, S).  A key row (HD halves) is read by HD/8 adjacent lanes with
// one 16-byte load each, so a wave covers 64/(HD/8) consecutive keys per load.
// Every such lane group keeps its own online-softmax state (running max m,
// denominator l, 8 output columns per lane) over the keys it is dealt, round
// robin over all groups of all S workgroups of the head -- the grid is fixed
// and the key range comes from DevState, so the same captured launch serves
// every KV length.  Groups are merged through LDS, workgroups through a
// partial buffer; the last workgroup of a head to arrive (device-scope counter)
// merges the S partials and writes o.
template <int HD>
__global__ __launch_bounds__(LL_WG) void attn_decode_kernel(
    const float* __restrict__ q, const half_t* __restrict__ kc, const half_t* __restrict__ vc,
    const DevState* __restrict__ st, float* part, unsigned* cnt, float* __restrict__ o,
    int max_seq) {
  constexpr int LPR = HD / 8;      // lanes per key row
  constexpr int GPW = 64 / LPR;    // lane groups per wave
  constexpr int NG = (LL_WG / 64) * GPW;
  constexpr int UK = 4;            // keys in flight per group
  constexpr int PS = HD + 2;       // floats per partial: m, l, acc[HD]
  __shared__ float s_m[NG], s_l[NG], s_acc[NG][HD];
  __shared__ int s_last;

  const int h = blockIdx.x, s = blockIdx.y, S = gridDim.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int gi = lane / LPR, li = lane % LPR;
  const int n_keys = st->pos + 1;
  const float scale = 1.0f / sqrtf((float)HD);

  float qv[8];
  {
    const f4 q0 = *reinterpret_cast<const f4*>(q + h * HD + li * 8);
    const f4 q1 = *reinterpret_cast<const f4*>(q + h * HD + li * 8 + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { qv[e] = q0[e] * scale; qv[4 + e] = q1[e] * scale; }
  }
  const half_t* kh = kc + (size_t)h * max_seq * HD + li * 8;
  const half_t* vh = vc + (size_t)h * max_seq * HD + li * 8;

  float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;

  const int stride = S * (LL_WG / 64) * GPW;
  for (int base = (s * (LL_WG / 64) + wave) * GPW; base < n_keys; base += stride * UK) {
    h8 kk[UK], vv[UK];
#pragma unroll
    for (int j = 0; j < UK; ++j) {
      const int u = min(base + j * stride + gi, n_keys - 1);
      kk[j] = *reinterpret_cast<const h8*>(kh + (size_t)u * HD);
      vv[j] = *reinterpret_cast<const h8*>(vh + (size_t)u * HD);
    }
#pragma unroll
    for (int j = 0; j < UK; ++j) {
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dot += qv[e] * (float)kk[j][e];
      dot = group_sum<LPR>(dot);
      if (base + j * stride + gi < n_keys) {
        const float mn = fmaxf(m, dot);
        const float corr = __expf(m - mn);
        const float p = __expf(dot - mn);
        l = l * corr + p;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * corr + p * (float)vv[j][e];
        m = mn;
      }
    }
  }

  const int g = wave * GPW + gi;
  if (li == 0) { s_m[g] = m; s_l[g] = l; }
#pragma unroll
  for (int e = 0; e < 8; ++e) s_acc[g][li * 8 + e] = acc[e];
  __syncthreads();

  float* mypart = part + ((size_t)h * S + s) * PS;
  if (tid < HD) {
    float M = -INFINITY;
    for (int i = 0; i < NG; ++i) M = fmaxf(M, s_m[i]);
    float L = 0.f, A = 0.f;
    if (M > -INFINITY) {
      for (int i = 0; i < NG; ++i) {
        const float w = __expf(s_m[i] - M);   // empty groups: exp(-inf) = 0
        L += s_l[i] * w;
        A += s_acc[i][tid] * w;
      }
    }
    if (tid == 0) {
      __hip_atomic_store(mypart + 0, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(mypart + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __hip_atomic_store(mypart + 2 + tid, A, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // Publishing without a cache flush: the partial was written with device-scope
  // atomic stores, which are coherent across the per-XCD L2s on their own, and
  // the counter increment is issued only after every such store of this
  // workgroup has completed (wait for the vector-memory counter, then the
  // workgroup barrier).  The reader's loads below are device-scope atomics
  // too and are issued after its own increment has returned.  A release fence
  // here would write back the whole L2 in every workgroup, which costs far
  // more than the attention itself.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) {
    const unsigned t = __hip_atomic_fetch_add(cnt + h, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (t == (unsigned)(S - 1));
  }
  __syncthreads();
  if (!s_last) return;
  if (tid < HD) {
    const float* hp = part + (size_t)h * S * PS;
    float M = -INFINITY;
    for (int i = 0; i < S; ++i)
      M = fmaxf(M, __hip_atomic_load(hp + i * PS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    float L = 0.f, A = 0.f;
    for (int i = 0; i < S; ++i) {
      const float mi = __hip_atomic_load(hp + i * PS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const float w = (mi > -INFINITY) ? __expf(mi - M) : 0.f;
      L += __hip_atomic_load(hp + i * PS + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * w;
      A += __hip_atomic_load(hp + i * PS + 2 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * w;
    }
    o[h * HD + tid] = A / L;
  }
  if (tid == 0) __hip_atomic_store(cnt + h, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Final argmax over the per-workgroup candidates of the LM head (ties: lowest
// index), then the state advance that makes the next replay self-contained:
// the token becomes next_token, the position moves on, and the id is written
// to a pinned host ring the caller reads after synchronising.
//   prefill = 1: pos := n_prompt, steps := 1, ring[0] := token
//   prefill = 0: pos += 1, ring[steps] := token, steps += 1
__global__ __launch_bounds__(LL_WG) void sample_kernel(const float* __restrict__ pval,
                                                       const int* __restrict__ pidx, int nparts,
                                                       DevState* st, int* host_ring, int ring_size,
                                                       int prefill) {
  __shared__ float sv[LL_WG];
  __shared__ int si[LL_WG];
  const int tid = threadIdx.x;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = tid; i < nparts; i += LL_WG) {
    const float v = pval[i];
    const int ix = pidx[i];
    if (v > bv || (v == bv && ix < bi)) { bv = v; bi = ix; }
  }
  sv[tid] = bv;
  si[tid] = bi;
  __syncthreads();
  for (int off = LL_WG / 2; off > 0; off >>= 1) {
    if (tid < off) {
      const float v = sv[tid + off];
      const int ix = si[tid + off];
      if (v > sv[tid] || (v == sv[tid] && ix < si[tid])) { sv[tid] = v; si[tid] = ix; }
    }
    __syncthreads();
  }
  if (tid == 0) {
    int tok = si[0];
    if (tok == 0x7fffffff) tok = 0;   // every logit NaN: still a valid id
    int idx;
    if (prefill) {
      st->pos = st->n_prompt;
      idx = 0;
      st->steps = 1;
    } else {
      st->pos = st->pos + 1;
      idx = st->steps;
      st->steps = idx + 1;
    }
    st->next_token = tok;
    if (idx < ring_size) host_ring[idx] = tok;
  }
}

// Plain device-to-device copy with the same 16-byte streaming loads the GEMVs
// use.  It exists to calibrate hardware traffic counters against a known byte
// count; nothing on the decode path calls it.
__global__ __launch_bounds__(LL_WG) void stream_copy_kernel(const h8* __restrict__ src,
                                                            h8* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * LL_WG;
  for (size_t i = (size_t)blockIdx.x * LL_WG + threadIdx.x; i < n16; i += stride)
    dst[i] = __builtin_nontemporal_load(src + i);
}
