// Token selection and state advance, the last kernel of every step: greedy
// argmax, or temperature / top-k / top-p sampling with a counter-based random
// draw.  The paper leaves sampling to its host-side dynamic domain (Sec. III-A,
// III-C) and lists stochastic operations as what keeps it outside graph replay
// (Sec. VI-C); here it is one single-workgroup kernel inside the captured graph:
// its parameters and the draw index live in device memory, so replays stay
// bit-reproducible for a given seed and a reset replays the same stream.
//
// Definition (every open choice of the textbook procedure fixed as stated):
//   z_i = logit_i * float(1 / T); candidates C = the top_k largest z (ties by lower index);
//   e_i = exp(z_i - max z) over C, S = sum; nucleus F = candidates above the threshold value tau
//   plus the first n_tie equal to it (lower index first), tau = largest value whose upper set has
//   mass >= top_p * S, n_tie = ceil((top_p * S - mass above) / e_tau) >= 1; the draw walks F in
//   order of increasing INDEX and returns the first token whose running sum of e exceeds u * sum_F;
//   u = (x0 >> 8) * 2^-24, x0 = first word of Philox4x32-10(counter = (draw index, 0, 0, 0), key = seed).
//
// No sort is needed: the k-th largest value and the nucleus threshold are found by bisecting the
// 32 bits of an order-preserving integer image of z, one block-wide count or sum per bit, with
// every thread holding 32 consecutive tokens in registers (vocabularies up to 32768).
#pragma once
#include "ll_device.h"

#define SMP_THREADS 1024
#define SMP_PER 32                               // consecutive tokens per thread
#define SMP_MAX_VOCAB (SMP_THREADS * SMP_PER)

struct SampleCfg {
  float inv_temp;      // float(1 / T); 0 selects greedy argmax
  int32_t top_k;       // 0 or >= vocab: no top-k cut
  float top_p;         // 1: no nucleus cut
  uint32_t seed_lo, seed_hi;
  int32_t pad[11];
};

__device__ __forceinline__ void philox4x32_10(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
    c[0] = n0; c[1] = (uint32_t)p1; c[2] = n2; c[3] = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}

// larger float <=> larger key; every real value maps above key 0, which marks "no token"
__device__ __forceinline__ uint32_t order_key(float z) {
  const uint32_t b = __builtin_bit_cast(uint32_t, z);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Block-wide sums over SMP_THREADS threads; every thread gets the result.  `red` holds one
// slot per wave; two barriers per call keep consecutive calls from overlapping.
__device__ __forceinline__ float smp_block_sum(float v, float* red) {
  v = wave_sum(v);
  const int tid = threadIdx.x;
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < SMP_THREADS / 64; ++w) s += red[w];
  __syncthreads();
  return s;
}
__device__ __forceinline__ int smp_block_sum_int(int v, float* red) {
  // counts stay below 2^24, so they are exact in the float lanes of the wave reduction
  return (int)(smp_block_sum((float)v, red) + 0.5f);
}

//   prefill = 1: pos := n_prompt, steps := 1, ring[0] := token (draw index 0)
//   prefill = 0: pos += 1, ring[steps] := token, steps += 1   (draw index = steps before the step)
__global__ __launch_bounds__(SMP_THREADS) void sample_kernel(const float* __restrict__ pval,
                                                             const int* __restrict__ pidx, int nparts,
                                                             const float* __restrict__ logits, int vocab,
                                                             const SampleCfg* __restrict__ cfg,
                                                             DevState* st, int* host_ring, int ring_size,
                                                             int prefill) {
  __shared__ float sv[SMP_THREADS];
  __shared__ int si[SMP_THREADS];
  __shared__ float red[SMP_THREADS / 64];
  __shared__ float scan[SMP_THREADS];
  __shared__ int found;
  const int tid = threadIdx.x;
  const float inv_temp = cfg->inv_temp;
  int tok;

  if (inv_temp == 0.f || vocab > SMP_MAX_VOCAB) {
    // ---- greedy: reduce the LM head's per-workgroup (max, lowest index) candidates
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = tid; i < nparts; i += SMP_THREADS) {
      const float v = pval[i];
      const int ix = pidx[i];
      if (v > bv || (v == bv && ix < bi)) { bv = v; bi = ix; }
    }
    sv[tid] = bv;
    si[tid] = bi;
    __syncthreads();
    for (int off = SMP_THREADS / 2; off > 0; off >>= 1) {
      if (tid < off) {
        const float v = sv[tid + off];
        const int ix = si[tid + off];
        if (v > sv[tid] || (v == sv[tid] && ix < si[tid])) { sv[tid] = v; si[tid] = ix; }
      }
      __syncthreads();
    }
    tok = si[0];
    if (tok == 0x7fffffff) tok = 0;   // every logit NaN: still a valid id
  } else {
    // ---- stochastic: thread t holds tokens 32 t .. 32 t + 31
    const int base = tid * SMP_PER;
    uint32_t key[SMP_PER];
    float zmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < SMP_PER; ++j) {
      const int i = base + j;
      const float z = i < vocab ? __fmul_rn(logits[i], inv_temp) + 0.f : 0.f;   // + 0: -0 and +0 are one value
      key[j] = i < vocab ? order_key(z) : 0u;
      if (i < vocab) zmax = fmaxf(zmax, z);
    }
    // block max through the sum helper's storage: max is exact in any order
    {
      float m = zmax;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
      if ((tid & 63) == 0) red[tid >> 6] = m;
      __syncthreads();
      m = red[0];
#pragma unroll
      for (int w = 1; w < SMP_THREADS / 64; ++w) m = fmaxf(m, red[w]);
      __syncthreads();
      zmax = m;
    }

    // (1) top-k: the k-th largest key by bisection, then the ties at that key by index order
    const int top_k = cfg->top_k;
    uint32_t cut = 1u;          // candidates: key > cut, or key == cut among the first tie_take ties
    int tie_take = 0x7fffffff;  // (cut = 1 with all ties taken keeps every real token: keys are >= 0x007FFFFF)
    if (top_k >= 1 && top_k < vocab) {
      uint32_t prefix = 0u;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t c = prefix | (1u << bit);
        int n = 0;
#pragma unroll
        for (int j = 0; j < SMP_PER; ++j) n += key[j] >= c;
        if (smp_block_sum_int(n, red) >= top_k) prefix = c;
      }
      cut = prefix;
      int gt = 0;
#pragma unroll
      for (int j = 0; j < SMP_PER; ++j) gt += key[j] > cut;
      tie_take = top_k - smp_block_sum_int(gt, red);
    }
    // exclusive count of ties before this thread, in index order
    auto ties_before = [&](uint32_t at) {
      int mine = 0;
#pragma unroll
      for (int j = 0; j < SMP_PER; ++j) mine += key[j] == at;
      scan[tid] = (float)mine;
      __syncthreads();
      for (int off = 1; off < SMP_THREADS; off <<= 1) {
        const float add = tid >= off ? scan[tid - off] : 0.f;
        __syncthreads();
        scan[tid] += add;
        __syncthreads();
      }
      const int before = (int)(scan[tid] + 0.5f) - mine;
      __syncthreads();
      return before;
    };
    float e[SMP_PER];
    {
      int seen = (tie_take != 0x7fffffff) ? ties_before(cut) : 0;
#pragma unroll
      for (int j = 0; j < SMP_PER; ++j) {
        bool in = key[j] > cut;
        if (key[j] == cut && key[j] != 0u) { in = seen < tie_take; ++seen; }
        if (!in) key[j] = 0u;                       // dropped tokens leave the key space
        const float z = (base + j) < vocab ? __fmul_rn(logits[base + j], inv_temp) + 0.f : 0.f;
        e[j] = in ? expf(z - zmax) : 0.f;
      }
    }

    // (2) top-p: largest key whose upper set holds top_p of the mass, ties by index order
    const float top_p = cfg->top_p;
    if (top_p < 1.f) {
      float mine = 0.f;
#pragma unroll
      for (int j = 0; j < SMP_PER; ++j) mine += e[j];
      const float want = top_p * smp_block_sum(mine, red);
      uint32_t prefix = 0u;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t c = prefix | (1u << bit);
        float m = 0.f;
#pragma unroll
        for (int j = 0; j < SMP_PER; ++j) m += key[j] >= c ? e[j] : 0.f;
        if (smp_block_sum(m, red) >= want) prefix = c;
      }
      if (prefix != 0u) {                            // prefix = 0: rounding left the total below the target, keep all
        float above = 0.f, etau = 0.f;
#pragma unroll
        for (int j = 0; j < SMP_PER; ++j) {
          above += key[j] > prefix ? e[j] : 0.f;
          if (key[j] == prefix) etau = e[j];
        }
        above = smp_block_sum(above, red);
        // every tie has the same e; take it from whichever thread holds one
        {
          float m = etau;
#pragma unroll
          for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
          if ((tid & 63) == 0) red[tid >> 6] = m;
          __syncthreads();
          m = red[0];
#pragma unroll
          for (int w = 1; w < SMP_THREADS / 64; ++w) m = fmaxf(m, red[w]);
          __syncthreads();
          etau = m;
        }
        int n_tie = (int)ceilf((want - above) / etau);
        if (n_tie < 1) n_tie = 1;
        int seen = ties_before(prefix);
#pragma unroll
        for (int j = 0; j < SMP_PER; ++j) {
          bool in = key[j] > prefix;
          if (key[j] == prefix) { in = seen < n_tie; ++seen; }
          if (!in) { key[j] = 0u; e[j] = 0.f; }
        }
      }
    }

    // (3) the draw: running sum of e in index order against u * total
    float mine = 0.f;
#pragma unroll
    for (int j = 0; j < SMP_PER; ++j) mine += e[j];
    scan[tid] = mine;
    if (tid == 0) found = 0x7fffffff;
    __syncthreads();
    for (int off = 1; off < SMP_THREADS; off <<= 1) {
      const float add = tid >= off ? scan[tid - off] : 0.f;
      __syncthreads();
      scan[tid] += add;
      __syncthreads();
    }
    const float total = scan[SMP_THREADS - 1];
    uint32_t ctr[4] = {(uint32_t)(prefill ? 0 : st->steps), 0u, 0u, 0u};
    philox4x32_10(ctr, cfg->seed_lo, cfg->seed_hi);
    const float target = (float)(ctr[0] >> 8) * (1.0f / 16777216.0f) * total;
    // every thread continues the walk from the running sum in front of its range; the lowest
    // token whose running sum exceeds the target wins, exactly as in a sequential walk
    {
      float run = tid > 0 ? scan[tid - 1] : 0.f;
      int pick = 0x7fffffff;
#pragma unroll
      for (int j = 0; j < SMP_PER; ++j) {
        if (e[j] > 0.f) {
          run += e[j];
          if (pick == 0x7fffffff && run > target) pick = base + j;
        }
      }
      if (pick != 0x7fffffff) atomicMin(&found, pick);
    }
    __syncthreads();
    if (found == 0x7fffffff) {
      // rounding left no running sum above the target: the last kept token
      __syncthreads();
      if (tid == 0) found = -1;
      __syncthreads();
      int last = -1;
#pragma unroll
      for (int j = 0; j < SMP_PER; ++j) if (e[j] > 0.f) last = base + j;
      if (last >= 0) atomicMax(&found, last);
      __syncthreads();
    }
    tok = found < 0 ? 0 : found;
  }

  if (tid == 0) {
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
