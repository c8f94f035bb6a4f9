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
#define SMP_Z_WORDS (SMP_THREADS * (SMP_PER + 1))   // dynamic LDS of sample_kernel, in 4-byte words

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

__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __builtin_bit_cast(float, (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Block-wide sums of three values at once over SMP_THREADS threads; every thread gets the
// results.  `red` holds two banks of 3 x 16 wave slots used alternately (`phase` counts the
// calls), so one barrier per call is enough: a bank is rewritten only two calls later, and
// nobody can be two barriers ahead of a thread that still reads it.
struct Sum3 { float a, b, c; };
__device__ __forceinline__ Sum3 smp_block_sum3(float a, float b, float c, float* red, int& phase) {
  constexpr int NW = SMP_THREADS / 64;
  a = wave_sum(a);
  b = wave_sum(b);
  c = wave_sum(c);
  const int tid = threadIdx.x;
  float* bank = red + (phase & 1) * 3 * NW;
  ++phase;
  if ((tid & 63) == 0) { bank[tid >> 6] = a; bank[NW + (tid >> 6)] = b; bank[2 * NW + (tid >> 6)] = c; }
  __syncthreads();
  Sum3 s = {0.f, 0.f, 0.f};
#pragma unroll
  for (int w = 0; w < NW; ++w) { s.a += bank[w]; s.b += bank[NW + w]; s.c += bank[2 * NW + w]; }
  return s;
}
__device__ __forceinline__ float smp_block_sum(float v, float* red, int& phase) {
  return smp_block_sum3(v, 0.f, 0.f, red, phase).a;
}
// counts stay below 2^24, so they are exact in the float lanes of the reduction
__device__ __forceinline__ int smp_block_sum_int(int v, float* red, int& phase) {
  return (int)(smp_block_sum(v, red, phase) + 0.5f);
}
__device__ __forceinline__ float smp_block_max(float m, float* red, int& phase) {
  constexpr int NW = SMP_THREADS / 64;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  const int tid = threadIdx.x;
  float* bank = red + (phase & 1) * 3 * NW;
  ++phase;
  if ((tid & 63) == 0) bank[tid >> 6] = m;
  __syncthreads();
  m = bank[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) m = fmaxf(m, bank[w]);
  return m;
}

// Exclusive prefix sum over the threads in thread order (and the grand total), one barrier:
// shuffle scan inside each wave, then every thread adds the totals of the waves before its own,
// always in the same order, so the result is reproducible.
__device__ __forceinline__ float smp_block_scan_excl(float v, float* red, int& phase, float* total) {
  constexpr int NW = SMP_THREADS / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const float up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  float* bank = red + (phase & 1) * 3 * NW;
  ++phase;
  if (lane == 63) bank[wave] = incl;
  __syncthreads();
  float before = 0.f, all = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    if (w < wave) before += bank[w];
    all += bank[w];
  }
  *total = all;
  const float prev = __shfl_up(incl, 1);
  return before + (lane > 0 ? prev : 0.f);
}

// k-th largest key over PER slots per thread (0 marks an empty slot) by bisecting the key's 32
// bits two at a time; a wave counts with ballots, so a slot costs one compare per candidate prefix.
// Returns 0 when fewer than k slots are filled.
template <int PER>
__device__ __forceinline__ uint32_t smp_kth_largest(const uint32_t (&key)[PER], int k, float* red, int& phase) {
  constexpr int NW = SMP_THREADS / 64;
  const int tid = threadIdx.x;
  uint32_t prefix = 0u;
  for (int bit = 31; bit >= 1; bit -= 2) {
    const uint32_t c1 = prefix | (1u << (bit - 1)), c2 = prefix | (2u << (bit - 1)), c3 = prefix | (3u << (bit - 1));
    int n1 = 0, n2 = 0, n3 = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      n1 += __builtin_popcountll(__ballot(key[j] >= c1));
      n2 += __builtin_popcountll(__ballot(key[j] >= c2));
      n3 += __builtin_popcountll(__ballot(key[j] >= c3));
    }
    int* bank = reinterpret_cast<int*>(red) + (phase & 1) * 3 * NW;
    ++phase;
    if ((tid & 63) == 0) { bank[tid >> 6] = n1; bank[NW + (tid >> 6)] = n2; bank[2 * NW + (tid >> 6)] = n3; }
    __syncthreads();
    int t1 = 0, t2 = 0, t3 = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { t1 += bank[w]; t2 += bank[NW + w]; t3 += bank[2 * NW + w]; }
    prefix = t3 >= k ? c3 : t2 >= k ? c2 : t1 >= k ? c1 : prefix;
  }
  return prefix;
}

// Top-k cut over PER slots per thread (thread order = index order): slots outside the k largest
// keys (equal keys enter by lower index) get key 0; every kept slot gets e = exp(z - zmax).
// top_k = 0 keeps every filled slot.
template <int PER>
__device__ __forceinline__ void smp_apply_topk(uint32_t (&key)[PER], float (&e)[PER], int top_k, float zmax,
                                               float* red, int& phase) {
  uint32_t cut = 1u;          // kept: key > cut, or key == cut among the first tie_take ties
  int tie_take = 0x7fffffff;  // (cut = 1 with all ties taken keeps every real token: real keys are >= 0x007FFFFF)
  int seen = 0;
  if (top_k > 0) {
    cut = smp_kth_largest<PER>(key, top_k, red, phase);
    int gt = 0, mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) { gt += key[j] > cut; mine += key[j] == cut; }
    tie_take = top_k - smp_block_sum_int(gt, red, phase);
    float all;
    seen = (int)(smp_block_scan_excl((float)mine, red, phase, &all) + 0.5f);   // ties before this thread
  }
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    bool in = key[j] > cut;
    if (key[j] == cut && key[j] != 0u) { in = seen < tie_take; ++seen; }
    if (!in) key[j] = 0u;
    e[j] = in ? expf(key_to_float(key[j]) - zmax) : 0.f;
  }
}

// Nucleus cut and draw over PER kept-or-dropped slots per thread; slot j of a thread is token
// id0 + j and thread order is index order.  Dropped slots have key 0 and e 0.
template <int PER>
__device__ __forceinline__ int smp_nucleus_and_draw(uint32_t (&key)[PER], float (&e)[PER], int id0, float top_p,
                                                    float u, float* red, int& phase, int* found) {
  const int tid = threadIdx.x;
  auto ties_before = [&](uint32_t at) {
    int mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) mine += key[j] == at;
    float all;
    return (int)(smp_block_scan_excl((float)mine, red, phase, &all) + 0.5f);   // counts < 2^24: exact
  };
  // top-p: largest key whose upper set holds top_p of the mass, ties by index order
  if (top_p < 1.f) {
    float mine = 0.f;
#pragma unroll
    for (int j = 0; j < PER; ++j) mine += e[j];
    const float want = top_p * smp_block_sum(mine, red, phase);
    uint32_t prefix = 0u;
    for (int bit = 31; bit >= 1; bit -= 2) {      // two bits per pass: three candidate prefixes, one reduction
      const uint32_t c1 = prefix | (1u << (bit - 1)), c2 = prefix | (2u << (bit - 1)), c3 = prefix | (3u << (bit - 1));
      float m1 = 0.f, m2 = 0.f, m3 = 0.f;
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        m1 += key[j] >= c1 ? e[j] : 0.f;
        m2 += key[j] >= c2 ? e[j] : 0.f;
        m3 += key[j] >= c3 ? e[j] : 0.f;
      }
      const Sum3 m = smp_block_sum3(m1, m2, m3, red, phase);
      prefix = m.c >= want ? c3 : m.b >= want ? c2 : m.a >= want ? c1 : prefix;
    }
    if (prefix != 0u) {                            // prefix = 0: rounding left the total below the target, keep all
      float above = 0.f, etau = 0.f;
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        above += key[j] > prefix ? e[j] : 0.f;
        if (key[j] == prefix) etau = e[j];
      }
      above = smp_block_sum(above, red, phase);
      etau = smp_block_max(etau, red, phase);      // every tie has the same e; take it from whichever thread holds one
      int n_tie = (int)ceilf((want - above) / etau);
      if (n_tie < 1) n_tie = 1;
      int seen = ties_before(prefix);
#pragma unroll
      for (int j = 0; j < PER; ++j) {
        bool in = key[j] > prefix;
        if (key[j] == prefix) { in = seen < n_tie; ++seen; }
        if (!in) { key[j] = 0u; e[j] = 0.f; }
      }
    }
  }

  // the draw: running sum of e in index order against u * total
  float mine = 0.f;
#pragma unroll
  for (int j = 0; j < PER; ++j) mine += e[j];
  if (tid == 0) *found = 0x7fffffff;
  float total;
  const float run0 = smp_block_scan_excl(mine, red, phase, &total);   // (its barrier also publishes *found)
  const float target = u * total;
  // every thread continues the walk from the running sum in front of its range; the lowest
  // token whose running sum exceeds the target wins, exactly as in a sequential walk
  {
    float run = run0;
    int pick = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (e[j] > 0.f) {
        run += e[j];
        if (pick == 0x7fffffff && run > target) pick = id0 + j;
      }
    }
    if (pick != 0x7fffffff) atomicMin(found, pick);
  }
  __syncthreads();
  if (*found == 0x7fffffff) {
    // rounding left no running sum above the target: the last kept token
    __syncthreads();
    if (tid == 0) *found = -1;
    __syncthreads();
    int last = -1;
#pragma unroll
    for (int j = 0; j < PER; ++j) if (e[j] > 0.f) last = id0 + j;
    if (last >= 0) atomicMax(found, last);
    __syncthreads();
  }
  return *found < 0 ? 0 : *found;
}

// One draw from logits[0 .. vocab) by a workgroup of SMP_THREADS threads (all of them call this;
// vocab <= SMP_MAX_VOCAB, cfg->inv_temp != 0).  smp_z: SMP_Z_WORDS words of LDS; si, sk: SMP_THREADS
// words each; red: 6 words per wave; found: one word.  Returns the token in every thread.
__device__ __forceinline__ int smp_draw_token(const float* __restrict__ logits, int vocab,
                                              const SampleCfg* __restrict__ cfg, uint32_t draw_index,
                                              float* smp_z, int* si, uint32_t* sk, float* red, int* found) {
  const int tid = threadIdx.x;
  const float inv_temp = cfg->inv_temp;
  int phase = 0;
  int tok;
  // Thread t holds tokens 32 t .. 32 t + 31.  The logits are read once, coalesced, into LDS rows of
  // 32 padded to 33 words, from which a thread takes its row without bank conflicts (read straight
  // from global memory, every load instruction of a wave would touch 64 cache lines).
  for (int i = tid; i < vocab; i += SMP_THREADS) smp_z[i + (i >> 5)] = logits[i];
  __syncthreads();
  const int base = tid * SMP_PER;
  uint32_t key[SMP_PER];
  float zmax = -INFINITY;
#pragma unroll
  for (int j = 0; j < SMP_PER; ++j) {
    const int i = base + j;
    const float z = i < vocab ? __fmul_rn(smp_z[base + tid + j], inv_temp) + 0.f : 0.f;   // + 0: -0 and +0 are one value
    key[j] = i < vocab ? order_key(z) : 0u;
    if (i < vocab) zmax = fmaxf(zmax, z);
  }
  zmax = smp_block_max(zmax, red, phase);

  uint32_t ctr[4] = {draw_index, 0u, 0u, 0u};
  philox4x32_10(ctr, cfg->seed_lo, cfg->seed_hi);
  const float u = (float)(ctr[0] >> 8) * (1.0f / 16777216.0f);
  const int top_k = (cfg->top_k >= 1 && cfg->top_k < vocab) ? cfg->top_k : 0;

  // (1) With a top-k cut of at most one candidate per thread, almost all of the vocabulary can be
  // discarded cheaply first: the k-th largest of the threads' own maxima is a lower bound of the
  // k-th largest key (at least k keys reach it), found with one slot per thread.  What reaches the
  // bound is packed, in index order, one per thread, and every later pass costs one slot, not 32.
  bool done = false;
  if (top_k > 0 && top_k <= SMP_THREADS) {
    uint32_t tmax[1] = {0u};
#pragma unroll
    for (int j = 0; j < SMP_PER; ++j) tmax[0] = key[j] > tmax[0] ? key[j] : tmax[0];
    const uint32_t bound = smp_kth_largest<1>(tmax, top_k, red, phase);
    int reach = 0;
#pragma unroll
    for (int j = 0; j < SMP_PER; ++j) reach += key[j] >= bound;
    float all;
    int at = (int)(smp_block_scan_excl((float)reach, red, phase, &all) + 0.5f);
    const int nreach = (int)(all + 0.5f);
    if (bound != 0u && nreach <= SMP_THREADS) {            // uniform: `all` is the same in every thread
#pragma unroll
      for (int j = 0; j < SMP_PER; ++j) {
        if (key[j] >= bound) {
          sk[at] = key[j];
          si[at] = base + j;
          ++at;
        }
      }
      __syncthreads();
      uint32_t k1[1] = {tid < nreach ? sk[tid] : 0u};
      float e1[1];
      const int id = tid < nreach ? si[tid] : 0;
      __syncthreads();
      smp_apply_topk<1>(k1, e1, top_k, zmax, red, phase);
      tok = smp_nucleus_and_draw<1>(k1, e1, id, cfg->top_p, u, red, phase, found);
      done = true;
    }
  }
  // (2) otherwise: the cut (if any), the nucleus and the draw over all 32 slots per thread
  if (!done) {
    float e[SMP_PER];
    smp_apply_topk<SMP_PER>(key, e, top_k, zmax, red, phase);
    tok = smp_nucleus_and_draw<SMP_PER>(key, e, base, cfg->top_p, u, red, phase, found);
  }
  return tok;
}

//   prefill = 1: pos += n_prompt (rows of the last prompt chunk), steps := 1, ring[0] := token (draw index 0)
//   prefill = 0: pos += 1, ring[steps] := token, steps += 1   (draw index = steps before the step)
// It also gathers the selected token's embedding row into x_next (when given), the input of the next
// decode step, which therefore needs no gather kernel of its own (what x_next held, the step's final
// residual stream, is kept in x_keep for the read-back hook); and it reports token -1 to the host
// when a kernel of the step raised DevState::fault (the device state still advances with a valid id).
__global__ __launch_bounds__(SMP_THREADS) void sample_kernel(const float* __restrict__ pval,
                                                             const int* __restrict__ pidx, int nparts,
                                                             const float* __restrict__ logits, int vocab,
                                                             const SampleCfg* __restrict__ cfg,
                                                             DevState* st, int* host_ring, int ring_size,
                                                             int prefill, const half_t* __restrict__ emb,
                                                             float* __restrict__ x_next, float* __restrict__ x_keep,
                                                             int d) {
  extern __shared__ float smp_z[];     // SMP_Z_WORDS words, used by the stochastic path only
  __shared__ float sv[SMP_THREADS];
  __shared__ int si[SMP_THREADS];
  __shared__ uint32_t sk[SMP_THREADS];
  __shared__ float red[2 * 3 * (SMP_THREADS / 64)];
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
    tok = smp_draw_token(logits, vocab, cfg, (uint32_t)(prefill ? 0 : st->steps), smp_z, si, sk, red, &found);
  }

  if (tid == 0) found = tok;        // one value for every thread, whichever path chose it
  __syncthreads();
  tok = found;
  if (x_next) {
    for (int i = tid * 8; i < d; i += SMP_THREADS * 8) {
      const h8 e = load_h8(emb + (size_t)tok * d + i);
      if (!prefill) {
        *reinterpret_cast<f4*>(x_keep + i) = *reinterpret_cast<const f4*>(x_next + i);
        *reinterpret_cast<f4*>(x_keep + i + 4) = *reinterpret_cast<const f4*>(x_next + i + 4);
      }
      *reinterpret_cast<f4*>(x_next + i) = f4{(float)e[0], (float)e[1], (float)e[2], (float)e[3]};
      *reinterpret_cast<f4*>(x_next + i + 4) = f4{(float)e[4], (float)e[5], (float)e[6], (float)e[7]};
    }
  }

  if (tid == 0) {
    int idx;
    if (prefill) {
      st->pos = st->pos + st->n_prompt;
      idx = 0;
      st->steps = 1;
    } else {
      st->pos = st->pos + 1;
      idx = st->steps;
      st->steps = idx + 1;
    }
    st->next_token = tok;
    if (idx < ring_size) host_ring[idx] = st->fault ? -1 : tok;
  }
}
