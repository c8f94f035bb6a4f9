// One persistent kernel for the whole decode step.
//
// Launched as ONE node of the decode graph with one 768-thread workgroup per
// compute unit.  The step's phases (per layer: QKV -> attention -> O -> gate/up
// -> down; then LM head -> sampling) run inside the kernel, separated by grid
// barriers, instead of as ~160 kernels whose ramp-up and drain leave HBM idle
// for about 3 us each.  What makes that pay: the weight stream does not depend
// on the activations, so before a compute wave reaches a barrier it has
// already put the 16 x 16-byte loads of its FIRST row pair of the NEXT phase in
// flight.  With 11 compute waves per CU that is ~180 KB per CU of weight
// traffic covering the barrier, the re-staging of the input vector and (for
// the O projection) the whole attention phase.
//
// Wave roles.  Waves 0..10 stream weights and leave raw dot products in LDS;
// they never store to global memory, so they never have to drain their
// vector-memory counter (which would also wait for the prefetched loads).
// Wave 11 is the service wave: at the end of a phase it applies the epilogue
// (RMSNorm factor, RoPE, SwiGLU, residual, argmax), stores the results, waits
// for those stores to complete, arrives at the grid barrier and spins on it.
//
// Coherence: the 8 XCDs have private L2s.  Everything one workgroup writes
// for another to read inside this launch (x, q, o, m, the new K/V row, split-K
// partials, argmax candidates) is written with device-scope atomic stores and
// read with device-scope atomic loads, which are coherent across the L2s on
// their own; ordering comes from completion (the service wave drains its
// vector-memory counter before it arrives).  No release/acquire fence is
// used: on this chip a device-scope release writes back the whole L2 of the
// XCD.  Weights and KV rows of earlier steps are read with ordinary loads.
//
// Every wave reaches every barrier; the spin is bounded (an error word is set
// and token -1 is reported on a timeout), so the grid always drains.
#pragma once
#include "ll_device.h"

#define MK_THREADS 768
#define MK_WAVES (MK_THREADS / 64)
#define MK_CW (MK_WAVES - 1)   // compute waves; wave MK_CW is the service wave
#define MK_U 8                 // 512-element chunks per row and item: one item = 2 rows x 4096 columns
#define MK_MAX_ITEMS 192       // local (pair, K-segment) items of one phase in one workgroup
#define MK_BAR_GROUPS 8
#define MK_BAR_STRIDE 32       // uints between barrier words (own 128-byte line each)
#define MK_BAR_GLOBAL (MK_BAR_GROUPS * MK_BAR_STRIDE)
#define MK_BAR_EPOCH ((MK_BAR_GROUPS + 1) * MK_BAR_STRIDE)   // barriers completed by earlier launches
#define MK_BAR_ERROR ((MK_BAR_GROUPS + 2) * MK_BAR_STRIDE)   // set when a barrier timed out
#define MK_BAR_WORDS ((MK_BAR_GROUPS + 3) * MK_BAR_STRIDE)

enum MkMode { MK_QKV = 0, MK_ORES = 1, MK_GATEUP = 2, MK_DOWN = 3, MK_LMHEAD = 4, MK_NONE = 5 };

struct MkLayer {
  const half_t *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
  half_t *kc, *vc;
};

struct MkArgs {
  const MkLayer* layers;   // device table, n_layers entries
  const half_t *tok_emb, *final_norm, *lm_head;
  float *x, *q, *o, *m, *logits, *attn_part;
  unsigned* attn_cnt;
  float* amax_val;
  int* amax_idx;
  const float2* rope;
  DevState* st;
  int* host_ring;
  unsigned* bar;           // MK_BAR_WORDS uints
  int ring_size;
  int n_layers, d, n_heads, head_dim, F, vocab, max_seq, attn_splits;
  float eps;
  int spin_limit;
  unsigned long long* trace;   // optional: 5 timestamps per phase from workgroup 0's service wave
};

struct MkPhase {
  const half_t *w0, *w1, *w2;
  int mode, npairs, K, nch, nseg, cps;   // nch chunks of 512 in K, split in nseg segments of cps chunks
};

struct MkCtx {
  int tid, lane, wave, b, nb;
  unsigned epoch;      // barriers completed before this launch (all launches ever)
  unsigned gen;        // barriers arrived at in this launch
  unsigned grp_size;   // workgroups in this workgroup's barrier group
  int* s_abort;        // LDS flag: a barrier timed out
  float* lds;          // dynamic LDS: staged input vector (+ zero chunk) | attention scratch
  float* red;          // MK_WAVES floats of reduction scratch
  float* res;          // [MK_MAX_ITEMS][2] raw dot products of the phase
  int phase_no;        // running phase index (trace slot)
  unsigned long long* s_trace;   // LDS [MK_TRACE_PHASES][8]
};

#define MK_TRACE_PHASES 162
// Timestamps go to LDS and are written out once at the end of the kernel, so
// that tracing adds no global stores to the waves it observes.
__device__ __forceinline__ void mk_stamp(const MkArgs& a, const MkCtx& c, int point) {
  if (a.trace && c.b == 0 && c.phase_no < MK_TRACE_PHASES) c.s_trace[c.phase_no * 8 + point] = wall_clock64();
}
__device__ __forceinline__ void mk_trace(const MkArgs& a, const MkCtx& c, int point) {
  if (c.tid == MK_CW * 64) mk_stamp(a, c, point);
}

// Service wave only: all of its stores have completed -> arrive (group counter
// first, the last of a group forwards to the global counter) -> spin until the
// barrier completes.  The other waves wait at the workgroup barrier that follows.
__device__ __forceinline__ void svc_arrive_and_wait(const MkArgs& a, MkCtx& c) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (c.lane == 0) mk_stamp(a, c, 3);
  if (c.lane == 0 && !*c.s_abort) {
    const unsigned gen = c.gen + 1;
    const unsigned t = __hip_atomic_fetch_add(a.bar + (c.b % MK_BAR_GROUPS) * MK_BAR_STRIDE, 1u,
                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t + 1u == (c.epoch + gen) * c.grp_size)
      __hip_atomic_fetch_add(a.bar + MK_BAR_GLOBAL, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int ngroups = c.nb < MK_BAR_GROUPS ? c.nb : MK_BAR_GROUPS;
    const unsigned target = (c.epoch + gen) * (unsigned)ngroups;
    int spins = 0;
    while ((int)(__hip_atomic_load(a.bar + MK_BAR_GLOBAL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) -
                 target) < 0) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins > a.spin_limit) {
        *c.s_abort = 1;
        __hip_atomic_store(a.bar + MK_BAR_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
  }
}

// number of row pairs of a phase this workgroup owns (pair p belongs to workgroup p % nb)
__device__ __forceinline__ int local_pairs(const MkPhase& ph, const MkCtx& c) {
  return c.b < ph.npairs ? (ph.npairs - c.b + c.nb - 1) / c.nb : 0;
}

struct MkItem {
  const half_t *pa, *pb;
  int rowA, rowB, sec, pair, seg;
  bool valid;
};

// local item li of a phase -> (pair, K segment) -> the two weight rows
__device__ __forceinline__ MkItem mk_item(const MkArgs& a, const MkPhase& ph, const MkCtx& c, int li) {
  MkItem it;
  const int lp = li / ph.nseg;
  it.seg = li - lp * ph.nseg;
  it.pair = lp * c.nb + c.b;
  it.valid = ph.mode != MK_NONE && li >= 0 && it.pair < ph.npairs;
  it.sec = 0;
  it.rowA = it.rowB = 0;
  it.pa = it.pb = ph.w0;
  if (!it.valid) return it;
  const int p = it.pair, K = ph.K;
  if (ph.mode == MK_QKV) {
    const int d_half = a.d >> 1;
    it.sec = p / d_half;
    const int pp = p - it.sec * d_half;
    const half_t* base = it.sec == 0 ? ph.w0 : (it.sec == 1 ? ph.w1 : ph.w2);
    if (it.sec < 2) {
      const int hh = a.head_dim >> 1;
      const int head = pp / hh, j = pp - head * hh;
      it.rowA = head * a.head_dim + j;
      it.rowB = it.rowA + hh;
    } else {
      it.rowA = 2 * pp;
      it.rowB = it.rowA + 1;
    }
    it.pa = base + (size_t)it.rowA * K;
    it.pb = base + (size_t)it.rowB * K;
  } else if (ph.mode == MK_GATEUP) {
    it.rowA = it.rowB = p;
    it.pa = ph.w0 + (size_t)p * K;
    it.pb = ph.w1 + (size_t)p * K;
  } else {
    const int nrows = ph.mode == MK_LMHEAD ? a.vocab : a.d;
    it.rowA = 2 * p;
    it.rowB = min(it.rowA + 1, nrows - 1);
    it.pa = ph.w0 + (size_t)it.rowA * K;
    it.pb = ph.w0 + (size_t)it.rowB * K;
  }
  return it;
}

__device__ __forceinline__ void mk_load(const MkPhase& ph, const MkItem& it, int lane, h8 (&wa)[MK_U],
                                        h8 (&wb)[MK_U]) {
  if (!it.valid) return;
  const int gc0 = it.seg * ph.cps;
#pragma unroll
  for (int u = 0; u < MK_U; ++u) {
    const int k = min((gc0 + u) * 512 + lane * 8, ph.K - 8);
    wa[u] = load_stream(it.pa + k);
    wb[u] = load_stream(it.pb + k);
  }
}

__device__ __forceinline__ void mk_dot(const MkPhase& ph, const MkItem& it, const MkCtx& c,
                                       const h8 (&wa)[MK_U], const h8 (&wb)[MK_U], float& accA,
                                       float& accB) {
  const int gc0 = it.seg * ph.cps;
  accA = accB = 0.f;
#pragma unroll
  for (int u = 0; u < MK_U; ++u) {
    const int gc = gc0 + u;
    const int xc = (u < ph.cps && gc < ph.nch) ? gc : ph.nch;   // chunk nch of the staging area is zero
    const float* xp = c.lds + xc * 512 + c.lane * 4;
    const f4 x0 = *reinterpret_cast<const f4*>(xp);
    const f4 x1 = *reinterpret_cast<const f4*>(xp + 256);
    accA = dot8(wa[u], x0, x1, accA);
    accB = dot8(wb[u], x0, x1, accB);
  }
  accA = wave_sum(accA);
  accB = wave_sum(accB);
}

// Stage the phase's input vector in LDS (lane-major chunks, one zero chunk
// behind the data) from device-coherent memory; with NORM, multiply by the
// gain and return rsqrt(mean x^2 + eps).  `emb` (layer 0 only) replaces x by
// the fp16 embedding row of the token being fed.
__device__ __forceinline__ float mk_stage(const MkCtx& c, const float* xin, const half_t* emb,
                                          const half_t* gain, int K, int nch, float eps, bool norm) {
  float ss = 0.f;
  const int n2 = (nch + 1) * 256;   // float2 slots including the zero chunk
  for (int i = c.tid; i < n2; i += MK_THREADS) {
    const int k = i * 2;
    float2 v = make_float2(0.f, 0.f);
    if (k < K) {
      if (emb) {
        const unsigned int e2 = *as_global(reinterpret_cast<const unsigned int*>(emb + k));
        v.x = (float)__builtin_bit_cast(half_t, (unsigned short)(e2 & 0xffffu));
        v.y = (float)__builtin_bit_cast(half_t, (unsigned short)(e2 >> 16));
      } else {
        v = ld_dev2(xin + k);
      }
      if (norm) {
        ss += v.x * v.x + v.y * v.y;
        const unsigned int g2 = *as_global(reinterpret_cast<const unsigned int*>(gain + k));
        v.x *= (float)__builtin_bit_cast(half_t, (unsigned short)(g2 & 0xffffu));
        v.y *= (float)__builtin_bit_cast(half_t, (unsigned short)(g2 >> 16));
      }
    }
    const int ch = k >> 9, r = k & 511;
    *reinterpret_cast<float2*>(c.lds + ch * 512 + ((r >> 2) & 1) * 256 + (r >> 3) * 4 + (r & 3)) = v;
  }
  float inv = 1.f;
  if (norm) {
    ss = wave_sum(ss);
    if (c.lane == 0) c.red[c.wave] = ss;
  }
  __syncthreads();
  if (norm) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < MK_WAVES; ++w) t += c.red[w];
    inv = 1.0f / sqrtf(t / (float)K + eps);
  }
  return inv;
}

// Epilogue of one row pair, run by one lane of the service wave.
template <int MODE>
__device__ __forceinline__ void mk_epilogue(const MkArgs& a, const MkItem& it, float accA, float accB,
                                            const half_t* emb, int layer, int pos, float& best_v,
                                            int& best_i) {
  if (MODE == MK_QKV) {
    if (it.sec < 2) {
      const int hh = a.head_dim >> 1;
      const int head = it.rowA / a.head_dim, j = it.rowA - head * a.head_dim;
      const float2 cs = a.rope[(size_t)pos * hh + j];
      const float ra = accA * cs.x - accB * cs.y;
      const float rb = accB * cs.x + accA * cs.y;
      if (it.sec == 0) {
        st_dev(a.q + it.rowA, ra);
        st_dev(a.q + it.rowB, rb);
      } else {
        half_t* kr = a.layers[layer].kc + ((size_t)head * a.max_seq + pos) * a.head_dim;
        st_dev_h(kr + j, ra);
        st_dev_h(kr + j + hh, rb);
      }
    } else {
      const int head = it.rowA / a.head_dim, e = it.rowA - head * a.head_dim;
      half_t* vr = a.layers[layer].vc + ((size_t)head * a.max_seq + pos) * a.head_dim;
      st_dev_h(vr + e, accA);
      st_dev_h(vr + e + 1, accB);
    }
  } else if (MODE == MK_GATEUP) {
    st_dev(a.m + it.pair, accA / (1.0f + expf(-accA)) * accB);
  } else if (MODE == MK_ORES || MODE == MK_DOWN) {
    // layer 0: the residual stream is still the embedding row of the fed token
    const float oldA = emb ? (float)as_global(emb)[it.rowA] : ld_dev(a.x + it.rowA);
    st_dev(a.x + it.rowA, oldA + accA);
    if (it.rowB != it.rowA) {
      const float oldB = emb ? (float)as_global(emb)[it.rowB] : ld_dev(a.x + it.rowB);
      st_dev(a.x + it.rowB, oldB + accB);
    }
  } else {   // MK_LMHEAD
    a.logits[it.rowA] = accA;
    if (accA > best_v) { best_v = accA; best_i = it.rowA; }        // rows ascend per lane:
    if (it.rowB != it.rowA) {                                      // '>' keeps the lowest index
      a.logits[it.rowB] = accB;
      if (accB > best_v) { best_v = accB; best_i = it.rowB; }
    }
  }
}

// One GEMV phase.  On entry the workgroup has passed the grid barrier that
// guards the phase's input, and wa/wb of every compute wave hold (in flight)
// its first item of the phase; on exit they hold its first item of `next` and
// the workgroup has passed the barrier that publishes this phase's output.
template <int MODE>
__device__ __forceinline__ void mk_gemv_phase(const MkArgs& a, MkCtx& c, const MkPhase& ph,
                                              const MkPhase& next, const float* xin,
                                              const half_t* emb_stage, const half_t* emb_res,
                                              const half_t* gain, int layer, h8 (&wa)[MK_U],
                                              h8 (&wb)[MK_U]) {
  constexpr bool NORM = (MODE == MK_QKV || MODE == MK_GATEUP || MODE == MK_LMHEAD);
  mk_trace(a, c, 0);
  const float inv = mk_stage(c, xin, emb_stage, gain, ph.K, ph.nch, a.eps, NORM);
  mk_trace(a, c, 1);
  const int n_pairs = local_pairs(ph, c);
  const int n_items = n_pairs * ph.nseg;

  if (c.wave < MK_CW) {
    bool prefetched = false;
    for (int li = c.wave; li < n_items || !prefetched; li += MK_CW) {
      const bool have = li < n_items;
      float accA = 0.f, accB = 0.f;
      MkItem it = mk_item(a, ph, c, have ? li : -1);
      if (c.tid == 0 && li == 0) mk_stamp(a, c, 5);
      if (have) mk_dot(ph, it, c, wa, wb, accA, accB);
      if (c.tid == 0 && li == 0) mk_stamp(a, c, 6);
      // keep the weight stream going: next item of this phase, else first item of the next phase
      if (li + MK_CW < n_items) {
        mk_load(ph, mk_item(a, ph, c, li + MK_CW), c.lane, wa, wb);
      } else {
        mk_load(next, mk_item(a, next, c, c.wave), c.lane, wa, wb);
        prefetched = true;
      }
      if (c.tid == 0 && li == 0) mk_stamp(a, c, 7);
      if (have && c.lane == 0) {
        c.res[li * 2] = accA;
        c.res[li * 2 + 1] = accB;
      }
    }
  }
  __syncthreads();   // raw dot products are in LDS
  mk_trace(a, c, 2);

  if (c.wave == MK_CW) {
    const int pos = a.st->pos;
    float best_v = -INFINITY;
    int best_i = 0x7fffffff;
    for (int lp = c.lane; lp < n_pairs; lp += 64) {
      float accA = 0.f, accB = 0.f;
      for (int s = 0; s < ph.nseg; ++s) {   // K segments in a fixed order
        accA += c.res[(lp * ph.nseg + s) * 2];
        accB += c.res[(lp * ph.nseg + s) * 2 + 1];
      }
      const MkItem it = mk_item(a, ph, c, lp * ph.nseg);
      mk_epilogue<MODE>(a, it, accA * inv, accB * inv, emb_res, layer, pos, best_v, best_i);
    }
    if (MODE == MK_LMHEAD) {
      // wave argmax (value desc, index asc)
      for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(best_v, off);
        const int oi = __shfl_xor(best_i, off);
        if (ov > best_v || (ov == best_v && oi < best_i)) { best_v = ov; best_i = oi; }
      }
      if (c.lane == 0) {
        st_dev(a.amax_val + c.b, best_v);
        st_dev_i(a.amax_idx + c.b, best_i);
      }
    }
    svc_arrive_and_wait(a, c);
  }
  mk_trace(a, c, 4);
  c.gen += 1;
  c.phase_no += 1;
  __syncthreads();   // grid barrier passed
}

// Attention phase: workgroups [0, n_heads * S) each take (head, split); same
// lane-group online softmax as the stand-alone kernel, 12 waves per workgroup.
template <int HD>
__device__ __forceinline__ void mk_attn_phase(const MkArgs& a, MkCtx& c, int layer) {
  constexpr int LPR = HD / 8, GPW = 64 / LPR, NG = MK_WAVES * GPW, UK = 2, PS = HD + 2;
  const int S = a.attn_splits;
  const bool active = c.b < a.n_heads * S;
  mk_trace(a, c, 0);
  float* s_m = c.lds;               // [NG]
  float* s_l = c.lds + NG;          // [NG]
  float* s_acc = c.lds + 2 * NG;    // [NG][HD]
  float* s_part = c.lds + 2 * NG + NG * HD;   // [PS] this workgroup's merged partial
  const int h = active ? c.b / S : 0, s = active ? c.b - h * S : 0;
  if (active) {
    const int gi = c.lane / LPR, li = c.lane % LPR;
    const int pos = a.st->pos, n_keys = pos + 1;
    const float scale = 1.0f / sqrtf((float)HD);
    float qv[8];
    {
      const float* qp = a.q + h * HD + li * 8;
      const float2 q0 = ld_dev2(qp), q1 = ld_dev2(qp + 2), q2 = ld_dev2(qp + 4), q3 = ld_dev2(qp + 6);
      qv[0] = q0.x * scale; qv[1] = q0.y * scale; qv[2] = q1.x * scale; qv[3] = q1.y * scale;
      qv[4] = q2.x * scale; qv[5] = q2.y * scale; qv[6] = q3.x * scale; qv[7] = q3.y * scale;
    }
    const half_t* kh = a.layers[layer].kc + (size_t)h * a.max_seq * HD + li * 8;
    const half_t* vh = a.layers[layer].vc + (size_t)h * a.max_seq * HD + li * 8;
    float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const int stride = S * MK_WAVES * GPW;
    for (int base = (s * MK_WAVES + c.wave) * GPW; base < n_keys; base += stride * UK) {
      h8 kk[UK], vv[UK];
#pragma unroll
      for (int j = 0; j < UK; ++j) {
        const int u = min(base + j * stride + gi, n_keys - 1);
        if (u == pos) {   // the row this launch wrote: read it coherently
          kk[j] = ld_dev_h8(kh + (size_t)u * HD);
          vv[j] = ld_dev_h8(vh + (size_t)u * HD);
        } else {
          kk[j] = load_h8(kh + (size_t)u * HD);
          vv[j] = load_h8(vh + (size_t)u * HD);
        }
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
    const int g = c.wave * GPW + gi;
    if (li == 0) { s_m[g] = m; s_l[g] = l; }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[g * HD + li * 8 + e] = acc[e];
  }
  __syncthreads();
  if (active && c.tid < HD) {   // merge the lane groups of this workgroup (LDS only)
    float M = -INFINITY;
    for (int i = 0; i < NG; ++i) M = fmaxf(M, s_m[i]);
    float L = 0.f, A = 0.f;
    if (M > -INFINITY) {
      for (int i = 0; i < NG; ++i) {
        const float w = __expf(s_m[i] - M);
        L += s_l[i] * w;
        A += s_acc[i * HD + c.tid] * w;
      }
    }
    if (c.tid == 0) { s_part[0] = M; s_part[1] = L; }
    s_part[2 + c.tid] = A;
  }
  __syncthreads();
  mk_trace(a, c, 2);
  if (c.wave == MK_CW) {
    if (active) {
      float* mypart = a.attn_part + ((size_t)h * S + s) * PS;
      for (int i = c.lane; i < PS; i += 64) st_dev(mypart + i, s_part[i]);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      unsigned t = 0;
      if (c.lane == 0)
        t = __hip_atomic_fetch_add(a.attn_cnt + h, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      t = (unsigned)__builtin_amdgcn_readfirstlane((int)t);
      if (t == (unsigned)(S - 1)) {   // last split of this head to arrive merges all S
        const float* hp = a.attn_part + (size_t)h * S * PS;
        float M = -INFINITY;
        for (int i = 0; i < S; ++i) M = fmaxf(M, ld_dev(hp + i * PS));
        for (int dcol = c.lane; dcol < HD; dcol += 64) {
          float L = 0.f, A = 0.f;
          for (int i = 0; i < S; ++i) {
            const float mi = ld_dev(hp + i * PS);
            const float w = (mi > -INFINITY) ? __expf(mi - M) : 0.f;
            L += ld_dev(hp + i * PS + 1) * w;
            A += ld_dev(hp + i * PS + 2 + dcol) * w;
          }
          st_dev(a.o + h * HD + dcol, A / L);
        }
        if (c.lane == 0) __hip_atomic_store(a.attn_cnt + h, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    svc_arrive_and_wait(a, c);
  }
  mk_trace(a, c, 4);
  c.gen += 1;
  c.phase_no += 1;
  __syncthreads();
}

__device__ __forceinline__ MkPhase mk_phase(const MkArgs& a, int mode, int layer) {
  MkPhase p;
  p.w0 = p.w1 = p.w2 = nullptr;
  p.mode = mode;
  p.npairs = 0;
  p.K = a.d;
  if (mode != MK_NONE && mode != MK_LMHEAD) {
    const MkLayer& L = a.layers[layer];
    if (mode == MK_QKV) { p.w0 = L.wq; p.w1 = L.wk; p.w2 = L.wv; p.npairs = 3 * (a.d >> 1); }
    else if (mode == MK_ORES) { p.w0 = L.wo; p.npairs = a.d >> 1; }
    else if (mode == MK_GATEUP) { p.w0 = L.w_gate; p.w1 = L.w_up; p.npairs = a.F; }
    else { p.w0 = L.w_down; p.npairs = a.d >> 1; p.K = a.F; }
  } else if (mode == MK_LMHEAD) {
    p.w0 = a.lm_head;
    p.npairs = (a.vocab + 1) >> 1;
  }
  p.nch = (p.K + 511) >> 9;
  p.nseg = (p.nch + MK_U - 1) / MK_U;
  p.cps = (p.nch + p.nseg - 1) / p.nseg;
  return p;
}

__global__ __launch_bounds__(MK_THREADS) void decode_mega_kernel(MkArgs a) {
  extern __shared__ float mk_lds[];
  __shared__ float s_red[MK_WAVES];
  __shared__ float s_res[MK_MAX_ITEMS * 2];
  __shared__ int s_abort;
  __shared__ unsigned long long s_trace[MK_TRACE_PHASES * 8];
  MkCtx c;
  c.tid = threadIdx.x;
  c.lane = c.tid & 63;
  c.wave = c.tid >> 6;
  c.b = blockIdx.x;
  c.nb = gridDim.x;
  c.epoch = a.bar[MK_BAR_EPOCH];
  c.gen = 0;
  c.phase_no = 0;
  {
    const int g = c.b % MK_BAR_GROUPS;
    c.grp_size = (unsigned)((c.nb - g + MK_BAR_GROUPS - 1) / MK_BAR_GROUPS);
  }
  c.s_abort = &s_abort;
  c.lds = mk_lds;
  c.red = s_red;
  c.res = s_res;
  c.s_trace = s_trace;
  if (a.trace && c.b == 0)
    for (int i = c.tid; i < MK_TRACE_PHASES * 8; i += MK_THREADS) s_trace[i] = 0;
  if (c.tid == 0) s_abort = 0;
  __syncthreads();

  const int tok = a.st->next_token;
  const half_t* emb_row = a.tok_emb + (size_t)tok * a.d;

  h8 wa[MK_U], wb[MK_U];
  MkPhase cur = mk_phase(a, MK_QKV, 0);
  if (c.wave < MK_CW) mk_load(cur, mk_item(a, cur, c, c.wave), c.lane, wa, wb);

  for (int l = 0; l < a.n_layers; ++l) {
    const MkLayer& L = a.layers[l];
    const half_t* emb = (l == 0) ? emb_row : nullptr;
    MkPhase nxt = mk_phase(a, MK_ORES, l);
    mk_gemv_phase<MK_QKV>(a, c, cur, nxt, a.x, emb, nullptr, L.attn_norm, l, wa, wb);
    if (a.head_dim == 128) mk_attn_phase<128>(a, c, l);
    else mk_attn_phase<64>(a, c, l);
    cur = nxt;
    nxt = mk_phase(a, MK_GATEUP, l);
    mk_gemv_phase<MK_ORES>(a, c, cur, nxt, a.o, nullptr, emb, nullptr, l, wa, wb);
    cur = nxt;
    nxt = mk_phase(a, MK_DOWN, l);
    mk_gemv_phase<MK_GATEUP>(a, c, cur, nxt, a.x, nullptr, nullptr, L.ffn_norm, l, wa, wb);
    cur = nxt;
    nxt = (l + 1 < a.n_layers) ? mk_phase(a, MK_QKV, l + 1) : mk_phase(a, MK_LMHEAD, 0);
    mk_gemv_phase<MK_DOWN>(a, c, cur, nxt, a.m, nullptr, nullptr, nullptr, l, wa, wb);
    cur = nxt;
  }
  {
    const MkPhase none = mk_phase(a, MK_NONE, 0);
    mk_gemv_phase<MK_LMHEAD>(a, c, cur, none, a.x, nullptr, nullptr, a.final_norm, 0, wa, wb);
  }

  if (a.trace && c.b == 0) {
    __syncthreads();
    const int n = (c.phase_no < MK_TRACE_PHASES ? c.phase_no : MK_TRACE_PHASES) * 8;
    for (int i = c.tid; i < n; i += MK_THREADS) a.trace[i] = s_trace[i];
  }

  // sampling: workgroup 0 reduces the per-workgroup candidates and advances the state
  if (c.b == 0 && c.wave == MK_CW) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = c.lane; i < c.nb; i += 64) {
      const float v = ld_dev(a.amax_val + i);
      const int ix = ld_dev_i(a.amax_idx + i);
      if (v > bv || (v == bv && ix < bi)) { bv = v; bi = ix; }
    }
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (c.lane == 0) {
      int t = bi == 0x7fffffff ? 0 : bi;
      if (s_abort || a.bar[MK_BAR_ERROR]) t = -1;
      const int idx = a.st->steps;
      a.st->pos = a.st->pos + 1;
      a.st->steps = idx + 1;
      a.st->next_token = t < 0 ? 0 : t;
      a.bar[MK_BAR_EPOCH] = c.epoch + c.gen;
      if (idx < a.ring_size) a.host_ring[idx] = t;
    }
  }
}
