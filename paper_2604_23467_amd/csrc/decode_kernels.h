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

#define ATTN_THREADS 1024
#define ATTN_MERGE_MAX 4     // attention partials per head that the O projection's prologue merges
#define ATTN_PART_STRIDE(HD) ((HD) + 4)   // floats per attention partial: m, l, 2 pad, acc[HD] (16-byte aligned)

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
  // O projection prologue: the input vector is the merge of attn_splits split-K partials per head
  const float* attn_part;
  int attn_splits;
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
// Threads per workgroup: the O projection, whose every workgroup merges all of the attention partials
// while it stages them, runs workgroups of 8 waves (half as many stagings for the same row pairs)
#define GEMV_WG(MODE) ((MODE) == GM_ORES ? 2 * LL_WG : LL_WG)
template <int MODE, int U>
__global__ __launch_bounds__(GEMV_WG(MODE)) void gemv_kernel(GemvArgs a) {
  extern __shared__ float lds[];
  constexpr int WG = GEMV_WG(MODE);
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

  const int gw = blockIdx.x * (WG / 64) + wave, GW = gridDim.x * (WG / 64);

  const float* xin = a.xin;
  if (MODE == GM_LMHEAD && a.x_row_from_prompt) xin += (size_t)(a.st->n_prompt - 1) * K;

  // Staging of the input vector, four float4 per thread and pass, all of a pass's loads issued before
  // any is used (one L2 round trip, not four).  For the O projection in two separate steps (loads;
  // arithmetic and LDS writes) and branch-free (addresses clamped, values selected afterwards), so that
  // the weight loads can be requested in between and the wait in front of the LDS writes leaves exactly
  // them in flight.
  // O projection: its input is the merge of the attention kernel's (at most ATTN_MERGE_MAX) partials per
  // head, o = sum_s w_s acc_s with w_s = exp(m_s - M) / sum_s l_s exp(m_s - M).  Every thread
  // fetches the (m, l) headers next to the accumulators it stages and forms the weights
  // itself, so the whole merge costs one L2 round trip and no extra barrier.
  constexpr int SU = MODE == GM_ORES ? 2 : 4;      // 512 threads x 2 x 4 elements cover d_model 4096 in one pass
  constexpr int MP = MODE == GM_ORES ? ATTN_MERGE_MAX : 1;    // partials merged in the prologue
  struct StageRegs {
    f4 v[MP][SU];
    float2 hd[MP][SU];           // (m, l) of the partials
  };
  auto stage_load = [&](int i0, StageRegs& R) {
#pragma unroll
    for (int j = 0; j < SU; ++j) {
      const int k = (i0 + j * WG) * 4;
      const int kc = min(k, K - 4);                     // K % 8 == 0
      // o[k..k+3] of head k / head_dim: the partial accumulators; without partials (long-context
      // instances merge in a kernel of their own) the merged vector itself
      const int HD = a.head_dim, PS = ATTN_PART_STRIDE(HD);
      const int head = kc / HD, dcol = kc - head * HD;
      const bool parts = a.attn_part != nullptr;
      const float* hb = parts ? a.attn_part + (size_t)head * a.attn_splits * PS : xin;
      const float* hp = parts ? hb + 4 + dcol : xin + kc;
#pragma unroll
      for (int sp = 0; sp < MP; ++sp) {
        const int off = parts ? min(sp, a.attn_splits - 1) * PS : 0;    // a missing partial re-reads the last one
        R.v[sp][j] = *reinterpret_cast<const f4*>(hp + off);
        R.hd[sp][j] = *reinterpret_cast<const float2*>(hb + off);
      }
    }
  };
  float ss = 0.f;
  auto stage_store = [&](int i0, const StageRegs& R) {
#pragma unroll
    for (int j = 0; j < SU; ++j) {
      const int k = (i0 + j * WG) * 4;
      if (k >= nchp * 512) continue;
      const bool parts = a.attn_part != nullptr;
      const int np = parts ? a.attn_splits : 0;
      float M = -INFINITY;
#pragma unroll
      for (int sp = 0; sp < MP; ++sp) M = fmaxf(M, sp < np ? R.hd[sp][j].x : -INFINITY);
      float e[MP], den = 0.f;
#pragma unroll
      for (int sp = 0; sp < MP; ++sp) {
        const float m = R.hd[sp][j].x;
        e[sp] = (sp < np && m > -INFINITY) ? __expf(m - M) : 0.f;
        den += R.hd[sp][j].y * e[sp];
      }
      const float rl = 1.0f / den;
      f4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int sp = 0; sp < MP; ++sp) {
        const float w = parts ? e[sp] * rl : (sp == 0 ? 1.0f : 0.f);
        t[0] += R.v[sp][j][0] * w; t[1] += R.v[sp][j][1] * w; t[2] += R.v[sp][j][2] * w; t[3] += R.v[sp][j][3] * w;
      }
      if (k >= K) t = f4{0.f, 0.f, 0.f, 0.f};          // padding up to a whole group of chunks
      const int c = k >> 9, r = k & 511;
      *reinterpret_cast<f4*>(lds + c * 512 + ((r >> 2) & 1) * 256 + (r >> 3) * 4) = t;
    }
  };

  // Order of the first requests.  The weight stream does not depend on the input vector, and the time
  // of these kernels is the time of that stream: the first loads of this wave's first row pair go out
  // before anything else (measured: the staging loads in front of them cost 1 % of a step).  The O
  // projection is the exception: at one row pair per wave those first loads are ALL of its weights, and
  // loads return in order, so staging requested behind them would start only when the stream has ended;
  // there the (small, cached) partials are requested first and merged while the weights arrive.
  if constexpr (MODE == GM_ORES) {
    StageRegs R;
    stage_load(tid, R);
    __builtin_amdgcn_sched_barrier(0);
    select_rows(min(gw, P - 1));                       // a wave without a pair fetches the last one's start: no branch
    load_group(0);
    __builtin_amdgcn_sched_barrier(0);
    stage_store(tid, R);
    for (int i0 = tid + WG * SU; i0 < nchp * 128; i0 += WG * SU) {   // K > 4096 (8192 with 8 waves)
      stage_load(i0, R);
      stage_store(i0, R);
    }
  } else if constexpr (MODE == GM_QKV || MODE == GM_GATEUP) {
    // Normalising projections of a layer (the LM head, with many row pairs per wave, measured no gain):
    // the raw vector and the gains go global -> LDS directly (no registers), requested in front of the
    // weights, each wave its own chunks; when they have landed (the weight
    // loads behind them stay in flight) the same lanes multiply the gains in, in place, and add up the
    // squares.  The prologue thus never waits for the weight stream's first loads.
    half_t* gl = reinterpret_cast<half_t*>(red + 16);
    for (int c = wave; c < nch; c += LL_WG / 64) {
      const int k = min(c * 512 + lane * 8, K - 8);            // K % 8 == 0: a lane's 8 elements are all in or all out
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)(xin + k),
                                       (__attribute__((address_space(3))) void*)(lds + c * 512), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)(xin + k + 4),
                                       (__attribute__((address_space(3))) void*)(lds + c * 512 + 256), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)(a.gain + k),
                                       (__attribute__((address_space(3))) void*)(gl + c * 512), 16, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    select_rows(min(gw, P - 1));          // unconditional: the wait below counts on 16 younger loads in every wave
    load_group(0);
    __builtin_amdgcn_sched_barrier(0);
    wait_vm_at_most<16>();
    asm volatile("" ::: "memory");
    for (int c = wave; c < nchp; c += LL_WG / 64) {
      float* xp = lds + c * 512 + lane * 4;
      f4 x0 = {0.f, 0.f, 0.f, 0.f}, x1 = x0;
      if (c < nch && c * 512 + lane * 8 < K) {
        x0 = *reinterpret_cast<const f4*>(xp);
        x1 = *reinterpret_cast<const f4*>(xp + 256);
        const h8 gv = *reinterpret_cast<const h8*>(gl + c * 512 + lane * 8);
        ss += x0[0] * x0[0] + x0[1] * x0[1] + x0[2] * x0[2] + x0[3] * x0[3] +
              x1[0] * x1[0] + x1[1] * x1[1] + x1[2] * x1[2] + x1[3] * x1[3];
#pragma unroll
        for (int e = 0; e < 4; ++e) { x0[e] *= (float)gv[e]; x1[e] *= (float)gv[4 + e]; }
      }
      *reinterpret_cast<f4*>(xp) = x0;                          // also the zero padding beyond K and up to nchp chunks
      *reinterpret_cast<f4*>(xp + 256) = x1;
    }
  } else {
    if (gw < P) {
      select_rows(gw);
      load_group(0);
    }
    for (int i0 = tid; i0 < nchp * 128; i0 += LL_WG * SU) {
      f4 v[SU];
      h4 g[SU];
#pragma unroll
      for (int j = 0; j < SU; ++j) {
        const int k = (i0 + j * LL_WG) * 4;
        v[j] = f4{0.f, 0.f, 0.f, 0.f};
        g[j] = h4{0, 0, 0, 0};
        if (k < K) {
          v[j] = *reinterpret_cast<const f4*>(xin + k);
          if (NORM) g[j] = *reinterpret_cast<const h4*>(a.gain + k);
        }
      }
#pragma unroll
      for (int j = 0; j < SU; ++j) {
        const int k = (i0 + j * LL_WG) * 4;
        if (k >= nchp * 512) continue;
        f4 t = v[j];
        if (NORM) {
          ss += t[0] * t[0] + t[1] * t[1] + t[2] * t[2] + t[3] * t[3];
          t[0] *= (float)g[j][0]; t[1] *= (float)g[j][1]; t[2] *= (float)g[j][2]; t[3] *= (float)g[j][3];
        }
        const int c = k >> 9, r = k & 511;
        *reinterpret_cast<f4*>(lds + c * 512 + ((r >> 2) & 1) * 256 + (r >> 3) * 4) = t;
      }
    }
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
  int qkv_pos = 0;
  if (MODE == GM_QKV) qkv_pos = a.st->pos;

  for (int p = gw; p < P; p += GW) {
    if (p != gw) select_rows(p);
    // What the epilogue will need besides the sums does not depend on them: fetch it now, so the
    // row pair ends without a memory round trip (the residual it adds to, or its RoPE factors).
    float pre0 = 0.f, pre1 = 0.f;
    float2 pcs = make_float2(1.f, 0.f);
    if (MODE == GM_ORES || MODE == GM_DOWN) {
      if (lane == 0) { pre0 = *as_global(a.out + rowA); pre1 = *as_global(a.out + rowB); }
    } else if (MODE == GM_QKV) {
      if (sec < 2) {
        const int head = rowA / a.head_dim, j = rowA - head * a.head_dim;
        pcs = a.rope[(size_t)qkv_pos * (a.head_dim >> 1) + j];
      }
    }
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
      const int pos = qkv_pos;
      if (sec < 2) {
        const int hh = a.head_dim >> 1;
        const int head = rowA / a.head_dim, j = rowA - head * a.head_dim;
        const float2 cs = pcs;
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
        a.out[rowA] = pre0 + accA;
        if (rowB != rowA) a.out[rowB] = pre1 + accB;
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

// Residual GEMV for long rows (K > 4096, i.e. the down projection): x += W m.
// A 22 KB row pair handled by one wave is a serial chain of three load groups;
// here every wave takes one K segment of at most 8 chunks instead, so ALL loads
// of the kernel are issued up front.  Workgroup = 4 row pairs x NSEG segments
// (NSEG waves per pair, adjacent), the NSEG partial sums meet in LDS.  grid =
// ceil(pairs / 4), one pass, no loop.
template <int NSEG>
__global__ __launch_bounds__(NSEG * 256, 6) void gemv_ksplit_kernel(GemvArgs a) {
  extern __shared__ float lds[];
  constexpr int NT = NSEG * 256;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K;
  const int nch = (K + 511) >> 9;
  const int cps = (nch + NSEG - 1) / NSEG;      // chunks per segment, <= 8
  float* part = lds + (nch + 1) * 512;          // [4 * NSEG][2]
  const int P = a.N >> 1;
  const int pl = wave / NSEG, seg = wave - pl * NSEG;
  const int p = blockIdx.x * 4 + pl;
  const bool valid = p < P;
  const int rowA = 2 * min(p, P - 1), rowB = rowA + 1;
  const half_t* pa = a.w0 + (size_t)rowA * K;
  const half_t* pb = a.w0 + (size_t)rowB * K;
  const int gc0 = seg * cps;

  // The input vector goes global -> LDS directly, requested BEFORE the weights.  This kernel requests all
  // of its weights at once and loads return in order, so staging requested behind them would start only
  // when the weight stream has ended; in front of them it needs no registers (16-byte direct loads, lane
  // l of half-chunk (c, f) fetching x[c * 512 + l * 8 + 4 f ..], which is exactly the lane-major layout
  // the dot products read) and is over long before the first weights arrive.
  constexpr int XL = (22 * 2 + NT / 64 - 1) / (NT / 64);      // direct loads per wave for K <= 11264
  const bool direct = nch <= 22;
  if (direct) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int c2 = wave + i * (NT / 64);                     // wave-uniform
      if (c2 >= 2 * nch) break;
      const int c = c2 >> 1, f = c2 & 1;
      const int k = min(c * 512 + lane * 8 + 4 * f, K - 4);    // ragged tail: clamped here, zeroed below
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)(a.xin + k),
                                       (__attribute__((address_space(3))) void*)(lds + c * 512 + f * 256), 16, 0, 0);
    }
  }
  h8 wa[8], wb[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int k = min((gc0 + u) * 512 + lane * 8, K - 8);
    wa[u] = load_stream(pa + k);
    wb[u] = load_stream(pb + k);
  }
  // the residual values the last step adds to, fetched up front
  float pre0 = 0.f, pre1 = 0.f;
  if (valid && seg == 0 && lane == 0) { pre0 = *as_global(a.out + rowA); pre1 = *as_global(a.out + rowB); }

  if (direct) {
    wait_vm_at_most<16>();          // the direct loads have landed; the 16 weight loads behind them may be in flight
    asm volatile("" ::: "memory");
    // zeros: chunk nch, and what lies beyond K in the last chunk (written by the wave that loaded there)
    for (int i = tid; i < 128; i += NT) *reinterpret_cast<f4*>(lds + nch * 512 + i * 4) = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int c2 = wave + i * (NT / 64);
      const int c = c2 >> 1, f = c2 & 1;
      if (c2 < 2 * nch && c * 512 + lane * 8 + 4 * f >= K)
        *reinterpret_cast<f4*>(lds + c * 512 + f * 256 + lane * 4) = f4{0.f, 0.f, 0.f, 0.f};
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();    // bare: __syncthreads() would wait for the weights
    asm volatile("" ::: "memory");
  } else {
    for (int i = tid; i < (nch + 1) * 128; i += NT) {   // chunk nch stays zero
      const int k = i * 4;
      f4 v = {0.f, 0.f, 0.f, 0.f};
      if (k < K) v = *reinterpret_cast<const f4*>(a.xin + k);
      const int c = k >> 9, r = k & 511;
      *reinterpret_cast<f4*>(lds + c * 512 + ((r >> 2) & 1) * 256 + (r >> 3) * 4) = v;
    }
    __syncthreads();
  }

  float accA = 0.f, accB = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int gc = gc0 + u;
    const int xc = (u < cps && gc < nch) ? gc : nch;
    const float* xp = lds + xc * 512 + lane * 4;
    const f4 x0 = *reinterpret_cast<const f4*>(xp);
    const f4 x1 = *reinterpret_cast<const f4*>(xp + 256);
    accA = dot8(wa[u], x0, x1, accA);
    accB = dot8(wb[u], x0, x1, accB);
  }
  accA = wave_sum(accA);
  accB = wave_sum(accB);
  if (lane == 0) { part[wave * 2] = accA; part[wave * 2 + 1] = accB; }
  __syncthreads();
  if (valid && seg == 0 && lane == 0) {
    for (int sg = 1; sg < NSEG; ++sg) { accA += part[(wave + sg) * 2]; accB += part[(wave + sg) * 2 + 1]; }
    a.out[rowA] = pre0 + accA;
    a.out[rowB] = pre1 + accB;
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
// grid = (heads, S), NTHR threads.  A key row (HD halves) is read by HD/8
// adjacent lanes with one 16-byte load each, so a wave covers 64/(HD/8)
// consecutive keys per load.  Every such lane group keeps its own
// online-softmax state (running max m, denominator l, 8 output columns per
// lane) over the keys it is dealt, round robin over all groups of all S
// workgroups of the head -- the grid is fixed and the key range comes from
// DevState, so the same captured launch serves every KV length.  With S = 4
// workgroups of 512 threads and 8 keys in flight per group one pass covers
// 1024 keys, and a CU has at most 128 KB of key and value rows to pull (a CU
// takes about 140 GB/s: with two workgroups of 1024 threads per head the kernel
// grew by 0.8 us per 440 keys).  Groups merge inside the wave by shuffles,
// waves through LDS; the S <= ATTN_MERGE_MAX partials (m, l, acc[HD]) of a head
// are merged by the consumer, the O-projection's prologue, underneath its weight
// stream, which saves this kernel a cross-workgroup hand-off (stores -> counter
// -> reload: about 5 us of pure latency).

template <int HD, int NTHR = ATTN_THREADS>
__global__ __launch_bounds__(NTHR) void attn_decode_kernel(
    const float* __restrict__ q, const half_t* __restrict__ kc, const half_t* __restrict__ vc,
    const DevState* __restrict__ st, float* __restrict__ part, int max_seq) {
  constexpr int LPR = HD / 8;      // lanes per key row
  constexpr int GPW = 64 / LPR;    // lane groups per wave
  constexpr int NW = NTHR / 64;
  constexpr int UK = 8;            // keys in flight per group
  constexpr int PS = ATTN_PART_STRIDE(HD);
  __shared__ float s_m[NW], s_l[NW], s_acc[NW][HD];

  const int h = blockIdx.x, s = blockIdx.y, S = gridDim.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int gi = lane / LPR, li = lane % LPR;
  const int n_keys = st->pos + 1;
  const float scale = 1.0f / sqrtf((float)HD);

  // The query is used unscaled (the score takes the factor): nothing is computed from it before the
  // first keys are requested, so its L2 round trip runs underneath theirs instead of in front of it.
  const f4 q0 = *reinterpret_cast<const f4*>(q + h * HD + li * 8);
  const f4 q1 = *reinterpret_cast<const f4*>(q + h * HD + li * 8 + 4);
  const half_t* kh = kc + (size_t)h * max_seq * HD + li * 8;
  const half_t* vh = vc + (size_t)h * max_seq * HD + li * 8;

  float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;

  const int stride = S * NW * GPW;
  auto batch = [&](int base) {
    h8 kk[UK], vv[UK];
#pragma unroll
    for (int j = 0; j < UK; ++j) {
      const int u = min(base + j * stride + gi, n_keys - 1);
      kk[j] = load_stream(kh + (size_t)u * HD);
      vv[j] = load_stream(vh + (size_t)u * HD);
    }
    __builtin_amdgcn_sched_barrier(0);     // all 16 requests out before the first use: one round trip, not several
    // One online-softmax step per batch, not per key: the batch's scores, one new maximum, one correction
    // of the running state, one exponential per key.  No branch around any of it: inside one the compiler
    // sinks a value row's load to where it is used and waits for it there, a second round trip behind the first.
    float dot[UK], mn = m;
#pragma unroll
    for (int j = 0; j < UK; ++j) {
      float t = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) t += q0[e] * (float)kk[j][e] + q1[e] * (float)kk[j][4 + e];
      t = group_sum<LPR>(t) * scale;
      dot[j] = (base + j * stride + gi < n_keys) ? t : -INFINITY;
      mn = fmaxf(mn, dot[j]);
    }
    const float corr = (m == mn) ? 1.0f : __expf(m - mn);     // also m = mn = -inf
    l *= corr;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= corr;
#pragma unroll
    for (int j = 0; j < UK; ++j) {
      const float p = (dot[j] > -INFINITY) ? __expf(dot[j] - mn) : 0.f;
      l += p;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += p * (float)vv[j][e];
    }
    m = mn;
  };
  // the first batch stands outside the loop: straight-line code, in which the wait for the query leaves
  // the keys and values requested after it in flight (a loop header waits for everything)
  const int base0 = (s * NW + wave) * GPW;
  if (base0 < n_keys) batch(base0);
  for (int base = base0 + stride * UK; base < n_keys; base += stride * UK) batch(base);
  // merge the lane groups of this wave: lanes with equal li hold the same columns
  {
    float M = m;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float w = (M > -INFINITY) ? __expf(m - M) : 0.f;   // empty groups (m = -inf) weigh 0
    l *= w;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= w;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
      l += __shfl_xor(l, off);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
    if (gi == 0) {
      if (li == 0) { s_m[wave] = M; s_l[wave] = l; }
#pragma unroll
      for (int e = 0; e < 8; ++e) s_acc[wave][li * 8 + e] = acc[e];
    }
  }
  __syncthreads();

  if (tid < HD) {   // merge the waves, publish this workgroup's partial
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < NW; ++i) M = fmaxf(M, s_m[i]);
    float L = 0.f, A = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        const float w = (s_m[i] > -INFINITY) ? __expf(s_m[i] - M) : 0.f;
        L += s_l[i] * w;
        A += s_acc[i][tid] * w;
      }
    }
    float* mypart = part + ((size_t)h * S + s) * PS;
    if (tid == 0) { mypart[0] = M; mypart[1] = L; }
    mypart[4 + tid] = A;
  }
}

// Attention and O projection of one layer in ONE launch: x += W_o * attention(q, K, V).
//
// The two are the pair furthest below the HBM roofline as separate kernels (a launch each of ramp-up
// and drain around 8-16 MB and 33.5 MB of traffic).  Here the first heads * S workgroups run the
// split-K attention exactly as attn_decode_kernel does, while the remaining workgroups, one row pair
// of W_o per wave, put ALL of W_o in flight at once (K <= 4096: 16 x 16-byte loads per lane and
// row pair), so the weight stream of the projection runs underneath the attention.  The hand-off
// is the one cross-workgroup dependency inside a launch on the default path: an attention workgroup
// stores its partial (m, l, acc[HD]) with device-scope stores, drains its vector-memory counter and
// then adds one to an arrival counter; one thread per projection workgroup polls that counter (bounded:
// on a time-out it raises DevState::fault and the step reports token -1 instead of hanging), after
// which the workgroup merges the partials into its LDS copy of o with device-scope loads and
// finishes its 16 row pairs from registers.  The grid never exceeds one workgroup per CU (host
// check), so every workgroup is resident and the attention workgroups, which wait for nobody, always
// finish.  The last projection workgroup to pass the wait clears both counters for the next launch.
#define ATTN_FUSED_MAX_SPLITS 2
struct AttnOArgs {
  const float* q;          // rotated query [d]
  const half_t* kc;        // this layer's keys   [head][max_seq][HD]
  const half_t* vc;        // this layer's values
  const DevState* st;
  float* part;             // [head][S][ATTN_PART_STRIDE(HD)] split-K partials
  const half_t* wo;        // [d][d]
  float* x;                // residual stream [d], updated in place
  unsigned* sync;          // [0]: attention workgroups arrived; [32]: projection workgroups past the wait
  int* fault;              // &DevState::fault
  int d, n_heads, splits, max_seq;
  int spin_limit;
};

template <int HD>
__global__ __launch_bounds__(ATTN_THREADS) void attn_oproj_kernel(AttnOArgs a) {
  constexpr int LPR = HD / 8, GPW = 64 / LPR, NW = ATTN_THREADS / 64, UK = 8;
  constexpr int PS = ATTN_PART_STRIDE(HD);
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_attn = a.n_heads * a.splits;

  if ((int)blockIdx.x < n_attn) {
    // ---------------- attention workgroup (head h, split s): see attn_decode_kernel
    float* s_m = lds;                  // [NW]
    float* s_l = lds + NW;             // [NW]
    float* s_acc = lds + 2 * NW;       // [NW][HD]
    const int h = blockIdx.x / a.splits, s = blockIdx.x - h * a.splits, S = a.splits;
    const int gi = lane / LPR, li = lane % LPR;
    const int n_keys = a.st->pos + 1;
    const float scale = 1.0f / sqrtf((float)HD);
    float qv[8];
    {
      const f4 q0 = *reinterpret_cast<const f4*>(a.q + h * HD + li * 8);
      const f4 q1 = *reinterpret_cast<const f4*>(a.q + h * HD + li * 8 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { qv[e] = q0[e] * scale; qv[4 + e] = q1[e] * scale; }
    }
    const half_t* kh = a.kc + (size_t)h * a.max_seq * HD + li * 8;
    const half_t* vh = a.vc + (size_t)h * a.max_seq * HD + li * 8;
    float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const int stride = S * NW * GPW;
    for (int base = (s * NW + wave) * GPW; base < n_keys; base += stride * UK) {
      h8 kk[UK], vv[UK];
#pragma unroll
      for (int j = 0; j < UK; ++j) {
        const int u = min(base + j * stride + gi, n_keys - 1);
        kk[j] = load_h8(kh + (size_t)u * HD);
        vv[j] = load_h8(vh + (size_t)u * HD);
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
    {
      float M = m;
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
      const float w = (M > -INFINITY) ? __expf(m - M) : 0.f;
      l *= w;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] *= w;
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) {
        l += __shfl_xor(l, off);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off);
      }
      if (gi == 0) {
        if (li == 0) { s_m[wave] = M; s_l[wave] = l; }
#pragma unroll
        for (int e = 0; e < 8; ++e) s_acc[wave * HD + li * 8 + e] = acc[e];
      }
    }
    __syncthreads();
    if (tid < HD) {
      float M = -INFINITY;
#pragma unroll
      for (int i = 0; i < NW; ++i) M = fmaxf(M, s_m[i]);
      float L = 0.f, A = 0.f;
      if (M > -INFINITY) {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
          const float w = (s_m[i] > -INFINITY) ? __expf(s_m[i] - M) : 0.f;
          L += s_l[i] * w;
          A += s_acc[i * HD + tid] * w;
        }
      }
      float* mypart = a.part + (size_t)blockIdx.x * PS;
      if (tid == 0) { st_dev(mypart, M); st_dev(mypart + 1, L); }
      st_dev(mypart + 4 + tid, A);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the partial is out before anyone is told
    }
    __syncthreads();
    if (tid == 0) __hip_atomic_fetch_add(as_global(a.sync), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }

  // ---------------- projection workgroup: 16 row pairs of W_o, one per wave
  const int K = a.d, P = a.d >> 1;
  const int nch = (K + 511) >> 9;                      // <= 8 (host check)
  const int p = ((int)blockIdx.x - n_attn) * NW + wave;
  const bool valid = p < P;
  const int rowA = 2 * min(p, P - 1), rowB = rowA + 1;
  const half_t* pa = a.wo + (size_t)rowA * K;
  const half_t* pb = a.wo + (size_t)rowB * K;
  h8 wa[8], wb[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int k = min(u * 512 + lane * 8, K - 8);
    wa[u] = load_stream(pa + k);
    wb[u] = load_stream(pb + k);
  }
  float pre0 = 0.f, pre1 = 0.f;
  if (valid && lane == 0) { pre0 = *as_global(a.x + rowA); pre1 = *as_global(a.x + rowB); }

  if (tid == 0) {
    int spins = 0;
    while (ld_dev_u(a.sync) < (unsigned)n_attn) {
      __builtin_amdgcn_s_sleep(2);
      if (++spins > a.spin_limit) { st_dev_i(a.fault, 1); break; }
    }
  }
  __syncthreads();

  // o = merge of the S partials of every head, staged lane-major for the dot products (chunk 8 stays zero)
  for (int i = tid; i < 9 * 128; i += ATTN_THREADS) {
    const int k = i * 4;
    f4 t = {0.f, 0.f, 0.f, 0.f};
    if (k < K) {
      const int head = k / HD, dcol = k - head * HD;
      const float* hb = a.part + (size_t)head * a.splits * PS;
      float2 hd[ATTN_FUSED_MAX_SPLITS], v0[ATTN_FUSED_MAX_SPLITS], v1[ATTN_FUSED_MAX_SPLITS];
#pragma unroll
      for (int sp = 0; sp < ATTN_FUSED_MAX_SPLITS; ++sp) {          // all loads first: one round trip
        hd[sp] = make_float2(-INFINITY, 0.f);
        v0[sp] = v1[sp] = make_float2(0.f, 0.f);
        if (sp < a.splits) {
          hd[sp] = ld_dev2(hb + sp * PS);
          v0[sp] = ld_dev2(hb + sp * PS + 4 + dcol);
          v1[sp] = ld_dev2(hb + sp * PS + 6 + dcol);
        }
      }
      float M = -INFINITY;
#pragma unroll
      for (int sp = 0; sp < ATTN_FUSED_MAX_SPLITS; ++sp) M = fmaxf(M, hd[sp].x);
      float L = 0.f;
#pragma unroll
      for (int sp = 0; sp < ATTN_FUSED_MAX_SPLITS; ++sp) {
        const float w = (hd[sp].x > -INFINITY) ? __expf(hd[sp].x - M) : 0.f;
        L += hd[sp].y * w;
        t[0] += v0[sp].x * w; t[1] += v0[sp].y * w; t[2] += v1[sp].x * w; t[3] += v1[sp].y * w;
      }
      const float rl = 1.0f / L;
      t[0] *= rl; t[1] *= rl; t[2] *= rl; t[3] *= rl;
    }
    const int c = k >> 9, r = k & 511;
    *reinterpret_cast<f4*>(lds + c * 512 + ((r >> 2) & 1) * 256 + (r >> 3) * 4) = t;
  }
  __syncthreads();

  float accA = 0.f, accB = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int xc = u < nch ? u : 8;
    const float* xp = lds + xc * 512 + lane * 4;
    const f4 x0 = *reinterpret_cast<const f4*>(xp);
    const f4 x1 = *reinterpret_cast<const f4*>(xp + 256);
    accA = dot8(wa[u], x0, x1, accA);
    accB = dot8(wb[u], x0, x1, accB);
  }
  accA = wave_sum(accA);
  accB = wave_sum(accB);
  if (valid && lane == 0) {
    a.x[rowA] = pre0 + accA;
    a.x[rowB] = pre1 + accB;
  }
  // every projection workgroup is past its wait when the last one gets here: clear the counters
  if (tid == 0) {
    const unsigned n_proj = gridDim.x - n_attn;
    const unsigned t = __hip_atomic_fetch_add(as_global(a.sync + 32), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t + 1u == n_proj) { st_dev_u(a.sync, 0u); st_dev_u(a.sync + 32, 0u); }
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

// Read-only pass over a buffer in the decode GEMVs' access shape: a wave takes 16 KB at a time (two
// "rows" of 8 KB, 16 x 16-byte streaming loads in flight per lane, a wave's load covering 1 KB), waves
// stride over the buffer.  Each workgroup may leave one word so that the loads cannot be dropped.  It
// measures the HBM read rate a kernel of this shape reaches on the chip at hand (the ceiling the
// decode step is compared with besides the nominal peak); nothing on the decode path calls it.
__global__ __launch_bounds__(LL_WG) void stream_read_kernel(const h8* __restrict__ src, size_t n16,
                                                            unsigned* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const size_t gw = (size_t)blockIdx.x * (LL_WG / 64) + (threadIdx.x >> 6), GW = (size_t)gridDim.x * (LL_WG / 64);
  const size_t nblk = n16 / 1024;                 // whole 16 KB blocks; a tail shorter than that is not read
  unsigned acc = 0;
  for (size_t b = gw; b < nblk; b += GW) {
    const h8* p = src + b * 1024 + lane;
    h8 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = __builtin_nontemporal_load(as_global(p + u * 64));
#pragma unroll
    for (int u = 0; u < 16; ++u) acc ^= __builtin_bit_cast(unsigned, __builtin_shufflevector(v[u], v[u], 0, 1));
  }
  acc ^= __shfl_xor(acc, 32);
  if (lane == 0 && acc == 0x9e3779b9u) sink[blockIdx.x] = acc;   // (practically never true: no store traffic)
}
