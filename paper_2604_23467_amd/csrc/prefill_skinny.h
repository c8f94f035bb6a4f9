// Projections of a SHORT prompt (at most 32 rows) for gfx950: the TTFT regime's
// low end (10-25 tokens, Sec. IV-E / Table I), where the layer is bound by
// streaming its weights once, exactly like a decode step, and a square-tiled
// GEMM wastes most of its tile.
//
// One workgroup of 8 waves owns a block of 16 output rows over the WHOLE of K,
// so nothing is accumulated across workgroups: no split-K atomics, no zeroing,
// and the epilogue of the layer (RoPE + KV-cache write, SwiGLU, residual add)
// runs on the finished sums inside the same kernel, as in the decode GEMVs.
//
//  * The weights never touch LDS.  v_mfma_f32_16x16x32_f16 takes, per lane, 8
//    consecutive k of one row (row = lane % 16, k = 8 * (lane / 16) ..), which is
//    exactly a 16-byte streaming load from that weight row: a wave's load
//    covers 16 rows x 64 contiguous bytes and goes straight into the A operand.
//  * The activations (B operand, 16 tokens per block, TB = 1 or 2 blocks) are at
//    most 32 x K and stay in L2.  Their producers store them fragment-major
//    (act_offset), so a B fragment is one contiguous 1 KB load; read row-major
//    with the weights' addressing, the 16 rows of a fragment sit a power of two
//    apart and pile onto one L2 channel (measured: 53 us per layer and token block).
//  * The 8 waves split K into 8 contiguous ranges; their partial 16 x 16 tiles
//    meet in LDS, and the epilogue threads sum the 8 partials.
//  * Weight loads are non-temporal, like the decode GEMVs': every byte is used once, and the stream then
//    leaves the activations and the norm factors alone in L2 (TTFT 2.98 -> 2.85 ms at 10 tokens, 3.30 ->
//    3.15 ms at 25; gate/up 34.3 -> 32.4 us, Q/K/V 21.4 -> 20.8, down 19.9 -> 18.9, O 9.2 -> 8.4).  A look-ahead
//    of a whole row block instead of half of one (twice the bytes in flight per wave) measured no gain on top.
//
// The two wide projections (Q/K/V, gate/up) normally run in the persistent form
// further down, which keeps a wave's activation fragments in registers; the
// kernel right below serves O and down, and any K too long for that.
//
// Row blocks are chosen so that the epilogue's partners share a block: a
// q/k block holds rows j..j+7 and j+hd/2..j+hd/2+7 of one head (the RoPE
// pairs), a gate/up block holds gate rows r..r+7 and up rows r..r+7.
//
// RMSNorm costs no kernel of its own.  The kernel that finishes a residual
// update (SK_RES, or the embedding gather for layer 0) also stores the fp16
// operand x * gain of the NEXT projection and, per token, the sum of squares of
// the 16 columns its workgroup owns into a slot of its own; the consuming
// projection (SK_QKV / SK_GATEUP) adds a token's slots in a fixed order and
// multiplies its finished sums by rsqrt(mean x^2 + eps), which commutes with
// the contraction: W (x g) s = s W (x g).  No atomics: every run of the same
// input gives the same bits.
#pragma once
#include "ll_device.h"

enum SkinnyMode { SK_QKV = 0, SK_RES = 1, SK_GATEUP = 2, SK_LOGITS = 3 };

struct SkinnyArgs {
  const half_t* X;        // 16 TB token rows x K fp16 activations, fragment-major; rows >= n hold anything
  const half_t* W[3];     // [N][K] fp16 each (QKV: q, k, v; GATEUP: gate, up; RES: one matrix)
  const half_t* Wf;       // optional copy of the same matrices in the kernels' own operand order (see
                          // sk_shuffle_kernel): the 16 x 32 piece of row block u and K step s is the 1 KB at
                          // ((u * ceil(K / 32) + s) * 64 + lane) * 8, zero beyond K.  Null: read W row-major
  const DevState* st;
  int N, K;
  float* Xres;            // RES: residual stream [rows][N] fp32, updated in place for rows < n
  const half_t* gain_next;// RES: gain of the norm in front of the next projection (null: none follows)
  half_t* Xh_next;        // RES: fp16 x * gain_next, fragment-major, operand of the next projection
  float* ss_out;          // RES: [16 TB][ss_stride] per-token sums of squares of the updated residual, slot
                          //      blockIdx.x = the 16 columns of this workgroup
  const float* ss_in;     // QKV / GATEUP / LOGITS: [16 TB][ss_stride], slots 0 .. ss_parts - 1 of a token add up
                          //      to the sum of squares of the operand's source row
  int ss_stride, ss_parts;
  float eps;
  half_t* Hout;           // GATEUP: 16 TB rows x N fp16, fragment-major
  half_t* Q;              // QKV: [rows][N] fp16 rotated queries
  half_t* kc;             // QKV: this layer's K cache [head][max_seq][head_dim]
  half_t* vc;
  const float2* rope;     // [max_seq][head_dim / 2] (cos, sin)
  long zeros_off;         // element offset from X of >= 16 bytes of zeros (same allocation as X)
                          // positions: row r of the prompt chunk sits at position st->pos + r
  int head_dim, max_seq;
  // batched decode (rows = sequences of a batch instead of rows of one prompt):
  const int* row_pos;     // QKV: position of row r (null: st->pos + r)
  const int* page_table;  // QKV: [rows][pt_stride] first cache row of each page of row r's sequence (null: cache row = position)
  int pt_stride, page_tokens;
  float* logits;          // LOGITS: [rows][N] fp32, normalised like QKV / GATEUP outputs
};

// position of row tok, and the cache row that holds a position of row tok's sequence
__device__ __forceinline__ int sk_row_pos(const SkinnyArgs& a, int p0, int tok) {
  return a.row_pos ? a.row_pos[tok] : p0 + tok;
}
__device__ __forceinline__ int sk_cache_row(const SkinnyArgs& a, int tok, int pos) {
  if (!a.page_table) return pos;
  const int pg = pos / a.page_tokens;
  return a.page_table[tok * a.pt_stride + pg] + (pos - pg * a.page_tokens);
}

#define SK_WAVES 8
#define SK_THREADS (SK_WAVES * 64)
#define SK_PSTRIDE 20      // floats per (wave, token) row of partials: 16 + pad, keeps 16-byte alignment

// floats between two tokens' slots of partial sums of squares: one slot per 16-column block of a
// d_model-wide residual row, rounded up to whole 64-byte groups
__host__ __device__ inline int sk_ss_stride(int d_model) { return ((d_model + 15) / 16 + 15) / 16 * 16; }

// rsqrt(mean x^2 + eps) of the 16 TB token rows into LDS: 16 lanes per token add its slots in a
// fixed order (strided partial sums, then a DPP tree).  Needs 256 TB threads.  Two steps, so that
// the loads can be put in flight ahead of a kernel's weight stream and their values used after
// it has started: the wait for them then leaves the younger weight loads in flight.  The
// caller's next workgroup barrier publishes s_scale.
struct SkSsLoads { float v[16]; float tail; };
template <int TB>
__device__ __forceinline__ void sk_ss_issue(const float* ss_in, int ss_stride, int ss_parts, int tid, SkSsLoads& L) {
  L.tail = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) L.v[i] = 0.f;
  if (tid < TB * 256) {
    const int tok = tid >> 4, j = tid & 15;
    const float* p = ss_in + (size_t)tok * ss_stride;
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (j + 16 * i < ss_parts) L.v[i] = *as_global(p + j + 16 * i);
    for (int i = j + 256; i < ss_parts; i += 16) L.tail += *as_global(p + i);   // d_model > 4096 only
  }
}
template <int TB>
__device__ __forceinline__ void sk_ss_finish(const SkSsLoads& L, int K, float eps, float* s_scale, int tid) {
  float s = L.tail;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += L.v[i];
  s = group_sum<16>(s);
  if (tid < TB * 256 && (tid & 15) == 0) s_scale[tid >> 4] = 1.0f / sqrtf(s / (float)K + eps);
}

// number of 16-row blocks the kernel's grid has to cover
__host__ __device__ inline int skinny_units(int mode, int N) {
  return mode == SK_QKV ? 3 * (N / 16) : mode == SK_GATEUP ? N / 8 : N / 16;
}

// NB > 0: the host promises ceil(K steps per wave / 8) == NB and the batch pipeline is unrolled
// with exact wait counts; NB = 0 walks any K with a loop that over-fetches one batch.
template <int MODE, int TB, int NB>
__global__ __launch_bounds__(SK_THREADS, 1) void pf_skinny_kernel(SkinnyArgs a) {
  constexpr int RB = 1;
  __shared__ __attribute__((aligned(16))) float part[SK_WAVES * TB * 16 * SK_PSTRIDE];
  __shared__ float s_scale[TB * 16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, g = lane >> 4;
  const int K = a.K, N = a.N;
  const int n = a.st->n_prompt, p0 = a.st->pos;   // rows of this chunk, positions cached before it
  const int units = skinny_units(MODE, N);
  const int hh = a.head_dim >> 1;

  // weight row this lane streams
  const half_t* wrow;
  {
    const int u = blockIdx.x;
    if (MODE == SK_RES) {
      wrow = a.W[0] + (size_t)(u * 16 + r) * K;
    } else if (MODE == SK_GATEUP) {
      wrow = a.W[r >> 3] + (size_t)(u * 8 + (r & 7)) * K;
    } else {
      const int per = N / 16, z = u / per, v = u - z * per;
      int row;
      if (z == 2) {
        row = v * 16 + r;
      } else {
        const int bph = hh / 8, head = v / bph, j0 = (v - head * bph) * 8;
        row = head * a.head_dim + j0 + (r & 7) + (r >> 3) * hh;
      }
      wrow = a.W[z] + (size_t)row * K;
    }
  }

  // with a fragment-major copy a wave's load is 1 KB of consecutive bytes instead of 16 rows x 64 bytes
  const bool frag = a.Wf != nullptr;
  const half_t* wfrag = frag ? a.Wf + ((size_t)blockIdx.x * ((K + 31) >> 5) * 64 + lane) * 8 : nullptr;

  f4 acc[TB];
#pragma unroll
  for (int t = 0; t < TB; ++t) acc[t] = f4{0.f, 0.f, 0.f, 0.f};

  // SK_RES: thread o < 32 TB finishes rows 8 (o & 1) .. + 8 of token o >> 1.  What it adds to
  // (the residual) and scales by (the next norm's gain) does not depend on the contraction, so
  // it is fetched now and has long arrived when the sums are ready.
  f4 ex0 = {0.f, 0.f, 0.f, 0.f}, ex1 = ex0;
  h8 egain = {0, 0, 0, 0, 0, 0, 0, 0};
  const bool efin = MODE == SK_RES && tid < TB * 32 && (tid >> 1) < n;
  if (MODE == SK_RES && efin) {
    const int c0 = blockIdx.x * 16 + (tid & 1) * 8;
    const float* xp = a.Xres + (size_t)(tid >> 1) * N + c0;
    ex0 = *as_global(reinterpret_cast<const f4*>(xp));
    ex1 = *as_global(reinterpret_cast<const f4*>(xp + 4));
    if (a.gain_next) egain = load_h8(a.gain_next + c0);
  }
  if (MODE != SK_RES) {
    SkSsLoads sl;
    sk_ss_issue<TB>(a.ss_in, a.ss_stride, a.ss_parts, tid, sl);
    sk_ss_finish<TB>(sl, K, a.eps, s_scale, tid);
  }
  __builtin_amdgcn_sched_barrier(0);

  // K range of this wave, in 32-wide MFMA steps, walked in batches of U steps.  Two batches
  // of registers alternate, so a batch's loads are in flight while the previous one is
  // multiplied.  A step outside the range (or a lane's 8 halves past K) re-reads the row
  // start and takes its B fragment from a block of zeros: no load is ever predicated.
  const int ksteps = (K + 31) >> 5;
  const int per_wave = (ksteps + SK_WAVES - 1) / SK_WAVES;
  const int s_begin = wave * per_wave, s_end = min(s_begin + per_wave, ksteps);
  constexpr int U = 8;
  h8 fa[2][U], fb[2][U][TB];
  auto issue = [&](int s0, h8 (&A)[U], h8 (&B)[U][TB]) {
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int st = s0 + i, k = st * 32 + g * 8;
      const bool in = st < s_end && k < K;           // K % 8 == 0: 8 halves are all in or all out
      A[i] = load_stream(frag ? wfrag + (in ? (long)st * 512 : 0) : wrow + (in ? k : 0));
#pragma unroll
      for (int t = 0; t < TB; ++t)
        B[i][t] = load_h8(a.X + (in ? (long)(st * TB + t) * 512 + lane * 8 : a.zeros_off));
    }
  };
  auto multiply = [&](const h8 (&A)[U], const h8 (&B)[U][TB]) {
#pragma unroll
    for (int i = 0; i < U; ++i)
#pragma unroll
      for (int t = 0; t < TB; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[i], B[i][t], acc[t], 0, 0, 0);
  };
  // The scheduling fences keep each batch's loads together and ahead of the other batch's
  // MFMAs; left alone the compiler sinks every load next to its use to save registers, which
  // serialises the memory latency.
  issue(s_begin, fa[0], fb[0]);
  if constexpr (NB > 0) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      __builtin_amdgcn_sched_barrier(0);
      if (b + 1 < NB) issue(s_begin + (b + 1) * U, fa[(b + 1) & 1], fb[(b + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
      multiply(fa[b & 1], fb[b & 1]);
    }
  } else {
    for (int s0 = s_begin; s0 < s_end; s0 += 2 * U) {
      __builtin_amdgcn_sched_barrier(0);
      issue(s0 + U, fa[1], fb[1]);        // unconditional: past the range these are cache hits on the row start
      __builtin_amdgcn_sched_barrier(0);
      multiply(fa[0], fb[0]);
      __builtin_amdgcn_sched_barrier(0);
      issue(s0 + 2 * U, fa[0], fb[0]);
      __builtin_amdgcn_sched_barrier(0);
      multiply(fa[1], fb[1]);
    }
  }

  // accumulator layout of the 16x16 MFMA: lane holds token column (lane % 16) and weight
  // rows 4 * (lane / 16) + 0..3; partials are stored as part[wave][token][row]
#pragma unroll
  for (int t = 0; t < TB; ++t)
    *reinterpret_cast<f4*>(part + ((wave * TB + t) * 16 + r) * SK_PSTRIDE + g * 4) = acc[t];
  // bare barrier: the look-ahead loads of the last round are still in flight and nobody needs them
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // Epilogue: one thread finishes 8 consecutive rows of one token (16-byte stores throughout).
  // sum8(b, tok, h): rows 8h..8h+7 of block b for token tok, summed over the 8 waves' partials
  auto sum8 = [&](int b, int tok, int h, float (&v)[8]) {
    f4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
    for (int w = 0; w < SK_WAVES; ++w) {
      const float* pp = part + (((w * RB + b) * TB) * 16 + tok) * SK_PSTRIDE + h * 8;
      s0 += *reinterpret_cast<const f4*>(pp);
      s1 += *reinterpret_cast<const f4*>(pp + 4);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[j] = s0[j]; v[4 + j] = s1[j]; }
  };

  if (MODE == SK_RES) {
    float ss = 0.f;
    if (efin) {
      const int h = tid & 1, tok = tid >> 1;
      float v[8];
      sum8(0, tok, h, v);
      const int c0 = blockIdx.x * 16 + h * 8;
      float* xp = a.Xres + (size_t)tok * N + c0;
#pragma unroll
      for (int j = 0; j < 4; ++j) { v[j] += ex0[j]; v[4 + j] += ex1[j]; }
      *reinterpret_cast<f4*>(xp) = f4{v[0], v[1], v[2], v[3]};
      *reinterpret_cast<f4*>(xp + 4) = f4{v[4], v[5], v[6], v[7]};
      if (a.gain_next) {
        h8 xh;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          xh[j] = (half_t)(v[j] * (float)egain[j]);
          ss += v[j] * v[j];
        }
        *reinterpret_cast<h8*>(a.Xh_next + act_offset(tok, c0, N, TB)) = xh;
      }
    }
    if (tid < TB * 32) {
      ss += dpp_mov<0xB1>(ss);                     // the token's other half sits in the neighbouring lane
      if (efin && (tid & 1) == 0 && a.gain_next) a.ss_out[(size_t)(tid >> 1) * a.ss_stride + blockIdx.x] = ss;
    }
  } else {
    for (int o = tid; o < RB * TB * 16; o += SK_THREADS) {
      const int tok = o % (TB * 16), b = o / (TB * 16);
      const int u = blockIdx.x * RB + b;
      if (u >= units || tok >= n) continue;
      const float rs = s_scale[tok];
      float lo[8], hi[8];
      sum8(b, tok, 0, lo);
      sum8(b, tok, 1, hi);
#pragma unroll
      for (int j = 0; j < 8; ++j) { lo[j] *= rs; hi[j] *= rs; }
      h8 o0, o1;
      if (MODE == SK_GATEUP) {
#pragma unroll
        for (int j = 0; j < 8; ++j) o0[j] = (half_t)(lo[j] / (1.0f + expf(-lo[j])) * hi[j]);
        *reinterpret_cast<h8*>(a.Hout + act_offset(tok, u * 8, N, TB)) = o0;
      } else {
        const int per = N / 16, z = u / per, v = u - z * per;
        if (z == 2) {
          const int c0 = v * 16, head = c0 / a.head_dim, e = c0 - head * a.head_dim;   // 16 rows of one head
#pragma unroll
          for (int j = 0; j < 8; ++j) { o0[j] = (half_t)lo[j]; o1[j] = (half_t)hi[j]; }
          const int pos = sk_row_pos(a, p0, tok);
          half_t* vr = a.vc + ((size_t)head * a.max_seq + sk_cache_row(a, tok, pos)) * a.head_dim + e;
          *reinterpret_cast<h8*>(vr) = o0;
          *reinterpret_cast<h8*>(vr + 8) = o1;
        } else {
          const int bph = hh / 8, head = v / bph, j0 = (v - head * bph) * 8;
          const int pos = sk_row_pos(a, p0, tok);                     // row tok of a prompt chunk sits at position p0 + tok
          const float2* cs = a.rope + (size_t)pos * hh + j0;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float2 t2 = cs[j];
            o0[j] = (half_t)(lo[j] * t2.x - hi[j] * t2.y);
            o1[j] = (half_t)(hi[j] * t2.x + lo[j] * t2.y);
          }
          half_t* dst = z == 0 ? a.Q + (size_t)tok * N + head * a.head_dim
                               : a.kc + ((size_t)head * a.max_seq + sk_cache_row(a, tok, pos)) * a.head_dim;
          *reinterpret_cast<h8*>(dst + j0) = o0;
          *reinterpret_cast<h8*>(dst + j0 + hh) = o1;
        }
      }
    }
  }
}

// Persistent form of the two wide projections (SK_QKV, SK_GATEUP) for K <= 4096 and at most 32
// tokens: one workgroup per CU walks row blocks u = blockIdx.x, + gridDim.x, ...  A wave keeps
// the same K range for every block, so its B fragments (16 K steps x TB) are loaded ONCE into
// registers and the activations cause no further traffic; and the first half of the next
// block's weights is requested before the current block's partials are exchanged, so the
// weight stream never drains while a block is being finished.  The finishing (8 partials ->
// epilogue) rotates over the waves, one block each, on all 64 lanes (2 or 4 row pairs of a token per
// lane); partials are double-buffered in LDS so a single barrier per block orders writers and the
// finishing wave.  The other waves meet the finishing wave again at the next block's barrier, so what
// its epilogue costs is on every block's path: spread over 64 lanes instead of one lane per token, and
// with the RoPE factors fetched when the block starts, Q/K/V went from 20.6 to 19.3 us and gate/up from
// 32.2 to 31.3 us at 16 rows (without any epilogue: 18.6 / 30.4 us).
#define SKP_KSTEPS 16     // K steps per wave held in registers: K <= 8 waves * 16 * 32
template <int MODE, int TB>
__global__ __launch_bounds__(SK_THREADS, 1) void pf_skinny_persist_kernel(SkinnyArgs a) {
  static_assert(MODE != SK_RES, "wide projections only");
  __shared__ __attribute__((aligned(16))) float part[2][SK_WAVES * TB * 16 * SK_PSTRIDE];
  __shared__ float s_scale[TB * 16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, g = lane >> 4;
  const int K = a.K, N = a.N;
  const int n = a.st->n_prompt, p0 = a.st->pos;   // rows of this chunk, positions cached before it
  const int units = skinny_units(MODE, N);
  const int hh = a.head_dim >> 1;
  const int ksteps = (K + 31) >> 5;
  const int per_wave = (ksteps + SK_WAVES - 1) / SK_WAVES;      // <= SKP_KSTEPS (host checked)
  const int s_begin = wave * per_wave, s_end = min(s_begin + per_wave, ksteps);
  constexpr int HALF = SKP_KSTEPS / 2;

  bool in[SKP_KSTEPS];
#pragma unroll
  for (int i = 0; i < SKP_KSTEPS; ++i) in[i] = (s_begin + i < s_end) && ((s_begin + i) * 32 + g * 8 < K);

  // weight row of this lane in row block u
  auto row_ptr = [&](int u) -> const half_t* {
    if (MODE == SK_GATEUP) return ((r >> 3) ? a.W[1] : a.W[0]) + (size_t)(u * 8 + (r & 7)) * K;   // no indexed read of the arguments
    if (MODE == SK_LOGITS) return a.W[0] + (size_t)(u * 16 + r) * K;
    const int per = N / 16, z = u / per, v = u - z * per;
    int row;
    if (z == 2) {
      row = v * 16 + r;
    } else {
      const int bph = hh / 8, head = v / bph, j0 = (v - head * bph) * 8;
      row = head * a.head_dim + j0 + (r & 7) + (r >> 3) * hh;
    }
    return a.W[z] + (size_t)row * K;
  };
  // element offset of K step i in a weight row; steps outside the wave's range re-read the row
  // start instead (always valid memory) and meet a zero B fragment
  // (with a fragment-major copy: its 1 KB pieces, 512 halves per K step, instead of 16 rows x 64 bytes)
  const bool frag = a.Wf != nullptr;
  int koff[SKP_KSTEPS];
#pragma unroll
  for (int i = 0; i < SKP_KSTEPS; ++i) koff[i] = !in[i] ? 0 : frag ? (s_begin + i) * 512 : (s_begin + i) * 32 + g * 8;
  auto blk_ptr = [&](int u) -> const half_t* {
    return frag ? a.Wf + ((size_t)u * ksteps * 64 + lane) * 8 : row_ptr(u);
  };

  // a few small loads for the tokens' norm factors, then the weight stream, then the (cached) activations
  SkSsLoads sl;
  sk_ss_issue<TB>(a.ss_in, a.ss_stride, a.ss_parts, tid, sl);
  __builtin_amdgcn_sched_barrier(0);
  int u = blockIdx.x;
  h8 fa0[HALF], fa1[HALF];
  {
    const half_t* wp = blk_ptr(u < units ? u : 0);
#pragma unroll
    for (int i = 0; i < HALF; ++i) fa0[i] = load_stream(wp + koff[i]);
  }
  __builtin_amdgcn_sched_barrier(0);
  h8 fb[SKP_KSTEPS][TB];
#pragma unroll
  for (int i = 0; i < SKP_KSTEPS; ++i)
#pragma unroll
    for (int t = 0; t < TB; ++t)
      fb[i][t] = load_h8(a.X + (in[i] ? ((long)((s_begin + i) * TB + t) * 64 + lane) * 8 : a.zeros_off));
  __builtin_amdgcn_sched_barrier(0);
  sk_ss_finish<TB>(sl, K, a.eps, s_scale, tid);   // published by the first block's barrier
  __builtin_amdgcn_sched_barrier(0);
  // The epilogue of a block runs on all 64 lanes of the wave whose turn it is: lane = (eq, etok) finishes NP
  // of the 8 (lo, hi) row pairs of token etok.  What it needs from memory besides the sums (the token's
  // position and cache row, its RoPE factors) is fetched when the block starts, so that the block ends
  // without a memory round trip.
  constexpr int ET = TB * 16, NP = 8 * ET / 64;              // tokens; pairs per lane (2 or 4)
  typedef float EV __attribute__((ext_vector_type(NP)));
  typedef half_t EH __attribute__((ext_vector_type(NP)));
  const int etok = lane % ET, eq = lane / ET;
  int epos = 0, ecrow = 0;
  if (MODE == SK_QKV && etok < n) {
    epos = sk_row_pos(a, p0, etok);
    ecrow = sk_cache_row(a, etok, epos);
  }
  constexpr bool EPRE = TB == 1;      // 32 token rows leave no registers for the early RoPE factors
  float2 ecs[NP];
  int round = 0;
  for (; u < units; u += gridDim.x, ++round) {
    {
      const half_t* wp = blk_ptr(u);
#pragma unroll
      for (int i = 0; i < HALF; ++i) fa1[i] = load_stream(wp + koff[HALF + i]);
    }
    if (MODE == SK_QKV && EPRE && wave == (round & (SK_WAVES - 1)) && etok < n) {
      const int per = N / 16, z = u / per, v = u - z * per;
      if (z < 2) {
        const int bph = hh / 8, head = v / bph, j0 = (v - head * bph) * 8 + eq * NP;
        const float2* cs = a.rope + (size_t)epos * hh + j0;
#pragma unroll
        for (int j = 0; j < NP; ++j) ecs[j] = cs[j];
      }
    }
    f4 acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t) acc[t] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < HALF; ++i)
#pragma unroll
      for (int t = 0; t < TB; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa0[i], fb[i][t], acc[t], 0, 0, 0);
    // always issued, so that the waits below are exact: after the last block the target is
    // row block 0, which every workgroup re-reads from cache
    {
      const int un = u + gridDim.x;
      const half_t* wp = blk_ptr(un < units ? un : 0);
#pragma unroll
      for (int i = 0; i < HALF; ++i) fa0[i] = load_stream(wp + koff[i]);
    }
#pragma unroll
    for (int i = 0; i < HALF; ++i)
#pragma unroll
      for (int t = 0; t < TB; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa1[i], fb[HALF + i][t], acc[t], 0, 0, 0);

    float* pb = part[round & 1];
#pragma unroll
    for (int t = 0; t < TB; ++t)
      *reinterpret_cast<f4*>(pb + ((wave * TB + t) * 16 + r) * SK_PSTRIDE + g * 4) = acc[t];
    // LDS writes done, then a bare barrier: a full __syncthreads() would also drain the weight loads in flight
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    if (wave == (round & (SK_WAVES - 1)) && etok < n) {
      // lane (eq, etok): pairs eq * NP .. + NP - 1 of token etok, i.e. rows eq * NP .. (lo) and 8 + eq * NP .. (hi)
      const float scale = s_scale[etok];
      float lo[NP], hi[NP];
#pragma unroll
      for (int j = 0; j < NP; ++j) lo[j] = hi[j] = 0.f;
#pragma unroll
      for (int w = 0; w < SK_WAVES; ++w) {
        const float* pp = pb + ((w * TB) * 16 + etok) * SK_PSTRIDE + eq * NP;
        const EV a0 = *reinterpret_cast<const EV*>(pp), a1 = *reinterpret_cast<const EV*>(pp + 8);
#pragma unroll
        for (int j = 0; j < NP; ++j) { lo[j] += a0[j]; hi[j] += a1[j]; }
      }
#pragma unroll
      for (int j = 0; j < NP; ++j) { lo[j] *= scale; hi[j] *= scale; }
      EH o0, o1;
      if (MODE == SK_GATEUP) {
#pragma unroll
        for (int j = 0; j < NP; ++j) o0[j] = (half_t)(lo[j] / (1.0f + expf(-lo[j])) * hi[j]);
        *reinterpret_cast<EH*>(a.Hout + act_offset(etok, u * 8 + eq * NP, N, TB)) = o0;
      } else if (MODE == SK_LOGITS) {
        float* lp = a.logits + (size_t)etok * N + u * 16 + eq * NP;
        EV v0, v1;
#pragma unroll
        for (int j = 0; j < NP; ++j) { v0[j] = lo[j]; v1[j] = hi[j]; }
        *reinterpret_cast<EV*>(lp) = v0;
        *reinterpret_cast<EV*>(lp + 8) = v1;
      } else {
        const int per = N / 16, z = u / per, v = u - z * per;
        if (z == 2) {
          const int c0 = v * 16, head = c0 / a.head_dim, e = c0 - head * a.head_dim;
#pragma unroll
          for (int j = 0; j < NP; ++j) { o0[j] = (half_t)lo[j]; o1[j] = (half_t)hi[j]; }
          half_t* vr = a.vc + ((size_t)head * a.max_seq + ecrow) * a.head_dim + e + eq * NP;
          *reinterpret_cast<EH*>(vr) = o0;
          *reinterpret_cast<EH*>(vr + 8) = o1;
        } else {
          const int bph = hh / 8, head = v / bph, j0 = (v - head * bph) * 8 + eq * NP;
          if (!EPRE) {
            const float2* cs = a.rope + (size_t)epos * hh + j0;
#pragma unroll
            for (int j = 0; j < NP; ++j) ecs[j] = cs[j];
          }
#pragma unroll
          for (int j = 0; j < NP; ++j) {
            const float2 t2 = ecs[j];
            o0[j] = (half_t)(lo[j] * t2.x - hi[j] * t2.y);
            o1[j] = (half_t)(hi[j] * t2.x + lo[j] * t2.y);
          }
          half_t* dst = z == 0 ? a.Q + (size_t)etok * N + head * a.head_dim
                               : a.kc + ((size_t)head * a.max_seq + ecrow) * a.head_dim;
          *reinterpret_cast<EH*>(dst + j0) = o0;
          *reinterpret_cast<EH*>(dst + j0 + hh) = o1;
        }
      }
    }
  }
}

// One-off re-layout of a projection's weights into the short-prompt kernels' operand order (run once
// per matrix group at initialisation).  Read row-major, the A operand of a 16 x 16 x 32 product is 16
// rows x 64 bytes per wave and load, a shape this chip streams at 5.7 TB/s where 1 KB of consecutive
// bytes per load reaches 6.8 (measured with plain read kernels); the copy puts the 16 x 32 piece of
// row block u and K step s, in lane order, at ((u * ksteps + s) * 64 + lane) * 8 halves, so the
// projections stream it like the decode GEMVs stream rows.  Row blocks are the kernels' own (RoPE
// partners, gate / up pairs).  grid = (row blocks, ceil(ksteps / 4)), 256 threads: one wave per piece.
template <int MODE>
__global__ __launch_bounds__(LL_WG) void sk_shuffle_kernel(const half_t* __restrict__ w0, const half_t* __restrict__ w1,
                                                           const half_t* __restrict__ w2, int N, int K, int head_dim,
                                                           half_t* __restrict__ out) {
  const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int ksteps = (K + 31) >> 5, u = blockIdx.x, s = blockIdx.y * (LL_WG / 64) + (threadIdx.x >> 6);
  if (s >= ksteps) return;
  const half_t* W[3] = {w0, w1, w2};
  const half_t* src;
  if (MODE == SK_RES || MODE == SK_LOGITS) {
    src = W[0] + (size_t)(u * 16 + r) * K;
  } else if (MODE == SK_GATEUP) {
    src = W[r >> 3] + (size_t)(u * 8 + (r & 7)) * K;
  } else {
    const int hh = head_dim >> 1, per = N / 16, z = u / per, v = u - z * per;
    int row;
    if (z == 2) {
      row = v * 16 + r;
    } else {
      const int bph = hh / 8, head = v / bph, j0 = (v - head * bph) * 8;
      row = head * head_dim + j0 + (r & 7) + (r >> 3) * hh;
    }
    src = W[z] + (size_t)row * K;
  }
  const int k = s * 32 + g * 8;
  h8 v8 = {0, 0, 0, 0, 0, 0, 0, 0};
  if (k < K) v8 = load_h8(src + k);                      // K % 8 == 0: a piece is all in or all out
  *reinterpret_cast<h8*>(out + (((size_t)u * ksteps + s) * 64 + lane) * 8) = v8;
}

// Layer-0 front end of the short-prompt path: X[r] = float(E[tokens[r]]) (zero for r >= n),
// Xh = fp16 (x * gain) fragment-major, slot 0 of ss[r] = sum x^2 (the first projection adds one slot).
// grid = 16 TB rows, one workgroup per row.
__global__ __launch_bounds__(LL_WG) void pf_embed_norm_kernel(const half_t* __restrict__ emb,
                                                              const int* __restrict__ tokens,
                                                              const DevState* __restrict__ st,
                                                              const half_t* __restrict__ gain,
                                                              float* __restrict__ X, half_t* __restrict__ Xh,
                                                              float* __restrict__ ss, int ss_stride,
                                                              int d, int tb) {
  __shared__ float red[LL_WG / 64];
  const int r = blockIdx.x, tid = threadIdx.x;
  const bool live = r < st->n_prompt;
  const half_t* e = emb + (size_t)(live ? tokens[r] : 0) * d;
  float acc = 0.f;
  for (int i = tid * 8; i < d; i += LL_WG * 8) {
    h8 v = load_h8(e + i);
    const h8 gn = load_h8(gain + i);
    h8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float x = live ? (float)v[j] : 0.f;
      X[(size_t)r * d + i + j] = x;
      o[j] = (half_t)(x * (float)gn[j]);
      acc += x * x;
    }
    *reinterpret_cast<h8*>(Xh + act_offset(r, i, d, tb)) = o;
  }
  acc = wave_sum(acc);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) ss[(size_t)r * ss_stride] = red[0] + red[1] + red[2] + red[3];
}
