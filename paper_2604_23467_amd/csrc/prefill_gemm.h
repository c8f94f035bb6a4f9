// Prefill projection GEMM for gfx950, prompts of 33..512 tokens (Sec. IV-E / Table I, the upper
// part of the TTFT range): C[M][ldc] (fp32) += A[M][K] (fp16 activations) * W_z[N][K]^T (fp16).
//
// v_mfma_f32_32x32x16_f16, the full-rate fp16 matrix instruction of this chip (measured: 2.0
// PFLOP/s with one wave per SIMD and 8 independent accumulators; the 16x16x32 form reaches
// 0.83), activations as the A operand, weights as the B operand.
//
// Workgroup tile = BM rows x 256 columns x 64 k per slab, 4 waves side by side along N and WM
// along M: BM = 128 with 8 waves of 64 x 64 (two waves per SIMD hide each other's waits: measured
// 3 % faster than 4 waves of 128 x 64), BM = 64 with 4 waves of 64 x 64 for prompts of at most 64
// rows.  A 256 x 256 tile with two stages was also tried and lost (fewer tiles, shallower
// pipeline).  Every slab moves (BM + 256) x 128 bytes from L2 for BM x 256 x 128 flop; the same direct
// loads alone run at 53 B/clk per CU from L2 (measured), three times what the kernel needs, so it is
// not that traffic by itself that bounds these GEMMs but how badly the phases of a slab overlap (see
// the timing-only decomposition further down).
//
// Both operands go global -> LDS directly (global_load_lds_dwordx4: no staging registers)
// into a ring of NS stages, refilled as soon as every wave holds a slab's last fragments in registers.  A direct load
// writes the 64 lanes' 16-byte pieces to consecutive LDS addresses, so rows are stored
// unpadded (128 bytes) and 16-byte chunk c of row r lives at chunk position c ^ (r & 7);
// fragment reads of 32 rows x 2 chunks then run at the LDS's full rate (measured).  Pieces
// outside the matrices (K tail, rows >= N, slabs past the split's end) are fetched from a block
// of zeros, so no lane is ever switched off and the wait counts are static.
//
// Work is dealt out in runs of K slabs: the K loops of all column tiles, laid end to end, are
// cut into equal runs of `quota` slabs, one run per workgroup.  With few tiles the host makes
// the quota a whole fraction of a tile's K loop (split-K: every piece starts a fresh pipeline,
// so pieces should not be cut twice); with more tiles than divide well over the CUs it deals
// stream-K fashion, a run ending in the middle of a tile and continuing with the next one, so
// that every CU gets the same share whatever the tile count.  Each piece of a tile stores its partial product as a slice of a scratch buffer with plain
// stores, and the kernel that consumes the GEMM's output anyway (RoPE, SwiGLU, the next RMSNorm)
// adds the slices of a tile up (SliceMap).  Measured alternatives: fp32 atomic adds onto one
// buffer complete at about 1.1 TB/s on this chip (40 % of the GEMM time at 128 rows), and whole
// tiles per workgroup leave CUs idle or cost a second, mostly empty round (344 tiles on 256 CUs
// take as long as 512).  The M tiles of a column tile run as sibling workgroups over the same
// run of slabs on one XCD (workgroups are dealt to the 8 XCDs round robin), so the re-reads of
// a weight tile hit that XCD's L2.
#pragma once
#include "ll_device.h"

struct GemmArgs {
  const half_t* A;        // [>= mtiles * BM rows][K]
  const half_t* W[3];
  const half_t* Wf;       // optional: matrix 0 in the short-prompt kernels' fragment-major order (16-row blocks x
                          // 32-wide K steps, 1 KB each, zero beyond K; see sk_shuffle_kernel with plain row blocks);
                          // kernels instantiated with WFRAG read the weights from it in whole 1 KB pieces
  float* C;               // slices: [slice][rows][ldc]
  const DevState* st;
  const half_t* zeros;    // >= 16 bytes of zeros in global memory
  int N, K, ldc, nmat;
  int mtiles;             // tiles of BM rows
  int runs;               // workgroups per M tile that have work
  SliceMap map;
};

#define PF_BN 256
#define PF_SLAB 64            // K slabs as the host's plan counts them; a kernel may walk one in BK-wide halves
#define PF_GEMM_LDS_BYTES(BM, NS, BK) ((NS) * ((BM) + PF_BN) * (BK) * 2)
#define PF_GEMM_THREADS_OF(WM, WN) ((WM) * (WN) * 64)


// BM x 256 tile, WM x WN waves of (BM / WM) x (256 / WN) each, NS ring stages of BK-wide slabs.
//   <128, 3, 2, 4, 64>  8 waves of 64 x 64: prompts of 65..255 rows
//   <64, 3, 1, 4, 64>   4 waves of 64 x 64: prompts of at most 64 rows
// Measured and not instantiated: <256, 4 or 5, 2, 2, 32>, four waves of 128 x 128 (one per SIMD, 256
// accumulator registers) on 32-wide slabs so that four or five stages fit the LDS.  A wave's k-step
// then reads 4 + 4 fragments from LDS for 16 matrix instructions instead of 2 + 2 for 4, and the tile
// takes a third less from L2 per flop; at 500 tokens Q/K/V, O, gate/up, down ran in 68.9 / 30.8 /
// 107.1 / 58.7 us (five stages; 73.6 / 31.6 / 111.3 / 61.5 with four) against 71 / 29 / 116 / 60 for
// the 128 x 256 tile, the consumers of the then more numerous slices took 11 us per layer longer, and
// at 250 tokens the prefill was 0.4 ms slower: neither LDS reads (SQ_WAIT_INST_LDS under 1 % of the
// wave cycles) nor bytes in flight (+33 % with the fifth stage bought 4-6 %) are what holds these
// GEMMs at 35-40 % of the matrix cores' time.  Two workgroups per CU (<128, 3, 2, 2, 32, 2>: four waves
// of 64 x 128 each, the plan dealing two rounds' worth of runs) lost outright: 82 / 32 / 123 / 67 us; the
// 256 x 256 tile as eight waves of 64 x 128 (<256, 5, 4, 2, 32>) gave 75 / 33 / 115 / 63 us.  Where the
// time goes at 500 tokens, from two timing-only builds of the 128 x 256 kernel: without the global
// loads (matrix instructions, LDS reads, barriers and the stores of the slices) the four projections take
// 41 / 18 / 65 / 34 us, i.e. with 64 x 64 waves the LDS reads alone take as long as the matrix
// instructions and the two overlap poorly; without the matrix instructions (loads, LDS reads, stores)
// 58 / 21 / 96 / 47 us; together 72 / 27 / 118 / 57 us.  FETCH_SIZE counts 210 / 42 / 364 / 157 MB from
// HBM per launch against 101 / 34 / 180 / 90 MB of weights: the four row tiles of a column tile, placed
// on one XCD, share about half of their weight fetches through its L2.  With every workgroup reading the
// same (L2-resident) weight and activation tile the projections still take 62 / 26 / 102 / 55 us (74 / 28 /
// 122 / 58 on the same box): cache misses are a sixth of the time at most.
// Three more structures measured at 500 tokens and not kept: operands staged global -> registers -> ds_write
// instead of direct loads (two slabs in flight in registers): 10 % slower on all four projections; the
// weights' fragments loaded global -> registers from the fragment-major copy, only the activations through LDS
// (four waves of 128 x 64, a third of the LDS traffic): O 28.0 -> 27.2, down 57.3 -> 54.7 us, nothing at 250
// tokens, slower at 128; four waves of 128 x 64 on this kernel: within 2 % either way.  A timing-only build
// that never waits for the direct loads runs as long as the real one, and one without the loads takes 37 / 17 /
// 59 / 32 us: the loads cost their stand-alone time on top of the rest whether or not anybody waits for them.
template <int BM, int NS, int WM, int WN, int BK, int OCC = 1, bool WFRAG = false, bool WNT = (BM == 64)>
__global__ __launch_bounds__(PF_GEMM_THREADS_OF(WM, WN), OCC) void pf_gemm_kernel(GemmArgs g) {
  static_assert(!WFRAG || BK == 64, "the fragment-major weight path pairs two 32-wide K steps per slab");
  constexpr int NWAVES = WM * WN;
  constexpr int MT = BM / WM / 32;                     // 32-row accumulators per wave
  constexpr int NT = PF_BN / WN / 32;                  // 32-column accumulators per wave
  constexpr int SUB = PF_SLAB / BK;                    // ring slabs per plan slab
  constexpr int CPR = BK / 8;                          // 16-byte chunks per LDS row
  constexpr int RPL = 64 / CPR;                        // rows one 1 KB direct load covers
  constexpr int A_LD = BM / RPL / NWAVES;              // direct loads per wave and ring slab
  constexpr int W_LD = PF_BN / RPL / NWAVES;
  constexpr int PER_SLAB = A_LD + W_LD;
  constexpr int STAGE_HALVES = (BM + PF_BN) * BK;
  // Cache policy of the weight loads (WNT).  With one row tile per column tile (prompts of at most 128 rows)
  // every weight byte is used once and is loaded non-temporal (4.29 -> 4.12 ms at 50 tokens); with sibling row
  // tiles the copies that the siblings find in L2 matter more (non-temporal: 11.14 -> 11.40 ms at 500).
  constexpr int W_AUX = WNT ? 2 : 0;
  static_assert(BK == 64 || BK == 32, "swizzles below are for 128- and 64-byte rows");
  static_assert(A_LD >= 1 && W_LD >= 1 && PER_SLAB * NS < 64, "vmcnt is a 6-bit counter");
  extern __shared__ __attribute__((aligned(16))) half_t pf_lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // slot t of XCD x: run (t / mtiles) * 8 + x of the slab sequence, M tile t % mtiles
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int run = (slot / g.mtiles) * 8 + xcd;
  const int m0 = (slot % g.mtiles) * BM;
  if (run >= g.runs || m0 >= g.st->n_prompt) return;
  const int K = g.K, S = g.map.nslabs;                  // S may be padded beyond the K loop's real slabs ...
  const int s_real = (K + PF_SLAB - 1) / PF_SLAB;       // ... so that runs end where tiles end
  const int total_units = g.map.ntiles * g.nmat * S;
  const int r = lane & 31, half = lane >> 5;
  // LDS rows are unpadded; 16-byte chunk c of row r sits at chunk position c ^ swz(r), which spreads
  // the 8 lanes the LDS serves per clock over all of its banks (128-byte rows: 8 rows x 8 chunk
  // positions; 64-byte rows: rows of equal parity share a bank range, 4 of them x 4 positions)
  auto swz = [](int row) { return BK == 64 ? (row & 7) : ((row >> 1) & 3); };
  int u = run * g.map.quota;
  const int u_end = min(u + g.map.quota, total_units);
  while (u < u_end) {
  const int nt_all = u / S;
  const int sl0 = u - nt_all * S;
  const int span = min(S - sl0, u_end - u);
  u += span;
  const int cnt = min(span, s_real - sl0);              // >= 1 by the host's choice of S and quota
  const int slice = run - (nt_all * S) / g.map.quota;
  const int z = nt_all / g.map.ntiles, n0 = (nt_all - z * g.map.ntiles) * PF_BN;

  // this lane's piece of every group of RPL rows: row (lane / CPR), physical chunk (lane % CPR),
  // which holds logical chunk (lane % CPR) ^ swz(row)
  const int lrow = lane / CPR, lchunk = (lane % CPR) ^ swz(lrow);
  const half_t* arow[A_LD];
  const half_t* wrow[W_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i)
    arow[i] = g.A + (size_t)(m0 + (wave * A_LD + i) * RPL + lrow) * K + lchunk * 8;
  const int ksteps32 = (K + 31) >> 5;
#pragma unroll
  for (int i = 0; i < W_LD; ++i) {
    if (WFRAG) {
      // piece f of the stage = 16-row block f / 2 of the tile, K step f % 2 of the slab: 1 KB of consecutive bytes
      const int f = wave * W_LD + i, blk = n0 / 16 + (f >> 1);
      wrow[i] = (blk * 16 < g.N) ? g.Wf + (((size_t)blk * ksteps32 + (f & 1)) * 64 + lane) * 8 : nullptr;
    } else {
      const int n = n0 + (wave * W_LD + i) * RPL + lrow;
      wrow[i] = (n < g.N) ? g.W[z] + (size_t)n * K + lchunk * 8 : nullptr;
    }
  }
  // Every workgroup walks its K range from a different starting slab (and wraps around): all
  // tiles reading the same 128-byte column of their weight rows at the same time would keep
  // hitting the same few memory channels, since the rows lie a multiple of 2 K bytes apart.
  const int rot = (nt_all * 7) % cnt;
  const int iters = cnt * SUB;
  // one of a slab's PER_SLAB direct loads (the activations' first): ring slab `it` into `stage`
  auto issue_one = [&](int it, int stage, int idx) {
    half_t* sa = pf_lds + stage * STAGE_HALVES;
    half_t* sw = sa + BM * BK;
    const int ps = it / SUB, sub = it - ps * SUB;         // plan slab (rotated below) and the BK-wide part of it
    const int sl = sl0 + (ps + rot < cnt ? ps + rot : ps + rot - cnt);
    const int k0 = sl * PF_SLAB + sub * BK;
    const bool kin = it < iters && k0 + lchunk * 8 < K;   // K % 8 == 0: a chunk is all in or all out
    if (idx < A_LD) {
      const half_t* src = kin ? arow[idx] + k0 : g.zeros;
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)src,
                                       (__attribute__((address_space(3))) void*)(sa + (wave * A_LD + idx) * RPL * BK),
                                       16, 0, 0);
    } else {
      const int i = idx - A_LD;
      const half_t* src;
      if (WFRAG) {          // K step 2 sl + (piece % 2); the copy is zero beyond K, steps past its end come from the zeros
        const int st = sl * 2 + ((wave * W_LD + i) & 1);
        src = (it < iters && st < ksteps32 && wrow[i]) ? wrow[i] + (size_t)sl * 1024 : g.zeros;
      } else {
        src = (kin && wrow[i]) ? wrow[i] + k0 : g.zeros;
      }
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)src,
                                       (__attribute__((address_space(3))) void*)(sw + (wave * W_LD + i) * RPL * BK),
                                       16, 0, W_AUX);
    }
  };

  f16v acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  constexpr int KS = BK / 16;
  static_assert(KS % 2 == 0, "the fragment double buffer keeps its parity across slabs");
  // A refill's direct loads are not issued in one burst behind the barrier but dealt over the k-steps that
  // follow, one behind a matrix instruction each: slot 0 is the slab's last k-step (behind the hand-over),
  // slot s is k-step s - 1 of the next slab.  A wave issues in order, so a wave waiting to issue the next load
  // of a burst cannot issue its matrix instructions either (measured at 500 tokens: Q/K/V 62.9 -> 61.6 us,
  // gate/up 103.9 -> 102.6 us).
  auto slot_of = [](int idx) { return idx * KS / PER_SLAB; };
  constexpr int N_SLOT0 = (PER_SLAB + KS - 1) / KS;      // loads with slot_of(idx) == 0
  static_assert(N_SLOT0 <= MT * NT, "one load behind each matrix instruction at most");

  __syncthreads();        // a previous piece's last fragment reads are over before its ring is refilled
  // slabs 0 .. NS - 2 whole, and slot 0 of slab NS - 1: what the loop's first k-steps expect to be under way
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
#pragma unroll
    for (int idx = 0; idx < PER_SLAB; ++idx) issue_one(s, s, idx);
#pragma unroll
  for (int idx = 0; idx < PER_SLAB; ++idx)
    if (slot_of(idx) == 0) issue_one(NS - 1, NS - 1, idx);

  // fragments of the next k-step are read from LDS while the matrix cores work on the current one
  auto load_frags = [&](int stage, int ks, h8 (&fa)[MT], h8 (&fb)[NT]) {
    const half_t* sa = pf_lds + stage * STAGE_HALVES + (wm * (BM / WM) + r) * BK;
    const half_t* sw = pf_lds + stage * STAGE_HALVES + (BM + wn * (PF_BN / WN) + r) * BK;
    const int pc = ((ks * 2 + half) ^ swz(r)) * 8;    // all fragment rows start at multiples of 32
#pragma unroll
    for (int i = 0; i < MT; ++i) fa[i] = *reinterpret_cast<const h8*>(sa + i * 32 * BK + pc);
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      if (WFRAG) {
        // row R of the tile sits in piece (R / 16) * 2 + ks / 2 at lane position ((ks % 2) * 2 + half) * 16 + R % 16:
        // 8 lanes read 128 consecutive bytes, no swizzle needed
        const int R = wn * (PF_BN / WN) + j * 32 + r;
        fb[j] = *reinterpret_cast<const h8*>(pf_lds + stage * STAGE_HALVES + BM * BK +
                                             ((((R >> 4) * 2 + (ks >> 1)) * 64) + ((ks & 1) * 2 + half) * 16 + (R & 15)) * 8);
      } else {
        fb[j] = *reinterpret_cast<const h8*>(sw + j * 32 * BK + pc);
      }
    }
  };
  // The slab hand-over sits in front of a slab's LAST k-step, not behind it: by then a wave holds the
  // slab's last fragments in registers, so once every wave is there the slab's stage is free and its refill
  // starts at once, and the first fragments of the next slab are read while the matrix cores still work on
  // this one; the barrier and the LDS reads that open a slab are hidden behind a k-step of matrix
  // instructions instead of leaving them idle.
  auto hand_over = [&]() {
    // This wave's pieces of the next slab have landed: behind them stands exactly one slab's worth of
    // younger loads per ring stage beyond two (slot 0 of a refill is issued in the k-step after this, the
    // other slots in the k-steps before the next hand-over) ...
    wait_vm_at_most<PER_SLAB * (NS - 2)>();
    // ... its fragment reads of this slab are done, and after the barrier so are everybody else's.
    // A bare s_barrier: __syncthreads() carries a fence that would drain ALL loads in flight.
    wait_lgkm_at_most<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  h8 fa[2][MT], fb[2][NT];
  wait_vm_at_most<PER_SLAB * (NS - 2) + N_SLOT0>();      // slab 0 is in
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  load_frags(0, 0, fa[0], fb[0]);
  // Scheduling fences pin the pipeline: per k-step the wait for this k-step's fragments, the LDS reads of the
  // next k-step, then the matrix instructions with the refill's loads between them.  Left alone the compiler
  // sinks every read to just before its use, and it waits for ALL outstanding LDS reads wherever it waits for
  // one (it does not count them here): requested behind the new reads, this k-step's fragments would cost a
  // whole LDS round trip in front of every second k-step.  Measured at 500 tokens, Q/K/V / O / gate/up / down:
  // 64.5 / 26.4 / 105.9 / 54.1 us with the compiler's waits, 61.6 / 25.4 / 102.6 / 52.2 us as below.
  __builtin_amdgcn_sched_barrier(0);
  for (int it = 0; it < iters; ++it) {
    const int stage = it % NS;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) {
        // the last k-step's fragments were waited for by the hand-over
        wait_lgkm_at_most<0>();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(stage, ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
      }
      // refill `rf` (slab rf + NS into stage rf % NS, free since the hand-over of slab rf): this k-step's share
      const int rf = ks == KS - 1 ? it : it - 1;
      const int rstage = ks == KS - 1 ? stage : (stage == 0 ? NS - 1 : stage - 1);
      const int slot = (ks + 1) % KS;
      const int first = (slot * PER_SLAB + KS - 1) / KS;      // lowest idx with slot_of(idx) == slot
#pragma unroll
      for (int t = 0; t < MT * NT; ++t) {
        const int i = t % MT, j = t / MT;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (first + t < PER_SLAB && slot_of(first + t) == slot) {
          issue_one(rf + NS, rstage, first + t);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (ks == KS - 2) {
        hand_over();
        load_frags((it + 1) % NS, 0, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  wait_vm_at_most<0>();   // the zero-filled look-ahead loads must not outlive the workgroup's LDS

  // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32) and
  // rows 8*(e/4) + 4*(lane/32) + e%4 for e = 0..15
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int col = n0 + wn * (PF_BN / WN) + j * 32 + r;
    if (col >= g.N) continue;
    float* cbase = g.C + slice * g.map.slice_floats + (size_t)z * g.N + col +
                   (size_t)(m0 + wm * (BM / WM) + 4 * half) * g.ldc;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e)
        *as_global(cbase + (size_t)(i * 32 + 8 * (e >> 2) + (e & 3)) * g.ldc) = acc[i][j][e];
  }
  }   // next piece of this workgroup's run
}

