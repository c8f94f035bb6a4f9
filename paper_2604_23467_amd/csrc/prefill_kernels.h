// Short-prompt prefill kernels for gfx950 (prompts of 10-500 tokens, the
// paper's TTFT regime, Sec. IV-E / Table I): the same layer as the decode path
// but for n rows at positions 0..n-1, so the projections are real dense
// contractions and run on the matrix cores (v_mfma_f32_32x32x16_f16, fp16
// operands, fp32 accumulate), and attention is LDS-tiled and causal.
//
// Every kernel is launched on a grid sized for a prompt-length bucket Mb and
// reads the true n from DevState, so one captured graph per bucket serves all
// prompts that fit it.  Rows >= n are zero on entry and never reach the KV
// cache or the logits.
#pragma once
#include "ll_device.h"

// X[r] = float(E[tokens[r]]) for r < n, 0 otherwise.  grid = (Mb, ceil(d / 2048))
__global__ __launch_bounds__(LL_WG) void pf_embed_kernel(const half_t* __restrict__ emb,
                                                         const int* __restrict__ tokens,
                                                         const DevState* __restrict__ st,
                                                         float* __restrict__ X, int d) {
  const int r = blockIdx.x;
  const int i = (blockIdx.y * LL_WG + threadIdx.x) * 8;
  if (i >= d) return;
  float* xr = X + (size_t)r * d + i;
  if (r < st->n_prompt) {
    const h8 e = *reinterpret_cast<const h8*>(emb + (size_t)tokens[r] * d + i);
#pragma unroll
    for (int j = 0; j < 8; ++j) xr[j] = (float)e[j];
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) xr[j] = 0.f;
  }
}

// Row-wise RMSNorm of the fp32 residual stream into fp16 GEMM operands, one
// workgroup per row.  As a side job each workgroup clears its row of the fp32
// buffer the following split-K GEMM accumulates into.  frag_tb != 0 writes the
// operands in the short-prompt kernels' fragment-major layout.
__global__ __launch_bounds__(LL_WG) void pf_rmsnorm_kernel(const float* __restrict__ X,
                                                           const half_t* __restrict__ gain,
                                                           half_t* __restrict__ Xn, int d, float eps,
                                                           float* __restrict__ zero_buf,
                                                           int zero_row_floats, int frag_tb) {
  __shared__ float red[LL_WG / 64];
  const int r = blockIdx.x, tid = threadIdx.x;
  const float* xr = X + (size_t)r * d;
  float ss = 0.f;
  for (int i = tid * 4; i < d; i += LL_WG * 4) {
    const f4 v = *reinterpret_cast<const f4*>(xr + i);
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const float inv = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
  for (int i = tid * 4; i < d; i += LL_WG * 4) {
    const f4 v = *reinterpret_cast<const f4*>(xr + i);
    const h4 g = *reinterpret_cast<const h4*>(gain + i);
    h4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (half_t)(v[j] * inv * (float)g[j]);
    *reinterpret_cast<h4*>(Xn + act_offset(r, i, d, frag_tb)) = o;
  }
  float* z = zero_buf + (size_t)r * zero_row_floats;
  const f4 zero = {0.f, 0.f, 0.f, 0.f};
  for (int i = tid * 4; i < zero_row_floats; i += LL_WG * 4) *reinterpret_cast<f4*>(z + i) = zero;
}

// C[M][ldc] (fp32) += A[M][K] (fp16) * W_z[N][K]^T (fp16) for z < nmat, output
// columns z*N + n.  BM x 128 tile per workgroup (BM = 64 for the short-prompt
// bucket, 128 otherwise), four waves in a 2 x 2 arrangement, each owning a
// (BM/2) x 64 block = BM/64 x 2 MFMA accumulators of 32 x 32.
//
// K is walked in 64-wide slabs through a ring of PF_STAGES LDS buffers that is
// filled by direct global->LDS loads (global_load_lds_dwordx4: no staging
// registers), PF_STAGES - 1 slabs ahead of the one being multiplied.  With
// both operands in LDS a 64 x 64 wave tile moves 1 KB of LDS per MFMA, which
// is what bounds this kernel (measured: dropping the MFMAs changes nothing,
// dropping the loads gains 25 %), so LDS capacity is better spent on a second
// resident workgroup than on deeper prefetch: 2 stages for the 128-row tile
// (measured against 3 and 4).  The 64-row tile of the short-prompt bucket is
// bound by the weight stream instead and gets 3 stages.  A direct load writes the 64 lanes' 16-byte pieces to consecutive LDS addresses, so
// rows are stored unpadded (128 bytes) and bank conflicts are avoided by an XOR
// swizzle instead: 16-byte chunk c of row r lives at chunk position c ^ (r & 7).
// Pieces outside the matrices (K tail, rows >= N) are fetched from a block of
// zeros, so no lane is ever switched off.
//
// Split-K over blockIdx.y with fp32 atomic adds when the prompt gives too few
// output tiles to spread the weight stream (read once) over all CUs; with one
// split the tile is added with plain read-modify-writes.  Workgroup -> tile
// mapping keeps the M-tiles that share a weight tile on one XCD (workgroups
// are dealt to the 8 XCDs round robin), so the re-reads hit that XCD's L2.
struct GemmArgs {
  const half_t* A;
  const half_t* W[3];
  float* C;
  const DevState* st;
  const half_t* zeros;  // >= 16 bytes of zeros in global memory
  int N, K, ldc, nmat;
  int mtiles, ntiles;   // tiles of BM rows / 128 columns (per matrix)
  int kt_per_split;     // 64-wide K slabs per blockIdx.y
  int atomic;           // more than one K split: accumulate with atomics
};

#define PF_BN 128
#define PF_BK 64
#define PF_GEMM_LDS_BYTES(BM, STAGES) ((STAGES) * ((BM) + PF_BN) * PF_BK * 2)

template <int N>
__device__ __forceinline__ void wait_vm_at_most() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int BM, int PF_STAGES>
__global__ __launch_bounds__(LL_WG) void pf_gemm_kernel(GemmArgs g) {
  constexpr int MT = BM / 64;             // 32-row MFMA tiles per wave
  constexpr int A_LD = BM / 32;           // 1 KB direct loads per wave and slab for A (8 rows each)
  constexpr int W_LD = PF_BN / 32;
  constexpr int STAGE_HALVES = (BM + PF_BN) * PF_BK;
  extern __shared__ __attribute__((aligned(16))) half_t pf_lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // XCD-aware tile order: slot t of XCD x handles n-tile (t / mtiles) * 8 + x, m-tile t % mtiles
  const int total_nt = g.ntiles * g.nmat;
  const int b = blockIdx.x;
  const int xcd = b & 7, slot = b >> 3;
  const int nt_all = (slot / g.mtiles) * 8 + xcd;
  const int mt = slot % g.mtiles;
  if (nt_all >= total_nt) return;
  const int z = nt_all / g.ntiles, nt = nt_all - z * g.ntiles;
  const int m0 = mt * BM, n0 = nt * PF_BN;
  if (m0 >= g.st->n_prompt) return;

  const int K = g.K;
  const int ktiles = (K + PF_BK - 1) / PF_BK;
  const int kt0 = blockIdx.y * g.kt_per_split;
  const int kt1 = min(kt0 + g.kt_per_split, ktiles);
  if (kt0 >= kt1) return;

  // this lane's piece of every 8-row block: row (lane / 8), physical chunk (lane % 8),
  // which holds logical chunk (lane % 8) ^ (row & 7) = (lane % 8) ^ (lane / 8)
  const int lrow = lane >> 3;
  const int lchunk = (lane & 7) ^ lrow;
  const half_t* arow[A_LD];
  const half_t* wrow[W_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i)
    arow[i] = g.A + (size_t)(m0 + (wave * A_LD + i) * 8 + lrow) * K + lchunk * 8;
#pragma unroll
  for (int i = 0; i < W_LD; ++i) {
    const int n = n0 + (wave * W_LD + i) * 8 + lrow;
    wrow[i] = (n < g.N) ? g.W[z] + (size_t)n * K + lchunk * 8 : nullptr;
  }
  auto issue = [&](int kt, int stage) {
    half_t* sa = pf_lds + stage * STAGE_HALVES;
    half_t* sw = sa + BM * PF_BK;
    const bool kin = kt < kt1 && kt * PF_BK + lchunk * 8 < K;   // K % 8 == 0: a chunk is all in or all out
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
      const half_t* src = kin ? arow[i] + kt * PF_BK : g.zeros;
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)src,
                                       (__attribute__((address_space(3))) void*)(sa + (wave * A_LD + i) * 8 * PF_BK),
                                       16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < W_LD; ++i) {
      const half_t* src = (kin && wrow[i]) ? wrow[i] + kt * PF_BK : g.zeros;
      __builtin_amdgcn_global_load_lds((const LL_GLOBAL void*)src,
                                       (__attribute__((address_space(3))) void*)(sw + (wave * W_LD + i) * 8 * PF_BK),
                                       16, 0, 0);
    }
  };

  const int wm = wave >> 1, wn = wave & 1;
  f16v acc[MT][2];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

#pragma unroll
  for (int s = 0; s < PF_STAGES - 1; ++s) issue(kt0 + s, s);

  for (int kt = kt0; kt < kt1; ++kt) {
    const int stage = (kt - kt0) % PF_STAGES;
    // this wave's pieces of slab kt have landed (later slabs may still be in flight) ...
    wait_vm_at_most<(A_LD + W_LD) * (PF_STAGES - 2)>();
    // ... and so have everybody else's; everybody is also done reading slab kt - 1.
    // A bare s_barrier: __syncthreads() carries a fence that would drain ALL loads in flight.
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(kt + PF_STAGES - 1, (stage + PF_STAGES - 1) % PF_STAGES);
    const half_t* sa = pf_lds + stage * STAGE_HALVES;
    const half_t* sw = sa + BM * PF_BK;
    // fragments of k-step ks + 1 are read from LDS while the matrix cores work on k-step ks
    const int r = lane & 31;
    auto load_frags = [&](int ks, h8 (&fa)[MT], h8 (&fb)[2]) {
      const int c = ks * 2 + (lane >> 5);           // logical 16-byte chunk of the row
      const int pc = (c ^ (r & 7)) * 8;              // all tile rows start at multiples of 8
#pragma unroll
      for (int i = 0; i < MT; ++i)
        fa[i] = *reinterpret_cast<const h8*>(sa + (wm * (BM / 2) + i * 32 + r) * PF_BK + pc);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const h8*>(sw + (wn * 64 + j * 32 + r) * PF_BK + pc);
    };
    h8 fa[2][MT], fb[2][2];
    load_frags(0, fa[0], fb[0]);
#pragma unroll
    for (int ks = 0; ks < PF_BK / 16; ++ks) {
      if (ks + 1 < PF_BK / 16) load_frags(ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
    }
  }
  wait_vm_at_most<0>();   // the zero-filled look-ahead loads must not outlive the workgroup's LDS

  // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32) and
  // rows 8*(e/4) + 4*(lane/32) + e%4 for e = 0..15
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = n0 + wn * 64 + j * 32 + (lane & 31);
    if (col >= g.N) continue;
    float* cbase = g.C + (size_t)z * g.N + col;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm * (BM / 2) + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        float* cp = cbase + (size_t)row * g.ldc;
        if (g.atomic) unsafeAtomicAdd(cp, acc[i][j][e]);
        else *cp += acc[i][j][e];
      }
  }
}

// RoPE on the q and k thirds of QKV[r] (fp32, [Mb][3d]) at position r, then
// q -> fp16 Q[r], k/v -> the KV cache rows of position r.  grid = (Mb), rows >= n idle.
__global__ __launch_bounds__(LL_WG) void pf_rope_kv_kernel(const float* __restrict__ QKV,
                                                           const float2* __restrict__ rope,
                                                           const DevState* __restrict__ st,
                                                           half_t* __restrict__ Q,
                                                           half_t* __restrict__ kc,
                                                           half_t* __restrict__ vc, int d,
                                                           int head_dim, int max_seq) {
  const int r = blockIdx.x;
  if (r >= st->n_prompt) return;
  const int hh = head_dim >> 1;
  const float* row = QKV + (size_t)r * 3 * d;
  for (int p = threadIdx.x; p < d / 2; p += LL_WG) {
    const int head = p / hh, j = p - head * hh;
    const int ia = head * head_dim + j, ib = ia + hh;
    const float2 cs = rope[(size_t)r * hh + j];
    const float qa = row[ia], qb = row[ib];
    Q[(size_t)r * d + ia] = (half_t)(qa * cs.x - qb * cs.y);
    Q[(size_t)r * d + ib] = (half_t)(qb * cs.x + qa * cs.y);
    const float ka = row[d + ia], kb = row[d + ib];
    half_t* kr = kc + ((size_t)head * max_seq + r) * head_dim;
    kr[j] = (half_t)(ka * cs.x - kb * cs.y);
    kr[j + hh] = (half_t)(kb * cs.x + ka * cs.y);
    half_t* vr = vc + ((size_t)head * max_seq + r) * head_dim;
    vr[j] = (half_t)row[2 * d + ia];
    vr[j + hh] = (half_t)row[2 * d + ib];
  }
}

// Causal attention of one head for a block of 64 queries, on the matrix cores.
// grid = (heads, Mb / 64), 128 threads: each of the two waves owns 32 queries
// and walks the keys in tiles of 32 with an online softmax.
//
// Both products are computed transposed so that the softmax needs no transpose:
//   S^T[key][q] = sum_d K[key][d] Q[q][d]      A = K tile (LDS), B = Q (registers)
//   O^T[d][q]  += sum_key V[key][d] P[q][key]  A = V^T tile (LDS), B = P^T (registers)
// In the 32x32 accumulator layout a lane holds ONE query column (lane % 32) and
// 16 of the 32 key rows (the other 16 sit in lane ^ 32), so the row max / sum is
// 15 register operations plus one cross-half shuffle, the rescale of O^T is a
// per-lane scalar, and the probabilities are already in B-operand position:
// k-slot j of lane half hf in k-step s holds key 16 s + 8 (j / 4) + 4 hf + j % 4.
// The V tile is written to LDS transposed with its keys in exactly that order,
// so an A fragment of V^T is one 16-byte LDS read.
template <int HD>
__global__ __launch_bounds__(128) void pf_attn_kernel(const half_t* __restrict__ Q,
                                                      const half_t* __restrict__ kc,
                                                      const half_t* __restrict__ vc,
                                                      const DevState* __restrict__ st,
                                                      half_t* __restrict__ O, int d, int max_seq,
                                                      int frag_tb) {
  constexpr int QB = 64, TK = 32, KS = HD / 16, DT = HD / 32, CPR = HD / 8;
  constexpr int K_STRIDE = HD + 8;   // halves: 16-byte fragment reads of 8 rows hit 8 distinct bank groups
  constexpr int V_STRIDE = 40;       // halves per d row of V^T (32 keys + pad)
  __shared__ __attribute__((aligned(16))) half_t Ks[TK * K_STRIDE];
  __shared__ __attribute__((aligned(16))) half_t Vt[HD * V_STRIDE];
  const int h = blockIdx.x, q0 = blockIdx.y * QB;
  const int n = st->n_prompt;
  if (q0 >= n) return;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qi = q0 + wave * 32 + ql;
  const int wave_last_q = q0 + wave * 32 + 31;
  const float scale = 1.0f / sqrtf((float)HD);

  h8 qf[KS];
  {
    const half_t* qp = Q + (size_t)min(qi, n - 1) * d + h * HD + hf * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = load_h8(qp + ks * 16);
  }
  f16v acc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  float m = -INFINITY, l = 0.f;

  const half_t* kh = kc + (size_t)h * max_seq * HD;
  const half_t* vh = vc + (size_t)h * max_seq * HD;
  const int last_key = min(q0 + QB, n) - 1;   // the block's last valid query attends it

  for (int k0 = 0; k0 <= last_key; k0 += TK) {
    __syncthreads();   // the previous tile has been consumed
    for (int idx = tid; idx < TK * CPR; idx += 128) {
      const int key = idx / CPR, c = idx - key * CPR;
      const int kr = min(k0 + key, n - 1);
      *reinterpret_cast<h8*>(Ks + key * K_STRIDE + c * 8) = load_h8(kh + (size_t)kr * HD + c * 8);
      const h8 v = load_h8(vh + (size_t)kr * HD + c * 8);
      // position of this key inside a V^T row: k-step s = key / 16, then half and slot as above
      const int r16 = key & 15;
      const int pos = ((key >> 4) * 2 + ((r16 & 7) >> 2)) * 8 + (r16 >> 3) * 4 + (r16 & 3);
#pragma unroll
      for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * V_STRIDE + pos] = v[e];
    }
    __syncthreads();
    if (k0 > wave_last_q) continue;   // whole tile above this wave's diagonal

    f16v sc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const h8 a = *reinterpret_cast<const h8*>(Ks + ql * K_STRIDE + ks * 16 + hf * 8);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, qf[ks], sc, 0, 0, 0);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int key = k0 + 8 * (e >> 2) + 4 * hf + (e & 3);
      sc[e] = (key <= qi) ? sc[e] * scale : -INFINITY;
      mx = fmaxf(mx, sc[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mn = fmaxf(m, mx);            // finite: tile 0 always holds key 0 <= qi
    const float corr = __expf(m - mn);
    float rs = 0.f;
    h8 pb[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const float p = __expf(sc[e] - mn);
      rs += p;
      pb[e >> 3][e & 7] = (half_t)p;
    }
    rs += __shfl_xor(rs, 32);
    l = l * corr + rs;
    m = mn;
#pragma unroll
    for (int t = 0; t < DT; ++t) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] *= corr;
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const h8 a = *reinterpret_cast<const h8*>(Vt + (t * 32 + ql) * V_STRIDE + (s2 * 2 + hf) * 8);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[s2], acc[t], 0, 0, 0);
      }
    }
  }

  if (qi < n) {
    const float rl = 1.0f / l;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {   // rows 32 t + 8 g4 + 4 hf + (0..3) of O^T = 4 consecutive columns of O
        h4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = (half_t)(acc[t][g4 * 4 + j] * rl);
        *reinterpret_cast<h4*>(O + act_offset(qi, h * HD + t * 32 + g4 * 8 + hf * 4, d, frag_tb)) = o;
      }
  }
}

// Hm[r][i] = silu(G[r][i]) * U[r][i] with GU = [Mb][2F] fp32 (gate | up).  grid = (Mb, ceil(F/1024))
__global__ __launch_bounds__(LL_WG) void pf_swiglu_kernel(const float* __restrict__ GU,
                                                          const DevState* __restrict__ st,
                                                          half_t* __restrict__ Hm, int F) {
  const int r = blockIdx.x;
  const int i = (blockIdx.y * LL_WG + threadIdx.x) * 4;
  if (i >= F) return;
  h4 o = {0, 0, 0, 0};
  if (r < st->n_prompt) {
    const f4 g = *reinterpret_cast<const f4*>(GU + (size_t)r * 2 * F + i);
    const f4 u = *reinterpret_cast<const f4*>(GU + (size_t)r * 2 * F + F + i);
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (half_t)(g[j] / (1.0f + expf(-g[j])) * u[j]);
  }
  *reinterpret_cast<h4*>(Hm + (size_t)r * F + i) = o;
}
