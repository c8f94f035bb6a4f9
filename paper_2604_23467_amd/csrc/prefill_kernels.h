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
// buffer the following split-K GEMM accumulates into.
__global__ __launch_bounds__(LL_WG) void pf_rmsnorm_kernel(const float* __restrict__ X,
                                                           const half_t* __restrict__ gain,
                                                           half_t* __restrict__ Xn, int d, float eps,
                                                           float* __restrict__ zero_buf,
                                                           int zero_row_floats) {
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
    *reinterpret_cast<h4*>(Xn + (size_t)r * d + i) = o;
  }
  float* z = zero_buf + (size_t)r * zero_row_floats;
  const f4 zero = {0.f, 0.f, 0.f, 0.f};
  for (int i = tid * 4; i < zero_row_floats; i += LL_WG * 4) *reinterpret_cast<f4*>(z + i) = zero;
}

// C[M][ldc] (fp32) += A[M][K] (fp16) * W_z[N][K]^T (fp16) for z < nmat, output
// columns z*N + n.  64x64 tile per workgroup, K walked in 64-wide slabs through
// LDS with the next slab prefetched into registers; four waves each own one
// 32x32 MFMA accumulator.  Split-K over blockIdx.y with fp32 atomic adds: the
// prompt lengths here give few output tiles, and it is the weight stream (read
// once) that has to be spread over all CUs.  Workgroup -> tile mapping keeps
// the M-tiles that share a weight tile on one XCD (workgroups are dealt to the
// 8 XCDs round robin), so the re-reads hit that XCD's L2.
struct GemmArgs {
  const half_t* A;
  const half_t* W[3];
  float* C;
  const DevState* st;
  int N, K, ldc, nmat;
  int mtiles, ntiles;   // tiles of 64 rows / 64 columns (per matrix)
  int kt_per_split;     // 64-wide K slabs per blockIdx.y
};

#define PF_BM 64
#define PF_BN 64
#define PF_BK 64
#define PF_LDS_STRIDE 72   // halves; 144-byte rows keep 16-byte fragment reads spread over banks

__global__ __launch_bounds__(LL_WG) void pf_gemm_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(16))) half_t As[PF_BM * PF_LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) half_t Ws[PF_BN * PF_LDS_STRIDE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // XCD-aware tile order: slot t of XCD x handles n-tile (t / mtiles) * 8 + x, m-tile t % mtiles
  const int total_nt = g.ntiles * g.nmat;
  const int b = blockIdx.x;
  const int xcd = b & 7, slot = b >> 3;
  const int nt_all = (slot / g.mtiles) * 8 + xcd;
  const int mt = slot % g.mtiles;
  if (nt_all >= total_nt) return;
  const int z = nt_all / g.ntiles, nt = nt_all - z * g.ntiles;
  const int m0 = mt * PF_BM, n0 = nt * PF_BN;
  if (m0 >= g.st->n_prompt) return;

  const int K = g.K;
  const int ktiles = (K + PF_BK - 1) / PF_BK;
  const int kt0 = blockIdx.y * g.kt_per_split;
  const int kt1 = min(kt0 + g.kt_per_split, ktiles);
  if (kt0 >= kt1) return;

  const half_t* A = g.A;
  const half_t* W = g.W[z];

  // global -> register staging: 2 x 16 bytes of A and of W per thread per slab
  int lrow[2], lk[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int idx = tid + i * LL_WG;
    lrow[i] = idx >> 3;
    lk[i] = (idx & 7) * 8;
  }
  h8 ra[2], rw[2];
  const h8 hz = {0, 0, 0, 0, 0, 0, 0, 0};
  auto fetch = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int k = kt * PF_BK + lk[i];
      const bool kin = k < K;   // K is a multiple of 8, so a 16-byte chunk is all in or all out
      ra[i] = kin ? *reinterpret_cast<const h8*>(A + (size_t)(m0 + lrow[i]) * K + k) : hz;
      const int n = n0 + lrow[i];
      rw[i] = (kin && n < g.N) ? load_stream(W + (size_t)n * K + k) : hz;
    }
  };

  const int wm = wave >> 1, wn = wave & 1;
  f16v acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  fetch(kt0);
  for (int kt = kt0; kt < kt1; ++kt) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *reinterpret_cast<h8*>(As + lrow[i] * PF_LDS_STRIDE + lk[i]) = ra[i];
      *reinterpret_cast<h8*>(Ws + lrow[i] * PF_LDS_STRIDE + lk[i]) = rw[i];
    }
    __syncthreads();
    if (kt + 1 < kt1) fetch(kt + 1);
#pragma unroll
    for (int ks = 0; ks < PF_BK / 16; ++ks) {
      const int kk = ks * 16 + (lane >> 5) * 8;
      const h8 fa = *reinterpret_cast<const h8*>(As + (wm * 32 + (lane & 31)) * PF_LDS_STRIDE + kk);
      const h8 fb = *reinterpret_cast<const h8*>(Ws + (wn * 32 + (lane & 31)) * PF_LDS_STRIDE + kk);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa, fb, acc, 0, 0, 0);
    }
    __syncthreads();
  }

  // accumulator layout of the 32x32 MFMA: lane holds column (lane % 32) and
  // rows 8*(i/4) + 4*(lane/32) + i%4 for i = 0..15
  const int col = n0 + wn * 32 + (lane & 31);
  if (col < g.N) {
    float* cbase = g.C + (size_t)z * g.N + col;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = m0 + wm * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
      unsafeAtomicAdd(cbase + (size_t)row * g.ldc, acc[i]);
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

// Causal attention for a block of 32 queries of one head.  grid = (heads, Mb/32).
// Eight lanes share a query (HD/8 columns each); key/value tiles of 32 rows are
// staged in LDS and every query walks them with an online softmax.
template <int HD>
__global__ __launch_bounds__(LL_WG) void pf_attn_kernel(const half_t* __restrict__ Q,
                                                        const half_t* __restrict__ kc,
                                                        const half_t* __restrict__ vc,
                                                        const DevState* __restrict__ st,
                                                        half_t* __restrict__ O, int d, int max_seq) {
  constexpr int QB = 32, TK = 32, SEG = HD / 8;
  __shared__ __attribute__((aligned(16))) half_t Ks[TK * HD];
  __shared__ __attribute__((aligned(16))) half_t Vs[TK * HD];
  const int h = blockIdx.x, q0 = blockIdx.y * QB;
  const int n = st->n_prompt;
  if (q0 >= n) return;
  const int tid = threadIdx.x;
  const int qi = q0 + (tid >> 3), seg = tid & 7;
  const float scale = 1.0f / sqrtf((float)HD);

  float qv[SEG], acc[SEG];
  {
    const half_t* qp = Q + (size_t)min(qi, n - 1) * d + h * HD + seg * SEG;
#pragma unroll
    for (int e = 0; e < SEG; ++e) { qv[e] = (float)qp[e] * scale; acc[e] = 0.f; }
  }
  float m = -INFINITY, l = 0.f;
  const half_t* kh = kc + (size_t)h * max_seq * HD;
  const half_t* vh = vc + (size_t)h * max_seq * HD;
  const int last_key = min(q0 + QB, n) - 1;   // inclusive, the block's last valid query attends it

  for (int k0 = 0; k0 <= last_key; k0 += TK) {
    __syncthreads();
    for (int i = tid; i < TK * HD / 8; i += LL_WG) {
      const int kr = min(k0 + i / (HD / 8), n - 1);
      const int c = (i % (HD / 8)) * 8;
      *reinterpret_cast<h8*>(Ks + (i / (HD / 8)) * HD + c) =
          *reinterpret_cast<const h8*>(kh + (size_t)kr * HD + c);
      *reinterpret_cast<h8*>(Vs + (i / (HD / 8)) * HD + c) =
          *reinterpret_cast<const h8*>(vh + (size_t)kr * HD + c);
    }
    __syncthreads();
    const int kend = min(TK, last_key - k0 + 1);
    for (int t = 0; t < kend; ++t) {
      const half_t* kp = Ks + t * HD + seg * SEG;
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < SEG; ++e) dot += qv[e] * (float)kp[e];
      dot = group_sum<8>(dot);
      if (k0 + t <= qi) {
        const half_t* vp = Vs + t * HD + seg * SEG;
        const float mn = fmaxf(m, dot);
        const float corr = __expf(m - mn);
        const float p = __expf(dot - mn);
        l = l * corr + p;
#pragma unroll
        for (int e = 0; e < SEG; ++e) acc[e] = acc[e] * corr + p * (float)vp[e];
        m = mn;
      }
    }
  }
  if (qi < n) {
    half_t* op = O + (size_t)qi * d + h * HD + seg * SEG;
    const float rl = 1.0f / l;
#pragma unroll
    for (int e = 0; e < SEG; ++e) op[e] = (half_t)(acc[e] * rl);
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
