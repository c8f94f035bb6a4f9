// Short-prompt prefill kernels for gfx950 (prompts of 10-500 tokens, the
// paper's TTFT regime, Sec. IV-E / Table I): the same layer as the decode path
// but for n rows at positions 0..n-1: the elementwise kernels around the
// projection GEMM (prefill_gemm.h) and the causal attention on the matrix cores.
//
// Every kernel is launched on a grid sized for a prompt-length bucket Mb and
// reads the true n from DevState, so one captured graph per bucket serves all
// prompts that fit it.  Rows >= n are zero on entry and never reach the KV
// cache or the logits.  A prompt longer than the largest bucket is fed in
// chunks: DevState.pos holds the number of positions already cached (p0), row r
// of the chunk sits at position p0 + r, and attention also covers the p0 keys
// of the earlier chunks.
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

// Sum of np split-K slices at p (slice stride in floats), four loads in flight at a time.
__device__ __forceinline__ f4 pf_slice_sum(const float* p, int np, size_t slice_floats) {
  f4 v = {0.f, 0.f, 0.f, 0.f};
  int s = 0;
  for (; s + 4 <= np; s += 4) {
    const f4 a = *reinterpret_cast<const f4*>(p + (size_t)s * slice_floats);
    const f4 b = *reinterpret_cast<const f4*>(p + (size_t)(s + 1) * slice_floats);
    const f4 c = *reinterpret_cast<const f4*>(p + (size_t)(s + 2) * slice_floats);
    const f4 e = *reinterpret_cast<const f4*>(p + (size_t)(s + 3) * slice_floats);
    v += (a + b) + (c + e);
  }
  for (; s < np; ++s) v += *reinterpret_cast<const f4*>(p + (size_t)s * slice_floats);
  return v;
}

// Row-wise RMSNorm of the fp32 residual stream into fp16 GEMM operands, one
// 1024-thread workgroup per row.  The residual GEMM in front of it may have left
// its result as np split-K slices ([np][rows][d] at part): they are added to X
// here, X is stored back, and the norm is taken of the sum.  Rows past the prompt
// give zero operands.  frag_tb != 0 writes the operands in the short-prompt
// kernels' fragment-major layout.
#define PF_NORM_THREADS 1024
__global__ __launch_bounds__(PF_NORM_THREADS) void pf_rmsnorm_kernel(float* __restrict__ X,
                                                                     const half_t* __restrict__ gain,
                                                                     half_t* __restrict__ Xn, int d, float eps,
                                                                     const DevState* __restrict__ st,
                                                                     const float* __restrict__ part, SliceMap map,
                                                                     int frag_tb) {
  __shared__ float red[PF_NORM_THREADS / 64];
  const int r = blockIdx.x, tid = threadIdx.x;
  if (r >= st->n_prompt) {
    const h4 zero = {0, 0, 0, 0};
    for (int i = tid * 4; i < d; i += PF_NORM_THREADS * 4)
      *reinterpret_cast<h4*>(Xn + act_offset(r, i, d, frag_tb)) = zero;
    return;
  }
  float* xr = X + (size_t)r * d;
  const float* pr = part + (size_t)r * d;
  float ss = 0.f;
  for (int i = tid * 4; i < d; i += PF_NORM_THREADS * 4) {
    f4 v = *reinterpret_cast<const f4*>(xr + i);
    if (part) {
      v += pf_slice_sum(pr + i, slice_count(map, i), map.slice_floats);
      *reinterpret_cast<f4*>(xr + i) = v;
    }
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < PF_NORM_THREADS / 64; ++w) tot += red[w];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = tid * 4; i < d; i += PF_NORM_THREADS * 4) {
    const f4 v = *reinterpret_cast<const f4*>(xr + i);      // this thread's own stores of the loop above
    const h4 g = *reinterpret_cast<const h4*>(gain + i);
    h4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (half_t)(v[j] * inv * (float)g[j]);
    *reinterpret_cast<h4*>(Xn + act_offset(r, i, d, frag_tb)) = o;
  }
}

// X[r] += the slices of the last residual GEMM (nothing follows it that could).
// grid = (rows, ceil(d / 1024))
__global__ __launch_bounds__(LL_WG) void pf_fold_kernel(float* __restrict__ X, const DevState* __restrict__ st,
                                                        const float* __restrict__ part, SliceMap map, int d) {
  const int r = blockIdx.x, i = (blockIdx.y * LL_WG + threadIdx.x) * 4;
  if (r >= st->n_prompt || i >= d) return;
  float* x = X + (size_t)r * d + i;
  *reinterpret_cast<f4*>(x) = *reinterpret_cast<const f4*>(x) + pf_slice_sum(part + (size_t)r * d + i, slice_count(map, i), map.slice_floats);
}

// RoPE on the q and k thirds of the QKV projection (fp32, slices of [Mb][3d], summed here) at
// position p0 + r, then q -> fp16 Q[r], k/v -> the KV cache rows of position p0 + r.  Four rotation
// pairs per thread with 16-byte loads, every load of a thread issued before the first use
// (head_dim % 8 == 0).  grid = (Mb, ceil(n_heads * head_dim / 8 / LL_WG)), rows >= n idle.
__global__ __launch_bounds__(LL_WG) void pf_rope_kv_kernel(const float* __restrict__ QKV, SliceMap map,
                                                            const float2* __restrict__ rope,
                                                            const DevState* __restrict__ st,
                                                            half_t* __restrict__ Q,
                                                            half_t* __restrict__ kc,
                                                            half_t* __restrict__ vc, int d,
                                                            int head_dim, int max_seq) {
  const int r = blockIdx.x;
  if (r >= st->n_prompt) return;
  const int hh = head_dim >> 1, per_head = hh >> 2;
  const int item = blockIdx.y * LL_WG + threadIdx.x;
  const int head = item / per_head, j = (item - head * per_head) * 4;
  if (head * head_dim >= d) return;
  const int pos = st->pos + r;
  const int ia = head * head_dim + j, ib = ia + hh;
  const float* row = QKV + (size_t)r * 3 * d;
  const f4 c01 = *reinterpret_cast<const f4*>(rope + (size_t)pos * hh + j);       // (cos, sin) of pairs j, j + 1
  const f4 c23 = *reinterpret_cast<const f4*>(rope + (size_t)pos * hh + j + 2);
  auto val = [&](int i) { return pf_slice_sum(row + i, slice_count(map, i), map.slice_floats); };
  const f4 qa = val(ia), qb = val(ib), ka = val(d + ia), kb = val(d + ib), va = val(2 * d + ia), vb = val(2 * d + ib);
  const f4 cs = {c01[0], c01[2], c23[0], c23[2]}, sn = {c01[1], c01[3], c23[1], c23[3]};
  h4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (half_t)(qa[e] * cs[e] - qb[e] * sn[e]);
  *reinterpret_cast<h4*>(Q + (size_t)r * d + ia) = o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (half_t)(qb[e] * cs[e] + qa[e] * sn[e]);
  *reinterpret_cast<h4*>(Q + (size_t)r * d + ib) = o;
  half_t* kr = kc + ((size_t)head * max_seq + pos) * head_dim;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (half_t)(ka[e] * cs[e] - kb[e] * sn[e]);
  *reinterpret_cast<h4*>(kr + j) = o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (half_t)(kb[e] * cs[e] + ka[e] * sn[e]);
  *reinterpret_cast<h4*>(kr + j + hh) = o;
  half_t* vr = vc + ((size_t)head * max_seq + pos) * head_dim;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (half_t)va[e];
  *reinterpret_cast<h4*>(vr + j) = o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (half_t)vb[e];
  *reinterpret_cast<h4*>(vr + j + hh) = o;
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
//
// Long prompts make the last query blocks walk many key tiles, one after the other with nothing
// else on the CU to hide a tile's chain of LDS round trips, matrix instructions and exponentials.
// So G groups of two waves share a query block: group g takes the key tiles g, g + G, ... with
// tile buffers of its own, and group 0 merges the groups' (max, sum, O^T) at the end.
#define PF_ATTN_TILE_HALVES(HD) (32 * ((HD) + 8) + (HD) * 36)
#define PF_ATTN_LDS_BYTES(HD, G) \
  ((G) * PF_ATTN_TILE_HALVES(HD) * 2 > ((G) - 1) * 128 * ((HD) / 2 + 2) * 4 \
       ? (G) * PF_ATTN_TILE_HALVES(HD) * 2 : ((G) - 1) * 128 * ((HD) / 2 + 2) * 4)

template <int HD, int G>
__global__ __launch_bounds__(128 * G) void pf_attn_kernel(const half_t* __restrict__ Q,
                                                          const half_t* __restrict__ kc,
                                                          const half_t* __restrict__ vc,
                                                          const DevState* __restrict__ st,
                                                          half_t* __restrict__ O, int d, int max_seq,
                                                          int frag_tb) {
  constexpr int QB = 64, TK = 32, KS = HD / 16, DT = HD / 32, CPR = HD / 8;
  constexpr int K_STRIDE = HD + 8;   // halves: 16-byte fragment reads of 8 rows hit 8 distinct bank groups
  constexpr int V_STRIDE = 36;       // halves per d row of V^T (32 keys + pad): rows 18 words apart, see stash()
  extern __shared__ __attribute__((aligned(16))) half_t pf_attn_lds[];
  const int h = blockIdx.x, q0 = blockIdx.y * QB;
  const int n = st->n_prompt, p0 = st->pos;   // rows of this chunk, positions cached before it
  if (q0 >= n) return;
  const int tid = threadIdx.x & 127, lane = tid & 63, hf = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7);
  half_t* Ks = pf_attn_lds + grp * PF_ATTN_TILE_HALVES(HD);
  half_t* Vt = Ks + TK * K_STRIDE;
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
  const int last_key = p0 + min(q0 + QB, n) - 1;   // the block's last valid query attends it

  // K/V tiles travel global -> registers -> LDS; the loads run two tiles ahead of the tile being
  // multiplied, so their latency (the whole cost of a tile otherwise) hides behind two tiles' work
  constexpr int ITEMS = TK * CPR / 128;      // 16-byte pieces of K (and of V) per thread and tile
  static_assert(TK * CPR % 128 == 0, "tile pieces divide over the workgroup");
  // V pieces are dealt differently: a thread takes the same 8 d values of TWO neighbouring keys,
  // which sit side by side in a V^T row, so the transposed store is 8 dwords instead of 16
  // halves; and lanes run over 8 column pieces x 8 key pairs, which lands a wave's 64 dwords of
  // one store in (almost) distinct banks: d rows are 18 words apart, 8 rows (one piece) 144.
  // (With a key's 16 pieces on neighbouring lanes every store hit two banks 16 ways.)
  constexpr int VITEMS = TK / 2 * CPR / 128;                  // key pairs x pieces per thread
  static_assert(TK / 2 * CPR % 128 == 0 && CPR % 8 == 0, "V pieces divide over the workgroup");
  auto v_item = [&](int it, int& c, int& key) {     // piece and even key (inside the tile) of this thread's item
    const int x = (tid >> 6) + 2 * it;              // lanes: 8 pieces x 8 key pairs; wave and item: the high parts
    c = (tid & 7) + 8 * (x % (CPR / 8));
    key = 2 * (((tid >> 3) & 7) + 8 * (x / (CPR / 8)));
  };
  h8 kpre[2][ITEMS], vpre[2][2 * VITEMS];
  auto fetch = [&](int k0, h8 (&kk)[ITEMS], h8 (&vv)[2 * VITEMS]) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int idx = tid + it * 128;
      const int key = idx / CPR, c = idx - key * CPR;
      const int kr = min(k0 + key, p0 + n - 1);
      kk[it] = load_h8(kh + (size_t)kr * HD + c * 8);
    }
#pragma unroll
    for (int it = 0; it < VITEMS; ++it) {
      int c, key;
      v_item(it, c, key);
      vv[2 * it] = load_h8(vh + (size_t)min(k0 + key, p0 + n - 1) * HD + c * 8);
      vv[2 * it + 1] = load_h8(vh + (size_t)min(k0 + key + 1, p0 + n - 1) * HD + c * 8);
    }
  };
  auto stash = [&](const h8 (&kk)[ITEMS], const h8 (&vv)[2 * VITEMS]) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int idx = tid + it * 128;
      const int key = idx / CPR, c = idx - key * CPR;
      *reinterpret_cast<h8*>(Ks + key * K_STRIDE + c * 8) = kk[it];
    }
#pragma unroll
    for (int it = 0; it < VITEMS; ++it) {
      int c, key;
      v_item(it, c, key);
      // position of this key inside a V^T row: k-step s = key / 16, then half and slot as above
      const int r16 = key & 15;
      const int pos = ((key >> 4) * 2 + ((r16 & 7) >> 2)) * 8 + (r16 >> 3) * 4 + (r16 & 3);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const h2 pr = {vv[2 * it][e], vv[2 * it + 1][e]};
        *reinterpret_cast<h2*>(Vt + (c * 8 + e) * V_STRIDE + pos) = pr;
      }
    }
  };
  auto tile = [&](int k0) {
    if (k0 > p0 + wave_last_q) return;   // whole tile above this wave's diagonal

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
      sc[e] = (key <= p0 + qi) ? sc[e] * scale : -INFINITY;
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
        const half_t* vp = Vt + (t * 32 + ql) * V_STRIDE + (s2 * 2 + hf) * 8;     // 8-byte aligned: rows are 72 bytes
        const h4 a0 = *reinterpret_cast<const h4*>(vp), a1 = *reinterpret_cast<const h4*>(vp + 4);
        const h8 a = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb[s2], acc[t], 0, 0, 0);
      }
    }
  };

  // group g walks tiles g, g + G, ...; every group makes the same number of trips (barriers)
  constexpr int STEP = G * TK;
  const int kg = grp * TK;
  if (kg <= last_key) fetch(kg, kpre[0], vpre[0]);
  if (kg + STEP <= last_key) fetch(kg + STEP, kpre[1], vpre[1]);
  for (int kb = 0; kb <= last_key; kb += 2 * STEP) {
    const int k0 = kb + kg;
    __syncthreads();   // the previous tile has been consumed
    if (k0 <= last_key) stash(kpre[0], vpre[0]);
    __syncthreads();
    if (k0 + 2 * STEP <= last_key) fetch(k0 + 2 * STEP, kpre[0], vpre[0]);
    if (k0 <= last_key) tile(k0);
    if (kb + STEP > last_key) break;
    __syncthreads();
    if (k0 + STEP <= last_key) stash(kpre[1], vpre[1]);
    __syncthreads();
    if (k0 + 3 * STEP <= last_key) fetch(k0 + 3 * STEP, kpre[1], vpre[1]);
    if (k0 + STEP <= last_key) tile(k0 + STEP);
  }

  if constexpr (G > 1) {
    // merge: groups 1.. leave (m, l, O^T) in LDS, [group - 1][value][thread of the group]
    float* mg = reinterpret_cast<float*>(pf_attn_lds);
    constexpr int VALS = DT * 16 + 2;
    __syncthreads();   // all tiles consumed: the tile buffers are free
    if (grp > 0) {
      float* mine = mg + (size_t)(grp - 1) * VALS * 128 + tid;
      mine[0] = m;
      mine[128] = l;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) mine[(2 + t * 16 + e) * 128] = acc[t][e];
    }
    __syncthreads();
    if (grp > 0) return;
#pragma unroll
    for (int g = 1; g < G; ++g) {
      const float* other = mg + (size_t)(g - 1) * VALS * 128 + tid;
      const float mo = other[0], lo = other[128];
      const float mn = fmaxf(m, mo);                 // finite: group 0 always holds key 0
      const float ca = __expf(m - mn), cb = __expf(mo - mn);   // a group without an unmasked key has mo = -inf, cb = 0
      l = l * ca + lo * cb;
      m = mn;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = acc[t][e] * ca + other[(2 + t * 16 + e) * 128] * cb;
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

// Hm[r][i] = silu(G[r][i]) * U[r][i] with GU = slices of [Mb][2F] fp32 (gate | up), summed here.
// grid = (Mb, ceil(F/1024))
__global__ __launch_bounds__(LL_WG) void pf_swiglu_kernel(const float* __restrict__ GU, SliceMap map,
                                                          const DevState* __restrict__ st,
                                                          half_t* __restrict__ Hm, int F) {
  const int r = blockIdx.x;
  const int i = (blockIdx.y * LL_WG + threadIdx.x) * 4;
  if (i >= F) return;
  h4 o = {0, 0, 0, 0};
  if (r < st->n_prompt) {
    const float* row = GU + (size_t)r * 2 * F;
    const f4 g = pf_slice_sum(row + i, slice_count(map, i), map.slice_floats);
    const f4 u = pf_slice_sum(row + F + i, slice_count(map, F + i), map.slice_floats);
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (half_t)(g[j] / (1.0f + expf(-g[j])) * u[j]);
  }
  *reinterpret_cast<h4*>(Hm + (size_t)r * F + i) = o;
}
