// Batched lock-step decoding over a paged KV cache: the kernels that have no counterpart in the
// single-sequence path.  The paper embeds a paged-KV attention library for its cache (Sec. II-C,
// Sec. V-A) and keeps batch 1 (Sec. V-A); this is the batch > 1 regime it leaves open, where the
// projections of a step become 16- or 32-row matrix products (the short-prompt kernels of
// prefill_skinny.h, one row per sequence) instead of GEMVs.
//
// A sequence owns pages of `page_tokens` consecutive cache rows; page_table[slot][i] is the first
// cache row of its i-th page, so position p of slot b lives in cache row
// page_table[b][p / page_tokens] + p % page_tokens of the per-layer pools [head][pool rows][head_dim].
// Free slots point at page 0, which no sequence ever owns: whatever they compute lands there.
#pragma once
#include "ll_device.h"
#include "sample_kernels.h"

#define BT_MAX_BATCH 32

struct BatchState {
  int32_t pos[BT_MAX_BATCH];         // cached positions of slot b = position of the token it feeds next
  int32_t next_token[BT_MAX_BATCH];  // token slot b feeds next
  int32_t active[BT_MAX_BATCH];      // 0: free slot
  int32_t steps[BT_MAX_BATCH];       // tokens slot b's sequence has produced (the draw index of stochastic selection)
};

// Attention of slot b's new query (position pos[b], already written to the cache) for one head.
// grid = (heads, rows of the step = 16 or 32), 512 threads (two workgroups per CU; two trips of 128 keys
// in flight); tb = rows / 16 selects the output's fragment-major layout.  As in the single-sequence kernel a key row is read
// by HD / 8 adjacent lanes with one 16-byte load each and every lane group keeps an online-softmax
// state over the keys it is dealt; groups merge by shuffles, waves through LDS.  Output: fp16,
// in the fragment-major operand layout of the O projection.
#define BT_ATTN_THREADS 512
template <int HD>
__global__ __launch_bounds__(BT_ATTN_THREADS) void bt_attn_kernel(
    const half_t* __restrict__ Q, const half_t* __restrict__ kc, const half_t* __restrict__ vc,
    const BatchState* __restrict__ bs, const int* __restrict__ page_table, int pt_stride, int page_tokens,
    half_t* __restrict__ O, int d, int pool_rows, int tb) {
  constexpr int LPR = HD / 8;      // lanes per key row
  constexpr int GPW = 64 / LPR;    // lane groups per wave
  constexpr int NW = BT_ATTN_THREADS / 64;
  constexpr int UK = 4;            // keys in flight per group
  __shared__ float s_m[NW], s_l[NW], s_acc[NW][HD];
  extern __shared__ int s_pt[];    // this slot's page-table row: a key's address then costs no global round trip
  const int h = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int gi = lane / LPR, li = lane % LPR;
  // One round trip for everything the key loop needs: the slot's state, the query and the WHOLE page-table
  // row (entries past the sequence's end are not used; reading them saves waiting for the position first).
  const int active = bs->active[b];
  const int n_keys = bs->pos[b] + 1;
  const h8 q = load_h8(Q + (size_t)b * d + h * HD + li * 8);
  for (int i = tid; i < pt_stride; i += BT_ATTN_THREADS) s_pt[i] = page_table[b * pt_stride + i];
  if (!active) {
    if (tid < HD / 8) *reinterpret_cast<h8*>(O + act_offset(b, h * HD + tid * 8, d, tb)) = h8{0, 0, 0, 0, 0, 0, 0, 0};
    return;
  }
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)HD);
  float qv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) qv[e] = (float)q[e] * scale;
  const half_t* kh = kc + (size_t)h * pool_rows * HD + li * 8;
  const half_t* vh = vc + (size_t)h * pool_rows * HD + li * 8;

  float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  constexpr int STRIDE = NW * GPW, TRIP = STRIDE * UK;     // keys one trip of the workgroup covers
  // Trips are double-buffered: the requests of trip t + 1 go out before trip t is used, so a long sequence
  // costs one memory round trip plus the arithmetic of its trips, not a round trip per trip.  A trip past
  // the sequence's end is still requested (every key clamped to the last one: cache hits), which keeps
  // the number of loads in flight the same on every path and the waits exact.
  auto issue = [&](int base, h8 (&kk)[UK], h8 (&vv)[UK]) {
#pragma unroll
    for (int j = 0; j < UK; ++j) {
      const int u = min(base + j * STRIDE + gi, n_keys - 1);
      const int pg = u / page_tokens;
      const size_t row = (size_t)(s_pt[pg] + (u - pg * page_tokens));
      kk[j] = load_stream(kh + row * HD);
      vv[j] = load_stream(vh + row * HD);
    }
  };
  // One online-softmax step per trip, not per key: the trip's scores first, then one new maximum, one
  // correction of the running state and one exponential per key (branch-free: inside a branch the
  // compiler sinks a value row's load to its use and waits for it there).
  auto consume = [&](int base, const h8 (&kk)[UK], const h8 (&vv)[UK]) {
    float dot[UK], mn = m;
#pragma unroll
    for (int j = 0; j < UK; ++j) {
      float t = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) t += qv[e] * (float)kk[j][e];
      t = group_sum<LPR>(t);
      dot[j] = (base + j * STRIDE + gi < n_keys) ? t : -INFINITY;
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
  h8 ka[UK], va[UK], kb[UK], vb[UK];
  issue(wave * GPW, ka, va);
  for (int base = wave * GPW; base < n_keys; base += 2 * TRIP) {
    issue(base + TRIP, kb, vb);
    __builtin_amdgcn_sched_barrier(0);
    consume(base, ka, va);
    __builtin_amdgcn_sched_barrier(0);
    issue(base + 2 * TRIP, ka, va);
    __builtin_amdgcn_sched_barrier(0);
    consume(base + TRIP, kb, vb);
    __builtin_amdgcn_sched_barrier(0);
  }
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
  if (tid < HD / 8) {
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < NW; ++i) M = fmaxf(M, s_m[i]);
    float L = 0.f, A[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      const float w = (s_m[i] > -INFINITY) ? __expf(s_m[i] - M) : 0.f;    // M is finite: key 0 is always attended
      L += s_l[i] * w;
#pragma unroll
      for (int e = 0; e < 8; ++e) A[e] += s_acc[i][tid * 8 + e] * w;
    }
    const float rl = 1.0f / L;
    h8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (half_t)(A[e] * rl);
    *reinterpret_cast<h8*>(O + act_offset(b, h * HD + tid * 8, d, tb)) = o;
  }
}

// Token of every slot and the slots' state advance: greedy (lowest index among equal maxima), or
// the stochastic selection of sample_kernels.h with the slot's own draw index, so a sequence draws
// the same stream in a batch as alone.  grid = rows of the step, SMP_THREADS threads, SMP_Z_WORDS
// words of dynamic LDS; out = device-visible host memory, -1 for free slots.
__global__ __launch_bounds__(SMP_THREADS) void bt_select_kernel(const float* __restrict__ logits, int vocab,
                                                                const SampleCfg* __restrict__ cfg,
                                                                BatchState* bs, int* out) {
  extern __shared__ float bt_z[];
  __shared__ float sv[SMP_THREADS];
  __shared__ int si[SMP_THREADS];
  __shared__ uint32_t sk[SMP_THREADS];
  __shared__ float red[2 * 3 * (SMP_THREADS / 64)];
  __shared__ int found;
  const int b = blockIdx.x, tid = threadIdx.x;
  if (!bs->active[b]) {
    if (tid == 0) out[b] = -1;
    return;
  }
  const float* row = logits + (size_t)b * vocab;
  int tok;
  if (cfg->inv_temp == 0.f || vocab > SMP_MAX_VOCAB) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = tid * 4; i < vocab; i += SMP_THREADS * 4) {     // vocab % 16 == 0 (checked when the batch is opened)
      const f4 v = *reinterpret_cast<const f4*>(row + i);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (v[e] > bv) { bv = v[e]; bi = i + e; }                // indices ascend: the first maximum stays
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
    if (tok == 0x7fffffff) tok = 0;          // every logit NaN: still a valid id
  } else {
    tok = smp_draw_token(row, vocab, cfg, (uint32_t)bs->steps[b], bt_z, si, sk, red, &found);
  }
  if (tid == 0) {
    bs->next_token[b] = tok;
    bs->pos[b] = bs->pos[b] + 1;
    bs->steps[b] = bs->steps[b] + 1;
    out[b] = tok;
  }
}

// After a prompt has been prefilled into the contiguous single-sequence cache: copy its rows
// 0 .. n - 1 into the pages of slot b.  grid = (n, layers * 2); a workgroup moves one cache row of
// every head of one layer's K or V.
__global__ __launch_bounds__(LL_WG) void bt_scatter_kernel(const half_t* __restrict__ src_kv, size_t src_layer_halves,
                                                           int src_rows, half_t* __restrict__ dst_kv,
                                                           size_t dst_layer_halves, int dst_rows,
                                                           const int* __restrict__ page_table, int pt_stride,
                                                           int page_tokens, int slot, int n_heads, int head_dim) {
  const int r = blockIdx.x, lk = blockIdx.y;      // lk = layer * 2 + (0: K, 1: V)
  const int pg = r / page_tokens;
  const size_t drow = (size_t)(page_table[slot * pt_stride + pg] + (r - pg * page_tokens));
  const half_t* s = src_kv + (size_t)lk * src_layer_halves;
  half_t* d = dst_kv + (size_t)lk * dst_layer_halves;
  const int per_head = head_dim / 8;
  for (int i = threadIdx.x; i < n_heads * per_head; i += LL_WG) {
    const int h = i / per_head, c = i - h * per_head;
    *reinterpret_cast<h8*>(d + ((size_t)h * dst_rows + drow) * head_dim + c * 8) =
        load_h8(s + ((size_t)h * src_rows + r) * head_dim + c * 8);
  }
}

// Page-table entries that changed since the last step, passed by value: one small launch in
// front of the step instead of a host-to-device copy of the table.
struct PageUpdates {
  int n;
  int index[BT_MAX_BATCH];      // slot * pt_stride + page number
  int row[BT_MAX_BATCH];        // first cache row of the page
};
__global__ __launch_bounds__(64) void bt_page_update_kernel(int* __restrict__ page_table, PageUpdates u) {
  const int i = threadIdx.x;
  if (i < u.n) page_table[u.index[i]] = u.row[i];
}
