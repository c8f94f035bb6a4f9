// C ABI of the decode / prefill path (see include/ll.h): workspace carving,
// kernel chains, hipGraph capture and replay, device-resident step state.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <chrono>
#include <future>
#include <string>
#include <vector>

#include "../../include/ll.h"
#include "decode_kernels.h"
#include "sample_kernels.h"
#include "decode_mega.h"
#include "prefill_kernels.h"
#include "prefill_skinny.h"
#include "prefill_gemm.h"
#include "batch_kernels.h"

// Scratch of ll_prefill_static(): the buffers a short prefill needs besides its inputs and outputs
// (activations, per-token partial sums, logits, selection candidates, the staged prompt ids), for
// callers that cannot bring device memory of their own for them.  One copy per GPU the library runs
// on, held until the process ends.  In host code this name is a stand-in, not a device address: the
// address on the current device comes from hipGetSymbolAddress (static_scratch_ptr below).
#define LL_STATIC_SCRATCH_BYTES (4u << 20)
static __device__ __align__(256) unsigned char scratch[LL_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIPCHK(expr)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return fail(LL_E_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                  __LINE__);                                                              \
  } while (0)

constexpr int kGemvU = 8;          // 512-element chunks of a weight row in flight per lane and row
constexpr int kGemvWgsPerCu = 4;   // measured best of 2/3/4 on the 7B shapes
constexpr int kAttnMaxSplits = 16;
constexpr int kMaxPromptBucket = 1024;   // rows of the largest prefill graph; longer prompts go through in chunks of it
constexpr int kGemmMinSlabs = 8;
constexpr size_t kAlign = 256;
constexpr size_t kAttnOLdsBytes = 9 * 512 * sizeof(float);   // staged o of the fused attention + O kernel (8 chunks + a zero chunk)

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Compute units of the current device, the unit every launch shape is sized in (workgroups per CU for
// the GEMVs, one round of workgroups for the prefill GEMM's plan, one workgroup per CU for the
// persistent projections).  Queried once; 256, the MI355X's count, where no device can be asked (the
// host-only plan hooks on a machine without a GPU).
int g_num_cus = 0;
int num_cus() {
  if (g_num_cus > 0) return g_num_cus;
  int dev = 0, cus = 0, ndev = 0;
  if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0 && hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
    g_num_cus = cus;
  else
    g_num_cus = 256;
  return g_num_cus;
}

bool config_ok(const ll_config* c, const char** why) {
  const char* w = nullptr;
  if (!c) w = "null config";
  else if (c->n_layers < 1 || c->vocab < 1) w = "n_layers and vocab must be >= 1";
  else if (c->head_dim != 64 && c->head_dim != 128) w = "head_dim must be 64 or 128";
  else if (c->n_heads < 1 || (int64_t)c->n_heads * c->head_dim != c->d_model) w = "n_heads * head_dim != d_model";
  else if (c->d_model % 8 || c->ffn_hidden % 8 || c->ffn_hidden < 8) w = "d_model and ffn_hidden must be multiples of 8";
  else if (c->max_seq < 2 || c->max_seq > (1 << 20)) w = "max_seq out of range";
  else if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) w = "bad rope_theta / rms_eps";
  if (why) *why = w;
  return w == nullptr;
}

int prompt_bucket(int n) {   // smallest of {64,128,256,512,1024} holding n rows
  int b = 64;
  while (b < n) b <<= 1;
  return b;
}

// Shapes the short-prompt kernels accept: 16-row blocks that keep RoPE pairs / gate-up pairs together
bool skinny_ok(const ll_config& c) {
  return c.d_model % 16 == 0 && c.head_dim % 16 == 0 && c.ffn_hidden % 8 == 0;
}

// Row tile of the projection GEMM and how its K loops are dealt out: the 64-wide slabs of all
// 256-column tiles form one sequence, cut into runs of `quota` slabs; with `mtiles` row tiles
// the grid has runs x mtiles workgroups.  Whatever splits a tile stays within one workgroup per CU
// (a second, partial round would cost as much as a full one) and keeps runs of at least
// kGemmMinSlabs slabs; whole tiles may take several rounds when they fill them well.
// O and down (one matrix of d_model columns, i.e. few column tiles) take two 64-row tiles at 65..128 rows:
// twice the workgroups per column tile, so half as many K pieces per tile for the consumer to add up, and
// the second row tile finds the weights in L2 (measured at 100 tokens: 4.89 -> 4.81 ms to first token).
int gemm_bm(int Mb, int nmat = 0) { return (Mb > 128 || (Mb == 128 && nmat != 1)) ? 128 : 64; }

struct GemmPlan {
  int mtiles, runs;
  int max_slices;          // most pieces any tile is cut into
  SliceMap map;
};

GemmPlan gemm_plan(int N, int K, int nmat, int Mb, int ldc) {
  GemmPlan p{};
  const int kGemmWantWgs = num_cus();               // one round of workgroups
  p.mtiles = Mb / gemm_bm(Mb, nmat);
  p.map.nslabs = (K + 63) / 64;
  p.map.ntiles = (N + 255) / 256;
  p.map.N = N;
  p.map.slice_floats = (size_t)Mb * ldc;
  const int tiles = p.map.ntiles * nmat, S = p.map.nslabs;
  // split-K: ks whole fractions of every tile, at most one round of workgroups over the CUs
  int ks = kGemmWantWgs / (tiles * p.mtiles);
  if (ks > S / kGemmMinSlabs) ks = S / kGemmMinSlabs;
  if (ks < 1) ks = 1;
  while (ks > 1 && (S + ks - 1) / ks * (ks - 1) >= S) --ks;      // no empty piece
  const int wgs = tiles * p.mtiles * ks, rounds = (wgs + kGemmWantWgs - 1) / kGemmWantWgs;
  if (ks == 1 && wgs * 5 < rounds * kGemmWantWgs * 4) {
    // whole tiles would leave a fifth of a round idle: equal runs across tile borders instead
    const int units = tiles * S;
    int runs = kGemmWantWgs / p.mtiles;
    if (runs > units / kGemmMinSlabs) runs = units / kGemmMinSlabs;
    if (runs < 1) runs = 1;
    p.map.quota = (units + runs - 1) / runs;
    p.runs = (units + p.map.quota - 1) / p.map.quota;
    p.max_slices = (S - 1) / p.map.quota + 2;
  } else {
    p.map.quota = (S + ks - 1) / ks;
    p.map.nslabs = p.map.quota * ks;          // padded: tile t owns units t * nslabs .., the last piece is short
    p.runs = tiles * ks;
    p.max_slices = ks;
  }
  return p;
}

struct Layout {
  size_t kv, rope, x, x_keep, q, o, m, attn_part, attn_cnt, logits, amax_val, amax_idx, state, tokens;
  size_t pf_x, pf_xn, pf_part, pf_q, pf_o, pf_h, pf_ss;
  size_t mk_layers, mk_bar, mk_amax_val, mk_amax_idx, mk_trace, zeros, sample_cfg, ao_sync;
  size_t wf;                // fragment-major copy of the projection weights for the short-prompt kernels (0 bytes without it)
  size_t wf_qkv, wf_o, wf_gu, wf_down, wf_layer, wf_lm;   // offsets inside a layer's part, bytes per layer, offset of the LM head's copy
  size_t total;
  int attn_splits, attn_threads, lm_wgs, max_prompt, mb_max;
  size_t kv_layer_halves;   // halves per layer per K or V
};

int gemv_grid(int pairs, int wg_threads = LL_WG) {
  // a few workgroups per CU keep enough 16-byte loads in flight; never more waves than row pairs
  const int wpw = wg_threads / 64;
  const int want = num_cus() * kGemvWgsPerCu * LL_WG / wg_threads;
  const int need = (pairs + wpw - 1) / wpw;
  if (need < want) return need < 1 ? 1 : need;
  // a grid within a quarter of that which gives every wave the same number of row pairs is worth more than
  // the last quarter of the workgroups (Q/K/V at d_model 4096: 768 workgroups of 2 pairs per wave 17.1 us,
  // 1024 of 1.5 pairs 17.7 us, 512 of 3 pairs 18.3 us)
  for (int g = want; g >= want - want / 4; --g)
    if (pairs % (g * wpw) == 0) return g;
  return want;
}

Layout make_layout(const ll_config& c) {
  Layout L{};
  const size_t d = c.d_model, F = c.ffn_hidden, V = c.vocab;
  // Workgroups per head of the decode attention: four, of 512 threads up to 2 K positions and of 1024
  // threads in long-context instances (two of 1024 when attention and O projection run as one launch,
  // which takes at most two).  Their partials are merged by the O projection's prologue underneath its
  // weight stream.  Measured at the 7B shape: 4 x 512 against 2 x 1024 threads 6.2 against 7.5 us per layer
  // at 500..800 keys; against a merge kernel of its own in a max_seq 4096 instance 2.57 / 2.62 / 2.81 ms
  // against 2.64 / 2.70 / 2.90 ms per step at 1000 / 2000 / 4000 keys.
  const bool fused = (c.flags & LL_FLAG_FUSED_ATTN_OPROJ) != 0;
  L.attn_splits = c.n_heads * 2 > 512 ? 1 : (c.max_seq <= 2048 && fused) ? 2 : 4;
  L.attn_threads = (c.max_seq <= 2048 && L.attn_splits == 4) ? 512 : ATTN_THREADS;
  L.lm_wgs = gemv_grid((c.vocab + 1) / 2);
  L.max_prompt = c.max_seq - 1;                   // longer than the largest bucket: fed in chunks
  L.mb_max = prompt_bucket(L.max_prompt < kMaxPromptBucket ? L.max_prompt : kMaxPromptBucket);
  L.kv_layer_halves = (size_t)c.n_heads * c.max_seq * c.head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.kv = take((size_t)c.n_layers * 2 * L.kv_layer_halves * 2);
  L.rope = take((size_t)c.max_seq * (c.head_dim / 2) * sizeof(float2));
  L.x = take(d * 4);
  L.x_keep = take(d * 4);
  L.q = take(d * 4);
  L.o = take(d * 4);
  L.m = take(F * 4);
  L.attn_part = take((size_t)c.n_heads * kAttnMaxSplits * (c.head_dim + 4) * 4);
  L.attn_cnt = take((size_t)c.n_heads * 4);
  L.logits = take(V * 4);
  L.amax_val = take((size_t)L.lm_wgs * 4);
  L.amax_idx = take((size_t)L.lm_wgs * 4);
  L.state = take(sizeof(DevState));
  L.tokens = take((size_t)L.mb_max * 4);
  const size_t M = L.mb_max;
  L.pf_x = take(M * d * 4);
  L.pf_xn = take(M * ((d + 31) / 32 * 32) * 2);          // K rounded up: fragment-major layout
  L.pf_q = take(M * d * 2);
  L.pf_o = take(M * ((d + 31) / 32 * 32) * 2);
  size_t part = 0;                                       // slices of the widest GEMM output of any bucket
  for (int mb = 64; mb <= L.mb_max; mb <<= 1) {
    const GemmPlan plans[4] = {gemm_plan(d, d, 3, mb, 3 * d), gemm_plan(d, d, 1, mb, d),
                               gemm_plan(F, d, 2, mb, 2 * F), gemm_plan(d, F, 1, mb, d)};
    for (const GemmPlan& p : plans) part = std::max(part, p.max_slices * p.map.slice_floats);
  }
  L.pf_part = take(part * 4);
  L.pf_h = take(M * ((F + 31) / 32 * 32) * 2);
  L.pf_ss = take((size_t)2 * 32 * sk_ss_stride(c.d_model) * 4);
  L.zeros = take(256);
  L.sample_cfg = take(sizeof(SampleCfg));
  L.ao_sync = take(64 * 4);                 // arrival counters of the fused attention + O kernel, a line apart
  L.mk_layers = take((size_t)c.n_layers * sizeof(MkLayer));
  L.mk_bar = take((size_t)MK_BAR_WORDS * 4);
  L.mk_amax_val = take(1024 * 4);   // one candidate per workgroup of the persistent kernel
  L.mk_amax_idx = take(1024 * 4);
  L.mk_trace = take((size_t)(5 * c.n_layers + 2) * 8 * 8);
  // Second copy of the weights in the short-prompt kernels' operand order (see sk_shuffle_kernel):
  // [layer][q,k,v | o | gate,up | down] then the LM head, 1 KB per 16-row block and 32-wide K step.
  if (skinny_ok(c) && !(c.flags & LL_FLAG_LEAN_WORKSPACE)) {
    const size_t kd = (d + 31) / 32, kf = (F + 31) / 32;
    L.wf_qkv = 0;
    L.wf_o = L.wf_qkv + align_up((size_t)skinny_units(SK_QKV, c.d_model) * kd * 1024);
    L.wf_gu = L.wf_o + align_up((size_t)skinny_units(SK_RES, c.d_model) * kd * 1024);
    L.wf_down = L.wf_gu + align_up((size_t)skinny_units(SK_GATEUP, c.ffn_hidden) * kd * 1024);
    L.wf_layer = L.wf_down + align_up((size_t)skinny_units(SK_RES, c.d_model) * kf * 1024);
    L.wf_lm = L.wf_layer * c.n_layers;
    L.wf = take(L.wf_lm + (c.vocab % 16 == 0 ? (size_t)skinny_units(SK_LOGITS, c.vocab) * kd * 1024 : 0));
  } else {
    L.wf_layer = 0;
    L.wf = off;
  }
  L.total = off;
  return L;
}

// Buffers of a prefill call (and of the head of a decode step) that hold nothing the caller needs once
// the call has returned: activations, partial sums, logits, selection candidates.  The KV rows, the
// state block and the token ring are the call's outputs and live elsewhere.
struct PfBuffers {
  float* X;          // residual stream [rows][d] fp32
  half_t* Xn;        // normalised operand of the next projection (fragment-major for <= 32 rows)
  half_t* Q;         // rotated queries [rows][d]
  half_t* O;         // attention output
  half_t* H;         // SwiGLU output [rows][F]
  float* part;       // slices of the prefill GEMM (prompts of more than 32 tokens)
  float* ss;         // two sets of per-token partial sums of squares
  int* tokens;       // prompt ids of the chunk in flight
  float* logits;     // [vocab]
  float* amax_val;   // per-workgroup argmax candidates of the LM head
  int* amax_idx;
  half_t* zeros;     // 256 bytes of zeros
};

// Device address of `scratch` on each GPU, looked up once per device with that device current
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_ptr(int dev, void** out) {
  if (dev < 0 || dev >= kMaxDevices) return fail(LL_E_HIP, "device ordinal %d out of range", dev);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || reinterpret_cast<uintptr_t>(p) % kAlign)
      return fail(LL_E_HIP, "hipGetSymbolAddress(scratch) returned %p", p);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LL_OK;
}

// The buffers of a prefill of at most 32 rows, laid out from `base`; returns the bytes they take
size_t carve_short_prefill(const ll_config& c, int lm_wgs, char* base, PfBuffers* out) {
  const size_t d = c.d_model, F = c.ffn_hidden, M = 32;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return base + o; };
  PfBuffers B{};
  B.X = reinterpret_cast<float*>(take(M * d * 4));
  B.Xn = reinterpret_cast<half_t*>(take(M * ((d + 31) / 32 * 32) * 2));
  B.Q = reinterpret_cast<half_t*>(take(M * d * 2));
  B.O = reinterpret_cast<half_t*>(take(M * ((d + 31) / 32 * 32) * 2));
  B.H = reinterpret_cast<half_t*>(take(M * ((F + 31) / 32 * 32) * 2));
  B.part = nullptr;                               // no GEMM slices: the short-prompt kernels sum inside a workgroup
  B.ss = reinterpret_cast<float*>(take((size_t)2 * 32 * sk_ss_stride(c.d_model) * 4));
  B.tokens = reinterpret_cast<int*>(take(M * 4));
  B.logits = reinterpret_cast<float*>(take((size_t)c.vocab * 4));
  B.amax_val = reinterpret_cast<float*>(take((size_t)lm_wgs * 4));
  B.amax_idx = reinterpret_cast<int*>(take((size_t)lm_wgs * 4));
  B.zeros = reinterpret_cast<half_t*>(take(256));
  if (out) *out = B;
  return off;
}

struct Batch;
void destroy_batch(Batch* B);

struct Instance {
  ll_config cfg;
  Batch* batch = nullptr;       // batched decoding over a paged cache, opened on top of the instance
  Layout L;
  std::vector<ll_layer_weights> layers;
  ll_weights w;
  char* ws = nullptr;
  PfBuffers pf{};               // the workspace's set of these buffers
  int device = 0;               // GPU the instance lives on
  char* static_scratch = nullptr;   // that GPU's copy of the library's static scratch array
  const float* last_logits = nullptr;   // where the most recent step left its logits / residual rows
  const float* last_rows = nullptr;
  hipStream_t stream = nullptr;
  bool own_stream = false;
  hipGraph_t dec_graph = nullptr;
  hipGraphExec_t dec_exec = nullptr;
  bool skinny = false;          // prompts of <= 32 tokens take the short-prompt kernels
  std::vector<int> pf_buckets;
  std::vector<hipGraph_t> pf_graph;
  std::vector<hipGraphExec_t> pf_exec;
  hipGraph_t pf_body_graph = nullptr;       // largest bucket without LM head and sampling: all but the last chunk
  hipGraphExec_t pf_body_exec = nullptr;    // of a prompt longer than that bucket
  int last_chunk_rows = 0;                  // rows of the most recent prefill's last chunk
  int* host_ring = nullptr;      // pinned, device-visible; kernels write generated ids here
  int* dev_ring = nullptr;       // device address of host_ring
  int ring_size = 0;
  int* host_stage = nullptr;     // pinned staging for the prompt ids + DevState
  // host mirror of the device state (never read back from the GPU on the hot path)
  int pos = 0, steps = 0;
  bool last_was_prefill = false;
  // profiling hook: when set, every decode launch is bracketed by events
  std::vector<hipEvent_t>* prof_events = nullptr;
  std::vector<int>* prof_class = nullptr;
  bool use_mega = false;         // decode step = one persistent kernel
  bool fused_attn = false;       // attention and O projection of a layer in one launch
  int mega_grid = 0;
  size_t mega_lds = 0;
  int mega_splits = 1;
  // the paper's mechanism as an option: one decode graph per KV length in a rolling buffer
  struct LenGraph { int len = -1; hipGraph_t graph = nullptr; hipGraphExec_t exec = nullptr; uint64_t used = 0; };
  bool per_length = false;
  std::vector<LenGraph> lg;      // at most kLenGraphBuffer entries
  uint64_t lg_clock = 0;
  hipStream_t cap_stream = nullptr;
  std::future<int> lg_future;    // capture of the next length, running on a second thread
  LenGraph lg_pending;
  std::string lg_pending_err;
  int64_t lg_stats[4] = {0, 0, 0, 0};   // replays of a buffered graph, blocking captures, overlapped captures, capture ns
  int only_class = -1;           // timing hook: launch only this kernel class of the decode chain
  bool runs(int klass) const { return only_class < 0 || only_class == klass; }

  template <class T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
  half_t* kcache(int layer) const { return at<half_t>(L.kv) + (size_t)layer * 2 * L.kv_layer_halves; }
  half_t* vcache(int layer) const { return kcache(layer) + L.kv_layer_halves; }
  DevState* state() const { return at<DevState>(L.state); }
  // fragment-major copy of one matrix group of a layer (null without the copy)
  const half_t* wfrag(int layer, size_t group_off) const {
    return L.wf_layer ? at<half_t>(L.wf + (size_t)layer * L.wf_layer + group_off) : nullptr;
  }
  const half_t* wfrag_lm() const { return L.wf_layer && cfg.vocab % 16 == 0 ? at<half_t>(L.wf + L.wf_lm) : nullptr; }
};

Instance* g = nullptr;

size_t gemv_lds_bytes(int K, bool norm) {
  const int nch = (K + 511) / 512;
  const int nchp = (nch + kGemvU - 1) / kGemvU * kGemvU;
  // input vector, reduction scratch, and for the normalising projections the staged gains
  return ((size_t)nchp * 512 + 16) * sizeof(float) + (norm ? (size_t)nch * 512 * sizeof(half_t) : 0);
}

struct ProfScope {
  Instance* I;
  hipStream_t s;
  ProfScope(Instance* inst, hipStream_t st, int klass) : I(inst), s(st) {
    if (I->prof_events) {
      hipEvent_t e;
      (void)hipEventCreate(&e);
      (void)hipEventRecord(e, s);
      I->prof_events->push_back(e);
      I->prof_class->push_back(klass);
    }
  }
  ~ProfScope() {
    if (I->prof_events) {
      hipEvent_t e;
      (void)hipEventCreate(&e);
      (void)hipEventRecord(e, s);
      I->prof_events->push_back(e);
    }
  }
};

template <int MODE>
void launch_gemv(const GemvArgs& a, int pairs, int grid_override, hipStream_t s) {
  const int grid = grid_override > 0 ? grid_override : gemv_grid(pairs, GEMV_WG(MODE));
  hipLaunchKernelGGL((gemv_kernel<MODE, kGemvU>), dim3(grid), dim3(GEMV_WG(MODE)),
                     gemv_lds_bytes(a.K, MODE == GM_QKV || MODE == GM_GATEUP || MODE == GM_LMHEAD), s, a);
}

// final RMSNorm + LM head + argmax + state advance, shared by decode and prefill
void enqueue_head(Instance* I, hipStream_t s, const PfBuffers& B, const float* xin, int from_prompt_row, int prefill) {
  const ll_config& c = I->cfg;
  if (I->runs(LL_KC_LMHEAD)) {
    ProfScope ps(I, s, LL_KC_LMHEAD);
    GemvArgs a{};
    a.w0 = (const half_t*)I->w.lm_head;
    a.xin = xin;
    a.gain = (const half_t*)I->w.final_norm;
    a.out = B.logits;
    a.N = c.vocab;
    a.K = c.d_model;
    a.eps = c.rms_eps;
    a.st = I->state();
    a.amax_val = B.amax_val;
    a.amax_idx = B.amax_idx;
    a.x_row_from_prompt = from_prompt_row;
    launch_gemv<GM_LMHEAD>(a, (c.vocab + 1) / 2, I->L.lm_wgs, s);
  }
  if (I->runs(LL_KC_SAMPLE)) {
    ProfScope ps(I, s, LL_KC_SAMPLE);
    hipLaunchKernelGGL(sample_kernel, dim3(1), dim3(SMP_THREADS), SMP_Z_WORDS * 4, s, B.amax_val,
                       B.amax_idx, I->L.lm_wgs, B.logits, c.vocab,
                       I->at<SampleCfg>(I->L.sample_cfg), I->state(), I->dev_ring, I->ring_size, prefill,
                       (const half_t*)I->w.tok_emb, I->use_mega ? nullptr : I->at<float>(I->L.x),
                       I->at<float>(I->L.x_keep), c.d_model);
  }
}

void enqueue_decode_multi(Instance* I, hipStream_t s) {
  const ll_config& c = I->cfg;
  const int d = c.d_model, F = c.ffn_hidden;
  float* x = I->at<float>(I->L.x);
  float* q = I->at<float>(I->L.q);
  float* o = I->at<float>(I->L.o);
  float* m = I->at<float>(I->L.m);
  // x already holds the embedding row of the token to feed: the selection kernel of the previous
  // step (or of the prefill) gathered it, and ll_dbg_force_next_token refreshes it
  if (I->use_mega && I->runs(LL_KC_EMBED)) {      // (the timing hooks of a persistent-kernel instance: its selection gathers nothing)
    ProfScope ps(I, s, LL_KC_EMBED);
    hipLaunchKernelGGL(embed_kernel, dim3((d + LL_WG * 8 - 1) / (LL_WG * 8)), dim3(LL_WG), 0, s,
                       (const half_t*)I->w.tok_emb, I->state(), x, d);
  }
  for (int l = 0; l < c.n_layers; ++l) {
    const ll_layer_weights& W = I->layers[l];
    if (I->runs(LL_KC_QKV)) {
      ProfScope ps(I, s, LL_KC_QKV);
      GemvArgs a{};
      a.w0 = (const half_t*)W.wq; a.w1 = (const half_t*)W.wk; a.w2 = (const half_t*)W.wv;
      a.xin = x; a.gain = (const half_t*)W.attn_norm; a.out = q;
      a.N = d; a.K = d; a.eps = c.rms_eps;
      a.kcache = I->kcache(l); a.vcache = I->vcache(l);
      a.rope = I->at<float2>(I->L.rope); a.st = I->state();
      a.head_dim = c.head_dim; a.max_seq = c.max_seq;
      launch_gemv<GM_QKV>(a, 3 * d / 2, 0, s);
    }
    if (I->fused_attn) {
      // attention + O projection in one launch (counted under the attention class by the timing hooks)
      if (I->runs(LL_KC_ATTN)) {
        ProfScope ps(I, s, LL_KC_ATTN);
        AttnOArgs a{};
        a.q = q; a.kc = I->kcache(l); a.vc = I->vcache(l); a.st = I->state();
        a.part = I->at<float>(I->L.attn_part); a.wo = (const half_t*)W.wo; a.x = x;
        a.sync = I->at<unsigned>(I->L.ao_sync); a.fault = &I->state()->fault;
        a.d = d; a.n_heads = c.n_heads; a.splits = I->L.attn_splits; a.max_seq = c.max_seq;
        a.spin_limit = 1 << 20;      // about a second, then the step reports an error instead of hanging
        const int grid = c.n_heads * I->L.attn_splits + (d / 2 + ATTN_THREADS / 64 - 1) / (ATTN_THREADS / 64);
        if (c.head_dim == 128)
          hipLaunchKernelGGL(attn_oproj_kernel<128>, dim3(grid), dim3(ATTN_THREADS), kAttnOLdsBytes, s, a);
        else
          hipLaunchKernelGGL(attn_oproj_kernel<64>, dim3(grid), dim3(ATTN_THREADS), kAttnOLdsBytes, s, a);
      }
    } else {
    if (I->runs(LL_KC_ATTN)) {
      ProfScope ps(I, s, LL_KC_ATTN);
      dim3 grid(c.n_heads, I->L.attn_splits);
      if (c.head_dim == 128 && I->L.attn_threads == 512)
        hipLaunchKernelGGL((attn_decode_kernel<128, 512>), grid, dim3(512), 0, s, q, I->kcache(l),
                           I->vcache(l), I->state(), I->at<float>(I->L.attn_part), c.max_seq);
      else if (c.head_dim == 128)
        hipLaunchKernelGGL(attn_decode_kernel<128>, grid, dim3(ATTN_THREADS), 0, s, q, I->kcache(l),
                           I->vcache(l), I->state(), I->at<float>(I->L.attn_part), c.max_seq);
      else if (I->L.attn_threads == 512)
        hipLaunchKernelGGL((attn_decode_kernel<64, 512>), grid, dim3(512), 0, s, q, I->kcache(l),
                           I->vcache(l), I->state(), I->at<float>(I->L.attn_part), c.max_seq);
      else
        hipLaunchKernelGGL(attn_decode_kernel<64>, grid, dim3(ATTN_THREADS), 0, s, q, I->kcache(l),
                           I->vcache(l), I->state(), I->at<float>(I->L.attn_part), c.max_seq);
    }
    if (I->runs(LL_KC_OPROJ)) {
      ProfScope ps(I, s, LL_KC_OPROJ);
      GemvArgs a{};
      a.w0 = (const half_t*)W.wo; a.xin = o; a.out = x; a.N = d; a.K = d;
      a.attn_part = I->at<float>(I->L.attn_part);
      a.attn_splits = I->L.attn_splits; a.head_dim = c.head_dim;
      launch_gemv<GM_ORES>(a, d / 2, 0, s);
    }
    }
    if (I->runs(LL_KC_GATEUP)) {
      ProfScope ps(I, s, LL_KC_GATEUP);
      GemvArgs a{};
      a.w0 = (const half_t*)W.w_gate; a.w1 = (const half_t*)W.w_up;
      a.xin = x; a.gain = (const half_t*)W.ffn_norm; a.out = m;
      a.N = F; a.K = d; a.eps = c.rms_eps;
      launch_gemv<GM_GATEUP>(a, F, 0, s);
    }
    if (I->runs(LL_KC_DOWN)) {
      ProfScope ps(I, s, LL_KC_DOWN);
      GemvArgs a{};
      a.w0 = (const half_t*)W.w_down; a.xin = m; a.out = x; a.N = d; a.K = F;
      const int nch = (F + 511) / 512, nseg = (nch + 7) / 8;
      const size_t lds = ((size_t)(nch + 1) * 512 + 4 * 4 * 2) * sizeof(float);
      const int grid = (d / 2 + 3) / 4;
      if (nseg == 2) hipLaunchKernelGGL(gemv_ksplit_kernel<2>, dim3(grid), dim3(512), lds, s, a);
      else if (nseg == 3) hipLaunchKernelGGL(gemv_ksplit_kernel<3>, dim3(grid), dim3(768), lds, s, a);
      else if (nseg == 4) hipLaunchKernelGGL(gemv_ksplit_kernel<4>, dim3(grid), dim3(1024), lds, s, a);
      else launch_gemv<GM_DOWN>(a, d / 2, 0, s);   // short rows, or too long to split over one workgroup
    }
  }
  enqueue_head(I, s, I->pf, x, 0, 0);
}

// Can the whole step run as one persistent kernel on this device / shape?
bool mega_plan(Instance* I, std::string* why) {
  const ll_config& c = I->cfg;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
    *why = "cannot query the CU count";
    return false;
  }
  if (cus > 1024) cus = 1024;
  const int nch_d = (c.d_model + 511) / 512, nch_f = (c.ffn_hidden + 511) / 512;
  if (nch_d > MK_U) { *why = "d_model > 4096"; return false; }
  if (c.n_heads > cus) { *why = "more heads than CUs"; return false; }
  auto items = [&](int npairs, int nch) { return ((npairs + cus - 1) / cus) * ((nch + MK_U - 1) / MK_U); };
  int worst = items(3 * c.d_model / 2, nch_d);
  worst = std::max(worst, items(c.ffn_hidden, nch_d));
  worst = std::max(worst, items(c.d_model / 2, nch_f));
  worst = std::max(worst, items((c.vocab + 1) / 2, nch_d));
  if (worst > MK_MAX_ITEMS) { *why = "too many row pairs per workgroup"; return false; }
  const int gpw = 64 / (c.head_dim / 8), ng = MK_WAVES * gpw;
  const size_t stage = (size_t)(std::max(nch_d, nch_f) + 1) * 512;
  const size_t attn = (size_t)2 * ng + (size_t)ng * c.head_dim + c.head_dim + 2;
  I->mega_lds = std::max(stage, attn) * sizeof(float);
  if (I->mega_lds > 64 * 1024) { *why = "input vector does not fit the LDS staging area"; return false; }
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_mega_kernel, MK_THREADS, I->mega_lds) !=
          hipSuccess || per_cu < 1) {
    *why = "persistent workgroup does not fit a CU";
    return false;
  }
  I->mega_grid = cus;   // one workgroup per CU: all co-resident, which the grid barrier needs
  int splits = cus / c.n_heads;
  I->mega_splits = splits > kAttnMaxSplits ? kAttnMaxSplits : splits;
  return true;
}

void enqueue_decode_mega(Instance* I, hipStream_t s, bool trace = false) {
  const ll_config& c = I->cfg;
  MkArgs a{};
  a.layers = I->at<MkLayer>(I->L.mk_layers);
  a.tok_emb = (const half_t*)I->w.tok_emb;
  a.final_norm = (const half_t*)I->w.final_norm;
  a.lm_head = (const half_t*)I->w.lm_head;
  a.x = I->at<float>(I->L.x); a.q = I->at<float>(I->L.q); a.o = I->at<float>(I->L.o);
  a.m = I->at<float>(I->L.m); a.logits = I->at<float>(I->L.logits);
  a.attn_part = I->at<float>(I->L.attn_part);
  a.attn_cnt = I->at<unsigned>(I->L.attn_cnt);
  a.amax_val = I->at<float>(I->L.mk_amax_val);
  a.amax_idx = I->at<int>(I->L.mk_amax_idx);
  a.rope = I->at<float2>(I->L.rope);
  a.st = I->state();
  a.host_ring = I->dev_ring;
  a.bar = I->at<unsigned>(I->L.mk_bar);
  a.ring_size = I->ring_size;
  a.n_layers = c.n_layers; a.d = c.d_model; a.n_heads = c.n_heads; a.head_dim = c.head_dim;
  a.F = c.ffn_hidden; a.vocab = c.vocab; a.max_seq = c.max_seq; a.attn_splits = I->mega_splits;
  a.eps = c.rms_eps;
  a.trace = trace ? I->at<unsigned long long>(I->L.mk_trace) : nullptr;
  a.spin_limit = 4000000;   // a few seconds, then the step reports an error instead of hanging
  hipLaunchKernelGGL(decode_mega_kernel, dim3(I->mega_grid), dim3(MK_THREADS), I->mega_lds, s, a);
}

void enqueue_decode(Instance* I, hipStream_t s) {
  if (I->use_mega && I->only_class < 0 && !I->prof_events) enqueue_decode_mega(I, s);
  else enqueue_decode_multi(I, s);
}



// Projection GEMM A W_z^T into the slice buffer; the returned map tells the consuming kernel
// which slices to add up for which column.
SliceMap launch_gemm(Instance* I, hipStream_t s, const PfBuffers& B, const half_t* A, const void* w0, const void* w1,
                     const void* w2, int nmat, int ldc, int N, int K, int Mb, const half_t* wf = nullptr) {
  const GemmPlan p = gemm_plan(N, K, nmat, Mb, ldc);
  GemmArgs ga{};
  ga.A = A;
  ga.W[0] = (const half_t*)w0; ga.W[1] = (const half_t*)w1; ga.W[2] = (const half_t*)w2;
  ga.C = B.part;
  ga.st = I->state();
  ga.zeros = B.zeros;
  ga.N = N; ga.K = K; ga.ldc = ldc; ga.nmat = nmat;
  ga.mtiles = p.mtiles; ga.runs = p.runs; ga.map = p.map;
  dim3 grid((p.runs + 7) / 8 * 8 * p.mtiles);      // runs are dealt to the 8 XCDs
  ga.Wf = wf;
  const bool once = p.mtiles == 1;      // a single row tile: every weight byte is used once
  if (gemm_bm(Mb, nmat) == 128 && wf && nmat == 1 && once)
    hipLaunchKernelGGL((pf_gemm_kernel<128, 3, 2, 4, 64, 1, true, true>), grid, dim3(PF_GEMM_THREADS_OF(2, 4)), PF_GEMM_LDS_BYTES(128, 3, 64), s, ga);
  else if (gemm_bm(Mb, nmat) == 128 && wf && nmat == 1)
    hipLaunchKernelGGL((pf_gemm_kernel<128, 3, 2, 4, 64, 1, true>), grid, dim3(PF_GEMM_THREADS_OF(2, 4)), PF_GEMM_LDS_BYTES(128, 3, 64), s, ga);
  else if (gemm_bm(Mb, nmat) == 128 && once)
    hipLaunchKernelGGL((pf_gemm_kernel<128, 3, 2, 4, 64, 1, false, true>), grid, dim3(PF_GEMM_THREADS_OF(2, 4)), PF_GEMM_LDS_BYTES(128, 3, 64), s, ga);
  else if (gemm_bm(Mb, nmat) == 128)
    hipLaunchKernelGGL((pf_gemm_kernel<128, 3, 2, 4, 64>), grid, dim3(PF_GEMM_THREADS_OF(2, 4)), PF_GEMM_LDS_BYTES(128, 3, 64), s, ga);
  else if (wf && nmat == 1 && !once)
    hipLaunchKernelGGL((pf_gemm_kernel<64, 3, 1, 4, 64, 1, true, false>), grid, dim3(PF_GEMM_THREADS_OF(1, 4)), PF_GEMM_LDS_BYTES(64, 3, 64), s, ga);
  else if (wf && nmat == 1)
    hipLaunchKernelGGL((pf_gemm_kernel<64, 3, 1, 4, 64, 1, true>), grid, dim3(PF_GEMM_THREADS_OF(1, 4)), PF_GEMM_LDS_BYTES(64, 3, 64), s, ga);
  else
    hipLaunchKernelGGL((pf_gemm_kernel<64, 3, 1, 4, 64>), grid, dim3(PF_GEMM_THREADS_OF(1, 4)), PF_GEMM_LDS_BYTES(64, 3, 64), s, ga);
  return p.map;
}


template <int MODE>
void launch_skinny(hipStream_t s, const PfBuffers& B, SkinnyArgs a, int Mb) {
  a.zeros_off = B.zeros - a.X;
  if constexpr (MODE != SK_RES) {
    const int per_wave = (((a.K + 31) >> 5) + SK_WAVES - 1) / SK_WAVES;
    if (per_wave <= SKP_KSTEPS) {
      const int units = skinny_units(MODE, a.N);
      dim3 grid(units < g_num_cus ? units : g_num_cus), block(SK_THREADS);
      if (Mb == 16) hipLaunchKernelGGL((pf_skinny_persist_kernel<MODE, 1>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((pf_skinny_persist_kernel<MODE, 2>), grid, block, 0, s, a);
      return;
    }
  }
  dim3 grid(skinny_units(MODE, a.N)), block(SK_THREADS);
  const int per_wave = (((a.K + 31) >> 5) + SK_WAVES - 1) / SK_WAVES, nb = (per_wave + 7) / 8;
  if constexpr (MODE == SK_RES) {       // the 7B shapes get the unrolled pipelines: K = 4096 and K = 11008
    if (nb == 2) {
      if (Mb == 16) hipLaunchKernelGGL((pf_skinny_kernel<MODE, 1, 2>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((pf_skinny_kernel<MODE, 2, 2>), grid, block, 0, s, a);
      return;
    }
    if (nb == 6) {
      if (Mb == 16) hipLaunchKernelGGL((pf_skinny_kernel<MODE, 1, 6>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((pf_skinny_kernel<MODE, 2, 6>), grid, block, 0, s, a);
      return;
    }
  }
  if (Mb == 16) hipLaunchKernelGGL((pf_skinny_kernel<MODE, 1, 0>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((pf_skinny_kernel<MODE, 2, 0>), grid, block, 0, s, a);
}

// Prompts of at most 32 tokens: five kernels per layer, every projection streams its weights
// once and finishes its own epilogue; the norms ride on the projections around them.
void enqueue_prefill_skinny(Instance* I, hipStream_t s, const PfBuffers& B, int Mb, bool with_head) {
  const ll_config& c = I->cfg;
  const int d = c.d_model, F = c.ffn_hidden;
  float* X = B.X;
  half_t *Xn = B.Xn, *Qh = B.Q, *Oh = B.O, *Hm = B.H;
  const int sst = sk_ss_stride(d), parts = d / 16;
  float* ss_attn = B.ss;                          // sums of squares in front of the attention block
  float* ss_ffn = ss_attn + (size_t)32 * sst;     // ... and in front of the FFN
  const int tb = Mb / 16;       // token blocks: the activations' fragment-major layout depends on it
  hipLaunchKernelGGL(pf_embed_norm_kernel, dim3(Mb), dim3(LL_WG), 0, s, (const half_t*)I->w.tok_emb,
                     B.tokens, I->state(), (const half_t*)I->layers[0].attn_norm, X, Xn, ss_attn, sst, d, tb);
  for (int l = 0; l < c.n_layers; ++l) {
    const ll_layer_weights& W = I->layers[l];
    SkinnyArgs a{};
    a.st = I->state(); a.head_dim = c.head_dim; a.max_seq = c.max_seq; a.eps = c.rms_eps; a.ss_stride = sst;
    a.X = Xn; a.W[0] = (const half_t*)W.wq; a.W[1] = (const half_t*)W.wk; a.W[2] = (const half_t*)W.wv;
    a.N = d; a.K = d; a.Q = Qh; a.kc = I->kcache(l); a.vc = I->vcache(l); a.rope = I->at<float2>(I->L.rope);
    a.ss_in = ss_attn; a.ss_parts = l == 0 ? 1 : parts;     // the embedding gather leaves whole sums in slot 0
    a.Wf = I->wfrag(l, I->L.wf_qkv);
    launch_skinny<SK_QKV>(s, B, a, Mb);
    dim3 agrid(c.n_heads, 1);
    if (c.head_dim == 128)
      hipLaunchKernelGGL((pf_attn_kernel<128, 1>), agrid, dim3(128), PF_ATTN_LDS_BYTES(128, 1), s, Qh, I->kcache(l),
                         I->vcache(l), I->state(), Oh, d, c.max_seq, tb);
    else
      hipLaunchKernelGGL((pf_attn_kernel<64, 1>), agrid, dim3(128), PF_ATTN_LDS_BYTES(64, 1), s, Qh, I->kcache(l),
                         I->vcache(l), I->state(), Oh, d, c.max_seq, tb);
    a.X = Oh; a.W[0] = (const half_t*)W.wo; a.W[1] = a.W[2] = nullptr; a.N = d; a.K = d; a.Xres = X;
    a.gain_next = (const half_t*)W.ffn_norm; a.Xh_next = Xn; a.ss_out = ss_ffn;
    a.Wf = I->wfrag(l, I->L.wf_o);
    launch_skinny<SK_RES>(s, B, a, Mb);
    a.X = Xn; a.W[0] = (const half_t*)W.w_gate; a.W[1] = (const half_t*)W.w_up; a.N = F; a.K = d; a.Hout = Hm;
    a.ss_in = ss_ffn; a.ss_parts = parts;
    a.Wf = I->wfrag(l, I->L.wf_gu);
    launch_skinny<SK_GATEUP>(s, B, a, Mb);
    a.X = Hm; a.W[0] = (const half_t*)W.w_down; a.W[1] = nullptr; a.N = d; a.K = F; a.Xres = X;
    a.gain_next = l + 1 < c.n_layers ? (const half_t*)I->layers[l + 1].attn_norm : nullptr;
    a.Xh_next = Xn; a.ss_out = ss_attn;
    a.Wf = I->wfrag(l, I->L.wf_down);
    launch_skinny<SK_RES>(s, B, a, Mb);
  }
  if (with_head) enqueue_head(I, s, B, X, 1, 1);
}

// Prefill attention of layer l for a bucket of Mb >= 64 rows: the longer the prompt, the more
// key groups share a query block (a chunk of a long prompt attends everything cached before it)
template <int HD>
void launch_attn_hd(Instance* I, hipStream_t s, const PfBuffers& B, int l, int Mb) {
  const ll_config& c = I->cfg;
  dim3 grid(c.n_heads, Mb / 64);
  const half_t* Qh = B.Q;
  half_t* Oh = B.O;
  const int groups = (Mb >= 256 || c.max_seq - 1 > kMaxPromptBucket) ? 4 : Mb >= 128 ? 2 : 1;
  if (groups == 4)
    hipLaunchKernelGGL((pf_attn_kernel<HD, 4>), grid, dim3(512), PF_ATTN_LDS_BYTES(HD, 4), s, Qh, I->kcache(l),
                       I->vcache(l), I->state(), Oh, c.d_model, c.max_seq, 0);
  else if (groups == 2)
    hipLaunchKernelGGL((pf_attn_kernel<HD, 2>), grid, dim3(256), PF_ATTN_LDS_BYTES(HD, 2), s, Qh, I->kcache(l),
                       I->vcache(l), I->state(), Oh, c.d_model, c.max_seq, 0);
  else
    hipLaunchKernelGGL((pf_attn_kernel<HD, 1>), grid, dim3(128), PF_ATTN_LDS_BYTES(HD, 1), s, Qh, I->kcache(l),
                       I->vcache(l), I->state(), Oh, c.d_model, c.max_seq, 0);
}

void launch_attn(Instance* I, hipStream_t s, const PfBuffers& B, int l, int Mb) {
  if (I->cfg.head_dim == 128) launch_attn_hd<128>(I, s, B, l, Mb);
  else launch_attn_hd<64>(I, s, B, l, Mb);
}

void enqueue_prefill(Instance* I, hipStream_t s, int Mb, bool with_head = true) {
  const PfBuffers& B = I->pf;
  if (Mb <= 32 && I->skinny) return enqueue_prefill_skinny(I, s, B, Mb, with_head);
  const ll_config& c = I->cfg;
  const int d = c.d_model, F = c.ffn_hidden;
  float* X = B.X;
  half_t *Xn = B.Xn, *Qh = B.Q, *Oh = B.O, *Hm = B.H;
  const float* P = B.part;                         // slices of the GEMM that ran last
  hipLaunchKernelGGL(pf_embed_kernel, dim3(Mb, (d + LL_WG * 8 - 1) / (LL_WG * 8)), dim3(LL_WG), 0, s,
                     (const half_t*)I->w.tok_emb, B.tokens, I->state(), X, d);
  SliceMap res{};                                  // the residual GEMM whose slices are still to be added to X
  const float* res_part = nullptr;
  for (int l = 0; l < c.n_layers; ++l) {
    const ll_layer_weights& W = I->layers[l];
    hipLaunchKernelGGL(pf_rmsnorm_kernel, dim3(Mb), dim3(PF_NORM_THREADS), 0, s, X, (const half_t*)W.attn_norm,
                       Xn, d, c.rms_eps, I->state(), res_part, res, 0);
    const SliceMap qkv = launch_gemm(I, s, B, Xn, W.wq, W.wk, W.wv, 3, 3 * d, d, d, Mb);
    hipLaunchKernelGGL(pf_rope_kv_kernel, dim3(Mb, (d / 8 + LL_WG - 1) / LL_WG), dim3(LL_WG), 0, s, P, qkv,
                       I->at<float2>(I->L.rope), I->state(), Qh, I->kcache(l), I->vcache(l), d,
                       c.head_dim, c.max_seq);
    launch_attn(I, s, B, l, Mb);
    res = launch_gemm(I, s, B, Oh, W.wo, nullptr, nullptr, 1, d, d, d, Mb, I->wfrag(l, I->L.wf_o));
    res_part = P;
    hipLaunchKernelGGL(pf_rmsnorm_kernel, dim3(Mb), dim3(PF_NORM_THREADS), 0, s, X, (const half_t*)W.ffn_norm,
                       Xn, d, c.rms_eps, I->state(), res_part, res, 0);
    const SliceMap gu = launch_gemm(I, s, B, Xn, W.w_gate, W.w_up, nullptr, 2, 2 * F, F, d, Mb);
    hipLaunchKernelGGL(pf_swiglu_kernel, dim3(Mb, (F + LL_WG * 4 - 1) / (LL_WG * 4)), dim3(LL_WG), 0,
                       s, P, gu, I->state(), Hm, F);
    res = launch_gemm(I, s, B, Hm, W.w_down, nullptr, nullptr, 1, d, d, F, Mb, I->wfrag(l, I->L.wf_down));
  }
  if (with_head && res_part)    // (a chunk that is not the prompt's last needs nothing of X any more)
    hipLaunchKernelGGL(pf_fold_kernel, dim3(Mb, (d + LL_WG * 4 - 1) / (LL_WG * 4)), dim3(LL_WG), 0, s, X,
                       I->state(), P, res, d);
  if (with_head) enqueue_head(I, s, B, X, 1, 1);
}

int capture_on(Instance* I, hipStream_t cs, hipGraph_t* graph, hipGraphExec_t* exec, int prefill_bucket,
               bool with_head = true) {
  HIPCHK(hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal));
  if (prefill_bucket) enqueue_prefill(I, cs, prefill_bucket, with_head);
  else enqueue_decode(I, cs);
  hipError_t e = hipStreamEndCapture(cs, graph);
  if (e != hipSuccess) return fail(LL_E_HIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
  HIPCHK(hipGraphInstantiate(exec, *graph, nullptr, nullptr, 0));
  return LL_OK;
}

int capture(Instance* I, hipGraph_t* graph, hipGraphExec_t* exec, int prefill_bucket) {
  return capture_on(I, I->stream, graph, exec, prefill_bucket);
}

int write_state(Instance* I, int pos, int next_token, int n_prompt, int steps) {
  DevState* hs = reinterpret_cast<DevState*>(I->host_stage);
  memset(hs, 0, sizeof(DevState));
  hs->pos = pos; hs->next_token = next_token; hs->n_prompt = n_prompt; hs->steps = steps;
  HIPCHK(hipMemcpyAsync(I->state(), hs, sizeof(DevState), hipMemcpyHostToDevice, I->stream));
  return LL_OK;
}

void destroy(Instance* I) {
  if (!I) return;
  destroy_batch(I->batch);
  I->batch = nullptr;
  if (I->lg_future.valid()) (void)I->lg_future.get();
  if (I->lg_pending.exec) (void)hipGraphExecDestroy(I->lg_pending.exec);
  if (I->lg_pending.graph) (void)hipGraphDestroy(I->lg_pending.graph);
  for (auto& e : I->lg) {
    if (e.exec) (void)hipGraphExecDestroy(e.exec);
    if (e.graph) (void)hipGraphDestroy(e.graph);
  }
  if (I->cap_stream) (void)hipStreamDestroy(I->cap_stream);
  if (I->dec_exec) (void)hipGraphExecDestroy(I->dec_exec);
  if (I->dec_graph) (void)hipGraphDestroy(I->dec_graph);
  if (I->pf_body_exec) (void)hipGraphExecDestroy(I->pf_body_exec);
  if (I->pf_body_graph) (void)hipGraphDestroy(I->pf_body_graph);
  for (auto e : I->pf_exec) if (e) (void)hipGraphExecDestroy(e);
  for (auto gr : I->pf_graph) if (gr) (void)hipGraphDestroy(gr);
  if (I->host_ring) (void)hipHostFree(I->host_ring);
  if (I->host_stage) (void)hipHostFree(I->host_stage);
  if (I->own_stream && I->stream) (void)hipStreamDestroy(I->stream);
  delete I;
}

bool eager(const Instance* I) { return (I->cfg.flags & LL_FLAG_EAGER) != 0; }

// ---- one graph per KV length (Alg. 1; Sec. IV-A): rolling buffer, LRU eviction, the next length
// captured by a second thread on a second stream while the current graph replays.  The kernels
// read the length from the device state, so every one of these graphs is the same graph: what
// this mode measures is what capturing per length costs.
constexpr size_t kLenGraphBuffer = 8;

Instance::LenGraph* lg_find(Instance* I, int len) {
  for (auto& e : I->lg) if (e.len == len) return &e;
  return nullptr;
}

// the stream is idle when this runs, so nothing that is evicted can still be executing
void lg_insert(Instance* I, const Instance::LenGraph& ng) {
  if (I->lg.size() >= kLenGraphBuffer) {
    size_t victim = 0;
    for (size_t i = 1; i < I->lg.size(); ++i) if (I->lg[i].used < I->lg[victim].used) victim = i;
    (void)hipGraphExecDestroy(I->lg[victim].exec);
    (void)hipGraphDestroy(I->lg[victim].graph);
    I->lg[victim] = ng;
  } else {
    I->lg.push_back(ng);
  }
}

int lg_capture(Instance* I, int len, Instance::LenGraph* out, std::string* err) {
  const auto t0 = std::chrono::steady_clock::now();
  out->len = len;
  out->used = 0;
  const int rc = capture_on(I, I->cap_stream, &out->graph, &out->exec, 0);
  if (rc != LL_OK && err) *err = g_err;          // this thread's message, for the caller's thread
  I->lg_stats[3] += std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0).count();
  return rc;
}

int lg_join(Instance* I) {
  if (!I->lg_future.valid()) return LL_OK;
  const int rc = I->lg_future.get();
  if (rc != LL_OK) {
    I->lg_pending = Instance::LenGraph();
    return fail(rc, "capture of the next length failed: %s", I->lg_pending_err.c_str());
  }
  lg_insert(I, I->lg_pending);
  I->lg_pending = Instance::LenGraph();
  return LL_OK;
}

int run_decode_steps_per_length(Instance* I, int k) {
  for (int i = 0; i < k; ++i) {
    const int len = I->pos + i;                  // cached positions when this step starts
    Instance::LenGraph* e = lg_find(I, len);
    if (e) {
      ++I->lg_stats[0];
    } else {
      Instance::LenGraph ng;
      const int rc = lg_capture(I, len, &ng, nullptr);
      if (rc != LL_OK) return rc;
      ++I->lg_stats[1];
      lg_insert(I, ng);
      e = lg_find(I, len);
    }
    e->used = ++I->lg_clock;
    HIPCHK(hipGraphLaunch(e->exec, I->stream));
    if (len + 1 < I->cfg.max_seq && !lg_find(I, len + 1)) {
      ++I->lg_stats[2];
      I->lg_future = std::async(std::launch::async, [I, len] {
        return lg_capture(I, len + 1, &I->lg_pending, &I->lg_pending_err);
      });
    }
    HIPCHK(hipStreamSynchronize(I->stream));     // the replay and the capture overlap here
    const int rc = lg_join(I);
    if (rc != LL_OK) return rc;
  }
  return LL_OK;
}

int run_decode_steps(Instance* I, int k) {
  if (I->per_length) return run_decode_steps_per_length(I, k);
  for (int i = 0; i < k; ++i) {
    if (eager(I)) enqueue_decode(I, I->stream);
    else HIPCHK(hipGraphLaunch(I->dec_exec, I->stream));
  }
  if (eager(I)) HIPCHK(hipGetLastError());
  return LL_OK;
}


// ---- batched lock-step decoding over a paged KV cache (batch_kernels.h) ----
struct BatchLayout {
  size_t kv, page_table, state, dstate, logits, total;
  size_t kv_layer_halves;     // halves per layer per K or V pool
  int pool_rows, pt_stride;
};

BatchLayout make_batch_layout(const ll_config& c, int page_tokens, int n_pages) {
  BatchLayout B{};
  B.pool_rows = page_tokens * n_pages;
  B.pt_stride = (c.max_seq + page_tokens - 1) / page_tokens;
  B.kv_layer_halves = (size_t)c.n_heads * B.pool_rows * c.head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  B.kv = take((size_t)c.n_layers * 2 * B.kv_layer_halves * 2);
  B.page_table = take((size_t)BT_MAX_BATCH * B.pt_stride * 4);
  B.state = take(sizeof(BatchState));
  B.dstate = take(sizeof(DevState));
  B.logits = take((size_t)BT_MAX_BATCH * c.vocab * 4);
  B.total = off;
  return B;
}

struct Batch {
  BatchLayout L;
  char* pool = nullptr;
  int max_batch = 0, page_tokens = 0, n_pages = 0;
  int rows = 16;                               // rows of a step: 16 up to 16 slots, else 32
  std::vector<int> free_pages;                 // page 0 is never handed out: free slots write there
  std::vector<std::vector<int>> pages;         // pages of every slot, in order
  BatchState* h_state = nullptr;               // pinned mirrors of the device state and page table
  int* h_table = nullptr;
  int* h_out = nullptr;                        // pinned, device-visible: tokens of the last step
  int* d_out = nullptr;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(pool + off); }
  half_t* kpool(int layer) const { return at<half_t>(L.kv) + (size_t)layer * 2 * L.kv_layer_halves; }
  half_t* vpool(int layer) const { return kpool(layer) + L.kv_layer_halves; }
};

void destroy_batch(Batch* B) {
  if (!B) return;
  if (B->exec) (void)hipGraphExecDestroy(B->exec);
  if (B->graph) (void)hipGraphDestroy(B->graph);
  if (B->h_state) (void)hipHostFree(B->h_state);
  if (B->h_table) (void)hipHostFree(B->h_table);
  if (B->h_out) (void)hipHostFree(B->h_out);
  delete B;
}

// One decode step of all slots: the 16 or 32 rows of the short-prompt kernels are the slots.
void enqueue_batch_step(Instance* I, hipStream_t s) {
  Batch* B = I->batch;
  const PfBuffers& P = I->pf;
  const ll_config& c = I->cfg;
  const int d = c.d_model, F = c.ffn_hidden, Mb = B->rows, tb = Mb / 16;
  float* X = P.X;
  half_t *Xn = P.Xn, *Qh = P.Q, *Oh = P.O, *Hm = P.H;
  const int sst = sk_ss_stride(d), parts = d / 16;
  float* ss_attn = P.ss;
  float* ss_ffn = ss_attn + (size_t)32 * sst;
  BatchState* bs = B->at<BatchState>(B->L.state);
  const DevState* st = B->at<DevState>(B->L.dstate);          // n_prompt = rows of the step, pos unused
  const int* table = B->at<int>(B->L.page_table);
  hipLaunchKernelGGL(pf_embed_norm_kernel, dim3(Mb), dim3(LL_WG), 0, s, (const half_t*)I->w.tok_emb,
                     bs->next_token, st, (const half_t*)I->layers[0].attn_norm, X, Xn, ss_attn, sst, d, tb);
  for (int l = 0; l < c.n_layers; ++l) {
    const ll_layer_weights& W = I->layers[l];
    SkinnyArgs a{};
    a.st = st; a.head_dim = c.head_dim; a.max_seq = B->L.pool_rows; a.eps = c.rms_eps; a.ss_stride = sst;
    a.X = Xn; a.W[0] = (const half_t*)W.wq; a.W[1] = (const half_t*)W.wk; a.W[2] = (const half_t*)W.wv;
    a.N = d; a.K = d; a.Q = Qh; a.kc = B->kpool(l); a.vc = B->vpool(l); a.rope = I->at<float2>(I->L.rope);
    a.ss_in = ss_attn; a.ss_parts = l == 0 ? 1 : parts;
    a.row_pos = bs->pos; a.page_table = table; a.pt_stride = B->L.pt_stride; a.page_tokens = B->page_tokens;
    a.Wf = I->wfrag(l, I->L.wf_qkv);
    launch_skinny<SK_QKV>(s, P, a, Mb);
    dim3 agrid(c.n_heads, Mb);
    if (c.head_dim == 128)
      hipLaunchKernelGGL(bt_attn_kernel<128>, agrid, dim3(BT_ATTN_THREADS), (size_t)B->L.pt_stride * 4, s, Qh, B->kpool(l), B->vpool(l), bs,
                         table, B->L.pt_stride, B->page_tokens, Oh, d, B->L.pool_rows, tb);
    else
      hipLaunchKernelGGL(bt_attn_kernel<64>, agrid, dim3(BT_ATTN_THREADS), (size_t)B->L.pt_stride * 4, s, Qh, B->kpool(l), B->vpool(l), bs,
                         table, B->L.pt_stride, B->page_tokens, Oh, d, B->L.pool_rows, tb);
    a.row_pos = nullptr; a.page_table = nullptr;
    a.X = Oh; a.W[0] = (const half_t*)W.wo; a.W[1] = a.W[2] = nullptr; a.N = d; a.K = d; a.Xres = X;
    a.gain_next = (const half_t*)W.ffn_norm; a.Xh_next = Xn; a.ss_out = ss_ffn;
    a.Wf = I->wfrag(l, I->L.wf_o);
    launch_skinny<SK_RES>(s, P, a, Mb);
    a.X = Xn; a.W[0] = (const half_t*)W.w_gate; a.W[1] = (const half_t*)W.w_up; a.N = F; a.K = d; a.Hout = Hm;
    a.ss_in = ss_ffn; a.ss_parts = parts;
    a.Wf = I->wfrag(l, I->L.wf_gu);
    launch_skinny<SK_GATEUP>(s, P, a, Mb);
    a.X = Hm; a.W[0] = (const half_t*)W.w_down; a.W[1] = nullptr; a.N = d; a.K = F; a.Xres = X;
    a.gain_next = l + 1 < c.n_layers ? (const half_t*)I->layers[l + 1].attn_norm : (const half_t*)I->w.final_norm;
    a.Xh_next = Xn; a.ss_out = ss_attn;
    a.Wf = I->wfrag(l, I->L.wf_down);
    launch_skinny<SK_RES>(s, P, a, Mb);
  }
  {
    // LM head of all rows: the wide persistent projection with a plain fp32 epilogue
    SkinnyArgs a{};
    a.st = st; a.eps = c.rms_eps; a.head_dim = c.head_dim; a.max_seq = c.max_seq;
    a.X = Xn; a.W[0] = (const half_t*)I->w.lm_head; a.N = c.vocab; a.K = d;
    a.ss_in = ss_attn; a.ss_stride = sst; a.ss_parts = parts; a.logits = B->at<float>(B->L.logits);
    a.Wf = I->wfrag_lm();
    a.zeros_off = P.zeros - a.X;
    const int units = skinny_units(SK_LOGITS, c.vocab);
    dim3 grid(units < g_num_cus ? units : g_num_cus);
    if (tb == 1) hipLaunchKernelGGL((pf_skinny_persist_kernel<SK_LOGITS, 1>), grid, dim3(SK_THREADS), 0, s, a);
    else hipLaunchKernelGGL((pf_skinny_persist_kernel<SK_LOGITS, 2>), grid, dim3(SK_THREADS), 0, s, a);
  }
  hipLaunchKernelGGL(bt_select_kernel, dim3(Mb), dim3(SMP_THREADS), SMP_Z_WORDS * 4, s, B->at<float>(B->L.logits),
                     c.vocab, I->at<SampleCfg>(I->L.sample_cfg), bs, B->d_out);
}

int push_batch_state(Instance* I) {
  Batch* B = I->batch;
  HIPCHK(hipMemcpyAsync(B->at<BatchState>(B->L.state), B->h_state, sizeof(BatchState), hipMemcpyHostToDevice, I->stream));
  HIPCHK(hipMemcpyAsync(B->at<int>(B->L.page_table), B->h_table, (size_t)BT_MAX_BATCH * B->L.pt_stride * 4,
                        hipMemcpyHostToDevice, I->stream));
  return LL_OK;
}

}  // namespace

extern "C" {

const char* ll_last_error(void) { return g_err.c_str(); }

size_t ll_workspace_bytes(const ll_config* cfg) {
  if (!config_ok(cfg, nullptr)) return 0;
  return make_layout(*cfg).total;
}

int ll_init(const ll_config* cfg, const ll_weights* w, void* workspace, size_t workspace_bytes,
            void* hip_stream) {
  if (g) return fail(LL_E_ALREADY_INIT, "ll_init: already initialised; call ll_shutdown first");
  const char* why = nullptr;
  if (!config_ok(cfg, &why)) return fail(LL_E_BAD_CONFIG, "ll_init: %s", why);
  if (!w || !w->tok_emb || !w->layers || !w->final_norm || !w->lm_head)
    return fail(LL_E_BAD_ARG, "ll_init: null weight pointer");
  for (int l = 0; l < cfg->n_layers; ++l) {
    const ll_layer_weights& lw = w->layers[l];
    if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.ffn_norm || !lw.w_gate ||
        !lw.w_up || !lw.w_down)
      return fail(LL_E_BAD_ARG, "ll_init: null weight pointer in layer %d", l);
  }
  if (!workspace) return fail(LL_E_BAD_ARG, "ll_init: null workspace");
  Layout L = make_layout(*cfg);
  if (workspace_bytes < L.total)
    return fail(LL_E_WORKSPACE, "ll_init: workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign)
    return fail(LL_E_WORKSPACE, "ll_init: workspace must be %zu-byte aligned", kAlign);
  if (gemv_lds_bytes(cfg->ffn_hidden, false) > 64 * 1024 || gemv_lds_bytes(cfg->d_model, true) > 64 * 1024)
    return fail(LL_E_BAD_CONFIG, "ll_init: d_model / ffn_hidden too large for the LDS-staged GEMV (at most 12288)");
  if (cfg->n_heads > 256)
    return fail(LL_E_BAD_CONFIG, "ll_init: n_heads = %d, at most 256 (two attention workgroups per head)", cfg->n_heads);

  Instance* I = new Instance();
  I->cfg = *cfg;
  I->L = L;
  I->layers.assign(w->layers, w->layers + cfg->n_layers);
  I->w = *w;
  I->w.layers = I->layers.data();
  I->ws = static_cast<char*>(workspace);
  I->pf = PfBuffers{I->at<float>(L.pf_x), I->at<half_t>(L.pf_xn), I->at<half_t>(L.pf_q), I->at<half_t>(L.pf_o),
                    I->at<half_t>(L.pf_h), I->at<float>(L.pf_part), I->at<float>(L.pf_ss), I->at<int>(L.tokens),
                    I->at<float>(L.logits), I->at<float>(L.amax_val), I->at<int>(L.amax_idx), I->at<half_t>(L.zeros)};
  I->last_logits = I->pf.logits;
  int rc = LL_OK;
  {
    void* sp = nullptr;
    if (hipGetDevice(&I->device) != hipSuccess) { delete I; return fail(LL_E_HIP, "ll_init: hipGetDevice failed"); }
    if ((rc = static_scratch_ptr(I->device, &sp)) != LL_OK) { delete I; return rc; }
    I->static_scratch = static_cast<char*>(sp);
  }
  auto bail = [&](int code) { destroy(I); return code; };

  if (hip_stream) {
    I->stream = static_cast<hipStream_t>(hip_stream);
  } else {
    hipError_t e = hipStreamCreateWithFlags(&I->stream, hipStreamNonBlocking);
    if (e != hipSuccess) return bail(fail(LL_E_HIP, "hipStreamCreate: %s", hipGetErrorString(e)));
    I->own_stream = true;
  }

  I->ring_size = cfg->max_seq + 1;
  auto hip_or_bail = [&](hipError_t e, const char* what) {
    if (e != hipSuccess) { rc = fail(LL_E_HIP, "%s: %s", what, hipGetErrorString(e)); return false; }
    return true;
  };
  if (!hip_or_bail(hipHostMalloc((void**)&I->host_ring, (size_t)I->ring_size * 4, hipHostMallocMapped),
                   "hipHostMalloc(ring)")) return bail(rc);
  if (!hip_or_bail(hipHostGetDevicePointer((void**)&I->dev_ring, I->host_ring, 0),
                   "hipHostGetDevicePointer")) return bail(rc);
  if (!hip_or_bail(hipHostMalloc((void**)&I->host_stage, sizeof(DevState) + (size_t)L.mb_max * 4 + 64,
                                 hipHostMallocDefault), "hipHostMalloc(stage)")) return bail(rc);
  memset(I->host_ring, 0, (size_t)I->ring_size * 4);

  // RoPE table: angle pos * theta^(-2j/head_dim) and its cos/sin in double, stored as float
  {
    const int hh = cfg->head_dim / 2;
    std::vector<float2> tab((size_t)cfg->max_seq * hh);
    std::vector<double> inv_freq(hh);
    for (int j = 0; j < hh; ++j)
      inv_freq[j] = std::pow((double)cfg->rope_theta, -2.0 * (double)j / (double)cfg->head_dim);
    for (int p = 0; p < cfg->max_seq; ++p)
      for (int j = 0; j < hh; ++j) {
        const double phi = (double)p * inv_freq[j];
        tab[(size_t)p * hh + j] = make_float2((float)std::cos(phi), (float)std::sin(phi));
      }
    if (!hip_or_bail(hipMemcpy(I->at<float2>(L.rope), tab.data(), tab.size() * sizeof(float2),
                               hipMemcpyHostToDevice), "hipMemcpy(rope)")) return bail(rc);
  }
  if (!hip_or_bail(hipMemset(I->at<unsigned>(L.attn_cnt), 0, (size_t)cfg->n_heads * 4), "hipMemset(cnt)"))
    return bail(rc);
  if (!hip_or_bail(hipMemset(I->state(), 0, sizeof(DevState)), "hipMemset(state)")) return bail(rc);
  if (!hip_or_bail(hipMemset(I->at<int>(L.tokens), 0, (size_t)L.mb_max * 4), "hipMemset(tokens)"))
    return bail(rc);
  if (!hip_or_bail(hipMemset(I->at<char>(L.zeros), 0, 256), "hipMemset(zeros)")) return bail(rc);
  if (!hip_or_bail(hipMemset(I->at<char>(L.ao_sync), 0, 64 * 4), "hipMemset(sync)")) return bail(rc);
  if (!hip_or_bail(hipMemset(I->at<char>(L.sample_cfg), 0, sizeof(SampleCfg)), "hipMemset(sampling)"))
    return bail(rc);                                           // inv_temp = 0: greedy
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&sample_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMP_Z_WORDS * 4),
                   "hipFuncSetAttribute(sample)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&bt_select_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMP_Z_WORDS * 4),
                   "hipFuncSetAttribute(batch select)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<128, 3, 2, 4, 64, 1, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_GEMM_LDS_BYTES(128, 3, 64)),
                   "hipFuncSetAttribute(gemm 128, fragment-major weights)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<128, 3, 2, 4, 64>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_GEMM_LDS_BYTES(128, 3, 64)),
                   "hipFuncSetAttribute(gemm 128)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<128, 3, 2, 4, 64, 1, true, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_GEMM_LDS_BYTES(128, 3, 64)),
                   "hipFuncSetAttribute(gemm 128, fragment-major weights used once)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<128, 3, 2, 4, 64, 1, false, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_GEMM_LDS_BYTES(128, 3, 64)),
                   "hipFuncSetAttribute(gemm 128, weights used once)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<64, 3, 1, 4, 64, 1, true, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_GEMM_LDS_BYTES(64, 3, 64)),
                   "hipFuncSetAttribute(gemm 64, fragment-major weights shared by two row tiles)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<64, 3, 1, 4, 64>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_GEMM_LDS_BYTES(64, 3, 64)),
                   "hipFuncSetAttribute(gemm 64)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_gemm_kernel<64, 3, 1, 4, 64, 1, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_GEMM_LDS_BYTES(64, 3, 64)),
                   "hipFuncSetAttribute(gemm 64, fragment-major weights)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_attn_kernel<128, 4>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_ATTN_LDS_BYTES(128, 4)),
                   "hipFuncSetAttribute(attention 128 x 4)")) return bail(rc);
  if (!hip_or_bail(hipFuncSetAttribute(reinterpret_cast<const void*>(&pf_attn_kernel<64, 4>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, PF_ATTN_LDS_BYTES(64, 4)),
                   "hipFuncSetAttribute(attention 64 x 4)")) return bail(rc);
  if (!hip_or_bail(hipMemset(I->at<unsigned>(L.mk_bar), 0, (size_t)MK_BAR_WORDS * 4), "hipMemset(bar)"))
    return bail(rc);
  {
    std::vector<MkLayer> tab(cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l) {
      const ll_layer_weights& lw = I->layers[l];
      tab[l] = MkLayer{(const half_t*)lw.attn_norm, (const half_t*)lw.wq, (const half_t*)lw.wk,
                       (const half_t*)lw.wv, (const half_t*)lw.wo, (const half_t*)lw.ffn_norm,
                       (const half_t*)lw.w_gate, (const half_t*)lw.w_up, (const half_t*)lw.w_down,
                       I->kcache(l), I->vcache(l)};
    }
    if (!hip_or_bail(hipMemcpy(I->at<MkLayer>(L.mk_layers), tab.data(), tab.size() * sizeof(MkLayer),
                               hipMemcpyHostToDevice), "hipMemcpy(layer table)")) return bail(rc);
  }
  if (L.wf_layer) {
    // the short-prompt kernels' copy of the projection weights, written once (the weights must not
    // change while the instance lives)
    const int d = cfg->d_model, F = cfg->ffn_hidden, kd = (d + 31) / 32, kf = (F + 31) / 32;
    auto shuffle = [&](auto kernel, int units, int ksteps, const void* w0, const void* w1, const void* w2, int N, int K,
                       const half_t* out) {
      hipLaunchKernelGGL(kernel, dim3(units, (ksteps + LL_WG / 64 - 1) / (LL_WG / 64)), dim3(LL_WG), 0, I->stream,
                         (const half_t*)w0, (const half_t*)w1, (const half_t*)w2, N, K, cfg->head_dim, const_cast<half_t*>(out));
    };
    for (int l = 0; l < cfg->n_layers; ++l) {
      const ll_layer_weights& lw = I->layers[l];
      shuffle(sk_shuffle_kernel<SK_QKV>, skinny_units(SK_QKV, d), kd, lw.wq, lw.wk, lw.wv, d, d, I->wfrag(l, L.wf_qkv));
      shuffle(sk_shuffle_kernel<SK_RES>, skinny_units(SK_RES, d), kd, lw.wo, nullptr, nullptr, d, d, I->wfrag(l, L.wf_o));
      shuffle(sk_shuffle_kernel<SK_GATEUP>, skinny_units(SK_GATEUP, F), kd, lw.w_gate, lw.w_up, nullptr, F, d, I->wfrag(l, L.wf_gu));
      shuffle(sk_shuffle_kernel<SK_RES>, skinny_units(SK_RES, d), kf, lw.w_down, nullptr, nullptr, d, F, I->wfrag(l, L.wf_down));
    }
    if (I->wfrag_lm())
      shuffle(sk_shuffle_kernel<SK_LOGITS>, skinny_units(SK_LOGITS, cfg->vocab), kd, I->w.lm_head, nullptr, nullptr,
              cfg->vocab, d, I->wfrag_lm());
    if (!hip_or_bail(hipGetLastError(), "weight re-layout launch")) return bail(rc);
  }
  if ((cfg->flags & LL_FLAG_PERSISTENT) && !(cfg->flags & (LL_FLAG_EAGER | LL_FLAG_MULTIKERNEL))) {
    std::string why;
    I->use_mega = mega_plan(I, &why);
    if (!I->use_mega) return bail(fail(LL_E_BAD_CONFIG, "ll_init: persistent kernel unavailable: %s", why.c_str()));
  }
  if (cfg->flags & LL_FLAG_PER_LENGTH_GRAPHS) {
    if (cfg->flags & (LL_FLAG_EAGER | LL_FLAG_PERSISTENT))
      return bail(fail(LL_E_BAD_CONFIG, "ll_init: LL_FLAG_PER_LENGTH_GRAPHS replays the multi-kernel graph; "
                                        "it excludes LL_FLAG_EAGER and LL_FLAG_PERSISTENT"));
    I->per_length = true;
    if (!hip_or_bail(hipStreamCreateWithFlags(&I->cap_stream, hipStreamNonBlocking), "hipStreamCreate(capture)"))
      return bail(rc);
  }
  if (!hip_or_bail(hipDeviceSynchronize(), "hipDeviceSynchronize")) return bail(rc);

  I->skinny = skinny_ok(*cfg);
  (void)num_cus();
  for (int b = I->skinny ? 16 : 64; b <= L.mb_max; b <<= 1) I->pf_buckets.push_back(b);
  // Opt-in: attention and O projection in one launch.  It needs the whole of W_o in the registers of one
  // round of workgroups (rows of at most 4096), at most two attention workgroups per head, and a CU
  // for every workgroup of the launch (the projection's wait needs them all resident).
  if (cfg->flags & LL_FLAG_FUSED_ATTN_OPROJ) {
    const int wgs = cfg->n_heads * L.attn_splits + (cfg->d_model / 2 + ATTN_THREADS / 64 - 1) / (ATTN_THREADS / 64);
    if (cfg->d_model > 4096 || L.attn_splits > ATTN_FUSED_MAX_SPLITS || wgs > g_num_cus)
      return bail(fail(LL_E_BAD_CONFIG, "ll_init: LL_FLAG_FUSED_ATTN_OPROJ needs d_model <= 4096, max_seq <= 2048 and "
                                        "2 * n_heads + d_model / 32 = %d workgroups <= %d CUs", wgs, g_num_cus));
    I->fused_attn = true;
  }

  // Warm-up: one eager pass of every kernel chain (loads the code objects, so
  // nothing is compiled or loaded inside a capture), on state that is reset
  // afterwards.  Token 0 at position 0 / a one-token prompt touch only valid memory.
  if ((rc = write_state(I, 0, 0, 1, 0)) != LL_OK) return bail(rc);
  enqueue_decode(I, I->stream);
  for (int b : I->pf_buckets) {
    if ((rc = write_state(I, 0, 0, 1, 0)) != LL_OK) return bail(rc);
    enqueue_prefill(I, I->stream, b);
  }
  if (!hip_or_bail(hipStreamSynchronize(I->stream), "warm-up")) return bail(rc);
  if (!hip_or_bail(hipGetLastError(), "warm-up launch")) return bail(rc);

  if (!(cfg->flags & LL_FLAG_EAGER)) {
    if ((rc = capture(I, &I->dec_graph, &I->dec_exec, 0)) != LL_OK) return bail(rc);
    I->pf_graph.assign(I->pf_buckets.size(), nullptr);
    I->pf_exec.assign(I->pf_buckets.size(), nullptr);
    for (size_t i = 0; i < I->pf_buckets.size(); ++i)
      if ((rc = capture(I, &I->pf_graph[i], &I->pf_exec[i], I->pf_buckets[i])) != LL_OK) return bail(rc);
    if (L.max_prompt > L.mb_max &&
        (rc = capture_on(I, I->stream, &I->pf_body_graph, &I->pf_body_exec, L.mb_max, false)) != LL_OK)
      return bail(rc);
  }
  if ((rc = write_state(I, 0, 0, 0, 0)) != LL_OK) return bail(rc);
  if (!hip_or_bail(hipStreamSynchronize(I->stream), "init sync")) return bail(rc);
  I->pos = 0;
  I->steps = 0;
  g = I;
  g_err.clear();
  return LL_OK;
}

int ll_shutdown(void) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_shutdown: not initialised");
  (void)hipStreamSynchronize(g->stream);
  destroy(g);
  g = nullptr;
  return LL_OK;
}

int ll_reset(void) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_reset: not initialised");
  int rc = write_state(g, 0, 0, 0, 0);
  if (rc != LL_OK) return rc;
  // also clears a barrier time-out left behind by a failed step
  HIPCHK(hipMemsetAsync(g->at<unsigned>(g->L.mk_bar), 0, (size_t)MK_BAR_WORDS * 4, g->stream));
  HIPCHK(hipMemsetAsync(g->at<unsigned>(g->L.attn_cnt), 0, (size_t)g->cfg.n_heads * 4, g->stream));
  HIPCHK(hipMemsetAsync(g->at<char>(g->L.ao_sync), 0, 64 * 4, g->stream));
  HIPCHK(hipStreamSynchronize(g->stream));
  g->pos = 0;
  g->steps = 0;
  return LL_OK;
}

int ll_set_sampling(float temperature, int32_t top_k, float top_p, uint64_t seed) {
  if (!(temperature >= 0.f) || !(temperature < INFINITY))
    return fail(LL_E_BAD_ARG, "ll_set_sampling: temperature = %g, need a finite value >= 0", (double)temperature);
  if (top_k < 0) return fail(LL_E_BAD_ARG, "ll_set_sampling: top_k = %d < 0", top_k);
  if (!(top_p > 0.f && top_p <= 1.f))
    return fail(LL_E_BAD_ARG, "ll_set_sampling: top_p = %g outside (0, 1]", (double)top_p);
  if (!g) return fail(LL_E_NOT_INIT, "ll_set_sampling: not initialised");
  Instance* I = g;
  if (temperature > 0.f && I->use_mega)
    return fail(LL_E_STATE, "ll_set_sampling: the persistent-kernel mode selects greedily only");
  if (temperature > 0.f && I->cfg.vocab > SMP_MAX_VOCAB)
    return fail(LL_E_CAPACITY, "ll_set_sampling: vocab = %d > %d", I->cfg.vocab, SMP_MAX_VOCAB);
  SampleCfg* h = reinterpret_cast<SampleCfg*>(I->host_stage);
  memset(h, 0, sizeof(SampleCfg));
  h->inv_temp = temperature > 0.f ? (float)(1.0 / (double)temperature) : 0.f;
  h->top_k = top_k;
  h->top_p = top_p;
  h->seed_lo = (uint32_t)(seed & 0xffffffffu);
  h->seed_hi = (uint32_t)(seed >> 32);
  HIPCHK(hipMemcpyAsync(I->at<SampleCfg>(I->L.sample_cfg), h, sizeof(SampleCfg), hipMemcpyHostToDevice, I->stream));
  HIPCHK(hipStreamSynchronize(I->stream));
  return LL_OK;
}

int32_t ll_max_prompt(void) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_max_prompt: not initialised");
  return g->L.max_prompt;
}

int32_t ll_position(void) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_position: not initialised");
  return g->pos;
}

}  // extern "C"

namespace {

// Checks shared by the two prefill entry points
int prefill_check(Instance* I, const char* who, const int32_t* tokens, int32_t n) {
  if (!tokens) return fail(LL_E_BAD_ARG, "%s: null tokens", who);
  if (n < 1) return fail(LL_E_BAD_ARG, "%s: n = %d < 1", who, n);
  if (I->pos != 0) return fail(LL_E_STATE, "%s: context holds %d positions; call ll_reset", who, I->pos);
  if (n + 1 > I->cfg.max_seq) return fail(LL_E_CAPACITY, "%s: n + 1 = %d > max_seq = %d", who, n + 1, I->cfg.max_seq);
  if (n > I->L.max_prompt) return fail(LL_E_CAPACITY, "%s: n = %d > ll_max_prompt() = %d", who, n, I->L.max_prompt);
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= I->cfg.vocab)
      return fail(LL_E_BAD_ARG, "%s: tokens[%d] = %d outside [0, %d)", who, i, tokens[i], I->cfg.vocab);
  return LL_OK;
}

}  // namespace

extern "C" {

int32_t ll_prefill(const int32_t* tokens, int32_t n) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_prefill: not initialised");
  Instance* I = g;
  const int chk = prefill_check(I, "ll_prefill", tokens, n);
  if (chk != LL_OK) return chk;

  // prompt ids and the state block travel in one pinned staging buffer.  A prompt longer than the
  // largest bucket goes through in chunks of that size: every chunk but the last runs the layers
  // only (its rows just fill the KV cache), the last one also produces the first token.
  DevState* hs = reinterpret_cast<DevState*>(I->host_stage);
  int* htok = reinterpret_cast<int*>(reinterpret_cast<char*>(I->host_stage) + sizeof(DevState));
  for (int p0 = 0; p0 < n;) {
    const int m = n - p0 > I->L.mb_max ? I->L.mb_max : n - p0;
    const bool last = p0 + m == n;
    const int Mb = (I->skinny && m <= 32) ? (m <= 16 ? 16 : 32) : prompt_bucket(m);
    memset(hs, 0, sizeof(DevState));
    hs->pos = p0;
    hs->n_prompt = m;
    memcpy(htok, tokens + p0, (size_t)m * 4);
    HIPCHK(hipMemcpyAsync(I->state(), hs, sizeof(DevState), hipMemcpyHostToDevice, I->stream));
    HIPCHK(hipMemcpyAsync(I->pf.tokens, htok, (size_t)m * 4, hipMemcpyHostToDevice, I->stream));
    if (eager(I)) {
      enqueue_prefill(I, I->stream, Mb, last);
      HIPCHK(hipGetLastError());
    } else if (!last) {
      HIPCHK(hipGraphLaunch(I->pf_body_exec, I->stream));
    } else {
      size_t bi = 0;
      while (I->pf_buckets[bi] != Mb) ++bi;
      HIPCHK(hipGraphLaunch(I->pf_exec[bi], I->stream));
    }
    HIPCHK(hipStreamSynchronize(I->stream));       // the staging buffer is reused by the next chunk
    I->last_chunk_rows = m;
    p0 += m;
  }
  I->pos = n;
  I->steps = 1;
  I->last_was_prefill = true;
  I->last_logits = I->pf.logits;
  I->last_rows = I->pf.X;
  return I->host_ring[0];
}

int32_t ll_prefill_static(const int32_t* tokens, int32_t n) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_prefill_static: not initialised");
  Instance* I = g;
  const int chk = prefill_check(I, "ll_prefill_static", tokens, n);
  if (chk != LL_OK) return chk;
  if (n > 32)
    return fail(LL_E_CAPACITY, "ll_prefill_static: n = %d tokens, at most 32 fit the static scratch; use ll_prefill", n);
  if (!I->skinny)
    return fail(LL_E_BAD_CONFIG, "ll_prefill_static: needs d_model %% 16 == 0, head_dim %% 16 == 0 and ffn_hidden %% 8 == 0");
  PfBuffers B{};
  const size_t need = carve_short_prefill(I->cfg, I->L.lm_wgs, I->static_scratch, &B);
  if (need > LL_STATIC_SCRATCH_BYTES)
    return fail(LL_E_CAPACITY, "ll_prefill_static: this model needs %zu bytes of scratch, the static array holds %u; "
                               "use ll_prefill", need, (unsigned)LL_STATIC_SCRATCH_BYTES);

  // The array keeps what the last call left: the block of zeros that out-of-range operand loads are
  // aimed at is cleared here; everything else is written by this call before it is read.
  HIPCHK(hipMemsetAsync(B.zeros, 0, 256, I->stream));
  DevState* hs = reinterpret_cast<DevState*>(I->host_stage);
  int* htok = reinterpret_cast<int*>(reinterpret_cast<char*>(I->host_stage) + sizeof(DevState));
  memset(hs, 0, sizeof(DevState));
  hs->n_prompt = n;
  memcpy(htok, tokens, (size_t)n * 4);
  HIPCHK(hipMemcpyAsync(I->state(), hs, sizeof(DevState), hipMemcpyHostToDevice, I->stream));
  HIPCHK(hipMemcpyAsync(B.tokens, htok, (size_t)n * 4, hipMemcpyHostToDevice, I->stream));
  enqueue_prefill_skinny(I, I->stream, B, n <= 16 ? 16 : 32, true);     // launched kernel by kernel: no graph holds these addresses
  HIPCHK(hipGetLastError());
  HIPCHK(hipStreamSynchronize(I->stream));
  I->last_chunk_rows = n;
  I->pos = n;
  I->steps = 1;
  I->last_was_prefill = true;
  I->last_logits = B.logits;
  I->last_rows = B.X;
  return I->host_ring[0];
}

int32_t ll_decode_n(int32_t k, int32_t* out_tokens) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_decode_n: not initialised");
  Instance* I = g;
  if (k < 1) return fail(LL_E_BAD_ARG, "ll_decode_n: k = %d < 1", k);
  if (I->pos == 0) return fail(LL_E_STATE, "ll_decode: empty context; call ll_prefill first");
  if (I->pos + k > I->cfg.max_seq)
    return fail(LL_E_CAPACITY, "ll_decode: %d cached + %d steps > max_seq = %d", I->pos, k, I->cfg.max_seq);
  if (I->steps + k > I->ring_size)
    return fail(LL_E_CAPACITY, "ll_decode: token ring full");
  int rc = run_decode_steps(I, k);
  if (rc != LL_OK) return rc;
  HIPCHK(hipStreamSynchronize(I->stream));
  for (int i = 0; i < k; ++i)
    if (I->host_ring[I->steps + i] < 0)
      return fail(LL_E_HIP, "ll_decode: a bounded wait between workgroups of one launch ran out (are other "
                            "kernels occupying the GPU?); call ll_reset");
  if (out_tokens) memcpy(out_tokens, I->host_ring + I->steps, (size_t)k * 4);
  I->pos += k;
  I->steps += k;
  I->last_was_prefill = false;
  I->last_logits = I->pf.logits;
  return I->host_ring[I->steps - 1];
}

int32_t ll_decode_step(void) { return ll_decode_n(1, nullptr); }

/* ---- batched lock-step decoding over a paged KV cache ---- */

size_t ll_batch_pool_bytes(int32_t page_tokens, int32_t n_pages) {
  if (!g || page_tokens < 1 || n_pages < 2) return 0;
  return make_batch_layout(g->cfg, page_tokens, n_pages).total;
}

int ll_batch_open(int32_t max_batch, int32_t page_tokens, int32_t n_pages, void* pool, size_t pool_bytes) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_open: not initialised");
  Instance* I = g;
  if (I->batch) return fail(LL_E_STATE, "ll_batch_open: already open; call ll_batch_close first");
  if (max_batch < 1 || max_batch > BT_MAX_BATCH)
    return fail(LL_E_BAD_ARG, "ll_batch_open: max_batch = %d outside [1, %d]", max_batch, BT_MAX_BATCH);
  if (page_tokens < 1 || n_pages < 2)
    return fail(LL_E_BAD_ARG, "ll_batch_open: need page_tokens >= 1 and n_pages >= 2 (page 0 is reserved)");
  if (!pool) return fail(LL_E_BAD_ARG, "ll_batch_open: null pool");
  const ll_config& c = I->cfg;
  const int per_wave = (((c.d_model + 31) >> 5) + SK_WAVES - 1) / SK_WAVES;
  if (!I->skinny || c.vocab % 16 != 0 || per_wave > SKP_KSTEPS || (c.head_dim != 64 && c.head_dim != 128))
    return fail(LL_E_BAD_CONFIG, "ll_batch_open: needs d_model %% 16 == 0, d_model <= 4096, ffn_hidden %% 8 == 0, "
                                 "vocab %% 16 == 0 and head_dim 64 or 128");
  if (I->use_mega || I->per_length)
    return fail(LL_E_STATE, "ll_batch_open: available with the multi-kernel graph and eager modes only");
  const BatchLayout BL = make_batch_layout(c, page_tokens, n_pages);
  if (BL.pt_stride > 8192)
    return fail(LL_E_BAD_ARG, "ll_batch_open: max_seq / page_tokens = %d pages per sequence, at most 8192 "
                              "(the attention kernel keeps a sequence's page list in LDS)", BL.pt_stride);
  if (pool_bytes < BL.total)
    return fail(LL_E_WORKSPACE, "ll_batch_open: pool has %zu bytes, %zu needed", pool_bytes, BL.total);
  if (reinterpret_cast<uintptr_t>(pool) % kAlign)
    return fail(LL_E_WORKSPACE, "ll_batch_open: pool must be %zu-byte aligned", kAlign);

  Batch* B = new Batch();
  B->L = BL;
  B->pool = static_cast<char*>(pool);
  B->max_batch = max_batch; B->page_tokens = page_tokens; B->n_pages = n_pages;
  B->rows = max_batch <= 16 ? 16 : 32;
  for (int p = n_pages - 1; p >= 1; --p) B->free_pages.push_back(p);
  B->pages.resize(BT_MAX_BATCH);
  int rc = LL_OK;
  auto bail = [&](int code) { I->batch = nullptr; destroy_batch(B); return code; };
  auto ok = [&](hipError_t e, const char* what) {
    if (e != hipSuccess) { rc = fail(LL_E_HIP, "%s: %s", what, hipGetErrorString(e)); return false; }
    return true;
  };
  if (!ok(hipHostMalloc((void**)&B->h_state, sizeof(BatchState), hipHostMallocDefault), "hipHostMalloc(batch state)"))
    return bail(rc);
  if (!ok(hipHostMalloc((void**)&B->h_table, (size_t)BT_MAX_BATCH * BL.pt_stride * 4, hipHostMallocDefault),
          "hipHostMalloc(page table)")) return bail(rc);
  if (!ok(hipHostMalloc((void**)&B->h_out, BT_MAX_BATCH * 4, hipHostMallocMapped), "hipHostMalloc(batch out)"))
    return bail(rc);
  if (!ok(hipHostGetDevicePointer((void**)&B->d_out, B->h_out, 0), "hipHostGetDevicePointer(batch out)")) return bail(rc);
  memset(B->h_state, 0, sizeof(BatchState));
  memset(B->h_table, 0, (size_t)BT_MAX_BATCH * BL.pt_stride * 4);          // every slot: page 0
  for (int b = 0; b < BT_MAX_BATCH; ++b) B->h_out[b] = -1;
  I->batch = B;
  {
    DevState* hs = reinterpret_cast<DevState*>(I->host_stage);
    memset(hs, 0, sizeof(DevState));
    hs->n_prompt = B->rows;
    if (!ok(hipMemcpyAsync(B->at<DevState>(BL.dstate), hs, sizeof(DevState), hipMemcpyHostToDevice, I->stream),
            "hipMemcpy(batch rows)")) return bail(rc);
    if (!ok(hipStreamSynchronize(I->stream), "batch init sync")) return bail(rc);
  }
  // page 0 must hold finite numbers: free slots attend nothing, but their K/V rows are written there
  if (!ok(hipMemsetAsync(B->at<char>(BL.kv), 0, (size_t)c.n_layers * 2 * BL.kv_layer_halves * 2, I->stream),
          "hipMemset(pool)")) return bail(rc);
  if ((rc = push_batch_state(I)) != LL_OK) return bail(rc);
  enqueue_batch_step(I, I->stream);                                         // warm-up on empty slots
  if (!ok(hipStreamSynchronize(I->stream), "batch warm-up")) return bail(rc);
  if (!ok(hipGetLastError(), "batch warm-up launch")) return bail(rc);
  if (!eager(I)) {
    hipError_t e = hipStreamBeginCapture(I->stream, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return bail(fail(LL_E_HIP, "hipStreamBeginCapture: %s", hipGetErrorString(e)));
    enqueue_batch_step(I, I->stream);
    e = hipStreamEndCapture(I->stream, &B->graph);
    if (e != hipSuccess) return bail(fail(LL_E_HIP, "hipStreamEndCapture: %s", hipGetErrorString(e)));
    if (!ok(hipGraphInstantiate(&B->exec, B->graph, nullptr, nullptr, 0), "hipGraphInstantiate(batch)")) return bail(rc);
  }
  return LL_OK;
}

int ll_batch_close(void) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_close: not initialised");
  if (!g->batch) return fail(LL_E_STATE, "ll_batch_close: not open");
  (void)hipStreamSynchronize(g->stream);
  destroy_batch(g->batch);
  g->batch = nullptr;
  return LL_OK;
}

int32_t ll_batch_add(const int32_t* tokens, int32_t n, int32_t* first_token) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_add: not initialised");
  Instance* I = g;
  Batch* B = I->batch;
  if (!B) return fail(LL_E_STATE, "ll_batch_add: call ll_batch_open first");
  if (!tokens || !first_token) return fail(LL_E_BAD_ARG, "ll_batch_add: null argument");
  if (n < 1) return fail(LL_E_BAD_ARG, "ll_batch_add: n = %d < 1", n);
  if (n + 1 > I->cfg.max_seq) return fail(LL_E_CAPACITY, "ll_batch_add: n + 1 = %d > max_seq = %d", n + 1, I->cfg.max_seq);
  int slot = -1;
  for (int b = 0; b < B->max_batch && slot < 0; ++b)
    if (!B->h_state->active[b]) slot = b;
  if (slot < 0) return fail(LL_E_CAPACITY, "ll_batch_add: all %d slots are taken", B->max_batch);
  const int need = (n + 1 + B->page_tokens - 1) / B->page_tokens;       // the prompt and the first generated position
  if ((int)B->free_pages.size() < need)
    return fail(LL_E_CAPACITY, "ll_batch_add: %d pages needed, %zu free", need, B->free_pages.size());

  for (int i = 0; i < n; ++i)                     // before anything is touched: ll_prefill's own check comes after the reset
    if (tokens[i] < 0 || tokens[i] >= I->cfg.vocab)
      return fail(LL_E_BAD_ARG, "ll_batch_add: tokens[%d] = %d outside [0, %d)", i, tokens[i], I->cfg.vocab);
  // the prompt runs through the single-sequence prefill (whose context it replaces) ...
  int rc = ll_reset();
  if (rc != LL_OK) return rc;
  const int32_t t1 = ll_prefill(tokens, n);
  if (t1 < 0) return t1;
  // ... and its cache rows move into the slot's pages
  for (int i = 0; i < need; ++i) {
    const int pg = B->free_pages.back();
    B->free_pages.pop_back();
    B->pages[slot].push_back(pg);
    B->h_table[slot * B->L.pt_stride + i] = pg * B->page_tokens;
  }
  B->h_state->pos[slot] = n;
  B->h_state->next_token[slot] = t1;
  B->h_state->active[slot] = 1;
  B->h_state->steps[slot] = 1;                  // the prefill drew with index 0
  if ((rc = push_batch_state(I)) != LL_OK) return rc;
  const ll_config& c = I->cfg;
  hipLaunchKernelGGL(bt_scatter_kernel, dim3(n, c.n_layers * 2), dim3(LL_WG), 0, I->stream, I->kcache(0),
                     I->L.kv_layer_halves, c.max_seq, B->kpool(0), B->L.kv_layer_halves, B->L.pool_rows,
                     B->at<int>(B->L.page_table), B->L.pt_stride, B->page_tokens, slot, c.n_heads, c.head_dim);
  HIPCHK(hipGetLastError());
  HIPCHK(hipStreamSynchronize(I->stream));
  *first_token = t1;
  return slot;
}

int ll_batch_remove(int32_t slot) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_remove: not initialised");
  Batch* B = g->batch;
  if (!B) return fail(LL_E_STATE, "ll_batch_remove: call ll_batch_open first");
  if (slot < 0 || slot >= B->max_batch || !B->h_state->active[slot])
    return fail(LL_E_BAD_ARG, "ll_batch_remove: slot %d holds no sequence", slot);
  for (int pg : B->pages[slot]) B->free_pages.push_back(pg);
  B->pages[slot].clear();
  for (int i = 0; i < B->L.pt_stride; ++i) B->h_table[slot * B->L.pt_stride + i] = 0;
  B->h_state->pos[slot] = 0;
  B->h_state->next_token[slot] = 0;
  B->h_state->active[slot] = 0;
  B->h_state->steps[slot] = 0;
  int rc = push_batch_state(g);
  if (rc != LL_OK) return rc;
  HIPCHK(hipStreamSynchronize(g->stream));
  return LL_OK;
}

int ll_batch_step(int32_t* out_tokens) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_step: not initialised");
  Instance* I = g;
  Batch* B = I->batch;
  if (!B) return fail(LL_E_STATE, "ll_batch_step: call ll_batch_open first");
  if (!out_tokens) return fail(LL_E_BAD_ARG, "ll_batch_step: null output");
  // this step writes position pos[b] of every active slot: check capacity and pages before anything runs
  int fresh = 0, live = 0;
  for (int b = 0; b < B->max_batch; ++b) {
    if (!B->h_state->active[b]) continue;
    ++live;
    const int p = B->h_state->pos[b];
    if (p + 1 > I->cfg.max_seq)
      return fail(LL_E_CAPACITY, "ll_batch_step: slot %d holds %d positions, max_seq = %d", b, p, I->cfg.max_seq);
    if (p / B->page_tokens >= (int)B->pages[b].size()) ++fresh;
  }
  if (!live) return fail(LL_E_STATE, "ll_batch_step: no sequence in the batch");
  if (fresh > (int)B->free_pages.size())
    return fail(LL_E_CAPACITY, "ll_batch_step: %d new pages needed, %zu free", fresh, B->free_pages.size());
  // Pages are handed out on the device first (the new table entries travel by value in front of the
  // step); the host's lists and pool follow only once the step has run, so a launch or
  // synchronisation that fails leaves the bookkeeping as it was.
  PageUpdates up{};                                // at most one new page per slot and step
  int up_slot[BT_MAX_BATCH];
  if (fresh) {
    size_t next_free = B->free_pages.size();
    for (int b = 0; b < B->max_batch; ++b) {
      if (!B->h_state->active[b]) continue;
      const int i = B->h_state->pos[b] / B->page_tokens;
      if (i < (int)B->pages[b].size()) continue;
      const int pg = B->free_pages[--next_free];
      up_slot[up.n] = b;
      up.index[up.n] = b * B->L.pt_stride + i;
      up.row[up.n++] = pg * B->page_tokens;
    }
    hipLaunchKernelGGL(bt_page_update_kernel, dim3(1), dim3(64), 0, I->stream, B->at<int>(B->L.page_table), up);
    HIPCHK(hipGetLastError());
  }
  if (eager(I)) {
    enqueue_batch_step(I, I->stream);
    HIPCHK(hipGetLastError());
  } else {
    HIPCHK(hipGraphLaunch(B->exec, I->stream));
  }
  HIPCHK(hipStreamSynchronize(I->stream));
  for (int j = 0; j < up.n; ++j) {                 // the step ran: the pages are the slots' now
    B->free_pages.pop_back();
    B->pages[up_slot[j]].push_back(up.row[j] / B->page_tokens);
    B->h_table[up.index[j]] = up.row[j];
  }
  for (int b = 0; b < BT_MAX_BATCH; ++b) {
    const int t = b < B->max_batch ? B->h_out[b] : -1;
    if (b < B->max_batch) out_tokens[b] = t;
    if (b < B->max_batch && B->h_state->active[b]) {       // the host mirror follows the device state
      B->h_state->pos[b] += 1;
      B->h_state->steps[b] += 1;
      B->h_state->next_token[b] = t;
    }
  }
  return LL_OK;
}

int ll_batch_dbg_get_logits(int32_t slot, float* host_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_dbg_get_logits: not initialised");
  Batch* B = g->batch;
  if (!B) return fail(LL_E_STATE, "ll_batch_dbg_get_logits: call ll_batch_open first");
  if (slot < 0 || slot >= B->max_batch || !host_out) return fail(LL_E_BAD_ARG, "ll_batch_dbg_get_logits: bad argument");
  HIPCHK(hipStreamSynchronize(g->stream));
  HIPCHK(hipMemcpy(host_out, B->at<float>(B->L.logits) + (size_t)slot * g->cfg.vocab, (size_t)g->cfg.vocab * 4,
                   hipMemcpyDeviceToHost));
  return LL_OK;
}

int ll_batch_dbg_force_next_token(int32_t slot, int32_t tok) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_dbg_force_next_token: not initialised");
  Batch* B = g->batch;
  if (!B) return fail(LL_E_STATE, "ll_batch_dbg_force_next_token: call ll_batch_open first");
  if (slot < 0 || slot >= B->max_batch || !B->h_state->active[slot] || tok < 0 || tok >= g->cfg.vocab)
    return fail(LL_E_BAD_ARG, "ll_batch_dbg_force_next_token: bad argument");
  B->h_state->next_token[slot] = tok;
  int rc = push_batch_state(g);
  if (rc != LL_OK) return rc;
  HIPCHK(hipStreamSynchronize(g->stream));
  return LL_OK;
}

int ll_batch_dbg_time_steps(int32_t k, float* ms_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_batch_dbg_time_steps: not initialised");
  Instance* I = g;
  Batch* B = I->batch;
  if (!B) return fail(LL_E_STATE, "ll_batch_dbg_time_steps: call ll_batch_open first");
  if (k < 1 || !ms_out) return fail(LL_E_BAD_ARG, "ll_batch_dbg_time_steps: bad argument");
  // k steps back to back: the pages those steps will write are taken up front
  int fresh = 0;
  for (int b = 0; b < B->max_batch; ++b) {
    if (!B->h_state->active[b]) continue;
    if (B->h_state->pos[b] + k > I->cfg.max_seq)
      return fail(LL_E_CAPACITY, "ll_batch_dbg_time_steps: slot %d would pass max_seq", b);
    const int want = (B->h_state->pos[b] + k - 1) / B->page_tokens + 1;
    if (want > (int)B->pages[b].size()) fresh += want - (int)B->pages[b].size();
  }
  if (fresh > (int)B->free_pages.size())
    return fail(LL_E_CAPACITY, "ll_batch_dbg_time_steps: %d new pages needed, %zu free", fresh, B->free_pages.size());
  if (fresh) {
    for (int b = 0; b < B->max_batch; ++b) {
      if (!B->h_state->active[b]) continue;
      const int want = (B->h_state->pos[b] + k - 1) / B->page_tokens + 1;
      while ((int)B->pages[b].size() < want) {
        const int pg = B->free_pages.back();
        B->free_pages.pop_back();
        B->h_table[b * B->L.pt_stride + (int)B->pages[b].size()] = pg * B->page_tokens;
        B->pages[b].push_back(pg);
      }
    }
    HIPCHK(hipMemcpyAsync(B->at<int>(B->L.page_table), B->h_table, (size_t)BT_MAX_BATCH * B->L.pt_stride * 4,
                          hipMemcpyHostToDevice, I->stream));
  }
  hipEvent_t e0, e1;
  HIPCHK(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(LL_E_HIP, "ll_batch_dbg_time_steps: hipEventCreate"); }
  hipError_t te = hipEventRecord(e0, I->stream);
  for (int i = 0; i < k && te == hipSuccess; ++i) {
    if (eager(I)) enqueue_batch_step(I, I->stream);
    else te = hipGraphLaunch(B->exec, I->stream);
  }
  if (te == hipSuccess) te = hipEventRecord(e1, I->stream);
  if (te == hipSuccess) te = hipStreamSynchronize(I->stream);
  if (te == hipSuccess) te = hipEventElapsedTime(ms_out, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (te != hipSuccess) return fail(LL_E_HIP, "ll_batch_dbg_time_steps: %s", hipGetErrorString(te));
  for (int b = 0; b < B->max_batch; ++b)
    if (B->h_state->active[b]) { B->h_state->pos[b] += k; B->h_state->steps[b] += k; B->h_state->next_token[b] = B->h_out[b]; }
  return LL_OK;
}

int ll_decode_mode(void) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_decode_mode: not initialised");
  if (g->cfg.flags & LL_FLAG_EAGER) return LL_MODE_EAGER;
  if (g->per_length) return LL_MODE_PER_LENGTH_GRAPHS;
  return g->use_mega ? LL_MODE_PERSISTENT_GRAPH : LL_MODE_MULTIKERNEL_GRAPH;
}

int ll_dbg_gemm_plan(int32_t N, int32_t K, int32_t nmat, int32_t rows, int32_t* out6) {
  if (!out6 || N < 1 || K < 1 || nmat < 1 || nmat > 3 || (rows != 64 && rows != 128 && rows != 256 && rows != 512 && rows != 1024))
    return fail(LL_E_BAD_ARG, "ll_dbg_gemm_plan: bad argument");
  const GemmPlan p = gemm_plan(N, K, nmat, rows, nmat * N);
  out6[0] = gemm_bm(rows, nmat); out6[1] = p.mtiles; out6[2] = p.runs; out6[3] = p.map.quota;
  out6[4] = p.map.nslabs; out6[5] = p.max_slices;
  return LL_OK;
}

int ll_dbg_gemm_slice_count(int32_t N, int32_t K, int32_t nmat, int32_t rows, int32_t col) {
  if (N < 1 || K < 1 || nmat < 1 || nmat > 3 || (rows != 64 && rows != 128 && rows != 256 && rows != 512 && rows != 1024) ||
      col < 0 || col >= nmat * N)
    return fail(LL_E_BAD_ARG, "ll_dbg_gemm_slice_count: bad argument");
  const GemmPlan p = gemm_plan(N, K, nmat, rows, nmat * N);
  return slice_count(p.map, col);
}

int ll_dbg_graph_stats(int64_t* out4) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_graph_stats: not initialised");
  if (!out4) return fail(LL_E_BAD_ARG, "ll_dbg_graph_stats: null output");
  for (int i = 0; i < 4; ++i) out4[i] = g->lg_stats[i];
  return LL_OK;
}

int ll_dbg_get_logits(float* host_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_get_logits: not initialised");
  if (!host_out) return fail(LL_E_BAD_ARG, "ll_dbg_get_logits: null output");
  HIPCHK(hipStreamSynchronize(g->stream));
  HIPCHK(hipMemcpy(host_out, g->last_logits, (size_t)g->cfg.vocab * 4, hipMemcpyDeviceToHost));
  return LL_OK;
}

int ll_dbg_get_hidden(float* host_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_get_hidden: not initialised");
  if (!host_out) return fail(LL_E_BAD_ARG, "ll_dbg_get_hidden: null output");
  if (g->pos == 0) return fail(LL_E_STATE, "ll_dbg_get_hidden: no step has run");
  HIPCHK(hipStreamSynchronize(g->stream));
  const float* src = g->last_was_prefill
                         ? g->last_rows + (size_t)(g->last_chunk_rows - 1) * g->cfg.d_model
                         : g->at<float>(g->use_mega ? g->L.x : g->L.x_keep);
  HIPCHK(hipMemcpy(host_out, src, (size_t)g->cfg.d_model * 4, hipMemcpyDeviceToHost));
  return LL_OK;
}

int ll_dbg_force_next_token(int32_t tok) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_force_next_token: not initialised");
  if (tok < 0 || tok >= g->cfg.vocab) return fail(LL_E_BAD_ARG, "ll_dbg_force_next_token: bad token %d", tok);
  if (g->pos == 0) return fail(LL_E_STATE, "ll_dbg_force_next_token: empty context");
  int* h = g->host_stage;
  *h = tok;
  HIPCHK(hipMemcpyAsync(&g->state()->next_token, h, 4, hipMemcpyHostToDevice, g->stream));
  if (!g->use_mega) {            // the step reads the token's embedding row from x, not the id
    const int d = g->cfg.d_model;
    hipLaunchKernelGGL(embed_kernel, dim3((d + LL_WG * 8 - 1) / (LL_WG * 8)), dim3(LL_WG), 0, g->stream,
                       (const half_t*)g->w.tok_emb, g->state(), g->at<float>(g->L.x), d);
    HIPCHK(hipGetLastError());
  }
  HIPCHK(hipStreamSynchronize(g->stream));
  return LL_OK;
}

int ll_dbg_get_kv(int32_t layer, int32_t which, int32_t n_pos, float* host_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_get_kv: not initialised");
  const ll_config& c = g->cfg;
  if (layer < 0 || layer >= c.n_layers || (which != 0 && which != 1) || n_pos < 0 || n_pos > c.max_seq || !host_out)
    return fail(LL_E_BAD_ARG, "ll_dbg_get_kv: bad argument");
  HIPCHK(hipStreamSynchronize(g->stream));
  std::vector<uint16_t> tmp(g->L.kv_layer_halves);
  const half_t* src = which ? g->vcache(layer) : g->kcache(layer);
  HIPCHK(hipMemcpy(tmp.data(), src, tmp.size() * 2, hipMemcpyDeviceToHost));
  for (int h = 0; h < c.n_heads; ++h)
    for (int p = 0; p < n_pos; ++p)
      for (int e = 0; e < c.head_dim; ++e) {
        uint16_t bits = tmp[((size_t)h * c.max_seq + p) * c.head_dim + e];
        _Float16 v;
        memcpy(&v, &bits, 2);
        host_out[(size_t)p * c.d_model + h * c.head_dim + e] = (float)v;
      }
  return LL_OK;
}

int ll_dbg_profile_decode(int32_t steps, float* us_out, int32_t* launches_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_profile_decode: not initialised");
  Instance* I = g;
  if (steps < 1 || !us_out) return fail(LL_E_BAD_ARG, "ll_dbg_profile_decode: bad argument");
  if (I->pos == 0) return fail(LL_E_STATE, "ll_dbg_profile_decode: empty context");
  if (I->pos + steps > I->cfg.max_seq || I->steps + steps > I->ring_size)
    return fail(LL_E_CAPACITY, "ll_dbg_profile_decode: would run past max_seq");
  double sum[LL_KC_COUNT] = {0};
  long cnt[LL_KC_COUNT] = {0};
  for (int sidx = 0; sidx < steps; ++sidx) {
    std::vector<hipEvent_t> ev;
    std::vector<int> kc;
    I->prof_events = &ev;
    I->prof_class = &kc;
    enqueue_decode(I, I->stream);
    I->prof_events = nullptr;
    I->prof_class = nullptr;
    hipError_t e = hipStreamSynchronize(I->stream);
    if (e == hipSuccess) {
      for (size_t i = 0; i < kc.size(); ++i) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]);
        sum[kc[i]] += ms * 1000.0;
        cnt[kc[i]] += 1;
      }
    }
    for (auto x : ev) (void)hipEventDestroy(x);
    if (e != hipSuccess) return fail(LL_E_HIP, "profile: %s", hipGetErrorString(e));
  }
  I->pos += steps;
  I->steps += steps;
  I->last_was_prefill = false;
  I->last_logits = I->pf.logits;
  for (int i = 0; i < LL_KC_COUNT; ++i) {
    us_out[i] = cnt[i] ? (float)(sum[i] / cnt[i]) : 0.f;
    if (launches_out) launches_out[i] = (int32_t)(cnt[i] / steps);
  }
  return LL_OK;
}

int ll_dbg_trace_decode(uint64_t* ticks_out, int32_t max_phases) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_trace_decode: not initialised");
  Instance* I = g;
  if (!I->use_mega) return fail(LL_E_STATE, "ll_dbg_trace_decode: persistent kernel not in use");
  const int phases = 5 * I->cfg.n_layers + 1;
  if (!ticks_out || max_phases < phases) return fail(LL_E_BAD_ARG, "ll_dbg_trace_decode: need room for %d phases", phases);
  if (I->pos == 0) return fail(LL_E_STATE, "ll_dbg_trace_decode: empty context");
  if (I->pos + 1 > I->cfg.max_seq || I->steps + 1 > I->ring_size)
    return fail(LL_E_CAPACITY, "ll_dbg_trace_decode: cache full");
  HIPCHK(hipMemsetAsync(I->at<char>(I->L.mk_trace), 0, (size_t)phases * 8 * 8, I->stream));
  enqueue_decode_mega(I, I->stream, true);
  HIPCHK(hipGetLastError());
  HIPCHK(hipStreamSynchronize(I->stream));
  HIPCHK(hipMemcpy(ticks_out, I->at<char>(I->L.mk_trace), (size_t)phases * 8 * 8, hipMemcpyDeviceToHost));
  I->pos += 1;
  I->steps += 1;
  I->last_was_prefill = false;
  I->last_logits = I->pf.logits;
  return phases;
}

int ll_dbg_stream_copy(void* dst, const void* src, size_t bytes) {
  if (!dst || !src || bytes == 0 || bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 ||
      reinterpret_cast<uintptr_t>(src) % 16)
    return fail(LL_E_BAD_ARG, "ll_dbg_stream_copy: pointers and size must be 16-byte multiples");
  hipStream_t s = g ? g->stream : nullptr;
  hipLaunchKernelGGL(stream_copy_kernel, dim3(num_cus() * 8), dim3(LL_WG), 0, s, (const h8*)src, (h8*)dst,
                     bytes / 16);
  HIPCHK(hipGetLastError());
  HIPCHK(hipStreamSynchronize(s));
  return LL_OK;
}

int ll_dbg_poison_scratch(void) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_poison_scratch: not initialised");
  Instance* I = g;
  const Layout& L = I->L;
  // every buffer a step or a prefill is meant to (re)write before it reads it; what carries state from
  // call to call (KV rows, RoPE table, state block, the next step's input row x, sampling settings,
  // barrier and arrival counters, the block of zeros) stays
  const size_t regions[][2] = {
      {L.x_keep, L.q}, {L.q, L.o}, {L.o, L.m}, {L.m, L.attn_part}, {L.attn_part, L.attn_cnt}, {L.logits, L.amax_val},
      {L.amax_val, L.amax_idx}, {L.amax_idx, L.state}, {L.tokens, L.pf_x}, {L.pf_x, L.pf_xn}, {L.pf_xn, L.pf_q},
      {L.pf_q, L.pf_o}, {L.pf_o, L.pf_part}, {L.pf_part, L.pf_h}, {L.pf_h, L.pf_ss}, {L.pf_ss, L.zeros}};
  HIPCHK(hipStreamSynchronize(I->stream));
  for (const auto& r : regions) {
    if (r[1] <= r[0]) return fail(LL_E_STATE, "ll_dbg_poison_scratch: layout order changed");
    HIPCHK(hipMemsetAsync(I->ws + r[0], 0xFF, r[1] - r[0], I->stream));      // all-ones bytes: NaN as fp16 and as fp32
  }
  HIPCHK(hipStreamSynchronize(I->stream));
  return LL_OK;
}

int ll_dbg_stream_read(const void* src, size_t bytes, int32_t reps, void* sink, float* gbps_out) {
  if (!src || !sink || !gbps_out || bytes == 0 || bytes % 16 || reps < 1 || reinterpret_cast<uintptr_t>(src) % 16)
    return fail(LL_E_BAD_ARG, "ll_dbg_stream_read: bad argument");
  hipStream_t s = g ? g->stream : nullptr;
  const int grid = num_cus() * kGemvWgsPerCu;
  hipEvent_t e0, e1;
  HIPCHK(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(LL_E_HIP, "ll_dbg_stream_read: hipEventCreate"); }
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(LL_WG), 0, s, (const h8*)src, bytes / 16, (unsigned*)sink);   // untimed
  (void)hipEventRecord(e0, s);
  for (int r = 0; r < reps; ++r)
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(LL_WG), 0, s, (const h8*)src, bytes / 16, (unsigned*)sink);
  (void)hipEventRecord(e1, s);
  hipError_t e = hipStreamSynchronize(s);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return fail(LL_E_HIP, "ll_dbg_stream_read: %s", hipGetErrorString(e));
  *gbps_out = (float)((double)(bytes / 16384 * 16384) * reps / (ms * 1e-3) / 1e9);   // the kernel reads whole 16 KiB blocks
  return LL_OK;
}

int ll_dbg_time_kernel_class(int32_t klass, int32_t reps, float* us_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_time_kernel_class: not initialised");
  Instance* I = g;
  if (klass < LL_KC_QKV || klass > LL_KC_LMHEAD || reps < 1 || !us_out)
    return fail(LL_E_BAD_ARG, "ll_dbg_time_kernel_class: bad argument");
  if (I->pos == 0) return fail(LL_E_STATE, "ll_dbg_time_kernel_class: empty context");
  if (I->pos >= I->cfg.max_seq) return fail(LL_E_CAPACITY, "ll_dbg_time_kernel_class: cache full");
  if (klass == LL_KC_OPROJ && I->fused_attn)
    return fail(LL_E_STATE, "ll_dbg_time_kernel_class: the O projection runs inside the attention launch in this instance");
  hipEvent_t e0, e1;
  HIPCHK(hipEventCreate(&e0));
  HIPCHK(hipEventCreate(&e1));
  I->only_class = klass;
  enqueue_decode(I, I->stream);   // untimed pass
  (void)hipEventRecord(e0, I->stream);
  for (int r = 0; r < reps; ++r) enqueue_decode(I, I->stream);
  (void)hipEventRecord(e1, I->stream);
  I->only_class = -1;
  hipError_t e = hipStreamSynchronize(I->stream);
  float ms = 0.f;
  if (e == hipSuccess) (void)hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return fail(LL_E_HIP, "time_kernel_class: %s", hipGetErrorString(e));
  const int per_pass = klass == LL_KC_LMHEAD ? 1 : I->cfg.n_layers;
  *us_out = ms * 1000.f / (float)(reps * per_pass);
  return LL_OK;
}

int ll_dbg_time_decode(int32_t k, float* ms_out) {
  if (!g) return fail(LL_E_NOT_INIT, "ll_dbg_time_decode: not initialised");
  Instance* I = g;
  if (k < 1 || !ms_out) return fail(LL_E_BAD_ARG, "ll_dbg_time_decode: bad argument");
  if (I->pos == 0) return fail(LL_E_STATE, "ll_dbg_time_decode: empty context");
  if (I->pos + k > I->cfg.max_seq || I->steps + k > I->ring_size)
    return fail(LL_E_CAPACITY, "ll_dbg_time_decode: would run past max_seq");
  hipEvent_t e0, e1;
  HIPCHK(hipEventCreate(&e0));
  HIPCHK(hipEventCreate(&e1));
  HIPCHK(hipEventRecord(e0, I->stream));
  int rc = run_decode_steps(I, k);
  if (rc == LL_OK) {
    (void)hipEventRecord(e1, I->stream);
    hipError_t e = hipStreamSynchronize(I->stream);
    if (e != hipSuccess) rc = fail(LL_E_HIP, "time_decode: %s", hipGetErrorString(e));
    else (void)hipEventElapsedTime(ms_out, e0, e1);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != LL_OK) return rc;
  I->pos += k;
  I->steps += k;
  I->last_was_prefill = false;
  I->last_logits = I->pf.logits;
  return LL_OK;
}

}  // extern "C"
