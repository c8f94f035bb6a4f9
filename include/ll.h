/*
 * ll.h -- C ABI of the MI355X (gfx950) batch-1 LLaMA decode / prefill path.
 *
 * The problem is the one the paper states in Alg. 1: given a prompt P and
 * model weights W, emit tokens t_1..t_n, one per decoding step, on a single
 * GPU at batch 1 (Sec. IV-E).  The paper replays one captured graph per
 * sequence length and keeps sampling, KV-cache update and position handling on
 * the host side (Sec. III-A, III-B).  This library instead captures ONE decode
 * graph for all lengths: position, KV length and the next token id live in a
 * device-resident state block that the kernels read and the last kernel of the
 * step advances, so the decode loop needs no host round trip.
 *
 * One process-global instance.  Not thread-safe: one caller thread.
 *
 * Memory: every pointer inside ll_weights, and `workspace`, are DEVICE
 * pointers owned by the caller (allocated e.g. through PyTorch) and must stay
 * valid until ll_shutdown().  `tokens`, `out_tokens` and every ll_dbg_* output
 * are HOST pointers.  After ll_init() the library allocates no device memory
 * and never frees caller memory; it owns only its graphs, two small pinned
 * host buffers and host bookkeeping.
 *
 * Weights are IEEE binary16, row-major [out, in] (y = W x); RMSNorm gains are
 * binary16 [d_model]; tok_emb and lm_head are [vocab, d_model] and not tied.  They must not
 * change between ll_init() and ll_shutdown(): the library keeps a re-ordered copy of the
 * projection matrices in the workspace (see LL_FLAG_LEAN_WORKSPACE).
 *
 * Errors: every call returns >= 0 on success and a negative LL_E_* code on
 * failure; ll_last_error() then describes it.  A call that fails its argument,
 * state or capacity checks (every error but LL_E_HIP) has run nothing and
 * leaves the decoder state unchanged.  After LL_E_HIP (a launch, copy or
 * synchronisation failed part-way, e.g. in the second chunk of a long prompt)
 * the context is undefined: call ll_reset().  No exception crosses this boundary.
 *
 * Reproducibility: no kernel on any path accumulates in arrival order (there
 * are no floating-point atomics), so the same call sequence on the same
 * weights gives the same bits, run after run.
 */
#ifndef LL_H
#define LL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  LL_OK = 0,
  LL_E_NOT_INIT = -1,   /* call needs a successful ll_init() first */
  LL_E_BAD_CONFIG = -2, /* unsupported or inconsistent ll_config */
  LL_E_BAD_ARG = -3,    /* null pointer, n < 1, token outside [0, vocab) ... */
  LL_E_CAPACITY = -4,   /* the request would run past max_seq cached positions */
  LL_E_WORKSPACE = -5,  /* workspace smaller than ll_workspace_bytes() or misaligned */
  LL_E_STATE = -6,      /* e.g. ll_prefill on a non-empty context, decode on an empty one */
  LL_E_HIP = -7,        /* a HIP runtime call failed; see ll_last_error() */
  LL_E_ALREADY_INIT = -8
};

/* ll_config.flags */
enum {
  LL_FLAG_EAGER = 1,       /* launch every kernel individually instead of replaying graphs
                              (same kernels, same order: isolates the dispatch cost the
                              paper's Sec. I-B / III-B attribute to per-kernel launches) */
  LL_FLAG_MULTIKERNEL = 2, /* decode step = graph of one kernel per fused operator (~160 nodes) */
  LL_FLAG_PERSISTENT = 4,  /* decode step = graph of ONE persistent kernel with in-kernel grid
                              barriers (needs d_model <= 4096 and one resident workgroup per
                              CU; ll_init fails with LL_E_BAD_CONFIG otherwise).  With neither
                              of the two flags the library picks the faster one it has measured
                              for the 7B shape, currently the multi-kernel graph. */
  LL_FLAG_PER_LENGTH_GRAPHS = 8,
                           /* the paper's own mechanism, kept as an ablation (Alg. 1, Sec. IV-A):
                              one decode graph PER KV LENGTH in a rolling buffer of 8 with
                              least-recently-used eviction; a miss captures before it replays,
                              and the graph of the next length is captured by a second thread on
                              a second stream while the current one replays.  Same kernels as
                              the multi-kernel graph (they read the length from device memory);
                              excludes LL_FLAG_EAGER and LL_FLAG_PERSISTENT. */
  LL_FLAG_LEAN_WORKSPACE = 32,
                           /* do without the second copy of the projection weights that ll_init otherwise
                              writes into the workspace in the short-prompt kernels' operand order (about
                              the size of the layers' weights again: 13 GB at the 7B shape; prompts of at
                              most 32 tokens and batched steps then read the caller's row-major weights,
                              some 15 % slower) */
  LL_FLAG_FUSED_ATTN_OPROJ = 16
                           /* a measured experiment, off by default: decode attention and O projection of
                              a layer in ONE launch, the projection's workgroups holding all of W_o in
                              registers while they wait (bounded) for the attention workgroups' partials.
                              It removes a kernel boundary per layer and comes out level with the two
                              kernels (the hand-off through memory costs what the boundary cost).
                              LL_E_BAD_CONFIG unless d_model <= 4096, max_seq <= 2048 and
                              2 n_heads + d_model / 32 workgroups fit one per CU. */
};

/* what ll_decode_step() replays, see ll_decode_mode() */
enum {
  LL_MODE_PERSISTENT_GRAPH = 0,   /* graph of ONE persistent kernel with in-kernel grid barriers */
  LL_MODE_MULTIKERNEL_GRAPH = 1,  /* graph of one kernel per fused operator */
  LL_MODE_EAGER = 2,              /* the multi-kernel chain launched kernel by kernel */
  LL_MODE_PER_LENGTH_GRAPHS = 3   /* the multi-kernel graph, captured once per KV length */
};

/* Model shape.  Constraints: n_heads * head_dim == d_model; head_dim is 64 or
 * 128; d_model and ffn_hidden are multiples of 8; max_seq >= 2. */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, ffn_hidden, vocab, max_seq;
  float rope_theta; /* RoPE base, e.g. 10000 */
  float rms_eps;    /* added to the mean square inside the root */
  int32_t flags;    /* LL_FLAG_* */
} ll_config;

typedef struct {
  const void *attn_norm;              /* [d_model] */
  const void *wq, *wk, *wv, *wo;      /* [d_model, d_model] */
  const void *ffn_norm;               /* [d_model] */
  const void *w_gate, *w_up;          /* [ffn_hidden, d_model] */
  const void *w_down;                 /* [d_model, ffn_hidden] */
} ll_layer_weights;

typedef struct {
  const void *tok_emb;                /* [vocab, d_model] */
  const ll_layer_weights *layers;     /* HOST array of n_layers entries (device pointers inside) */
  const void *final_norm;             /* [d_model] */
  const void *lm_head;                /* [vocab, d_model] */
} ll_weights;

/* Bytes of device workspace ll_init() needs for this shape: the KV cache, the RoPE table, the
 * state block and the ONE activation arena that every captured graph shares (the paper lets all
 * of its graphs reuse one activation workspace, Sec. IV-B): activations, split-K partials, logits.
 * Host arithmetic only (it asks the current device for its CU count, 256 without a device, because
 * the prefill GEMM's slice buffer is sized for one round of workgroups); returns 0 for a
 * configuration ll_init() would reject. */
size_t ll_workspace_bytes(const ll_config *cfg);

/* The initialisation step of Alg. 1 (streams created, graphs pre-captured; Sec. IV-A): binds the
 * weights W, carves the workspace (256-byte aligned device pointer), uploads the RoPE cos/sin
 * table, warms every kernel up and captures the decode graph (ONE for all lengths, where the paper
 * pre-captures lengths 1-50) and one prefill graph per prompt-length bucket on `hip_stream`, a
 * hipStream_t of default priority that every later call also runs on.  NULL makes the library
 * create a private non-blocking stream of its own: work the caller queued on other streams (e.g.
 * weight uploads) must then have completed before ll_init is called.  Launch shapes follow the
 * device's CU count; the chip it is tuned for has 256 CUs in 8 XCDs.  Context starts empty. */
int ll_init(const ll_config *cfg, const ll_weights *w, void *workspace, size_t workspace_bytes,
            void *hip_stream);

/* Time-to-first-token call (the paper's TTFT metric, Sec. IV-E / Table I):
 * runs the whole prompt (1 <= n, n + 1 <= max_seq, n <= ll_max_prompt())
 * through the MFMA prefill path, fills KV positions 0..n-1 and returns the
 * first generated token t_1 (greedy by default: lowest index among the maxima of
 * the logits at position n-1; see ll_set_sampling).  Requires an empty context (after ll_init or
 * ll_reset), else LL_E_STATE.  Blocks until the token is on the host. */
int32_t ll_prefill(const int32_t *tokens, int32_t n);

/* ll_prefill() for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc) and so cannot bring the prefill's share of a
 * workspace: the same kernels, launched one by one, with everything a short prefill needs besides its
 * inputs and outputs (activations, per-token partial sums, logits, selection candidates, the staged
 * ids) in a static device array of the library (4 MiB, one copy per GPU, held until the process
 * ends) instead of the workspace.  Same arguments, result, state change and errors as ll_prefill;
 * the KV rows, the state block and the token go where ll_prefill puts them, so ll_decode_step()
 * continues from either.  Limits, LL_E_CAPACITY beyond them: n <= 32 tokens, and a model whose
 * short-prompt buffers fit the array (about 336 d_model + 64 ffn_hidden + 4 vocab bytes <= 4 MiB;
 * the 7B shape takes 2.2 MiB); LL_E_BAD_CONFIG unless d_model % 16 == 0 and ffn_hidden % 8 == 0.
 * Calls no hipMalloc / hipFree or other allocating routine.  Every call on a GPU shares that GPU's
 * array, which keeps the last call's contents (the call clears what must start at zero): calls that
 * overlap on one GPU race. */
int32_t ll_prefill_static(const int32_t *tokens, int32_t n);

/* One decoding step (Alg. 1 loop body): feeds the previous step's token at the
 * next position, appends its key/value rows, returns the next token (greedy by
 * default, see ll_set_sampling).
 * Blocks until the token is on the host.  LL_E_STATE on an empty context,
 * LL_E_CAPACITY once max_seq positions are cached. */
int32_t ll_decode_step(void);

/* k iterations of the decoding loop of Alg. 1 enqueued back to back with ONE synchronisation at
 * the end (the loop needs no host round trip: position, KV length and token stay on the device);
 * out_tokens (host, k entries, may be NULL) receives the generated ids.  Returns the last token.
 * Same errors as ll_decode_step, checked for all k steps before anything runs. */
int32_t ll_decode_n(int32_t k, int32_t *out_tokens);

/* Starts a new request (a new prompt P for the loop of Alg. 1, whose initialisation is not repeated):
 * empties the context (position 0, no cached keys; the KV rows need no clearing because the length
 * is what bounds attention); weights, graphs and the workspace binding are kept. */
int ll_reset(void);

/* Token selection of every following ll_prefill / ll_decode_step.  The paper keeps "token
 * sampling" in its host-side dynamic domain (Sec. III-A, III-C) and names stochastic operations
 * as what stays outside graph replay (Sec. VI-C); here the selection runs inside the captured
 * graph and its parameters live in device memory, so no graph is re-captured.
 *   temperature = 0: greedy argmax (the state after ll_init).
 *   temperature > 0: z = logits * float(1 / temperature); keep the top_k largest z (0 = all,
 *     equal values by lower index); softmax over them; keep the smallest set of highest
 *     probabilities whose mass reaches top_p (1 = all, equal values by lower index); draw by
 *     walking the kept tokens in index order with u = (x >> 8) * 2^-24, x = first word of
 *     Philox4x32-10(counter = (i, 0, 0, 0), key = seed), i = tokens produced since the last
 *     ll_reset.  A reset therefore replays the same token stream.
 * LL_E_BAD_ARG for temperature < 0 or not finite, top_k < 0, top_p outside (0, 1];
 * LL_E_CAPACITY for temperature > 0 with vocab > 32768; LL_E_STATE for temperature > 0 in the
 * persistent-kernel mode.  The setting survives ll_reset. */
int ll_set_sampling(float temperature, int32_t top_k, float top_p, uint64_t seed);

/* The clean-up step of Alg. 1: waits for the stream, then destroys the graphs and the host
 * buffers; caller memory is untouched. */
int ll_shutdown(void);

/* Longest prompt ll_prefill() accepts for the current instance: max_seq - 1.  Prompts of more
 * than 1024 tokens are fed through the prefill kernels in chunks of 1024 (the "longer contexts"
 * direction of Sec. VI-E); the chunking is invisible to the caller. */
int32_t ll_max_prompt(void);

/* Number of cached positions (0 when empty), or LL_E_NOT_INIT. */
int32_t ll_position(void);

/* LL_MODE_* of the current instance. */
int ll_decode_mode(void);

/* Text of the most recent failure on this thread ("" if none). */
const char *ll_last_error(void);

/* ---- batched lock-step decoding over a paged KV cache ----
 *
 * The paper stays at batch 1 and takes its KV cache from a paged-attention library (Sec. II-C,
 * Sec. V-A); these calls open the regime it leaves out on top of an initialised instance: up to 32
 * sequences advance one token per call, each projection of the step is one 16- or 32-row matrix
 * product over the weights instead of that many GEMVs, and every sequence keeps its K/V rows in pages of
 * `page_tokens` positions taken from a common pool, so memory follows the sequences' real lengths.
 * Tokens are selected as ll_set_sampling says (greedy by default); every slot draws with its own
 * index, so a sequence sees the same stream in a batch as alone.  Available in the default
 * (multi-kernel graph) and eager modes; the step is one captured graph, like the single-sequence step.
 *
 * Ownership: `pool` is device memory of ll_batch_pool_bytes() bytes, 256-byte aligned, owned by the
 * caller and kept alive until ll_batch_close (or ll_shutdown, which closes the batch).  The calls
 * share the instance's stream and prefill scratch: ll_batch_add runs the prompt through the
 * single-sequence prefill, which REPLACES the context of ll_prefill / ll_decode_step.
 * Errors: negative LL_E_* codes, state unchanged; not thread-safe. */

/* Bytes of `pool` for pages of page_tokens positions, n_pages of them (page 0 is reserved, so
 * n_pages - 1 are usable); 0 without an instance or for arguments ll_batch_open would reject. */
size_t ll_batch_pool_bytes(int32_t page_tokens, int32_t n_pages);
/* Opens batched decoding for up to max_batch (1..32) concurrent sequences (a step computes 16 rows
 * up to 16 slots, 32 beyond).  LL_E_BAD_CONFIG unless
 * d_model % 16 == 0, d_model <= 4096, ffn_hidden % 8 == 0, vocab % 16 == 0, head_dim 64 or 128. */
int ll_batch_open(int32_t max_batch, int32_t page_tokens, int32_t n_pages, void *pool, size_t pool_bytes);
/* Adds a sequence: prefills tokens[0..n) (host pointer), moves its cache rows into freshly taken
 * pages, stores the first generated token in *first_token and returns the slot (>= 0) the sequence
 * occupies.  LL_E_CAPACITY when no slot or not enough pages are free, or n + 1 > max_seq; those and
 * the argument checks come first and leave everything as it was.  Past them the single-sequence
 * context is replaced, whether or not the prefill then succeeds. */
int32_t ll_batch_add(const int32_t *tokens, int32_t n, int32_t *first_token);
/* One decode step of every sequence in the batch.  out_tokens (host, max_batch entries) receives
 * the new token of every occupied slot and -1 for free slots.  A sequence that crosses a page border
 * takes a page first: LL_E_CAPACITY (nothing ran) when the pool is exhausted or a sequence is at
 * max_seq - remove one and call again.  The host's page lists change only after the step has run. */
int ll_batch_step(int32_t *out_tokens);
/* Ends the sequence in `slot` and returns its pages to the pool. */
int ll_batch_remove(int32_t slot);
/* Closes batched decoding (graphs and host buffers; the pool goes back to the caller). */
int ll_batch_close(void);
/* Test hooks: logits [vocab] of `slot` from the most recent ll_batch_step; override of the token the
 * slot feeds next; k steps back to back timed on the device (milliseconds in *ms_out; the pages the
 * k steps write are taken first, LL_E_CAPACITY and nothing run if the pool cannot supply them). */
int ll_batch_dbg_get_logits(int32_t slot, float *host_out);
int ll_batch_dbg_force_next_token(int32_t slot, int32_t tok);
int ll_batch_dbg_time_steps(int32_t k, float *ms_out);

/* ---- measurement and test hooks (not part of the four-call contract) ---- */

/* Per-length graph mode: out4 = { replays that found their graph in the buffer, captures that
 * blocked a step, captures overlapped with a replay, nanoseconds spent capturing }. */
int ll_dbg_graph_stats(int64_t *out4);

/* How the prefill projection GEMM out[rows][nmat * N] = A[rows][K] W^T deals its work (prompts of
 * more than 32 tokens; host arithmetic only, needs no instance and no GPU):
 * out6 = { rows per tile, row tiles, runs (workgroups per row tile), K slabs per run, K slabs per
 * column tile as the runs count them (padded when runs end at tile borders), most slices any
 * column tile is cut into }.  rows is a prompt bucket (64, 128, 256, 512 or 1024). */
int ll_dbg_gemm_plan(int32_t N, int32_t K, int32_t nmat, int32_t rows, int32_t *out6);
/* Number of slices that hold the partial products of output column col (0 <= col < nmat * N)
 * under that plan, or a negative LL_E_* code. */
int ll_dbg_gemm_slice_count(int32_t N, int32_t K, int32_t nmat, int32_t rows, int32_t col);

/* Logits [vocab] of the most recent prefill/decode step, copied to the host. */
int ll_dbg_get_logits(float *host_out);
/* Residual stream [d_model] before the final norm of the most recent step. */
int ll_dbg_get_hidden(float *host_out);
/* Overrides the token the next decode step will feed (teacher forcing). */
int ll_dbg_force_next_token(int32_t tok);
/* Cached keys (which = 0) or values (which = 1) of one layer, positions
 * [0, n_pos), converted to float, laid out [n_pos][d_model] on the host. */
int ll_dbg_get_kv(int32_t layer, int32_t which, int32_t n_pos, float *host_out);

/* Runs `steps` decode steps eagerly with a hipEvent pair around every kernel
 * launch and returns per-kernel-class mean durations.  The context advances by
 * `steps` tokens.  us_out[LL_KC_COUNT] receives microseconds per launch and
 * launches_out[LL_KC_COUNT] (nullable) the launches per step of each class. */
enum {
  LL_KC_EMBED = 0,
  LL_KC_QKV = 1,     /* RMSNorm + QKV GEMV + RoPE + KV write */
  LL_KC_ATTN = 2,    /* split-K decode attention + combine (+ the O projection where the two share a launch) */
  LL_KC_OPROJ = 3,   /* O GEMV + residual (no launches of its own where it runs inside the attention launch) */
  LL_KC_GATEUP = 4,  /* RMSNorm + gate/up GEMV + SwiGLU */
  LL_KC_DOWN = 5,    /* down GEMV + residual */
  LL_KC_LMHEAD = 6,  /* final RMSNorm + LM-head GEMV + block argmax */
  LL_KC_SAMPLE = 7,  /* final argmax + state advance */
  LL_KC_COUNT = 8
};
int ll_dbg_profile_decode(int32_t steps, float *us_out, int32_t *launches_out);

/* Mean device time of one launch of kernel class `klass` (LL_KC_QKV ..
 * LL_KC_LMHEAD): `reps` passes over all layers, launching only that class back
 * to back (each layer's own weights, so nothing is re-read from cache) between
 * one hipEvent pair on the library's stream.  The position does not advance,
 * but the activation buffers are left undefined: call ll_reset() afterwards. */
int ll_dbg_time_kernel_class(int32_t klass, int32_t reps, float *us_out);

/* One decode step of the persistent kernel with phase tracing: for each of its
 * 5 * n_layers + 1 phases (QKV, attention, O, gate/up, down per layer, then the
 * LM head) workgroup 0 records 100 MHz timestamps, 8 slots per phase: [0] phase
 * entry, [1] input staged, [2] dot products done, [3] results stored, [4] grid
 * barrier passed (service wave); [5] first dot product starts, [6] ends, [7] its
 * next loads issued (compute wave 0); slots a phase does not use stay 0.
 * ticks_out (host) receives [phases][8] values (at most 162 phases are traced);
 * returns the phase count.  The context advances by one token. */
int ll_dbg_trace_decode(uint64_t *ticks_out, int32_t max_phases);

/* Copies `bytes` (a multiple of 16; both DEVICE pointers 16-byte aligned) with
 * the same 16-byte streaming loads the decode GEMVs use, and waits for it.  A
 * calibration kernel of known traffic for hardware counters; works with or
 * without an initialised instance. */
int ll_dbg_stream_copy(void *dst, const void *src, size_t bytes);

/* Debug aid against stale reads: fills every workspace buffer that a step or a prefill is meant to
 * write before it reads (activations, attention partials, logits, selection candidates, the prefill
 * buffers and GEMM slices) with NaN bit patterns; the KV rows, the state and what else carries over
 * between calls stay.  A following step must give the same result as without the call. */
int ll_dbg_poison_scratch(void);

/* Read rate in GB/s of a read-only pass over `bytes` (a multiple of 16) at DEVICE pointer `src`
 * (16-byte aligned) with the decode GEMVs' streaming loads, `reps` passes between one hipEvent pair;
 * `sink` is a DEVICE buffer of at least 4 KiB that the kernel may write a word to.  The measured
 * streaming ceiling of the chip at hand, reported next to the nominal peak; works with or without an
 * initialised instance. */
int ll_dbg_stream_read(const void *src, size_t bytes, int32_t reps, void *sink, float *gbps_out);

/* Device time of `k` decode-step replays measured with one hipEvent pair on
 * the library's stream (milliseconds for all k steps), tokens discarded. */
int ll_dbg_time_decode(int32_t k, float *ms_out);

#ifdef __cplusplus
}
#endif
#endif /* LL_H */
