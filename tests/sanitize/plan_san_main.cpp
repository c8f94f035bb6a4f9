// Drives the host-only logic of the runtime (workspace layout, the prefill GEMM's work plan and slice
// map, argument validation in front of every entry point) under AddressSanitizer +
// UndefinedBehaviorSanitizer.  Linked with ll_runtime.hip compiled with host sanitizers; makes no call
// that reaches a GPU, so it runs on a machine without one.
//
//   hipcc -O1 -g -std=c++17 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined -Xarch_host -fno-sanitize-recover=all \
//         paper_2604_23467_amd/csrc/ll_runtime.hip tests/sanitize/plan_san_main.cpp -o plan_san && ./plan_san
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/ll.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d): %s\n", #c, __LINE__, ll_last_error()); return 1; } } while (0)

int main() {
  // ---- workspace layout over a sweep of shapes: never 0 for a valid shape, 256-byte multiples, grows with max_seq
  const int dims[][5] = {{2, 4, 64, 688, 1024}, {1, 2, 128, 344, 777}, {1, 3, 128, 1000, 501}, {32, 32, 128, 11008, 32000},
                         {1, 33, 128, 64, 64}, {2, 2, 64, 136, 33}, {1, 2, 64, 8712, 100}, {80, 64, 128, 28672, 128256}};
  for (const auto& d : dims) {
    size_t prev = 0;
    for (int max_seq : {2, 17, 64, 1024, 1025, 2049, 4096, 65536}) {
      ll_config c{};
      c.n_layers = d[0]; c.n_heads = d[1]; c.head_dim = d[2]; c.d_model = d[1] * d[2]; c.ffn_hidden = d[3]; c.vocab = d[4];
      c.max_seq = max_seq; c.rope_theta = 10000.f; c.rms_eps = 1e-5f; c.flags = 0;
      const size_t b = ll_workspace_bytes(&c);
      CHECK(b > 0 && b % 256 == 0 && b >= prev);
      prev = b;
    }
  }
  {
    ll_config bad{};
    CHECK(ll_workspace_bytes(&bad) == 0 && ll_workspace_bytes(nullptr) == 0);
    ll_weights w{};
    CHECK(ll_init(&bad, &w, nullptr, 0, nullptr) == LL_E_BAD_CONFIG);
    CHECK(ll_init(nullptr, &w, nullptr, 0, nullptr) == LL_E_BAD_CONFIG);
    ll_config ok{2, 256, 4, 64, 688, 1024, 64, 10000.f, 1e-5f, 0};
    CHECK(ll_init(&ok, nullptr, nullptr, 0, nullptr) == LL_E_BAD_ARG);
    std::vector<ll_layer_weights> layers(2);            // null pointers inside: refused before anything is touched
    w.layers = layers.data();
    int dummy = 0;
    w.tok_emb = w.final_norm = w.lm_head = &dummy;
    CHECK(ll_init(&ok, &w, nullptr, 0, nullptr) == LL_E_BAD_ARG);
  }
  // ---- every entry point before ll_init
  int32_t toks[4] = {1, 2, 3, 4}, out[32];
  float f[8];
  int64_t st[4];
  CHECK(ll_prefill(toks, 4) == LL_E_NOT_INIT && ll_prefill_static(toks, 4) == LL_E_NOT_INIT);
  CHECK(ll_decode_step() == LL_E_NOT_INIT && ll_decode_n(2, out) == LL_E_NOT_INIT && ll_reset() == LL_E_NOT_INIT);
  CHECK(ll_shutdown() == LL_E_NOT_INIT && ll_max_prompt() == LL_E_NOT_INIT && ll_position() == LL_E_NOT_INIT);
  CHECK(ll_decode_mode() == LL_E_NOT_INIT && ll_set_sampling(1.f, 0, 1.f, 0) == LL_E_NOT_INIT);
  CHECK(ll_set_sampling(-1.f, 0, 1.f, 0) == LL_E_BAD_ARG && ll_set_sampling(1.f, -1, 1.f, 0) == LL_E_BAD_ARG);
  CHECK(ll_set_sampling(1.f, 0, 0.f, 0) == LL_E_BAD_ARG);
  CHECK(ll_batch_pool_bytes(16, 8) == 0 && ll_batch_open(2, 8, 4, &out, 1) == LL_E_NOT_INIT);
  CHECK(ll_batch_add(toks, 4, out) == LL_E_NOT_INIT && ll_batch_step(out) == LL_E_NOT_INIT);
  CHECK(ll_batch_remove(0) == LL_E_NOT_INIT && ll_batch_close() == LL_E_NOT_INIT);
  CHECK(ll_batch_dbg_get_logits(0, f) == LL_E_NOT_INIT && ll_batch_dbg_force_next_token(0, 1) == LL_E_NOT_INIT);
  CHECK(ll_batch_dbg_time_steps(1, f) == LL_E_NOT_INIT && ll_dbg_graph_stats(st) == LL_E_NOT_INIT);
  CHECK(ll_dbg_get_logits(f) == LL_E_NOT_INIT && ll_dbg_get_hidden(f) == LL_E_NOT_INIT);
  CHECK(ll_dbg_force_next_token(1) == LL_E_NOT_INIT && ll_dbg_get_kv(0, 0, 1, f) == LL_E_NOT_INIT);
  CHECK(ll_dbg_profile_decode(1, f, out) == LL_E_NOT_INIT && ll_dbg_time_kernel_class(LL_KC_QKV, 1, f) == LL_E_NOT_INIT);
  CHECK(ll_dbg_trace_decode(nullptr, 0) == LL_E_NOT_INIT && ll_dbg_time_decode(1, f) == LL_E_NOT_INIT);
  CHECK(ll_dbg_stream_copy(nullptr, nullptr, 16) == LL_E_BAD_ARG && ll_dbg_stream_copy(out, toks, 15) == LL_E_BAD_ARG);
  CHECK(ll_dbg_stream_read(nullptr, 16, 1, out, f) == LL_E_BAD_ARG && ll_dbg_stream_read(toks, 16, 0, out, f) == LL_E_BAD_ARG);
  CHECK(std::strlen(ll_last_error()) > 0);

  // ---- the prefill GEMM's plan: every 64-wide K slab of every column tile is covered exactly once by the
  //      runs, and slice counts agree with the plan
  int32_t p[6];
  CHECK(ll_dbg_gemm_plan(0, 64, 1, 64, p) == LL_E_BAD_ARG && ll_dbg_gemm_plan(64, 64, 4, 64, p) == LL_E_BAD_ARG);
  CHECK(ll_dbg_gemm_plan(64, 64, 1, 65, p) == LL_E_BAD_ARG && ll_dbg_gemm_plan(64, 64, 1, 64, nullptr) == LL_E_BAD_ARG);
  CHECK(ll_dbg_gemm_slice_count(64, 64, 1, 64, 64) == LL_E_BAD_ARG && ll_dbg_gemm_slice_count(64, 64, 1, 64, -1) == LL_E_BAD_ARG);
  long plans = 0;
  for (int rows : {64, 128, 256, 512, 1024})
    for (int nmat = 1; nmat <= 3; ++nmat)
      for (int N : {8, 136, 256, 344, 688, 1000, 4096, 4224, 11008, 28672})
        for (int K : {8, 64, 136, 256, 384, 1000, 4096, 8712, 11008, 28672}) {
          CHECK(ll_dbg_gemm_plan(N, K, nmat, rows, p) == LL_OK);
          const int row_tile = p[0], row_tiles = p[1], runs = p[2], quota = p[3], tile_slabs = p[4], max_slices = p[5];
          CHECK((row_tile == 64 || row_tile == 128 || row_tile == 256) && row_tile * row_tiles == rows && runs >= 1 && quota >= 1);
          const int slabs = (K + 63) / 64, tiles = (N + 255) / 256 * nmat;
          CHECK(tile_slabs >= slabs && max_slices >= 1);
          CHECK((long)runs * quota >= (long)tiles * tile_slabs);        // the runs reach the end of the last tile
          CHECK((long)(runs - 1) * quota < (long)tiles * tile_slabs);   // and none of them is empty
          int most = 0;
          for (int col = 0; col < nmat * N; col += 97) {
            const int sc = ll_dbg_gemm_slice_count(N, K, nmat, rows, col);
            CHECK(sc >= 1 && sc <= max_slices);
            // pieces of the tile that owns this column, counted from the plan itself
            const int z = col / N, t = z * ((N + 255) / 256) + (col - z * N) / 256;
            const long u0 = (long)t * tile_slabs, u1 = u0 + tile_slabs - 1;
            CHECK(sc == (int)(u1 / quota - u0 / quota + 1));
            most = sc > most ? sc : most;
          }
          ++plans;
        }
  std::printf("runtime host-logic sanitizer run ok (%ld GEMM plans)\n", plans);
  return 0;
}
