// Drives the argument and state checks of the C ABI (include/c2t.h) with the library's host code
// built under -fsanitize=address,undefined (tests/test_sanitizers.py; CPU only, no GPU needed: every
// call here is refused on the host before anything is enqueued, or fails cleanly at the launch).
#include "../../include/c2t.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>

#define EXPECT(cond) do { if (!(cond)) { std::printf("abi driver: %s failed at line %d\n", #cond, __LINE__); return 1; } } while (0)

static c2t_config base() {
  c2t_config c;
  std::memset(&c, 0, sizeof c);
  c.batch = 3; c.vocab = 1000; c.max_frontier = 4; c.top_k = 4; c.max_depth = 3; c.budget = 10; c.hidden = 8;
  c.logits_dtype = C2T_BF16; c.beta = 0.5f; c.entropy_top_m = 0; c.rerank = 0;
  return c;
}

int main() {
  size_t need = 0;
  c2t_config c = base();
  EXPECT(c2t_workspace_bytes(&c, &need) == C2T_OK && need > 0);
  EXPECT(c2t_workspace_bytes(nullptr, &need) == C2T_ERR_INVALID_ARG);
  EXPECT(c2t_workspace_bytes(&c, nullptr) == C2T_ERR_INVALID_ARG);
  { c2t_config b = base(); b.batch = 0; EXPECT(c2t_workspace_bytes(&b, &need) == C2T_ERR_INVALID_ARG); }
  { c2t_config b = base(); b.top_k = 65; b.max_frontier = 1; EXPECT(c2t_workspace_bytes(&b, &need) == C2T_ERR_UNSUPPORTED); }
  { c2t_config b = base(); b.beta = 1.0f; EXPECT(c2t_workspace_bytes(&b, &need) == C2T_ERR_INVALID_ARG); }
  { c2t_config b = base(); b.rerank = 1; b.max_depth = 64; b.max_frontier = 32; b.top_k = 32; EXPECT(c2t_workspace_bytes(&b, &need) == C2T_ERR_UNSUPPORTED); }
  for (int rerank = 0; rerank < 2; ++rerank) {
    for (int dtype = 0; dtype < 2; ++dtype) {
      c = base(); c.rerank = rerank; c.logits_dtype = dtype; c.entropy_top_m = dtype ? 0 : 50;
      EXPECT(c2t_workspace_bytes(&c, &need) == C2T_OK);
      // never dereferenced on the host: only its alignment and size are looked at
      void* ws = (void*)(uintptr_t)0x10000000;
      c2t_ctx* x = nullptr;
      EXPECT(c2t_create(&c, nullptr, need, &x) == C2T_ERR_WORKSPACE && !x);
      EXPECT(c2t_create(&c, (char*)ws + 8, need, &x) == C2T_ERR_WORKSPACE);
      EXPECT(c2t_create(&c, ws, need - 1, &x) == C2T_ERR_WORKSPACE);
      EXPECT(c2t_create(&c, ws, need, nullptr) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_create(&c, ws, need, &x) == C2T_OK && x);
      EXPECT(c2t_reset(x, nullptr) == C2T_ERR_STATE);                       // classifier not set
      EXPECT(c2t_expand_layer(x, ws, c.vocab, nullptr) == C2T_ERR_STATE);  // before the first reset
      EXPECT(c2t_expand_layer(x, nullptr, c.vocab, nullptr) == C2T_ERR_INVALID_ARG);
      c2t_tree_out o;
      std::memset(&o, 0, sizeof o);
      EXPECT(c2t_finalize_tree(x, &o, nullptr) == C2T_ERR_INVALID_ARG);    // NULL output buffers
      EXPECT(c2t_finalize_tree(x, nullptr, nullptr) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_finalize_tree_reranked(x, &o, 4, nullptr) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_finalize_tree_reranked_static(x, &o, 4, nullptr) == C2T_ERR_INVALID_ARG);
      o.tokens = o.parent = o.position = o.n_nodes = (int32_t*)ws; o.conf = o.joint_prob = o.entropy = (float*)ws;
      o.mask = (uint8_t*)ws; o.status = (uint32_t*)ws;
      EXPECT(c2t_finalize_tree(x, &o, nullptr) == C2T_ERR_STATE);          // nothing expanded yet
      EXPECT(c2t_finalize_tree_reranked(x, &o, 0, nullptr) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_finalize_tree_reranked(x, &o, C2T_MAX_BUDGET + 1, nullptr) == C2T_ERR_UNSUPPORTED);
      EXPECT(c2t_finalize_tree_reranked(x, &o, 4, nullptr) == C2T_ERR_STATE);
      EXPECT(c2t_finalize_tree_reranked_static(x, &o, 4, nullptr) == C2T_ERR_STATE);
      const int32_t *a = nullptr, *b = nullptr, *d = nullptr;
      EXPECT(c2t_get_frontier(x, &a, &b, &d) == C2T_OK && a && b && d);
      EXPECT(c2t_get_frontier(x, nullptr, nullptr, nullptr) == C2T_OK);
      EXPECT(c2t_get_candidates(x, &a, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == C2T_OK);
      EXPECT(c2t_get_layer_rows(x, &a) == C2T_OK && c2t_get_layer_rows(x, nullptr) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_set_row_splits(x, -1, 0) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_set_row_splits(x, 1 << 20, 1) == C2T_ERR_UNSUPPORTED);
      EXPECT(c2t_set_row_splits(x, 0, 0) == C2T_OK && c2t_set_row_splits(x, 2, 3) == C2T_OK);
      EXPECT(c2t_profile_enable(x, -1) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_profile_sample(x, 0, 0) == C2T_ERR_INVALID_ARG && c2t_profile_sample(x, 4, 4) == C2T_ERR_INVALID_ARG);
      EXPECT(c2t_profile_sample(x, 4, 2) == C2T_OK);
      float ms[4]; int32_t n = 4;
      EXPECT(c2t_profile_read(x, ms, &n) == C2T_OK && n == 0);
      EXPECT(c2t_profile_read(x, nullptr, &n) == C2T_ERR_INVALID_ARG);
      float W1[24] = {0}, b1[8] = {0}, w2[8] = {0};
      EXPECT(c2t_set_classifier(x, nullptr, b1, w2, 0.f, nullptr) == C2T_ERR_INVALID_ARG);
      // with a GPU this enqueues small kernels; without one the launch fails and the call reports it
      const int rc = c2t_set_classifier(x, W1, b1, w2, 0.25f, nullptr);
      EXPECT(rc == C2T_OK || rc == C2T_ERR_HIP);
      c2t_destroy(x);
    }
  }
  c2t_destroy(nullptr);
  EXPECT(c2t_stream_read(nullptr, 16, nullptr, nullptr) == C2T_ERR_INVALID_ARG);
  EXPECT(c2t_stream_read_rows((void*)(uintptr_t)0x1000, 0, 16, 16, (uint32_t*)(uintptr_t)0x1000, nullptr) == C2T_ERR_INVALID_ARG);
  for (int e = 0; e >= -7; --e) EXPECT(c2t_strerror(e) != nullptr && std::strlen(c2t_strerror(e)) > 0);
  std::printf("abi driver ok\n");
  return 0;
}
