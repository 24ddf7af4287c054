// Host-side exercise of libdisco under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only: no kernel
// is launched; every call either fails its host-side validation or only touches host handles).  Linked
// against a build of the library whose HOST code is instrumented.  Exits non-zero on an unexpected result;
// the sanitizers abort on a finding.
#include "../../include/disco.h"
#include "../../include/disco_bench.h"

#include <cstdio>
#include <cstring>
#include <vector>

static int g_failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, disco_last_error()); ++g_failures; } } while (0)

static void* const FAKE = reinterpret_cast<void*>(0x7F0000000000ull);   // 256-byte aligned, never dereferenced

static int make_model(disco_model** out, int family, int n_layers, int d_model, int n_heads, int d_head, int n_kv, int d_ff, int vocab) {
  disco_model_desc d{};
  d.family = family; d.n_layers = n_layers; d.d_model = d_model; d.n_heads = n_heads; d.d_head = d_head; d.n_kv_heads = n_kv;
  d.d_ff = d_ff; d.vocab = vocab; d.max_pos = 64; d.norm_eps = 1e-5f; d.rope_base = 10000.f;
  std::vector<disco_layer_weights> layers(n_layers > 0 ? n_layers : 1);
  for (auto& L : layers) {
    L.norm1_g = static_cast<const float*>(FAKE); L.norm1_b = static_cast<const float*>(FAKE); L.wqkv = FAKE; L.wo = FAKE;
    L.norm2_g = static_cast<const float*>(FAKE); L.norm2_b = static_cast<const float*>(FAKE); L.w_in = FAKE; L.w_out = FAKE;
  }
  disco_model_weights w{};
  w.tok_emb = FAKE; w.tok_emb_stride = d_model; w.pos_emb = FAKE; w.layers = layers.data();
  w.normf_g = static_cast<const float*>(FAKE); w.normf_b = static_cast<const float*>(FAKE); w.wlm = FAKE;
  return disco_model_create(&d, &w, out);      // the library copies the layer array: `layers` may die here
}

int main() {
  disco_model* m = nullptr;
  EXPECT(make_model(&m, DISCO_FAMILY_B, 2, 64, 2, 64, 2, 128, 256) == DISCO_OK && m != nullptr);
  disco_model* bad = nullptr;
  EXPECT(make_model(&bad, 7, 2, 64, 2, 64, 2, 128, 256) == DISCO_EINVAL);
  EXPECT(make_model(&bad, DISCO_FAMILY_A, 2, 65, 2, 64, 2, 128, 256) == DISCO_EINVAL);
  EXPECT(make_model(&bad, DISCO_FAMILY_A, 2, 64, 3, 64, 2, 128, 256) == DISCO_EINVAL);
  EXPECT(make_model(&bad, DISCO_FAMILY_B, 2, 64, 2, 48, 2, 128, 256) == DISCO_EINVAL);
  EXPECT(disco_model_create(nullptr, nullptr, &bad) == DISCO_EINVAL);
  // a model the persistent launch structure accepts (its layer table is built at creation)
  disco_model* big = nullptr;
  EXPECT(make_model(&big, DISCO_FAMILY_B, 3, 768, 12, 64, 12, 3072, 32000) == DISCO_OK);

  // sizes and handles
  EXPECT(disco_kv_bytes(m, 40, 16) > 0 && disco_kv_bytes(m, 0, 16) == 0 && disco_kv_bytes(nullptr, 40, 16) == 0);
  EXPECT(disco_workspace_bytes(m, 16, 100) > 0 && disco_workspace_bytes(m, 17, 100) == 0);
  EXPECT(disco_workspace_bytes(big, 16, 2048) > disco_workspace_bytes(m, 16, 2048));
  EXPECT(disco_prefill_workspace_bytes(m, 100, 128) > disco_workspace_bytes(m, 16, 128));
  EXPECT(disco_prefill_workspace_bytes(m, DISCO_PREFILL_MAX + 1, 128) == 0);
  disco_kv* kv = nullptr;
  const size_t kvb = disco_kv_bytes(m, 40, 16);
  EXPECT(disco_kv_create(m, FAKE, kvb, 40, 16, nullptr, &kv) == DISCO_OK && kv != nullptr);
  EXPECT(disco_kv_len(kv) == 0 && disco_kv_pages_in_use(kv) == 0);
  disco_kv* kv2 = nullptr;
  EXPECT(disco_kv_create(m, FAKE, kvb - 1, 40, 16, nullptr, &kv2) == DISCO_ECAP);
  EXPECT(disco_kv_create(m, FAKE, kvb, 40, 6, nullptr, &kv2) == DISCO_EINVAL);
  EXPECT(disco_kv_create(m, static_cast<char*>(FAKE) + 8, kvb, 40, 16, nullptr, &kv2) == DISCO_EINVAL);
  const int32_t dup[3] = {0, 0, 2};
  EXPECT(disco_kv_create(m, FAKE, kvb, 40, 16, dup, &kv2) == DISCO_EINVAL);           // not a permutation
  const int32_t oob[3] = {0, 1, 3};
  EXPECT(disco_kv_create(m, FAKE, kvb, 40, 16, oob, &kv2) == DISCO_EINVAL);
  EXPECT(disco_kv_rollback(kv, 1) == DISCO_ESTATE && disco_kv_rollback(kv, -1) == DISCO_ESTATE && disco_kv_rollback(kv, 0) == DISCO_OK);
  EXPECT(disco_kv_rollback(nullptr, 0) == DISCO_EINVAL && disco_kv_len(nullptr) == DISCO_EINVAL);
  EXPECT(disco_kv_fill(kv, FAKE, 1000, nullptr) == DISCO_ECAP);

  // the five calls: argument errors are found before any launch
  const size_t wsb = disco_workspace_bytes(m, 16, 40);
  int32_t* tok = static_cast<int32_t*>(FAKE);
  float* logits = static_cast<float*>(FAKE);
  EXPECT(disco_draft_step(m, kv, tok, 0, logits, FAKE, wsb, nullptr, nullptr) == DISCO_ECAP);
  EXPECT(disco_draft_step(m, kv, tok, 17, logits, FAKE, wsb, nullptr, nullptr) == DISCO_ECAP);
  EXPECT(disco_draft_step(m, kv, tok, 1, logits, FAKE, wsb - 1, nullptr, nullptr) == DISCO_EINVAL);
  EXPECT(disco_draft_step(m, kv, tok, 1, nullptr, FAKE, wsb, nullptr, nullptr) == DISCO_EINVAL);
  EXPECT(disco_draft_step(big, kv, tok, 1, logits, FAKE, wsb, nullptr, nullptr) == DISCO_ESTATE);    // cache of another model
  EXPECT(disco_verify(m, kv, tok, 16, nullptr, nullptr, FAKE, wsb, nullptr) == DISCO_EINVAL);
  EXPECT(disco_verify(m, kv, tok, 41, tok, nullptr, FAKE, wsb, nullptr) == DISCO_ECAP);
  disco_clf clf{static_cast<const float*>(FAKE), 0};
  disco_clf_out* co = static_cast<disco_clf_out*>(FAKE);
  EXPECT(disco_classify(&clf, logits, 256, 1.f, .5f, 0, co, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == DISCO_EINVAL);
  EXPECT(disco_classify(nullptr, logits, 70000, 1.f, .5f, 0, co, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == DISCO_EINVAL);
  EXPECT(disco_classify_static(nullptr, logits, 65537, 1.f, .5f, 0, co, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == DISCO_ECAP);
  disco_accept_out* ao = static_cast<disco_accept_out*>(FAKE);
  EXPECT(disco_accept(tok, tok, 0, nullptr, ao, nullptr, nullptr) == DISCO_ECAP);
  EXPECT(disco_accept(tok, nullptr, 4, nullptr, ao, nullptr, nullptr) == DISCO_EINVAL);
  clf.hidden = 64;
  disco_loop_out* lo = static_cast<disco_loop_out*>(FAKE);
  EXPECT(disco_draft_loop(m, kv, &clf, tok, 1, 16, 0, 1.f, .5f, nullptr, logits, co, lo, nullptr, FAKE, wsb, nullptr) == DISCO_ECAP);
  EXPECT(disco_draft_loop(m, kv, &clf, tok, 3, 4, 0, 1.f, .5f, nullptr, logits, co, lo, nullptr, FAKE, wsb, nullptr) == DISCO_EINVAL);
  EXPECT(disco_draft_loop(m, kv, &clf, tok, 1, 4, 5, 1.f, .5f, nullptr, logits, co, lo, nullptr, FAKE, wsb, nullptr) == DISCO_EINVAL);
  disco_loop_opts opts{};
  opts.ppl_threshold = 2.f;
  EXPECT(disco_draft_loop_ex(m, kv, &clf, tok, 1, 4, 0, 1.f, .5f, &opts, logits, co, lo, nullptr, FAKE, wsb, nullptr) == DISCO_EINVAL);
  disco_loop_opts cont{};
  cont.block_offset = 9;
  EXPECT(disco_draft_loop_ex(m, kv, &clf, tok, 1, 8, 0, 1.f, .5f, &cont, logits, co, lo, nullptr, FAKE, wsb, nullptr) == DISCO_ECAP);
  // the iteration driver: everything below is refused before the first launch
  disco_iter_buffers ib{tok, logits, co, lo, lo, tok, ao, ao};
  disco_iter_result ir{};
  const int32_t pending[3] = {1, 2, 3};
  EXPECT(disco_iterate(nullptr, kv, FAKE, wsb, m, kv, FAKE, wsb, &clf, pending, 1, 4, 0, 0, 1.f, .5f, nullptr, &ib, &ir, nullptr) == DISCO_EINVAL);
  EXPECT(disco_iterate(m, kv, FAKE, wsb, m, kv, FAKE, wsb, &clf, pending, 3, 4, 0, 0, 1.f, .5f, nullptr, &ib, &ir, nullptr) == DISCO_EINVAL);
  EXPECT(disco_iterate(m, kv, FAKE, wsb, m, kv, FAKE, wsb, &clf, pending, 1, 16, 0, 0, 1.f, .5f, nullptr, &ib, &ir, nullptr) == DISCO_ECAP);
  EXPECT(disco_iterate(m, kv, FAKE, wsb, m, kv, FAKE, wsb, &clf, pending, 1, 4, 0, -2, 1.f, .5f, nullptr, &ib, &ir, nullptr) == DISCO_EINVAL);
  EXPECT(disco_iterate(m, kv, FAKE, wsb, m, kv, FAKE, wsb, &clf, pending, 1, 4, 0, 0, 1.f, .5f, &cont, &ib, &ir, nullptr) == DISCO_EINVAL);
  disco_iter_buffers ib_bad = ib;
  ib_bad.host_accept_out = nullptr;
  EXPECT(disco_iterate(m, kv, FAKE, wsb, m, kv, FAKE, wsb, &clf, pending, 1, 4, 0, 0, 1.f, .5f, nullptr, &ib_bad, &ir, nullptr) == DISCO_EINVAL);
  EXPECT(disco_prefill_ex(m, kv, tok, 16, nullptr, 8u, FAKE, wsb, nullptr) == DISCO_EINVAL);
  EXPECT(disco_sample(logits, 1, 1001, 1001, 1.f, logits, nullptr, tok, nullptr) == DISCO_EINVAL);
  EXPECT(disco_sample(logits, 1, 1000, 1000, 0.f, logits, nullptr, tok, nullptr) == DISCO_EINVAL);
  EXPECT(disco_accept_sample(tok, 2, nullptr, nullptr, logits, 1000, 1.f, nullptr, logits, ao, nullptr, nullptr) == DISCO_EINVAL);
  EXPECT(disco_clf_train(logits, tok, DISCO_TRAIN_MAX_N + 1, 64, 10, .5f, logits, nullptr, nullptr) == DISCO_ECAP);
  EXPECT(disco_clf_eval(&clf, logits, tok, 10, .5f, nullptr, nullptr, nullptr) == DISCO_EINVAL);
  EXPECT(disco_clf_examples(co, 0, tok, logits, tok, nullptr, nullptr) == DISCO_EINVAL);
  EXPECT(disco_prefill(m, kv, tok, 0, nullptr, FAKE, wsb, nullptr) == DISCO_ECAP);
  EXPECT(disco_pack_weight(FAKE, 17, 32, FAKE, nullptr) == DISCO_EINVAL);
  EXPECT(disco_pack_gate_up(FAKE, FAKE, 16, 33, FAKE, nullptr) == DISCO_EINVAL);

  // host-only arithmetic and switches
  EXPECT(disco_heuristic_next(5, 5, 5, 2, 1, 10) == 7 && disco_heuristic_next(1, 1, 0, 2, 1, 10) == 1);
  EXPECT(disco_heuristic_next(0, 1, 0, 2, 1, 10) == DISCO_EINVAL);
  const int prev = disco_set_launch_mode(1);
  EXPECT(prev == 0 || prev == 1);
  EXPECT(disco_set_launch_mode(prev) == 1 && disco_set_launch_mode(5) == DISCO_EINVAL);
  EXPECT(disco_probe_read_ms() < 0.f);
  EXPECT(std::strlen(disco_last_error()) > 0);

  disco_kv_destroy(kv);
  disco_kv_destroy(nullptr);
  disco_model_destroy(m);
  disco_model_destroy(big);
  disco_model_destroy(nullptr);
  std::printf("%s: %d unexpected results\n", g_failures ? "FAILED" : "ok", g_failures);
  return g_failures ? 1 : 0;
}
