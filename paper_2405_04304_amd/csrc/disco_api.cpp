// C boundary of the DISCO hot path: handles, host-side validation, workspace carving and the launch
// sequences of a draft step, a verification forward and the fused draft loop.  Every check runs on
// the host before the first launch, so argument errors are reported without touching the GPU.
#include "../../include/disco.h"
#include "../../include/disco_bench.h"
#include "disco_internal.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace disco;

namespace {

thread_local char g_err[512] = "";

// measurement probe (disco_bench.h)
std::mutex g_probe_mu;
int g_probe_layer = -1;
bool g_probe_taken = false;
hipEvent_t g_probe_ev[2] = {nullptr, nullptr};

// Records event `which` (0 before, 1 after the bracketed launch) if the probe is set on `layer`.
hipError_t probe_record(int layer, int which, hipStream_t s) {
  std::lock_guard<std::mutex> lock(g_probe_mu);
  if (layer != g_probe_layer || g_probe_ev[which] == nullptr) return hipSuccess;
  const hipError_t e = hipEventRecord(g_probe_ev[which], s);
  if (e == hipSuccess && which == 1) g_probe_taken = true;
  return e;
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(DISCO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

struct disco_model {
  disco_model_desc d;
  disco_model_weights w;
  std::vector<disco_layer_weights> layers;
  int d_q, d_kv, d_qkv;
  // one launch per forward (RMSNorm / rotary / SwiGLU family with shapes the persistent kernel tiles)
  bool persist_ok, persist_big;
  std::vector<FwdLayer> fwd_layers;      // copied into every workspace by disco_workspace_init
  int loop_steps;                        // draft-loop steps the workspace holds panel versions for (1: none beyond one forward)
};

struct disco_kv {
  const disco_model* model;
  bf16_t* pages;
  int32_t* dev_page_table;   // inside the caller's buffer, or nullptr for the identity order
  float* dev_rope;           // inside the caller's buffer: [capacity][d_head / 2][cos, sin] (family B), else nullptr
  bool rope_ready;           // the table is written by the first forward that uses the cache, on its stream
  int page_tokens, n_pages, capacity, len;
  size_t layer_stride;       // elements between layers
};

namespace {

struct Ws {
  float* h; float* q; bf16_t* xn; bf16_t* xattn; bf16_t* xact; float* part; float* gpart; float* logits;
  float* ssq; int* gemm_counters; int* attn_counters; int n_counters; float* clf_scratch;
  uint32_t* gate; int32_t* sl_count; int32_t* tok_next;
  int* head_ready; unsigned* abort_word;     // fused QKV + attention launch: per-head counters, sticky failure flag
  // LayerNorm family: per-tile sums beside ssq, and the correction vectors of the deferred norms (W . g, W . b) of
  // every matrix that reads a normalised row: per layer [wg | wb] of the QKV matrix (2 d_qkv floats) and of the MLP
  // input matrix (2 d_ff), then the LM head's (2 vocab); written by disco_workspace_init
  float* sum; float* ln_vec; size_t ln_layer_stride;
  // persistent forward: panel versions (a fresh address per phase and step), the layer table, barrier words
  bf16_t* xn_v; bf16_t* xattn_v; bf16_t* xact_v; float* q_v; size_t xn_stride, xattn_stride, xact_stride;
  FwdLayer* fwd_layers; unsigned* bar;
  size_t total;
};

// Launch structure (disco_set_launch_mode): 0 = one launch per phase, the QKV projection and the attention of a layer
// in one launch where the model allows it (default), 1 = one cooperative launch per forward / draft loop, 2 = one
// launch per phase, nothing fused.  DISCO_PERSISTENT=1 in the environment selects 1 at load time.
int g_launch_mode = [] { const char* e = getenv("DISCO_PERSISTENT"); return (e && e[0] == '1') ? 1 : 0; }();
bool persistent_enabled() { return g_launch_mode == 1; }
int g_wait_limit = 1 << 20;     // polls before a wait inside a launch gives up (disco_set_wait_limit)

// Carve the workspace; with base == nullptr only the total is meaningful.
Ws carve(const disco_model* m, int max_block, int max_ctx, void* base) {
  (void)max_block;  // buffers are sized for DISCO_MAX_BLOCK tokens
  const disco_model_desc& d = m->d;
  char* p = static_cast<char*>(base);
  size_t off = 0;
  auto take = [&](size_t bytes) { void* r = p ? p + off : nullptr; off += round_up(bytes, 256); return r; };
  Ws w;
  w.h = static_cast<float*>(take(sizeof(float) * 16 * d.d_model));
  w.q = static_cast<float*>(take(sizeof(float) * 16 * m->d_q));
  w.xn = static_cast<bf16_t*>(take(sizeof(bf16_t) * 2 * 16 * d.d_model));
  w.xattn = static_cast<bf16_t*>(take(sizeof(bf16_t) * 2 * 16 * m->d_q));
  w.xact = static_cast<bf16_t*>(take(sizeof(bf16_t) * 2 * 16 * d.d_ff));
  // partial tiles and ticket counters of split row groups: sized for the widest matrix of the model
  int max_rows = d.vocab;
  if (m->d_qkv > max_rows) max_rows = m->d_qkv;
  if (2 * d.d_ff > max_rows) max_rows = 2 * d.d_ff;
  if (d.d_model > max_rows) max_rows = d.d_model;
  const int max_tiles = max_rows / 16;
  w.gpart = static_cast<float*>(take(sizeof(float) * GEMM_MAX_SPLIT * 256 * (size_t)max_tiles));
  w.logits = static_cast<float*>(take(sizeof(float) * 16 * (size_t)d.vocab));
  w.ssq = static_cast<float*>(take(sizeof(float) * 16 * (size_t)(d.d_model / 16)));
  w.sum = nullptr; w.ln_vec = nullptr; w.ln_layer_stride = 2 * ((size_t)m->d_qkv + d.d_ff);
  if (d.family == DISCO_FAMILY_A) {
    w.sum = static_cast<float*>(take(sizeof(float) * 16 * (size_t)(d.d_model / 16)));
    w.ln_vec = static_cast<float*>(take(sizeof(float) * (w.ln_layer_stride * d.n_layers + 2 * (size_t)d.vocab)));
  }
  w.n_counters = max_tiles + d.n_heads;
  w.gemm_counters = static_cast<int*>(take(sizeof(int) * (size_t)w.n_counters));
  w.attn_counters = w.gemm_counters ? w.gemm_counters + max_tiles : nullptr;
  w.clf_scratch = static_cast<float*>(take(CLASSIFY_SCRATCH_BYTES));
  w.gate = static_cast<uint32_t*>(take(256));
  w.sl_count = reinterpret_cast<int32_t*>(w.gate ? w.gate + 16 : nullptr);
  w.tok_next = reinterpret_cast<int32_t*>(w.gate ? w.gate + 32 : nullptr);
  w.abort_word = w.gate ? w.gate + 48 : nullptr;
  w.head_ready = static_cast<int*>(take(sizeof(int) * QKV_ATTN_READY_SLOT * (size_t)d.n_heads));
  w.xn_stride = (size_t)2 * 16 * d.d_model + 2 * (size_t)d.d_model;      // two panels + d floats of sums of squares
  w.xattn_stride = (size_t)2 * 16 * m->d_q; w.xact_stride = (size_t)2 * 16 * d.d_ff;
  w.xn_v = w.xattn_v = w.xact_v = nullptr; w.q_v = nullptr; w.fwd_layers = nullptr; w.bar = nullptr;
  if (m->persist_ok) {
    const size_t steps = (size_t)m->loop_steps, L = (size_t)d.n_layers;
    w.xn_v = static_cast<bf16_t*>(take(sizeof(bf16_t) * w.xn_stride * (2 * L + 1) * steps));
    w.xattn_v = static_cast<bf16_t*>(take(sizeof(bf16_t) * w.xattn_stride * L * steps));
    w.xact_v = static_cast<bf16_t*>(take(sizeof(bf16_t) * w.xact_stride * L * steps));
    w.q_v = static_cast<float*>(take(sizeof(float) * 16 * m->d_q * L * steps));
    w.fwd_layers = static_cast<FwdLayer*>(take(sizeof(FwdLayer) * L));
    w.bar = static_cast<unsigned*>(take(sizeof(unsigned) * FWD_BAR_WORDS));
  }
  // the only buffer whose size depends on max_ctx goes last, so that every other offset (the ticket
  // counters above all) is the same for every call on this workspace
  const int n_splits = (max_ctx + DISCO_MAX_BLOCK + ATTN_SPLIT_LEN - 1) / ATTN_SPLIT_LEN;
  w.part = static_cast<float*>(take(sizeof(float) * (size_t)d.n_heads * n_splits * 16 * (d.d_head + 2)));
  w.total = off;
  return w;
}

int check_forward_args(const disco_model* m, const disco_kv* kv, const int32_t* tokens, int n,
                       const void* ws, size_t ws_bytes) {
  if (!m || !kv || !tokens || !ws) return fail(DISCO_EINVAL, "null argument");
  if (kv->model != m) return fail(DISCO_ESTATE, "KV cache belongs to another model");
  if (n < 1 || n > DISCO_MAX_BLOCK) return fail(DISCO_ECAP, "block of %d tokens outside [1, %d]", n, DISCO_MAX_BLOCK);
  if (kv->len + n > kv->capacity) return fail(DISCO_ECAP, "KV capacity %d exceeded (len %d + %d)", kv->capacity, kv->len, n);
  if (m->d.family == DISCO_FAMILY_A && kv->len + n > m->d.max_pos)
    return fail(DISCO_ECAP, "position table of %d rows exceeded", m->d.max_pos);
  if (!aligned(tokens, 4) || !aligned(ws, 256)) return fail(DISCO_EINVAL, "misaligned pointer");
  const size_t need = carve(m, n, kv->len + n, nullptr).total;
  if (ws_bytes < need) return fail(DISCO_EINVAL, "workspace of %zu bytes, %zu needed", ws_bytes, need);
  return DISCO_OK;
}

#define HIP_TRY(expr, what) do { hipError_t e__ = (expr); if (e__ != hipSuccess) return hip_fail(e__, what); } while (0)

// The model / cache / workspace part of a persistent launch's arguments.
FwdArgs forward_args(const disco_model* m, const disco_kv* kv, const Ws& ws) {
  const disco_model_desc& d = m->d;
  FwdArgs f{};
  f.n_layers = d.n_layers; f.d = d.d_model; f.d_q = m->d_q; f.d_qkv = m->d_qkv; f.d_ff = d.d_ff; f.nq = d.n_heads;
  f.nkv = d.n_kv_heads; f.dh = d.d_head; f.vocab = d.vocab; f.eps = d.norm_eps; f.attn_scale = 1.0f / sqrtf((float)d.d_head);
  f.layers = ws.fwd_layers; f.normf_g = m->w.normf_g; f.wlm = static_cast<const bf16_t*>(m->w.wlm);
  f.tok_emb = static_cast<const bf16_t*>(m->w.tok_emb); f.tok_stride = m->w.tok_emb_stride;
  f.h = ws.h; f.q = ws.q_v; f.xn = ws.xn_v; f.xattn = ws.xattn_v; f.xact = ws.xact_v;
  f.xn_stride = ws.xn_stride; f.xattn_stride = ws.xattn_stride; f.xact_stride = ws.xact_stride;
  f.part = ws.part; f.planes = ws.gpart; f.gemm_counters = ws.gemm_counters; f.attn_counters = ws.attn_counters;
  f.kv_pages = kv->pages; f.kv_layer_stride = kv->layer_stride; f.page_table = kv->dev_page_table;
  f.page_tokens = kv->page_tokens; f.rope = kv->dev_rope;
  f.bar = ws.bar; f.n_steps = 1;
  return f;
}

// One forward of n tokens at positions kv->len ..: the shared body of draft step and verification.
// logits_out: [vocab] of the last token (only_last) or [n x vocab].
int forward_block(const disco_model* m, disco_kv* kv, const int32_t* dev_tokens, int n, float* logits_out,
                  bool only_last, const Ws& ws, const uint32_t* gate, hipStream_t s) {
  const disco_model_desc& d = m->d;
  const int pos0 = kv->len;
  const bool fam_a = d.family == DISCO_FAMILY_A;
  if (kv->dev_rope && !kv->rope_ready) {
    HIP_TRY(launch_rope_fill(kv->dev_rope, kv->capacity, d.d_head, d.rope_base, s), "rotary table launch");
    kv->rope_ready = true;
  }

  const int n_tiles = d.d_model / 16;            // one sum-of-squares slot per 16 columns of h
  if (m->persist_ok && ws.bar != nullptr && gate == nullptr && persistent_enabled()) {
    // embedding launch (residual rows, first panel version, sums of squares), then the whole forward in one launch
    NormArgs n0{};
    n0.h = ws.h; n0.d = d.d_model; n0.M = n; n0.eps = d.norm_eps; n0.Xout = ws.xn_v; n0.pos0 = pos0; n0.vocab = d.vocab;
    n0.max_pos = d.max_pos; n0.ssq_out = reinterpret_cast<float*>(ws.xn_v + (size_t)32 * d.d_model); n0.n_ssq_out = n_tiles;
    n0.g = m->layers[0].norm1_g;
    n0.tokens = dev_tokens; n0.tok_emb = static_cast<const bf16_t*>(m->w.tok_emb); n0.tok_stride = m->w.tok_emb_stride;
    HIP_TRY(launch_norm(n0, s), "embedding launch");
    HIP_TRY(launch_zero(reinterpret_cast<int*>(ws.bar), FWD_BAR_WORDS, s), "barrier reset launch");
    FwdArgs f = forward_args(m, kv, ws);
    f.M = n; f.pos0 = pos0; f.logits = logits_out; f.only_last = only_last ? 1 : 0;
    HIP_TRY(launch_forward(f, m->persist_big, false, s), "forward launch");
    kv->len = pos0 + n;
    return DISCO_OK;
  }
  const int split_o = gemm_split_for(d.d_model, m->d_q / 32, n), split_dn = gemm_split_for(d.d_model, d.d_ff / 32, n);

  NormArgs na{};
  na.h = ws.h; na.d = d.d_model; na.M = n; na.layernorm = fam_a; na.eps = d.norm_eps;
  na.Xout = ws.xn; na.gate = gate; na.pos0 = pos0; na.vocab = d.vocab; na.max_pos = d.max_pos;
  na.ssq_out = ws.ssq; na.n_ssq_out = n_tiles;                   // every norm is deferred to the consumer GEMM
  if (fam_a) na.sum_out = ws.sum;

  // Every GEMM that reads a normalised row reads gain * h panels and applies the norm in its epilogue: 1 / rms
  // (family B), or rstd * (y - mean * W.g) + W.b with the vectors that disco_workspace_init left (family A);
  // the residual-update GEMMs write those panels and the per-tile sums.
  auto normed_input = [&](GemmArgs& g, const float* ln_vec, int n_rows) {
    g.X = ws.xn; g.KT = d.d_model / 32;
    g.ssq = ws.ssq; g.n_ssq = n_tiles; g.d_in = d.d_model; g.eps = d.norm_eps;
    if (fam_a) { g.sum = ws.sum; g.wg = ln_vec; g.wb = ln_vec + n_rows; }
  };
  auto residual_update = [&](GemmArgs& g, const void* w, const bf16_t* x, int k, int split, const float* next_gain) {
    g.M = n; g.gate = gate; g.W = static_cast<const bf16_t*>(w); g.X = x; g.KT = k / 32;
    g.n_rows = d.d_model; g.h = ws.h; g.ld_out = d.d_model; g.only_row = -1;
    g.n_split = split; g.planes = ws.gpart; g.counters = ws.gemm_counters;
    g.Xout = ws.xn; g.KT_out = d.d_model / 32; g.gain = next_gain; g.ssq_out = ws.ssq; g.n_ssq_out = n_tiles;
    if (fam_a) g.sum_out = ws.sum;
  };

  {
    NormArgs n0 = na;
    n0.g = m->layers[0].norm1_g; n0.b = m->layers[0].norm1_b;
    n0.tokens = dev_tokens; n0.tok_emb = static_cast<const bf16_t*>(m->w.tok_emb);
    n0.tok_stride = m->w.tok_emb_stride; n0.pos_emb = static_cast<const bf16_t*>(m->w.pos_emb);
    HIP_TRY(launch_norm(n0, s), "embedding launch");
  }
  for (int l = 0; l < d.n_layers; ++l) {
    const disco_layer_weights& L = m->layers[l];
    const bool last = (l + 1 == d.n_layers);
    const float* next_g = last ? m->w.normf_g : m->layers[l + 1].norm1_g;

    GemmArgs g{};
    g.M = n; g.gate = gate; g.planes = ws.gpart; g.counters = ws.gemm_counters;
    // QKV projection, rotary, KV append
    const float* ln_l = fam_a ? ws.ln_vec + ws.ln_layer_stride * l : nullptr;
    g.W = static_cast<const bf16_t*>(L.wqkv); normed_input(g, ln_l, m->d_qkv); g.n_rows = m->d_qkv;
    g.grp = d.d_head / 32; g.q = ws.q; g.ldq = m->d_q; g.nq = d.n_heads; g.nkv = d.n_kv_heads; g.dh = d.d_head;
    g.pos0 = pos0; g.rope_tab = kv->dev_rope;
    g.kv_layer = kv->pages + (size_t)l * kv->layer_stride; g.page_table = kv->dev_page_table;
    g.page_tokens = kv->page_tokens;
    AttnArgs at{};
    at.q = ws.q; at.ldq = m->d_q; at.kv_layer = g.kv_layer; at.page_table = kv->dev_page_table;
    at.page_tokens = kv->page_tokens; at.nq = d.n_heads; at.nkv = d.n_kv_heads; at.dh = d.d_head; at.M = n;
    at.pos0 = pos0; at.scale = 1.0f / sqrtf((float)d.d_head); at.part = ws.part;
    at.split_len = attn_split_len(pos0 + n); at.n_splits = (pos0 + n + at.split_len - 1) / at.split_len;
    at.Xout = ws.xattn; at.counters = ws.attn_counters; at.gate = gate;
    bool fused = false;
    // (a bounded wait inside the fused launch that runs out sets the workspace's abort word: the LM head then stores
    // NaN logits, the arg-max and loop-finish kernels report -1)
    if (g_launch_mode != 2)
      HIP_TRY(launch_qkv_attn(g, at, ws.head_ready, ws.abort_word, g_wait_limit, &fused, s), "qkv + attention launch");
    if (!fused) {
      HIP_TRY(launch_gemm(g, EPI_QKV, s), "qkv launch");
      HIP_TRY(launch_attn(at, s), "attention launch");
    }

    GemmArgs o{};
    residual_update(o, L.wo, ws.xattn, m->d_q, split_o, L.norm2_g);
    HIP_TRY(launch_gemm(o, EPI_PARTIAL, s), "o-proj launch");

    GemmArgs u{};
    u.M = n; u.gate = gate; u.planes = ws.gpart; u.counters = ws.gemm_counters;
    u.W = static_cast<const bf16_t*>(L.w_in); normed_input(u, fam_a ? ln_l + 2 * (size_t)m->d_qkv : nullptr, d.d_ff);
    u.n_rows = fam_a ? d.d_ff : 2 * d.d_ff; u.grp = 1; u.Xout = ws.xact; u.KT_out = d.d_ff / 32;
    HIP_TRY(probe_record(l, 0, s), "probe event");
    HIP_TRY(launch_gemm(u, fam_a ? EPI_GELU : EPI_SWIGLU, s), "mlp-in launch");
    HIP_TRY(probe_record(l, 1, s), "probe event");

    GemmArgs dn{};
    residual_update(dn, L.w_out, ws.xact, d.d_ff, split_dn, next_g);
    HIP_TRY(launch_gemm(dn, EPI_PARTIAL, s), "mlp-out launch");

  }
  GemmArgs lm{};
  lm.M = n; lm.gate = gate; lm.planes = ws.gpart; lm.counters = ws.gemm_counters;
  lm.W = static_cast<const bf16_t*>(m->w.wlm); normed_input(lm, fam_a ? ws.ln_vec + ws.ln_layer_stride * d.n_layers : nullptr, d.vocab);
  lm.n_rows = d.vocab; lm.out = logits_out; lm.ld_out = d.vocab; lm.only_row = only_last ? n - 1 : -1;
  lm.abort_word = ws.abort_word;
  HIP_TRY(launch_gemm(lm, EPI_STORE, s), "lm-head launch");
  kv->len = pos0 + n;
  return DISCO_OK;
}

// ---- dense prompt pass -----------------------------------------------------------------------------

// Workspace of the prompt pass: the ordinary workspace first (its ticket counters and split planes serve
// the LM head of the last token), then the buffers of n_groups groups of 16 tokens.
struct PfWs {
  Ws base;
  float* h; float* q; bf16_t* xn; bf16_t* xattn; bf16_t* xact; float* ssq; float* rstd;
  size_t total;
};

PfWs carve_prefill(const disco_model* m, int n_groups, int max_ctx, void* base) {
  const disco_model_desc& d = m->d;
  PfWs w;
  w.base = carve(m, DISCO_MAX_BLOCK, max_ctx, base);
  char* p = static_cast<char*>(base);
  size_t off = w.base.total;
  auto take = [&](size_t bytes) { void* r = p ? p + off : nullptr; off += round_up(bytes, 256); return r; };
  const size_t rows = (size_t)16 * n_groups;
  w.h = static_cast<float*>(take(sizeof(float) * rows * d.d_model));
  w.q = static_cast<float*>(take(sizeof(float) * rows * m->d_q));
  w.xn = static_cast<bf16_t*>(take(sizeof(bf16_t) * 2 * rows * d.d_model));
  w.xattn = static_cast<bf16_t*>(take(sizeof(bf16_t) * 2 * rows * m->d_q));
  w.xact = static_cast<bf16_t*>(take(sizeof(bf16_t) * 2 * rows * d.d_ff));
  w.ssq = static_cast<float*>(take(sizeof(float) * rows * (size_t)(d.d_model / 16)));
  w.rstd = static_cast<float*>(take(sizeof(float) * rows));
  w.total = off;
  return w;
}

}  // namespace

extern "C" {

size_t disco_prefill_workspace_bytes(const disco_model* m, int n_tokens, int max_ctx) {
  if (!m || n_tokens < 1 || n_tokens > DISCO_PREFILL_MAX || max_ctx < 0) return 0;
  return carve_prefill(m, (n_tokens + 15) / 16, max_ctx, nullptr).total;
}

int disco_prefill(const disco_model* m, disco_kv* kv, const int32_t* dev_tokens, int n_tokens, float* dev_logits_last,
                  void* dev_ws, size_t ws_bytes, disco_stream s) {
  return disco_prefill_ex(m, kv, dev_tokens, n_tokens, dev_logits_last, 0u, dev_ws, ws_bytes, s);
}

int disco_prefill_ex(const disco_model* m, disco_kv* kv, const int32_t* dev_tokens, int n_tokens, float* dev_logits_last,
                     unsigned flags, void* dev_ws, size_t ws_bytes, disco_stream s) {
  if (!m || !kv || !dev_tokens || !dev_ws) return fail(DISCO_EINVAL, "null argument");
  if (flags & ~(unsigned)DISCO_PREFILL_BF16_ACTIVATIONS) return fail(DISCO_EINVAL, "unknown prompt-pass flag 0x%x", flags);
  const int hi_only = (flags & DISCO_PREFILL_BF16_ACTIVATIONS) ? 1 : 0;
  if (kv->model != m) return fail(DISCO_ESTATE, "KV cache belongs to another model");
  const disco_model_desc& d = m->d;
  const bool fam_a = d.family == DISCO_FAMILY_A;
  if (n_tokens < 1 || n_tokens > DISCO_PREFILL_MAX) return fail(DISCO_ECAP, "prompt of %d tokens outside [1, %d]", n_tokens, DISCO_PREFILL_MAX);
  const int G = (n_tokens + 15) / 16, pos0 = kv->len;
  if (pos0 + 16 * G > kv->capacity)
    return fail(DISCO_ECAP, "KV capacity %d below len %d + %d (the prompt rounded up to groups of 16)", kv->capacity, pos0, 16 * G);
  if (fam_a && pos0 + n_tokens > d.max_pos) return fail(DISCO_ECAP, "position table of %d rows exceeded", d.max_pos);
  if (!aligned(dev_tokens, 4) || !aligned(dev_ws, 256) || !aligned(dev_logits_last, 16)) return fail(DISCO_EINVAL, "misaligned pointer");
  const int n_in = fam_a ? d.d_ff : 2 * d.d_ff;      // rows of the MLP input matrix
  if (m->d_qkv % 64 || n_in % 64) return fail(DISCO_EINVAL, "projection widths must be multiples of 64 for the prompt pass");
  const size_t need = carve_prefill(m, G, pos0 + 16 * G, nullptr).total;
  if (ws_bytes < need) return fail(DISCO_EINVAL, "workspace of %zu bytes, %zu needed", ws_bytes, need);
  const PfWs ws = carve_prefill(m, G, pos0 + 16 * G, dev_ws);
  hipStream_t st = static_cast<hipStream_t>(s);
  if (kv->dev_rope && !kv->rope_ready) {
    HIP_TRY(launch_rope_fill(kv->dev_rope, kv->capacity, d.d_head, d.rope_base, st), "rotary table launch");
    kv->rope_ready = true;
  }
  const int n_tiles = d.d_model / 16;
  const size_t xs_d = (size_t)32 * d.d_model, xs_q = (size_t)32 * m->d_q, xs_ff = (size_t)32 * d.d_ff;

  // Family B defers every RMSNorm into the consumer GEMM (gain * h panels and per-tile sums of squares
  // from the producer, one 1 / rms per row from k_rstd_groups); family A runs LayerNorm launches.
  NormArgs na{};
  na.h = ws.h; na.d = d.d_model; na.M = 16; na.n_groups = G; na.layernorm = fam_a; na.eps = d.norm_eps;
  na.Xout = ws.xn; na.pos0 = pos0; na.vocab = d.vocab; na.max_pos = d.max_pos;
  if (!fam_a) { na.ssq_out = ws.ssq; na.n_ssq_out = n_tiles; }
  {
    NormArgs n0 = na;
    n0.g = m->layers[0].norm1_g; n0.b = m->layers[0].norm1_b;
    n0.tokens = dev_tokens; n0.n_tok = n_tokens; n0.tok_emb = static_cast<const bf16_t*>(m->w.tok_emb);
    n0.tok_stride = m->w.tok_emb_stride; n0.pos_emb = static_cast<const bf16_t*>(m->w.pos_emb);
    HIP_TRY(launch_norm(n0, st), "embedding launch");
  }
  auto dense = [&](const void* w, const bf16_t* x, size_t xs, int k, int n_rows) {
    DenseArgs a{};
    a.g.M = 16; a.g.W = static_cast<const bf16_t*>(w); a.g.X = x; a.g.KT = k / 32; a.g.n_rows = n_rows; a.g.grp = 1;
    a.g.only_row = -1; a.n_groups = G; a.xs = xs; a.hi_only = hi_only;
    return a;
  };
  auto residual_update = [&](DenseArgs& a, const float* next_gain) {
    a.g.h = ws.h; a.hs = (size_t)16 * d.d_model; a.g.ld_out = d.d_model;
    if (!fam_a) {
      a.g.gain = next_gain; a.g.Xout = ws.xn; a.xouts = xs_d; a.g.KT_out = d.d_model / 32;
      a.g.ssq_out = ws.ssq; a.ssq_outs = (size_t)n_tiles * 16;
    }
  };
  for (int l = 0; l < d.n_layers; ++l) {
    const disco_layer_weights& L = m->layers[l];
    const bool last = (l + 1 == d.n_layers);
    const float* next_g = last ? m->w.normf_g : m->layers[l + 1].norm1_g;
    const float* next_b = last ? m->w.normf_b : m->layers[l + 1].norm1_b;
    bf16_t* kv_layer = kv->pages + (size_t)l * kv->layer_stride;

    if (!fam_a) HIP_TRY(launch_rstd_groups(ws.ssq, n_tiles, d.d_model, d.norm_eps, ws.rstd, G, st), "rstd launch");
    DenseArgs qa = dense(L.wqkv, ws.xn, xs_d, d.d_model, m->d_qkv);
    qa.rstd = fam_a ? nullptr : ws.rstd; qa.g.grp = d.d_head / 32; qa.g.q = ws.q; qa.qs = (size_t)16 * m->d_q; qa.g.ldq = m->d_q;
    qa.g.nq = d.n_heads; qa.g.nkv = d.n_kv_heads; qa.g.dh = d.d_head; qa.g.pos0 = pos0; qa.g.rope_tab = kv->dev_rope;
    qa.g.kv_layer = kv_layer; qa.g.page_table = kv->dev_page_table; qa.g.page_tokens = kv->page_tokens;
    HIP_TRY(launch_gemm_dense(qa, EPI_QKV, st), "qkv launch");

    AttnArgs at{};
    at.q = ws.q; at.ldq = m->d_q; at.kv_layer = kv_layer; at.page_table = kv->dev_page_table;
    at.page_tokens = kv->page_tokens; at.nq = d.n_heads; at.nkv = d.n_kv_heads; at.dh = d.d_head; at.M = 16;
    at.pos0 = pos0; at.scale = 1.0f / sqrtf((float)d.d_head); at.Xout = ws.xattn;
    HIP_TRY(launch_attn_groups(at, G, xs_q, hi_only != 0, st), "attention launch");

    DenseArgs oa = dense(L.wo, ws.xattn, xs_q, m->d_q, d.d_model);
    residual_update(oa, L.norm2_g);
    HIP_TRY(launch_gemm_dense(oa, EPI_PARTIAL, st), "o-proj launch");

    if (fam_a) {
      NormArgs n2 = na;
      n2.g = L.norm2_g; n2.b = L.norm2_b;
      HIP_TRY(launch_norm(n2, st), "norm launch");
    } else {
      HIP_TRY(launch_rstd_groups(ws.ssq, n_tiles, d.d_model, d.norm_eps, ws.rstd, G, st), "rstd launch");
    }
    DenseArgs ua = dense(L.w_in, ws.xn, xs_d, d.d_model, n_in);
    ua.rstd = fam_a ? nullptr : ws.rstd; ua.g.Xout = ws.xact; ua.xouts = xs_ff; ua.g.KT_out = d.d_ff / 32;
    HIP_TRY(probe_record(l, 0, st), "probe event");
    HIP_TRY(launch_gemm_dense(ua, fam_a ? EPI_GELU : EPI_SWIGLU, st), "mlp-in launch");
    HIP_TRY(probe_record(l, 1, st), "probe event");

    DenseArgs da = dense(L.w_out, ws.xact, xs_ff, d.d_ff, d.d_model);
    residual_update(da, next_g);
    HIP_TRY(launch_gemm_dense(da, EPI_PARTIAL, st), "mlp-out launch");

    if (fam_a && (!last || dev_logits_last)) {
      NormArgs n3 = na;
      n3.g = next_g; n3.b = next_b;
      HIP_TRY(launch_norm(n3, st), "norm launch");
    }
  }
  if (dev_logits_last) {
    // logits of the prompt's last token: the skinny LM head on the last group's panels
    GemmArgs lm{};
    lm.M = 16; lm.planes = ws.base.gpart; lm.counters = ws.base.gemm_counters;
    lm.W = static_cast<const bf16_t*>(m->w.wlm); lm.X = ws.xn + (size_t)(G - 1) * xs_d; lm.KT = d.d_model / 32;
    if (!fam_a) { lm.ssq = ws.ssq + (size_t)(G - 1) * n_tiles * 16; lm.n_ssq = n_tiles; lm.d_in = d.d_model; lm.eps = d.norm_eps; }
    lm.n_rows = d.vocab; lm.out = dev_logits_last; lm.ld_out = d.vocab; lm.only_row = (n_tokens - 1) % 16;
    HIP_TRY(launch_gemm(lm, EPI_STORE, st), "lm-head launch");
  }
  kv->len = pos0 + n_tokens;
  return DISCO_OK;
}

const char* disco_last_error(void) { return g_err; }

int disco_pack_weight(const void* dev_src, int64_t n, int64_t k, void* dev_dst, disco_stream s) {
  if (!dev_src || !dev_dst) return fail(DISCO_EINVAL, "null pointer");
  if (n <= 0 || k <= 0 || n % 16 || k % 32) return fail(DISCO_EINVAL, "matrix %lld x %lld: rows %% 16 and columns %% 32 must be 0", (long long)n, (long long)k);
  if (!aligned(dev_src, 16) || !aligned(dev_dst, 16)) return fail(DISCO_EINVAL, "misaligned pointer");
  HIP_TRY(launch_pack(static_cast<const bf16_t*>(dev_src), n, k, static_cast<bf16_t*>(dev_dst), 1, 0, static_cast<hipStream_t>(s)), "pack launch");
  return DISCO_OK;
}

int disco_pack_gate_up(const void* dev_gate, const void* dev_up, int64_t d_ff, int64_t k, void* dev_dst, disco_stream s) {
  if (!dev_gate || !dev_up || !dev_dst) return fail(DISCO_EINVAL, "null pointer");
  if (d_ff <= 0 || k <= 0 || d_ff % 16 || k % 32) return fail(DISCO_EINVAL, "matrix %lld x %lld: rows %% 16 and columns %% 32 must be 0", (long long)d_ff, (long long)k);
  if (!aligned(dev_gate, 16) || !aligned(dev_up, 16) || !aligned(dev_dst, 16)) return fail(DISCO_EINVAL, "misaligned pointer");
  hipStream_t st = static_cast<hipStream_t>(s);
  HIP_TRY(launch_pack(static_cast<const bf16_t*>(dev_gate), d_ff, k, static_cast<bf16_t*>(dev_dst), 2, 0, st), "pack launch");
  HIP_TRY(launch_pack(static_cast<const bf16_t*>(dev_up), d_ff, k, static_cast<bf16_t*>(dev_dst), 2, 1, st), "pack launch");
  return DISCO_OK;
}

int disco_model_create(const disco_model_desc* desc, const disco_model_weights* w, disco_model** out) {
  if (!desc || !w || !out) return fail(DISCO_EINVAL, "null argument");
  const disco_model_desc& d = *desc;
  if (d.family != DISCO_FAMILY_A && d.family != DISCO_FAMILY_B) return fail(DISCO_EINVAL, "unknown family %d", d.family);
  if (d.n_layers < 1 || d.d_model < 32 || d.d_model % 32 || d.d_ff < 32 || d.d_ff % 32 || d.vocab < 16 || d.vocab % 16)
    return fail(DISCO_EINVAL, "d_model and d_ff must be multiples of 32, vocab of 16");
  if (d.d_model % 64) return fail(DISCO_EINVAL, "d_model must be a multiple of 64");
  if (d.d_model > 8192) return fail(DISCO_EINVAL, "d_model %d above 8192 unsupported", d.d_model);
  if (d.d_head != 64 && d.d_head != 128) return fail(DISCO_EINVAL, "d_head %d unsupported (64 or 128)", d.d_head);
  if (d.n_heads < 1 || d.n_kv_heads < 1 || d.n_heads % d.n_kv_heads) return fail(DISCO_EINVAL, "n_heads must be a multiple of n_kv_heads");
  if (d.family == DISCO_FAMILY_A && (d.max_pos < 1 || !w->pos_emb)) return fail(DISCO_EINVAL, "family A needs a position table");
  if (!(d.norm_eps > 0.f)) return fail(DISCO_EINVAL, "norm_eps must be positive");
  if (!w->tok_emb || !w->layers || !w->normf_g || !w->wlm) return fail(DISCO_EINVAL, "null weight pointer");
  if (w->tok_emb_stride < d.d_model || w->tok_emb_stride % 4) return fail(DISCO_EINVAL, "bad embedding stride");
  if (d.family == DISCO_FAMILY_A && !w->normf_b) return fail(DISCO_EINVAL, "family A needs norm biases");
  if (!aligned(w->tok_emb, 16) || !aligned(w->wlm, 16) || !aligned(w->normf_g, 16) || !aligned(w->normf_b, 16) || !aligned(w->pos_emb, 16))
    return fail(DISCO_EINVAL, "misaligned weight pointer");
  for (int l = 0; l < d.n_layers; ++l) {
    const disco_layer_weights& L = w->layers[l];
    if (!L.norm1_g || !L.norm2_g || !L.wqkv || !L.wo || !L.w_in || !L.w_out) return fail(DISCO_EINVAL, "null weight pointer in layer %d", l);
    if (d.family == DISCO_FAMILY_A && (!L.norm1_b || !L.norm2_b)) return fail(DISCO_EINVAL, "family A needs norm biases (layer %d)", l);
    const void* ps[] = {L.norm1_g, L.norm1_b, L.norm2_g, L.norm2_b, L.wqkv, L.wo, L.w_in, L.w_out};
    for (const void* p : ps) if (!aligned(p, 16)) return fail(DISCO_EINVAL, "misaligned weight pointer in layer %d", l);
  }
  disco_model* m = new (std::nothrow) disco_model();
  if (!m) return fail(DISCO_EINVAL, "out of host memory");
  m->d = d; m->w = *w;
  m->layers.assign(w->layers, w->layers + d.n_layers);
  m->w.layers = m->layers.data();
  if (d.family == DISCO_FAMILY_B) { m->w.pos_emb = nullptr; m->w.normf_b = nullptr; for (auto& L : m->layers) { L.norm1_b = nullptr; L.norm2_b = nullptr; } }
  m->d_q = d.n_heads * d.d_head; m->d_kv = d.n_kv_heads * d.d_head; m->d_qkv = m->d_q + 2 * m->d_kv;
  m->persist_big = d.d_model >= 2048;
  m->persist_ok = d.family == DISCO_FAMILY_B && forward_shape_ok(d.d_model, m->d_q, m->d_qkv, d.d_ff, d.d_head, d.vocab, m->persist_big);
  m->loop_steps = 1;
  if (m->persist_ok) {
    for (const auto& L : m->layers)
      m->fwd_layers.push_back(FwdLayer{static_cast<const bf16_t*>(L.wqkv), static_cast<const bf16_t*>(L.wo), static_cast<const bf16_t*>(L.w_in),
                                       static_cast<const bf16_t*>(L.w_out), L.norm1_g, L.norm2_g});
    // a draft loop in one launch needs panel versions for every step: kept for small models only
    const size_t per_step = sizeof(bf16_t) * 34 * ((size_t)(2 * d.n_layers + 1) * d.d_model + (size_t)d.n_layers * (2 * m->d_q + d.d_ff));
    if (per_step <= ((size_t)4 << 20) && d.d_model <= 4096) m->loop_steps = DISCO_MAX_BLOCK;
  }
  *out = m;
  return DISCO_OK;
}

void disco_model_destroy(disco_model* m) { delete m; }

static size_t kv_table_bytes(int n_pages) { return round_up(sizeof(int32_t) * (size_t)n_pages, 256); }
// rotary table of a family B cache: (cos, sin) per position and channel pair
static size_t kv_rope_bytes(const disco_model* m, int n_pages, int page_tokens) {
  if (m->d.family != DISCO_FAMILY_B) return 0;
  return round_up(sizeof(float) * 2 * (size_t)n_pages * page_tokens * (m->d.d_head / 2), 256);
}

size_t disco_kv_bytes(const disco_model* m, int capacity_tokens, int page_tokens) {
  if (!m || capacity_tokens < 1 || page_tokens < 1) return 0;
  const int n_pages = (capacity_tokens + page_tokens - 1) / page_tokens;
  const size_t page_elems = (size_t)2 * m->d.n_kv_heads * page_tokens * m->d.d_head;
  return kv_table_bytes(n_pages) + kv_rope_bytes(m, n_pages, page_tokens) + sizeof(bf16_t) * page_elems * n_pages * m->d.n_layers;
}

int disco_kv_create(const disco_model* m, void* dev_pages, size_t bytes, int capacity_tokens, int page_tokens,
                    const int32_t* host_page_order, disco_kv** out) {
  if (!m || !dev_pages || !out) return fail(DISCO_EINVAL, "null argument");
  if (capacity_tokens < 1 || page_tokens < 4 || page_tokens % 4) return fail(DISCO_EINVAL, "capacity must be positive and the page size a positive multiple of 4");
  if (!aligned(dev_pages, 256)) return fail(DISCO_EINVAL, "KV buffer must be 256-byte aligned");
  const size_t need = disco_kv_bytes(m, capacity_tokens, page_tokens);
  if (bytes < need) return fail(DISCO_ECAP, "KV buffer of %zu bytes, %zu needed", bytes, need);
  const int n_pages = (capacity_tokens + page_tokens - 1) / page_tokens;
  if (host_page_order) {
    std::vector<char> seen(n_pages, 0);
    for (int i = 0; i < n_pages; ++i) {
      const int p = host_page_order[i];
      if (p < 0 || p >= n_pages || seen[p]) return fail(DISCO_EINVAL, "page order is not a permutation");
      seen[p] = 1;
    }
  }
  disco_kv* kv = new (std::nothrow) disco_kv();
  if (!kv) return fail(DISCO_EINVAL, "out of host memory");
  kv->model = m; kv->page_tokens = page_tokens; kv->n_pages = n_pages;
  kv->capacity = n_pages * page_tokens; kv->len = 0;
  const size_t rope_bytes = kv_rope_bytes(m, n_pages, page_tokens);
  kv->dev_rope = rope_bytes ? reinterpret_cast<float*>(static_cast<char*>(dev_pages) + kv_table_bytes(n_pages)) : nullptr;
  kv->pages = reinterpret_cast<bf16_t*>(static_cast<char*>(dev_pages) + kv_table_bytes(n_pages) + rope_bytes);
  kv->layer_stride = (size_t)2 * m->d.n_kv_heads * page_tokens * m->d.d_head * n_pages;
  kv->dev_page_table = nullptr;
  if (host_page_order) {
    kv->dev_page_table = static_cast<int32_t*>(dev_pages);
    hipError_t e = hipMemcpy(kv->dev_page_table, host_page_order, sizeof(int32_t) * n_pages, hipMemcpyHostToDevice);
    if (e != hipSuccess) { delete kv; return hip_fail(e, "page table upload"); }
  }
  kv->rope_ready = false;
  *out = kv;
  return DISCO_OK;
}

void disco_kv_destroy(disco_kv* kv) { delete kv; }
int disco_kv_len(const disco_kv* kv) { return kv ? kv->len : DISCO_EINVAL; }
int disco_kv_pages_in_use(const disco_kv* kv) {
  return kv ? (kv->len + kv->page_tokens - 1) / kv->page_tokens : DISCO_EINVAL;
}

int disco_kv_fill(disco_kv* kv, const void* dev_src, int ctx, disco_stream s) {
  if (!kv || !dev_src) return fail(DISCO_EINVAL, "null argument");
  if (ctx < 0 || ctx > kv->capacity) return fail(DISCO_ECAP, "fill of %d positions exceeds capacity %d", ctx, kv->capacity);
  if (!aligned(dev_src, 16)) return fail(DISCO_EINVAL, "misaligned pointer");
  if (ctx > 0) {
    const disco_model_desc& d = kv->model->d;
    HIP_TRY(launch_kv_fill(static_cast<const bf16_t*>(dev_src), kv->pages, kv->dev_page_table, d.n_layers, kv->n_pages,
                           kv->page_tokens, d.n_kv_heads, d.d_head, ctx, static_cast<hipStream_t>(s)), "kv fill launch");
  }
  kv->len = ctx;
  return DISCO_OK;
}

size_t disco_workspace_bytes(const disco_model* m, int max_block, int max_ctx) {
  if (!m || max_block < 1 || max_block > DISCO_MAX_BLOCK || max_ctx < 0) return 0;
  return carve(m, max_block, max_ctx, nullptr).total;
}

int disco_workspace_init(const disco_model* m, void* dev_ws, size_t ws_bytes, int max_block, int max_ctx, disco_stream s) {
  if (!m || !dev_ws) return fail(DISCO_EINVAL, "null argument");
  if (!aligned(dev_ws, 256)) return fail(DISCO_EINVAL, "misaligned workspace");
  const size_t need = disco_workspace_bytes(m, max_block, max_ctx);
  if (need == 0 || ws_bytes < need) return fail(DISCO_EINVAL, "workspace of %zu bytes, %zu needed", ws_bytes, need);
  const Ws ws = carve(m, max_block, max_ctx, dev_ws);
  const disco_model_desc& d0 = m->d;
  HIP_TRY(launch_zero(ws.gemm_counters, ws.n_counters, static_cast<hipStream_t>(s)), "workspace init launch");
  HIP_TRY(launch_zero(reinterpret_cast<int*>(ws.clf_scratch), 64, static_cast<hipStream_t>(s)), "workspace init launch");
  HIP_TRY(launch_zero(ws.head_ready, QKV_ATTN_READY_SLOT * d0.n_heads, static_cast<hipStream_t>(s)), "workspace init launch");
  HIP_TRY(launch_zero(reinterpret_cast<int*>(ws.gate), 64, static_cast<hipStream_t>(s)), "workspace init launch");
  if (ws.ln_vec != nullptr) {
    // correction vectors of the deferred LayerNorms: one-token GEMVs of every consumer matrix with the gain vector
    // and with the bias vector of the norm in front of it (a missing bias gives zeros)
    const disco_model_desc& d = m->d;
    hipStream_t st = static_cast<hipStream_t>(s);
    auto gemv = [&](const void* W, int n_rows, const float* vec, float* out) -> int {
      HIP_TRY(launch_vec_panel(vec, d.d_model, ws.xn, st), "norm vector panel launch");
      GemmArgs g{};
      g.M = 1; g.W = static_cast<const bf16_t*>(W); g.X = ws.xn; g.KT = d.d_model / 32; g.n_rows = n_rows; g.grp = 1;
      g.n_split = 1; g.out = out; g.ld_out = n_rows; g.only_row = 0;
      HIP_TRY(launch_gemm(g, EPI_STORE, st), "norm vector launch");
      return DISCO_OK;
    };
    for (int l = 0; l < d.n_layers; ++l) {
      const disco_layer_weights& L = m->layers[l];
      float* v = ws.ln_vec + ws.ln_layer_stride * l;
      int rc = gemv(L.wqkv, m->d_qkv, L.norm1_g, v); if (rc) return rc;
      rc = gemv(L.wqkv, m->d_qkv, L.norm1_b, v + m->d_qkv); if (rc) return rc;
      v += 2 * (size_t)m->d_qkv;
      rc = gemv(L.w_in, d.d_ff, L.norm2_g, v); if (rc) return rc;
      rc = gemv(L.w_in, d.d_ff, L.norm2_b, v + d.d_ff); if (rc) return rc;
    }
    float* v = ws.ln_vec + ws.ln_layer_stride * d.n_layers;
    int rc = gemv(m->w.wlm, d.vocab, m->w.normf_g, v); if (rc) return rc;
    rc = gemv(m->w.wlm, d.vocab, m->w.normf_b, v + d.vocab); if (rc) return rc;
  }
  if (ws.fwd_layers != nullptr) {
    HIP_TRY(hipMemcpyAsync(ws.fwd_layers, m->fwd_layers.data(), sizeof(FwdLayer) * m->fwd_layers.size(), hipMemcpyHostToDevice,
                           static_cast<hipStream_t>(s)), "layer table upload");
    HIP_TRY(launch_zero(reinterpret_cast<int*>(ws.bar), FWD_BAR_WORDS, static_cast<hipStream_t>(s)), "workspace init launch");
  }
  return DISCO_OK;
}

int disco_classify_scratch_init(void* dev_scratch, disco_stream s) {
  if (!dev_scratch || !aligned(dev_scratch, 256)) return fail(DISCO_EINVAL, "scratch pointer null or not 256-byte aligned");
  HIP_TRY(launch_zero(static_cast<int*>(dev_scratch), 64, static_cast<hipStream_t>(s)), "scratch init launch");
  return DISCO_OK;
}

int disco_draft_step(const disco_model* draft, disco_kv* kv, const int32_t* dev_tokens_in, int n_in, float* dev_logits,
                     void* dev_ws, size_t ws_bytes, const uint32_t* dev_gate, disco_stream s) {
  int rc = check_forward_args(draft, kv, dev_tokens_in, n_in, dev_ws, ws_bytes);
  if (rc) return rc;
  if (!dev_logits || !aligned(dev_logits, 16)) return fail(DISCO_EINVAL, "logits pointer null or misaligned");
  if (dev_gate && !aligned(dev_gate, 4)) return fail(DISCO_EINVAL, "misaligned gate pointer");
  const Ws ws = carve(draft, n_in, kv->len + n_in, dev_ws);
  return forward_block(draft, kv, dev_tokens_in, n_in, dev_logits, true, ws, dev_gate, static_cast<hipStream_t>(s));
}

static int classify_impl(const disco_clf* clf, float* dev_logits, int vocab, float pos_feature, float tau, int force_halt,
                         disco_clf_out* dev_out, int32_t* dev_token_next, int32_t* dev_block_slot, uint32_t* dev_gate,
                         int32_t* dev_sl_count, const int32_t* dev_force_token, float* scratch, hipStream_t st) {
  if (!dev_logits || !dev_out) return fail(DISCO_EINVAL, "null argument");
  if (vocab < 1 || vocab > 65536) return fail(DISCO_EINVAL, "vocab %d outside [1, 65536]", vocab);
  if (!aligned(dev_logits, 16) || !aligned(dev_out, 4) || !aligned(dev_token_next, 4) || !aligned(dev_block_slot, 4) ||
      !aligned(dev_gate, 4) || !aligned(dev_sl_count, 4) || !aligned(dev_force_token, 4) || !aligned(scratch, 256))
    return fail(DISCO_EINVAL, "misaligned pointer");
  if (clf) {
    if (!clf->dev_params || !aligned(clf->dev_params, 4)) return fail(DISCO_EINVAL, "classifier parameters null or misaligned");
    if (clf->hidden < 1 || clf->hidden > DISCO_CLF_HIDDEN_MAX) return fail(DISCO_EINVAL, "classifier hidden size %d outside [1, %d]", clf->hidden, DISCO_CLF_HIDDEN_MAX);
  }
  ClassifyArgs a{};
  a.logits = dev_logits; a.vocab = vocab; a.clf_params = clf ? clf->dev_params : nullptr; a.hidden = clf ? clf->hidden : 0;
  a.pos_feature = pos_feature; a.tau = tau; a.force_halt = force_halt; a.out = dev_out; a.token_next = dev_token_next;
  a.block_slot = dev_block_slot; a.gate = dev_gate; a.sl_count = dev_sl_count; a.force_token = dev_force_token;
  a.scratch = scratch;
  HIP_TRY(launch_classify(a, st), "classify launch");
  return DISCO_OK;
}

int disco_classify(const disco_clf* clf, float* dev_logits, int vocab, float pos_feature, float tau, int force_halt,
                   disco_clf_out* dev_out, int32_t* dev_token_next, int32_t* dev_block_slot, uint32_t* dev_gate,
                   int32_t* dev_sl_count, const int32_t* dev_force_token, void* dev_scratch, disco_stream s) {
  return classify_impl(clf, dev_logits, vocab, pos_feature, tau, force_halt, dev_out, dev_token_next, dev_block_slot, dev_gate,
                       dev_sl_count, dev_force_token, static_cast<float*>(dev_scratch), static_cast<hipStream_t>(s));
}

int disco_classify_static(const disco_clf* clf, float* dev_logits, int vocab, float pos_feature, float tau, int force_halt,
                          disco_clf_out* dev_out, int32_t* dev_token_next, int32_t* dev_block_slot, uint32_t* dev_gate,
                          int32_t* dev_sl_count, const int32_t* dev_force_token, disco_stream s) {
  // the array holds one record per 1024 logits: 64 records
  if (vocab > DISCO_CLASSIFY_STATIC_MAX_VOCAB)
    return fail(DISCO_ECAP, "vocab %d above the %d logits that the library's own scratch array serves", vocab, DISCO_CLASSIFY_STATIC_MAX_VOCAB);
  float* scratch = nullptr;
  HIP_TRY(classify_static_scratch(&scratch), "address of the scratch array");
  hipStream_t st = static_cast<hipStream_t>(s);
  // the array keeps the last call's contents: the ticket word must start at zero (a fill kernel, which
  // a captured graph replays correctly)
  HIP_TRY(launch_zero(reinterpret_cast<int*>(scratch), 64, st), "scratch clear launch");
  return classify_impl(clf, dev_logits, vocab, pos_feature, tau, force_halt, dev_out, dev_token_next, dev_block_slot, dev_gate,
                       dev_sl_count, dev_force_token, scratch, st);
}

int disco_verify(const disco_model* target, disco_kv* kv, const int32_t* dev_block, int n_block, int32_t* dev_argmax,
                 float* dev_logits, void* dev_ws, size_t ws_bytes, disco_stream s) {
  int rc = check_forward_args(target, kv, dev_block, n_block, dev_ws, ws_bytes);
  if (rc) return rc;
  if (!dev_argmax || !aligned(dev_argmax, 4)) return fail(DISCO_EINVAL, "argmax pointer null or misaligned");
  if (dev_logits && !aligned(dev_logits, 16)) return fail(DISCO_EINVAL, "misaligned logits pointer");
  const Ws ws = carve(target, n_block, kv->len + n_block, dev_ws);
  float* logits = dev_logits ? dev_logits : ws.logits;
  hipStream_t st = static_cast<hipStream_t>(s);
  rc = forward_block(target, kv, dev_block, n_block, logits, false, ws, nullptr, st);
  if (rc) return rc;
  const bool persistent = target->persist_ok && ws.bar != nullptr && persistent_enabled();
  HIP_TRY(launch_argmax_rows(logits, n_block, target->d.vocab, dev_argmax, persistent ? ws.bar + FWD_BAR_ABORT_WORD : ws.abort_word, st), "argmax launch");
  return DISCO_OK;
}

int disco_accept(const int32_t* dev_block, const int32_t* dev_argmax, int n_block, const int32_t* dev_n_block,
                 disco_accept_out* dev_out, disco_accept_out* host_out, disco_stream s) {
  if (!dev_block || !dev_argmax || !dev_out) return fail(DISCO_EINVAL, "null argument");
  if (n_block < 1 || n_block > DISCO_MAX_BLOCK) return fail(DISCO_ECAP, "block of %d tokens outside [1, %d]", n_block, DISCO_MAX_BLOCK);
  if (!aligned(dev_block, 4) || !aligned(dev_argmax, 4) || !aligned(dev_out, 4) || !aligned(host_out, 4) || !aligned(dev_n_block, 4))
    return fail(DISCO_EINVAL, "misaligned pointer");
  HIP_TRY(launch_accept(dev_block, dev_argmax, n_block, dev_n_block, dev_out, host_out, static_cast<hipStream_t>(s)), "accept launch");
  return DISCO_OK;
}

int disco_kv_rollback(disco_kv* kv, int new_len) {
  if (!kv) return fail(DISCO_EINVAL, "null argument");
  if (new_len < 0 || new_len > kv->len) return fail(DISCO_ESTATE, "rollback to %d outside [0, %d]", new_len, kv->len);
  kv->len = new_len;
  return DISCO_OK;
}

static int draft_loop_impl(const disco_model* draft, disco_kv* kv, const disco_clf* clf, const int32_t* dev_tokens_in, int n_in,
                           int cap, int static_sl, float pos_feature0, float tau, const disco_loop_opts& o, float* dev_logits,
                           disco_clf_out* dev_steps, disco_loop_out* dev_out, disco_loop_out* host_out,
                           void* dev_ws, size_t ws_bytes, disco_stream s) {
  const int32_t* dev_force_tokens = o.dev_force_tokens; const int32_t* dev_ref_tokens = o.dev_ref_tokens;
  const float temperature = o.temperature; const float* dev_u_draft = o.dev_u_draft; float* dev_draft_probs = o.dev_draft_probs;
  const float ppl_threshold = o.ppl_threshold;
  const int k0 = o.block_offset;
  const bool sampled = dev_u_draft != nullptr;
  if (k0 < 0 || k0 + cap > DISCO_MAX_BLOCK - 1) return fail(DISCO_ECAP, "block offset %d + cap %d outside [0, %d]", k0, cap, DISCO_MAX_BLOCK - 1);
  if (k0 > 0 && (sampled || n_in != 1)) return fail(DISCO_EINVAL, "a continued block feeds one token and is not sampled");
  if (!aligned(dev_ref_tokens, 4)) return fail(DISCO_EINVAL, "misaligned pointer");
  if (sampled && (dev_ref_tokens || dev_force_tokens)) return fail(DISCO_EINVAL, "sampling excludes forced and reference tokens");
  if (!(ppl_threshold >= 0.f)) return fail(DISCO_EINVAL, "perplexity threshold must be >= 0 (0 = off)");
  if (ppl_threshold > 0.f && (sampled || dev_ref_tokens || clf || static_sl > 0))
    return fail(DISCO_EINVAL, "the perplexity rule excludes sampling, reference tokens, a classifier and a static lookahead");
  if (sampled) {
    if (!(temperature > 0.f)) return fail(DISCO_EINVAL, "temperature must be positive");
    if (!dev_draft_probs || !aligned(dev_u_draft, 4) || !aligned(dev_draft_probs, 16)) return fail(DISCO_EINVAL, "sampling buffers null or misaligned");
    if (draft && (draft->d.vocab > 65536)) return fail(DISCO_EINVAL, "vocab above 65536 unsupported for sampling");
  }
  if (cap < 1 || cap > DISCO_MAX_BLOCK - 1) return fail(DISCO_ECAP, "cap %d outside [1, %d]", cap, DISCO_MAX_BLOCK - 1);
  if (static_sl < 0 || static_sl > cap) return fail(DISCO_EINVAL, "static_sl %d outside [0, cap]", static_sl);
  if (n_in < 1 || n_in > 2) return fail(DISCO_EINVAL, "n_in must be 1 or 2");
  int rc = check_forward_args(draft, kv, dev_tokens_in, n_in, dev_ws, ws_bytes);
  if (rc) return rc;
  if (kv->len + n_in + cap - 1 > kv->capacity) return fail(DISCO_ECAP, "KV capacity %d exceeded by the draft loop", kv->capacity);
  if (draft->d.family == DISCO_FAMILY_A && kv->len + n_in + cap - 1 > draft->d.max_pos) return fail(DISCO_ECAP, "position table exceeded by the draft loop");
  if (!dev_logits || !dev_steps || !dev_out) return fail(DISCO_EINVAL, "null argument");
  if (!aligned(dev_logits, 16) || !aligned(dev_steps, 4) || !aligned(dev_out, 4) || !aligned(host_out, 4) || !aligned(dev_force_tokens, 4))
    return fail(DISCO_EINVAL, "misaligned pointer");
  if (clf) {
    if (!clf->dev_params || clf->hidden < 1 || clf->hidden > DISCO_CLF_HIDDEN_MAX) return fail(DISCO_EINVAL, "bad classifier");
  }
  if (carve(draft, 2, kv->len + n_in + cap, nullptr).total > ws_bytes) return fail(DISCO_EINVAL, "workspace too small for the draft loop");
  hipStream_t st = static_cast<hipStream_t>(s);
  const Ws ws = carve(draft, 2, kv->len + n_in + cap, dev_ws);
  if (k0 == 0) HIP_TRY(launch_loop_init(ws.gate, ws.sl_count, dev_tokens_in, n_in, dev_out, st), "loop init launch");
  const int steps = static_sl > 0 ? static_sl : cap;
  dev_steps += k0;                                 // records and block slots of this call's steps
  int32_t* block_base = dev_out->block + k0;
  if (draft->persist_ok && ws.bar != nullptr && !sampled && steps <= draft->loop_steps && persistent_enabled()) {
    // the whole loop in one launch: the kernel leaves at the first halting step
    const disco_model_desc& d = draft->d;
    const int pos0 = kv->len;
    if (kv->dev_rope && !kv->rope_ready) {
      HIP_TRY(launch_rope_fill(kv->dev_rope, kv->capacity, d.d_head, d.rope_base, st), "rotary table launch");
      kv->rope_ready = true;
    }
    NormArgs n0{};
    n0.h = ws.h; n0.d = d.d_model; n0.M = n_in; n0.eps = d.norm_eps; n0.Xout = ws.xn_v; n0.pos0 = pos0; n0.vocab = d.vocab;
    n0.max_pos = d.max_pos; n0.ssq_out = reinterpret_cast<float*>(ws.xn_v + (size_t)32 * d.d_model); n0.n_ssq_out = d.d_model / 16;
    n0.g = draft->layers[0].norm1_g;
    n0.tokens = dev_tokens_in; n0.tok_emb = static_cast<const bf16_t*>(draft->w.tok_emb); n0.tok_stride = draft->w.tok_emb_stride;
    HIP_TRY(launch_norm(n0, st), "embedding launch");
    HIP_TRY(launch_zero(reinterpret_cast<int*>(ws.bar), FWD_BAR_WORDS, st), "barrier reset launch");
    FwdArgs f = forward_args(draft, kv, ws);
    f.M = n_in; f.pos0 = pos0; f.logits = dev_logits; f.only_last = 1; f.n_steps = steps; f.open_end = o.open_end ? 1 : 0;
    ClassifyArgs& a = f.clf;
    a.logits = dev_logits; a.vocab = d.vocab; a.clf_params = clf ? clf->dev_params : nullptr; a.hidden = clf ? clf->hidden : 0;
    a.pos_feature = pos_feature0; a.tau = static_sl > 0 ? -1.0e30f : tau; a.out = dev_steps; a.token_next = ws.tok_next;
    a.block_slot = block_base + 1; a.gate = ws.gate; a.sl_count = ws.sl_count; a.force_token = dev_force_tokens;
    a.ref_token = dev_ref_tokens; a.ppl_threshold = ppl_threshold; a.scratch = ws.clf_scratch;
    HIP_TRY(launch_forward(f, draft->persist_big, true, st), "draft loop launch");
    kv->len = pos0 + n_in + steps - 1;
    HIP_TRY(launch_loop_finish(ws.sl_count, ws.gate, dev_out, host_out, ws.bar + FWD_BAR_ABORT_WORD, st), "loop finish launch");
    return DISCO_OK;
  }
  const int len_entry = kv->len;
  for (int j = 1; j <= steps; ++j) {
    rc = forward_block(draft, kv, j == 1 ? dev_tokens_in : ws.tok_next, j == 1 ? n_in : 1, dev_logits, true, ws, ws.gate, st);
    if (rc) { kv->len = len_entry; return rc; }   // a launch failed: the cache length is as on entry (see disco.h)
    if (sampled) {
      // the draft token of this step is drawn before the classifier may close the gate on it
      SampleArgs sa{};
      sa.logits = dev_logits; sa.ld = draft->d.vocab; sa.vocab = draft->d.vocab; sa.inv_t = 1.0f / temperature;
      sa.u = dev_u_draft + (j - 1); sa.probs = dev_draft_probs + (size_t)(j - 1) * draft->d.vocab;
      sa.tokens = ws.tok_next; sa.block_slot = block_base + j; sa.gate = ws.gate;
      { const hipError_t e = launch_sample_rows(sa, 1, st); if (e != hipSuccess) { kv->len = len_entry; return hip_fail(e, "sample launch"); } }
    }
    ClassifyArgs a{};
    a.logits = dev_logits; a.vocab = draft->d.vocab; a.clf_params = clf ? clf->dev_params : nullptr; a.hidden = clf ? clf->hidden : 0;
    a.pos_feature = pos_feature0 + (float)(j - 1);
    a.tau = static_sl > 0 ? -1.0e30f : tau;
    a.force_halt = (j == steps && !o.open_end) ? 1 : 0;
    a.out = dev_steps + (j - 1); a.token_next = sampled ? nullptr : ws.tok_next;
    a.block_slot = sampled ? nullptr : block_base + j; a.gate = ws.gate;
    a.sl_count = ws.sl_count; a.force_token = dev_force_tokens ? dev_force_tokens + (j - 1) : nullptr;
    a.ref_token = dev_ref_tokens ? dev_ref_tokens + (j - 1) : nullptr;
    a.ppl_threshold = ppl_threshold;
    a.scratch = ws.clf_scratch;
    { const hipError_t e = launch_classify(a, st); if (e != hipSuccess) { kv->len = len_entry; return hip_fail(e, "classify launch"); } }
  }
  HIP_TRY(launch_loop_finish(ws.sl_count, ws.gate, dev_out, host_out, ws.abort_word, st), "loop finish launch");
  return DISCO_OK;
}

int disco_draft_loop(const disco_model* draft, disco_kv* kv, const disco_clf* clf, const int32_t* dev_tokens_in, int n_in,
                     int cap, int static_sl, float pos_feature0, float tau, const int32_t* dev_force_tokens,
                     float* dev_logits, disco_clf_out* dev_steps, disco_loop_out* dev_out, disco_loop_out* host_out,
                     void* dev_ws, size_t ws_bytes, disco_stream s) {
  disco_loop_opts o{};
  o.dev_force_tokens = dev_force_tokens;
  return draft_loop_impl(draft, kv, clf, dev_tokens_in, n_in, cap, static_sl, pos_feature0, tau, o, dev_logits, dev_steps, dev_out,
                         host_out, dev_ws, ws_bytes, s);
}

int disco_draft_loop_ex(const disco_model* draft, disco_kv* kv, const disco_clf* clf, const int32_t* dev_tokens_in, int n_in,
                        int cap, int static_sl, float pos_feature0, float tau, const disco_loop_opts* opts, float* dev_logits,
                        disco_clf_out* dev_steps, disco_loop_out* dev_out, disco_loop_out* host_out, void* dev_ws,
                        size_t ws_bytes, disco_stream s) {
  disco_loop_opts o{};
  if (opts) o = *opts;
  return draft_loop_impl(draft, kv, clf, dev_tokens_in, n_in, cap, static_sl, pos_feature0, tau, o, dev_logits, dev_steps, dev_out,
                         host_out, dev_ws, ws_bytes, s);
}

int disco_draft_loop_sampled(const disco_model* draft, disco_kv* kv, const disco_clf* clf, const int32_t* dev_tokens_in,
                             int n_in, int cap, int static_sl, float pos_feature0, float tau, float temperature,
                             const float* dev_u_draft, float* dev_draft_probs, float* dev_logits, disco_clf_out* dev_steps,
                             disco_loop_out* dev_out, disco_loop_out* host_out, void* dev_ws, size_t ws_bytes, disco_stream s) {
  if (!dev_u_draft) return fail(DISCO_EINVAL, "null argument");
  disco_loop_opts o{};
  o.temperature = temperature; o.dev_u_draft = dev_u_draft; o.dev_draft_probs = dev_draft_probs;
  return draft_loop_impl(draft, kv, clf, dev_tokens_in, n_in, cap, static_sl, pos_feature0, tau, o, dev_logits, dev_steps, dev_out,
                         host_out, dev_ws, ws_bytes, s);
}

int disco_iterate(const disco_model* target, disco_kv* kv_t, void* dev_ws_t, size_t ws_t_bytes, const disco_model* draft,
                  disco_kv* kv_d, void* dev_ws_d, size_t ws_d_bytes, const disco_clf* clf, const int32_t* host_pending,
                  int n_pending, int cap, int static_sl, int chunk, float pos_feature0, float tau, const disco_loop_opts* opts,
                  const disco_iter_buffers* buf, disco_iter_result* res, disco_stream s) {
  if (!target || !kv_t || !buf || !res || !host_pending) return fail(DISCO_EINVAL, "null argument");
  if (n_pending < 1 || n_pending > 2) return fail(DISCO_EINVAL, "n_pending must be 1 or 2");
  if (cap < 0 || cap > DISCO_MAX_BLOCK - 1) return fail(DISCO_ECAP, "cap %d outside [0, %d]", cap, DISCO_MAX_BLOCK - 1);
  if (chunk < 0) return fail(DISCO_EINVAL, "chunk must be >= 0");
  if (!buf->dev_loop_out || !buf->host_loop_out || !buf->dev_argmax || !buf->dev_accept_out || !buf->host_accept_out)
    return fail(DISCO_EINVAL, "null iteration buffer");
  disco_loop_opts o{};
  if (opts) o = *opts;
  if (o.dev_u_draft || o.block_offset || o.open_end) return fail(DISCO_EINVAL, "sampling and block continuation are not options of an iteration");
  if (!draft) cap = 0;
  if (cap > 0 && (!kv_d || !dev_ws_d || !buf->dev_tokens_in || !buf->dev_logits_draft || !buf->dev_steps)) return fail(DISCO_EINVAL, "null draft-side argument");
  hipStream_t st = static_cast<hipStream_t>(s);
  const int len_t0 = kv_t->len;
  int sl = 0, enq = 0, ran = 0;
  if (cap >= 1) {
    const int len_d0 = kv_d->len;
    HIP_TRY(launch_put_tokens(buf->dev_tokens_in, host_pending[0], n_pending > 1 ? host_pending[1] : 0, n_pending, nullptr, nullptr, st),
            "token upload launch");
    const int total = static_sl > 0 ? static_sl : cap;          // steps the block may take
    int c = chunk > 0 ? chunk : 3;                              // default: a look at the flag every third step
    if (static_sl > 0 || c > total) c = total;
    bool halted = false;
    while (!halted && enq < total) {
      const int todo = total - enq < c ? total - enq : c;
      disco_loop_opts oc = o;
      oc.block_offset = enq; oc.open_end = (enq + todo < total) ? 1 : 0;
      if (oc.dev_force_tokens) oc.dev_force_tokens += enq;
      if (oc.dev_ref_tokens) oc.dev_ref_tokens += enq;
      const int rc = draft_loop_impl(draft, kv_d, clf, enq == 0 ? buf->dev_tokens_in : buf->dev_loop_out->block + enq, enq == 0 ? n_pending : 1,
                                     todo, static_sl > 0 ? todo : 0, pos_feature0 + (float)enq, tau, oc, buf->dev_logits_draft,
                                     buf->dev_steps, buf->dev_loop_out, buf->host_loop_out, dev_ws_d, ws_d_bytes, s);
      if (rc) return rc;
      enq += todo;
      HIP_TRY(hipStreamSynchronize(st), "stream synchronisation");
      sl = buf->host_loop_out->sl;
      if (sl < 0) return fail(DISCO_EHIP, "the draft loop's grid barrier timed out");
      halted = buf->host_loop_out->halted != 0;
    }
    if (sl > DISCO_MAX_BLOCK - 1) return fail(DISCO_ESTATE, "draft loop reported %d tokens", sl);
    // with a reference the step whose token left it ran too
    ran = sl + ((o.dev_ref_tokens && sl < total) ? 1 : 0);
    if (ran > enq) ran = enq;
    const int rc = disco_kv_rollback(kv_d, len_d0 + n_pending + ran - 1);
    if (rc) return rc;
  } else {
    HIP_TRY(launch_put_tokens(nullptr, host_pending[0], n_pending > 1 ? host_pending[1] : 0, n_pending, buf->dev_loop_out, nullptr, st),
            "block launch");
  }
  int rc = disco_verify(target, kv_t, buf->dev_loop_out->block, sl + 1, buf->dev_argmax, nullptr, dev_ws_t, ws_t_bytes, s);
  if (rc) return rc;
  rc = disco_accept(buf->dev_loop_out->block, buf->dev_argmax, sl + 1, nullptr, buf->dev_accept_out, buf->host_accept_out, s);
  if (rc) return rc;
  HIP_TRY(hipStreamSynchronize(st), "stream synchronisation");
  const disco_accept_out& acc = *buf->host_accept_out;
  if (acc.n < 0 || acc.n > sl) return fail(DISCO_ESTATE, "acceptance reported %d of %d tokens", acc.n, sl);
  if (acc.emit[acc.n] < 0) return fail(DISCO_EHIP, "the verification forward's grid barrier timed out");
  rc = disco_kv_rollback(kv_t, len_t0 + acc.n + 1);
  if (rc) return rc;
  if (kv_d && kv_d->len > len_t0 + acc.n + 1) { rc = disco_kv_rollback(kv_d, len_t0 + acc.n + 1); if (rc) return rc; }
  res->sl = sl; res->n = acc.n; res->draft_forwards = ran; res->draft_steps_enqueued = enq;
  for (int i = 0; i < DISCO_MAX_BLOCK; ++i) {
    res->block[i] = (cap >= 1 && i <= sl) ? buf->host_loop_out->block[i] : 0;
    res->emit[i] = i <= acc.n ? acc.emit[i] : 0;
  }
  if (cap < 1) res->block[0] = host_pending[n_pending - 1];
  return DISCO_OK;
}

int disco_sample(const float* dev_logits, int n_rows, int vocab, int64_t ld_logits, float temperature, const float* dev_u,
                 float* dev_probs, int32_t* dev_tokens, disco_stream s) {
  if (!dev_logits || !dev_u || !dev_tokens) return fail(DISCO_EINVAL, "null argument");
  if (n_rows < 1 || n_rows > 65535) return fail(DISCO_EINVAL, "n_rows %d outside [1, 65535]", n_rows);
  if (vocab < 4 || vocab % 4 || vocab > 65536) return fail(DISCO_EINVAL, "vocab %d: must be a multiple of 4 in [4, 65536]", vocab);
  if (ld_logits < vocab || ld_logits % 4) return fail(DISCO_EINVAL, "row stride must be a multiple of 4 and at least vocab");
  if (!(temperature > 0.f)) return fail(DISCO_EINVAL, "temperature must be positive");
  if (!aligned(dev_logits, 16) || !aligned(dev_u, 4) || !aligned(dev_probs, 16) || !aligned(dev_tokens, 4)) return fail(DISCO_EINVAL, "misaligned pointer");
  SampleArgs a{};
  a.logits = dev_logits; a.ld = ld_logits; a.vocab = vocab; a.inv_t = 1.0f / temperature; a.u = dev_u; a.probs = dev_probs;
  a.tokens = dev_tokens;
  HIP_TRY(launch_sample_rows(a, n_rows, static_cast<hipStream_t>(s)), "sample launch");
  return DISCO_OK;
}

int disco_accept_sample(const int32_t* dev_block, int n_block, const int32_t* dev_n_block, const float* dev_draft_probs,
                        const float* dev_target_logits, int vocab, float temperature, const float* dev_u_accept,
                        const float* dev_u_resample, disco_accept_out* dev_out, disco_accept_out* host_out, disco_stream s) {
  if (!dev_block || !dev_target_logits || !dev_u_resample || !dev_out) return fail(DISCO_EINVAL, "null argument");
  if (n_block < 1 || n_block > DISCO_MAX_BLOCK) return fail(DISCO_ECAP, "block of %d tokens outside [1, %d]", n_block, DISCO_MAX_BLOCK);
  if (n_block > 1 && (!dev_draft_probs || !dev_u_accept)) return fail(DISCO_EINVAL, "null argument");
  if (vocab < 4 || vocab % 4 || vocab > 65536) return fail(DISCO_EINVAL, "vocab %d: must be a multiple of 4 in [4, 65536]", vocab);
  if (!(temperature > 0.f)) return fail(DISCO_EINVAL, "temperature must be positive");
  if (!aligned(dev_block, 4) || !aligned(dev_n_block, 4) || !aligned(dev_draft_probs, 16) || !aligned(dev_target_logits, 16) ||
      !aligned(dev_u_accept, 4) || !aligned(dev_u_resample, 4) || !aligned(dev_out, 4) || !aligned(host_out, 4))
    return fail(DISCO_EINVAL, "misaligned pointer");
  AcceptSampleArgs a{};
  a.block = dev_block; a.n_block = n_block; a.dev_n_block = dev_n_block; a.draft_probs = dev_draft_probs;
  a.target_logits = dev_target_logits; a.vocab = vocab; a.inv_t = 1.0f / temperature; a.u_accept = dev_u_accept;
  a.u_resample = dev_u_resample; a.out = dev_out; a.host_out = host_out;
  HIP_TRY(launch_accept_sample(a, static_cast<hipStream_t>(s)), "accept launch");
  return DISCO_OK;
}

int disco_clf_train(const float* dev_feats, const int32_t* dev_labels, int n, int hidden, int epochs, float lr,
                    float* dev_params, float* dev_loss, disco_stream s) {
  if (!dev_feats || !dev_labels || !dev_params) return fail(DISCO_EINVAL, "null argument");
  if (n < 1 || n > DISCO_TRAIN_MAX_N) return fail(DISCO_ECAP, "%d training samples outside [1, %d]", n, DISCO_TRAIN_MAX_N);
  if (hidden < 1 || hidden > DISCO_CLF_HIDDEN_MAX) return fail(DISCO_EINVAL, "classifier hidden size %d outside [1, %d]", hidden, DISCO_CLF_HIDDEN_MAX);
  if (epochs < 0 || !(lr > 0.f)) return fail(DISCO_EINVAL, "epochs must be >= 0 and the step positive");
  if (!aligned(dev_feats, 4) || !aligned(dev_labels, 4) || !aligned(dev_params, 4) || !aligned(dev_loss, 4)) return fail(DISCO_EINVAL, "misaligned pointer");
  TrainArgs a{};
  a.feats = dev_feats; a.labels = dev_labels; a.n = n; a.hidden = hidden; a.epochs = epochs; a.lr = lr; a.params = dev_params;
  a.loss = dev_loss;
  HIP_TRY(launch_clf_train(a, static_cast<hipStream_t>(s)), "train launch");
  return DISCO_OK;
}

int disco_clf_eval(const disco_clf* clf, const float* dev_feats, const int32_t* dev_labels, int n, float tau,
                   float* dev_scores, int32_t* dev_counts, disco_stream s) {
  if (!clf || !clf->dev_params || !dev_feats) return fail(DISCO_EINVAL, "null argument");
  if (clf->hidden < 1 || clf->hidden > DISCO_CLF_HIDDEN_MAX) return fail(DISCO_EINVAL, "classifier hidden size %d outside [1, %d]", clf->hidden, DISCO_CLF_HIDDEN_MAX);
  if (n < 1) return fail(DISCO_EINVAL, "n must be positive");
  if ((dev_counts != nullptr) != (dev_labels != nullptr)) return fail(DISCO_EINVAL, "labels and counts go together");
  if (!aligned(dev_feats, 4) || !aligned(dev_labels, 4) || !aligned(dev_scores, 4) || !aligned(dev_counts, 4) || !aligned(clf->dev_params, 4))
    return fail(DISCO_EINVAL, "misaligned pointer");
  EvalArgs a{};
  a.feats = dev_feats; a.labels = dev_labels; a.n = n; a.params = clf->dev_params; a.hidden = clf->hidden; a.tau = tau;
  a.scores = dev_scores; a.counts = dev_counts;
  HIP_TRY(launch_clf_eval(a, static_cast<hipStream_t>(s)), "eval launch");
  return DISCO_OK;
}

int disco_clf_examples(const disco_clf_out* dev_records, int n, const int32_t* dev_ref_tokens, float* dev_feats,
                       int32_t* dev_labels, int32_t* dev_tokens, disco_stream s) {
  if (!dev_records || !dev_ref_tokens || !dev_feats || !dev_labels) return fail(DISCO_EINVAL, "null argument");
  if (n < 1) return fail(DISCO_EINVAL, "n must be positive");
  if (!aligned(dev_records, 4) || !aligned(dev_ref_tokens, 4) || !aligned(dev_feats, 4) || !aligned(dev_labels, 4) || !aligned(dev_tokens, 4))
    return fail(DISCO_EINVAL, "misaligned pointer");
  HIP_TRY(launch_clf_examples(dev_records, n, dev_ref_tokens, dev_feats, dev_labels, dev_tokens, static_cast<hipStream_t>(s)), "examples launch");
  return DISCO_OK;
}

int disco_heuristic_next(int lookahead, int drafted, int accepted, int up, int down, int cap) {
  if (lookahead < 1 || drafted < 0 || accepted < 0 || accepted > drafted || up < 0 || down < 0 || cap < 1)
    return fail(DISCO_EINVAL, "heuristic: lookahead and cap must be >= 1, 0 <= accepted <= drafted, steps >= 0");
  if (drafted == 0) return lookahead > cap ? cap : lookahead;          // nothing was drafted: nothing was learnt
  int next = (accepted == drafted) ? lookahead + up : lookahead - down;
  if (next > cap) next = cap;
  if (next < 1) next = 1;
  return next;
}

int disco_set_launch_mode(int mode) {
  if (mode < 0 || mode > 2)
    return fail(DISCO_EINVAL, "launch mode %d: 0 (one launch per phase, QKV + attention in one), 1 (one launch per forward) or 2 (one launch per phase)", mode);
  const int prev = g_launch_mode;
  g_launch_mode = mode;
  return prev;
}

int disco_set_wait_limit(int polls) {
  const int prev = g_wait_limit;
  g_wait_limit = polls > (1 << 24) ? (1 << 24) : polls;
  return prev;
}

int disco_probe_enable(int layer) {
  std::lock_guard<std::mutex> lock(g_probe_mu);
  g_probe_taken = false;
  if (layer < 0) { g_probe_layer = -1; return DISCO_OK; }
  for (int i = 0; i < 2; ++i)
    if (!g_probe_ev[i]) HIP_TRY(hipEventCreate(&g_probe_ev[i]), "probe event create");
  g_probe_layer = layer;
  return DISCO_OK;
}

float disco_probe_read_ms(void) {
  std::lock_guard<std::mutex> lock(g_probe_mu);
  if (!g_probe_taken) return -1.0f;
  float ms = -1.0f;
  if (hipEventElapsedTime(&ms, g_probe_ev[0], g_probe_ev[1]) != hipSuccess) return -1.0f;
  return ms;
}

}  // extern "C"
