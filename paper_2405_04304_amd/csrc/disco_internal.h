// Internal launcher interface between the C boundary (disco_api.cpp) and the gfx950 kernels
// (disco_kernels.hip).  Plain structs and pointers; nothing here is exported.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace disco {

typedef uint16_t bf16_t;  // raw bfloat16 bits

// Epilogues of the skinny GEMM  Y[M x N] = X[M x K] . W[N x K]^T.
enum Epi {
  EPI_STORE = 1,   // out[m][n]  = y           (LM head logits)
  EPI_QKV = 2,     // rotary (optional) + q store + paged K/V append
  EPI_SWIGLU = 3,  // silu(gate) * up  -> packed activation panel
  EPI_GELU = 4,    // gelu(y)          -> packed activation panel
  EPI_PARTIAL = 5, // h[m][n] += y             (O-projection, MLP down; K may be split over workgroups,
                   //                           partial planes in `out`, last workgroup adds them up)
};

struct GemmArgs {
  const bf16_t* W;      // packed [N x K]
  const bf16_t* X;      // activation panels (see xpack layout in disco_kernels.hip)
  int KT;               // K / 32
  int M;                // live tokens, 1..16
  int n_rows;           // N
  int grp;              // row-tile pairing distance for two-tile workgroups (1 = adjacent tiles)
  const uint32_t* gate; // optional: skip when *gate != 0
  int n_split;          // K ranges (grid.y) of the one-unit-per-workgroup launch
  float* planes;        // partial tiles of row groups whose K range is shared by several workgroups:
                        // [row group][GEMM_MAX_SPLIT][tile of the group][64 lanes][4] fp32
  const float* ssq; int n_ssq; int d_in; float eps;   // deferred RMSNorm of the input (ssq == nullptr: none)
  // deferred LayerNorm of the input (sum != nullptr; needs ssq too): per-tile sums of the row beside the sums of
  // squares, and two vectors over the output rows, wg[n] = sum_k W[n][k] g[k] and wb[n] = sum_k W[n][k] b[k]:
  // W . LN(h) = rstd * (W . (g * h) - mean * wg) + wb
  const float* sum; const float* wg; const float* wb;
  int* counters;        // one zeroed ticket counter per row group (used when a K range is shared)
  float* h;             // PARTIAL: residual stream updated in place, row stride ld_out
  const float* gain; float* ssq_out; int n_ssq_out;   // PARTIAL with Xout: next norm's gain, sums of squares
  float* sum_out;                                     // PARTIAL with Xout, next norm a LayerNorm: per-tile sums too
  float* out;           // STORE target, row stride ld_out
  int64_t ld_out;
  int only_row;         // STORE: write only this token's row to out[0..N) (-1: all rows)
  const unsigned* abort_word;   // STORE, optional: when the word is set (a bounded wait of an earlier launch ran out) NaN is stored
  // QKV epilogue
  float* q; int ldq; int nq, nkv, dh; int pos0;
  const float* rope_tab;  // rotary table [position][d_head / 2][cos, sin], or nullptr for no rotation
  bf16_t* kv_layer; const int32_t* page_table; int page_tokens;
  // packed-activation epilogues
  bf16_t* Xout; int KT_out;
};

// Dense prompt pass: the same GEMM over n_groups groups of 16 tokens in one launch.  g describes
// group 0 (M = 16, two-panel layout); the strides give the distance to the next group's buffers.
struct DenseArgs {
  GemmArgs g;
  int n_groups;
  size_t xs, xouts;     // bf16 elements between the groups' input / output panels
  size_t hs, qs;        // floats between the groups' residual rows / query rows
  size_t ssq_outs;      // floats between the groups' sum-of-squares slots
  const float* rstd;    // [group][16]: 1 / rms of the input rows (epilogues that read a normalised input)
  int hi_only;          // bf16 activations: the lo panels are not read
  int tile_r, tile_t;   // set by the launcher: row blocks x token blocks walked by consecutive workgroups of an XCD
};

struct NormArgs {
  float* h; int d; int M; int layernorm; float eps;
  const float* g; const float* b;
  bf16_t* Xout;                      // packed panels, K = d
  float* ssq_out; int n_ssq_out;     // deferred RMSNorm: write gain * h panels and the row's sum of squares
  float* sum_out;                    // deferred LayerNorm (with ssq_out): the row's sum as well
  // embedding mode (tokens != nullptr): h = tok_emb[token] (+ pos_emb[pos0 + m]) first
  const int32_t* tokens; const bf16_t* tok_emb; int64_t tok_stride; const bf16_t* pos_emb;
  int pos0; int vocab; int max_pos;
  const uint32_t* gate;
  // prompt pass: n_groups > 0 launches 16 * n_groups token slots (M == 16); slots >= n_tok embed token 0
  int n_groups; int n_tok;
};

struct AttnArgs {
  const float* q; int ldq;
  const bf16_t* kv_layer; const int32_t* page_table; int page_tokens;
  int nq, nkv, dh, M, pos0; float scale;
  float* part; int n_splits; int split_len;
  bf16_t* Xout;                      // packed panels, K = nq * dh
  int* counters;                     // one zeroed ticket counter per query head
  const uint32_t* gate;
};

struct ClassifyArgs {
  float* logits; int vocab; const float* clf_params; int hidden;
  float pos_feature; float tau; int force_halt;
  void* out;                         // disco_clf_out*
  int32_t* token_next; int32_t* block_slot; uint32_t* gate; int32_t* sl_count;
  const int32_t* force_token;
  const int32_t* ref_token;          // optional: known continuation; a different arg-max ends the block and stays out of it
  float ppl_threshold;               // > 0: perplexity rule (needs sl_count; the float after it holds -sum ln p of the block)
  float* scratch;                    // optional: >= CLASSIFY_SCRATCH_BYTES, first word zero (ticket counter)
};
struct SampleArgs {
  const float* logits; int64_t ld; int vocab; float inv_t;
  const float* u;                    // one uniform in [0, 1) per row
  float* probs;                      // optional [rows x vocab] probability rows
  int32_t* tokens;                   // [rows]
  int32_t* token_next; int32_t* block_slot;   // optional extra copies of row 0's token
  const uint32_t* gate;
};

struct AcceptSampleArgs {
  const int32_t* block; int n_block; const int32_t* dev_n_block;
  const float* draft_probs;          // [n_block - 1][vocab], row j - 1 = distribution of block[j]
  const float* target_logits;        // [n_block][vocab]
  int vocab; float inv_t;
  const float* u_accept;             // [n_block - 1]
  const float* u_resample;           // [n_block], entry n is used
  void* out; void* host_out;         // disco_accept_out
};

struct TrainArgs {
  const float* feats; const int32_t* labels; int n; int hidden; int epochs; float lr;
  float* params;                     // in: initial (standardised space), out: trained, folded to raw features
  float* loss;                       // optional [epochs]: mean loss before each step
};

struct EvalArgs {
  const float* feats; const int32_t* labels; int n; const float* params; int hidden; float tau;
  float* scores; int* counts;
};

// One launch per forward (or per draft loop) for the RMSNorm / rotary / SwiGLU family: see k_forward.
struct FwdLayer { const bf16_t* wqkv; const bf16_t* wo; const bf16_t* w_in; const bf16_t* w_out; const float* norm1_g; const float* norm2_g; };

struct FwdArgs {
  // model
  int n_layers, d, d_q, d_qkv, d_ff, nq, nkv, dh, vocab; float eps; float attn_scale;
  const FwdLayer* layers;            // DEVICE array of n_layers entries
  const float* normf_g; const bf16_t* wlm;
  const bf16_t* tok_emb; int64_t tok_stride;
  // the forward: M tokens at positions pos0 ..; the residual rows h and the first panel version are already
  // written (embedding launch)
  int M, pos0;
  float* h;
  float* q;                                                // query versions: L per step, 16 x d_q floats each
  bf16_t* xn; bf16_t* xattn; bf16_t* xact;                 // panel versions: (2 L + 1), L and L per step; an xn version is
                                                           // two panels followed by its sums of squares (d floats)
  size_t xn_stride, xattn_stride, xact_stride;             // elements between versions
  float* part; float* planes; int* gemm_counters; int* attn_counters;
  bf16_t* kv_pages; size_t kv_layer_stride; const int32_t* page_table; int page_tokens; const float* rope;
  float* logits; int only_last;
  int split_o, split_dn, attn_split_len;                   // set by the launcher from the grid size
  unsigned* bar;                                           // FWD_BAR_WORDS words of the grid barrier, zeroed before the launch
  // draft loop: n_steps (forward, classify) pairs in one launch; step 0 feeds M tokens, later steps one;
  // clf holds the first step's classify arguments (pos_feature, out, block_slot, force_token, ref_token advance per step)
  int n_steps;
  int open_end;                      // the last step does not force a halt (the block goes on in a further launch)
  ClassifyArgs clf;
};

constexpr size_t CLASSIFY_SCRATCH_BYTES = 256 + 64 * 16 * sizeof(float);

hipError_t launch_pack(const bf16_t* src, int64_t n, int64_t k, bf16_t* dst, int64_t tile_mul,
                       int64_t tile_add, hipStream_t s);
hipError_t launch_gemm(const GemmArgs& a, int epi, hipStream_t s);
int gemm_split_for(int n_rows, int KT, int M);   // K ranges the PARTIAL epilogue should be launched with
hipError_t launch_norm(const NormArgs& a, hipStream_t s);
// one-token activation panel (hi + lo) of an fp32 vector of d elements (d % 32 == 0), or of zeros if v == nullptr
hipError_t launch_vec_panel(const float* v, int d, bf16_t* Xout, hipStream_t s);
bool forward_shape_ok(int d, int d_q, int d_qkv, int d_ff, int dh, int vocab, bool big);
hipError_t launch_forward(const FwdArgs& f, bool big, bool loop, hipStream_t s);
constexpr int FWD_BAR_WORDS = (2 * 16 + 2) * 64;   // group counters, top counter, release words, abort word: 256 bytes apart
constexpr int FWD_BAR_ABORT_WORD = (2 * 16 + 1) * 64;
hipError_t launch_attn(const AttnArgs& a, hipStream_t s);
// QKV projection (EPI_QKV arguments) and attention of one layer in one launch, where the shape allows it (every query
// head with its own K / V head, RMSNorm family): sets *launched; when it stays false nothing was enqueued and the caller
// launches the two kernels.  head_ready: one zeroed counter per query head, QKV_ATTN_READY_SLOT ints apart; abort_word:
// set when a bounded wait inside the launch ran out (results unusable).
constexpr int QKV_ATTN_READY_SLOT = 64;
// wait_limit: polls before a wait gives up (negative: at once).
hipError_t launch_qkv_attn(const GemmArgs& g, const AttnArgs& a, int* head_ready, unsigned* abort_word, int wait_limit, bool* launched,
                           hipStream_t s);
// dense prompt pass (groups of 16 tokens; every group holds 16 rows, surplus rows are padding)
hipError_t launch_gemm_dense(const DenseArgs& a, int epi, hipStream_t s);
hipError_t launch_rstd_groups(const float* ssq, int n_ssq, int d, float eps, float* rstd, int n_groups, hipStream_t s);
hipError_t launch_attn_groups(const AttnArgs& a, int n_groups, size_t x_stride, bool bf16_operands, hipStream_t s);
hipError_t launch_classify(const ClassifyArgs& a, hipStream_t s);
// device address of the current GPU's file-scope classify scratch (CLASSIFY_SCRATCH_BYTES; no allocation)
hipError_t classify_static_scratch(float** out);
hipError_t launch_sample_rows(const SampleArgs& a, int n_rows, hipStream_t s);
hipError_t launch_accept_sample(const AcceptSampleArgs& a, hipStream_t s);
hipError_t launch_clf_train(const TrainArgs& a, hipStream_t s);
hipError_t launch_clf_eval(const EvalArgs& a, hipStream_t s);
hipError_t launch_clf_examples(const void* rec, int n, const int32_t* ref_tokens, float* feats, int32_t* labels, int32_t* tokens,
                               hipStream_t s);
hipError_t launch_argmax_rows(const float* logits, int M, int vocab, int32_t* out, const unsigned* abort_word, hipStream_t s);
hipError_t launch_accept(const int32_t* block, const int32_t* argmax, int n_block,
                         const int32_t* dev_n_block, void* dev_out, void* host_out, hipStream_t s);
hipError_t launch_kv_fill(const bf16_t* src, bf16_t* pages, const int32_t* page_table, int n_layers,
                          int n_pages, int page_tokens, int nkv, int dh, int ctx, hipStream_t s);
hipError_t launch_zero(int* p, int n, hipStream_t s);
hipError_t launch_rope_fill(float* tab, int n_pos, int dh, float base, hipStream_t s);
hipError_t launch_loop_init(uint32_t* gate, int32_t* sl_count, const int32_t* tokens_in, int n_in,
                            void* dev_loop_out, hipStream_t s);
hipError_t launch_put_tokens(int32_t* tokens, int t0, int t1, int n, void* dev_loop_out, void* host_loop_out, hipStream_t s);
hipError_t launch_loop_finish(const int32_t* sl_count, const uint32_t* gate, void* dev_loop_out, void* host_loop_out,
                              const unsigned* abort_word, hipStream_t s);

constexpr int GEMM_MAX_SPLIT = 8;
constexpr int ATTN_SPLIT_LEN = 128;  // fewest cached positions per attention workgroup
int attn_split_len(int total);       // positions per workgroup for a context of `total` positions (a multiple of ATTN_SPLIT_LEN)

}  // namespace disco
