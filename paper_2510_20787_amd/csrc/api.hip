// C ABI of libltea (declared in include/ltea.h): host-side argument validation, workspace carving and
// dispatch to the kernel launchers.  Nothing here allocates, synchronises or keeps state.
#include <math.h>
#include <string.h>

#include <limits.h>

#include <atomic>

#include "ltea_kernels.h"
#include "train_common.h"

using namespace ltea;

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int elem_size(int dtype) { return dtype == LTEA_F32 ? 4 : 2; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
// workspaces are carved into 256-byte aligned parts that the kernels move in 16-byte pieces
bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

int check_cfg(const ltea_cfg* cfg) {
  if (!cfg) return LTEA_EINVAL;
  if (cfg->dtype != LTEA_F32 && cfg->dtype != LTEA_BF16) return LTEA_EINVAL;
  if (cfg->Hq < 1 || cfg->Hkv < 1 || cfg->Hq % cfg->Hkv != 0) return LTEA_EINVAL;
  if (cfg->window < 1 || cfg->budget < 0 || cfg->sink < 0) return LTEA_EINVAL;
  if (isnan(cfg->tau_logit) || isnan(cfg->softmax_scale)) return LTEA_EINVAL;
  if (cfg->D != 64 && cfg->D != 128) return LTEA_EUNSUPPORTED;
  return LTEA_OK;
}

int check_cnn(const ltea_cfg* cfg, const ltea_cnn* cnn) {
  if (!cnn) return LTEA_EINVAL;
  if (cnn->n_layers < 1 || cnn->n_layers > LTEA_MAX_CNN_LAYERS) return LTEA_EINVAL;
  for (int l = 0; l < cnn->n_layers; ++l) {
    if (cnn->kernel[l] < 1 || cnn->kernel[l] % 2 == 0) return LTEA_EINVAL;
    if (cnn->dilation[l] < 1 || cnn->c_out[l] < 1) return LTEA_EINVAL;
    if (!cnn->w[l] || !cnn->bias[l]) return LTEA_EINVAL;
  }
  if (!cnn->w_out || !cnn->b_out) return LTEA_EINVAL;
  if (cfg->window < 2 * cnn_rho(cnn) + 1) return LTEA_EINVAL;  // look-ahead must stay inside the window
  return LTEA_OK;
}

int check_seqs(const int32_t* cu, int32_t n_seqs, int64_t total, int32_t max_seqlen) {
  if (n_seqs < 0 || total < 0 || max_seqlen < 0) return LTEA_EINVAL;
  if (!cu) return LTEA_EINVAL;
  if (total > 0 && (n_seqs == 0 || max_seqlen == 0)) return LTEA_EINVAL;
  if (total > (int64_t)n_seqs * max_seqlen) return LTEA_EINVAL;
  if (total >= (int64_t)1 << 31) return LTEA_EUNSUPPORTED;  // cu_seqlens is int32
  return LTEA_OK;
}

// rows are moved in 16-byte pieces: base pointers and strides must keep every row 16-byte aligned
int check_view(const void* p, int64_t st, int64_t sh, int D, int esz) {
  if (!p) return LTEA_EINVAL;
  if (st < D || sh < D) return LTEA_EINVAL;
  const int64_t per16 = 16 / esz;
  if (st % per16 != 0 || sh % per16 != 0 || !aligned16(p)) return LTEA_EINVAL;
  return LTEA_OK;
}

int check_rope(const ltea_cfg* cfg, const ltea_rope* rope) {
  if (!rope->cos || !rope->sin || rope->n_pos < 1) return LTEA_EINVAL;
  if (rope->rot_dim < 16 || rope->rot_dim > cfg->D || rope->rot_dim % 16 != 0) return LTEA_EINVAL;
  if (rope->interleaved != 0 && rope->interleaved != 1) return LTEA_EINVAL;
  return LTEA_OK;
}

int check_cache(const ltea_cfg* cfg, const ltea_cache* c, bool need_window) {
  if (!c) return LTEA_EINVAL;
  if (!c->ret_count || !c->n_seen || !c->n_scored) return LTEA_EINVAL;
  if (cfg->budget > 0 && (!c->k_ret || !c->v_ret || !c->ret_score || !c->ret_pos)) return LTEA_EINVAL;
  if (need_window && (!c->k_win || !c->v_win || !c->win_score)) return LTEA_EINVAL;
  if (!aligned16(c->k_ret) || !aligned16(c->v_ret) || !aligned16(c->k_win) || !aligned16(c->v_win)) return LTEA_EINVAL;
  return LTEA_OK;
}

bool use_score_mfma(const ltea_cfg& cfg, const ltea_cnn& cnn) { return score_mfma_supported(cfg, cnn); }

size_t score_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn, int64_t total) {
  if (use_score_mfma(cfg, cnn)) return align_up(score_mfma_workspace(cfg, cnn), 256);
  if (score_deep_supported(cfg, cnn)) return align_up(score_deep_workspace(cfg, cnn), 256);
  return align_up(score_generic_workspace(cfg, cnn, total), 256);
}

int hip_status(hipError_t e) { return e == hipSuccess ? LTEA_OK : LTEA_EHIP; }

int do_score(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st, int64_t sh,
             const SeqView& sv, float* logits, void* ws, hipStream_t stream) {
  // The matrix-core kernels are chosen from (cfg, cnn) alone, which is also what sizes their workspace; a token
  // stride beyond their 32-bit row offsets (above a million elements) is refused rather than scored wrongly.
  const bool mfma = use_score_mfma(cfg, cnn), deep = !mfma && score_deep_supported(cfg, cnn);
  if ((mfma || deep) && !score_stride_ok(st)) return LTEA_EUNSUPPORTED;
  if (mfma) return hip_status(launch_score_mfma(cfg, cnn, k, v, st, sh, sv, logits, ws, stream));
  if (deep) return hip_status(launch_score_deep(cfg, cnn, k, v, st, sh, sv, logits, ws, stream));
  return hip_status(launch_score_generic(cfg, cnn, k, v, st, sh, sv, logits, ws, stream));
}

int do_attention(const ltea_cfg& cfg, const void* q, int64_t qst, int64_t qsh, const void* k, const void* v,
                 int64_t st, int64_t sh, const SeqView& sv, const ltea_cache& c, void* out, hipStream_t stream,
                 float* lse = nullptr) {
  if (attention_mfma_supported(cfg, st, sv.max_seqlen))
    return hip_status(launch_attention_mfma(cfg, q, qst, qsh, k, v, st, sh, sv, c, out, stream, nullptr, nullptr, lse));
  return hip_status(launch_attention_generic(cfg, q, qst, qsh, k, v, st, sh, sv, c, out, stream, lse));
}

// Saved state of a training forward, carved from the caller's workspace: an uncapped cache (compact arrays with
// max_seqlen rows per head), the delta scratch of the backward, then the scoring kernels' own workspace.
size_t carve_train(const ltea_cfg& cfg, int n_seqs, int64_t total, int max_seqlen, void* base, ltea_cache* c,
                   float** delta, float** far_dk = nullptr, float** far_dv = nullptr) {
  const size_t esz = (size_t)elem_size(cfg.dtype);
  const size_t heads = (size_t)n_seqs * cfg.Hkv;
  const size_t cap = (size_t)(max_seqlen > 1 ? max_seqlen : 1);
  // integer arithmetic: a size query carves from a null base
  uintptr_t p = reinterpret_cast<uintptr_t>(base);
  auto take = [&](size_t bytes) { char* r = reinterpret_cast<char*>(p); p += align_up(bytes > 0 ? bytes : 1, 256); return r; };
  void* k_ret = take(heads * cap * cfg.D * esz);
  void* v_ret = take(heads * cap * cfg.D * esz);
  float* ret_score = reinterpret_cast<float*>(take(heads * cap * 4));
  int32_t* ret_pos = reinterpret_cast<int32_t*>(take(heads * cap * 4));
  int32_t* ret_count = reinterpret_cast<int32_t*>(take(heads * 4));
  void* k_win = take(heads * cfg.window * cfg.D * esz);
  void* v_win = take(heads * cfg.window * cfg.D * esz);
  float* win_score = reinterpret_cast<float*>(take(heads * cfg.window * 4));
  int32_t* n_seen = reinterpret_cast<int32_t*>(take((size_t)n_seqs * 4));
  int32_t* n_scored = reinterpret_cast<int32_t*>(take((size_t)n_seqs * 4));
  float* d = reinterpret_cast<float*>(take((size_t)cfg.Hq * (size_t)total * 4));
  float* fk = reinterpret_cast<float*>(take((size_t)train_far_chunks(n_seqs, cfg.Hkv) * heads * cap * cfg.D * 4));
  float* fv = reinterpret_cast<float*>(take((size_t)train_far_chunks(n_seqs, cfg.Hkv) * heads * cap * cfg.D * 4));
  if (far_dk) *far_dk = fk;
  if (far_dv) *far_dv = fv;
  if (c) *c = ltea_cache{k_win, v_win, win_score, k_ret, v_ret, ret_score, ret_pos, ret_count, n_seen, n_scored};
  if (delta) *delta = d;
  return (size_t)(p - reinterpret_cast<uintptr_t>(base));
}

}  // namespace

extern "C" {

size_t ltea_cnn_panels_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn) {
  if (check_cfg(cfg) != LTEA_OK || check_cnn(cfg, cnn) != LTEA_OK) return 0;
  if (use_score_mfma(*cfg, *cnn)) return align_up(score_mfma_workspace(*cfg, *cnn), 256);
  if (score_deep_supported(*cfg, *cnn)) return align_up(score_deep_workspace(*cfg, *cnn), 256);
  return 0;
}

int ltea_cnn_prepare(const ltea_cfg* cfg, const ltea_cnn* cnn, void* panels, size_t panels_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st != LTEA_OK) return st;
  const size_t need = ltea_cnn_panels_bytes(cfg, cnn);
  if (need == 0) return LTEA_OK;                      // this configuration's kernels read the weights as they are
  if (!panels || !aligned16(panels) || panels_bytes < need) return LTEA_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (use_score_mfma(*cfg, *cnn)) return hip_status(launch_score_mfma_panels(*cfg, *cnn, panels, s));
  return hip_status(launch_score_deep_panels(*cfg, *cnn, panels, s));
}

const char* ltea_strerror(int status) {
  switch (status) {
    case LTEA_OK: return "ok";
    case LTEA_EINVAL: return "invalid argument (null pointer, size, stride, alignment or inconsistent config)";
    case LTEA_EUNSUPPORTED: return "configuration not supported by the gfx950 kernels";
    case LTEA_EWORKSPACE: return "workspace missing or too small (or the request exceeds the fixed scratch of a *_static entry point)";
    case LTEA_EHIP: return "HIP runtime rejected a kernel launch";
    default: return "unknown ltea status";
  }
}

size_t ltea_workspace_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn, int32_t n_seqs, int64_t total_tokens,
                            int32_t max_seqlen) {
  (void)n_seqs; (void)max_seqlen;
  if (check_cfg(cfg) != LTEA_OK || total_tokens < 0) return 0;
  size_t bytes = 0;
  if (cnn) {
    if (check_cnn(cfg, cnn) != LTEA_OK) return 0;
    bytes += align_up((size_t)cfg->Hkv * (size_t)total_tokens * sizeof(float), 256);  // logits when not returned
    bytes += score_workspace(*cfg, *cnn, total_tokens);
  }
  return bytes;
}

// The per-(sequence, head) scoring of the eager step keeps two generations of (2 rho + 1) activation rows in LDS.
static bool decode_pyramid_fits(const ltea_cfg* cfg, const ltea_cnn* cnn) {
  int row_floats = 2 * cfg->D;
  for (int l = 0; l < cnn->n_layers; ++l) row_floats = cnn->c_out[l] > row_floats ? cnn->c_out[l] : row_floats;
  return (size_t)2 * (2 * cnn_rho(cnn) + 1) * row_floats * sizeof(float) <= 48 * 1024;
}

static size_t decode_scored_workspace(const ltea_cfg* cfg, const ltea_cnn* cnn, int32_t n_seqs) {
  const int rho = cnn_rho(cnn);
  return align_up(decode_workspace(*cfg, n_seqs), 256) + align_up(decode_windows_layout(*cfg, rho, n_seqs, nullptr, nullptr), 256) +
         score_workspace(*cfg, *cnn, (int64_t)n_seqs * (2 * rho + 1));
}

size_t ltea_decode_workspace_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn, int32_t n_seqs) {
  if (check_cfg(cfg) != LTEA_OK || n_seqs < 0) return 0;
  if (cnn && check_cnn(cfg, cnn) != LTEA_OK) return 0;
  if (!cnn) return align_up(decode_workspace(*cfg, n_seqs), 256);
  const size_t full = align_up(decode_workspace_full(*cfg, *cnn, n_seqs), 256);
  if (decode_pyramid_fits(cfg, cnn)) return full;
  const size_t scored = decode_scored_workspace(cfg, cnn, n_seqs);   // such CNNs are scored through the prefill kernels
  return scored > full ? scored : full;
}

int ltea_score(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* k, const void* v, int64_t stride_tok,
               int64_t stride_head, const int32_t* cu_seqlens, int32_t n_seqs, int64_t total_tokens,
               int32_t max_seqlen, float* logits, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_seqs(cu_seqlens, n_seqs, total_tokens, max_seqlen);
  if (st != LTEA_OK) return st;
  if (total_tokens == 0) return LTEA_OK;
  const int esz = elem_size(cfg->dtype);
  if ((st = check_view(k, stride_tok, stride_head, cfg->D, esz)) != LTEA_OK) return st;
  if ((st = check_view(v, stride_tok, stride_head, cfg->D, esz)) != LTEA_OK) return st;
  if (!logits) return LTEA_EINVAL;
  const size_t need = score_workspace(*cfg, *cnn, total_tokens);
  if (need > 0 && (!workspace || workspace_bytes < need)) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  SeqView sv{cu_seqlens, n_seqs, total_tokens, max_seqlen};
  return do_score(*cfg, *cnn, k, v, stride_tok, stride_head, sv, logits, workspace, static_cast<hipStream_t>(stream));
}

int ltea_retain(const ltea_cfg* cfg, const float* logits, const void* k, const void* v, int64_t stride_tok,
                int64_t stride_head, const int32_t* cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                int32_t max_seqlen, int32_t rho, const ltea_cache* cache, void* workspace, size_t workspace_bytes,
                void* stream) {
  (void)workspace; (void)workspace_bytes;
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_seqs(cu_seqlens, n_seqs, total_tokens, max_seqlen);
  if (st == LTEA_OK) st = check_cache(cfg, cache, true);
  if (st != LTEA_OK) return st;
  if (rho < 0 || cfg->window < 2 * rho + 1) return LTEA_EINVAL;
  if (n_seqs == 0) return LTEA_OK;
  const int esz = elem_size(cfg->dtype);
  if (total_tokens > 0) {
    if ((st = check_view(k, stride_tok, stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(v, stride_tok, stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if (!logits) return LTEA_EINVAL;
  }
  SeqView sv{cu_seqlens, n_seqs, total_tokens, max_seqlen};
  return hip_status(launch_retain(*cfg, logits, k, v, stride_tok, stride_head, sv, rho, *cache,
                                  static_cast<hipStream_t>(stream)));
}

int ltea_sparse_attention(const ltea_cfg* cfg, const void* q, int64_t q_stride_tok, int64_t q_stride_head,
                          const void* k, const void* v, int64_t kv_stride_tok, int64_t kv_stride_head,
                          const int32_t* cu_seqlens, int32_t n_seqs, int64_t total_tokens, int32_t max_seqlen,
                          const ltea_cache* cache, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_seqs(cu_seqlens, n_seqs, total_tokens, max_seqlen);
  if (st == LTEA_OK) st = check_cache(cfg, cache, false);
  if (st != LTEA_OK) return st;
  if (total_tokens == 0) return LTEA_OK;
  const int esz = elem_size(cfg->dtype);
  if ((st = check_view(q, q_stride_tok, q_stride_head, cfg->D, esz)) != LTEA_OK) return st;
  if ((st = check_view(k, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
  if ((st = check_view(v, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
  if (!out || !aligned16(out)) return LTEA_EINVAL;
  SeqView sv{cu_seqlens, n_seqs, total_tokens, max_seqlen};
  return do_attention(*cfg, q, q_stride_tok, q_stride_head, k, v, kv_stride_tok, kv_stride_head, sv, *cache, out,
                      static_cast<hipStream_t>(stream));
}

int ltea_prefill_feat(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* q, int64_t q_stride_tok,
                      int64_t q_stride_head, const void* k, const void* v, const void* k_feat, int64_t kv_stride_tok,
                      int64_t kv_stride_head, const int32_t* cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                      int32_t max_seqlen, void* out, const ltea_cache* cache, float* logits_or_null, void* workspace,
                      size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_seqs(cu_seqlens, n_seqs, total_tokens, max_seqlen);
  if (st == LTEA_OK) st = check_cache(cfg, cache, true);
  if (st != LTEA_OK) return st;
  if (n_seqs == 0) return LTEA_OK;
  const int esz = elem_size(cfg->dtype);
  if (total_tokens > 0) {
    if ((st = check_view(q, q_stride_tok, q_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(k, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(v, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(k_feat, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if (!out || !aligned16(out)) return LTEA_EINVAL;
  }
  const size_t logits_bytes = align_up((size_t)cfg->Hkv * (size_t)total_tokens * sizeof(float), 256);
  const size_t score_ws = score_workspace(*cfg, *cnn, total_tokens);
  const size_t need = (logits_or_null ? 0 : logits_bytes) + score_ws;
  if (need > 0 && (!workspace || workspace_bytes < need)) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  char* ws = static_cast<char*>(workspace);
  float* logits = logits_or_null;
  if (!logits) { logits = reinterpret_cast<float*>(ws); ws += logits_bytes; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  SeqView sv{cu_seqlens, n_seqs, total_tokens, max_seqlen};
  if (total_tokens > 0) {
    st = do_score(*cfg, *cnn, k_feat, v, kv_stride_tok, kv_stride_head, sv, logits, ws, s);
    if (st != LTEA_OK) return st;
  }
  st = hip_status(launch_retain(*cfg, logits, k, v, kv_stride_tok, kv_stride_head, sv, cnn_rho(cnn), *cache, s));
  if (st != LTEA_OK) return st;
  if (total_tokens == 0) return LTEA_OK;
  return do_attention(*cfg, q, q_stride_tok, q_stride_head, k, v, kv_stride_tok, kv_stride_head, sv, *cache, out, s);
}

int ltea_prefill(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* q, int64_t q_stride_tok, int64_t q_stride_head,
                 const void* k, const void* v, int64_t kv_stride_tok, int64_t kv_stride_head,
                 const int32_t* cu_seqlens, int32_t n_seqs, int64_t total_tokens, int32_t max_seqlen, void* out,
                 const ltea_cache* cache, float* logits_or_null, void* workspace, size_t workspace_bytes,
                 void* stream) {
  return ltea_prefill_feat(cfg, cnn, q, q_stride_tok, q_stride_head, k, v, k, kv_stride_tok, kv_stride_head, cu_seqlens,
                           n_seqs, total_tokens, max_seqlen, out, cache, logits_or_null, workspace, workspace_bytes,
                           stream);
}

size_t ltea_append_workspace_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn, int32_t n_seqs, int64_t total_new,
                                   int32_t max_new) {
  (void)max_new;
  if (check_cfg(cfg) != LTEA_OK || !cnn || check_cnn(cfg, cnn) != LTEA_OK || n_seqs < 0 || total_new < 0) return 0;
  const int64_t ext = append_ext_tokens(*cfg, n_seqs, total_new);
  return align_up(append_workspace(*cfg, n_seqs, total_new, true), 256) + score_workspace(*cfg, *cnn, ext);
}

int ltea_prefill_append(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* q, int64_t q_stride_tok,
                        int64_t q_stride_head, const void* k, const void* v, int64_t kv_stride_tok,
                        int64_t kv_stride_head, const int32_t* cu_new, int32_t n_seqs, int64_t total_new,
                        int32_t max_new, void* out, const ltea_cache* cache, void* workspace, size_t workspace_bytes,
                        void* stream) {
  return ltea_prefill_append_feat(cfg, cnn, nullptr, q, q_stride_tok, q_stride_head, k, v, nullptr, kv_stride_tok,
                                  kv_stride_head, cu_new, n_seqs, total_new, max_new, out, cache, nullptr, workspace,
                                  workspace_bytes, stream);
}

int ltea_prefill_append_feat(const ltea_cfg* cfg, const ltea_cnn* cnn, const ltea_rope* rope, const void* q,
                             int64_t q_stride_tok, int64_t q_stride_head, const void* k, const void* v,
                             const void* k_feat, int64_t kv_stride_tok, int64_t kv_stride_head, const int32_t* cu_new,
                             int32_t n_seqs, int64_t total_new, int32_t max_new, void* out, const ltea_cache* cache,
                             int32_t* status, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_seqs(cu_new, n_seqs, total_new, max_new);
  if (st == LTEA_OK) st = check_cache(cfg, cache, true);
  if (st == LTEA_OK && rope) st = check_rope(cfg, rope);
  if (st != LTEA_OK) return st;
  // without the sinusoids there is no way back from the cached keys to the ones the CNN scored
  if (k_feat && !rope) return LTEA_EINVAL;
  if (n_seqs == 0) return LTEA_OK;
  const int esz = elem_size(cfg->dtype);
  if (total_new > 0) {
    if ((st = check_view(q, q_stride_tok, q_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(k, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(v, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if (k_feat && (st = check_view(k_feat, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if (!out || !aligned16(out)) return LTEA_EINVAL;
  }
  const int64_t ext_stride_tok = (int64_t)cfg->Hkv * cfg->D;
  const int64_t ext_len_max = (int64_t)cfg->budget + 2 * (int64_t)cfg->window + max_new;
  if (ext_len_max > INT32_MAX / 2) return LTEA_EUNSUPPORTED;
  const int64_t ext = append_ext_tokens(*cfg, n_seqs, total_new);
  if (ext >= (int64_t)1 << 31) return LTEA_EUNSUPPORTED;   // the packed extended sequences are indexed by int32 prefix sums
  const size_t build_ws = align_up(append_workspace(*cfg, n_seqs, total_new, rope != nullptr), 256);
  const size_t need = build_ws + score_workspace(*cfg, *cnn, ext);
  if (!workspace || workspace_bytes < need) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int rho = cnn_rho(cnn);
  AppendBuffers buf;
  st = hip_status(launch_append_build(*cfg, k, v, k_feat, kv_stride_tok, kv_stride_head, cu_new, n_seqs, total_new,
                                      max_new, rope, status, *cache, workspace, &buf, s));
  if (st != LTEA_OK) return st;
  SeqView sv_ext{buf.cu_ext, n_seqs, buf.total_ext, buf.max_ext_len};
  SeqView sv_score{buf.cu_score, n_seqs, buf.total_ext, 2 * buf.max_ext_len};
  st = do_score(*cfg, *cnn, buf.ext_kf, buf.ext_v, ext_stride_tok, cfg->D, sv_score, buf.ext_logits,
                static_cast<char*>(workspace) + build_ws, s);
  if (st != LTEA_OK) return st;
  st = hip_status(launch_append_keys(*cfg, n_seqs, total_new, *cache, rho, workspace, buf, s));
  if (st != LTEA_OK) return st;
  ltea_cfg sel = *cfg;
  sel.sink = 0;     // sinks already carry the key +inf in the extended sequence
  st = hip_status(launch_retain(sel, buf.ext_logits, buf.ext_k, buf.ext_v, ext_stride_tok, cfg->D, sv_ext, rho, *cache, s));
  if (st != LTEA_OK) return st;
  st = hip_status(launch_append_fixup(*cfg, cu_new, n_seqs, total_new, *cache, rho, workspace, s));
  if (st != LTEA_OK) return st;
  if (total_new == 0) return LTEA_OK;
  ltea_cache local = *cache;
  local.ret_pos = buf.local_pos;
  SeqView sv_q{cu_new, n_seqs, total_new, max_new};
  if (attention_mfma_supported(*cfg, ext_stride_tok, (int32_t)ext_len_max))
    return hip_status(launch_attention_mfma(*cfg, q, q_stride_tok, q_stride_head, buf.ext_k, buf.ext_v, ext_stride_tok,
                                            cfg->D, sv_q, local, out, s, buf.kv_start, buf.kv_len));
  return hip_status(launch_attention_generic(*cfg, q, q_stride_tok, q_stride_head, buf.ext_k, buf.ext_v, ext_stride_tok,
                                             cfg->D, sv_q, local, out, s, nullptr, buf.kv_start, buf.kv_len));
}

int ltea_decode_step(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* q, const void* k, const void* v, void* out,
                     const ltea_cache* cache, int32_t n_seqs, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_cache(cfg, cache, true);
  if (st != LTEA_OK) return st;
  if (n_seqs < 0) return LTEA_EINVAL;
  if (n_seqs == 0) return LTEA_OK;
  if (!q || !k || !v || !out) return LTEA_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return LTEA_EINVAL;
  // A CNN whose per-step activation rows do not fit LDS goes through the packed-window path (needs the workspace
  // ltea_decode_workspace_bytes(cfg, cnn, n_seqs) reports for it).
  if (!decode_pyramid_fits(cfg, cnn))
    return ltea_decode_step_feat(cfg, cnn, nullptr, q, k, v, nullptr, out, cache, n_seqs, nullptr, workspace,
                                 workspace_bytes, stream);
  const size_t need = align_up(decode_workspace(*cfg, n_seqs), 256);
  if (!workspace || workspace_bytes < need) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  return hip_status(launch_decode_step(*cfg, *cnn, q, k, v, out, *cache, n_seqs, workspace, workspace_bytes,
                                       static_cast<hipStream_t>(stream)));
}

// ---- the decode step for callers that cannot allocate ----------------------------------------------------------
// Its scratch (split partials, finalised logits, step indices: everything ltea_decode_step carves from a caller
// workspace) lives in a file-scope device array.  Host code never passes the array's name to a kernel: the name is a
// host-side stand-in, the device address comes from hipGetSymbolAddress, looked up once per device (each GPU holds
// its own copy at its own address) with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[LTEA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device; nullptr (and *err set) if the runtime refuses.
void* static_scratch(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // racing first calls store the same address
  }
  return p;
}
}  // namespace

int ltea_decode_step_static(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* q, const void* k, const void* v,
                            void* out, const ltea_cache* cache, int32_t n_seqs, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st != LTEA_OK) return st;
  if (n_seqs < 0) return LTEA_EINVAL;
  // beyond the fixed scratch: refused here, before anything is looked up or launched
  if (ltea_decode_workspace_bytes(cfg, cnn, n_seqs) > (size_t)LTEA_STATIC_SCRATCH_BYTES) return LTEA_EWORKSPACE;
  if (n_seqs == 0) return ltea_decode_step(cfg, cnn, q, k, v, out, cache, 0, nullptr, 0, stream);
  if (!q || !k || !v || !out || !cache) return LTEA_EINVAL;     // before the device is asked for the array's address
  hipError_t e = hipSuccess;
  void* ws = static_scratch(&e);
  if (ws == nullptr) return LTEA_EHIP;
  // nothing in the scratch has to start at zero: every part is written by the step's first launch before its
  // second launch reads it
  return ltea_decode_step(cfg, cnn, q, k, v, out, cache, n_seqs, ws, (size_t)LTEA_STATIC_SCRATCH_BYTES, stream);
}

size_t ltea_decode_feat_workspace_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn, int32_t n_seqs) {
  if (check_cfg(cfg) != LTEA_OK || check_cnn(cfg, cnn) != LTEA_OK || n_seqs < 0) return 0;
  return decode_scored_workspace(cfg, cnn, n_seqs);
}

int ltea_decode_step_feat(const ltea_cfg* cfg, const ltea_cnn* cnn, const ltea_rope* rope, const void* q, const void* k,
                          const void* v, const void* k_feat, void* out, const ltea_cache* cache, int32_t n_seqs,
                          int32_t* status, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_cache(cfg, cache, true);
  if (st == LTEA_OK && rope) st = check_rope(cfg, rope);
  if (st != LTEA_OK) return st;
  if (n_seqs < 0) return LTEA_EINVAL;
  if (k_feat && !rope) return LTEA_EINVAL;   // no way back from the cached keys without the sinusoids
  if (n_seqs == 0) return LTEA_OK;
  if (!q || !k || !v || !out) return LTEA_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || (k_feat && !aligned16(k_feat))) return LTEA_EINVAL;
  const int rho = cnn_rho(cnn);
  const int64_t rows = (int64_t)n_seqs * (2 * rho + 1);
  if (rows >= (int64_t)1 << 30) return LTEA_EUNSUPPORTED;
  const size_t step_ws = align_up(decode_workspace(*cfg, n_seqs), 256);
  const size_t win_ws = align_up(decode_windows_layout(*cfg, rho, n_seqs, nullptr, nullptr), 256);
  if (!workspace || workspace_bytes < step_ws + win_ws + score_workspace(*cfg, *cnn, rows)) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(workspace);
  DecodeWindows w;
  decode_windows_layout(*cfg, rho, n_seqs, base + step_ws, &w);
  st = hip_status(launch_decode_windows(*cfg, rho, k, v, k_feat, rope, status, *cache, n_seqs, w, s));
  if (st != LTEA_OK) return st;
  SeqView sv{w.cu2, 2 * n_seqs, rows, 2 * rho + 1};
  st = do_score(*cfg, *cnn, w.win_k, w.win_v, (int64_t)cfg->Hkv * cfg->D, cfg->D, sv, w.logits, base + step_ws + win_ws, s);
  if (st != LTEA_OK) return st;
  return hip_status(launch_decode_step_scored(*cfg, *cnn, q, k, v, out, *cache, n_seqs, workspace, w.logits, rows, s));
}

int32_t ltea_lazy_period(const ltea_cfg* cfg, const ltea_cnn* cnn) {
  if (check_cfg(cfg) != LTEA_OK || check_cnn(cfg, cnn) != LTEA_OK) return 0;
  return cfg->window - 2 * cnn_rho(cnn);
}

size_t ltea_rescore_workspace_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn, int32_t n_seqs) {
  if (check_cfg(cfg) != LTEA_OK || check_cnn(cfg, cnn) != LTEA_OK || n_seqs < 0) return 0;
  return align_up(rescore_workspace(*cfg, n_seqs, nullptr, nullptr), 256) +
         score_workspace(*cfg, *cnn, (int64_t)n_seqs * cfg->window);
}

int ltea_rescore(const ltea_cfg* cfg, const ltea_cnn* cnn, const ltea_rope* rope, const ltea_cache* cache,
                 int32_t n_seqs, int32_t* status, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_cache(cfg, cache, true);
  if (st != LTEA_OK) return st;
  if (n_seqs < 0) return LTEA_EINVAL;
  if (rope && (st = check_rope(cfg, rope)) != LTEA_OK) return st;
  if (n_seqs == 0) return LTEA_OK;
  const int64_t total = (int64_t)n_seqs * cfg->window;
  if (total >= (int64_t)1 << 31) return LTEA_EUNSUPPORTED;
  const size_t pack_ws = align_up(rescore_workspace(*cfg, n_seqs, nullptr, nullptr), 256);
  const size_t need = pack_ws + score_workspace(*cfg, *cnn, total);
  if (!workspace || workspace_bytes < need) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  RescoreBuffers buf;
  rescore_workspace(*cfg, n_seqs, &buf, workspace);
  st = hip_status(launch_rescore_pack(*cfg, rope, *cache, n_seqs, cnn_rho(cnn), status, buf, s));
  if (st != LTEA_OK) return st;
  SeqView sv{buf.cu, n_seqs, total, cfg->window};
  st = do_score(*cfg, *cnn, buf.pk, buf.pv, (int64_t)cfg->Hkv * cfg->D, cfg->D, sv, buf.logits,
                static_cast<char*>(workspace) + pack_ws, s);
  if (st != LTEA_OK) return st;
  return hip_status(launch_rescore_scatter(*cfg, *cache, n_seqs, buf, s));
}

int ltea_decode_step_lazy(const ltea_cfg* cfg, const void* q, const void* k, const void* v, void* out,
                          const ltea_cache* cache, int32_t n_seqs, int32_t* status, void* workspace,
                          size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cache(cfg, cache, true);
  if (st != LTEA_OK) return st;
  if (n_seqs < 0) return LTEA_EINVAL;
  if (n_seqs == 0) return LTEA_OK;
  if (!q || !k || !v || !out) return LTEA_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return LTEA_EINVAL;
  const size_t need = align_up(decode_workspace(*cfg, n_seqs), 256);
  if (!workspace || workspace_bytes < need) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  return hip_status(launch_decode_step_lazy(*cfg, q, k, v, out, *cache, n_seqs, status, workspace,
                                            static_cast<hipStream_t>(stream)));
}

size_t ltea_train_workspace_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn, int32_t n_seqs, int64_t total_tokens,
                                  int32_t max_seqlen) {
  if (check_cfg(cfg) != LTEA_OK || (cnn && check_cnn(cfg, cnn) != LTEA_OK) || n_seqs < 0 || total_tokens < 0 ||
      max_seqlen < 0)
    return 0;
  return carve_train(*cfg, n_seqs, total_tokens, max_seqlen, nullptr, nullptr, nullptr) +
         (cnn ? score_workspace(*cfg, *cnn, total_tokens) : 0);
}

int ltea_train_forward(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* q, int64_t q_stride_tok,
                       int64_t q_stride_head, const void* k, const void* v, int64_t kv_stride_tok,
                       int64_t kv_stride_head, const int32_t* cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                       int32_t max_seqlen, int32_t rho, void* out, float* lse, float* logits, void* workspace,
                       size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK && cnn) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_seqs(cu_seqlens, n_seqs, total_tokens, max_seqlen);
  if (st != LTEA_OK) return st;
  if (cnn) rho = cnn_rho(cnn);
  if (rho < 0 || cfg->window < 2 * rho + 1) return LTEA_EINVAL;
  if (n_seqs == 0) return LTEA_OK;
  const int esz = elem_size(cfg->dtype);
  if (total_tokens > 0) {
    if ((st = check_view(q, q_stride_tok, q_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(k, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(v, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if (!out || !aligned16(out) || !lse || !logits) return LTEA_EINVAL;
  }
  const size_t saved = carve_train(*cfg, n_seqs, total_tokens, max_seqlen, nullptr, nullptr, nullptr);
  const size_t need = saved + (cnn ? score_workspace(*cfg, *cnn, total_tokens) : 0);
  if (!workspace || workspace_bytes < need) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  ltea_cache cache;
  carve_train(*cfg, n_seqs, total_tokens, max_seqlen, workspace, &cache, nullptr);
  ltea_cfg open = *cfg;
  open.budget = max_seqlen;           // every candidate is kept: no cap during training
  hipStream_t s = static_cast<hipStream_t>(stream);
  SeqView sv{cu_seqlens, n_seqs, total_tokens, max_seqlen};
  if (cnn && total_tokens > 0) {
    st = do_score(*cfg, *cnn, k, v, kv_stride_tok, kv_stride_head, sv, logits, static_cast<char*>(workspace) + saved, s);
    if (st != LTEA_OK) return st;
  }
  st = hip_status(launch_retain(open, logits, k, v, kv_stride_tok, kv_stride_head, sv, rho, cache, s));
  if (st != LTEA_OK || total_tokens == 0) return st;
  return do_attention(open, q, q_stride_tok, q_stride_head, k, v, kv_stride_tok, kv_stride_head, sv, cache, out, s, lse);
}

int ltea_train_backward(const ltea_cfg* cfg, const void* q, int64_t q_stride_tok, int64_t q_stride_head, const void* k,
                        const void* v, int64_t kv_stride_tok, int64_t kv_stride_head, const int32_t* cu_seqlens,
                        int32_t n_seqs, int64_t total_tokens, int32_t max_seqlen, const void* out, const void* dout,
                        const float* lse, const float* logits, const float* lambda, void* dq, void* dk, void* dv,
                        float* dz, int32_t* counts, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_seqs(cu_seqlens, n_seqs, total_tokens, max_seqlen);
  if (st != LTEA_OK) return st;
  if (n_seqs == 0) return LTEA_OK;
  if (!lambda || !counts) return LTEA_EINVAL;
  const int esz = elem_size(cfg->dtype);
  if (total_tokens > 0) {
    if ((st = check_view(q, q_stride_tok, q_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(k, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if ((st = check_view(v, kv_stride_tok, kv_stride_head, cfg->D, esz)) != LTEA_OK) return st;
    if (!out || !dout || !lse || !logits || !dq || !dk || !dv || !dz) return LTEA_EINVAL;
  }
  const size_t saved = carve_train(*cfg, n_seqs, total_tokens, max_seqlen, nullptr, nullptr, nullptr);
  if (!workspace || workspace_bytes < saved) return LTEA_EWORKSPACE;
  if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  ltea_cache cache;
  float *delta = nullptr, *far_dk = nullptr, *far_dv = nullptr;
  carve_train(*cfg, n_seqs, total_tokens, max_seqlen, workspace, &cache, &delta, &far_dk, &far_dv);
  SeqView sv{cu_seqlens, n_seqs, total_tokens, max_seqlen};
  return hip_status(launch_train_backward(*cfg, q, q_stride_tok, q_stride_head, k, v, kv_stride_tok, kv_stride_head, sv,
                                          out, dout, lse, logits, lambda, cache, max_seqlen > 1 ? max_seqlen : 1, delta, far_dk, far_dv, dq, dk, dv, dz,
                                          counts,
                                          static_cast<hipStream_t>(stream)));
}

size_t ltea_cnn_backward_workspace_bytes(const ltea_cfg* cfg, const ltea_cnn* cnn, int64_t total_tokens) {
  if (check_cfg(cfg) != LTEA_OK || check_cnn(cfg, cnn) != LTEA_OK || total_tokens < 0) return 0;
  return align_up(cnn_backward_workspace(*cfg, *cnn, total_tokens), 256);
}

int ltea_cnn_backward(const ltea_cfg* cfg, const ltea_cnn* cnn, const void* k_feat, const void* v, int64_t stride_tok,
                      int64_t stride_head, const int32_t* cu_seqlens, int32_t n_seqs, int64_t total_tokens,
                      int32_t max_seqlen, const float* dz, const ltea_cnn_grad* grad, void* dk_feat, void* dv,
                      void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_cfg(cfg);
  if (st == LTEA_OK) st = check_cnn(cfg, cnn);
  if (st == LTEA_OK) st = check_seqs(cu_seqlens, n_seqs, total_tokens, max_seqlen);
  if (st != LTEA_OK) return st;
  if (!grad || !grad->w_out || !grad->b_out) return LTEA_EINVAL;
  for (int l = 0; l < cnn->n_layers; ++l)
    if (!grad->w[l] || !grad->bias[l]) return LTEA_EINVAL;
  if (total_tokens >= (int64_t)1 << 31) return LTEA_EUNSUPPORTED;   // token bounds are kept as int32
  if (total_tokens > 0) {
    if ((st = check_view(k_feat, stride_tok, stride_head, cfg->D, elem_size(cfg->dtype))) != LTEA_OK) return st;
    if ((st = check_view(v, stride_tok, stride_head, cfg->D, elem_size(cfg->dtype))) != LTEA_OK) return st;
    if (!dz) return LTEA_EINVAL;
    if ((dk_feat && !aligned16(dk_feat)) || (dv && !aligned16(dv))) return LTEA_EINVAL;
    if (!workspace || workspace_bytes < cnn_backward_workspace(*cfg, *cnn, total_tokens)) return LTEA_EWORKSPACE;
    if (workspace && !aligned256(workspace)) return LTEA_EINVAL;
  }
  SeqView sv{cu_seqlens, n_seqs, total_tokens, max_seqlen};
  return hip_status(launch_cnn_backward(*cfg, *cnn, k_feat, v, stride_tok, stride_head, sv, dz, *grad, dk_feat, dv,
                                        workspace, static_cast<hipStream_t>(stream)));
}

int ltea_lambda_update(float* lambda, const float* c_bar, int32_t n, float cap, float alpha) {
  if (!lambda || !c_bar || n < 0 || !(alpha > 0.f) || !(cap >= 0.f)) return LTEA_EINVAL;
  // The multiplier lives in fp32, so the floor is the fp32 image of 1e-9: a head that sits at the floor and whose
  // count is inside the dead band [0.95 cap, cap] stays at the floor instead of being flushed to zero by the
  // rounding of the floor itself.  Direction first (grow above the cap, shrink below 95 % of it, else hold), then
  // the clamps: at most 1, zero below the floor, and back to the floor when a zero head overshoots the cap.
  const float floor_l = 1e-9f;
  for (int i = 0; i < n; ++i) {
    const double c = c_bar[i];
    const bool over = c > (double)cap, under = c < 0.95 * (double)cap;
    const double step = over ? (double)alpha : under ? 1.0 / (double)alpha : 1.0;
    float l = (float)fmin((double)lambda[i] * step, 1.0);
    if (l < floor_l) l = over ? floor_l : 0.0f;
    lambda[i] = l;
  }
  return LTEA_OK;
}

}  // extern "C"
