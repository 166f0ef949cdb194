// C ABI of the MoE hot path: argument validation on the host, workspace planning, launches.
// Every entry point validates first, launches on the caller's stream, never allocates, never
// synchronises.  See include/moe_mi355x.h for the contract of each call.
#include <stdarg.h>
#include <stdio.h>
#include <math.h>

#include "common.h"

namespace moe {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

namespace {

#define REQUIRE(cond, code, ...)  \
  do {                            \
    if (!(cond)) {                \
      set_error(__VA_ARGS__);     \
      return code;                \
    }                             \
  } while (0)

moe_status_t check_cfg(const moe_config_t* c) {
  REQUIRE(c != nullptr, MOE_ERR_INVALID_ARG, "cfg is NULL");
  REQUIRE(c->n_tokens > 0 && c->d_model > 0 && c->n_experts > 0 && c->d_hidden > 0 && c->top_k > 0,
          MOE_ERR_INVALID_ARG, "sizes must be positive (N=%d M=%d E=%d H=%d k=%d)", c->n_tokens, c->d_model,
          c->n_experts, c->d_hidden, c->top_k);
  REQUIRE(c->top_k <= c->n_experts, MOE_ERR_INVALID_ARG, "top_k=%d exceeds n_experts=%d", c->top_k, c->n_experts);
  REQUIRE(c->dtype == MOE_F32 || c->dtype == MOE_BF16, MOE_ERR_INVALID_ARG, "unknown dtype %d", c->dtype);
  REQUIRE(c->act >= MOE_ACT_RELU && c->act <= MOE_ACT_GELU_ERF, MOE_ERR_INVALID_ARG, "unknown activation %d", c->act);
  REQUIRE(c->renormalize >= MOE_GATE_SOFTMAX_ALL && c->renormalize <= MOE_GATE_EXPERT_CHOICE, MOE_ERR_INVALID_ARG,
          "unknown gate-weight function %d", c->renormalize);
  REQUIRE(c->top_k <= 8, MOE_ERR_UNSUPPORTED, "top_k=%d: at most 8 is supported", c->top_k);
  if (c->renormalize == MOE_GATE_EXPERT_CHOICE)
    REQUIRE(c->top_k == c->n_experts && c->capacity > 0, MOE_ERR_INVALID_ARG,
            "expert choice: top_k=%d must equal n_experts=%d (one slot per expert) and capacity=%d must be positive",
            c->top_k, c->n_experts, c->capacity);
  REQUIRE(c->n_experts <= 256, MOE_ERR_UNSUPPORTED, "n_experts=%d: at most 256 is supported", c->n_experts);
  const int vec = c->dtype == MOE_BF16 ? 8 : 4;
  REQUIRE(c->d_model % vec == 0 && c->d_hidden % vec == 0, MOE_ERR_UNSUPPORTED,
          "d_model=%d and d_hidden=%d must be multiples of %d (16-byte rows)", c->d_model, c->d_hidden, vec);
  REQUIRE((long)c->n_tokens * c->top_k < (1l << 30), MOE_ERR_UNSUPPORTED, "n_tokens*top_k too large");
  return MOE_OK;
}

struct SavedPlan {
  size_t off[MOE_SAVED_N_], len[MOE_SAVED_N_], bytes;
};

SavedPlan saved_plan(const moe_config_t& c) {
  SavedPlan p;
  const size_t N = c.n_tokens, E = c.n_experts, k = c.top_k, M = c.d_model, H = c.d_hidden, b = elem_size(c.dtype);
  const size_t A = N * k;
  size_t len[MOE_SAVED_N_];
  len[MOE_SAVED_LOGITS] = N * E * 4;
  len[MOE_SAVED_PROBS] = N * E * 4;
  len[MOE_SAVED_TOPK_IDX] = A * 4;
  len[MOE_SAVED_TOPK_W] = A * 4;
  len[MOE_SAVED_POS] = A * 4;
  len[MOE_SAVED_ROW_OF] = A * 4;
  len[MOE_SAVED_COUNT] = E * 4;
  len[MOE_SAVED_OFFSETS] = (E + 1) * 4;
  len[MOE_SAVED_SRC_OF_ROW] = A * 4;
  len[MOE_SAVED_XE] = A * M * b;
  len[MOE_SAVED_A1] = A * H * b;
  len[MOE_SAVED_A3] = c.act == MOE_ACT_SWIGLU ? A * H * b : 0;
  len[MOE_SAVED_HH] = A * H * b;
  len[MOE_SAVED_Q] = A * M * b;
  size_t o = 0;
  for (int i = 0; i < MOE_SAVED_N_; ++i) {
    p.off[i] = o;
    p.len[i] = len[i];
    o += align_up(len[i], 256);
  }
  p.bytes = o;
  return p;
}

struct BwdPlan {
  size_t off_dq, off_dxe, off_dtw, off_expert, off_route, bytes;
};

BwdPlan bwd_plan(const moe_config_t& c) {
  BwdPlan p;
  const size_t A = (size_t)c.n_tokens * c.top_k, M = c.d_model, b = elem_size(c.dtype);
  size_t o = 0;
  p.off_dq = o; o += align_up(A * M * b, 256);
  p.off_dxe = o; o += align_up(A * M * b, 256);
  p.off_dtw = o; o += align_up(A * 4, 256);
  p.off_expert = o; o += align_up(expert_bwd_workspace_bytes(c), 256);
  p.off_route = o; o += align_up(route_bwd_workspace_bytes(c), 256);
  p.bytes = o;
  return p;
}

// The workspace ends in the row ranges of the chunked layer: begin[r][E], end[r][E], r <= MOE_MAX_CHUNKS.
size_t chunk_bounds_offset(const moe_config_t& c) {
  size_t w = route_workspace_bytes(c);
  size_t b = bwd_plan(c).bytes;
  return align_up(w > b ? w : b, 256);
}
size_t workspace_bytes(const moe_config_t& c) {
  return chunk_bounds_offset(c) + align_up((size_t)2 * MOE_MAX_CHUNKS * c.n_experts * sizeof(int32_t), 256);
}


inline hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

// a tensor argument: present, and aligned for the 16-byte vector accesses of the kernels
#define NOT_NULL(p)                                                                                        \
  do {                                                                                                     \
    REQUIRE((p) != nullptr, MOE_ERR_INVALID_ARG, "%s: argument '%s' is NULL", __func__, #p);               \
    REQUIRE((reinterpret_cast<uintptr_t>(p) & 15) == 0, MOE_ERR_INVALID_ARG,                               \
            "%s: argument '%s' is not 16-byte aligned", __func__, #p);                                     \
  } while (0)
#define CHECK_CFG(c)                   \
  do {                                 \
    moe_status_t st__ = check_cfg(c);  \
    if (st__ != MOE_OK) return st__;   \
  } while (0)
#define CHECK_WS(c, ws, ws_bytes)                                                                        \
  do {                                                                                                   \
    NOT_NULL(ws);                                                                                        \
    REQUIRE((ws_bytes) >= workspace_bytes(*(c)), MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes, need %zu", \
            __func__, (size_t)(ws_bytes), workspace_bytes(*(c)));                                        \
  } while (0)

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

int32_t moe_capacity(int32_t n_tokens, int32_t n_experts, int32_t top_k, double f) {
  if (n_tokens <= 0 || n_experts <= 0 || top_k <= 0 || !(f > 0.0)) return -1;
  const double t = (((double)top_k * f) * (double)n_tokens) / (double)n_experts;
  return (int32_t)ceil(t);
}

moe_status_t moe_workspace_bytes(const moe_config_t* cfg, size_t* ws_bytes, size_t* saved_bytes) {
  CHECK_CFG(cfg);
  if (ws_bytes != nullptr) *ws_bytes = workspace_bytes(*cfg);
  if (saved_bytes != nullptr) *saved_bytes = saved_plan(*cfg).bytes;
  return MOE_OK;
}

moe_status_t moe_saved_offset(const moe_config_t* cfg, int32_t which, size_t* byte_offset, size_t* n_bytes) {
  CHECK_CFG(cfg);
  REQUIRE(which >= 0 && which < MOE_SAVED_N_, MOE_ERR_INVALID_ARG, "moe_saved_offset: unknown tensor %d", which);
  SavedPlan p = saved_plan(*cfg);
  if (byte_offset != nullptr) *byte_offset = p.off[which];
  if (n_bytes != nullptr) *n_bytes = p.len[which];
  return MOE_OK;
}

moe_status_t moe_route(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate, float* logits,
                       float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                       int32_t* offsets, int32_t* src_of_row, void* workspace, size_t workspace_bytes_, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w_gate); NOT_NULL(logits); NOT_NULL(probs); NOT_NULL(topk_idx); NOT_NULL(topk_w);
  NOT_NULL(pos); NOT_NULL(row_of); NOT_NULL(count); NOT_NULL(offsets); NOT_NULL(src_of_row);
  CHECK_WS(cfg, workspace, workspace_bytes_);
  return launch_route(*cfg, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets, src_of_row,
                      workspace, as_stream(stream));
}

moe_status_t moe_route_static(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                              float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                              int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w_gate); NOT_NULL(logits); NOT_NULL(probs); NOT_NULL(topk_idx); NOT_NULL(topk_w);
  NOT_NULL(pos); NOT_NULL(row_of); NOT_NULL(count); NOT_NULL(offsets); NOT_NULL(src_of_row);
  return launch_route_static(*cfg, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets,
                             src_of_row, as_stream(stream));
}

moe_status_t moe_route_noisy(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                             const void* w_noise, const float* noise, float* logits, float* noise_logits, float* probs,
                             int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                             int32_t* offsets, int32_t* src_of_row, void* workspace, size_t workspace_bytes_,
                             void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w_gate); NOT_NULL(w_noise); NOT_NULL(noise); NOT_NULL(logits); NOT_NULL(noise_logits);
  NOT_NULL(probs); NOT_NULL(topk_idx); NOT_NULL(topk_w); NOT_NULL(pos); NOT_NULL(row_of); NOT_NULL(count);
  NOT_NULL(offsets); NOT_NULL(src_of_row);
  REQUIRE(cfg->renormalize != MOE_GATE_EXPERT_CHOICE, MOE_ERR_UNSUPPORTED, "moe_route_noisy: not with expert choice");
  CHECK_WS(cfg, workspace, workspace_bytes_);
  return launch_route_noisy(*cfg, x, w_gate, b_gate, w_noise, noise, logits, noise_logits, probs, topk_idx, topk_w, pos,
                            row_of, count, offsets, src_of_row, workspace, as_stream(stream));
}

moe_status_t moe_route_noisy_bwd(const moe_config_t* cfg, const void* x, const void* w_gate, const void* w_noise,
                                 const float* noise, const float* noise_logits, const float* probs,
                                 const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                                 float* db_gate, void* dw_noise, void* dx, void* workspace, size_t workspace_bytes_,
                                 void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w_gate); NOT_NULL(w_noise); NOT_NULL(noise); NOT_NULL(noise_logits); NOT_NULL(probs);
  NOT_NULL(topk_idx); NOT_NULL(pos); NOT_NULL(dtopk_w); NOT_NULL(dw_gate); NOT_NULL(dw_noise); NOT_NULL(dx);
  REQUIRE(cfg->renormalize != MOE_GATE_EXPERT_CHOICE, MOE_ERR_UNSUPPORTED, "moe_route_noisy_bwd: not with expert choice");
  CHECK_WS(cfg, workspace, workspace_bytes_);
  return launch_route_noisy_bwd(*cfg, x, w_gate, w_noise, noise, noise_logits, probs, topk_idx, pos, dtopk_w, dw_gate,
                                db_gate, dw_noise, dx, workspace, as_stream(stream));
}

static moe_status_t check_xmoe(const char* fn, const moe_config_t* cfg, int32_t d_proj, const void* workspace,
                               size_t workspace_bytes_) {
  REQUIRE(d_proj >= 4 && d_proj <= 256 && d_proj % 4 == 0, MOE_ERR_UNSUPPORTED,
          "%s: d_proj=%d must be a multiple of 4 in 4..256", fn, d_proj);
  REQUIRE(cfg->renormalize != MOE_GATE_EXPERT_CHOICE, MOE_ERR_UNSUPPORTED, "%s: not with expert choice", fn);
  REQUIRE(workspace != nullptr, MOE_ERR_INVALID_ARG, "%s: argument 'workspace' is NULL", fn);
  const size_t need = route_xmoe_workspace_bytes(*cfg, d_proj);
  REQUIRE(workspace_bytes_ >= need, MOE_ERR_WORKSPACE, "%s: workspace of %zu bytes, need %zu", fn, workspace_bytes_, need);
  return MOE_OK;
}

moe_status_t moe_route_xmoe_workspace_bytes(const moe_config_t* cfg, int32_t d_proj, size_t* ws_bytes) {
  CHECK_CFG(cfg);
  REQUIRE(ws_bytes != nullptr, MOE_ERR_INVALID_ARG, "moe_route_xmoe_workspace_bytes: argument 'ws_bytes' is NULL");
  REQUIRE(d_proj >= 4 && d_proj <= 256 && d_proj % 4 == 0, MOE_ERR_UNSUPPORTED,
          "moe_route_xmoe_workspace_bytes: d_proj=%d must be a multiple of 4 in 4..256", d_proj);
  *ws_bytes = route_xmoe_workspace_bytes(*cfg, d_proj);
  return MOE_OK;
}

moe_status_t moe_route_xmoe(const moe_config_t* cfg, const void* x, const void* w_proj, const void* w_gate,
                            int32_t d_proj, float* proj, float* logits, float* probs, int32_t* topk_idx, float* topk_w,
                            int32_t* pos, int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row,
                            void* workspace, size_t workspace_bytes_, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w_proj); NOT_NULL(w_gate); NOT_NULL(proj); NOT_NULL(logits); NOT_NULL(probs); NOT_NULL(topk_idx);
  NOT_NULL(topk_w); NOT_NULL(pos); NOT_NULL(row_of); NOT_NULL(count); NOT_NULL(offsets); NOT_NULL(src_of_row);
  moe_status_t st = check_xmoe("moe_route_xmoe", cfg, d_proj, workspace, workspace_bytes_);
  if (st != MOE_OK) return st;
  return launch_route_xmoe(*cfg, x, w_proj, w_gate, d_proj, proj, logits, probs, topk_idx, topk_w, pos, row_of, count,
                           offsets, src_of_row, workspace, as_stream(stream));
}

moe_status_t moe_route_xmoe_bwd(const moe_config_t* cfg, const void* x, const void* w_proj, const void* w_gate,
                                int32_t d_proj, const float* proj, const float* probs, const int32_t* topk_idx,
                                const int32_t* pos, const float* dtopk_w, void* dw_proj, void* dw_gate, void* dx,
                                void* workspace, size_t workspace_bytes_, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w_proj); NOT_NULL(w_gate); NOT_NULL(proj); NOT_NULL(probs); NOT_NULL(topk_idx); NOT_NULL(pos);
  NOT_NULL(dtopk_w); NOT_NULL(dw_proj); NOT_NULL(dw_gate); NOT_NULL(dx);
  moe_status_t st = check_xmoe("moe_route_xmoe_bwd", cfg, d_proj, workspace, workspace_bytes_);
  if (st != MOE_OK) return st;
  return launch_route_xmoe_bwd(*cfg, x, w_proj, w_gate, d_proj, proj, probs, topk_idx, pos, dtopk_w, dw_proj, dw_gate, dx,
                               workspace, as_stream(stream));
}

moe_status_t moe_dispatch(const moe_config_t* cfg, const void* x, const int32_t* row_of, void* xe, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(row_of); NOT_NULL(xe);
  return launch_dispatch(*cfg, x, row_of, xe, as_stream(stream));
}

moe_status_t moe_dispatch_bwd(const moe_config_t* cfg, const void* dxe, const int32_t* row_of, const void* dy, void* dx,
                              void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(dxe); NOT_NULL(row_of); NOT_NULL(dx);
  REQUIRE(!cfg->add_residual || dy != nullptr, MOE_ERR_INVALID_ARG, "moe_dispatch_bwd: add_residual needs dy");
  if (cfg->add_residual) NOT_NULL(dy);
  return launch_dispatch_bwd(*cfg, dxe, row_of, dy, dx, as_stream(stream));
}

moe_status_t moe_expert_ffn_fwd(const moe_config_t* cfg, const void* xe, const int32_t* offsets, const void* w1,
                                const void* w3, const void* w2, void* q, void* a1, void* a3, void* hh, void* workspace,
                                size_t workspace_bytes_, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(xe); NOT_NULL(offsets); NOT_NULL(w1); NOT_NULL(w2); NOT_NULL(q); NOT_NULL(a1); NOT_NULL(hh);
  if (cfg->act == MOE_ACT_SWIGLU) { NOT_NULL(w3); NOT_NULL(a3); }
  (void)workspace; (void)workspace_bytes_;
  return launch_expert_fwd(*cfg, xe, offsets, nullptr, w1, w3, w2, q, a1, a3, hh, as_stream(stream));
}

moe_status_t moe_expert_ffn_bwd(const moe_config_t* cfg, const void* dq, const void* xe, const int32_t* offsets,
                                const void* w1, const void* w3, const void* w2, const void* a1, const void* a3,
                                const void* hh, void* dxe, void* dw1, void* dw3, void* dw2, void* workspace,
                                size_t workspace_bytes_, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(dq); NOT_NULL(xe); NOT_NULL(offsets); NOT_NULL(w1); NOT_NULL(w2); NOT_NULL(a1); NOT_NULL(hh);
  NOT_NULL(dxe); NOT_NULL(dw1); NOT_NULL(dw2);
  if (cfg->act == MOE_ACT_SWIGLU) { NOT_NULL(w3); NOT_NULL(a3); NOT_NULL(dw3); }
  CHECK_WS(cfg, workspace, workspace_bytes_);
  return launch_expert_bwd(*cfg, dq, xe, offsets, w1, w3, w2, a1, a3, hh, dxe, dw1, dw3, dw2, workspace,
                           as_stream(stream));
}

moe_status_t moe_combine(const moe_config_t* cfg, const void* q, const float* topk_w, const int32_t* row_of,
                         const void* x, void* y, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(q); NOT_NULL(topk_w); NOT_NULL(row_of); NOT_NULL(y);
  REQUIRE(!cfg->add_residual || x != nullptr, MOE_ERR_INVALID_ARG, "moe_combine: add_residual needs x");
  if (cfg->add_residual) NOT_NULL(x);
  return launch_combine(*cfg, q, topk_w, row_of, x, y, as_stream(stream));
}

moe_status_t moe_combine_bwd(const moe_config_t* cfg, const void* dy, const void* q, const float* topk_w,
                             const int32_t* row_of, void* dq, float* dtopk_w, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(dy); NOT_NULL(q); NOT_NULL(topk_w); NOT_NULL(row_of); NOT_NULL(dq); NOT_NULL(dtopk_w);
  return launch_combine_bwd(*cfg, dy, q, topk_w, row_of, dq, dtopk_w, as_stream(stream));
}

moe_status_t moe_route_bwd(const moe_config_t* cfg, const void* x, const void* w_gate, const float* probs,
                           const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                           float* db_gate, void* dx, void* workspace, size_t workspace_bytes_, void* stream) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w_gate); NOT_NULL(probs); NOT_NULL(topk_idx); NOT_NULL(pos); NOT_NULL(dtopk_w);
  NOT_NULL(dw_gate); NOT_NULL(dx);
  CHECK_WS(cfg, workspace, workspace_bytes_);
  return launch_route_bwd(*cfg, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, workspace,
                          as_stream(stream));
}

static moe_status_t layer_fwd_impl(const char* fn, const moe_config_t* cfg, const void* x, const void* w_gate,
                                   const float* b_gate, const void* w1, const void* w3, const void* w2, void* y,
                                   void* saved, size_t saved_bytes, void* workspace, size_t workspace_bytes_, int r,
                                   void* stream, void* aux_stream, bool routed = false) {
  CHECK_CFG(cfg);
  NOT_NULL(x); NOT_NULL(w1); NOT_NULL(w2); NOT_NULL(y); NOT_NULL(saved);
  if (!routed) NOT_NULL(w_gate);
  if (cfg->act == MOE_ACT_SWIGLU) NOT_NULL(w3);
  REQUIRE(r >= 1 && r <= MOE_MAX_CHUNKS, MOE_ERR_INVALID_ARG, "%s: %d chunks, must be 1..%d", fn, r, MOE_MAX_CHUNKS);
  CHECK_WS(cfg, workspace, workspace_bytes_);
  SavedPlan sp = saved_plan(*cfg);
  REQUIRE(saved_bytes >= sp.bytes, MOE_ERR_WORKSPACE, "%s: saved blob of %zu bytes, need %zu", fn, saved_bytes, sp.bytes);
  unsigned char* sv = static_cast<unsigned char*>(saved);
  auto at = [&](int w) { return static_cast<void*>(sv + sp.off[w]); };
  hipStream_t s = as_stream(stream);
  void* a3 = cfg->act == MOE_ACT_SWIGLU ? at(MOE_SAVED_A3) : nullptr;
  const int32_t* offsets = (const int32_t*)at(MOE_SAVED_OFFSETS);
  moe_status_t st = MOE_OK;
  if (!routed) {  // routed: a moe_route* call has already written the routing tensors of `saved`
    st = launch_route(*cfg, x, w_gate, b_gate, (float*)at(MOE_SAVED_LOGITS), (float*)at(MOE_SAVED_PROBS),
                      (int32_t*)at(MOE_SAVED_TOPK_IDX), (float*)at(MOE_SAVED_TOPK_W), (int32_t*)at(MOE_SAVED_POS),
                      (int32_t*)at(MOE_SAVED_ROW_OF), (int32_t*)at(MOE_SAVED_COUNT), (int32_t*)at(MOE_SAVED_OFFSETS),
                      (int32_t*)at(MOE_SAVED_SRC_OF_ROW), workspace, s);
    if (st != MOE_OK) return st;
  }
  if (r == 1) {
    st = launch_dispatch(*cfg, x, (const int32_t*)at(MOE_SAVED_ROW_OF), at(MOE_SAVED_XE), s);
    if (st != MOE_OK) return st;
    st = launch_expert_fwd(*cfg, at(MOE_SAVED_XE), offsets, nullptr, w1, w3, w2, at(MOE_SAVED_Q), at(MOE_SAVED_A1), a3,
                           at(MOE_SAVED_HH), s);
    if (st != MOE_OK) return st;
  } else {
    // FSMoE Sec. 4.2 on one GPU: the rows of every expert are cut into r chunks; chunk c is dispatched (on the
    // auxiliary stream when there is one) while chunk c - 1 is in the expert FFN.  Rows are independent in
    // dispatch and in the FFN, so every byte of xe, a1, a3, hh, q is what r = 1 writes.
    int32_t* begin = reinterpret_cast<int32_t*>(static_cast<unsigned char*>(workspace) + chunk_bounds_offset(*cfg));
    int32_t* end = begin + (size_t)MOE_MAX_CHUNKS * cfg->n_experts;
    st = launch_chunk_bounds(*cfg, offsets, r, begin, end, s);
    if (st != MOE_OK) return st;
    hipStream_t aux = as_stream(aux_stream);
    // events of this call only (two calls on different stream pairs may run at once); an event may be
    // destroyed as soon as the work that waits on it has been enqueued
    struct Events {
      hipEvent_t e[MOE_MAX_CHUNKS + 1];
      int n = 0;
      ~Events() { for (int i = 0; i < n; ++i) (void)hipEventDestroy(e[i]); }
    } evs;
    hipEvent_t* ev = nullptr;
    if (aux_stream != nullptr && aux != s) {
      for (; evs.n < r + 1; ++evs.n)
        REQUIRE(hipEventCreateWithFlags(&evs.e[evs.n], hipEventDisableTiming) == hipSuccess, MOE_ERR_DEVICE,
                "%s: could not create an event", fn);
      ev = evs.e;
      REQUIRE(hipEventRecord(ev[r], s) == hipSuccess && hipStreamWaitEvent(aux, ev[r], 0) == hipSuccess, MOE_ERR_DEVICE,
              "%s: stream ordering failed", fn);
    }
    for (int c = 0; c < r; ++c) {
      const int32_t* bc = begin + (size_t)c * cfg->n_experts;
      const int32_t* ec = end + (size_t)c * cfg->n_experts;
      st = launch_dispatch_rows(*cfg, x, (const int32_t*)at(MOE_SAVED_SRC_OF_ROW), bc, ec, r, at(MOE_SAVED_XE),
                                ev != nullptr ? aux : s);
      if (st != MOE_OK) return st;
      if (ev != nullptr)
        REQUIRE(hipEventRecord(ev[c], aux) == hipSuccess && hipStreamWaitEvent(s, ev[c], 0) == hipSuccess, MOE_ERR_DEVICE,
                "%s: stream ordering failed", fn);
      st = launch_expert_fwd(*cfg, at(MOE_SAVED_XE), bc, ec, w1, w3, w2, at(MOE_SAVED_Q), at(MOE_SAVED_A1), a3,
                             at(MOE_SAVED_HH), s);
      if (st != MOE_OK) return st;
    }
  }
  return launch_combine(*cfg, at(MOE_SAVED_Q), (const float*)at(MOE_SAVED_TOPK_W), (const int32_t*)at(MOE_SAVED_ROW_OF),
                        x, y, s);
}

moe_status_t moe_layer_fwd(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                           const void* w1, const void* w3, const void* w2, void* y, void* saved, size_t saved_bytes,
                           void* workspace, size_t workspace_bytes_, void* stream) {
  return layer_fwd_impl("moe_layer_fwd", cfg, x, w_gate, b_gate, w1, w3, w2, y, saved, saved_bytes, workspace,
                        workspace_bytes_, 1, stream, nullptr);
}

moe_status_t moe_layer_fwd_chunked(const moe_config_t* cfg, const void* x, const void* w_gate, const float* b_gate,
                                   const void* w1, const void* w3, const void* w2, void* y, void* saved,
                                   size_t saved_bytes, void* workspace, size_t workspace_bytes_, int32_t n_chunks,
                                   void* stream, void* aux_stream) {
  return layer_fwd_impl("moe_layer_fwd_chunked", cfg, x, w_gate, b_gate, w1, w3, w2, y, saved, saved_bytes, workspace,
                        workspace_bytes_, n_chunks, stream, aux_stream);
}

static moe_status_t layer_bwd_impl(const char* fn, const moe_config_t* cfg, const void* dy, const void* x,
                                   const void* w_gate, const void* w1, const void* w3, const void* w2, const void* saved,
                                   size_t saved_bytes, void* dx, void* dw_gate, float* db_gate, void* dw1, void* dw3,
                                   void* dw2, void* workspace, size_t workspace_bytes_, int r, void* stream,
                                   float* dtopk_w_out = nullptr) {
  // dtopk_w_out: stop before the gate (its backward is the caller's next call) and leave the gradient of the
  // gate weights there
  const bool routed = dtopk_w_out != nullptr;
  CHECK_CFG(cfg);
  NOT_NULL(dy); NOT_NULL(w1); NOT_NULL(w2); NOT_NULL(saved); NOT_NULL(dx); NOT_NULL(dw1); NOT_NULL(dw2);
  if (!routed) { NOT_NULL(x); NOT_NULL(w_gate); NOT_NULL(dw_gate); }
  if (cfg->act == MOE_ACT_SWIGLU) { NOT_NULL(w3); NOT_NULL(dw3); }
  REQUIRE(r >= 1 && r <= MOE_MAX_CHUNKS, MOE_ERR_INVALID_ARG, "%s: %d chunks, must be 1..%d", fn, r, MOE_MAX_CHUNKS);
  CHECK_WS(cfg, workspace, workspace_bytes_);
  SavedPlan sp = saved_plan(*cfg);
  REQUIRE(saved_bytes >= sp.bytes, MOE_ERR_WORKSPACE, "%s: saved blob of %zu bytes, need %zu", fn, saved_bytes, sp.bytes);
  const unsigned char* sv = static_cast<const unsigned char*>(saved);
  auto at = [&](int w) { return static_cast<const void*>(sv + sp.off[w]); };
  BwdPlan bp = bwd_plan(*cfg);
  unsigned char* w = static_cast<unsigned char*>(workspace);
  void* dq = w + bp.off_dq;
  void* dxe = w + bp.off_dxe;
  float* dtw = routed ? dtopk_w_out : reinterpret_cast<float*>(w + bp.off_dtw);
  hipStream_t s = as_stream(stream);
  const int32_t* row_of = (const int32_t*)at(MOE_SAVED_ROW_OF);
  const int32_t* offsets = (const int32_t*)at(MOE_SAVED_OFFSETS);
  const void* a3 = cfg->act == MOE_ACT_SWIGLU ? at(MOE_SAVED_A3) : nullptr;
  moe_status_t st = launch_combine_bwd(*cfg, dy, at(MOE_SAVED_Q), (const float*)at(MOE_SAVED_TOPK_W), row_of, dq, dtw, s);
  if (st != MOE_OK) return st;
  if (r == 1) {
    st = launch_expert_bwd(*cfg, dq, at(MOE_SAVED_XE), offsets, w1, w3, w2, at(MOE_SAVED_A1), a3, at(MOE_SAVED_HH), dxe,
                           dw1, dw3, dw2, w + bp.off_expert, s);
    if (st != MOE_OK) return st;
  } else {
    // the row-wise products (dhh with the activation derivative, dxe) chunk by chunk; the weight gradients
    // contract over the rows of an expert and stay whole, so that their rounding is that of r = 1
    int32_t* begin = reinterpret_cast<int32_t*>(w + chunk_bounds_offset(*cfg));
    int32_t* end = begin + (size_t)MOE_MAX_CHUNKS * cfg->n_experts;
    st = launch_chunk_bounds(*cfg, offsets, r, begin, end, s);
    if (st != MOE_OK) return st;
    for (int c = 0; c < r; ++c) {
      st = launch_expert_bwd_dgrad(*cfg, dq, begin + (size_t)c * cfg->n_experts, end + (size_t)c * cfg->n_experts, w1, w3,
                                   w2, at(MOE_SAVED_A1), a3, dxe, w + bp.off_expert, 3, s);
      if (st != MOE_OK) return st;
    }
    st = launch_expert_bwd_wgrad(*cfg, dq, at(MOE_SAVED_XE), offsets, at(MOE_SAVED_HH), dw1, dw3, dw2, w + bp.off_expert,
                                 3, s);
    if (st != MOE_OK) return st;
  }
  if (routed) return launch_dispatch_bwd(*cfg, dxe, row_of, dy, dx, s);
  // backward of the ordering function and of the gate; dx is written once when the gate's share can be folded in
  return launch_dispatch_route_bwd(*cfg, dxe, row_of, dy, x, w_gate, (const float*)at(MOE_SAVED_PROBS),
                                   (const int32_t*)at(MOE_SAVED_TOPK_IDX), (const int32_t*)at(MOE_SAVED_POS), dtw, dw_gate,
                                   db_gate, dx, w + bp.off_route, s);
}

moe_status_t moe_layer_bwd(const moe_config_t* cfg, const void* dy, const void* x, const void* w_gate, const void* w1,
                           const void* w3, const void* w2, const void* saved, size_t saved_bytes, void* dx,
                           void* dw_gate, float* db_gate, void* dw1, void* dw3, void* dw2, void* workspace,
                           size_t workspace_bytes_, void* stream) {
  return layer_bwd_impl("moe_layer_bwd", cfg, dy, x, w_gate, w1, w3, w2, saved, saved_bytes, dx, dw_gate, db_gate, dw1,
                        dw3, dw2, workspace, workspace_bytes_, 1, stream);
}

moe_status_t moe_layer_bwd_chunked(const moe_config_t* cfg, const void* dy, const void* x, const void* w_gate,
                                   const void* w1, const void* w3, const void* w2, const void* saved, size_t saved_bytes,
                                   void* dx, void* dw_gate, float* db_gate, void* dw1, void* dw3, void* dw2,
                                   void* workspace, size_t workspace_bytes_, int32_t n_chunks, void* stream) {
  return layer_bwd_impl("moe_layer_bwd_chunked", cfg, dy, x, w_gate, w1, w3, w2, saved, saved_bytes, dx, dw_gate, db_gate,
                        dw1, dw3, dw2, workspace, workspace_bytes_, n_chunks, stream);
}

moe_status_t moe_layer_fwd_routed(const moe_config_t* cfg, const void* x, const void* w1, const void* w3, const void* w2,
                                  void* y, void* saved, size_t saved_bytes, void* workspace, size_t workspace_bytes_,
                                  int32_t n_chunks, void* stream, void* aux_stream) {
  return layer_fwd_impl("moe_layer_fwd_routed", cfg, x, nullptr, nullptr, w1, w3, w2, y, saved, saved_bytes, workspace,
                        workspace_bytes_, n_chunks, stream, aux_stream, true);
}

moe_status_t moe_layer_bwd_routed(const moe_config_t* cfg, const void* dy, const void* w1, const void* w3, const void* w2,
                                  const void* saved, size_t saved_bytes, void* dx, void* dw1, void* dw3, void* dw2,
                                  float* dtopk_w, void* workspace, size_t workspace_bytes_, int32_t n_chunks,
                                  void* stream) {
  REQUIRE(dtopk_w != nullptr, MOE_ERR_INVALID_ARG, "moe_layer_bwd_routed: argument 'dtopk_w' is NULL");
  return layer_bwd_impl("moe_layer_bwd_routed", cfg, dy, nullptr, nullptr, w1, w3, w2, saved, saved_bytes, dx, nullptr,
                        nullptr, dw1, dw3, dw2, workspace, workspace_bytes_, n_chunks, stream, dtopk_w);
}

const char* moe_last_error(void) { return moe::g_err; }

}  // extern "C"
