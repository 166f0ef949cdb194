// Expert FFNs as grouped GEMMs (FSMoE Sec. 2.1 "Experts": Q_e = e_e(rows of expert e); Sec. 3.1: GPT
// two-layer FFN and Mixtral three-matrix FFN; Sec. 4.4: backward = gradients of input and weights).
//
// Forward : a1 = xe.W1 (, a3 = xe.W3), hh = act(a1) | silu(a1)*a3   [one launch, activation fused]
//           q  = hh.W2
// Backward: dhh = dq.W2^T -> da1 (, da3) through the stored pre-activations [fused epilogue]
//           dW2 = hh^T.dq
//           dxe = da1.W1^T (+ da3.W3^T)
//           dW1 = xe^T.da1 (, dW3 = xe^T.da3)
// Every product is one launch over all experts; rows are ragged per expert (offsets[] on device).
#include <stdlib.h>

#include "common.h"
#include "gemm_params.h"

namespace moe {

namespace {

// MOE_FORCE_PLAIN_GEMM=1 routes every product through the plain FMA kernel (for A/B checks of the MFMA path)
bool force_plain() {
  const char* e = getenv("MOE_FORCE_PLAIN_GEMM");
  return e != nullptr && e[0] == '1';
}

moe_status_t gemm(const GemmP& p, int dtype, int epi, bool ragged_k, hipStream_t s) {
  if (!force_plain() && gemm_mfma_supported(p, dtype, epi, ragged_k)) return launch_gemm_mfma(p, epi, ragged_k, s);
  return launch_gemm_plain(p, dtype, epi, ragged_k, s);
}

int max_rows_per_expert(const moe_config_t& c) {
  long nk = (long)c.n_tokens * c.top_k;
  // an expert is chosen at most once per token, and never holds more than the capacity
  long m = c.n_tokens;
  if (c.capacity > 0 && c.capacity < m) m = c.capacity;
  return (int)(m < nk ? m : nk);
}

// rows [row_begin[e], row_end[e]) of every expert; row_end == NULL: whole experts (row_begin = offsets)
GemmP base(const moe_config_t& c, const int32_t* row_begin, const int32_t* row_end = nullptr) {
  GemmP p = {};
  p.offsets = row_begin;
  p.row_end = row_end != nullptr ? row_end : row_begin + 1;
  p.n_experts = c.n_experts;
  p.n_pairs = 1;
  p.act = c.act;
  p.accumulate = 0;
  p.max_rows = max_rows_per_expert(c);
  p.total_rows_bound = (long)c.n_tokens * c.top_k;
  return p;
}

}  // namespace

size_t expert_bwd_workspace_bytes(const moe_config_t& c) {
  size_t one = align_up((size_t)c.n_tokens * c.top_k * c.d_hidden * elem_size(c.dtype), 256);
  return c.act == MOE_ACT_SWIGLU ? 2 * one : one;
}

moe_status_t launch_expert_fwd(const moe_config_t& c, const void* xe, const int32_t* offsets, const int32_t* row_end,
                               const void* w1, const void* w3, const void* w2, void* q, void* a1, void* a3, void* hh,
                               hipStream_t s) {
  const long M = c.d_model, H = c.d_hidden;
  const bool glu = c.act == MOE_ACT_SWIGLU;
  {  // a1 (, a3), hh : [A,M] x [M,H]
    GemmP p = base(c, offsets, row_end);
    p.A[0] = xe; p.sAi = M; p.sAk = 1;
    p.B[0] = w1; p.B[1] = glu ? w3 : nullptr; p.sBk = H; p.sBn = 1; p.gB = M * H;
    p.C[0] = a1; p.C[1] = a3; p.C[2] = hh; p.ldc = H;
    p.N = (int)H; p.Kfix = (int)M;
    moe_status_t st = gemm(p, c.dtype, glu ? EPI_GLU_FWD : EPI_ACT_FWD, false, s);
    if (st != MOE_OK) return st;
  }
  {  // q : [A,H] x [H,M]
    GemmP p = base(c, offsets, row_end);
    p.A[0] = hh; p.sAi = H; p.sAk = 1;
    p.B[0] = w2; p.sBk = M; p.sBn = 1; p.gB = H * M;
    p.C[0] = q; p.ldc = M;
    p.N = (int)M; p.Kfix = (int)H;
    return gemm(p, c.dtype, EPI_PLAIN, false, s);
  }
}

// dhh = dq.W2^T with the activation derivative in the epilogue -> da1 (, da3) in the workspace, then
// dxe = da1.W1^T (+ da3.W3^T): the products with ragged M, on rows [offsets[e], row_end[e]) of every expert.
moe_status_t launch_expert_bwd_dgrad(const moe_config_t& c, const void* dq, const int32_t* offsets,
                                     const int32_t* row_end, const void* w1, const void* w3, const void* w2,
                                     const void* a1, const void* a3, void* dxe, void* ws, int which, hipStream_t s) {
  const long M = c.d_model, H = c.d_hidden;
  const bool glu = c.act == MOE_ACT_SWIGLU;
  unsigned char* w = static_cast<unsigned char*>(ws);
  void* da1 = w;
  void* da3 = glu ? w + align_up((size_t)c.n_tokens * c.top_k * H * elem_size(c.dtype), 256) : nullptr;
  if (which & 1) {  // dhh = dq.W2^T : [A,M] x [M,H] with B(k=m, n=h) = W2[h][m]; epilogue -> da1 (, da3)
    GemmP p = base(c, offsets, row_end);
    p.A[0] = dq; p.sAi = M; p.sAk = 1;
    p.B[0] = w2; p.sBk = 1; p.sBn = M; p.gB = H * M;
    p.C[0] = da1; p.C[1] = da3; p.X[0] = a1; p.X[1] = a3; p.ldc = H;
    p.N = (int)H; p.Kfix = (int)M;
    moe_status_t st = gemm(p, c.dtype, glu ? EPI_GLU_BWD : EPI_ACT_BWD, false, s);
    if (st != MOE_OK) return st;
  }
  if (which & 2) {  // dxe = da1.W1^T (+ da3.W3^T) : [A,H] x [H,M] with B(k=h, n=m) = W1[m][h]
    GemmP p = base(c, offsets, row_end);
    p.A[0] = da1; p.A[1] = da3; p.sAi = H; p.sAk = 1;
    p.B[0] = w1; p.B[1] = w3; p.sBk = 1; p.sBn = H; p.gB = M * H;
    p.n_pairs = glu ? 2 : 1;
    p.C[0] = dxe; p.ldc = M;
    p.N = (int)M; p.Kfix = (int)H;
    return gemm(p, c.dtype, EPI_PLAIN, false, s);
  }
  return MOE_OK;
}

// dW2_e = hh_e^T.dq_e and dW1_e = xe_e^T.da1_e (, dW3_e = xe_e^T.da3_e): the products that contract over the
// rows of an expert.  Always over whole experts: splitting the contraction would change the rounding.
moe_status_t launch_expert_bwd_wgrad(const moe_config_t& c, const void* dq, const void* xe, const int32_t* offsets,
                                     const void* hh, void* dw1, void* dw3, void* dw2, void* ws, int which,
                                     hipStream_t s) {
  const long M = c.d_model, H = c.d_hidden;
  const bool glu = c.act == MOE_ACT_SWIGLU;
  unsigned char* w = static_cast<unsigned char*>(ws);
  void* da1 = w;
  void* da3 = glu ? w + align_up((size_t)c.n_tokens * c.top_k * H * elem_size(c.dtype), 256) : nullptr;
  if (which & 1) {  // dW2_e = hh_e^T.dq_e : [H,rows] x [rows,M]
    GemmP p = base(c, offsets);
    p.A[0] = hh; p.sAi = 1; p.sAk = H;
    p.B[0] = dq; p.sBk = M; p.sBn = 1;
    p.C[0] = dw2; p.ldc = M; p.gC = H * M;
    p.Mfix = (int)H; p.N = (int)M;
    p.accumulate = c.accumulate_wgrad;
    moe_status_t st = gemm(p, c.dtype, EPI_PLAIN, true, s);
    if (st != MOE_OK) return st;
  }
  if (which & 2) {  // dW1_e = xe_e^T.da1_e (, dW3_e = xe_e^T.da3_e) : [M,rows] x [rows,H]
    GemmP p = base(c, offsets);
    p.A[0] = xe; p.sAi = 1; p.sAk = M;
    p.B[0] = da1; p.B[1] = da3; p.sBk = H; p.sBn = 1;
    p.n_pairs = glu ? 2 : 1;
    p.C[0] = dw1; p.C[1] = dw3; p.ldc = H; p.gC = M * H;
    p.Mfix = (int)M; p.N = (int)H;
    p.accumulate = c.accumulate_wgrad;
    return gemm(p, c.dtype, EPI_PLAIN, true, s);
  }
  return MOE_OK;
}

moe_status_t launch_expert_bwd(const moe_config_t& c, const void* dq, const void* xe, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2, const void* a1, const void* a3,
                               const void* hh, void* dxe, void* dw1, void* dw3, void* dw2, void* ws, hipStream_t s) {
  // dhh, dW2, dxe, dW1/dW3 (the order in which the operands are freshest in the caches)
  moe_status_t st = launch_expert_bwd_dgrad(c, dq, offsets, nullptr, w1, w3, w2, a1, a3, dxe, ws, 1, s);
  if (st != MOE_OK) return st;
  st = launch_expert_bwd_wgrad(c, dq, xe, offsets, hh, dw1, dw3, dw2, ws, 1, s);
  if (st != MOE_OK) return st;
  st = launch_expert_bwd_dgrad(c, dq, offsets, nullptr, w1, w3, w2, a1, a3, dxe, ws, 2, s);
  if (st != MOE_OK) return st;
  return launch_expert_bwd_wgrad(c, dq, xe, offsets, hh, dw1, dw3, dw2, ws, 2, s);
}

}  // namespace moe
