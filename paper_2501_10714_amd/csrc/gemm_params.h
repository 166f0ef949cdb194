// Description of one grouped (per-expert) GEMM launch of the expert FFN (FSMoE Sec. 2.1 "Experts",
// Sec. 4.4 for the backward products).  Shared by the plain fp32-FMA kernel and the bf16 MFMA kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moe_mi355x.h"

namespace moe {

enum Epilogue {
  EPI_PLAIN = 0,    // C = acc (or C += acc)
  EPI_ACT_FWD = 1,  // C0 = a1 = acc, C2 = hh = act(a1)
  EPI_GLU_FWD = 2,  // two accumulators: C0 = a1, C1 = a3, C2 = hh = silu(a1) * a3
  EPI_ACT_BWD = 3,  // acc = dhh: C0 = da1 = dhh * act'(X0)
  EPI_GLU_BWD = 4,  // acc = dhh: C0 = da1 = dhh * X1 * silu'(X0), C1 = da3 = dhh * silu(X0)
  EPI_ACCUM = 5     // C0 += acc, the old C0 read ahead like the saved activations (bf16 MFMA kernel only)
};

// Two shapes of raggedness:
//   ragged M (RAGGED_K = false): group e owns rows offsets[e]..offsets[e+1] of A and C; B is the
//     expert's weight (group stride gB); K = Kfix.  With n_pairs = 2 and a single accumulator the
//     two products A[0].B[0] + A[1].B[1] are summed (dxe = da1.W1^T + da3.W3^T).
//   ragged K (RAGGED_K = true): group e contracts over its rows; A(i,k) and B(k,n) are both indexed
//     by the expert row k; C is the expert's weight gradient (group stride gC), M = Mfix.  With
//     n_pairs = 2 there are 2E groups: group g uses A[0], B[g / E], C[g / E] for expert g % E.
struct GemmP {
  const void* A[2];
  const void* B[2];
  void* C[3];
  const void* X[2];        // saved activations read by the backward epilogues, same layout as C
  const int32_t* offsets;  // device: first row of every group ([E]; offsets[E] is only read through row_end)
  const int32_t* row_end;  // device: one past the last row of every group (offsets + 1 for whole experts; a
                           // chunk of the rows of every expert when the layer is run in chunks, FSMoE Sec. 4.2)
  long sAi, sAk;           // element strides of A(i,k)
  long sBk, sBn;           // element strides of B(k,n)
  long gB, gC;             // per-expert strides (elements) of weights / weight gradients
  long ldc;
  int n_experts, n_pairs;
  int Mfix, N, Kfix;
  int act, accumulate;
  int max_rows;            // upper bound on rows per expert known on the host
  long total_rows_bound;   // upper bound on A = offsets[E] known on the host (N*k)
};

// gemm_mfma.hip / gemm_plain.hip
bool gemm_mfma_supported(const GemmP& p, int dtype, int epi, bool ragged_k);
moe_status_t launch_gemm_mfma(const GemmP& p, int epi, bool ragged_k, hipStream_t s);
moe_status_t launch_gemm_plain(const GemmP& p, int dtype, int epi, bool ragged_k, hipStream_t s);

}  // namespace moe
