// Plain grouped GEMM: 64x64 output tile, fp32 FMA, any strides, any sizes.  It is the fp32 path of
// the expert FFN (FSMoE Sec. 2.1 "Experts", Sec. 4.4) and the path for bf16 shapes the MFMA kernel
// does not take.  Accumulation is fp32; bf16 operands are widened on load.
#include "common.h"
#include "gemm_params.h"

namespace moe {
namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T, int EPI, bool RAGGED_K>
__global__ __launch_bounds__(256) void gg_plain_kernel(GemmP p) {
  constexpr bool kDual = EPI == EPI_GLU_FWD;
  __shared__ float As[TK][TM + 1];
  __shared__ float Bs[kDual ? 2 : 1][TK][TN + 1];

  const int g = blockIdx.z;
  const int e = g % p.n_experts;
  const int set = g / p.n_experts;  // only > 0 for ragged-K launches with two outputs
  const int r0 = p.offsets[e], r1 = p.row_end[e];
  const int rows = r1 - r0;
  const int Mg = RAGGED_K ? p.Mfix : rows;
  const int Kg = RAGGED_K ? rows : p.Kfix;
  const int m0 = blockIdx.x * TM, n0 = blockIdx.y * TN;
  if (m0 >= Mg) return;

  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4], acc2[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = acc2[i][j] = 0.0f;

  const int sum_pairs = (!RAGGED_K && !kDual) ? p.n_pairs : 1;
  for (int pr = 0; pr < sum_pairs; ++pr) {
    const T* A = static_cast<const T*>(p.A[RAGGED_K ? 0 : pr]);
    const T* B = static_cast<const T*>(p.B[RAGGED_K ? set : pr]);
    const T* B2 = kDual ? static_cast<const T*>(p.B[1]) : nullptr;
    for (int k0 = 0; k0 < Kg; k0 += TK) {
      for (int i = threadIdx.x; i < TM * TK; i += 256) {
        // k fastest for ragged M (A rows are K-contiguous), i fastest for ragged K
        int kk = RAGGED_K ? i / TM : i % TK, ii = RAGGED_K ? i % TM : i / TK;
        int gi = m0 + ii, gk = k0 + kk;
        float v = 0.0f;
        if (gi < Mg && gk < Kg) {
          long off = RAGGED_K ? (long)(r0 + gk) * p.sAk + (long)gi * p.sAi : (long)(r0 + gi) * p.sAi + (long)gk * p.sAk;
          v = Elem<T>::ld(A + off);
        }
        As[kk][ii] = v;
      }
      for (int i = threadIdx.x; i < TN * TK; i += 256) {
        // n fastest when B rows are N-contiguous, k fastest otherwise
        int kk = p.sBn == 1 ? i / TN : i % TK, nn = p.sBn == 1 ? i % TN : i / TK;
        int gn = n0 + nn, gk = k0 + kk;
        float v = 0.0f, v2 = 0.0f;
        if (gn < p.N && gk < Kg) {
          long off = RAGGED_K ? (long)(r0 + gk) * p.sBk + (long)gn * p.sBn
                              : (long)e * p.gB + (long)gk * p.sBk + (long)gn * p.sBn;
          v = Elem<T>::ld(B + off);
          if (kDual) v2 = Elem<T>::ld(B2 + off);
        }
        Bs[0][kk][nn] = v;
        if (kDual) Bs[kDual ? 1 : 0][kk][nn] = v2;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < TK; ++kk) {
        float a[4], b[4], b2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          b[j] = Bs[0][kk][tx * 4 + j];
          if (kDual) b2[j] = Bs[kDual ? 1 : 0][kk][tx * 4 + j];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            if (kDual) acc2[i][j] = fmaf(a[i], b2[j], acc2[i][j]);
          }
      }
      __syncthreads();
    }
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gi = m0 + ty * 4 + i;
    if (gi >= Mg) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= p.N) continue;
      const long off = RAGGED_K ? (long)e * p.gC + (long)gi * p.ldc + gn : (long)(r0 + gi) * p.ldc + gn;
      const float v = acc[i][j];
      if (EPI == EPI_PLAIN) {
        T* c = static_cast<T*>(p.C[RAGGED_K ? set : 0]) + off;
        Elem<T>::st(c, p.accumulate ? Elem<T>::ld(c) + v : v);
      } else if (EPI == EPI_ACT_FWD) {
        Elem<T>::st(static_cast<T*>(p.C[0]) + off, v);
        Elem<T>::st(static_cast<T*>(p.C[2]) + off, act_fwd(v, p.act));
      } else if (EPI == EPI_GLU_FWD) {
        const float v3 = acc2[i][j];
        Elem<T>::st(static_cast<T*>(p.C[0]) + off, v);
        Elem<T>::st(static_cast<T*>(p.C[1]) + off, v3);
        Elem<T>::st(static_cast<T*>(p.C[2]) + off, siluf_(v) * v3);
      } else if (EPI == EPI_ACT_BWD) {
        const float a1 = Elem<T>::ld(static_cast<const T*>(p.X[0]) + off);
        Elem<T>::st(static_cast<T*>(p.C[0]) + off, v * act_grad(a1, p.act));
      } else {
        const float a1 = Elem<T>::ld(static_cast<const T*>(p.X[0]) + off);
        const float a3 = Elem<T>::ld(static_cast<const T*>(p.X[1]) + off);
        Elem<T>::st(static_cast<T*>(p.C[0]) + off, v * a3 * silu_gradf_(a1));
        Elem<T>::st(static_cast<T*>(p.C[1]) + off, v * siluf_(a1));
      }
    }
  }
}

// Experts with no rows: their weight gradients are zero (ragged-K launches skip the K loop and
// still run the epilogue with a zero accumulator, so nothing else is needed there).

template <typename T, int EPI, bool RAGGED_K>
moe_status_t launch_t(const GemmP& p, hipStream_t s) {
  const int mrows = RAGGED_K ? p.Mfix : p.max_rows;
  const int groups = (RAGGED_K && p.n_pairs == 2) ? 2 * p.n_experts : p.n_experts;
  if (mrows <= 0) return MOE_OK;
  dim3 grid(ceil_div(mrows, TM), ceil_div(p.N, TN), groups);
  hipLaunchKernelGGL((gg_plain_kernel<T, EPI, RAGGED_K>), grid, dim3(256), 0, s, p);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

template <typename T>
moe_status_t launch_dt(const GemmP& p, int epi, bool ragged_k, hipStream_t s) {
  if (ragged_k) return launch_t<T, EPI_PLAIN, true>(p, s);
  switch (epi) {
    case EPI_PLAIN: return launch_t<T, EPI_PLAIN, false>(p, s);
    case EPI_ACT_FWD: return launch_t<T, EPI_ACT_FWD, false>(p, s);
    case EPI_GLU_FWD: return launch_t<T, EPI_GLU_FWD, false>(p, s);
    case EPI_ACT_BWD: return launch_t<T, EPI_ACT_BWD, false>(p, s);
    default: return launch_t<T, EPI_GLU_BWD, false>(p, s);
  }
}

}  // namespace

moe_status_t launch_gemm_plain(const GemmP& p, int dtype, int epi, bool ragged_k, hipStream_t s) {
  return dtype == MOE_BF16 ? launch_dt<bf16_t>(p, epi, ragged_k, s) : launch_dt<float>(p, epi, ragged_k, s);
}

}  // namespace moe
