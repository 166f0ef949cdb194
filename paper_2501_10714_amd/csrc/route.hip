// Gate, top-k, capacity positions (FSMoE Sec. 2.1 "Gating Function" and the capacity rule of the
// ordering function) and the gate's backward pass (Sec. 4.4).
//
// Forward, up to four launches on one stream:
//   1. the gate: logits, top-k, G(I), and a histogram of choices per (expert, rank j, 64-token tile).  Three kernels,
//      chosen by shape (route_t):
//        gate_mfma_kernel (gate_mfma.hip)  bf16 inputs, up to 64 experts, the plain gate: product on the matrix cores,
//                          fp64 repair of the logits a close top-k decision rests on;
//        gate_small_kernel  everything else whose W_g rows of one 8-expert group fit in LDS: fp64 product on the
//                          vector ALU with the token rows in registers, every logit rounded once to fp32;
//        widen_gate_kernel + gate_topk_kernel  very large d_model (W_g widened to fp64, both operands staged through
//                          LDS in K chunks); gate_topk_kernel also runs the tail alone for gates that bring their
//                          own logits (X-MoE) and the product alone (the noise product of the noisy gate);
//   2. scan_hist_kernel    exclusive prefix over (j, tile) for every expert: the number of earlier
//                          assignments to that expert in rank-major, token-minor order
//   3. positions_kernel    count = min(total, T), offsets = exclusive prefix of count, then
//                          pos / row_of / src_of_row: tile base + rank among the wave's lanes
// Positions come from prefix sums only (no atomics decide an index), so the result is the same on
// every run and equals the serial walk "for j, for t".
//
// In the two fp64 gate kernels the logits are an fp64 product on the vector ALU: routing and logits that match an
// independent fp64 evaluation bit for bit whatever the summation order, at the price of being bound by that unit.
// The matrix-core gate keeps the routing at that bar and gives up bit-equality of the logits no decision rests on.
#include <stdlib.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "common.h"
#include "gemm_params.h"

namespace moe {
namespace {

constexpr int kTile = 64;          // tokens per block
constexpr int kGateThreads = 256;
constexpr int kKC = 64;            // k per staged chunk
constexpr int kXP = kTile + 2;     // pitch (doubles) of a k-row of the staged x chunk
constexpr int kMaxK = 8;

// what gate_topk_kernel does: the whole gate; the product only (logits out, nothing else written); or top-k,
// G(I) and the histogram on logits that are already there
enum GateMode { kGateFull = 0, kGateLogitsOnly = 1, kGateFromLogits = 2 };

struct RoutePlan {
  int ee;      // experts per pass (8,16,32,64)
  int ep;      // padded expert count (multiple of ee)
  int nkc;     // K chunks
  int mpad;    // padded rows of the fp64 gate matrix
  int nb;      // 64-token tiles
  size_t off_wd, off_hist, off_total, bytes;
};

// LDS of gate_topk_kernel with ee experts per pass: the two staged operands (double buffered), the tile's
// logits, the histogram of choices
size_t gate_lds_bytes(int ee, int n_experts, int top_k) {
  return (size_t)2 * kKC * kXP * sizeof(double) + (size_t)2 * kKC * ee * sizeof(double) +
         (size_t)kTile * (n_experts + 1) * sizeof(float) + (size_t)top_k * n_experts * sizeof(int32_t);
}

RoutePlan route_plan(const moe_config_t& c) {
  RoutePlan p;
  int e = c.n_experts;
  p.ee = e <= 8 ? 8 : e <= 16 ? 16 : e <= 32 ? 32 : 64;
  // many experts: fewer per pass, so that the logits of the tile still fit beside the operands (160 KB of LDS;
  // E = 256 with top_k = 8 fits at 16 per pass)
  while (p.ee > 8 && gate_lds_bytes(p.ee, e, c.top_k) > (size_t)160 * 1024) p.ee /= 2;
  p.ep = ceil_div(e, p.ee) * p.ee;
  p.nkc = ceil_div(c.d_model, kKC);
  p.mpad = p.nkc * kKC;
  p.nb = ceil_div(c.n_tokens, kTile);
  size_t o = 0;
  p.off_wd = o; o += align_up((size_t)p.mpad * p.ep * sizeof(double), 256);
  p.off_hist = o; o += align_up((size_t)e * c.top_k * p.nb * sizeof(int32_t), 256);
  p.off_total = o; o += align_up((size_t)e * sizeof(int32_t), 256);
  p.bytes = o;
  return p;
}

template <typename T>
__global__ void widen_gate_kernel(const T* __restrict__ w_gate, double* __restrict__ wd, int d_model, int n_experts,
                                  int mpad, int ep) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= mpad * ep) return;
  int m = i / ep, e = i % ep;
  wd[i] = (m < d_model && e < n_experts) ? (double)Elem<T>::ld(w_gate + (size_t)m * n_experts + e) : 0.0;
}

template <typename T> struct Widen;
template <> struct Widen<bf16_t> {
  static constexpr int kN = 8;
  __device__ static __forceinline__ void run(const uint4& r, double* d) {
    uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      d[2 * i] = (double)__uint_as_float(w[i] << 16);
      d[2 * i + 1] = (double)__uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
};
template <> struct Widen<float> {
  static constexpr int kN = 4;
  __device__ static __forceinline__ void run(const uint4& r, double* d) {
    d[0] = (double)__uint_as_float(r.x); d[1] = (double)__uint_as_float(r.y);
    d[2] = (double)__uint_as_float(r.z); d[3] = (double)__uint_as_float(r.w);
  }
};

// Everything after the product, for the tile of 64 tokens whose logits are in lg (or, mode kGateFromLogits, in
// memory): logits out, top-k and G(I) (one token per lane of wave 0), the histogram of choices.  Called by all
// threads of the block; hcnt has been cleared and lg written before the call (with a barrier in between).
__device__ __forceinline__ void gate_tail(float* __restrict__ lg, int32_t* __restrict__ hcnt, float* __restrict__ logits,
                                          float* __restrict__ probs, int32_t* __restrict__ topk_idx,
                                          float* __restrict__ topk_w, int32_t* __restrict__ hist, int n_tokens,
                                          int n_experts, int top_k, int renormalize, int nb, int mode, int nthreads) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int t0 = blockIdx.x * kTile;
  const int lgs = n_experts + 1;
  if (mode == kGateFromLogits) {  // the tile's logits come from memory
    for (int i = tid; i < kTile * n_experts; i += nthreads) {
      int tk = i / n_experts, e = i % n_experts;
      lg[tk * lgs + e] = t0 + tk < n_tokens ? logits[(size_t)(t0 + tk) * n_experts + e] : 0.0f;
    }
    __syncthreads();
  } else {  // logits out, coalesced over the tile
    for (int i = tid; i < kTile * n_experts; i += nthreads) {
      int tk = i / n_experts, e = i % n_experts;
      if (t0 + tk < n_tokens) logits[(size_t)(t0 + tk) * n_experts + e] = lg[tk * lgs + e];
    }
    if (mode == kGateLogitsOnly) return;  // the same for every thread of the block
    __syncthreads();  // wave 0 overwrites lg with G(I) below: every wave has copied its logits out by then
  }

  // top-k and G(I): one token per lane of wave 0
  if (wave == 0) {
    const int t = t0 + lane;
    if (t < n_tokens) {
      float* l = lg + lane * lgs;
      int sel[kMaxK];
      float selv[kMaxK];
      float prev_v = 0.0f;
      int prev_e = -1;
      for (int j = 0; j < top_k; ++j) {
        float bv = 0.0f;
        int be = -1;
        for (int e = 0; e < n_experts; ++e) {
          float v = l[e];
          bool eligible = (j == 0) || (v < prev_v) || (v == prev_v && e > prev_e);
          if (eligible && (be < 0 || v > bv)) { bv = v; be = e; }
        }
        if (be < 0) {  // only with NaN logits (every comparison false): lowest expert not yet taken, so indices stay valid
          for (int e = 0; e < n_experts && be < 0; ++e) {
            bool taken = false;
            for (int i = 0; i < j; ++i) taken |= sel[i] == e;
            if (!taken) { be = e; bv = l[e]; }
          }
        }
        sel[j] = be; selv[j] = bv; prev_v = bv; prev_e = be;
        topk_idx[(size_t)t * top_k + j] = be;
        atomicAdd(&hcnt[j * n_experts + be], 1);
      }
      const float mx = selv[0];
      if (renormalize == MOE_GATE_SIGMOID) {  // sigmoid gate: sigma(H_i), the choices do not interact
        for (int e = 0; e < n_experts; ++e) l[e] = 1.0f / (1.0f + expf(-l[e]));
        for (int j = 0; j < top_k; ++j) topk_w[(size_t)t * top_k + j] = l[sel[j]];
      } else if (renormalize) {
        float z[kMaxK], s = 0.0f;
        for (int j = 0; j < top_k; ++j) { z[j] = expf(selv[j] - mx); s += z[j]; }
        for (int e = 0; e < n_experts; ++e) l[e] = 0.0f;
        for (int j = 0; j < top_k; ++j) {
          float w = z[j] / s;
          l[sel[j]] = w;
          topk_w[(size_t)t * top_k + j] = w;
        }
      } else {
        float s = 0.0f;
        for (int e = 0; e < n_experts; ++e) { float z = expf(l[e] - mx); l[e] = z; s += z; }
        for (int e = 0; e < n_experts; ++e) l[e] = l[e] / s;
        for (int j = 0; j < top_k; ++j) topk_w[(size_t)t * top_k + j] = l[sel[j]];
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < kTile * n_experts; i += nthreads) {
    int tk = i / n_experts, e = i % n_experts;
    if (t0 + tk < n_tokens) probs[(size_t)(t0 + tk) * n_experts + e] = lg[tk * lgs + e];
  }
  for (int i = tid; i < top_k * n_experts; i += nthreads) {
    int j = i / n_experts, e = i % n_experts;
    hist[((size_t)e * top_k + j) * nb + blockIdx.x] = hcnt[i];
  }
}

// logits = fp32(x.W_g + b_g) with the products and the sum in fp64, then top-k, G(I) and the
// histogram of choices, for one tile of 64 tokens.  The fp64 GEMM is register tiled: a thread owns
// 8 tokens x 8 experts for a slice of every 64-wide K chunk; x (widened to fp64 while it is staged)
// and the fp64 copy of W_g come from LDS, double buffered, with the next chunk's global loads in
// flight under the FMAs.  (The fp64 matrix instruction was tried for this product and measured slower.)
// Eight consecutive lanes stage the same 16-byte column chunk of eight consecutive token rows, which
// keeps the transposed LDS writes of the widened chunk nearly conflict-free.  The K slices are then summed in slice order (fixed, so runs repeat).
template <typename T, int NEG>  // NEG groups of 8 experts per pass
__global__ __launch_bounds__(kGateThreads) void gate_topk_kernel(
    const T* __restrict__ x, const double* __restrict__ wd, const float* __restrict__ b_gate,
    float* __restrict__ logits, float* __restrict__ probs, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    int32_t* __restrict__ hist, int n_tokens, int d_model, int n_experts, int top_k, int renormalize, int ep, int nkc,
    int nb, const float* __restrict__ noise, const float* __restrict__ noise_logits, int mode) {
  constexpr int EE = 8 * NEG;         // experts per pass
  constexpr int NKS = 32 / NEG;       // K slices
  constexpr int KPS = kKC / NKS;      // k per slice and chunk
  constexpr int R = NKS / 4;          // slices summed per reduction round
  constexpr int V = Widen<T>::kN;     // elements per 16-byte load
  constexpr int XLD = kTile * kKC / V / kGateThreads;  // 16-byte x loads per thread and chunk
  constexpr int WLD = kKC * EE / 2 / kGateThreads;     // 16-byte W loads per thread and chunk
  extern __shared__ __align__(16) unsigned char smem[];
  double* xs = reinterpret_cast<double*>(smem);                        // [2][kKC][kXP]; later partial sums
  double* ws = xs + 2 * kKC * kXP;                                     // [2][kKC][EE]
  float* lg = reinterpret_cast<float*>(ws + 2 * kKC * EE);             // [kTile][n_experts + 1]
  int32_t* hcnt = reinterpret_cast<int32_t*>(lg + kTile * (n_experts + 1));  // [top_k][n_experts]
  double* part = xs;                    // [R][EE][kTile] after the K loop
  double* red = xs + R * EE * kTile;    // [EE][kTile]

  const int tid = threadIdx.x;
  const int tg = tid & 7, eg = (tid >> 3) % NEG, ks = tid / (8 * NEG);
  const int t0 = blockIdx.x * kTile;
  const int lgs = n_experts + 1;

  for (int i = tid; i < top_k * n_experts; i += kGateThreads) hcnt[i] = 0;

  const int ep_run = mode == kGateFromLogits ? 0 : ep;
  for (int ec = 0; ec < ep_run; ec += EE) {
    double acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = 0.0;

    uint4 xr[XLD];
    double2 wr[WLD];
    auto fetch = [&](int kc) {
#pragma unroll
      for (int r = 0; r < XLD; ++r) {
        const int q = tid + kGateThreads * r;
        const int row = (q & 7) + 8 * (q / (8 * (kKC / V))), c = (q >> 3) % (kKC / V);
        const int t = t0 + row, k = kc * kKC + c * V;
        xr[r] = (t < n_tokens && k < d_model) ? *reinterpret_cast<const uint4*>(x + (size_t)t * d_model + k)
                                              : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < WLD; ++r) {
        const int q = tid + kGateThreads * r;
        const int row = q / (EE / 2), c2 = q % (EE / 2);
        wr[r] = *reinterpret_cast<const double2*>(wd + (size_t)(kc * kKC + row) * ep + ec + 2 * c2);
      }
    };
    auto stash = [&](int buf) {
      double* xb = xs + buf * kKC * kXP;
      double* wb = ws + buf * kKC * EE;
#pragma unroll
      for (int r = 0; r < XLD; ++r) {
        const int q = tid + kGateThreads * r;
        const int row = (q & 7) + 8 * (q / (8 * (kKC / V))), c = (q >> 3) % (kKC / V);  // as in fetch
        double xd[V];
        Widen<T>::run(xr[r], xd);
#pragma unroll
        for (int i = 0; i < V; ++i) xb[(c * V + i) * kXP + row] = xd[i];
      }
#pragma unroll
      for (int r = 0; r < WLD; ++r) {
        const int q = tid + kGateThreads * r;
        const int row = q / (EE / 2), c2 = q % (EE / 2);
        *reinterpret_cast<double2*>(wb + row * EE + 2 * c2) = wr[r];
      }
    };

    __syncthreads();  // the LDS of the previous pass (partial sums) is free again
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kc = 0; kc < nkc; ++kc) {
      if (kc + 1 < nkc) fetch(kc + 1);
      const double* xb = xs + (kc & 1) * kKC * kXP + 8 * tg;
      const double* wb = ws + (kc & 1) * kKC * EE + 8 * eg;
#pragma unroll 2
      for (int kk = 0; kk < KPS; ++kk) {
        const int k = ks * KPS + kk;
        double xv[8], wv[8];
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
          const double2 a = *reinterpret_cast<const double2*>(xb + k * kXP + i);
          const double2 b = *reinterpret_cast<const double2*>(wb + k * EE + i);
          xv[i] = a.x; xv[i + 1] = a.y; wv[i] = b.x; wv[i + 1] = b.y;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[i][j] = fma(xv[i], wv[j], acc[i][j]);
      }
      if (kc + 1 < nkc) stash((kc + 1) & 1);  // that buffer was last read in iteration kc-1
      __syncthreads();
    }
    // sum the K slices in slice order: four rounds of R slices each
    for (int rd = 0; rd < 4; ++rd) {
      if (ks / R == rd) {
        double* pp = part + (size_t)(ks % R) * EE * kTile;
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int i = 0; i < 8; ++i) pp[(8 * eg + j) * kTile + 8 * tg + i] = acc[i][j];
      }
      __syncthreads();
      for (int o = tid; o < EE * kTile; o += kGateThreads) {
        double v = rd == 0 ? 0.0 : red[o];
#pragma unroll
        for (int sl = 0; sl < R; ++sl) v += part[(size_t)sl * EE * kTile + o];
        red[o] = v;
      }
      __syncthreads();
    }
    for (int i = tid; i < EE * kTile; i += kGateThreads) {
      int e = i / kTile, tk = i % kTile;
      if (ec + e < n_experts) {
        double v = red[e * kTile + tk];
        if (b_gate != nullptr) v += (double)b_gate[ec + e];
        float f = (float)v;
        if (noise != nullptr && t0 + tk < n_tokens) {
          // noisy gate (Sec. 2.1): H = I.W_g + noise * Softplus(I.W_noise), formed in fp64 from the two fp32
          // products and rounded once
          const size_t gi = (size_t)(t0 + tk) * n_experts + ec + e;
          const double z = (double)noise_logits[gi];
          const double sp = z > 0.0 ? z + log1p(exp(-z)) : log1p(exp(z));
          f = (float)((double)f + (double)noise[gi] * sp);
        }
        lg[tk * lgs + ec + e] = f;
      }
    }
    __syncthreads();
  }

  gate_tail(lg, hcnt, logits, probs, topk_idx, topk_w, hist, n_tokens, n_experts, top_k, renormalize, nb, mode, kGateThreads);
}

// ---- the product, 8 experts at a time.  Every x element then meets all experts of the group in one thread, so x
// needs no LDS: a wave owns 8 tokens, its lanes own consecutive 16-byte pieces of their rows (64 lanes = 1 KB of every
// row per step, read straight from memory into registers, one step ahead), and each lane keeps 8 tokens x 8
// experts of fp64 partial sums over the k it has seen.  W_g sits in LDS in its stored format (M rows of 8
// experts, zero padded; 16 bytes of padding after every lane's piece, so the 16-byte reads of 16 neighbouring
// lanes cover all banks) and is widened as it is used.  At the end the 64 partial sums of the 64 lanes are added
// by a butterfly in which every step halves what a lane holds (fixed order, so runs repeat): lane l ends with
// the logit of token l / 8, expert l % 8.
constexpr int kSmallThreads = 512;  // 8 waves x 8 tokens = the 64-token tile of the tail
constexpr int kSmallE = 8;

template <typename T> struct SmallGate;
template <> struct SmallGate<bf16_t> {
  static constexpr int kV = 8;  // k per 16-byte piece of an x row
  __device__ static __forceinline__ double x_at(const uint4& r, int j) {
    const uint32_t w = j < 2 ? r.x : j < 4 ? r.y : j < 6 ? r.z : r.w;
    return (double)__uint_as_float((j & 1) ? (w & 0xFFFF0000u) : (w << 16));
  }
  // row of 8 experts (16 bytes) -> doubles
  __device__ static __forceinline__ void w_row(const unsigned char* p, double* d) {
    Widen<bf16_t>::run(*reinterpret_cast<const uint4*>(p), d);
  }
};
template <> struct SmallGate<float> {
  static constexpr int kV = 4;
  __device__ static __forceinline__ double x_at(const uint4& r, int j) {
    return (double)__uint_as_float(j == 0 ? r.x : j == 1 ? r.y : j == 2 ? r.z : r.w);
  }
  __device__ static __forceinline__ void w_row(const unsigned char* p, double* d) {  // 32 bytes
    Widen<float>::run(*reinterpret_cast<const uint4*>(p), d);
    Widen<float>::run(*reinterpret_cast<const uint4*>(p + 16), d + 4);
  }
};
constexpr int kSmallPiece = 128 + 16;  // LDS bytes of the W rows of one lane's piece (kV rows of 8 experts) + padding

inline size_t small_gate_lds_bytes(int d_model, int n_experts, int top_k, int v) {
  const int pieces = ceil_div(d_model, 64 * v) * 64;
  return (size_t)pieces * kSmallPiece + (size_t)kTile * (n_experts + 1) * sizeof(float) +
         (size_t)top_k * n_experts * sizeof(int32_t);
}

template <typename T>
__global__ __launch_bounds__(kSmallThreads) void gate_small_kernel(
    const T* __restrict__ x, const T* __restrict__ w_gate, const float* __restrict__ b_gate, float* __restrict__ logits,
    float* __restrict__ probs, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int32_t* __restrict__ hist,
    int n_tokens, int d_model, int n_experts, int top_k, int renormalize, int nb, const float* __restrict__ noise,
    const float* __restrict__ noise_logits, int mode) {
  typedef SmallGate<T> G;
  constexpr int V = G::kV;
  constexpr int kRowBytes = kSmallE * (int)sizeof(T);
  extern __shared__ __align__(16) unsigned char smem[];
  const int nsteps = (d_model + 64 * V - 1) / (64 * V);
  const int pieces = nsteps * 64;
  unsigned char* wl = smem;                                                   // [pieces][kSmallPiece]
  float* lg = reinterpret_cast<float*>(wl + (size_t)pieces * kSmallPiece);    // [kTile][n_experts + 1]
  int32_t* hcnt = reinterpret_cast<int32_t*>(lg + kTile * (n_experts + 1));   // [top_k][n_experts]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lgs = n_experts + 1;
  const int tb = blockIdx.x * kTile + wave * 8;  // first token of this wave

  for (int i = tid; i < top_k * n_experts; i += kSmallThreads) hcnt[i] = 0;

  // experts in groups of 8; with more than one group the x rows are read again for every group (from L2 or the
  // memory-side cache: a workgroup's 64 rows are 64 * M elements)
  for (int e0 = 0; e0 < n_experts; e0 += kSmallE) {
    const int ge = min(kSmallE, n_experts - e0);  // experts in this group
    if (e0 > 0) __syncthreads();                  // every wave is done with the W rows of the group before
    // W_g -> LDS: element (k, e0 + e) at piece k / V, row k % V, column e; columns past the group and rows past M are zero
    if (ge == kSmallE && n_experts % kSmallE == 0 && (reinterpret_cast<uintptr_t>(w_gate) & 15) == 0) {  // 16 bytes at a time
      constexpr int kPer = kRowBytes / 16;  // 16-byte parts of a group's share of a row
      for (int i = tid; i < pieces * V * kPer; i += kSmallThreads) {
        const int k = i / kPer, part = i % kPer;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (k < d_model) v = reinterpret_cast<const uint4*>(w_gate + (size_t)k * n_experts + e0)[part];
        *reinterpret_cast<uint4*>(wl + (size_t)(k / V) * kSmallPiece + (k % V) * kRowBytes + part * 16) = v;
      }
    } else {
      for (int i = tid; i < pieces * V * kSmallE; i += kSmallThreads) {
        const int k = i / kSmallE, e = i % kSmallE;
        T v = 0;
        if (k < d_model && e < ge) v = w_gate[(size_t)k * n_experts + e0 + e];
        *reinterpret_cast<T*>(wl + (size_t)(k / V) * kSmallPiece + (k % V) * kRowBytes + e * sizeof(T)) = v;
      }
    }
    __syncthreads();

    double acc[8][kSmallE];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int e = 0; e < kSmallE; ++e) acc[i][e] = 0.0;
    uint4 cur[8], nxt[8];
    auto fetch = [&](int s, uint4(&r)[8]) {
      const int k0 = (s * 64 + lane) * V;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        r[i] = (k0 < d_model && tb + i < n_tokens) ? *reinterpret_cast<const uint4*>(x + (size_t)(tb + i) * d_model + k0)
                                                   : make_uint4(0, 0, 0, 0);
    };
    fetch(0, cur);
    for (int s = 0; s < nsteps; ++s) {
      if (s + 1 < nsteps) fetch(s + 1, nxt);
      const unsigned char* wp = wl + (size_t)(s * 64 + lane) * kSmallPiece;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        double wv[kSmallE];
        G::w_row(wp + j * kRowBytes, wv);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const double xv = G::x_at(cur[i], j);
#pragma unroll
          for (int e = 0; e < kSmallE; ++e) acc[i][e] = fma(xv, wv[e], acc[i][e]);
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) cur[i] = nxt[i];
    }

    // add the partial sums of the 64 lanes: after the step with distance b a lane holds b of the 64 (token, expert)
    // sums, those whose index agrees with its lane number in the bits above b
    double* v = &acc[0][0];
#pragma unroll
    for (int b = 32; b >= 1; b >>= 1) {
      const bool up = (lane & b) != 0;
#pragma unroll
      for (int j = 0; j < b; ++j) {
        const double keep = up ? v[j + b] : v[j];
        const double send = up ? v[j] : v[j + b];
        v[j] = keep + __shfl_xor(send, b, 64);
      }
    }
    const int i = lane >> 3, e = e0 + (lane & 7);
    if (e < n_experts) {
      double sum = v[0];
      if (b_gate != nullptr) sum += (double)b_gate[e];
      float f = (float)sum;
      if (noise != nullptr && tb + i < n_tokens) {  // noisy gate, as in gate_topk_kernel
        const size_t gi = (size_t)(tb + i) * n_experts + e;
        const double z = (double)noise_logits[gi];
        const double sp = z > 0.0 ? z + log1p(exp(-z)) : log1p(exp(z));
        f = (float)((double)f + (double)noise[gi] * sp);
      }
      lg[(wave * 8 + i) * lgs + e] = f;
    }
  }
  __syncthreads();
  gate_tail(lg, hcnt, logits, probs, topk_idx, topk_w, hist, n_tokens, n_experts, top_k, renormalize, nb, mode, kSmallThreads);
}

// One block per expert: in-place exclusive prefix over its (rank j, tile) histogram entries.
__global__ __launch_bounds__(256) void scan_hist_kernel(int32_t* __restrict__ hist, int32_t* __restrict__ total,
                                                        int len) {
  __shared__ int32_t part[256];
  int32_t* h = hist + (size_t)blockIdx.x * len;
  const int seg = (len + 255) / 256;
  const int lo = threadIdx.x * seg, hi = min(lo + seg, len);
  int32_t s = 0;
  for (int i = lo; i < hi; ++i) s += h[i];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {  // Hillis-Steele inclusive scan
    int32_t v = (int)threadIdx.x >= o ? part[threadIdx.x - o] : 0;
    __syncthreads();
    part[threadIdx.x] += v;
    __syncthreads();
  }
  int32_t run = part[threadIdx.x] - s;
  for (int i = lo; i < hi; ++i) {
    int32_t v = h[i];
    h[i] = run;
    run += v;
  }
  if (threadIdx.x == 255) total[blockIdx.x] = part[255];
}

// One wave per 64-token tile, one token per lane.  Every block first derives count = min(total, T)
// and offsets = exclusive prefix of count from the per-expert totals (E <= 256 values, redundantly per
// block; block 0 also writes them out).
__global__ __launch_bounds__(256) void positions_kernel(const int32_t* __restrict__ topk_idx,
                                                        const int32_t* __restrict__ base,
                                                        const int32_t* __restrict__ total, int32_t* __restrict__ count,
                                                        int32_t* __restrict__ offsets, int32_t* __restrict__ pos,
                                                        int32_t* __restrict__ row_of, int32_t* __restrict__ src_of_row,
                                                        int n_tokens, int n_experts, int top_k, int capacity, int nb) {
  __shared__ int32_t s_off[257];
  {
    const int e = threadIdx.x;
    int32_t c = 0;
    if (e < n_experts) {
      c = total[e];
      if (capacity > 0 && c > capacity) c = capacity;
    }
    s_off[e + 1] = c;
    if (e == 0) s_off[0] = 0;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {  // inclusive scan of s_off[1..256]
      const int32_t v = e >= o ? s_off[e + 1 - o] : 0;
      __syncthreads();
      s_off[e + 1] += v;
      __syncthreads();
    }
    if (blockIdx.x == 0) {
      if (e < n_experts) { count[e] = c; offsets[e] = s_off[e]; }
      if (e == 0) offsets[n_experts] = s_off[n_experts];
    }
  }
  const int lane = threadIdx.x & 63;
  const int tile = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int t = tile * kTile + lane;
  const bool live = tile < nb && t < n_tokens;
  if (tile < nb) {
    for (int j = 0; j < top_k; ++j) {
      const int e = live ? topk_idx[(size_t)t * top_k + j] : -1;
      // rank among the lanes of this wave that chose the same expert and come earlier
      int local = 0;
      unsigned long long todo = __ballot(live);
      while (todo != 0ull) {
        const int leader = __ffsll((long long)todo) - 1;
        const int e0 = __shfl(e, leader, 64);
        const unsigned long long same = __ballot(live && e == e0);
        if (live && e == e0) local = __popcll(same & ((1ull << lane) - 1ull));
        todo &= ~same;
      }
      if (live) {
        const int rank = base[((size_t)e * top_k + j) * nb + tile] + local;
        const bool kept = capacity <= 0 || rank < capacity;
        const int p = kept ? rank : -1;
        const int row = kept ? s_off[e] + rank : -1;
        pos[(size_t)t * top_k + j] = p;
        row_of[(size_t)t * top_k + j] = row;
        if (kept) src_of_row[row] = t * top_k + j;
      }
    }
  }
  // rows past A have no source
  const int a = s_off[n_experts];
  const int all = n_tokens * top_k;
  for (int r = a + blockIdx.x * blockDim.x + threadIdx.x; r < all; r += gridDim.x * blockDim.x) src_of_row[r] = -1;
}

// Kernels that use more than 64 KB of LDS need the attribute below once per device.  A host-side call (no stream
// work, so it is legal under stream capture); done on the first launch on each device, from whichever thread
// gets there first (setting it twice is harmless, so a racing second thread just sets it again).
template <typename K>
moe_status_t allow_full_lds(K kernel, std::atomic<uint64_t>& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    set_error("gate: no current device");
    return MOE_ERR_DEVICE;
  }
  const uint64_t bit = 1ull << dev;
  if (done.load(std::memory_order_acquire) & bit) return MOE_OK;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           160 * 1024);
  if (e != hipSuccess) {
    set_error("gate: hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: %s", hipGetErrorString(e));
    return MOE_ERR_DEVICE;
  }
  done.fetch_or(bit, std::memory_order_release);
  return MOE_OK;
}

template <typename T, int NEG>
moe_status_t launch_gate(const moe_config_t& c, const RoutePlan& p, const void* x, const double* wd, const float* b_gate,
                 float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* hist, const float* noise,
                 const float* noise_logits, int mode, hipStream_t s) {
  constexpr int EE = 8 * NEG;
  const size_t lds = gate_lds_bytes(EE, c.n_experts, c.top_k);
  static std::atomic<uint64_t> attr_done{0};
  const moe_status_t st = allow_full_lds(gate_topk_kernel<T, NEG>, attr_done);
  if (st != MOE_OK) return st;
  hipLaunchKernelGGL((gate_topk_kernel<T, NEG>), dim3(p.nb), dim3(kGateThreads), lds, s, (const T*)x, wd, b_gate, logits,
                     probs, topk_idx, topk_w, hist, c.n_tokens, c.d_model, c.n_experts, c.top_k, c.renormalize, p.ep,
                     p.nkc, p.nb, noise, noise_logits, mode);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

template <typename T>
// noise, noise_logits: NULL, or the inputs of the noisy gate (logits = x.W_g + b + noise * Softplus(noise_logits)).
// mode: kGateLogitsOnly stops after the product (logits out: noise_logits = x.W_noise, or the X-MoE projection);
// kGateFromLogits takes `logits` as they are and does the rest (x, w_gate, b_gate are not read).
moe_status_t route_t(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate, float* logits,
                     float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                     int32_t* offsets, int32_t* src_of_row, void* ws, const float* noise, const float* noise_logits,
                     int mode, hipStream_t s) {
  RoutePlan p = route_plan(c);
  unsigned char* w = static_cast<unsigned char*>(ws);
  double* wd = reinterpret_cast<double*>(w + p.off_wd);
  int32_t* hist = reinterpret_cast<int32_t*>(w + p.off_hist);
  int32_t* total = reinterpret_cast<int32_t*>(w + p.off_total);
  int nwd = p.mpad * p.ep;
  // the kernel that reads x straight into registers, whenever the W_g rows of 8 experts fit in LDS (M up to
  // about 8000 in bf16); measured faster than gate_topk_kernel at every shape tried (2x at E = 8, 1.1x at 32 and 64,
  // 1.4x at 256)
#ifdef MOE_DEBUG_SWITCHES
  static const bool force_wide = getenv("MOE_GATE_WIDE") != nullptr;  // for A/B timing of the two gate kernels
#else
  constexpr bool force_wide = false;
#endif
  const size_t small_lds = small_gate_lds_bytes(c.d_model, c.n_experts, c.top_k, SmallGate<T>::kV);
  // bf16, up to 64 experts, the plain gate: the product on the matrix cores, exact fp64 logits only for the tokens
  // whose top-k decision is close (gate_mfma.hip).  The other modes need every logit exact and take the kernels below.
  if (std::is_same<T, bf16_t>::value && mode == kGateFull && noise == nullptr && !force_wide && gate_mfma_supported(c)) {
    const moe_status_t mst = launch_gate_mfma(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, hist, p.nb, s);
    if (mst != MOE_OK) return mst;
  } else if (mode != kGateFromLogits && small_lds <= (size_t)160 * 1024 && !force_wide) {
    static std::atomic<uint64_t> attr_done{0};
    const moe_status_t ast = allow_full_lds(gate_small_kernel<T>, attr_done);
    if (ast != MOE_OK) return ast;
    hipLaunchKernelGGL(gate_small_kernel<T>, dim3(p.nb), dim3(kSmallThreads), small_lds, s, (const T*)x, (const T*)w_gate,
                       b_gate, logits, probs, topk_idx, topk_w, hist, c.n_tokens, c.d_model, c.n_experts, c.top_k,
                       c.renormalize, p.nb, noise, noise_logits, mode);
    MOE_CHECK_LAUNCH();
  } else {
  if (mode != kGateFromLogits) {
    hipLaunchKernelGGL(widen_gate_kernel<T>, dim3(ceil_div(nwd, 256)), dim3(256), 0, s, (const T*)w_gate, wd, c.d_model,
                       c.n_experts, p.mpad, p.ep);
    MOE_CHECK_LAUNCH();
  }
  moe_status_t gst;
  switch (p.ee) {
    case 8: gst = launch_gate<T, 1>(c, p, x, wd, b_gate, logits, probs, topk_idx, topk_w, hist, noise, noise_logits, mode, s); break;
    case 16: gst = launch_gate<T, 2>(c, p, x, wd, b_gate, logits, probs, topk_idx, topk_w, hist, noise, noise_logits, mode, s); break;
    case 32: gst = launch_gate<T, 4>(c, p, x, wd, b_gate, logits, probs, topk_idx, topk_w, hist, noise, noise_logits, mode, s); break;
    default: gst = launch_gate<T, 8>(c, p, x, wd, b_gate, logits, probs, topk_idx, topk_w, hist, noise, noise_logits, mode, s); break;
  }
  if (gst != MOE_OK) return gst;
  }
  if (mode == kGateLogitsOnly) return MOE_OK;
  hipLaunchKernelGGL(scan_hist_kernel, dim3(c.n_experts), dim3(256), 0, s, hist, total, c.top_k * p.nb);
  MOE_CHECK_LAUNCH();
  hipLaunchKernelGGL(positions_kernel, dim3(ceil_div(p.nb, 4)), dim3(256), 0, s, topk_idx, hist, total, count, offsets,
                     pos, row_of, src_of_row, c.n_tokens, c.n_experts, c.top_k, c.capacity, p.nb);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

// ----------------------------------------------------------------------------- backward of the gate

constexpr int kDwTokens = 256;   // tokens per partial-sum tile of dW_g
constexpr int kDwThreads = 128;
constexpr int kDxTokens = 16;    // tokens per block of the dx update
constexpr int kEc = 8;           // experts per register chunk

constexpr int kSplitTokens = 512;  // tokens per split-K group of the bf16 dW_g product

// steps of the gate's backward: dlogits (and the padded bf16 copies of the MFMA path); dx += dlogits.W_g^T; dW_g and db_g
enum RouteBwdParts { kPartDl = 1, kPartDx = 2, kPartDw = 4, kPartAll = 7 };

// bf16: the two products of the gate backward go through the MFMA grouped GEMM (fp32: plain kernels)
inline bool gate_bwd_on_mfma(const moe_config_t& c) { return c.dtype == MOE_BF16; }

struct RouteBwdPlan {
  int ntile;   // 256-token tiles (fp32 path partial sums, and the db_g column sums of both paths)
  int ep;      // experts padded to a multiple of 32 (bf16 path: K of the dx product, N of the dW_g product)
  int nsplit;  // split-K groups of the bf16 dW_g product
  size_t off_dl, off_part, off_bpart, off_dlb, off_wgp, off_tok, bytes;
};

RouteBwdPlan route_bwd_plan(const moe_config_t& c) {
  RouteBwdPlan p;
  const bool bf = gate_bwd_on_mfma(c);
  p.ntile = ceil_div(c.n_tokens, kDwTokens);
  p.ep = ceil_div(c.n_experts, 32) * 32;
  p.nsplit = ceil_div(c.n_tokens, kSplitTokens);
  size_t o = 0;
  p.off_dl = o; o += align_up((size_t)c.n_tokens * c.n_experts * sizeof(float), 256);
  p.off_part = o;  // fp32 path: [ntile][M][E] f32; bf16 path: [nsplit][M][ep] bf16
  o += align_up(bf ? (size_t)p.nsplit * c.d_model * p.ep * 2 : (size_t)p.ntile * c.d_model * c.n_experts * sizeof(float), 256);
  p.off_bpart = o; o += align_up((size_t)p.ntile * c.n_experts * sizeof(float), 256);
  p.off_dlb = o; o += bf ? align_up((size_t)c.n_tokens * p.ep * 2, 256) : 0;
  p.off_wgp = o; o += bf ? align_up((size_t)c.d_model * p.ep * 2, 256) : 0;
  p.off_tok = o; o += bf ? align_up((size_t)(p.nsplit + 3) * sizeof(int32_t), 256) : 0;
  p.bytes = o;
  return p;
}

// dlogits[t,e] = probs[t,e] * (g[t,e] - <g[t,:], probs[t,:]>), g = dtopk_w scattered to the kept choices;
// sigmoid gate: dlogits[t,e] = g[t,e] * probs[t,e] * (1 - probs[t,e])
__global__ __launch_bounds__(256) void dlogits_kernel(const float* __restrict__ probs,
                                                      const int32_t* __restrict__ topk_idx,
                                                      const int32_t* __restrict__ pos,
                                                      const float* __restrict__ dtopk_w, float* __restrict__ dl,
                                                      bf16_t* __restrict__ dlb, int n_tokens, int n_experts,
                                                      int top_k, int ep, int gate, const float* __restrict__ noise,
                                                      const float* __restrict__ noise_logits) {
  // one thread per (token, padded expert); dlb (optional) is the bf16 copy with zero columns up to ep
  const int width = dlb != nullptr ? ep : n_experts;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)n_tokens * width) return;
  const int t = (int)(i / width), e = (int)(i % width);
  float v = 0.0f;
  if (e < n_experts) {
    float s = 0.0f, g = 0.0f;
    for (int j = 0; j < top_k; ++j) {
      const size_t a = (size_t)t * top_k + j;
      if (pos[a] >= 0) {
        const int ej = topk_idx[a];
        const float d = dtopk_w[a];
        s = fmaf(d, probs[(size_t)t * n_experts + ej], s);
        if (ej == e) g = d;
      }
    }
    const float pe = probs[(size_t)t * n_experts + e];
    v = gate == MOE_GATE_SIGMOID ? g * pe * (1.0f - pe) : pe * (g - s);
    if (noise != nullptr) {  // noisy gate: gradient of the I.W_noise product, dH * noise * sigma(I.W_noise)
      const size_t gi = (size_t)t * n_experts + e;
      v *= noise[gi] / (1.0f + expf(-noise_logits[gi]));
    }
    dl[(size_t)t * n_experts + e] = v;
  }
  if (dlb != nullptr) dlb[i] = f32_to_bf16(v);
}

// bf16 copy of a gradient that is already there, with zero columns up to ep
__global__ __launch_bounds__(256) void pad_dl_kernel(const float* __restrict__ dl, bf16_t* __restrict__ dlb,
                                                     int n_tokens, int n_experts, int ep) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)n_tokens * ep) return;
  const int t = (int)(i / ep), e = (int)(i % ep);
  dlb[i] = f32_to_bf16(e < n_experts ? dl[(size_t)t * n_experts + e] : 0.0f);
}

// bf16 path helpers: W_g with zero columns up to ep, and the row ranges of the two grouped products
__global__ void pad_gate_kernel(const bf16_t* __restrict__ w_gate, bf16_t* __restrict__ wgp, int32_t* __restrict__ tok,
                                int d_model, int n_experts, int ep, int n_tokens, int nsplit) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < d_model * ep) {
    const int m = i / ep, e = i % ep;
    wgp[i] = e < n_experts ? w_gate[(size_t)m * n_experts + e] : (bf16_t)0;
  }
  // tok[0..nsplit] = split-K token ranges; tok[nsplit+1 .. nsplit+2] = {0, N}: the single group of the dx product
  if (i <= nsplit) tok[i] = min(i * kSplitTokens, n_tokens);
  if (i == 0) { tok[nsplit + 1] = 0; tok[nsplit + 2] = n_tokens; }
}

__global__ __launch_bounds__(256) void gate_dw_reduce_bf16_kernel(const bf16_t* __restrict__ part,
                                                                  bf16_t* __restrict__ dw_gate, int nsplit, int d_model,
                                                                  int n_experts, int ep) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < d_model * n_experts) {
    const int m = i / n_experts, e = i % n_experts;
    float s = 0.0f;
    for (int g = 0; g < nsplit; ++g) s += bf16_to_f32(part[((size_t)g * d_model + m) * ep + e]);
    dw_gate[i] = f32_to_bf16(s);
  }
}

// dx[t, m..m+V) += sum_e dl[t,e] * W_g[m.., e]; a thread owns one 16-byte column chunk for kDxTokens tokens
template <typename T>
__global__ __launch_bounds__(256) void gate_dx_kernel(const float* __restrict__ dl, const T* __restrict__ w_gate,
                                                      T* __restrict__ dx, int n_tokens, int d_model, int n_experts) {
  constexpr int V = Elem<T>::kVec;
  extern __shared__ float dls[];  // [kDxTokens][n_experts]
  const int t0 = blockIdx.x * kDxTokens;
  for (int i = threadIdx.x; i < kDxTokens * n_experts; i += 256) {
    int tk = i / n_experts;
    dls[i] = (t0 + tk < n_tokens) ? dl[(size_t)t0 * n_experts + i] : 0.0f;
  }
  __syncthreads();
  const int m = (blockIdx.y * 256 + threadIdx.x) * V;
  if (m >= d_model) return;
  float acc[kDxTokens][V];
#pragma unroll
  for (int tk = 0; tk < kDxTokens; ++tk)
#pragma unroll
    for (int i = 0; i < V; ++i) acc[tk][i] = 0.0f;
  for (int ec = 0; ec < n_experts; ec += kEc) {
    float w[V][kEc];
#pragma unroll
    for (int i = 0; i < V; ++i)
#pragma unroll
      for (int e = 0; e < kEc; ++e)
        w[i][e] = (ec + e < n_experts) ? Elem<T>::ld(w_gate + (size_t)(m + i) * n_experts + ec + e) : 0.0f;
#pragma unroll
    for (int tk = 0; tk < kDxTokens; ++tk)
#pragma unroll
      for (int e = 0; e < kEc; ++e) {
        const float d = (ec + e < n_experts) ? dls[tk * n_experts + ec + e] : 0.0f;
#pragma unroll
        for (int i = 0; i < V; ++i) acc[tk][i] = fmaf(d, w[i][e], acc[tk][i]);
      }
  }
#pragma unroll
  for (int tk = 0; tk < kDxTokens; ++tk) {
    if (t0 + tk < n_tokens) {
      Vec16<T> v;
      T* p = dx + (size_t)(t0 + tk) * d_model + m;
      v.load(p);
#pragma unroll
      for (int i = 0; i < V; ++i) v.v[i] += acc[tk][i];
      v.store(p);
    }
  }
}

// part[tile][m][e] = sum over the tile's tokens of x[t,m] * dl[t,e]; grid (tile, m block, expert chunk)
template <typename T>
__global__ __launch_bounds__(kDwThreads) void gate_dw_partial_kernel(const T* __restrict__ x,
                                                                     const float* __restrict__ dl,
                                                                     float* __restrict__ part, int n_tokens,
                                                                     int d_model, int n_experts) {
  constexpr int V = Elem<T>::kVec;
  constexpr int kSub = 64;
  __shared__ float dls[kSub][kEc];
  const int t0 = blockIdx.x * kDwTokens;
  const int m = (blockIdx.y * kDwThreads + threadIdx.x) * V;
  const int ec = blockIdx.z * kEc;
  float acc[V][kEc];
#pragma unroll
  for (int i = 0; i < V; ++i)
#pragma unroll
    for (int e = 0; e < kEc; ++e) acc[i][e] = 0.0f;
  for (int ts = 0; ts < kDwTokens; ts += kSub) {
    __syncthreads();
    for (int i = threadIdx.x; i < kSub * kEc; i += kDwThreads) {
      int tk = i / kEc, e = i % kEc;
      int t = t0 + ts + tk;
      dls[tk][e] = (t < n_tokens && ec + e < n_experts) ? dl[(size_t)t * n_experts + ec + e] : 0.0f;
    }
    __syncthreads();
    if (m < d_model) {
      for (int tk = 0; tk < kSub; ++tk) {
        int t = t0 + ts + tk;
        if (t >= n_tokens) break;
        Vec16<T> xv;
        xv.load(x + (size_t)t * d_model + m);
#pragma unroll
        for (int e = 0; e < kEc; ++e) {
          const float d = dls[tk][e];
#pragma unroll
          for (int i = 0; i < V; ++i) acc[i][e] = fmaf(xv.v[i], d, acc[i][e]);
        }
      }
    }
  }
  if (m < d_model) {
    float* p = part + ((size_t)blockIdx.x * d_model + m) * n_experts;
#pragma unroll
    for (int i = 0; i < V; ++i)
#pragma unroll
      for (int e = 0; e < kEc; ++e)
        if (ec + e < n_experts) p[(size_t)i * n_experts + ec + e] = acc[i][e];
  }
}

// db_g = column sums of dlogits, in two fixed-order steps (so runs repeat): per tile of kDwTokens tokens,
// 256 / E token lanes per column summed in lane order; then the tiles per column, 256 lanes and a tree.
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* __restrict__ dl, float* __restrict__ bpart,
                                                             int n_tokens, int n_experts) {
  __shared__ float sh[256];
  const int lanes = 256 / n_experts;  // token lanes per column (n_experts <= 256)
  const int e = threadIdx.x % n_experts, sub = threadIdx.x / n_experts;
  const int t0 = blockIdx.x * kDwTokens;
  float s = 0.0f;
  if (sub < lanes)
    for (int tk = sub; tk < kDwTokens && t0 + tk < n_tokens; tk += lanes) s += dl[(size_t)(t0 + tk) * n_experts + e];
  sh[threadIdx.x] = s;
  __syncthreads();
  if (sub == 0) {
    float v = 0.0f;
    for (int l = 0; l < lanes; ++l) v += sh[l * n_experts + e];
    bpart[(size_t)blockIdx.x * n_experts + e] = v;
  }
}

// block e: db_gate[e] = sum over tiles of bpart[tile][e]
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ bpart, float* __restrict__ db_gate,
                                                           int ntile, int n_experts) {
  __shared__ float sh[256];
  const int e = blockIdx.x;
  float s = 0.0f;
  for (int tl = threadIdx.x; tl < ntile; tl += 256) s += bpart[(size_t)tl * n_experts + e];
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) db_gate[e] = sh[0];
}

template <typename T>
__global__ __launch_bounds__(256) void gate_dw_reduce_kernel(const float* __restrict__ part, T* __restrict__ dw_gate,
                                                             int ntile, int d_model, int n_experts) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int n = d_model * n_experts;
  if (i < n) {
    float s = 0.0f;
    for (int tl = 0; tl < ntile; ++tl) s += part[(size_t)tl * n + i];
    Elem<T>::st(dw_gate + i, s);
  }
}

// plain FMA kernels (fp32).  dW_g through per-256-token partial sums reduced in tile order.
template <typename T>
moe_status_t route_bwd_plain(const moe_config_t& c, const void* x, const void* w_gate, const float* probs,
                             const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                             float* db_gate, void* dx, void* ws, const float* noise, const float* noise_logits,
                             const float* dl_ext, int parts, hipStream_t s) {
  constexpr int V = Elem<T>::kVec;
  RouteBwdPlan p = route_bwd_plan(c);
  unsigned char* w = static_cast<unsigned char*>(ws);
  const float* dl = dl_ext;
  float* part = reinterpret_cast<float*>(w + p.off_part);
  float* bpart = reinterpret_cast<float*>(w + p.off_bpart);
  if (dl_ext == nullptr) {
    float* dl_own = reinterpret_cast<float*>(w + p.off_dl);
    if (parts & kPartDl) {
      const size_t ne = (size_t)c.n_tokens * c.n_experts;
      hipLaunchKernelGGL(dlogits_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, s, probs, topk_idx, pos, dtopk_w,
                         dl_own, (bf16_t*)nullptr, c.n_tokens, c.n_experts, c.top_k, 0, c.renormalize, noise, noise_logits);
      MOE_CHECK_LAUNCH();
    }
    dl = dl_own;
  }
  if (parts & kPartDx) {
    hipLaunchKernelGGL(gate_dx_kernel<T>, dim3(ceil_div(c.n_tokens, kDxTokens), ceil_div(c.d_model, 256 * V)), dim3(256),
                       (size_t)kDxTokens * c.n_experts * sizeof(float), s, dl, (const T*)w_gate, (T*)dx, c.n_tokens,
                       c.d_model, c.n_experts);
    MOE_CHECK_LAUNCH();
  }
  if (!(parts & kPartDw)) return MOE_OK;
  hipLaunchKernelGGL(gate_dw_partial_kernel<T>,
                     dim3(p.ntile, ceil_div(c.d_model, kDwThreads * V), ceil_div(c.n_experts, kEc)), dim3(kDwThreads), 0,
                     s, (const T*)x, dl, part, c.n_tokens, c.d_model, c.n_experts);
  MOE_CHECK_LAUNCH();
  if (db_gate != nullptr) {
    hipLaunchKernelGGL(colsum_partial_kernel, dim3(p.ntile), dim3(256), 0, s, dl, bpart, c.n_tokens, c.n_experts);
    MOE_CHECK_LAUNCH();
    hipLaunchKernelGGL(colsum_final_kernel, dim3(c.n_experts), dim3(256), 0, s, bpart, db_gate, p.ntile, c.n_experts);
    MOE_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL(gate_dw_reduce_kernel<T>, dim3(ceil_div(c.d_model * c.n_experts, 256)), dim3(256), 0, s, part,
                     (T*)dw_gate, p.ntile, c.d_model, c.n_experts);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

// bf16: both products go through the MFMA grouped GEMM with dlogits rounded to bf16 (E padded to a
// multiple of 32 with zero columns):
//   dx += dl.W_g^T   one group of N rows, K = ep, accumulate epilogue          (HBM-bound: dx read + written)
//   dW_g = x^T.dl    split-K groups of 512 tokens, bf16 partials summed in group order   (HBM-bound: x read)
moe_status_t route_bwd_bf16(const moe_config_t& c, const void* x, const void* w_gate, const float* probs,
                            const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                            float* db_gate, void* dx, void* ws, const float* noise, const float* noise_logits,
                            const float* dl_ext, int parts, hipStream_t s) {
  RouteBwdPlan p = route_bwd_plan(c);
  unsigned char* w = static_cast<unsigned char*>(ws);
  const float* dl = dl_ext;
  bf16_t* part = reinterpret_cast<bf16_t*>(w + p.off_part);
  float* bpart = reinterpret_cast<float*>(w + p.off_bpart);
  bf16_t* dlb = reinterpret_cast<bf16_t*>(w + p.off_dlb);
  bf16_t* wgp = reinterpret_cast<bf16_t*>(w + p.off_wgp);
  int32_t* tok = reinterpret_cast<int32_t*>(w + p.off_tok);
  const size_t ne = (size_t)c.n_tokens * p.ep;
  if (dl_ext == nullptr) dl = reinterpret_cast<float*>(w + p.off_dl);
  if (parts & kPartDl) {
    if (dl_ext == nullptr) {
      hipLaunchKernelGGL(dlogits_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, s, probs, topk_idx, pos, dtopk_w,
                         reinterpret_cast<float*>(w + p.off_dl), dlb, c.n_tokens, c.n_experts, c.top_k, p.ep, c.renormalize,
                         noise, noise_logits);
    } else {
      hipLaunchKernelGGL(pad_dl_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, s, dl_ext, dlb, c.n_tokens,
                         c.n_experts, p.ep);
    }
    MOE_CHECK_LAUNCH();
    const int npad = c.d_model * p.ep > p.nsplit + 1 ? c.d_model * p.ep : p.nsplit + 1;
    hipLaunchKernelGGL(pad_gate_kernel, dim3(ceil_div(npad, 256)), dim3(256), 0, s, (const bf16_t*)w_gate, wgp, tok,
                       c.d_model, c.n_experts, p.ep, c.n_tokens, p.nsplit);
    MOE_CHECK_LAUNCH();
  }
  if (parts & kPartDx) {  // dx += dlb.wgp^T : [N,ep] x [ep,M], B(k=e, n=m) = wgp[m][e]
    GemmP g = {};
    g.offsets = tok + p.nsplit + 1; g.row_end = g.offsets + 1; g.n_experts = 1; g.n_pairs = 1;
    g.A[0] = dlb; g.sAi = p.ep; g.sAk = 1;
    g.B[0] = wgp; g.sBk = 1; g.sBn = p.ep; g.gB = 0;
    g.C[0] = dx; g.ldc = c.d_model; g.N = c.d_model; g.Kfix = p.ep;
    g.max_rows = c.n_tokens; g.total_rows_bound = c.n_tokens;
    moe_status_t st = launch_gemm_mfma(g, EPI_ACCUM, false, s);
    if (st != MOE_OK) return st;
  }
  if (!(parts & kPartDw)) return MOE_OK;
  {  // part[g] = x_g^T.dlb_g : [M,rows] x [rows,ep] for every 512-token group
    GemmP g = {};
    g.offsets = tok; g.row_end = g.offsets + 1; g.n_experts = p.nsplit; g.n_pairs = 1;
    g.A[0] = x; g.sAi = 1; g.sAk = c.d_model;
    g.B[0] = dlb; g.sBk = p.ep; g.sBn = 1;
    g.C[0] = part; g.ldc = p.ep; g.gC = (long)c.d_model * p.ep;
    g.Mfix = c.d_model; g.N = p.ep;
    g.max_rows = kSplitTokens; g.total_rows_bound = c.n_tokens;
    moe_status_t st = launch_gemm_mfma(g, EPI_PLAIN, true, s);
    if (st != MOE_OK) return st;
  }
  if (db_gate != nullptr) {
    hipLaunchKernelGGL(colsum_partial_kernel, dim3(p.ntile), dim3(256), 0, s, dl, bpart, c.n_tokens, c.n_experts);
    MOE_CHECK_LAUNCH();
    hipLaunchKernelGGL(colsum_final_kernel, dim3(c.n_experts), dim3(256), 0, s, bpart, db_gate, p.ntile, c.n_experts);
    MOE_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL(gate_dw_reduce_bf16_kernel, dim3(ceil_div(c.d_model * c.n_experts, 256)), dim3(256), 0, s, part,
                     (bf16_t*)dw_gate, p.nsplit, c.d_model, c.n_experts, p.ep);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

// the gate's products for dl (own: from probs / dtopk_w; or dl_ext), by dtype and expert count.
// parts: which steps run (all by default); the whole-layer backward runs kPartDl, then the backward of the ordering
// function with the dx product folded in, then kPartDw.
moe_status_t route_bwd_any(const moe_config_t& c, const void* x, const void* w_gate, const float* probs,
                           const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                           float* db_gate, void* dx, void* ws, const float* noise, const float* noise_logits,
                           const float* dl_ext, hipStream_t s, int parts = kPartAll) {
  if (gate_bwd_on_mfma(c))
    return route_bwd_bf16(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, noise, noise_logits, dl_ext,
                          parts, s);
  if (c.dtype == MOE_BF16)
    return route_bwd_plain<bf16_t>(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, noise,
                                   noise_logits, dl_ext, parts, s);
  return route_bwd_plain<float>(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, noise, noise_logits,
                                dl_ext, parts, s);
}

// ----------------------------------------------------------------------------- expert choice (Sec. 2.1)
// G(I) = Softmax(KeepTopK((I.W_g)^T, k)): every expert keeps the k tokens with its largest logits and weighs
// them by the softmax over those logits.  One block per expert walks its column of the logits: a radix select
// (four rounds of 8 bits on an order-preserving integer key) finds the k-th largest value, two prefix counts in
// token order then give every kept token its row (tokens above the threshold, and the earliest of those equal to
// it), and the softmax needs one sum.  Nothing depends on the order in which threads run.
constexpr int kEcThreads = 1024;

// larger float <=> larger key; -0 and +0 get the same key
__device__ __forceinline__ uint32_t ec_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// number of threads before this one (in thread order) whose flag is set, and the block's count; every thread calls it
__device__ __forceinline__ int ec_block_rank(bool flag, int* wave_tot, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long b = __ballot(flag);
  __syncthreads();  // the previous use of wave_tot is over
  if (lane == 0) wave_tot[wave] = __popcll(b);
  __syncthreads();
  int before = 0, tot = 0;
  for (int w = 0; w < kEcThreads / 64; ++w) {
    const int c = wave_tot[w];
    before += w < wave ? c : 0;
    tot += c;
  }
  total = tot;
  return before + __popcll(b & ((1ull << lane) - 1ull));
}

// sum over the block, lanes then waves in order (the same on every run); every thread calls it and gets the sum
__device__ __forceinline__ float ec_block_sum(float v, float* wave_sum) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.0f;
  for (int w = 0; w < kEcThreads / 64; ++w) s += wave_sum[w];
  return s;
}

__global__ __launch_bounds__(kEcThreads) void ec_select_kernel(const float* __restrict__ logits, float* __restrict__ probs,
                                                               int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                               int32_t* __restrict__ pos, int32_t* __restrict__ row_of,
                                                               int32_t* __restrict__ count, int32_t* __restrict__ offsets,
                                                               int32_t* __restrict__ src_of_row, int n_tokens,
                                                               int n_experts, int k_tokens) {
  __shared__ int hist[256];
  __shared__ int s_bucket, s_need;
  __shared__ int wave_tot[kEcThreads / 64];
  __shared__ float wave_sum[kEcThreads / 64];
  __shared__ float wave_max[kEcThreads / 64];
  const int e = blockIdx.x, tid = threadIdx.x;
  const int k = min(k_tokens, n_tokens);

  // the k-th largest key of the column, and how many of the keys equal to it are kept
  uint32_t prefix = 0u, mask = 0u;
  int need = k;
  float mx = -INFINITY;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int t = tid; t < n_tokens; t += kEcThreads) {
      const float l = logits[(size_t)t * n_experts + e];
      mx = fmaxf(mx, l);
      const uint32_t key = ec_key(l);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (tid == 0) {  // from the top bucket down to the one that holds the need-th largest
      int acc = 0, b = 255;
      while (b > 0 && acc + hist[b] < need) { acc += hist[b]; --b; }
      s_bucket = b;
      s_need = need - acc;
    }
    __syncthreads();
    prefix |= (uint32_t)s_bucket << shift;
    mask |= 0xFFu << shift;
    need = s_need;
    __syncthreads();  // hist, s_bucket, s_need are rewritten in the next round
  }
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if ((tid & 63) == 0) wave_max[tid >> 6] = mx;
  __syncthreads();
  for (int w = 0; w < kEcThreads / 64; ++w) mx = fmaxf(mx, wave_max[w]);

  // rows in token order, and the sum of the softmax
  float part = 0.0f;
  int run_eq = 0, run_sel = 0;
  for (int base = 0; base < n_tokens; base += kEcThreads) {
    const int t = base + tid;
    const bool live = t < n_tokens;
    const float l = live ? logits[(size_t)t * n_experts + e] : 0.0f;
    const uint32_t key = ec_key(l);
    const bool eq = live && key == prefix;
    int tot_eq, tot_sel;
    const int eq_rank = run_eq + ec_block_rank(eq, wave_tot, tot_eq);
    const bool sel = live && (key > prefix || (eq && eq_rank < need));
    const int p = run_sel + ec_block_rank(sel, wave_tot, tot_sel);
    run_eq += tot_eq;
    run_sel += tot_sel;
    if (live) {
      const size_t i = (size_t)t * n_experts + e;
      topk_idx[i] = e;
      pos[i] = sel ? p : -1;
      row_of[i] = sel ? e * k + p : -1;
      if (sel) {
        src_of_row[e * k + p] = t * n_experts + e;
        part += expf(l - mx);
      }
    }
  }
  const float sum = ec_block_sum(part, wave_sum);
  for (int t = tid; t < n_tokens; t += kEcThreads) {  // each thread meets the tokens it handled above
    const size_t i = (size_t)t * n_experts + e;
    const float w = pos[i] >= 0 ? expf(logits[i] - mx) / sum : 0.0f;
    topk_w[i] = w;
    probs[i] = w;
  }
  if (tid == 0) {
    count[e] = k;
    offsets[e] = e * k;
    if (e == n_experts - 1) offsets[n_experts] = n_experts * k;
  }
  // rows past the last expert's have no source
  for (int r = n_experts * k + e * kEcThreads + tid; r < n_tokens * n_experts; r += n_experts * kEcThreads) src_of_row[r] = -1;
}

// dl[t,e] = p[t,e] (g[t,e] - c_e) on the kept tokens of expert e, 0 elsewhere; c_e = sum over them of p g
// (the softmax runs down the column).  One block per expert.
__global__ __launch_bounds__(kEcThreads) void ec_dlogits_kernel(const float* __restrict__ probs,
                                                                const int32_t* __restrict__ pos,
                                                                const float* __restrict__ dtopk_w, float* __restrict__ dl,
                                                                int n_tokens, int n_experts) {
  __shared__ float wave_sum[kEcThreads / 64];
  const int e = blockIdx.x;
  float part = 0.0f;
  for (int t = threadIdx.x; t < n_tokens; t += kEcThreads) {
    const size_t i = (size_t)t * n_experts + e;
    if (pos[i] >= 0) part = fmaf(probs[i], dtopk_w[i], part);
  }
  const float c = ec_block_sum(part, wave_sum);
  for (int t = threadIdx.x; t < n_tokens; t += kEcThreads) {
    const size_t i = (size_t)t * n_experts + e;
    dl[i] = pos[i] >= 0 ? probs[i] * (dtopk_w[i] - c) : 0.0f;
  }
}

template <typename T>
moe_status_t route_ec_t(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate, float* logits,
                        float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                        int32_t* offsets, int32_t* src_of_row, void* ws, hipStream_t s) {
  moe_status_t st = route_t<T>(c, x, w_gate, b_gate, logits, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                               nullptr, ws, nullptr, nullptr, kGateLogitsOnly, s);
  if (st != MOE_OK) return st;
  hipLaunchKernelGGL(ec_select_kernel, dim3(c.n_experts), dim3(kEcThreads), 0, s, (const float*)logits, probs, topk_idx,
                     topk_w, pos, row_of, count, offsets, src_of_row, c.n_tokens, c.n_experts, c.capacity);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

// ----------------------------------------------------------------------------- X-MoE gate (Sec. 2.1)
// s_i = cos(W_proj I, W_g[:, i]): the token is projected to D dimensions (the gate kernel with W_proj in the
// place of W_g, logits only), projection and expert embeddings are scaled to unit length, and the scores
// are their dot products, formed in fp64 and rounded once to fp32 like the logits of the plain gate.

// wn[d][e] = W_g[d][e] / |W_g[:, e]| and col_norm[e] = |W_g[:, e]|, fp64; one thread per expert
template <typename T>
__global__ void xmoe_unit_columns_kernel(const T* __restrict__ w_gate, double* __restrict__ wn,
                                         double* __restrict__ col_norm, int d_proj, int n_experts) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_experts) return;
  double ss = 0.0;
  for (int d = 0; d < d_proj; ++d) {
    const double v = (double)Elem<T>::ld(w_gate + (size_t)d * n_experts + e);
    ss = fma(v, v, ss);
  }
  const double nrm = sqrt(ss);
  for (int d = 0; d < d_proj; ++d) wn[(size_t)d * n_experts + e] = (double)Elem<T>::ld(w_gate + (size_t)d * n_experts + e) / nrm;
  col_norm[e] = nrm;
}

// scores[t][e] = fp32(<proj[t,:], wn[:,e]> / |proj[t,:]|); one thread per (token, expert)
__global__ __launch_bounds__(256) void xmoe_scores_kernel(const float* __restrict__ proj, const double* __restrict__ wn,
                                                          float* __restrict__ scores, int n_tokens, int d_proj,
                                                          int n_experts) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)n_tokens * n_experts) return;
  const int t = (int)(i / n_experts), e = (int)(i % n_experts);
  const float* p = proj + (size_t)t * d_proj;
  double ss = 0.0, dot = 0.0;
  for (int d = 0; d < d_proj; ++d) {
    const double v = (double)p[d];
    ss = fma(v, v, ss);
    dot = fma(v, wn[(size_t)d * n_experts + e], dot);
  }
  scores[i] = (float)(dot / sqrt(ss));
}

// Backward through the unit scaling of the projection, one thread per token:
//   g[d] = sum_e ds[t,e] wn[d,e]   (gradient of the unit vector pn = p / |p|)
//   dp   = (g - pn <pn, g>) / |p|
// g is formed twice (once for <pn, g>, once for dp) instead of being kept.  pn is stored for the product
// d(wn) = pn^T . ds.
__global__ __launch_bounds__(256) void xmoe_bwd_token_kernel(const float* __restrict__ proj, const float* __restrict__ ds,
                                                             const double* __restrict__ wn, float* __restrict__ dp,
                                                             float* __restrict__ pn, int n_tokens, int d_proj,
                                                             int n_experts) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= n_tokens) return;
  const float* p = proj + (size_t)t * d_proj;
  const float* g_in = ds + (size_t)t * n_experts;
  double ss = 0.0, pg = 0.0;
  for (int d = 0; d < d_proj; ++d) {
    double g = 0.0;
    for (int e = 0; e < n_experts; ++e) g = fma((double)g_in[e], wn[(size_t)d * n_experts + e], g);
    const double v = (double)p[d];
    ss = fma(v, v, ss);
    pg = fma(v, g, pg);
  }
  const double inv = 1.0 / sqrt(ss);
  const double c = pg * inv;  // <pn, g>
  for (int d = 0; d < d_proj; ++d) {
    double g = 0.0;
    for (int e = 0; e < n_experts; ++e) g = fma((double)g_in[e], wn[(size_t)d * n_experts + e], g);
    const double u = (double)p[d] * inv;
    pn[(size_t)t * d_proj + d] = (float)u;
    dp[(size_t)t * d_proj + d] = (float)((g - u * c) * inv);
  }
}

// Backward through the unit scaling of the expert embeddings, one thread per expert:
//   dW_g[:,e] = (dwn[:,e] - wn[:,e] <wn[:,e], dwn[:,e]>) / |W_g[:,e]|
template <typename T>
__global__ void xmoe_embed_grad_kernel(const float* __restrict__ dwn, const double* __restrict__ wn,
                                       const double* __restrict__ col_norm, T* __restrict__ dw_gate, int d_proj,
                                       int n_experts) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_experts) return;
  double c = 0.0;
  for (int d = 0; d < d_proj; ++d) c = fma(wn[(size_t)d * n_experts + e], (double)dwn[(size_t)d * n_experts + e], c);
  const double inv = 1.0 / col_norm[e];
  for (int d = 0; d < d_proj; ++d) {
    const size_t i = (size_t)d * n_experts + e;
    Elem<T>::st(dw_gate + i, (float)(((double)dwn[i] - wn[i] * c) * inv));
  }
}

// the gate with D "experts": the projection I . W_proj and its backward are the plain gate product at that width
moe_config_t proj_config(const moe_config_t& c, int d_proj) {
  moe_config_t cd = c;
  cd.n_experts = d_proj;
  cd.top_k = 1;
  return cd;
}

struct XmoePlan {
  size_t off_wn, off_norm, off_ds, off_dp, off_pn, off_part, off_dwn, off_route, bytes;
};

XmoePlan xmoe_plan(const moe_config_t& c, int d_proj) {
  XmoePlan p;
  const moe_config_t cd = proj_config(c, d_proj);
  const size_t N = c.n_tokens, E = c.n_experts, D = d_proj;
  size_t o = 0;
  p.off_wn = o; o += align_up(D * E * sizeof(double), 256);
  p.off_norm = o; o += align_up(E * sizeof(double), 256);
  // forward: the workspace of the gate kernel at width D, then at width E; backward: the buffers below
  const size_t fwd = o + (route_plan(cd).bytes > route_plan(c).bytes ? route_plan(cd).bytes : route_plan(c).bytes);
  p.off_ds = o; o += align_up(N * E * sizeof(float), 256);
  p.off_dp = o; o += align_up(N * D * sizeof(float), 256);
  p.off_pn = o; o += align_up(N * D * sizeof(float), 256);
  p.off_part = o; o += align_up((size_t)ceil_div(c.n_tokens, kDwTokens) * D * E * sizeof(float), 256);
  p.off_dwn = o; o += align_up(D * E * sizeof(float), 256);
  p.off_route = o; o += route_bwd_plan(cd).bytes;
  p.bytes = o > fwd ? o : fwd;
  return p;
}

template <typename T>
moe_status_t route_xmoe_t(const moe_config_t& c, const void* x, const void* w_proj, const void* w_gate, int d_proj,
                          float* proj, float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                          int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row, void* ws, hipStream_t s) {
  const XmoePlan p = xmoe_plan(c, d_proj);
  unsigned char* w = static_cast<unsigned char*>(ws);
  double* wn = reinterpret_cast<double*>(w + p.off_wn);
  double* col_norm = reinterpret_cast<double*>(w + p.off_norm);
  void* gate_ws = w + p.off_ds;  // the gate kernel's own workspace (shares the space of the backward buffers)
  const moe_config_t cd = proj_config(c, d_proj);
  moe_status_t st = route_t<T>(cd, x, w_proj, nullptr, proj, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                               nullptr, gate_ws, nullptr, nullptr, kGateLogitsOnly, s);
  if (st != MOE_OK) return st;
  hipLaunchKernelGGL(xmoe_unit_columns_kernel<T>, dim3(ceil_div(c.n_experts, 64)), dim3(64), 0, s, (const T*)w_gate, wn,
                     col_norm, d_proj, c.n_experts);
  MOE_CHECK_LAUNCH();
  const size_t ne = (size_t)c.n_tokens * c.n_experts;
  hipLaunchKernelGGL(xmoe_scores_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, s, proj, wn, logits, c.n_tokens,
                     d_proj, c.n_experts);
  MOE_CHECK_LAUNCH();
  return route_t<T>(c, nullptr, nullptr, nullptr, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets, src_of_row,
                    gate_ws, nullptr, nullptr, kGateFromLogits, s);
}

template <typename T>
moe_status_t route_xmoe_bwd_t(const moe_config_t& c, const void* x, const void* w_proj, const void* w_gate, int d_proj,
                              const float* proj, const float* probs, const int32_t* topk_idx, const int32_t* pos,
                              const float* dtopk_w, void* dw_proj, void* dw_gate, void* dx, void* ws, hipStream_t s) {
  const XmoePlan p = xmoe_plan(c, d_proj);
  unsigned char* w = static_cast<unsigned char*>(ws);
  double* wn = reinterpret_cast<double*>(w + p.off_wn);
  double* col_norm = reinterpret_cast<double*>(w + p.off_norm);
  float* ds = reinterpret_cast<float*>(w + p.off_ds);
  float* dp = reinterpret_cast<float*>(w + p.off_dp);
  float* pn = reinterpret_cast<float*>(w + p.off_pn);
  float* part = reinterpret_cast<float*>(w + p.off_part);
  float* dwn = reinterpret_cast<float*>(w + p.off_dwn);
  const int ntile = ceil_div(c.n_tokens, kDwTokens);
  const size_t ne = (size_t)c.n_tokens * c.n_experts;
  // ds: gradient of the scores (the softmax or sigmoid Jacobian on the kept choices)
  hipLaunchKernelGGL(dlogits_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, s, probs, topk_idx, pos, dtopk_w,
                     ds, (bf16_t*)nullptr, c.n_tokens, c.n_experts, c.top_k, 0, c.renormalize, (const float*)nullptr,
                     (const float*)nullptr);
  MOE_CHECK_LAUNCH();
  hipLaunchKernelGGL(xmoe_unit_columns_kernel<T>, dim3(ceil_div(c.n_experts, 64)), dim3(64), 0, s, (const T*)w_gate, wn,
                     col_norm, d_proj, c.n_experts);
  MOE_CHECK_LAUNCH();
  hipLaunchKernelGGL(xmoe_bwd_token_kernel, dim3(ceil_div(c.n_tokens, 256)), dim3(256), 0, s, proj, ds, wn, dp, pn,
                     c.n_tokens, d_proj, c.n_experts);
  MOE_CHECK_LAUNCH();
  // d(wn) = pn^T . ds through per-tile partial sums in fp32, reduced in tile order
  hipLaunchKernelGGL(gate_dw_partial_kernel<float>, dim3(ntile, ceil_div(d_proj, kDwThreads * 4), ceil_div(c.n_experts, kEc)),
                     dim3(kDwThreads), 0, s, (const float*)pn, (const float*)ds, part, c.n_tokens, d_proj, c.n_experts);
  MOE_CHECK_LAUNCH();
  hipLaunchKernelGGL(gate_dw_reduce_kernel<float>, dim3(ceil_div(d_proj * c.n_experts, 256)), dim3(256), 0, s,
                     (const float*)part, dwn, ntile, d_proj, c.n_experts);
  MOE_CHECK_LAUNCH();
  hipLaunchKernelGGL(xmoe_embed_grad_kernel<T>, dim3(ceil_div(c.n_experts, 64)), dim3(64), 0, s, (const float*)dwn,
                     (const double*)wn, (const double*)col_norm, (T*)dw_gate, d_proj, c.n_experts);
  MOE_CHECK_LAUNCH();
  // p = I . W_proj: dW_proj = x^T . dp and dx += dp . W_proj^T, the gate's products at width D
  const moe_config_t cd = proj_config(c, d_proj);
  return route_bwd_any(cd, x, w_proj, nullptr, nullptr, nullptr, nullptr, dw_proj, nullptr, dx, w + p.off_route, nullptr,
                       nullptr, dp, s);
}

}  // namespace

size_t route_workspace_bytes(const moe_config_t& c) { return route_plan(c).bytes; }

// ----------------------------------------------------------------------------- moe_route_static
// The gate for callers that cannot allocate (code under stream capture, serving loops): the scratch that
// moe_route takes as a workspace (the fp64 copy of W_g of the wide gate kernel, the histogram of choices per
// (expert, rank, 64-token tile), the per-expert totals) lives in a device array of the library instead.  Every
// GPU holds its own copy at its own address, looked up once per device; host code uses that address and never
// the array's name.  Nothing in it has to start at zero: each kernel writes the parts the next one reads.
namespace {
static __device__ __align__(256) unsigned char scratch[MOE_ROUTE_STATIC_SCRATCH_BYTES];

moe_status_t static_scratch_address(void** out) {
  static std::mutex mu;
  static void* per_device[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    set_error("moe_route_static: no current device");
    return MOE_ERR_DEVICE;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (per_device[dev] == nullptr) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr) {
      set_error("moe_route_static: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
      return MOE_ERR_DEVICE;
    }
    per_device[dev] = ptr;
  }
  *out = per_device[dev];
  return MOE_OK;
}
}  // namespace

moe_status_t launch_route_static(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate,
                                 float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                                 int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row, hipStream_t s) {
  const size_t need = route_plan(c).bytes;
  if (need > (size_t)MOE_ROUTE_STATIC_SCRATCH_BYTES) {
    set_error("moe_route_static: this shape needs %zu bytes of scratch, the built-in buffer holds %zu (use moe_route)", need,
              (size_t)MOE_ROUTE_STATIC_SCRATCH_BYTES);
    return MOE_ERR_WORKSPACE;
  }
  void* ws = nullptr;
  const moe_status_t st = static_scratch_address(&ws);
  if (st != MOE_OK) return st;
  return launch_route(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets, src_of_row, ws, s);
}
size_t route_bwd_workspace_bytes(const moe_config_t& c) { return route_bwd_plan(c).bytes; }

moe_status_t launch_route(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate, float* logits,
                          float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                          int32_t* offsets, int32_t* src_of_row, void* ws, hipStream_t s) {
  if (c.renormalize == MOE_GATE_EXPERT_CHOICE)
    return c.dtype == MOE_BF16 ? route_ec_t<bf16_t>(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count,
                                                    offsets, src_of_row, ws, s)
                               : route_ec_t<float>(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count,
                                                   offsets, src_of_row, ws, s);
  return c.dtype == MOE_BF16 ? route_t<bf16_t>(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count,
                                               offsets, src_of_row, ws, nullptr, nullptr, kGateFull, s)
                             : route_t<float>(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count,
                                              offsets, src_of_row, ws, nullptr, nullptr, kGateFull, s);
}

// Noisy gate (Sec. 2.1): the gate kernel runs twice, first on W_noise (only its logits are kept: noise_logits),
// then on W_g with the noise term added before the top-k.
moe_status_t launch_route_noisy(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate,
                                const void* w_noise, const float* noise, float* logits, float* noise_logits, float* probs,
                                int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                                int32_t* offsets, int32_t* src_of_row, void* ws, hipStream_t s) {
  const bool bf = c.dtype == MOE_BF16;
  moe_status_t st = bf ? route_t<bf16_t>(c, x, w_noise, nullptr, noise_logits, probs, topk_idx, topk_w, pos, row_of, count,
                                         offsets, src_of_row, ws, nullptr, nullptr, kGateLogitsOnly, s)
                       : route_t<float>(c, x, w_noise, nullptr, noise_logits, probs, topk_idx, topk_w, pos, row_of, count,
                                        offsets, src_of_row, ws, nullptr, nullptr, kGateLogitsOnly, s);
  if (st != MOE_OK) return st;
  return bf ? route_t<bf16_t>(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets,
                              src_of_row, ws, noise, noise_logits, kGateFull, s)
            : route_t<float>(c, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, pos, row_of, count, offsets,
                             src_of_row, ws, noise, noise_logits, kGateFull, s);
}

moe_status_t launch_route_bwd(const moe_config_t& c, const void* x, const void* w_gate, const float* probs,
                              const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                              float* db_gate, void* dx, void* ws, hipStream_t s) {
  const float* dl_ext = nullptr;
  if (c.renormalize == MOE_GATE_EXPERT_CHOICE) {  // its own Jacobian (down the columns), then the gate's products
    float* dl = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + route_bwd_plan(c).off_dl);
    hipLaunchKernelGGL(ec_dlogits_kernel, dim3(c.n_experts), dim3(kEcThreads), 0, s, probs, pos, dtopk_w, dl, c.n_tokens,
                       c.n_experts);
    MOE_CHECK_LAUNCH();
    dl_ext = dl;
  }
  return route_bwd_any(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, nullptr, nullptr, dl_ext, s);
}

moe_status_t launch_dispatch_route_bwd(const moe_config_t& c, const void* dxe, const int32_t* row_of, const void* dy,
                                       const void* x, const void* w_gate, const float* probs, const int32_t* topk_idx,
                                       const int32_t* pos, const float* dtopk_w, void* dw_gate, float* db_gate, void* dx,
                                       void* ws, hipStream_t s) {
  if (c.renormalize == MOE_GATE_EXPERT_CHOICE || !dispatch_bwd_gate_supported(c)) {
    moe_status_t st = launch_dispatch_bwd(c, dxe, row_of, dy, dx, s);
    if (st != MOE_OK) return st;
    return launch_route_bwd(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, s);
  }
  moe_status_t st = route_bwd_any(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, nullptr, nullptr,
                                  nullptr, s, kPartDl);
  if (st != MOE_OK) return st;
  const float* dl = reinterpret_cast<const float*>(static_cast<unsigned char*>(ws) + route_bwd_plan(c).off_dl);
  st = launch_dispatch_bwd_gate(c, dxe, row_of, dy, dl, w_gate, dx, s);
  if (st != MOE_OK) return st;
  return route_bwd_any(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, nullptr, nullptr, nullptr, s,
                       kPartDw);
}

// Backward of the noisy gate: the ordinary gate backward for W_g (dH = dlogits), then the same products for
// W_noise with dH * noise * sigma(noise_logits) in place of dH; both add their share to dx.
moe_status_t launch_route_noisy_bwd(const moe_config_t& c, const void* x, const void* w_gate, const void* w_noise,
                                    const float* noise, const float* noise_logits, const float* probs,
                                    const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                                    float* db_gate, void* dw_noise, void* dx, void* ws, hipStream_t s) {
  moe_status_t st = launch_route_bwd(c, x, w_gate, probs, topk_idx, pos, dtopk_w, dw_gate, db_gate, dx, ws, s);
  if (st != MOE_OK) return st;
  return route_bwd_any(c, x, w_noise, probs, topk_idx, pos, dtopk_w, dw_noise, nullptr, dx, ws, noise, noise_logits, nullptr, s);
}

size_t route_xmoe_workspace_bytes(const moe_config_t& c, int d_proj) { return xmoe_plan(c, d_proj).bytes; }

moe_status_t launch_route_xmoe(const moe_config_t& c, const void* x, const void* w_proj, const void* w_gate, int d_proj,
                               float* proj, float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                               int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row, void* ws,
                               hipStream_t s) {
  return c.dtype == MOE_BF16 ? route_xmoe_t<bf16_t>(c, x, w_proj, w_gate, d_proj, proj, logits, probs, topk_idx, topk_w, pos,
                                                    row_of, count, offsets, src_of_row, ws, s)
                             : route_xmoe_t<float>(c, x, w_proj, w_gate, d_proj, proj, logits, probs, topk_idx, topk_w, pos,
                                                   row_of, count, offsets, src_of_row, ws, s);
}

moe_status_t launch_route_xmoe_bwd(const moe_config_t& c, const void* x, const void* w_proj, const void* w_gate, int d_proj,
                                   const float* proj, const float* probs, const int32_t* topk_idx, const int32_t* pos,
                                   const float* dtopk_w, void* dw_proj, void* dw_gate, void* dx, void* ws, hipStream_t s) {
  return c.dtype == MOE_BF16 ? route_xmoe_bwd_t<bf16_t>(c, x, w_proj, w_gate, d_proj, proj, probs, topk_idx, pos, dtopk_w,
                                                        dw_proj, dw_gate, dx, ws, s)
                             : route_xmoe_bwd_t<float>(c, x, w_proj, w_gate, d_proj, proj, probs, topk_idx, pos, dtopk_w,
                                                       dw_proj, dw_gate, dx, ws, s);
}

}  // namespace moe
