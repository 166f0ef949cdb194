// The gate of FSMoE Sec. 2.1 (H = I.W_g + b, top-k, G(I)) for bf16 inputs and up to 64 experts, bound by the
// HBM read of the tokens instead of by the fp64 vector ALU.
//
// The routing has to equal, index for index, the routing an independent fp64 evaluation decides on fp32-rounded
// logits.  It does not need fp64 everywhere for that: only for the tokens whose decision is close.
//
//   1. Fast pass.  The product runs on the matrix cores: bf16 x bf16 products are exact in fp32, an MFMA
//      16x16x32 adds 32 of them in fp32, two chained MFMAs give the partial sum of 64 k, and the partial sums are
//      added up in fp64 (exactly, for all purposes).  What is lost is the fp32 rounding inside a chain of 64
//      products.  Taking every addition inside the chain as rounded (64 roundings of at most 2^-24 of the running
//      magnitude) and doubling that for safety:
//          |approx[t,e] - exact[t,e]| <= 2^-17 * sum_k |x[t,k] w[k,e]| <= 2^-17 * |x[t,:]|_2 * |w[:,e]|_2 =: eps[t,e].
//      Both norms come from the matrix cores too (the diagonals of x.x^T and W^T.W), so the token rows are read
//      once and touched by no vector instruction.
//   2. Decision.  Top-k on the approximate fp32 logits.  A gap between neighbours among the k selected values that
//      exceeds 2 eps + 2 ulp stays a gap of the same sign between the exact values and between their fp32 roundings.
//      Only an expert with a logit within 2 eps + 2 ulp of the k-th selected value can belong to the exact top k
//      without having been selected.  So the logits that have to be exact are: both members of every close pair
//      among the selected, and, when some unselected expert is within reach of the k-th value, all those within
//      reach together with the k-th selected one.
//   3. Repair.  Those logits (a handful for a fraction of a percent of the tokens) are recomputed as fp64 dot
//      products with a fixed summation order and rounded once to fp32, as the fp64 gate kernels compute every logit;
//      the token is then decided again.  Every comparison that can change the result is taken on such values.
//
// Consequence for the outputs: routing integers are those of the exact gate; logits that were not repaired (and with
// them probs and topk_w) carry the fast pass's error, at most eps (1e-7 .. 1e-6 of the largest logit in practice;
// the bound above is 1e-4 .. 1e-3).
//
// Work split: one workgroup of 8 waves per 64 tokens (the tile of the position kernels' histogram): 4 token groups of
// 16 (the M of the MFMA) x 2 halves of K (even and odd super-steps of 256 k; the halves are added at the end).  A wave
// reads its 16 rows 512 contiguous bytes at a time into registers (two register sets: the next super-step's loads fly
// under this one's MFMAs), passes them through a private LDS patch, and reads them back as A operands (lane (g, i):
// row i, 8 k at 8 g of every 32).  W_g sits in LDS, in chunks of kc rows when it does not fit whole, laid out so that
// the B operand (8 consecutive k of one expert per lane) comes out of conflict-free ds_read_b64_tr_b16 reads, which
// transpose 4 k x 16 experts per 16 lanes.  After the product: top-k, the decision rule, repair, gate weights and
// the histogram, four lanes per token.
#include <math.h>

#include <atomic>

#include "common.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kTile = 64;       // tokens per workgroup
constexpr int kWaves = 8;       // 4 token groups of 16 x 2 halves of K
constexpr int kThreads = kWaves * 64;
constexpr int kTailThreads = 256;  // top-k, gate weights: four lanes per token
constexpr int kSS = 256;        // k per super-step (one round of loads of a wave)
constexpr int kXPitch = kSS * 2 + 16;  // bytes per row of a wave's LDS patch (16 bytes of padding: rows on different banks)
constexpr int kMaxK = 8;
constexpr float kEpsScale = 7.71e-6f;  // 2^-17 (the bound above), times 1.01 for the fp32 rounding of the two norms

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) {
  union { u32x4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// W_g in LDS: one array per tile of 16 experts, [kc rows][16 experts] (32-byte rows).  Inside every block of 32 k the
// rows are stored in the order the four k-groups of an MFMA operand read them: k = 32 b + 8 g + r sits at row
// 32 b + 4 r + g.  A ds_read_b64_tr_b16 of the 64 lanes (lane (g, i): row 4 (i / 4) + g, 8-byte piece i % 4) then covers
// 512 consecutive bytes, every bank twice: no conflicts.  (Rows in k order put the four groups 256 bytes apart, on the
// same banks.)
__device__ __forceinline__ int w_row(int k) { return (k & ~31) | ((k & 7) << 2) | ((k >> 3) & 3); }

// The MFMA operand of lane (g, i) for the 32 k starting at k32 (a multiple of 32, relative to the chunk) and tile t:
// expert i, k = k32 + 8 g .. + 7, four k per read.
__device__ __forceinline__ bf16x8 read_w(const unsigned char* wl, int tile_bytes, int k32, int t, int g, int i) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const unsigned char* p = wl + (size_t)t * tile_bytes + (size_t)(k32 + 4 * (i >> 2) + g) * 32 + (i & 3) * 8;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p);          // k = 8 g + i / 4
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 512));  // k + 4: sixteen rows further
  union { s16x4 h[2]; bf16x8 v; } u;
  u.h[0] = lo; u.h[1] = hi;
  return u.v;
}

__device__ __forceinline__ float pick4(const f32x4& v, int r) { return r == 0 ? v[0] : r == 1 ? v[1] : r == 2 ? v[2] : v[3]; }

template <int NT>  // 16-expert tiles: E <= 16 NT
__global__ __launch_bounds__(kThreads) void gate_mfma_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ w_gate, const float* __restrict__ b_gate,
    float* __restrict__ logits, float* __restrict__ probs, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    int32_t* __restrict__ hist, int n_tokens, int d_model, int n_experts, int top_k, int gate, int nb, int kc, int mpad) {
  constexpr int EP = NT * 16;       // experts in LDS (E rounded up to whole tiles)
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* wl = smem;                                                        // [NT][kc][16] bf16
  unsigned char* xs_all = smem + (size_t)kc * EP * 2;                              // [kWaves][16 rows][kXPitch]
  double* red = reinterpret_cast<double*>(xs_all + kWaves * 16 * kXPitch);         // [kWaves][4]
  float* lg = reinterpret_cast<float*>(red + kWaves * 4);                          // [kTile][E + 1]
  int32_t* hcnt = reinterpret_cast<int32_t*>(lg + kTile * (n_experts + 1));        // [top_k][E]
  float* nx = reinterpret_cast<float*>(hcnt + top_k * n_experts);                  // [kTile]  |x_t|^2
  float* nw = nx + kTile;                                                          // [EP]     |w_e|^2
  int32_t* amb = reinterpret_cast<int32_t*>(nw + EP);                              // [kTile][2]  bit e: logit e must be exact

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, i = lane & 15;  // k-group and row (or expert) of this lane inside an MFMA operand
  const int tg = wave & 3, half = wave >> 2;  // token group of 16; which super-steps of K (even or odd)
  const int t0 = blockIdx.x * kTile;
  const int lgs = n_experts + 1;
  const int E = n_experts, M = d_model;

  for (int q = tid; q < top_k * E; q += kThreads) hcnt[q] = 0;
  const int tile_bytes = kc * 32;  // one tile's [kc][16] array
  if (EP > E)  // the columns past E stay zero for every chunk
    for (int q = tid; q < kc * (EP - E); q += kThreads) {
      const int kr = q / (EP - E), e = E + q % (EP - E);
      *reinterpret_cast<bf16_t*>(wl + (size_t)(e >> 4) * tile_bytes + kr * 32 + (e & 15) * 2) = 0;
    }

  // W_g rows [k0, k0 + kc) -> LDS (layout: see read_w); rows past M are zero
  const bool vec_ok = (E % 8 == 0) && ((reinterpret_cast<uintptr_t>(w_gate) & 15) == 0);
  // (eight loads in flight per thread before the first LDS store: a load per iteration would pay the memory latency
  // kc * E / 4096 times in a row)
  auto stage = [&](int k0) {
    if (vec_ok) {
      const int per = E / 8;  // 16-byte parts of a row: part p holds experts 8 p .. 8 p + 7 = half p % 2 of tile p / 2
      const int total = kc * per;
      for (int v0 = tid; v0 < total; v0 += 8 * kThreads) {
        uint4 val[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int v = v0 + u * kThreads;
          const int kr = v / per, part = v % per;
          val[u] = make_uint4(0, 0, 0, 0);
          if (v < total && k0 + kr < M) val[u] = *reinterpret_cast<const uint4*>(w_gate + (size_t)(k0 + kr) * E + part * 8);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int v = v0 + u * kThreads;
          const int kr = v / per, part = v % per;
          if (v < total) *reinterpret_cast<uint4*>(wl + (size_t)(part >> 1) * tile_bytes + w_row(kr) * 32 + (part & 1) * 16) = val[u];
        }
      }
    } else {
      const int total = kc * E;
      for (int q0 = tid; q0 < total; q0 += 8 * kThreads) {
        bf16_t val[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int q = q0 + u * kThreads;
          const int kr = q / E, e = q % E;
          val[u] = (q < total && k0 + kr < M) ? w_gate[(size_t)(k0 + kr) * E + e] : (bf16_t)0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int q = q0 + u * kThreads;
          const int kr = q / E, e = q % E;
          if (q < total) *reinterpret_cast<bf16_t*>(wl + (size_t)(e >> 4) * tile_bytes + w_row(kr) * 32 + (e & 15) * 2) = val[u];
        }
      }
    }
  };

  // ---- the token rows of this wave.  A super-step is kSS = 256 k of the wave's 16 rows: eight wave-level loads, each
  //      two rows x 512 contiguous bytes (lane l: row 2 q + l / 32, bytes 16 (l % 32) ..), into registers; from there
  //      into the wave's own LDS patch [16 rows][512 + 16 bytes]; from there as A operands (lane (g, i): row i,
  //      8 k at 8 g of every 32).  Two register sets: the loads of the next super-step fly under the MFMAs of this one.
  unsigned char* xs = xs_all + (size_t)wave * 16 * kXPitch;
  const int row_a = lane >> 5;  // row inside the pair of a load
  auto load_ss = [&](int ss, u32x4(&r)[8]) {
    const int ko = ss * kSS + (lane & 31) * 8;  // first element of this lane's 16 bytes
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int tr = t0 + tg * 16 + 2 * q + row_a;
      r[q] = (tr < n_tokens && ko < M) ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + (size_t)tr * M + ko)) : zero;
    }
  };
  auto put_ss = [&](const u32x4(&r)[8]) {
#pragma unroll
    for (int q = 0; q < 8; ++q)
      *reinterpret_cast<u32x4*>(xs + (2 * q + row_a) * kXPitch + (lane & 31) * 16) = r[q];
  };

  double acc[NT][4];
  f32x4 gw[NT];
  f32x4 gx = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    gw[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[t][r] = 0.0;
  }

  int chunk_k0 = -kc;  // first k of the chunk in LDS
  // the MFMAs of super-step ss (this wave's rows are in xs); W_g chunk switched first when ss starts a new one: the two
  // halves of the workgroup reach a switch in the same iteration (kc is a multiple of 2 kSS), so the barriers match
  auto compute_ss = [&](int ss) {
    if (ss * kSS >= chunk_k0 + kc) {  // the same for all threads
      __syncthreads();               // every wave is done with the chunk before
      chunk_k0 += kc;
      stage(chunk_k0);
      __syncthreads();
    }
#pragma unroll
    for (int st = 0; st < kSS / 64; ++st) {
      const bf16x8 xa = as_bf16x8(*reinterpret_cast<const u32x4*>(xs + i * kXPitch + st * 128 + g * 16));
      const bf16x8 xb = as_bf16x8(*reinterpret_cast<const u32x4*>(xs + i * kXPitch + st * 128 + 64 + g * 16));
      const int kl = ss * kSS + st * 64 - chunk_k0;  // first k of the step inside the chunk
      gx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, xa, gx, 0, 0, 0);
      gx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xb, xb, gx, 0, 0, 0);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const bf16x8 b1 = read_w(wl, tile_bytes, kl, t, g, i);
        const bf16x8 b2 = read_w(wl, tile_bytes, kl + 32, t, g, i);
        f32x4 c = {0.f, 0.f, 0.f, 0.f};
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, b1, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xb, b2, c, 0, 0, 0);
        if ((t & 3) == tg) {  // |w_e|^2 does not depend on the tokens: token group t % 4 computes it for tile t
          gw[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b1, b1, gw[t], 0, 0, 0);
          gw[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b2, b2, gw[t], 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] += (double)c[r];
      }
    }
  };

  const int nss = mpad / kSS;  // a multiple of 4: each half of the workgroup takes an even number of super-steps
  u32x4 ra[8], rb[8];
  load_ss(half, ra);
  for (int ss = half; ss < nss; ss += 4) {
    load_ss(ss + 2, rb);  // ss + 2 < nss
    put_ss(ra);
    compute_ss(ss);
    if (ss + 4 < nss) load_ss(ss + 4, ra);
    put_ss(rb);
    compute_ss(ss + 2);
  }
  __syncthreads();  // every wave is done with its LDS patch and with W_g

  // ---- the two halves of K are added (second half into the first, through the patches' LDS), then logits -> lg.
  //      A lane holds rows 4 g + r, column i of every 16x16 result.
  double* xch = reinterpret_cast<double*>(xs_all) + (size_t)tg * (NT * 4 + 2 + NT * 2) * 64;  // per token group, per lane
  if (half == 1) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) xch[(t * 4 + r) * 64 + lane] = acc[t][r];
      reinterpret_cast<f32x4*>(xch + (NT * 4 + 2) * 64)[t * 64 + lane] = gw[t];
    }
    reinterpret_cast<f32x4*>(xch + NT * 4 * 64)[lane] = gx;
  }
  __syncthreads();
  if (half == 0) {
    const f32x4 gx1 = reinterpret_cast<const f32x4*>(xch + NT * 4 * 64)[lane];
#pragma unroll
    for (int r = 0; r < 4; ++r) gx[r] += gx1[r];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const f32x4 gw1 = reinterpret_cast<const f32x4*>(xch + (NT * 4 + 2) * 64)[t * 64 + lane];
      const int e = 16 * t + i;
      if (e < E) {
        const double b = b_gate != nullptr ? (double)b_gate[e] : 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          lg[(tg * 16 + 4 * g + r) * lgs + e] = (float)((acc[t][r] + xch[(t * 4 + r) * 64 + lane]) + b);
      }
      if ((t & 3) == tg && (i >> 2) == g) nw[16 * t + i] = pick4(gw[t], i & 3) + pick4(gw1, i & 3);  // diagonal of W^T.W
    }
    if ((i >> 2) == g) nx[tg * 16 + i] = pick4(gx, i & 3);  // diagonal of x.x^T
  }
  __syncthreads();

  // ---- top-k with four lanes per token
  const bool tail_thread = tid < kTailThreads;  // waves 0 .. 3; the others only keep the barriers company
  const int tk = (tid & (kTailThreads - 1)) >> 2, sub = tid & 3;
  const int t = t0 + tk;
  const bool live = tail_thread && t < n_tokens;
  float* l = lg + tk * lgs;
  int sel[kMaxK];
  float selv[kMaxK];
  auto select = [&]() {
    float prev_v = 0.0f;
    int prev_e = -1;
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
      if (j >= top_k) break;
      float bv = 0.0f;
      int be = -1;
      for (int e = sub; e < E; e += 4) {
        const float v = l[e];
        const bool eligible = (j == 0) || (v < prev_v) || (v == prev_v && e > prev_e);
        if (eligible && (be < 0 || v > bv)) { bv = v; be = e; }
      }
#pragma unroll
      for (int m = 1; m <= 2; m <<= 1) {  // best of the four lanes: larger value, lower expert among equal values
        const float ov = __shfl_xor(bv, m, 64);
        const int oe = __shfl_xor(be, m, 64);
        if (oe >= 0 && (be < 0 || ov > bv || (ov == bv && oe < be))) { bv = ov; be = oe; }
      }
      if (be < 0) {  // only with NaN logits (every comparison false): lowest expert not yet taken, so indices stay valid
        for (int e = 0; e < E && be < 0; ++e) {
          bool taken = false;
#pragma unroll
          for (int q = 0; q < kMaxK; ++q) taken |= (q < j) && sel[q] == e;
          if (!taken) { be = e; bv = l[e]; }
        }
      }
      sel[j] = be;
      selv[j] = bv;
      prev_v = bv;
      prev_e = be;
    }
  };
  if (tail_thread) select();

  // ---- which logits have to be exact for the decision to be certain?  (a) both members of a pair of neighbours among
  //      the k selected whose gap is inside the error bound; (b) when any expert other than the k-th selected one is
  //      within reach of the k-th value (l >= v_k - 2 eps - 2 ulp: only those can belong to the exact top k besides the
  //      ones selected with a clear gap), all the experts within reach.  Everything else keeps its fast-pass value:
  //      a clear gap stays a clear gap when one side is replaced by its exact value.
  if (tail_thread) {
    float wmax = 0.0f;
    for (int e = 0; e < E; ++e) wmax = fmaxf(wmax, nw[e]);
    const float eps = kEpsScale * sqrtf(nx[tk] * wmax);
    uint32_t m_lo = 0u, m_hi = 0u;
    auto mark = [&](int e) {
      if (e < 32) m_lo |= 1u << e; else m_hi |= 1u << (e - 32);
    };
    float vk = 0.0f;
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
      if (j >= top_k) break;
      if (j + 1 == top_k) vk = selv[j];
      if (j + 1 < kMaxK && j + 1 < top_k) {
        const float a = selv[j], b = selv[j + 1];
        const float thr = 2.0f * eps + 2.4e-7f * (fabsf(a) + fabsf(b));
        if (!(a - b > thr)) { mark(sel[j]); mark(sel[j + 1]); }  // NaN anywhere: not certain
      }
    }
    const float zone = vk - (2.0f * eps + 4.8e-7f * fabsf(vk));
    uint32_t s_lo = 0u, s_hi = 0u;  // the k selected experts
    int last = 0;                   // the k-th selected expert
#pragma unroll
    for (int j = 0; j < kMaxK; ++j)
      if (j < top_k) {
        if (sel[j] < 32) s_lo |= 1u << sel[j]; else s_hi |= 1u << (sel[j] - 32);
        last = sel[j];
      }
    uint32_t z_lo = 0u, z_hi = 0u;  // experts that were not selected but are within reach of the k-th value
    for (int e = sub; e < E; e += 4)
      if (!(l[e] < zone)) {
        if (e < 32) z_lo |= 1u << e; else z_hi |= 1u << (e - 32);
      }
#pragma unroll
    for (int m = 1; m <= 2; m <<= 1) {
      z_lo |= __shfl_xor(z_lo, m, 64);
      z_hi |= __shfl_xor(z_hi, m, 64);
    }
    z_lo &= ~s_lo;
    z_hi &= ~s_hi;
    if ((z_lo | z_hi) != 0u) { m_lo |= z_lo; m_hi |= z_hi; mark(last); }
    if (sub == 0) {
      amb[2 * tk] = live ? (int32_t)m_lo : 0;
      amb[2 * tk + 1] = live ? (int32_t)m_hi : 0;
    }
  }
  __syncthreads();

  // ---- repair: the logits marked above as fp64 dot products, one token at a time by the whole workgroup (threads
  //      stride over k in 16-byte pieces, up to four experts per pass over the row; butterfly inside a wave, the
  //      waves added in wave order; bias added in fp64; one rounding to fp32).
  for (int tk2 = 0; tk2 < kTile; ++tk2) {
    uint32_t r_lo = (uint32_t)amb[2 * tk2], r_hi = (uint32_t)amb[2 * tk2 + 1];  // the same for every thread
    if ((r_lo | r_hi) == 0u) continue;
    const bf16_t* xr = x + (size_t)(t0 + tk2) * M;
    while ((r_lo | r_hi) != 0u) {
      int ec[4], n = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        ec[c] = 0;
        if (r_lo != 0u) { ec[c] = __ffs(r_lo) - 1; r_lo &= r_lo - 1u; n = c + 1; }
        else if (r_hi != 0u) { ec[c] = 32 + __ffs(r_hi) - 1; r_hi &= r_hi - 1u; n = c + 1; }
      }
      double a4[4] = {0.0, 0.0, 0.0, 0.0};
      for (int k = tid * 8; k < M; k += kThreads * 8) {
        const uint4 xv = *reinterpret_cast<const uint4*>(xr + k);
        const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const double xk = (double)__uint_as_float((j & 1) ? (xw[j >> 1] & 0xFFFF0000u) : (xw[j >> 1] << 16));
          const bf16_t* wr = w_gate + (size_t)(k + j) * E;
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (c < n) a4[c] = fma(xk, (double)bf16_to_f32(wr[ec[c]]), a4[c]);
        }
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        double v = a4[c];
#pragma unroll
        for (int b = 32; b >= 1; b >>= 1) v += __shfl_xor(v, b, 64);
        if (lane == 0) red[wave * 4 + c] = v;
      }
      __syncthreads();
      if (tid < n) {
        const int e_out = tid == 0 ? ec[0] : tid == 1 ? ec[1] : tid == 2 ? ec[2] : ec[3];
        double v = red[tid];
#pragma unroll
        for (int wv = 1; wv < kWaves; ++wv) v += red[wv * 4 + tid];  // in wave order
        if (b_gate != nullptr) v += (double)b_gate[e_out];
        lg[tk2 * lgs + e_out] = (float)v;
      }
      __syncthreads();
    }
  }
  __syncthreads();
  if (tail_thread && (amb[2 * tk] | amb[2 * tk + 1]) != 0) select();  // the four lanes of a token agree

  // ---- outputs: logits, then G(I) in place of the logits in LDS, then probs and the histogram
  for (int q = tid; q < kTile * E; q += kThreads) {
    const int r = q / E, e = q % E;
    if (t0 + r < n_tokens) logits[(size_t)(t0 + r) * E + e] = lg[r * lgs + e];
  }
  __syncthreads();
  if (live) {
    const float mx = selv[0];
    float wj[kMaxK];
    if (gate == MOE_GATE_SIGMOID) {
      for (int e = sub; e < E; e += 4) l[e] = 1.0f / (1.0f + expf(-l[e]));
    } else if (gate == MOE_GATE_SOFTMAX_TOPK) {
      float s = 0.0f;
#pragma unroll
      for (int j = 0; j < kMaxK; ++j)
        if (j < top_k) { wj[j] = expf(selv[j] - mx); s += wj[j]; }
#pragma unroll
      for (int j = 0; j < kMaxK; ++j)
        if (j < top_k) wj[j] = wj[j] / s;
      for (int e = sub; e < E; e += 4) l[e] = 0.0f;
    } else {
      float s = 0.0f;
      for (int e = sub; e < E; e += 4) {
        const float z = expf(l[e] - mx);
        l[e] = z;
        s += z;
      }
      s += __shfl_xor(s, 1, 64);
      s += __shfl_xor(s, 2, 64);
      for (int e = sub; e < E; e += 4) l[e] = l[e] / s;
    }
    if (sub == 0) {  // LDS operations of one wave complete in order: the row is written by now
#pragma unroll
      for (int j = 0; j < kMaxK; ++j) {
        if (j >= top_k) break;
        float w;
        if (gate == MOE_GATE_SOFTMAX_TOPK) { w = wj[j]; l[sel[j]] = w; }
        else w = l[sel[j]];
        topk_w[(size_t)t * top_k + j] = w;
        topk_idx[(size_t)t * top_k + j] = sel[j];
        atomicAdd(&hcnt[j * E + sel[j]], 1);
      }
    }
  }
  __syncthreads();
  for (int q = tid; q < kTile * E; q += kThreads) {
    const int r = q / E, e = q % E;
    if (t0 + r < n_tokens) probs[(size_t)(t0 + r) * E + e] = lg[r * lgs + e];
  }
  for (int q = tid; q < top_k * E; q += kThreads) {
    const int j = q / E, e = q % E;
    hist[((size_t)e * top_k + j) * nb + blockIdx.x] = hcnt[q];
  }
}

struct Plan {
  int nt, kc, mpad;
  size_t lds;
};

// mpad: K rounded up to whole rounds of the main loop (two super-steps for each half of the workgroup).  kc: rows of W_g
// per LDS chunk: the whole matrix when it fits beside the waves' patches, else the largest multiple of 2 kSS that does (the
// two halves of the workgroup then switch chunks in the same iteration).
bool make_plan(const moe_config_t& c, Plan* p) {
  if (c.dtype != MOE_BF16 || c.n_experts > 64 || c.top_k > kMaxK) return false;
  p->nt = c.n_experts <= 16 ? 1 : c.n_experts <= 32 ? 2 : 4;
  const int ep = p->nt * 16;
  p->mpad = ceil_div(c.d_model, 4 * kSS) * 4 * kSS;
  const size_t rest = (size_t)kWaves * 16 * kXPitch + kWaves * 4 * sizeof(double) + (size_t)kTile * (c.n_experts + 1) * 4 +
                      (size_t)c.top_k * c.n_experts * 4 + kTile * 4 + ep * 4 + 2 * kTile * 4;
  const size_t budget = (size_t)160 * 1024 - rest - 256;
  if ((size_t)p->mpad * ep * 2 <= budget) {
    p->kc = p->mpad;
  } else {
    p->kc = (int)(budget / (ep * 2) / (2 * kSS)) * 2 * kSS;
    if (p->kc < 2 * kSS) return false;
  }
  p->lds = (size_t)p->kc * ep * 2 + rest;
  return p->lds <= (size_t)160 * 1024;
}

template <int NT>
moe_status_t launch_nt(const moe_config_t& c, const Plan& p, const void* x, const void* w_gate, const float* b_gate,
                       float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* hist, int nb, hipStream_t s) {
  static std::atomic<uint64_t> done{0};  // LDS above 64 KB: one attribute call per device (see route.hip)
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    set_error("gate: no current device");
    return MOE_ERR_DEVICE;
  }
  if (!(done.load(std::memory_order_acquire) & (1ull << dev))) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gate_mfma_kernel<NT>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) {
      set_error("gate: hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: %s", hipGetErrorString(e));
      return MOE_ERR_DEVICE;
    }
    done.fetch_or(1ull << dev, std::memory_order_release);
  }
  hipLaunchKernelGGL(gate_mfma_kernel<NT>, dim3(nb), dim3(kThreads), p.lds, s, (const bf16_t*)x, (const bf16_t*)w_gate,
                     b_gate, logits, probs, topk_idx, topk_w, hist, c.n_tokens, c.d_model, c.n_experts, c.top_k,
                     c.renormalize, nb, p.kc, p.mpad);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

}  // namespace

bool gate_mfma_supported(const moe_config_t& c) {
  Plan p;
  return make_plan(c, &p);
}

moe_status_t launch_gate_mfma(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate,
                              float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* hist, int nb,
                              hipStream_t s) {
  Plan p;
  if (!make_plan(c, &p)) {
    set_error("gate: shape not supported by the matrix-core gate kernel");
    return MOE_ERR_UNSUPPORTED;
  }
  switch (p.nt) {
    case 1: return launch_nt<1>(c, p, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, hist, nb, s);
    case 2: return launch_nt<2>(c, p, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, hist, nb, s);
    default: return launch_nt<4>(c, p, x, w_gate, b_gate, logits, probs, topk_idx, topk_w, hist, nb, s);
  }
}

}  // namespace moe
