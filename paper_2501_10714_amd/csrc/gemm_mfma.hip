// bf16 grouped GEMM on the CDNA4 matrix cores for the expert FFNs (FSMoE Sec. 2.1 "Experts",
// Sec. 4.4 for the backward products): the one dense contraction of the layer.
//
// One workgroup (256 lanes = 4 waves, one per SIMD) owns a 256x256 output tile and walks K in
// steps of 64 through a two-stage LDS pipeline.  Each wave owns a 128x128 quadrant = 4x4 MFMA
// 32x32x16 tiles, fp32 accumulators (256 registers per lane).
//
// Operand layouts in LDS (bf16):
//   KC  "K-contiguous rows"  [256 rows][64 k]   128-byte rows, 16-byte chunks XOR-swizzled by row.
//        A lane reads its 8 consecutive k of one row with one ds_read_b128.
//   TR  "transposed feed"    [64 k][256 cols]   512-byte rows, 32-byte segments XOR-swizzled by k.
//        The operand is N-contiguous in memory but the MFMA wants 8 consecutive k per lane:
//        ds_read_b64_tr_b16 hands a 16-lane group the 4(k) x 16(col) block transposed.
//   The three products need: forward  A=KC (activations), B=TR (W[k][n]);
//                            dgrad    A=KC, B=KC (W^T: W rows are the output columns);
//                            wgrad    A=TR, B=TR (both operands are indexed by the ragged expert row).
//
// MFMA is issued with the operands swapped (B fragment first), so a lane ends up with 4 consecutive
// output COLUMNS of one output row per accumulator quad: 8-byte bf16 stores and 8-byte loads of the
// saved activations in the fused epilogues.
//
// Tile order: hardware deals workgroup ids round-robin to the 8 XCDs (each with its own L2), so
// id -> (xcd, slot) is remapped to give every XCD a contiguous range of logical tiles; inside that
// range tiles are ordered in bands of 8 row-tiles x all column-tiles so the 32 CUs of an XCD share
// A and B panels in L2.  Rows are ragged per expert: the tile list is derived from offsets[] on
// the device by every workgroup (E <= 256 scalar steps), no host synchronisation.
#include <type_traits>

#include "common.h"
#include "gemm_params.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // native vector: stays in registers (HIP's uint4 struct copies as memcpy)
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int kOperandBytes = BM * BK * 2;      // 32 KB
constexpr int kStageBytes = 2 * kOperandBytes;  // A | B
constexpr int kLdsBytes = 2 * kStageBytes;      // two stages: 128 KB
constexpr int kBand = 8;                        // row-tiles per L2 band
constexpr int kSlots = 8;                       // 16-byte chunks per thread per operand per stage

enum Layout { KC = 0, TR = 1 };

__device__ __forceinline__ int kc_chunk_off(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }
__device__ __forceinline__ int tr_chunk_off(int krow, int c) {  // c: 16-byte chunk (8 cols) of the 512-byte k-row
  return krow * 512 + ((((c >> 1) ^ (krow & 15))) << 5) + ((c & 1) << 4);
}

// ---- fragment reads: 32 (rows or cols) x 16 k, as the MFMA 32x32x16 operand registers
__device__ __forceinline__ bf16x8 read_kc(const unsigned char* op, int row0, int s, int lane) {
  const int row = row0 + (lane & 31);
  const int c = 2 * s + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(op + kc_chunk_off(row, c));
}

__device__ __forceinline__ bf16x8 read_tr(const unsigned char* op, int col0, int s, int lane) {
  const int grp = lane >> 4, i = lane & 15;
  const int seg = (col0 >> 4) + (grp & 1);          // 16-column segment of the tile
  const int k = 16 * s + 8 * (grp >> 1) + (i >> 2);  // k-row this lane addresses for the first read
  const int a0 = k * 512 + ((seg ^ (k & 15)) << 5) + ((i & 3) << 3);
  const int k1 = k + 4;
  const int a1 = k1 * 512 + ((seg ^ (k1 & 15)) << 5) + ((i & 3) << 3);
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(op + a0));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(op + a1));
  union { s16x4 h[2]; bf16x8 v; } u;
  u.h[0] = lo; u.h[1] = hi;
  return u.v;
}

template <int LAYOUT>
__device__ __forceinline__ bf16x8 read_frag(const unsigned char* op, int base, int s, int lane) {
  return LAYOUT == KC ? read_kc(op, base, s, lane) : read_tr(op, base, s, lane);
}

__device__ __forceinline__ uint32_t pack2(float a, float b) {
  union { __bf16 h[2]; uint32_t u; } v;
  v.h[0] = (__bf16)a; v.h[1] = (__bf16)b;
  return v.u;
}
__device__ __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
  *reinterpret_cast<u32x2*>(p) = u32x2{pack2(a, b), pack2(c, d)};
}
__device__ __forceinline__ void load4(const bf16_t* p, float* v) {
  u32x2 r = *reinterpret_cast<const u32x2*>(p);
  v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xFFFF0000u);
  v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xFFFF0000u);
}

struct TileId {
  int e, set, mt, nt, r0, rows;
  bool valid;
};

// Logical tile index -> (expert, row tile, column tile).  Ragged M: row tiles per expert come from
// offsets[]; ragged K: every group has the same mt_fix row tiles.
template <bool RAGGED_K>
__device__ __forceinline__ TileId find_tile(const GemmP& p, int n_nt, int mt_fix) {
  TileId t;
  t.valid = false;
  const int groups = (RAGGED_K && p.n_pairs == 2) ? 2 * p.n_experts : p.n_experts;
  int total = 0;
  if (RAGGED_K) {
    total = groups * mt_fix * n_nt;
  } else {
    for (int e = 0; e < p.n_experts; ++e) total += ((p.offsets[e + 1] - p.offsets[e] + BM - 1) / BM) * n_nt;
  }
  // XCD-aware remap: workgroup id b runs on XCD b % 8; give XCD x the logical range [x*per, (x+1)*per)
  const int per = (total + 7) >> 3;
  const int slot = blockIdx.x >> 3;
  if (slot >= per) return t;
  int L = (blockIdx.x & 7) * per + slot;
  if (L >= total) return t;
  int g = 0, mt_g = mt_fix;
  if (RAGGED_K) {
    g = L / (mt_fix * n_nt);
    L -= g * mt_fix * n_nt;
  } else {
    for (;; ++g) {
      mt_g = (p.offsets[g + 1] - p.offsets[g] + BM - 1) / BM;
      const int cnt = mt_g * n_nt;
      if (L < cnt) break;
      L -= cnt;
    }
  }
  const int band = L / (kBand * n_nt);
  const int rem = L - band * kBand * n_nt;
  const int bsz = min(kBand, mt_g - band * kBand);
  t.nt = rem / bsz;
  t.mt = band * kBand + rem % bsz;
  t.e = g % p.n_experts;
  t.set = g / p.n_experts;
  t.r0 = p.offsets[t.e];
  t.rows = p.offsets[t.e + 1] - t.r0;
  t.valid = true;
  return t;
}

template <int LA, int LB, int EPI, bool RAGGED_K, int ACT>
__global__ __launch_bounds__(kThreads, 1) void gg_mfma_kernel(GemmP p, int n_nt, int mt_fix) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr bool kGluFwd = EPI == EPI_GLU_FWD;
  constexpr int kOutCols = kGluFwd ? BN / 2 : BN;  // output columns per tile

  const TileId t = find_tile<RAGGED_K>(p, n_nt, mt_fix);
  if (!t.valid) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const int Kg = RAGGED_K ? t.rows : p.Kfix;
  const int sum_pairs = (!RAGGED_K && !kGluFwd) ? p.n_pairs : 1;
  const int nk1 = (Kg + BK - 1) / BK;
  const int nk = nk1 * sum_pairs;

  // ---- per-thread global chunk bookkeeping (element offsets from the operand base, k0 = 0)
  const long lda = RAGGED_K ? p.sAk : p.sAi;  // row stride of the A array in memory
  const long ldb = RAGGED_K ? p.sBk : (LB == TR ? p.sBk : p.sBn);
  long aoff[kSlots], boff[kSlots];
  int alds[kSlots], blds[kSlots];
  int bsrc[kSlots];  // which B matrix (GLU forward only)
#pragma unroll
  for (int r = 0; r < kSlots; ++r) {
    const int q = tid + kThreads * r;
    if (LA == KC) {  // rows = output rows of this expert, clamped to its last row
      const int row = q >> 3, c = q & 7;
      const int grow = t.r0 + min(t.mt * BM + row, t.rows - 1);
      aoff[r] = (long)grow * lda + c * 8;
      alds[r] = kc_chunk_off(row, c);
    } else {  // ragged K: [k][i], i = output row (weight-gradient row), clamped to the matrix
      const int krow = q >> 5, c = q & 31;
      const int i0 = min(t.mt * BM + c * 8, p.Mfix - 8);
      aoff[r] = (long)i0;  // row part added per step
      alds[r] = tr_chunk_off(krow, c);
    }
    bsrc[r] = 0;
    if (LB == KC) {  // rows = output columns n, k contiguous
      const int row = q >> 3, c = q & 7;
      const int n = min(t.nt * BN + row, p.N - 1);
      boff[r] = (long)t.e * p.gB + (long)n * ldb + c * 8;
      blds[r] = kc_chunk_off(row, c);
    } else {
      const int krow = q >> 5, c = q & 31;
      int col;
      if (kGluFwd) {  // tile columns: [wn][W1 64 | W3 64]
        const int w = c >> 4, half = (c >> 3) & 1, nn = c & 7;
        col = t.nt * kOutCols + w * 64 + nn * 8;
        bsrc[r] = half;
      } else {
        col = t.nt * BN + c * 8;
      }
      col = min(col, p.N - 8);
      boff[r] = (RAGGED_K ? 0 : (long)t.e * p.gB) + col;  // row part added per step
      blds[r] = tr_chunk_off(krow, c);
    }
  }

  u32x4 areg[kSlots], breg[kSlots];
  auto fetch = [&](int it) {
    const int pr = it / nk1;
    const int k0 = (it - pr * nk1) * BK;
    const bf16_t* A = static_cast<const bf16_t*>(p.A[RAGGED_K ? 0 : pr]);
    const bf16_t* B0 = static_cast<const bf16_t*>(p.B[RAGGED_K ? t.set : pr]);
    const bf16_t* B1 = kGluFwd ? static_cast<const bf16_t*>(p.B[1]) : B0;
#pragma unroll
    for (int r = 0; r < kSlots; ++r) {
      if (LA == KC) {
        areg[r] = *reinterpret_cast<const u32x4*>(A + aoff[r] + k0);
      } else {
        const int k = k0 + ((tid + kThreads * r) >> 5);
        areg[r] = k < Kg ? *reinterpret_cast<const u32x4*>(A + (long)(t.r0 + k) * lda + aoff[r]) : u32x4{0u, 0u, 0u, 0u};
      }
      if (LB == KC) {
        breg[r] = *reinterpret_cast<const u32x4*>(B0 + boff[r] + k0);
      } else {
        int k = k0 + ((tid + kThreads * r) >> 5);
        if (RAGGED_K) k = t.r0 + min(k, Kg - 1);
        breg[r] = *reinterpret_cast<const u32x4*>((bsrc[r] ? B1 : B0) + (long)k * ldb + boff[r]);
      }
    }
  };
  // half h of the prefetched tile -> LDS stage
  auto stash_half = [&](int stage, int h) {
    unsigned char* a = lds + stage * kStageBytes;
    unsigned char* b = a + kOperandBytes;
#pragma unroll
    for (int r = h * (kSlots / 2); r < (h + 1) * (kSlots / 2); ++r) {
      *reinterpret_cast<u32x4*>(a + alds[r]) = areg[r];
      *reinterpret_cast<u32x4*>(b + blds[r]) = breg[r];
    }
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  auto load_frags = [&](bf16x8(&af)[4], bf16x8(&bf)[4], const unsigned char* a, const unsigned char* b, int s) {
#pragma unroll
    for (int f = 0; f < 4; ++f) af[f] = read_frag<LA>(a, wm * 128 + f * 32, s, lane);
#pragma unroll
    for (int f = 0; f < 4; ++f) bf[f] = read_frag<LB>(b, wn * 128 + f * 32, s, lane);
  };
  auto mfma_step = [&](const bf16x8(&af)[4], const bf16x8(&bf)[4]) {
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int fn = 0; fn < 4; ++fn)
        acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[fn], af[fm], acc[fm][fn], 0, 0, 0);
  };
  // LDS reads of one k-step spread over the 16 MFMAs of the previous one
  constexpr int kReads = (LA == KC ? 4 : 8) + (LB == KC ? 4 : 8);
  auto interleave = [&](int ds_writes, int vmem) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // 2 MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, (kReads + 7) / 8, 0);  // DS reads
      if (ds_writes) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // 1 DS write
      if (vmem) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);       // 2 VMEM reads
    }
  };

  // One K iteration on LDS stage `it & 1`.  While its 64 MFMAs run, the tile for iteration it+1
  // (already in registers) goes to the other stage and the loads for iteration it+2 are issued.
  // Straight-line code (no branches) so that the scheduler can interleave the four instruction kinds.
  auto iteration = [&](int it, auto more_tag) {
    constexpr bool kMore = decltype(more_tag)::value;
    const unsigned char* a = lds + (it & 1) * kStageBytes;
    const unsigned char* b = a + kOperandBytes;
    bf16x8 af0[4], bf0[4], af1[4], bf1[4];
    load_frags(af0, bf0, a, b, 0);
    load_frags(af1, bf1, a, b, 1);
    mfma_step(af0, bf0);  // k-step 0
    interleave(0, 0);
    load_frags(af0, bf0, a, b, 2);
    if (kMore) stash_half((it + 1) & 1, 0);  // that stage was last read in iteration it-1
    mfma_step(af1, bf1);  // k-step 1
    interleave(kMore, 0);
    load_frags(af1, bf1, a, b, 3);
    if (kMore) stash_half((it + 1) & 1, 1);
    mfma_step(af0, bf0);  // k-step 2
    interleave(kMore, 0);
    if (kMore) fetch(min(it + 2, nk - 1));  // the last iterations re-fetch the final tile: harmless, branch-free
    mfma_step(af1, bf1);  // k-step 3
    interleave(0, kMore);
    if (kMore) __syncthreads();
  };

  if (nk > 0) {
    fetch(0);
    stash_half(0, 0);
    stash_half(0, 1);
    __syncthreads();
    if (nk > 1) fetch(1);
    for (int it = 0; it < nk - 1; ++it) iteration(it, std::true_type{});
    iteration(nk - 1, std::false_type{});
  }

  // ---- epilogue.  acc[fm][fn][4*rg + j] = C[row][col + j],
  //      row = wm*128 + fm*32 + lane%32,  col = wn*128 + fn*32 + rg*8 + (lane/32)*4  (tile coordinates)
  const int lrow = lane & 31, lcol = (lane >> 5) * 4;
  const int m_limit = RAGGED_K ? p.Mfix : t.rows;
#pragma unroll
  for (int fm = 0; fm < 4; ++fm) {
    const int mrow = t.mt * BM + wm * 128 + fm * 32 + lrow;  // row inside the group
    if (mrow >= m_limit) continue;
    const long rbase = RAGGED_K ? (long)t.e * p.gC + (long)mrow * p.ldc : (long)(t.r0 + mrow) * p.ldc;
#pragma unroll
    for (int fn = 0; fn < (kGluFwd ? 2 : 4); ++fn) {
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int col = kGluFwd ? t.nt * kOutCols + wn * 64 + fn * 32 + rg * 8 + lcol
                                : t.nt * BN + wn * 128 + fn * 32 + rg * 8 + lcol;
        if (col >= p.N) continue;
        const long off = rbase + col;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc[fm][fn][4 * rg + j];
        if (EPI == EPI_PLAIN) {
          bf16_t* c = static_cast<bf16_t*>(p.C[RAGGED_K ? t.set : 0]) + off;
          if (p.accumulate) {
            float old[4];
            load4(c, old);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] += old[j];
          }
          store4(c, v[0], v[1], v[2], v[3]);
        } else if (EPI == EPI_ACT_FWD) {
          store4(static_cast<bf16_t*>(p.C[0]) + off, v[0], v[1], v[2], v[3]);
          store4(static_cast<bf16_t*>(p.C[2]) + off, act_fwd(v[0], ACT), act_fwd(v[1], ACT), act_fwd(v[2], ACT),
                 act_fwd(v[3], ACT));
        } else if (EPI == EPI_GLU_FWD) {
          float g[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) g[j] = acc[fm][fn + 2][4 * rg + j];
          store4(static_cast<bf16_t*>(p.C[0]) + off, v[0], v[1], v[2], v[3]);
          store4(static_cast<bf16_t*>(p.C[1]) + off, g[0], g[1], g[2], g[3]);
          store4(static_cast<bf16_t*>(p.C[2]) + off, siluf_(v[0]) * g[0], siluf_(v[1]) * g[1], siluf_(v[2]) * g[2],
                 siluf_(v[3]) * g[3]);
        } else if (EPI == EPI_ACT_BWD) {
          float a1[4];
          load4(static_cast<const bf16_t*>(p.X[0]) + off, a1);
          store4(static_cast<bf16_t*>(p.C[0]) + off, v[0] * act_grad(a1[0], ACT), v[1] * act_grad(a1[1], ACT),
                 v[2] * act_grad(a1[2], ACT), v[3] * act_grad(a1[3], ACT));
        } else {
          float a1[4], a3[4];
          load4(static_cast<const bf16_t*>(p.X[0]) + off, a1);
          load4(static_cast<const bf16_t*>(p.X[1]) + off, a3);
          store4(static_cast<bf16_t*>(p.C[0]) + off, v[0] * a3[0] * silu_gradf_(a1[0]), v[1] * a3[1] * silu_gradf_(a1[1]),
                 v[2] * a3[2] * silu_gradf_(a1[2]), v[3] * a3[3] * silu_gradf_(a1[3]));
          store4(static_cast<bf16_t*>(p.C[1]) + off, v[0] * siluf_(a1[0]), v[1] * siluf_(a1[1]), v[2] * siluf_(a1[2]),
                 v[3] * siluf_(a1[3]));
        }
      }
    }
  }
}

template <int LA, int LB, int EPI, bool RAGGED_K, int ACT = 0>
moe_status_t launch_cfg(const GemmP& p, hipStream_t s) {
  constexpr int out_cols = EPI == EPI_GLU_FWD ? BN / 2 : BN;
  const int n_nt = ceil_div(p.N, out_cols);
  int mt_fix = 0, max_tiles;
  if (RAGGED_K) {
    mt_fix = ceil_div(p.Mfix, BM);
    max_tiles = (p.n_pairs == 2 ? 2 : 1) * p.n_experts * mt_fix * n_nt;
  } else {
    // each expert adds at most one partial row tile on top of the dense count
    long rows_bound = (long)p.max_rows * p.n_experts;
    if (rows_bound > p.total_rows_bound) rows_bound = p.total_rows_bound;
    max_tiles = (int)((rows_bound + BM - 1) / BM + p.n_experts) * n_nt;
  }
  if (max_tiles <= 0) return MOE_OK;
  static bool attr_set = false;
  auto kern = gg_mfma_kernel<LA, LB, EPI, RAGGED_K, ACT>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kLdsBytes);
    if (e != hipSuccess) {
      set_error("hipFuncSetAttribute(max dynamic LDS %d): %s", kLdsBytes, hipGetErrorString(e));
      return MOE_ERR_DEVICE;
    }
    attr_set = true;
  }
  const int grid = ceil_div(max_tiles, 8) * 8;  // the XCD remap wants a multiple of 8
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), kLdsBytes, s, p, n_nt, mt_fix);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

}  // namespace

bool gemm_mfma_supported(const GemmP& p, int dtype, int epi, bool ragged_k) {
  if (dtype != MOE_BF16) return false;
  if (p.N % 8 != 0 || p.N < 8) return false;
  if (ragged_k) return p.Mfix % 8 == 0 && p.Mfix >= 8;
  (void)epi;
  return p.Kfix % BK == 0;
}

moe_status_t launch_gemm_mfma(const GemmP& p, int epi, bool ragged_k, hipStream_t s) {
  if (ragged_k) return launch_cfg<TR, TR, EPI_PLAIN, true>(p, s);
  const bool b_kc = p.sBk == 1;  // B(k,n) = W[n][k]: the dgrad products
  switch (epi) {
    case EPI_PLAIN:
      return b_kc ? launch_cfg<KC, KC, EPI_PLAIN, false>(p, s) : launch_cfg<KC, TR, EPI_PLAIN, false>(p, s);
    case EPI_ACT_FWD:
      if (p.act == MOE_ACT_RELU) return launch_cfg<KC, TR, EPI_ACT_FWD, false, MOE_ACT_RELU>(p, s);
      if (p.act == MOE_ACT_GELU_TANH) return launch_cfg<KC, TR, EPI_ACT_FWD, false, MOE_ACT_GELU_TANH>(p, s);
      return launch_cfg<KC, TR, EPI_ACT_FWD, false, MOE_ACT_GELU_ERF>(p, s);
    case EPI_GLU_FWD: return launch_cfg<KC, TR, EPI_GLU_FWD, false>(p, s);
    case EPI_ACT_BWD:
      if (p.act == MOE_ACT_RELU) return launch_cfg<KC, KC, EPI_ACT_BWD, false, MOE_ACT_RELU>(p, s);
      if (p.act == MOE_ACT_GELU_TANH) return launch_cfg<KC, KC, EPI_ACT_BWD, false, MOE_ACT_GELU_TANH>(p, s);
      return launch_cfg<KC, KC, EPI_ACT_BWD, false, MOE_ACT_GELU_ERF>(p, s);
    default: return launch_cfg<KC, KC, EPI_GLU_BWD, false>(p, s);
  }
}

}  // namespace moe
