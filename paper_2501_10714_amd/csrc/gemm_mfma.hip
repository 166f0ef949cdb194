// bf16 grouped GEMM on the CDNA4 matrix cores for the expert FFNs (FSMoE Sec. 2.1 "Experts",
// Sec. 4.4 for the backward products): the one dense contraction of the layer.
//
// One workgroup (256 lanes = 4 waves, one per SIMD) owns a 256x256 output tile.  Each wave owns a
// 128x128 quadrant = 4x4 MFMA 32x32x16 tiles, fp32 accumulators (256 registers per lane).
//
// Operands travel global -> LDS directly (global_load_lds_dwordx4: no registers, no ds_write).  A
// wave-level load drops 64 x 16 bytes into 1 KB of contiguous LDS, so the bank swizzle is applied on
// the global side: each lane fetches the chunk that belongs at its LDS slot.  Two K pipelines:
//
//   gg_mfma_kernel    four LDS stages of 32 k (32 KB each), three in flight, one barrier per 32 k.
//                     Used by the weight-gradient products (both operands row-major, K = the ragged
//                     expert rows) and by any product whose K is not a multiple of 64.
//   gg_mfma64_kernel  64-k batches in a ring of five 32 KB buffers, one barrier per 64 k (described
//                     at its definition).  Used when the A operand is K-contiguous and K % 64 == 0:
//                     a K-contiguous operand then arrives in whole 128-byte cache lines.
//
// In both, the buffers are separate __shared__ arrays and the K loop is unrolled over a full turn
// of the ring, so every LDS access names its buffer statically; fragments are double buffered in
// registers (the MFMAs of one 16-k step run while the fragments of the next are read).
//
// Operand layouts in LDS (bf16), 32-k stages:
//   KC  "K-contiguous rows"  [256 rows][32 k]   64-byte rows, 16-byte chunks XOR-swizzled by row.
//        A lane reads its 8 consecutive k of one row with one ds_read_b128.
//   TR  "transposed feed"    [32 k][256 cols]   512-byte rows, 32-byte segments XOR-swizzled by k.
//        The operand is N-contiguous in memory but the MFMA wants 8 consecutive k per lane:
//        ds_read_b64_tr_b16 hands a 16-lane group the 4(k) x 16(col) block transposed.
//   The three products need: forward  A=KC (activations), B=TR (W[k][n]);
//                            dgrad    A=KC, B=KC (W^T: W rows are the output columns);
//                            wgrad    A=TR, B=TR (both operands are indexed by the ragged expert row).
//
// MFMA is issued with the operands swapped (B fragment first), so a lane ends up with 4 consecutive
// output COLUMNS of one output row per accumulator quad; the epilogue turns the quadrant row-major
// through LDS so that global stores (and the loads of the saved activations) are full cache lines.
//
// Tile order: tiles are ordered per expert in bands of 8 row-tiles x all column-tiles and dealt to
// the 8 XCDs in chunks of 32 (see find_tile).  Rows are ragged per expert: the tile list is derived
// from offsets[] on the device by every workgroup (E <= 256 scalar steps), no host synchronisation.
#include <cstdlib>
#include <type_traits>

#include "common.h"
#include "gemm_params.h"

namespace moe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // native vectors stay in registers
typedef unsigned char __attribute__((address_space(3))) lds_byte;

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int kThreads = 256;
constexpr int kStages = 4;
constexpr int kOpBytes = BM * BK * 2;  // 16 KB: one operand, one stage
constexpr int kBand = 8;               // row-tiles per L2 band
constexpr int kChunk = 32;             // consecutive logical tiles per XCD turn
constexpr int kLoads = kOpBytes / 1024 / 4;  // wave-level 1 KB loads per wave per operand per stage (4)
constexpr int kPartBytes = kLoads * 1024;    // one wave's share of one operand of one stage (4 KB)
constexpr int kRegionBytes = 2 * kPartBytes; // a stage is four wave regions [A part | B part]

enum Layout { KC = 0, TR = 1 };

// One array per stage (A operand, then B operand): accesses name their stage statically (see the
// header comment).  Four objects, so the compiler can track the in-flight loads of each separately.
__shared__ __attribute__((aligned(1024))) unsigned char g_st0[2 * kOpBytes], g_st1[2 * kOpBytes], g_st2[2 * kOpBytes],
    g_st3[2 * kOpBytes];

template <int S> __device__ __forceinline__ unsigned char* stage_a() {
  if constexpr (S == 0) return g_st0; else if constexpr (S == 1) return g_st1; else if constexpr (S == 2) return g_st2; else return g_st3;
}
template <int S> __device__ __forceinline__ unsigned char* stage_b() { return stage_a<S>() + kPartBytes; }

// Direct global -> LDS load of 16 bytes per lane: lane i's data lands at M0 + OFF + 16 i.  The
// immediate offset is added to the global address as well, so callers pass the pointer minus OFF.
// One M0 write serves a whole stage (a wave stalls on every M0 write until the loads issued before
// it have left the queue): the wave's region of a stage is [A part | B part], M0 points between
// the two and the eight loads use offsets -4096 .. 3072.
// Issued as inline assembly so that the pipeline below, not the compiler's conservative tracking of
// in-flight LDS writes, decides where the waits go.
__device__ __forceinline__ void dma_set_base(uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(lds_addr) : "memory");
}
template <int OFF> __device__ __forceinline__ void dma16(const unsigned char* g) {
  asm volatile("global_load_lds_dwordx4 %0, off offset:%1" ::"v"(g - OFF), "n"(OFF) : "memory");
}
constexpr int kDmaBias = 4096;
// a wave-uniform pointer the compiler may hold in vector registers (tile indices come out of
// integer divisions, which run on the vector ALU) -> scalar registers
__device__ __forceinline__ const unsigned char* to_sgpr(const unsigned char* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const unsigned char*>(((uint64_t)hi << 32) | lo);
}
template <int OFF> __device__ __forceinline__ void dma16s(uint32_t voff, const unsigned char* sbase) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(voff), "s"(sbase), "n"(OFF) : "memory");
}
template <bool IS_B> __device__ __forceinline__ void dma_block_s(uint32_t voff, const unsigned char* sbase, int j) {
  constexpr int base = IS_B ? 0 : -kPartBytes;
  switch (j) {
    case 0: dma16s<base>(voff, sbase); break;
    case 1: dma16s<base + 1024>(voff, sbase); break;
    case 2: dma16s<base + 2048>(voff, sbase); break;
    default: dma16s<base + 3072>(voff, sbase); break;
  }
}
// block j of the A part (j = 0..3) or of the B part
template <bool IS_B> __device__ __forceinline__ void dma_block(const unsigned char* g, int j) {
  constexpr int base = IS_B ? 0 : -kPartBytes;
  switch (j) {
    case 0: dma16<base>(g); break;
    case 1: dma16<base + 1024>(g); break;
    case 2: dma16<base + 2048>(g); break;
    default: dma16<base + 3072>(g); break;
  }
}
__device__ __forceinline__ uint32_t lds_addr_of(const unsigned char* p) {
  return (uint32_t)(uintptr_t)(lds_byte*)p;
}
__device__ __forceinline__ void stage_barrier() {
  static_assert(2 * 2 * kLoads == 16, "the immediate below is vmcnt(16)");
  asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// ---- byte offset of a 16-byte chunk inside a stage
// KC operand: row r of the tile lives in wave region r / 64
__device__ __forceinline__ int kc_chunk_off(int row, int c) {
  return (row >> 6) * kRegionBytes + (row & 63) * 64 + ((c ^ ((row >> 2) & 3)) << 4);
}
// TR operand: 32-byte segment s of k-row k sits at position s ^ tr_swz(k): the 4 rows x 2 segments that
// two 16-lane groups of one transposed read touch then fall into 8 different bank groups
__device__ __forceinline__ int tr_swz(int k) { return (k & 3) << 1; }
// TR operand: k-row k of the stage lives in wave region k / 8
__device__ __forceinline__ int tr_row_off(int k) { return (k >> 3) * kRegionBytes + (k & 7) * 512; }

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
  const int a0 = tr_row_off(k) + ((seg ^ tr_swz(k)) << 5) + ((i & 3) << 3);
  const int k1 = k + 4;
  const int a1 = tr_row_off(k1) + ((seg ^ tr_swz(k1)) << 5) + ((i & 3) << 3);
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
// Outputs are written once and the saved activations read once per kernel: both are marked non-temporal, so
// that they do not push operand panels out of L2 (measured: 0.3 - 2.7 % of a layer step, by shape).
__device__ __forceinline__ void store8(bf16_t* p, const float* v) {
  const u32x4 r = u32x4{pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
  __builtin_nontemporal_store(r, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void load8(const bf16_t* p, float* v) {
  const u32x4 r = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = __uint_as_float(r[i] << 16);
    v[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
  }
}

struct TileId {
  int e, set, mt, nt, r0, rows;
  bool valid;
};

// Logical tile index -> (expert, row tile, column tile).  Ragged M: row tiles per expert come from
// offsets[]; ragged K: every group has the same mt_fix row tiles.
// Number of output tiles of a launch.  Ragged M: row tiles per expert come from offsets[]; ragged K: every
// group has the same mt_fix row tiles.
template <bool RAGGED_K>
__device__ __forceinline__ int count_tiles(const GemmP& p, int n_nt, int mt_fix) {
  if (RAGGED_K) return ((p.n_pairs == 2) ? 2 * p.n_experts : p.n_experts) * mt_fix * n_nt;
  int total = 0;
  for (int e = 0; e < p.n_experts; ++e) total += ((p.row_end[e] - p.offsets[e] + BM - 1) / BM) * n_nt;
  return total;
}
// Logical tile index L < count_tiles() -> (expert, row tile, column tile): per expert, bands of about kBand
// row tiles x all column tiles, row tile fastest inside a band.
template <bool RAGGED_K>
__device__ __forceinline__ TileId tile_at(const GemmP& p, int n_nt, int mt_fix, int L) {
  TileId t;
  int g = 0, mt_g = mt_fix;
  if (RAGGED_K) {
    g = L / (mt_fix * n_nt);
    L -= g * mt_fix * n_nt;
  } else {
    for (;; ++g) {
      mt_g = (p.row_end[g] - p.offsets[g] + BM - 1) / BM;
      const int cnt = mt_g * n_nt;
      if (L < cnt) break;
      L -= cnt;
    }
  }
  // The mt_g row tiles are cut into bands of nearly equal height, about kBand each (6 .. 11): a last band of one
  // or two row tiles would share its B panels among that few tiles only.
  const int nbands = max(1, (mt_g + kBand / 2) / kBand);
  const int bh = mt_g / nbands, tall = mt_g % nbands;  // the first `tall` bands hold bh + 1 row tiles
  const int tall_tiles = tall * (bh + 1) * n_nt;
  int band, bsz, rem;
  if (L < tall_tiles) {
    bsz = bh + 1;
    band = L / (bsz * n_nt);
    rem = L - band * bsz * n_nt;
  } else {
    bsz = bh;
    const int l2 = L - tall_tiles;
    band = tall + l2 / (bsz * n_nt);
    rem = l2 - (band - tall) * bsz * n_nt;
  }
  t.nt = rem / bsz;
  t.mt = band * bh + min(band, tall) + rem % bsz;
  t.e = g % p.n_experts;
  t.set = g / p.n_experts;
  t.r0 = p.offsets[t.e];
  t.rows = p.row_end[t.e] - t.r0;
  t.valid = true;
  return t;
}
// XCD-aware deal: workgroup id b runs on XCD b % 8 (each XCD has its own L2).  Logical tiles are dealt to
// the XCDs in chunks of `chunk` consecutive ones (32 = 8 row tiles x 4 column tiles, one per CU of an XCD):
// inside an XCD the tiles of a chunk share A and B panels in its L2, and the 8 chunks in flight across the
// chip are neighbours in the same band, so they share their A panels in the memory-side cache.
__device__ __forceinline__ int dealt_tile(int slot, int chunk) {
  return (((slot / chunk) << 3) + (blockIdx.x & 7)) * chunk + (slot % chunk);
}
template <bool RAGGED_K>
__device__ __forceinline__ TileId find_tile(const GemmP& p, int n_nt, int mt_fix) {
  const int L = dealt_tile(blockIdx.x >> 3, kChunk);
  if (L >= count_tiles<RAGGED_K>(p, n_nt, mt_fix)) {
    TileId t;
    t.valid = false;
    return t;
  }
  return tile_at<RAGGED_K>(p, n_nt, mt_fix, L);
}

// ---- epilogue.  In the accumulators a lane holds 4 consecutive columns of 32 different rows
// (acc[fm][fn][4 rg + j] = C[wm*128 + fm*32 + lane%32][wn*128 + fn*32 + rg*8 + (lane/32)*4 + j]);
// stored like that, every store instruction would scatter 16-byte pieces over 32 rows and the L2
// write path would set the pace.  Each wave therefore passes its quadrant through 16 KB of LDS of its
// own (`scr`), 32 rows at a time in fp32, and reads it back row-major: a lane then owns 8 consecutive
// columns, 16 lanes cover 256 contiguous bytes of a row, and all global loads and stores of the fused
// epilogues are 16-byte vectors on full cache lines.  Scratch row r (128 floats) keeps 16-byte chunk q
// at slot q ^ r: column writes (32 rows, one chunk) and row reads (one row, 16 chunks) both touch every
// bank once.  The caller makes sure that no wave still reads, and no load still fills, that LDS.
template <int EPI, bool RAGGED_K, int ACT>
__device__ __forceinline__ void tile_epilogue(const GemmP& p, const TileId& t, f32x16 (&acc)[4][4], float* scr, int wave, int lane) {
  constexpr bool kGluFwd = EPI == EPI_GLU_FWD;
  constexpr int kOutCols = kGluFwd ? BN / 2 : BN;
  const int wm = wave >> 1, wn = wave & 1;
  auto scr_at = [&](int r, int q) { return scr + r * 128 + ((q ^ r) << 2); };  // row r (0..31), 16-byte chunk q (0..31)
  const int m_limit = RAGGED_K ? p.Mfix : t.rows;
  constexpr int kLanesPerRow = kGluFwd ? 8 : 16;   // 8 columns per lane
  constexpr int kRowsPerPass = 64 / kLanesPerRow;
  constexpr int kPasses = 32 / kRowsPerPass;
  const int pr = lane / kLanesPerRow, c8 = (lane % kLanesPerRow) * 8;
  const int col = kGluFwd ? t.nt * kOutCols + wn * 64 + c8 : t.nt * BN + wn * 128 + c8;
  const bool col_ok = col < p.N;  // N is a multiple of 8
  auto out_off = [&](int mrow, int c) {
    return (RAGGED_K ? (long)t.e * p.gC + (long)mrow * p.ldc : (long)(t.r0 + mrow) * p.ldc) + c;
  };
  // The backward epilogues read the saved pre-activations at the output position.  The loads of a
  // 32-row block go out one block ahead (addresses clamped into the tensor, so they need no
  // predicate), and their latency passes under the LDS turn of the block before.
  constexpr int kNX = EPI == EPI_GLU_BWD ? 2 : (EPI == EPI_ACT_BWD || EPI == EPI_ACCUM) ? 1 : 0;
  u32x4 xin[2][kPasses][kNX > 0 ? kNX : 1];
  auto prefetch = [&](int fm) {
    if constexpr (kNX > 0) {
      const int cc = min(col, p.N - 8);
#pragma unroll
      for (int ps = 0; ps < kPasses; ++ps) {
        const int mrow = min(t.mt * BM + wm * 128 + fm * 32 + ps * kRowsPerPass + pr, m_limit - 1);
        const long off = out_off(mrow, cc);
#pragma unroll
        for (int x = 0; x < kNX; ++x)
          xin[fm & 1][ps][x] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(static_cast<const bf16_t*>(EPI == EPI_ACCUM ? p.C[0] : p.X[x]) + off));
      }
    }
  };
  auto widen8 = [](const u32x4& r, float* v) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(r[i] << 16);
      v[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  };
  prefetch(0);
#pragma unroll
  for (int fm = 0; fm < 4; ++fm) {
    if (fm + 1 < 4) prefetch(fm + 1);
#pragma unroll
    for (int fn = 0; fn < 4; ++fn)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        f32x4 v = {acc[fm][fn][4 * rg], acc[fm][fn][4 * rg + 1], acc[fm][fn][4 * rg + 2], acc[fm][fn][4 * rg + 3]};
        *reinterpret_cast<f32x4*>(scr_at(lane & 31, fn * 8 + rg * 2 + (lane >> 5))) = v;
      }
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
      const int r = ps * kRowsPerPass + pr;
      const int mrow = t.mt * BM + wm * 128 + fm * 32 + r;  // row inside the group
      float v[8];
      {
        const f32x4 lo = *reinterpret_cast<const f32x4*>(scr_at(r, c8 >> 2));
        const f32x4 hi = *reinterpret_cast<const f32x4*>(scr_at(r, (c8 >> 2) + 1));
#pragma unroll
        for (int j = 0; j < 4; ++j) { v[j] = lo[j]; v[4 + j] = hi[j]; }
      }
      float g[8];
      if (kGluFwd) {
        const f32x4 lo = *reinterpret_cast<const f32x4*>(scr_at(r, 16 + (c8 >> 2)));
        const f32x4 hi = *reinterpret_cast<const f32x4*>(scr_at(r, 17 + (c8 >> 2)));
#pragma unroll
        for (int j = 0; j < 4; ++j) { g[j] = lo[j]; g[4 + j] = hi[j]; }
      }
      if (mrow >= m_limit || !col_ok) continue;
      const long off = out_off(mrow, col);
      if (EPI == EPI_PLAIN) {
        bf16_t* c = static_cast<bf16_t*>(p.C[RAGGED_K ? t.set : 0]) + off;
        if (p.accumulate) {
          float old[8];
          load8(c, old);
#pragma unroll
          for (int j = 0; j < 8; ++j) v[j] += old[j];
        }
        store8(c, v);
      } else if (EPI == EPI_ACT_FWD) {
        store8(static_cast<bf16_t*>(p.C[0]) + off, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_fwd(v[j], ACT);
        store8(static_cast<bf16_t*>(p.C[2]) + off, v);
      } else if (EPI == EPI_GLU_FWD) {
        store8(static_cast<bf16_t*>(p.C[0]) + off, v);
        store8(static_cast<bf16_t*>(p.C[1]) + off, g);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = siluf_(v[j]) * g[j];
        store8(static_cast<bf16_t*>(p.C[2]) + off, v);
      } else if (EPI == EPI_ACCUM) {
        float old[8];
        widen8(xin[fm & 1][ps][0], old);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] += old[j];
        store8(static_cast<bf16_t*>(p.C[0]) + off, v);
      } else if (EPI == EPI_ACT_BWD) {
        float a1[8];
        widen8(xin[fm & 1][ps][0], a1);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] *= act_grad(a1[j], ACT);
        store8(static_cast<bf16_t*>(p.C[0]) + off, v);
      } else {
        float a1[8], a3[8], d1[8], d3[8];
        widen8(xin[fm & 1][ps][0], a1);
        widen8(xin[fm & 1][ps][kNX > 1 ? 1 : 0], a3);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float sg = sigmoidf_(a1[j]);
          d1[j] = v[j] * a3[j] * (sg * (1.0f + a1[j] * (1.0f - sg)));  // dhh * a3 * silu'(a1)
          d3[j] = v[j] * (a1[j] * sg);                                   // dhh * silu(a1)
        }
        store8(static_cast<bf16_t*>(p.C[0]) + off, d1);
        store8(static_cast<bf16_t*>(p.C[1]) + off, d3);
      }
    }
  }
}

template <int LA, int LB, int EPI, bool RAGGED_K, int ACT>
__global__ __launch_bounds__(kThreads, 1) void gg_mfma_kernel(GemmP p, int n_nt, int mt_fix) {
  constexpr bool kGluFwd = EPI == EPI_GLU_FWD;
  constexpr int kOutCols = kGluFwd ? BN / 2 : BN;  // output columns per tile

  const TileId t = find_tile<RAGGED_K>(p, n_nt, mt_fix);
  if (!t.valid) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const int Kg = RAGGED_K ? t.rows : p.Kfix;
  const int sum_pairs = (!RAGGED_K && !kGluFwd) ? p.n_pairs : 1;
  const int nk1 = (Kg + BK - 1) / BK;
  const int nk = nk1 * sum_pairs;

  // ---- global side of the direct-to-LDS loads.  Load j of this wave fills the 1 KB block
  //      blk = wave*4 + j of the stage; lane i owns bytes [16 i, 16 i + 16) of it and fetches the
  //      chunk the swizzle puts there.  Pointers advance by a uniform stride per K stage.
  const long lda = RAGGED_K ? p.sAk : p.sAi;  // row stride (elements) of the A array in memory
  const long ldb = RAGGED_K ? p.sBk : (LB == TR ? p.sBk : p.sBn);
  // Addresses: scalar base (steps along K) + 32-bit lane offset (fixed for the tile); see dma16s.
  // The Mixtral forward tile draws its columns from two tensors: its B loads keep 64-bit lane addresses.
  constexpr bool kBPtr = kGluFwd;
  uint32_t va[kLoads], vb[kLoads];
  const unsigned char* gb[kLoads];
  const unsigned char* sa;
  const unsigned char* sb;
  int ka[kLoads], kb[kLoads];  // row-major layouts: byte offset of this lane's k-row inside the stage (k-row * row pitch)
  {
    const bf16_t* A = static_cast<const bf16_t*>(p.A[0]);
    const bf16_t* B0 = static_cast<const bf16_t*>(p.B[RAGGED_K ? t.set : 0]);
    const bf16_t* B1 = kGluFwd ? static_cast<const bf16_t*>(p.B[1]) : B0;
    sa = to_sgpr(reinterpret_cast<const unsigned char*>(LA == KC ? A + (long)(t.r0 + t.mt * BM) * lda : A + (long)t.r0 * lda + t.mt * BM) - kDmaBias);
    {
      const long rowpart = (LB == TR && RAGGED_K) ? (long)t.r0 * ldb : (long)t.e * p.gB;
      sb = to_sgpr(reinterpret_cast<const unsigned char*>(B0 + rowpart + (LB == KC ? (long)t.nt * BN * ldb : (long)t.nt * BN)) - kDmaBias);
    }
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int blk = wave * kLoads + j;
      const uint32_t bias_a = (uint32_t)(kDmaBias - (-kPartBytes + 1024 * j)), bias_b = (uint32_t)(kDmaBias - 1024 * j);
      if (LA == KC) {  // 16 rows x 64 B per block; rows = output rows of this expert, clamped to its last row
        const int row = blk * 16 + (lane >> 2), slot = lane & 3;
        const int c = slot ^ ((row >> 2) & 3);
        const int rrow = min(t.mt * BM + row, t.rows - 1) - t.mt * BM;
        va[j] = (uint32_t)rrow * (uint32_t)(lda * 2) + c * 16 + bias_a;
        ka[j] = 0;
      } else {  // 2 k-rows x 512 B per block; ragged K: [k][i], i = weight-gradient row, clamped to the matrix
        const int krow = blk * 2 + (lane >> 5), pos = lane & 31;
        const int seg = (pos >> 1) ^ tr_swz(krow);
        const int ri = min(t.mt * BM + (seg * 2 + (pos & 1)) * 8, p.Mfix - 8) - t.mt * BM;
        va[j] = ri * 2 + bias_a;  // + the k-row part, added per load (clamped at the expert's last row)
        ka[j] = krow * (int)(lda * 2);
      }
      vb[j] = 0;
      gb[j] = nullptr;
      if (LB == KC) {  // rows = output columns n, k contiguous
        const int row = blk * 16 + (lane >> 2), slot = lane & 3;
        const int c = slot ^ ((row >> 2) & 3);
        const int rn = min(t.nt * BN + row, p.N - 1) - t.nt * BN;
        vb[j] = (uint32_t)rn * (uint32_t)(ldb * 2) + c * 16 + bias_b;
        kb[j] = 0;
      } else {
        const int krow = blk * 2 + (lane >> 5), pos = lane & 31;
        const int seg = (pos >> 1) ^ tr_swz(krow);
        const int cc = seg * 2 + (pos & 1);  // 8-column chunk of the tile
        if (kGluFwd) {  // tile columns: [wn][W1 64 | W3 64]
          const int col = min(t.nt * kOutCols + (cc >> 4) * 64 + (cc & 7) * 8, p.N - 8);
          const bf16_t* B = ((cc >> 3) & 1) ? B1 : B0;
          gb[j] = reinterpret_cast<const unsigned char*>(B + (long)t.e * p.gB + (long)krow * ldb + col);
        } else {
          const int rcol = min(t.nt * BN + cc * 8, p.N - 8) - t.nt * BN;
          vb[j] = rcol * 2 + bias_b;
        }
        kb[j] = krow * (int)(ldb * 2);
      }
    }
  }
  const long a_step = (LA == KC ? (long)BK : (long)BK * lda) * 2;  // bytes per K stage
  const long b_step = (LB == KC ? (long)BK : (long)BK * ldb) * 2;
  // second operand pair of a summed product (dxe = da1.W1^T + da3.W3^T): jump of the bases at it = nk1
  const long a_jump = sum_pairs == 2 ? reinterpret_cast<const unsigned char*>(p.A[1]) - reinterpret_cast<const unsigned char*>(p.A[0]) - nk1 * a_step : 0;
  const long b_jump = sum_pairs == 2 ? reinterpret_cast<const unsigned char*>(p.B[1]) - reinterpret_cast<const unsigned char*>(p.B[0]) - nk1 * b_step : 0;

  // Loads of K stage `it_load` into LDS stage S, one wave-level load per call (q = 0..7: A0 B0 A1 B1 ...);
  // after the last one the bases step to the next K stage.  Stages past the end re-fetch the last
  // one (never read), so the number of loads in flight is the same in every iteration.
  int it_load = 0;
  auto issue_one = [&](auto stage_tag, int q) {
    constexpr int S = decltype(stage_tag)::value;
    const int j = q >> 1;
    const bool is_b = q & 1;
    if (q == 0) dma_set_base(lds_addr_of(stage_a<S>()) + wave * kRegionBytes + kPartBytes);
    // ragged K: rows past the expert's last re-read its last row (finite data); the A rows are zeroed
    // in LDS once they have landed (see iteration()), so those products vanish.  The clamp is one
    // v_min against a scalar: min(k-row, last row of the expert inside this stage) * row pitch.
    const int last_row = RAGGED_K ? min(Kg - 1 - it_load * BK, BK) : BK;  // >= 0: stages past the end re-fetch the last one
    if (is_b) {
      if (kBPtr) dma_block<true>(gb[j], j);
      else dma_block_s<true>(vb[j] + (LB == TR ? (uint32_t)min(kb[j], last_row * (int)(ldb * 2)) : 0u), to_sgpr(sb), j);
    } else {
      dma_block_s<false>(va[j] + (LA == TR ? (uint32_t)min(ka[j], last_row * (int)(lda * 2)) : 0u), to_sgpr(sa), j);
    }
    if (q == 2 * kLoads - 1) {
      const bool last = it_load + 1 >= nk;
      const bool jump = it_load + 1 == nk1 && sum_pairs == 2;
      const long da_ = last ? 0 : a_step + (jump ? a_jump : 0);
      const long db_ = last ? 0 : b_step + (jump ? b_jump : 0);
      sa += da_;
      if (kBPtr) {
#pragma unroll
        for (int u = 0; u < kLoads; ++u) gb[u] += db_;
      } else {
        sb += db_;
      }
      it_load += last ? 0 : 1;
    }
  };
  auto issue = [&](auto stage_tag) {
#pragma unroll
    for (int q = 0; q < 2 * kLoads; ++q) issue_one(stage_tag, q);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  bf16x8 ax[4], bx[4], ay[4], by[4];  // fragment sets X (first 16 k of a stage) and Y (second 16 k)
  auto mfma_step = [&](const bf16x8(&af)[4], const bf16x8(&bf)[4]) {
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int fn = 0; fn < 4; ++fn)
        acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[fn], af[fm], acc[fm][fn], 0, 0, 0);
  };

  int it_cur = 0;
  // One K stage.  On entry set Y holds the second half of the previous stage (kFirst: nothing).
  auto iteration = [&](auto stage_tag, auto first_tag) {
    constexpr int S = decltype(stage_tag)::value;
    constexpr bool kFirst = decltype(first_tag)::value;
    // (a) all but the two youngest stages of this wave's loads have landed, so stage S is in LDS;
    // (b) this wave's fragment reads of stage S-1 have returned; then the barrier makes both true for
    // every wave.  A bare s_barrier, not __syncthreads(): the fence of the latter waits for ALL loads.
    stage_barrier();
    if (RAGGED_K) {
      if (it_cur == nk - 1 && (Kg & (BK - 1)) != 0) {  // ragged K tail: zero the A rows past the expert's last
#pragma unroll
        for (int j = 0; j < kLoads; ++j)
          if (it_cur * BK + (wave * kLoads + j) * 2 + (lane >> 5) >= Kg)
            *reinterpret_cast<u32x4*>(stage_a<S>() + wave * kRegionBytes + j * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};
        __syncthreads();
      }
      ++it_cur;
    }
    // Eight groups of 4 MFMAs, each with one load of stage S+3 and two fragment reads.  The address unit
    // of the CU takes ~16 cycles per load and four waves share it, so the loads are spread over the
    // whole stage instead of being bunched behind the barrier.
    // First half: this stage's first fragments (X) under the MFMAs of the previous stage's second half (Y).
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // B fragments first: the first MFMA on X needs all four of them, but only ax[0].
      // One MFMA, then at most one fragment read (1-2 LDS instructions) or one load: a wave has a
      // single instruction stream, and a run of other instructions between two MFMAs that lasts
      // longer than the 32 cycles of an MFMA leaves the matrix pipe idle.  The scheduler is held
      // to this order (sched_barrier): left alone it sinks the reads down to their use.
      if (j < 2) bx[2 * j] = read_frag<LB>(stage_b<S>(), wn * 128 + (2 * j) * 32, 0, lane);
      else ax[2 * j - 4] = read_frag<LA>(stage_a<S>(), wm * 128 + (2 * j - 4) * 32, 0, lane);
      if (!kFirst) acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[0], ay[j], acc[j][0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (j < 2) bx[2 * j + 1] = read_frag<LB>(stage_b<S>(), wn * 128 + (2 * j + 1) * 32, 0, lane);
      else ax[2 * j - 3] = read_frag<LA>(stage_a<S>(), wm * 128 + (2 * j - 3) * 32, 0, lane);
      if (!kFirst) acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[1], ay[j], acc[j][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      issue_one(std::integral_constant<int, (S + 3) % kStages>{}, j);
      if (!kFirst) acc[j][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[2], ay[j], acc[j][2], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (!kFirst) acc[j][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[3], ay[j], acc[j][3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // Second half: this stage's second fragments (Y) under the MFMAs of X.
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (j < 2) by[2 * j] = read_frag<LB>(stage_b<S>(), wn * 128 + (2 * j) * 32, 1, lane);
      else ay[2 * j - 4] = read_frag<LA>(stage_a<S>(), wm * 128 + (2 * j - 4) * 32, 1, lane);
      acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[0], ax[j], acc[j][0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (j < 2) by[2 * j + 1] = read_frag<LB>(stage_b<S>(), wn * 128 + (2 * j + 1) * 32, 1, lane);
      else ay[2 * j - 3] = read_frag<LA>(stage_a<S>(), wm * 128 + (2 * j - 3) * 32, 1, lane);
      acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[1], ax[j], acc[j][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      issue_one(std::integral_constant<int, (S + 3) % kStages>{}, 4 + j);
      acc[j][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[2], ax[j], acc[j][2], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      acc[j][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[3], ax[j], acc[j][3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  if (nk > 0) {
    issue(std::integral_constant<int, 0>{});
    issue(std::integral_constant<int, 1>{});
    issue(std::integral_constant<int, 2>{});
    iteration(std::integral_constant<int, 0>{}, std::true_type{});
    int it = 1;
    for (; it + 4 <= nk; it += 4) {
      iteration(std::integral_constant<int, 1>{}, std::false_type{});
      iteration(std::integral_constant<int, 2>{}, std::false_type{});
      iteration(std::integral_constant<int, 3>{}, std::false_type{});
      iteration(std::integral_constant<int, 0>{}, std::false_type{});
    }
    if (it < nk) iteration(std::integral_constant<int, 1>{}, std::false_type{});
    if (it + 1 < nk) iteration(std::integral_constant<int, 2>{}, std::false_type{});
    if (it + 2 < nk) iteration(std::integral_constant<int, 3>{}, std::false_type{});
    mfma_step(ay, by);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the re-fetches past the end must land before the LDS goes back to the pool
  }

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the re-fetches past the end have landed
  __syncthreads();                                  // every wave is done with the K stages
  tile_epilogue<EPI, RAGGED_K, ACT>(p, t, acc, reinterpret_cast<float*>(wave == 0 ? g_st0 : wave == 1 ? g_st1 : wave == 2 ? g_st2 : g_st3), wave, lane);
}

// ============================================================================================
// Second K pipeline, for products whose A operand is K-contiguous (all but the weight gradients)
// and whose K is a multiple of 64.
//
// The L1 fills whole 128-byte lines: a direct-to-LDS load that takes only 64 bytes of each line (a
// 32-k slice of a K-contiguous row) runs at half the rate of one that takes full lines (measured:
// 29 vs 58 bytes/clk/CU from L2), and with two such operands the load path, not the matrix cores,
// sets the pace.  Here a K-contiguous operand therefore arrives 64 k at a time: a batch is
// [256 rows][64 k] = 32 KB, a wave-level load covers 8 rows x 128 bytes.  (A row-major B batch is
// [64 k][256 columns], 2 k-rows x 512 bytes per load, as before.)
//
// LDS holds five batch buffers (160 KB).  Batches are issued in the order A0 B0 A1 B1 ..., batch j
// into buffer j mod 5.  A 64-k step m multiplies batches 2m and 2m+1 in two halves of 32 k; during
// its first half batch 2m+3 is issued (into the buffer that held A of step m-1), during its second
// half batch 2m+4 (the buffer of B of step m-1).  So a batch has between one and three half-steps
// to land, and one barrier per 64 k is enough: it says that every wave has batches 2m and 2m+1 and
// has finished reading step m-1.  The loop is unrolled over five steps (the buffer assignment
// repeats every ten batches), so every LDS access names its buffer statically.
constexpr int BK2 = 64;
constexpr int kBatchBytes = BM * BK2 * 2;  // 32 KB
static_assert(kBatchBytes == 2 * kOpBytes, "a batch buffer is one of the 32 KB stage arrays");
__shared__ __attribute__((aligned(1024))) unsigned char g_st4[kBatchBytes];

template <int B> __device__ __forceinline__ unsigned char* batch_buf() {
  if constexpr (B == 0) return g_st0; else if constexpr (B == 1) return g_st1; else if constexpr (B == 2) return g_st2;
  else if constexpr (B == 3) return g_st3; else return g_st4;
}
// load q (0..7) of a wave's 8 KB share of a batch; M0 points at the middle of that share
__device__ __forceinline__ void dma_block8s(uint32_t voff, const unsigned char* sbase, int q) {
  switch (q) {
    case 0: dma16s<-4096>(voff, sbase); break;
    case 1: dma16s<-3072>(voff, sbase); break;
    case 2: dma16s<-2048>(voff, sbase); break;
    case 3: dma16s<-1024>(voff, sbase); break;
    case 4: dma16s<0>(voff, sbase); break;
    case 5: dma16s<1024>(voff, sbase); break;
    case 6: dma16s<2048>(voff, sbase); break;
    default: dma16s<3072>(voff, sbase); break;
  }
}
__device__ __forceinline__ void batch_barrier() {
  asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// K-contiguous batch: 128-byte rows, 16-byte chunk c of row r at position c ^ ((r >> 1) & 7): the 16
// rows a quarter-wave reads with one ds_read_b128 pass then cover all 64 banks once
__device__ __forceinline__ int kc64_swz(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ bf16x8 read_kc64(const unsigned char* op, int row0, int ks, int lane) {
  const int row = row0 + (lane & 31);
  const int c = 2 * ks + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(op + row * 128 + ((c ^ kc64_swz(row)) << 4));
}
// row-major batch: k-row k at k * PITCH, segments swizzled as in the 32-k stages.  PITCH 512: one
// tensor, 256 columns.  PITCH 256: the Mixtral forward tile, whose batch is two halves of 16 KB,
// [64 k][128 columns of W1] then [64 k][128 columns of W3], so that a wave-level load (4 k-rows x
// 256 bytes) draws on one tensor and can take the scalar-base form.
template <int PITCH>
__device__ __forceinline__ bf16x8 read_tr64(const unsigned char* op, int col0, int ks, int lane) {
  const int grp = lane >> 4, i = lane & 15;
  const int seg = (col0 >> 4) + (grp & 1);
  const int k = 16 * ks + 8 * (grp >> 1) + (i >> 2);
  const int a0 = k * PITCH + ((seg ^ tr_swz(k)) << 5) + ((i & 3) << 3);
  const int k1 = k + 4;
  const int a1 = k1 * PITCH + ((seg ^ tr_swz(k1)) << 5) + ((i & 3) << 3);
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(op + a0));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(op + a1));
  union { s16x4 h[2]; bf16x8 v; } u;
  u.h[0] = lo; u.h[1] = hi;
  return u.v;
}

template <int LB, int EPI, int ACT>
__global__ __launch_bounds__(kThreads, 1) void gg_mfma64_kernel(GemmP p, int n_nt) {
  constexpr bool kGluFwd = EPI == EPI_GLU_FWD;
  constexpr int kOutCols = kGluFwd ? BN / 2 : BN;

  const TileId t = find_tile<false>(p, n_nt, 0);
  if (!t.valid) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const int sum_pairs = !kGluFwd ? p.n_pairs : 1;
  const int nb1 = p.Kfix / BK2;     // 64-k steps per operand pair
  const int nb = nb1 * sum_pairs;   // 64-k steps in all

  const long lda = p.sAi;
  const long ldb = LB == TR ? p.sBk : p.sBn;
  // Addresses of the direct-to-LDS loads: scalar base (steps along K) + 32-bit lane offset (fixed for the
  // tile).  A wave is held at such a load while its addresses go out, and the MFMA queue drains
  // meanwhile: about 18 cycles with a 64-bit address per lane, about 3 with a 32-bit offset (measured).
  // The instruction adds its immediate offset to the LDS address and to the global address alike, so
  // the lane offset carries kDmaBias - OFF and the scalar base is kDmaBias short.
  uint32_t va[8], vb[8];
  const unsigned char* sa;
  const unsigned char* sb;
  const unsigned char* sb3;  // Mixtral forward: W3 (sb is W1)
  {
    const bf16_t* A = static_cast<const bf16_t*>(p.A[0]);
    const bf16_t* B0 = static_cast<const bf16_t*>(p.B[0]);
    const bf16_t* B1 = kGluFwd ? static_cast<const bf16_t*>(p.B[1]) : B0;
    sa = to_sgpr(reinterpret_cast<const unsigned char*>(A + (long)(t.r0 + t.mt * BM) * lda) - kDmaBias);
    sb = to_sgpr(reinterpret_cast<const unsigned char*>(B0 + (long)t.e * p.gB + (LB == KC ? (long)t.nt * BN * ldb : (long)t.nt * kOutCols)) - kDmaBias);
    sb3 = to_sgpr(reinterpret_cast<const unsigned char*>(B1 + (long)t.e * p.gB + (long)t.nt * kOutCols) - kDmaBias);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t bias = (uint32_t)(kDmaBias - (-4096 + 1024 * j));
      // K-contiguous: load j of this wave = rows 64 wave + 8 j .. + 7, lane i -> (row i / 8, slot i % 8)
      const int row = wave * 64 + j * 8 + (lane >> 3), slot = lane & 7;
      const int c = slot ^ kc64_swz(row);
      const int rrow = min(t.mt * BM + row, t.rows - 1) - t.mt * BM;  // rows past the expert's last re-read it
      va[j] = (uint32_t)rrow * (uint32_t)(lda * 2) + c * 16 + bias;
      vb[j] = 0;
      if (LB == KC) {
        const int rn = min(t.nt * BN + row, p.N - 1) - t.nt * BN;
        vb[j] = (uint32_t)rn * (uint32_t)(ldb * 2) + c * 16 + bias;
      } else if (kGluFwd) {  // load j of half j / 4 = k-rows 16 wave + 4 (j % 4) .. + 3; lane i -> (k-row i / 16, slot i % 16)
        const int krow = wave * 16 + (j & 3) * 4 + (lane >> 4), pos = lane & 15;
        const int seg = (pos >> 1) ^ tr_swz(krow);
        const int rcol = min(t.nt * kOutCols + (seg * 2 + (pos & 1)) * 8, p.N - 8) - t.nt * kOutCols;
        vb[j] = (uint32_t)krow * (uint32_t)(ldb * 2) + rcol * 2 + (uint32_t)(kDmaBias - (-2048 + 1024 * (j & 3)));
      } else {  // row-major: load j = k-rows 16 wave + 2 j, + 1; lane i -> (k-row i / 32, 16-byte slot i % 32)
        const int krow = wave * 16 + j * 2 + (lane >> 5), pos = lane & 31;
        const int seg = (pos >> 1) ^ tr_swz(krow);
        const int rcol = min(t.nt * BN + (seg * 2 + (pos & 1)) * 8, p.N - 8) - t.nt * BN;
        vb[j] = (uint32_t)krow * (uint32_t)(ldb * 2) + rcol * 2 + bias;
      }
    }
  }
  const long a_step = (long)BK2 * 2;  // bytes per batch
  const long b_step = (LB == KC ? (long)BK2 : (long)BK2 * ldb) * 2;
  const long a_jump = sum_pairs == 2 ? reinterpret_cast<const unsigned char*>(p.A[1]) - reinterpret_cast<const unsigned char*>(p.A[0]) - nb1 * a_step : 0;
  const long b_jump = sum_pairs == 2 ? reinterpret_cast<const unsigned char*>(p.B[1]) - reinterpret_cast<const unsigned char*>(p.B[0]) - nb1 * b_step : 0;

  // One wave-level load of the next A (or B) batch into buffer BUF; after the eighth the base steps
  // to the following batch.  Batches past the end re-fetch the last one into a free buffer (never
  // read), so the number of loads in flight at a barrier is always the same.
  int ia = 0, ib = 0;
  auto issue_a = [&](auto buf_tag, int q) {
    constexpr int BUF = decltype(buf_tag)::value;
    if (q == 0) dma_set_base(lds_addr_of(batch_buf<BUF>()) + wave * 8192 + 4096);
    dma_block8s(va[q], to_sgpr(sa), q);
    if (q == 7) {
      const bool last = ia + 1 >= nb;
      sa += last ? 0 : a_step + ((ia + 1 == nb1 && sum_pairs == 2) ? a_jump : 0);
      ia += last ? 0 : 1;
    }
  };
  auto issue_b = [&](auto buf_tag, int q) {
    constexpr int BUF = decltype(buf_tag)::value;
    if (kGluFwd) {
      if ((q & 3) == 0) dma_set_base(lds_addr_of(batch_buf<BUF>()) + (q >> 2) * (kBatchBytes / 2) + wave * 4096 + 2048);
      const unsigned char* base = to_sgpr(q < 4 ? sb : sb3);
      switch (q & 3) {
        case 0: dma16s<-2048>(vb[q], base); break;
        case 1: dma16s<-1024>(vb[q], base); break;
        case 2: dma16s<0>(vb[q], base); break;
        default: dma16s<1024>(vb[q], base); break;
      }
    } else {
      if (q == 0) dma_set_base(lds_addr_of(batch_buf<BUF>()) + wave * 8192 + 4096);
      dma_block8s(vb[q], to_sgpr(sb), q);
    }
    if (q == 7) {
      const bool last = ib + 1 >= nb;
      const long d = last ? 0 : b_step + ((ib + 1 == nb1 && sum_pairs == 2) ? b_jump : 0);
      sb += d;
      sb3 += d;
      ib += last ? 0 : 1;
    }
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  bf16x8 ax[4], bx[4], ay[4], by[4];  // fragment sets X (first 16 k of a half-step) and Y (second 16 k)
  auto frag_a = [&](const unsigned char* buf, int f, int ks) { return read_kc64(buf, wm * 128 + f * 32, ks, lane); };
  auto frag_b = [&](const unsigned char* buf, int f, int ks) {
    if (LB == KC) return read_kc64(buf, wn * 128 + f * 32, ks, lane);
    if (kGluFwd) return read_tr64<256>(buf + (f >> 1) * (kBatchBytes / 2), wn * 64 + (f & 1) * 32, ks, lane);
    return read_tr64<512>(buf, wn * 128 + f * 32, ks, lane);
  };

  // Half-step PH of the ten in a period: 64-k step U = PH / 2 of five, half H = PH % 2.
  auto half_step = [&](auto ph_tag, auto first_tag) {
    constexpr int PH = decltype(ph_tag)::value;
    constexpr bool kFirst = decltype(first_tag)::value;
    constexpr int U = PH / 2, H = PH % 2;
    constexpr int ABUF = (2 * U) % 5, BBUF = (2 * U + 1) % 5;
    constexpr int LBUF = H == 0 ? (2 * U + 3) % 5 : (2 * U + 4) % 5;  // H = 0 issues a B batch, H = 1 an A batch
    const unsigned char* abuf = batch_buf<ABUF>();
    const unsigned char* bbuf = batch_buf<BBUF>();
    if (H == 0) batch_barrier();
    // Eight regions of 4 MFMAs, each with one load and two fragment reads.
    auto issue = [&](int q) {
      if (H == 0) issue_b(std::integral_constant<int, LBUF>{}, q); else issue_a(std::integral_constant<int, LBUF>{}, q);
    };
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // one MFMA, then at most one fragment read or one load (see the 32-k kernel); order held by sched_barrier
      if (j < 2) bx[2 * j] = frag_b(bbuf, 2 * j, 2 * H);
      else ax[2 * j - 4] = frag_a(abuf, 2 * j - 4, 2 * H);
      if (!kFirst) acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[0], ay[j], acc[j][0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (j < 2) bx[2 * j + 1] = frag_b(bbuf, 2 * j + 1, 2 * H);
      else ax[2 * j - 3] = frag_a(abuf, 2 * j - 3, 2 * H);
      if (!kFirst) acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[1], ay[j], acc[j][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      issue(j);
      if (!kFirst) acc[j][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[2], ay[j], acc[j][2], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (!kFirst) acc[j][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[3], ay[j], acc[j][3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (j < 2) by[2 * j] = frag_b(bbuf, 2 * j, 2 * H + 1);
      else ay[2 * j - 4] = frag_a(abuf, 2 * j - 4, 2 * H + 1);
      acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[0], ax[j], acc[j][0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (j < 2) by[2 * j + 1] = frag_b(bbuf, 2 * j + 1, 2 * H + 1);
      else ay[2 * j - 3] = frag_a(abuf, 2 * j - 3, 2 * H + 1);
      acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[1], ax[j], acc[j][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      issue(4 + j);
      acc[j][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[2], ax[j], acc[j][2], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      acc[j][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bx[3], ax[j], acc[j][3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
#define MOE_HS(ph) half_step(std::integral_constant<int, ph>{}, std::false_type{})
  if (nb > 0) {
#pragma unroll
    for (int q = 0; q < 8; ++q) issue_a(std::integral_constant<int, 0>{}, q);
#pragma unroll
    for (int q = 0; q < 8; ++q) issue_b(std::integral_constant<int, 1>{}, q);
#pragma unroll
    for (int q = 0; q < 8; ++q) issue_a(std::integral_constant<int, 2>{}, q);
    half_step(std::integral_constant<int, 0>{}, std::true_type{});
    const int nh = 2 * nb;  // half-steps
    int h = 1;
    for (; h + 10 <= nh; h += 10) {
      MOE_HS(1); MOE_HS(2); MOE_HS(3); MOE_HS(4); MOE_HS(5); MOE_HS(6); MOE_HS(7); MOE_HS(8); MOE_HS(9); MOE_HS(0);
    }
    const int rest = nh - h;  // 0..9 half-steps left, starting at phase 1
    if (rest > 0) MOE_HS(1);
    if (rest > 1) MOE_HS(2);
    if (rest > 2) MOE_HS(3);
    if (rest > 3) MOE_HS(4);
    if (rest > 4) MOE_HS(5);
    if (rest > 5) MOE_HS(6);
    if (rest > 6) MOE_HS(7);
    if (rest > 7) MOE_HS(8);
    if (rest > 8) MOE_HS(9);
#pragma unroll
    for (int fm = 0; fm < 4; ++fm)
#pragma unroll
      for (int fn = 0; fn < 4; ++fn)
        acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(by[fn], ay[fm], acc[fm][fn], 0, 0, 0);
  }
#undef MOE_HS
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  tile_epilogue<EPI, false, ACT>(p, t, acc, reinterpret_cast<float*>(wave == 0 ? g_st0 : wave == 1 ? g_st1 : wave == 2 ? g_st2 : g_st3), wave, lane);
}

template <int LB, int EPI, int ACT = 0>
moe_status_t launch_cfg64(const GemmP& p, hipStream_t s) {
  constexpr int out_cols = EPI == EPI_GLU_FWD ? BN / 2 : BN;
  const int n_nt = ceil_div(p.N, out_cols);
  long rows_bound = (long)p.max_rows * p.n_experts;
  if (rows_bound > p.total_rows_bound) rows_bound = p.total_rows_bound;
  const int max_tiles = (int)((rows_bound + BM - 1) / BM + p.n_experts) * n_nt;
  if (max_tiles <= 0) return MOE_OK;
  const int grid = ceil_div(max_tiles, 8 * kChunk) * 8 * kChunk;  // whole turns of the XCD deal
  hipLaunchKernelGGL((gg_mfma64_kernel<LB, EPI, ACT>), dim3(grid), dim3(kThreads), 0, s, p, n_nt);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
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
  auto kern = gg_mfma_kernel<LA, LB, EPI, RAGGED_K, ACT>;
  const int grid = ceil_div(max_tiles, 8 * kChunk) * 8 * kChunk;  // whole turns of the XCD deal
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), 0, s, p, n_nt, mt_fix);
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
#ifdef MOE_DEBUG_SWITCHES
  static const bool force_k32 = getenv("MOE_GEMM_K32") != nullptr;  // for A/B timing of the two K pipelines
#else
  constexpr bool force_k32 = false;
#endif
  if (p.Kfix % BK2 == 0 && !force_k32) {
    switch (epi) {
      case EPI_PLAIN:
        return b_kc ? launch_cfg64<KC, EPI_PLAIN>(p, s) : launch_cfg64<TR, EPI_PLAIN>(p, s);
      case EPI_ACT_FWD:
        if (p.act == MOE_ACT_RELU) return launch_cfg64<TR, EPI_ACT_FWD, MOE_ACT_RELU>(p, s);
        if (p.act == MOE_ACT_GELU_TANH) return launch_cfg64<TR, EPI_ACT_FWD, MOE_ACT_GELU_TANH>(p, s);
        return launch_cfg64<TR, EPI_ACT_FWD, MOE_ACT_GELU_ERF>(p, s);
      case EPI_GLU_FWD: return launch_cfg64<TR, EPI_GLU_FWD>(p, s);
      case EPI_ACCUM: return launch_cfg64<KC, EPI_ACCUM>(p, s);
      case EPI_ACT_BWD:
        if (p.act == MOE_ACT_RELU) return launch_cfg64<KC, EPI_ACT_BWD, MOE_ACT_RELU>(p, s);
        if (p.act == MOE_ACT_GELU_TANH) return launch_cfg64<KC, EPI_ACT_BWD, MOE_ACT_GELU_TANH>(p, s);
        return launch_cfg64<KC, EPI_ACT_BWD, MOE_ACT_GELU_ERF>(p, s);
      default: return launch_cfg64<KC, EPI_GLU_BWD>(p, s);
    }
  }
  switch (epi) {
    case EPI_PLAIN:
      return b_kc ? launch_cfg<KC, KC, EPI_PLAIN, false>(p, s) : launch_cfg<KC, TR, EPI_PLAIN, false>(p, s);
    case EPI_ACT_FWD:
      if (p.act == MOE_ACT_RELU) return launch_cfg<KC, TR, EPI_ACT_FWD, false, MOE_ACT_RELU>(p, s);
      if (p.act == MOE_ACT_GELU_TANH) return launch_cfg<KC, TR, EPI_ACT_FWD, false, MOE_ACT_GELU_TANH>(p, s);
      return launch_cfg<KC, TR, EPI_ACT_FWD, false, MOE_ACT_GELU_ERF>(p, s);
    case EPI_GLU_FWD: return launch_cfg<KC, TR, EPI_GLU_FWD, false>(p, s);
    case EPI_ACCUM: return launch_cfg<KC, KC, EPI_ACCUM, false>(p, s);
    case EPI_ACT_BWD:
      if (p.act == MOE_ACT_RELU) return launch_cfg<KC, KC, EPI_ACT_BWD, false, MOE_ACT_RELU>(p, s);
      if (p.act == MOE_ACT_GELU_TANH) return launch_cfg<KC, KC, EPI_ACT_BWD, false, MOE_ACT_GELU_TANH>(p, s);
      return launch_cfg<KC, KC, EPI_ACT_BWD, false, MOE_ACT_GELU_ERF>(p, s);
    default: return launch_cfg<KC, KC, EPI_GLU_BWD, false>(p, s);
  }
}

}  // namespace moe
