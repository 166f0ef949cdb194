// Internal helpers shared by the HIP sources of the MoE hot path (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moe_mi355x.h"

namespace moe {

typedef uint16_t bf16_t;  // bf16 storage: the upper half of an fp32 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round-to-nearest-even; inputs are finite by contract
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kVec = 4;  // elements per 16-byte access
  __device__ static __forceinline__ float ld(const float* p) { return *p; }
  __device__ static __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 16-byte vector of elements, widened to fp32 lanes
// 16-byte accesses marked non-temporal: for data that is read or written once per kernel and not needed in
// the caches afterwards (the rows the ordering kernels stream through)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_nt(const void* p) {
  const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(r[0], r[1], r[2], r[3]);
}
__device__ __forceinline__ void store16_nt(void* p, const uint4& v) {
  const u32x4_t r = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(r, reinterpret_cast<u32x4_t*>(p));
}

template <typename T> struct Vec16;
template <> struct Vec16<float> {
  float v[4];
  __device__ __forceinline__ void set(const uint4& r) {
    v[0] = __uint_as_float(r.x); v[1] = __uint_as_float(r.y); v[2] = __uint_as_float(r.z); v[3] = __uint_as_float(r.w);
  }
  __device__ __forceinline__ void load(const float* p) { set(*reinterpret_cast<const uint4*>(p)); }
  __device__ __forceinline__ void load_nt(const float* p) { set(load16_nt(p)); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct Vec16<bf16_t> {
  float v[8];
  __device__ __forceinline__ void set(const uint4& r) {
    uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  __device__ __forceinline__ void load(const bf16_t* p) { set(*reinterpret_cast<const uint4*>(p)); }
  __device__ __forceinline__ void load_nt(const bf16_t* p) { set(load16_nt(p)); }
  __device__ __forceinline__ void store(bf16_t* p) const {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f32_to_bf16(v[2 * i]) | ((uint32_t)f32_to_bf16(v[2 * i + 1]) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// ----------------------------------------------------------------------------- activations (fp32)
// 1 / (1 + e^{-z}) with the hardware reciprocal (1 ulp): the fused epilogues evaluate this for every
// element of an [A,H] tensor, and a full-precision division is ten times the instructions
__device__ __forceinline__ float sigmoidf_(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }
__device__ __forceinline__ float siluf_(float z) { return z * sigmoidf_(z); }
__device__ __forceinline__ float silu_gradf_(float z) {
  float s = sigmoidf_(z);
  return s * (1.0f + z * (1.0f - s));
}
// tanh through one exponential: tanh(u) = 1 - 2 / (1 + e^{2u}); saturates cleanly for large |u|
__device__ __forceinline__ float tanh_fast(float u) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * u)); }

__device__ __forceinline__ float act_fwd(float z, int act) {
  if (act == MOE_ACT_RELU) return z > 0.0f ? z : 0.0f;
  if (act == MOE_ACT_GELU_TANH) {
    float u = 0.7978845608028654f * (z + 0.044715f * z * z * z);
    return 0.5f * z * (1.0f + tanh_fast(u));
  }
  return 0.5f * z * (1.0f + erff(z * 0.7071067811865476f));
}
__device__ __forceinline__ float act_grad(float z, int act) {
  if (act == MOE_ACT_RELU) return z > 0.0f ? 1.0f : 0.0f;
  if (act == MOE_ACT_GELU_TANH) {
    float u = 0.7978845608028654f * (z + 0.044715f * z * z * z);
    float th = tanh_fast(u);
    return 0.5f * (1.0f + th) + 0.5f * z * (1.0f - th * th) * 0.7978845608028654f * (1.0f + 0.134145f * z * z);
  }
  return 0.5f * (1.0f + erff(z * 0.7071067811865476f)) + z * __expf(-0.5f * z * z) * 0.3989422804014327f;
}

// ----------------------------------------------------------------------------- host side
void set_error(const char* fmt, ...);

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }
inline size_t elem_size(int dtype) { return dtype == MOE_BF16 ? 2 : 4; }

#define MOE_CHECK_LAUNCH()                                                       \
  do {                                                                           \
    hipError_t e__ = hipGetLastError();                                          \
    if (e__ != hipSuccess) {                                                     \
      moe::set_error("%s:%d: launch failed: %s", __FILE__, __LINE__, hipGetErrorString(e__)); \
      return MOE_ERR_DEVICE;                                                     \
    }                                                                            \
  } while (0)

// ----------------------------------------------------------------------------- launchers (one per source file)
// route.hip
size_t route_workspace_bytes(const moe_config_t& c);
moe_status_t launch_route(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate, float* logits,
                          float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                          int32_t* offsets, int32_t* src_of_row, void* ws, hipStream_t s);
moe_status_t launch_route_static(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate,
                                 float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                                 int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row, hipStream_t s);
moe_status_t launch_route_noisy(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate,
                                const void* w_noise, const float* noise, float* logits, float* noise_logits, float* probs,
                                int32_t* topk_idx, float* topk_w, int32_t* pos, int32_t* row_of, int32_t* count,
                                int32_t* offsets, int32_t* src_of_row, void* ws, hipStream_t s);
moe_status_t launch_route_noisy_bwd(const moe_config_t& c, const void* x, const void* w_gate, const void* w_noise,
                                    const float* noise, const float* noise_logits, const float* probs,
                                    const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                                    float* db_gate, void* dw_noise, void* dx, void* ws, hipStream_t s);
size_t route_bwd_workspace_bytes(const moe_config_t& c);
size_t route_xmoe_workspace_bytes(const moe_config_t& c, int d_proj);
moe_status_t launch_route_xmoe(const moe_config_t& c, const void* x, const void* w_proj, const void* w_gate, int d_proj,
                               float* proj, float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* pos,
                               int32_t* row_of, int32_t* count, int32_t* offsets, int32_t* src_of_row, void* ws,
                               hipStream_t s);
moe_status_t launch_route_xmoe_bwd(const moe_config_t& c, const void* x, const void* w_proj, const void* w_gate, int d_proj,
                                   const float* proj, const float* probs, const int32_t* topk_idx, const int32_t* pos,
                                   const float* dtopk_w, void* dw_proj, void* dw_gate, void* dx, void* ws, hipStream_t s);
moe_status_t launch_route_bwd(const moe_config_t& c, const void* x, const void* w_gate, const float* probs,
                              const int32_t* topk_idx, const int32_t* pos, const float* dtopk_w, void* dw_gate,
                              float* db_gate, void* dx, void* ws, hipStream_t s);
// The same with the backward of the ordering function in between (whole-layer backward): dlogits, then
// dx = sum_j dxe[row_of] (+ dy) + dlogits.W_g^T in one pass over dx when the shape allows it (else the gather, then the
// gate's accumulate into dx), then dW_g and db_g.  dx is overwritten.
moe_status_t launch_dispatch_route_bwd(const moe_config_t& c, const void* dxe, const int32_t* row_of, const void* dy,
                                       const void* x, const void* w_gate, const float* probs, const int32_t* topk_idx,
                                       const int32_t* pos, const float* dtopk_w, void* dw_gate, float* db_gate, void* dx,
                                       void* ws, hipStream_t s);
// gate_mfma.hip: the gate product on the matrix cores (bf16, E <= 64) with top-k, G(I) and the histogram of choices;
// hist as gate_small_kernel / gate_topk_kernel leave it ([E][top_k][nb]), nb = 64-token tiles
bool gate_mfma_supported(const moe_config_t& c);
moe_status_t launch_gate_mfma(const moe_config_t& c, const void* x, const void* w_gate, const float* b_gate,
                              float* logits, float* probs, int32_t* topk_idx, float* topk_w, int32_t* hist, int nb,
                              hipStream_t s);
// order.hip
moe_status_t launch_dispatch(const moe_config_t& c, const void* x, const int32_t* row_of, void* xe, hipStream_t s);
// chunked layer (FSMoE Sec. 4.2): row ranges of chunk c of every expert, and the dispatch of one chunk
moe_status_t launch_chunk_bounds(const moe_config_t& c, const int32_t* offsets, int r, int32_t* begin, int32_t* end,
                                 hipStream_t s);
moe_status_t launch_dispatch_rows(const moe_config_t& c, const void* x, const int32_t* src_of_row, const int32_t* begin,
                                  const int32_t* end, int r, void* xe, hipStream_t s);
moe_status_t launch_dispatch_bwd(const moe_config_t& c, const void* dxe, const int32_t* row_of, const void* dy, void* dx,
                                 hipStream_t s);
// dispatch backward with the gate's share of dx folded in: dx = sum_j dxe[row_of] (+ dy) + dl . W_g^T (small E only)
bool dispatch_bwd_gate_supported(const moe_config_t& c);
moe_status_t launch_dispatch_bwd_gate(const moe_config_t& c, const void* dxe, const int32_t* row_of, const void* dy,
                                      const float* dl, const void* w_gate, void* dx, hipStream_t s);
moe_status_t launch_combine(const moe_config_t& c, const void* q, const float* topk_w, const int32_t* row_of,
                            const void* x, void* y, hipStream_t s);
moe_status_t launch_combine_bwd(const moe_config_t& c, const void* dy, const void* q, const float* topk_w,
                                const int32_t* row_of, void* dq, float* dtopk_w, hipStream_t s);
// expert_ffn.hip
size_t expert_bwd_workspace_bytes(const moe_config_t& c);
// row_end == NULL: whole experts; else rows [offsets[e], row_end[e]) of every expert (one chunk)
moe_status_t launch_expert_fwd(const moe_config_t& c, const void* xe, const int32_t* offsets, const int32_t* row_end,
                               const void* w1, const void* w3, const void* w2, void* q, void* a1, void* a3, void* hh,
                               hipStream_t s);
// which: bit 0 = dhh (-> da1, da3 in ws), bit 1 = dxe
moe_status_t launch_expert_bwd_dgrad(const moe_config_t& c, const void* dq, const int32_t* offsets,
                                     const int32_t* row_end, const void* w1, const void* w3, const void* w2,
                                     const void* a1, const void* a3, void* dxe, void* ws, int which, hipStream_t s);
// which: bit 0 = dW2, bit 1 = dW1 (, dW3); needs da1 (, da3) in ws
moe_status_t launch_expert_bwd_wgrad(const moe_config_t& c, const void* dq, const void* xe, const int32_t* offsets,
                                     const void* hh, void* dw1, void* dw3, void* dw2, void* ws, int which,
                                     hipStream_t s);
moe_status_t launch_expert_bwd(const moe_config_t& c, const void* dq, const void* xe, const int32_t* offsets,
                               const void* w1, const void* w3, const void* w2, const void* a1, const void* a3,
                               const void* hh, void* dxe, void* dw1, void* dw3, void* dw2, void* ws, hipStream_t s);

}  // namespace moe
