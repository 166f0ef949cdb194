// Ordering and I-ordering functions of the MoE layer (FSMoE Sec. 2.1) and their backward passes.
//
// All four kernels are HBM-bound row movers.  They walk TOKENS, not expert rows: a token's row is
// read once and fanned out to (or gathered from) its k expert rows, so the traffic is the
// algorithmic minimum  N*M*b + A*M*b.  Rows move as 16-byte vectors; a row is covered by a group
// of `tpr` consecutive lanes (a power of two), so one wave touches whole contiguous rows.
// Which accesses are marked non-temporal was chosen by timing each kernel inside the layer (the cache state
// its neighbours leave matters): the stores of the ordering function, the loads of the three gathers.
#include "common.h"

namespace moe {
namespace {

constexpr int kBlock = 256;
constexpr int kMaxK = 8;

struct RowMap {
  int tpr;  // threads per row (power of two, <= kBlock)
  int rpb;  // rows per block
};

inline RowMap row_map(int chunks_per_row) {
  int tpr = 1;
  while (tpr < chunks_per_row && tpr < kBlock) tpr <<= 1;
  return RowMap{tpr, kBlock / tpr};
}

// xe[row_of[t,j], :] = x[t, :]
template <typename T>
__global__ __launch_bounds__(kBlock) void dispatch_kernel(const T* __restrict__ x, const int32_t* __restrict__ row_of,
                                                          T* __restrict__ xe, int n_tokens, int d_model, int top_k,
                                                          int tpr) {
  constexpr int V = Elem<T>::kVec;
  const int rpb = kBlock / tpr;
  const int t = blockIdx.x * rpb + threadIdx.x / tpr;
  if (t >= n_tokens) return;
  const int lane = threadIdx.x % tpr;
  const int chunks = d_model / V;
  int rows[kMaxK];
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) rows[j] = j < top_k ? row_of[(size_t)t * top_k + j] : -1;
  const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)t * d_model);
  for (int c = lane; c < chunks; c += tpr) {
    uint4 v = src[c];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j)
      if (rows[j] >= 0) store16_nt(reinterpret_cast<uint4*>(xe + (size_t)rows[j] * d_model) + c, v);
  }
}

// One chunk of the ordering function, expert rows [begin[e], end[e]) of every expert e (blockIdx.y):
// xe[row, :] = x[src_of_row[row] / top_k, :].  Walks expert rows, so x is read once per kept assignment.
template <typename T>
__global__ __launch_bounds__(kBlock) void dispatch_rows_kernel(const T* __restrict__ x, const int32_t* __restrict__ src_of_row,
                                                               const int32_t* __restrict__ begin,
                                                               const int32_t* __restrict__ end, T* __restrict__ xe,
                                                               int d_model, int top_k, int tpr) {
  constexpr int V = Elem<T>::kVec;
  const int rpb = kBlock / tpr;
  const int row = begin[blockIdx.y] + blockIdx.x * rpb + threadIdx.x / tpr;
  if (row >= end[blockIdx.y]) return;
  const int lane = threadIdx.x % tpr;
  const int chunks = d_model / V;
  const int t = src_of_row[row] / top_k;
  const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)t * d_model);
  uint4* dst = reinterpret_cast<uint4*>(xe + (size_t)row * d_model);
  for (int c = lane; c < chunks; c += tpr) dst[c] = src[c];
}

// Chunk c of r of expert e holds its rows floor(c n / r) .. floor((c + 1) n / r) - 1, n = rows of the expert
// (FSMoE Sec. 4.2: the capacity dimension is cut into r parts).  begin, end: [r][E].
__global__ void chunk_bounds_kernel(const int32_t* __restrict__ offsets, int n_experts, int r,
                                    int32_t* __restrict__ begin, int32_t* __restrict__ end) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= r * n_experts) return;
  const int c = i / n_experts, e = i % n_experts;
  const long n = offsets[e + 1] - offsets[e];
  begin[i] = offsets[e] + (int)(c * n / r);
  end[i] = offsets[e] + (int)((c + 1) * n / r);
}

// out[t,:] = sum_j scale_j * src[row_of[t,j], :] (+ res[t,:]);  scale_j = w[t,j] or 1
template <typename T, bool kWeighted>
__global__ __launch_bounds__(kBlock) void gather_sum_kernel(const T* __restrict__ src, const float* __restrict__ w,
                                                            const int32_t* __restrict__ row_of,
                                                            const T* __restrict__ res, T* __restrict__ out,
                                                            int n_tokens, int d_model, int top_k, int tpr) {
  constexpr int V = Elem<T>::kVec;
  const int rpb = kBlock / tpr;
  const int t = blockIdx.x * rpb + threadIdx.x / tpr;
  if (t >= n_tokens) return;
  const int lane = threadIdx.x % tpr;
  const int chunks = d_model / V;
  int rows[kMaxK];
  float sc[kMaxK];
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    rows[j] = j < top_k ? row_of[(size_t)t * top_k + j] : -1;
    sc[j] = (kWeighted && j < top_k) ? w[(size_t)t * top_k + j] : 1.0f;
  }
  for (int c = lane; c < chunks; c += tpr) {
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
      if (rows[j] >= 0) {
        Vec16<T> v;
        v.load_nt(src + (size_t)rows[j] * d_model + c * V);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = kWeighted ? fmaf(sc[j], v.v[i], acc[i]) : acc[i] + v.v[i];
      }
    }
    if (res != nullptr) {
      Vec16<T> r;
      r.load_nt(res + (size_t)t * d_model + c * V);
#pragma unroll
      for (int i = 0; i < V; ++i) acc[i] += r.v[i];
    }
    Vec16<T> o;
#pragma unroll
    for (int i = 0; i < V; ++i) o.v[i] = acc[i];
    o.store(out + (size_t)t * d_model + c * V);
  }
}

// Backward of the ordering function with the gate's share of dx folded in (FSMoE Sec. 4.4):
//   dx[t,:] = sum_j dxe[row_of[t,j], :] (+ dy[t,:]) + dlogits[t,:] . W_g^T
// so that dx is written once instead of being written by the gather and read and written again by the gate's backward.
// A lane owns the same CH 16-byte column chunks for every token it meets and keeps the W_g rows of those columns in
// registers (CH x V x GE fp32 values, experts past E zero); a workgroup walks token groups in a grid-stride loop.
template <typename T, int CH, int GE>
__global__ __launch_bounds__(kBlock) void gather_gate_kernel(const T* __restrict__ src, const int32_t* __restrict__ row_of,
                                                             const T* __restrict__ res, const float* __restrict__ dl,
                                                             const T* __restrict__ w_gate, T* __restrict__ out,
                                                             int n_tokens, int d_model, int n_experts, int top_k, int tpr) {
  constexpr int V = Elem<T>::kVec;
  const int rpb = kBlock / tpr;
  const int lane = threadIdx.x % tpr, sub = threadIdx.x / tpr;
  const int chunks = d_model / V;
  float wreg[CH][V][GE];
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    const int c = lane + ch * tpr;
#pragma unroll
    for (int i = 0; i < V; ++i)
#pragma unroll
      for (int e = 0; e < GE; ++e)
        wreg[ch][i][e] = (c < chunks && e < n_experts) ? Elem<T>::ld(w_gate + (size_t)(c * V + i) * n_experts + e) : 0.0f;
  }
  const int groups = (n_tokens + rpb - 1) / rpb;
  for (int tb = blockIdx.x; tb < groups; tb += gridDim.x) {
    const int t = tb * rpb + sub;
    if (t >= n_tokens) continue;
    int rows[kMaxK];
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) rows[j] = j < top_k ? row_of[(size_t)t * top_k + j] : -1;
    float dlv[GE];
#pragma unroll
    for (int e = 0; e < GE; ++e) dlv[e] = e < n_experts ? dl[(size_t)t * n_experts + e] : 0.0f;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int c = lane + ch * tpr;
      if (c >= chunks) break;
      float acc[V];
#pragma unroll
      for (int i = 0; i < V; ++i) acc[i] = 0.0f;
#pragma unroll
      for (int j = 0; j < kMaxK; ++j) {
        if (rows[j] >= 0) {
          Vec16<T> v;
          v.load_nt(src + (size_t)rows[j] * d_model + c * V);
#pragma unroll
          for (int i = 0; i < V; ++i) acc[i] += v.v[i];
        }
      }
      if (res != nullptr) {
        Vec16<T> r;
        r.load_nt(res + (size_t)t * d_model + c * V);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += r.v[i];
      }
#pragma unroll
      for (int e = 0; e < GE; ++e)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = fmaf(dlv[e], wreg[ch][i][e], acc[i]);
      Vec16<T> o;
#pragma unroll
      for (int i = 0; i < V; ++i) o.v[i] = acc[i];
      o.store(out + (size_t)t * d_model + c * V);
    }
  }
}

// dq[row_of[t,j], :] = w[t,j] * dy[t, :];  dtopk_w[t,j] = <dy[t,:], q[row_of[t,j],:]>
template <typename T>
__global__ __launch_bounds__(kBlock) void combine_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ q,
                                                             const float* __restrict__ w,
                                                             const int32_t* __restrict__ row_of, T* __restrict__ dq,
                                                             float* __restrict__ dtopk_w, int n_tokens, int d_model,
                                                             int top_k, int tpr) {
  constexpr int V = Elem<T>::kVec;
  __shared__ float red[kMaxK][kBlock / 64];
  const int rpb = kBlock / tpr;
  const int t = blockIdx.x * rpb + threadIdx.x / tpr;
  const bool live = t < n_tokens;
  const int lane = threadIdx.x % tpr;
  const int chunks = d_model / V;
  int rows[kMaxK];
  float sc[kMaxK], dot[kMaxK];
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    rows[j] = (live && j < top_k) ? row_of[(size_t)t * top_k + j] : -1;
    sc[j] = (live && j < top_k) ? w[(size_t)t * top_k + j] : 0.0f;
    dot[j] = 0.0f;
  }
  if (live) {
    for (int c = lane; c < chunks; c += tpr) {
      Vec16<T> g;
      g.load_nt(dy + (size_t)t * d_model + c * V);
#pragma unroll
      for (int j = 0; j < kMaxK; ++j) {
        if (rows[j] >= 0) {
          Vec16<T> qv, o;
          qv.load_nt(q + (size_t)rows[j] * d_model + c * V);
#pragma unroll
          for (int i = 0; i < V; ++i) {
            dot[j] = fmaf(g.v[i], qv.v[i], dot[j]);
            o.v[i] = sc[j] * g.v[i];
          }
          o.store(dq + (size_t)rows[j] * d_model + c * V);
        }
      }
    }
  }
  // reduce the partial dots over the tpr lanes of the row: butterflies inside a wave, LDS across waves
  const int in_wave = tpr < 64 ? tpr : 64;
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    if (j < top_k) {
      float v = dot[j];
      for (int o = in_wave >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      dot[j] = v;
    }
  }
  if (tpr > 64) {  // a row spans tpr / 64 waves: sum their partials in wave order
    const int wave = threadIdx.x >> 6;
    const int wpr = tpr >> 6;
    if ((threadIdx.x & 63) == 0)
      for (int j = 0; j < top_k; ++j) red[j][wave] = dot[j];
    __syncthreads();
    if (lane < top_k && live) {
      const int first = (threadIdx.x / tpr) * wpr;
      float v = 0.0f;
      for (int wv = 0; wv < wpr; ++wv) v += red[lane][first + wv];
      dtopk_w[(size_t)t * top_k + lane] = v;  // dropped choices never accumulated: 0
    }
  } else if (live && lane == 0) {
#pragma unroll
    for (int j = 0; j < kMaxK; ++j)
      if (j < top_k) dtopk_w[(size_t)t * top_k + j] = dot[j];
  }
}

template <typename T>
moe_status_t dispatch_t(const moe_config_t& c, const void* x, const int32_t* row_of, void* xe, hipStream_t s) {
  RowMap m = row_map(c.d_model / Elem<T>::kVec);
  hipLaunchKernelGGL(dispatch_kernel<T>, dim3(ceil_div(c.n_tokens, m.rpb)), dim3(kBlock), 0, s, (const T*)x, row_of,
                     (T*)xe, c.n_tokens, c.d_model, c.top_k, m.tpr);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

template <typename T, bool kWeighted>
moe_status_t gather_t(const moe_config_t& c, const void* src, const float* w, const int32_t* row_of, const void* res,
                      void* out, hipStream_t s) {
  RowMap m = row_map(c.d_model / Elem<T>::kVec);
  hipLaunchKernelGGL((gather_sum_kernel<T, kWeighted>), dim3(ceil_div(c.n_tokens, m.rpb)), dim3(kBlock), 0, s,
                     (const T*)src, w, row_of, (const T*)res, (T*)out, c.n_tokens, c.d_model, c.top_k, m.tpr);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

template <typename T>
moe_status_t combine_bwd_t(const moe_config_t& c, const void* dy, const void* q, const float* w, const int32_t* row_of,
                           void* dq, float* dtopk_w, hipStream_t s) {
  RowMap m = row_map(c.d_model / Elem<T>::kVec);
  hipLaunchKernelGGL(combine_bwd_kernel<T>, dim3(ceil_div(c.n_tokens, m.rpb)), dim3(kBlock), 0, s, (const T*)dy,
                     (const T*)q, w, row_of, (T*)dq, dtopk_w, c.n_tokens, c.d_model, c.top_k, m.tpr);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

}  // namespace

moe_status_t launch_dispatch(const moe_config_t& c, const void* x, const int32_t* row_of, void* xe, hipStream_t s) {
  return c.dtype == MOE_BF16 ? dispatch_t<bf16_t>(c, x, row_of, xe, s) : dispatch_t<float>(c, x, row_of, xe, s);
}

moe_status_t launch_chunk_bounds(const moe_config_t& c, const int32_t* offsets, int r, int32_t* begin, int32_t* end,
                                 hipStream_t s) {
  const int n = r * c.n_experts;
  hipLaunchKernelGGL(chunk_bounds_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, s, offsets, c.n_experts, r, begin, end);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

moe_status_t launch_dispatch_rows(const moe_config_t& c, const void* x, const int32_t* src_of_row, const int32_t* begin,
                                  const int32_t* end, int r, void* xe, hipStream_t s) {
  const bool bf16 = c.dtype == MOE_BF16;
  const RowMap m = row_map(c.d_model / (bf16 ? 8 : 4));
  // an expert is chosen at most once per token and holds at most the capacity: a chunk has at most ceil(that / r) rows
  long rows = c.n_tokens;
  if (c.capacity > 0 && c.capacity < rows) rows = c.capacity;
  const int per_chunk = (int)((rows + r - 1) / r);
  const dim3 grid(ceil_div(per_chunk, m.rpb), c.n_experts);
  if (bf16)
    hipLaunchKernelGGL(dispatch_rows_kernel<bf16_t>, grid, dim3(kBlock), 0, s, static_cast<const bf16_t*>(x), src_of_row,
                       begin, end, static_cast<bf16_t*>(xe), c.d_model, c.top_k, m.tpr);
  else
    hipLaunchKernelGGL(dispatch_rows_kernel<float>, grid, dim3(kBlock), 0, s, static_cast<const float*>(x), src_of_row,
                       begin, end, static_cast<float*>(xe), c.d_model, c.top_k, m.tpr);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}

moe_status_t launch_dispatch_bwd(const moe_config_t& c, const void* dxe, const int32_t* row_of, const void* dy, void* dx,
                                 hipStream_t s) {
  const void* res = c.add_residual ? dy : nullptr;
  return c.dtype == MOE_BF16 ? gather_t<bf16_t, false>(c, dxe, nullptr, row_of, res, dx, s)
                             : gather_t<float, false>(c, dxe, nullptr, row_of, res, dx, s);
}

// The fused form needs the W_g rows of a lane's chunks in registers: CH chunks per lane x GE experts <= 16.
namespace {
struct GateFold { int ch, ge; };
bool gate_fold_plan(const moe_config_t& c, GateFold* g) {
  const RowMap m = row_map(c.d_model / (c.dtype == MOE_BF16 ? 8 : 4));
  const int chunks = c.d_model / (c.dtype == MOE_BF16 ? 8 : 4);
  const int ch = ceil_div(chunks, m.tpr);
  const int ge = c.n_experts <= 8 ? 8 : 16;
  if (c.n_experts > 16 || ch > 2 || ch * ge > 16) return false;
  g->ch = ch; g->ge = ge;
  return true;
}
template <typename T, int CH, int GE>
moe_status_t gather_gate_t(const moe_config_t& c, const void* dxe, const int32_t* row_of, const void* res, const float* dl,
                           const void* w_gate, void* dx, hipStream_t s) {
  const RowMap m = row_map(c.d_model / Elem<T>::kVec);
  const int groups = ceil_div(c.n_tokens, m.rpb);
  const int grid = groups < 1024 ? groups : 1024;  // four workgroups per compute unit walk the token groups
  hipLaunchKernelGGL((gather_gate_kernel<T, CH, GE>), dim3(grid), dim3(kBlock), 0, s, (const T*)dxe, row_of, (const T*)res,
                     dl, (const T*)w_gate, (T*)dx, c.n_tokens, c.d_model, c.n_experts, c.top_k, m.tpr);
  MOE_CHECK_LAUNCH();
  return MOE_OK;
}
}  // namespace

bool dispatch_bwd_gate_supported(const moe_config_t& c) {
  GateFold g;
  return gate_fold_plan(c, &g);
}

moe_status_t launch_dispatch_bwd_gate(const moe_config_t& c, const void* dxe, const int32_t* row_of, const void* dy,
                                      const float* dl, const void* w_gate, void* dx, hipStream_t s) {
  GateFold g;
  if (!gate_fold_plan(c, &g)) {
    set_error("dispatch backward with the gate folded in: shape not supported");
    return MOE_ERR_UNSUPPORTED;
  }
  const void* res = c.add_residual ? dy : nullptr;
  const bool bf = c.dtype == MOE_BF16;
  if (g.ch == 1 && g.ge == 8)
    return bf ? gather_gate_t<bf16_t, 1, 8>(c, dxe, row_of, res, dl, w_gate, dx, s)
              : gather_gate_t<float, 1, 8>(c, dxe, row_of, res, dl, w_gate, dx, s);
  if (g.ch == 1)
    return bf ? gather_gate_t<bf16_t, 1, 16>(c, dxe, row_of, res, dl, w_gate, dx, s)
              : gather_gate_t<float, 1, 16>(c, dxe, row_of, res, dl, w_gate, dx, s);
  return bf ? gather_gate_t<bf16_t, 2, 8>(c, dxe, row_of, res, dl, w_gate, dx, s)
            : gather_gate_t<float, 2, 8>(c, dxe, row_of, res, dl, w_gate, dx, s);
}

moe_status_t launch_combine(const moe_config_t& c, const void* q, const float* topk_w, const int32_t* row_of,
                            const void* x, void* y, hipStream_t s) {
  const void* res = c.add_residual ? x : nullptr;
  return c.dtype == MOE_BF16 ? gather_t<bf16_t, true>(c, q, topk_w, row_of, res, y, s)
                             : gather_t<float, true>(c, q, topk_w, row_of, res, y, s);
}

moe_status_t launch_combine_bwd(const moe_config_t& c, const void* dy, const void* q, const float* topk_w,
                                const int32_t* row_of, void* dq, float* dtopk_w, hipStream_t s) {
  return c.dtype == MOE_BF16 ? combine_bwd_t<bf16_t>(c, dy, q, topk_w, row_of, dq, dtopk_w, s)
                             : combine_bwd_t<float>(c, dy, q, topk_w, row_of, dq, dtopk_w, s);
}

}  // namespace moe
