// Tensor importance reduction (Eq. 2) and the masked optimizer update (Section 8), both driven
// by a device table of tensor chunks so that one launch covers every tensor of the model.
//
// importance: I_k = sum_i g_i * (w_snapshot_i - w_i).  Stage 1: one 256-thread workgroup per
// chunk of at most SEG_ELEMS elements; every thread streams 16-byte loads of g, w and w_snapshot
// (coalesced across the wave), keeps four fp32 partial sums, then the workgroup combines them in
// double precision with cross-lane shuffles inside each 64-lane wave and a 4-entry LDS exchange.
// Stage 2: one thread per tensor adds that tensor's chunk sums in ascending order.  No atomics:
// the result is bit-reproducible.
//
// update: one workgroup per chunk; a chunk whose tensor is not in the selection bit set returns
// at once, so unselected weights and optimizer state are neither read nor written.
#include "kernels.h"

namespace et {
namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// METRIC 0: Eq. 2, g * (w_snap - w);  1: |w| (weight magnitude);  2: |g| (gradient magnitude) -- the two
// non-additive metrics of the ablation in Section 8 go through the same segmented reduction
template <int METRIC>
__device__ __forceinline__ float metric_term(float g, float w, float ws) {
  return METRIC == 0 ? g * (ws - w) : (METRIC == 1 ? fabsf(w) : fabsf(g));
}

template <bool BF16W, int METRIC>
__global__ __launch_bounds__(256) void importance_stage1(const TensorSeg* __restrict__ segs,
                                                         double* __restrict__ partial) {
  __shared__ double red[4];
  const TensorSeg sg = segs[blockIdx.x];
  const float* __restrict__ g = sg.g;
  const uint32_t n = sg.n;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (BF16W) {
    const bf16* __restrict__ w = (const bf16*)sg.w;
    const bf16* __restrict__ ws = (const bf16*)sg.w_snap;
    const bool vec = (((uintptr_t)g | (uintptr_t)w | (uintptr_t)ws) & 15) == 0;
    const uint32_t n8 = vec ? n / 8 : 0;
    for (uint32_t i = threadIdx.x; i < n8; i += 256) {
      const float4 g0 = ((const float4*)g)[2 * i], g1 = ((const float4*)g)[2 * i + 1];
      const bf16x8 wv = ((const bf16x8*)w)[i];
      bf16x8 sv = wv;
      if (METRIC == 0) sv = ((const bf16x8*)ws)[i];
      a0 += metric_term<METRIC>(g0.x, (float)wv[0], (float)sv[0]) + metric_term<METRIC>(g0.y, (float)wv[1], (float)sv[1]);
      a1 += metric_term<METRIC>(g0.z, (float)wv[2], (float)sv[2]) + metric_term<METRIC>(g0.w, (float)wv[3], (float)sv[3]);
      a2 += metric_term<METRIC>(g1.x, (float)wv[4], (float)sv[4]) + metric_term<METRIC>(g1.y, (float)wv[5], (float)sv[5]);
      a3 += metric_term<METRIC>(g1.z, (float)wv[6], (float)sv[6]) + metric_term<METRIC>(g1.w, (float)wv[7], (float)sv[7]);
    }
    for (uint32_t i = n8 * 8 + threadIdx.x; i < n; i += 256)
      a0 += metric_term<METRIC>(g[i], (float)w[i], METRIC == 0 ? (float)ws[i] : 0.f);
  } else {
    const float* __restrict__ w = (const float*)sg.w;
    const float* __restrict__ ws = (const float*)sg.w_snap;
    const bool vec = (((uintptr_t)g | (uintptr_t)w | (uintptr_t)ws) & 15) == 0;
    const uint32_t n4 = vec ? n / 4 : 0;
    for (uint32_t i = threadIdx.x; i < n4; i += 256) {
      const float4 gv = ((const float4*)g)[i], wv = ((const float4*)w)[i];
      float4 sv = wv;
      if (METRIC == 0) sv = ((const float4*)ws)[i];
      a0 += metric_term<METRIC>(gv.x, wv.x, sv.x);
      a1 += metric_term<METRIC>(gv.y, wv.y, sv.y);
      a2 += metric_term<METRIC>(gv.z, wv.z, sv.z);
      a3 += metric_term<METRIC>(gv.w, wv.w, sv.w);
    }
    for (uint32_t i = n4 * 4 + threadIdx.x; i < n; i += 256) a0 += metric_term<METRIC>(g[i], w[i], METRIC == 0 ? ws[i] : 0.f);
  }
  double s = wave_sum_d(((double)a0 + (double)a1) + ((double)a2 + (double)a3));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ void importance_stage2(const double* __restrict__ partial, const uint32_t* __restrict__ seg_begin,
                                  int n_tensors, double* __restrict__ out) {
  // one wave per tensor: lane l adds the chunks l, l+64, ... in order, then a fixed butterfly
  const int k = blockIdx.x;
  if (k >= n_tensors) return;
  double s = 0.0;
  for (uint32_t i = seg_begin[k] + threadIdx.x; i < seg_begin[k + 1]; i += 64) s += partial[i];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (threadIdx.x == 0) out[k] = s;
}

template <bool BF16W>
__global__ __launch_bounds__(256) void masked_update_kernel(const UpdateSeg* __restrict__ segs, SelectionBits sel,
                                                            OptParams p) {
  const UpdateSeg sg = segs[blockIdx.x];
  if (!((sel.bits[sg.tensor >> 6] >> (sg.tensor & 63)) & 1ull)) return;
  const float* __restrict__ g = sg.g;
  float* __restrict__ m = sg.m;
  float* __restrict__ v = sg.v;
  float* __restrict__ wf = BF16W ? sg.master : (float*)sg.w;
  bf16* __restrict__ wb = (bf16*)sg.w;
  // one element: returns the new weight, updates the moments in place (unless dry)
  auto one = [&](float gi, float w_old, float& mi, float& vi) -> float {
    if (p.kind == 0) {
      const float m_new = p.beta1 * mi + (1.f - p.beta1) * gi;
      const float v_new = p.beta2 * vi + (1.f - p.beta2) * gi * gi;
      const float w = w_old - p.lr * (m_new / p.bc1) / (sqrtf(v_new / p.bc2) + p.eps);
      if (!p.dry) { mi = m_new; vi = v_new; }
      return w;
    }
    const float m_new = p.momentum * mi + gi;
    const float w = w_old - p.lr * m_new - p.lr * p.wd * w_old;
    if (!p.dry) mi = m_new;
    return w;
  };
  // chunks start at multiples of 16 384 elements of 256-byte aligned tensors: 16-byte vectors of 4 elements
  const uint32_t n4 = sg.n >> 2;
  for (uint32_t i = threadIdx.x; i < n4; i += 256) {
    const float4 g4 = ((const float4*)g)[i];
    float4 w4 = ((const float4*)wf)[i];
    float4 m4 = ((const float4*)m)[i];
    float4 v4 = p.kind == 0 ? ((const float4*)v)[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 w_old = w4;
    w4.x = one(g4.x, w4.x, m4.x, v4.x);
    w4.y = one(g4.y, w4.y, m4.y, v4.y);
    w4.z = one(g4.z, w4.z, m4.z, v4.z);
    w4.w = one(g4.w, w4.w, m4.w, v4.w);
    // a dry run (profiling) moves the same bytes and leaves every value as it was
    ((float4*)m)[i] = m4;
    if (p.kind == 0) ((float4*)v)[i] = v4;
    ((float4*)wf)[i] = p.dry ? w_old : w4;
    if (BF16W) {
      typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
      bf16x4 o;
      if (p.dry) {
        o = ((const bf16x4*)wb)[i];
      } else {
        o[0] = (bf16)w4.x; o[1] = (bf16)w4.y; o[2] = (bf16)w4.z; o[3] = (bf16)w4.w;
      }
      ((bf16x4*)wb)[i] = o;
    }
  }
  for (uint32_t i = (n4 << 2) + threadIdx.x; i < sg.n; i += 256) {   // at most three elements
    float mi = m[i], vi = p.kind == 0 ? v[i] : 0.f;
    const float w_old = wf[i];
    const float w = one(g[i], w_old, mi, vi);
    m[i] = mi;
    if (p.kind == 0) v[i] = vi;
    wf[i] = p.dry ? w_old : w;
    if (BF16W) wb[i] = p.dry ? wb[i] : (bf16)w;
  }
}

}  // namespace

hipError_t importance_reduce(const TensorSeg* segs_dev, int n_segs, const uint32_t* seg_begin_dev, int n_tensors,
                             bool bf16_weights, double* partial_dev, double* out_dev, hipStream_t s, int metric) {
  if (n_segs <= 0 || n_tensors <= 0 || metric < 0 || metric > 2) return hipErrorInvalidValue;
#define ET_IMP(B, M) hipLaunchKernelGGL((importance_stage1<B, M>), dim3(n_segs), dim3(256), 0, s, segs_dev, partial_dev)
  if (bf16_weights) {
    if (metric == 0) ET_IMP(true, 0); else if (metric == 1) ET_IMP(true, 1); else ET_IMP(true, 2);
  } else {
    if (metric == 0) ET_IMP(false, 0); else if (metric == 1) ET_IMP(false, 1); else ET_IMP(false, 2);
  }
#undef ET_IMP
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(importance_stage2, dim3(n_tensors), dim3(64), 0, s, partial_dev, seg_begin_dev,
                     n_tensors, out_dev);
  return hipGetLastError();
}

hipError_t masked_update(const UpdateSeg* segs_dev, int n_segs, bool bf16_weights, const SelectionBits& sel,
                         OptParams p, hipStream_t s) {
  if (n_segs <= 0) return hipErrorInvalidValue;
  if (bf16_weights)
    hipLaunchKernelGGL((masked_update_kernel<true>), dim3(n_segs), dim3(256), 0, s, segs_dev, sel, p);
  else
    hipLaunchKernelGGL((masked_update_kernel<false>), dim3(n_segs), dim3(256), 0, s, segs_dev, sel, p);
  return hipGetLastError();
}

}  // namespace et
