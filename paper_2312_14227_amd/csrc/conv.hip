// HBM-bound kernels of the convolutional workload (Section 5: every convolution weight, folded
// BatchNorm gain and shift is one tensor of the chain).  Activations are NHWC bf16, so a
// convolution is a matrix product over the rows of an im2col matrix [B*Ho*Wo][k*k*C] (column
// order ky, kx, c — the order of the weights [out][ky][kx][c]); everything here moves 16-byte
// vectors of 8 channels.  All sums have a fixed order.
#include "kernels.h"

namespace et {
namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int j = 0; j < 8; j++) z[j] = (bf16)0.f;
  return z;
}

// ---------------------------------------------------------------------------------------------
// im2col, channels a multiple of 8: one thread per (row, tap, 8 channels)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void im2col_vec_kernel(const bf16* __restrict__ x, bf16* __restrict__ cols,
                                                         ConvGeom g, long long total) {
  const int c8n = g.C >> 3, taps = g.k * g.k;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int c8 = (int)(i % c8n);
    const long long r = i / c8n;
    const int t = (int)(r % taps);
    const long long m = r / taps;
    const int ow = (int)(m % g.Wo), oh = (int)((m / g.Wo) % g.Ho), b = (int)(m / ((long long)g.Wo * g.Ho));
    const int h = oh * g.stride - g.pad + t / g.k, w = ow * g.stride - g.pad + t % g.k;
    bf16x8 v = zero8();
    if (h >= 0 && h < g.H && w >= 0 && w < g.W)
      v = *(const bf16x8*)(x + (((long long)b * g.H + h) * g.W + w) * g.C + c8 * 8);
    *(bf16x8*)(cols + m * g.Kc + (long long)t * g.C + c8 * 8) = v;
  }
}

// any channel count (the 3-channel stem): one thread per 8 consecutive columns, scalar gathers;
// columns from k*k*C up to Kc are zero
__global__ __launch_bounds__(256) void im2col_any_kernel(const bf16* __restrict__ x, bf16* __restrict__ cols,
                                                         ConvGeom g, long long total) {
  const int k8n = g.Kc >> 3, K = g.k * g.k * g.C;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int j8 = (int)(i % k8n);
    const long long m = i / k8n;
    const int ow = (int)(m % g.Wo), oh = (int)((m / g.Wo) % g.Ho), b = (int)(m / ((long long)g.Wo * g.Ho));
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const int col = j8 * 8 + e;
      bf16 val = (bf16)0.f;
      if (col < K) {
        const int t = col / g.C, ch = col % g.C;
        const int h = oh * g.stride - g.pad + t / g.k, w = ow * g.stride - g.pad + t % g.k;
        if (h >= 0 && h < g.H && w >= 0 && w < g.W) val = x[(((long long)b * g.H + h) * g.W + w) * g.C + ch];
      }
      v[e] = val;
    }
    *(bf16x8*)(cols + m * g.Kc + j8 * 8) = v;
  }
}

// ---------------------------------------------------------------------------------------------
// adjoint of im2col in gather form: every input pixel adds the (at most k*k) column entries that
// were copied from it, taps in ascending order; then out = (sum + add) * (mask > 0)
// ---------------------------------------------------------------------------------------------
// The column matrix is float32 for kernels larger than 1x1 (the taps are summed before the one
// rounding of the input gradient) and bf16 for a strided 1x1 convolution (a pure scatter).
template <typename TC>
__global__ __launch_bounds__(256) void col2im_kernel(const TC* __restrict__ dcols, const bf16* __restrict__ add,
                                                     const bf16* __restrict__ mask, bf16* __restrict__ out, ConvGeom g,
                                                     long long total) {
  const int c8n = g.C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int c8 = (int)(i % c8n);
    const long long pix = i / c8n;
    const int w = (int)(pix % g.W), h = (int)((pix / g.W) % g.H), b = (int)(pix / ((long long)g.W * g.H));
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; j++) acc[j] = 0.f;
    for (int ky = 0; ky < g.k; ky++) {
      const int hh = h + g.pad - ky;
      if (hh < 0 || hh % g.stride) continue;
      const int oh = hh / g.stride;
      if (oh >= g.Ho) continue;
      for (int kx = 0; kx < g.k; kx++) {
        const int ww = w + g.pad - kx;
        if (ww < 0 || ww % g.stride) continue;
        const int ow = ww / g.stride;
        if (ow >= g.Wo) continue;
        const TC* src = dcols + (((long long)b * g.Ho + oh) * g.Wo + ow) * g.Kc + (long long)(ky * g.k + kx) * g.C + c8 * 8;
        if constexpr (sizeof(TC) == 4) {
          const float4 v0 = *(const float4*)src, v1 = *(const float4*)(src + 4);
          acc[0] += v0.x; acc[1] += v0.y; acc[2] += v0.z; acc[3] += v0.w;
          acc[4] += v1.x; acc[5] += v1.y; acc[6] += v1.z; acc[7] += v1.w;
        } else {
          const bf16x8 v = *(const bf16x8*)src;
#pragma unroll
          for (int j = 0; j < 8; j++) acc[j] += (float)v[j];
        }
      }
    }
    const long long o = pix * g.C + c8 * 8;
    if (add) {
      const bf16x8 a = *(const bf16x8*)(add + o);
#pragma unroll
      for (int j = 0; j < 8; j++) acc[j] += (float)a[j];
    }
    bf16x8 r;
    if (mask) {
      const bf16x8 mk = *(const bf16x8*)(mask + o);
#pragma unroll
      for (int j = 0; j < 8; j++) r[j] = (float)mk[j] > 0.f ? (bf16)acc[j] : (bf16)0.f;
    } else {
#pragma unroll
      for (int j = 0; j < 8; j++) r[j] = (bf16)acc[j];
    }
    *(bf16x8*)(out + o) = r;
  }
}

// ---------------------------------------------------------------------------------------------
// folded BatchNorm: out = act(z1*g1 + b1 + [z2*g2 + b2 | z2]), act = ReLU or identity
// ---------------------------------------------------------------------------------------------
template <bool Z32>
__global__ __launch_bounds__(256) void affine_kernel(const bf16* __restrict__ z1, const float* __restrict__ z1f,
                                                     const bf16* __restrict__ g1, const bf16* __restrict__ b1,
                                                     const bf16* __restrict__ z2, const bf16* __restrict__ g2,
                                                     const bf16* __restrict__ b2, int relu, bf16* __restrict__ out,
                                                     long long n8, int C) {
  const int c8n = C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (long long)gridDim.x * blockDim.x) {
    const int c = (int)(i % c8n) * 8;
    float v[8];
    if (Z32) {
      const float4 a = *(const float4*)(z1f + i * 8), b = *(const float4*)(z1f + i * 8 + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
      const bf16x8 a = *(const bf16x8*)(z1 + i * 8);
#pragma unroll
      for (int j = 0; j < 8; j++) v[j] = (float)a[j];
    }
    const bf16x8 g = *(const bf16x8*)(g1 + c), s = *(const bf16x8*)(b1 + c);
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = v[j] * (float)g[j] + (float)s[j];
    if (z2) {
      const bf16x8 a = *(const bf16x8*)(z2 + i * 8);
      if (g2) {
        const bf16x8 gg = *(const bf16x8*)(g2 + c), ss = *(const bf16x8*)(b2 + c);
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] += (float)a[j] * (float)gg[j] + (float)ss[j];
      } else {
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] += (float)a[j];
      }
    }
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; j++) r[j] = (bf16)(relu ? fmaxf(v[j], 0.f) : v[j]);
    *(bf16x8*)(out + i * 8) = r;
  }
}

// out = d * gain[c]
__global__ __launch_bounds__(256) void scale_cols_kernel(const bf16* __restrict__ d, const bf16* __restrict__ gain,
                                                         bf16* __restrict__ out, long long n8, int C) {
  const int c8n = C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (long long)gridDim.x * blockDim.x) {
    const bf16x8 a = *(const bf16x8*)(d + i * 8), g = *(const bf16x8*)(gain + (int)(i % c8n) * 8);
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; j++) r[j] = (bf16)((float)a[j] * (float)g[j]);
    *(bf16x8*)(out + i * 8) = r;
  }
}

// out = (a + b) * (0 < mask < hi); b may be null; mask may be null (plain sum)
__global__ __launch_bounds__(256) void add_mask_kernel(const bf16* __restrict__ a, const bf16* __restrict__ b,
                                                       const bf16* __restrict__ mask, bf16* __restrict__ out,
                                                       long long n8, float hi) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (long long)gridDim.x * blockDim.x) {
    const bf16x8 x = *(const bf16x8*)(a + i * 8);
    bf16x8 r = x;
    if (b) {
      const bf16x8 y = *(const bf16x8*)(b + i * 8);
#pragma unroll
      for (int j = 0; j < 8; j++) r[j] = (bf16)((float)x[j] + (float)y[j]);
    }
    if (mask) {
      const bf16x8 mk = *(const bf16x8*)(mask + i * 8);
#pragma unroll
      for (int j = 0; j < 8; j++) r[j] = ((float)mk[j] > 0.f && (float)mk[j] < hi) ? r[j] : (bf16)0.f;
    }
    *(bf16x8*)(out + i * 8) = r;
  }
}

// ---------------------------------------------------------------------------------------------
// 3x3 depthwise convolution (zero padding 1, stride 1 or 2) on NHWC, 8 channels per thread; weights
// [C][9].  Forward: z = sum over taps (fp32), stored rounded; y = clamp(z * gain + shift, 0, 6)
// from the rounded z.  Input gradient in gather form: every input pixel sums the output
// gradients of the windows it belongs to; then + add (nullable), times the ReLU6 mask of the
// activation in front of the convolution (nullable).
// ---------------------------------------------------------------------------------------------
struct DwGeom { int B, H, W, C, stride, Ho, Wo; };

// the 72 weights of 8 consecutive channels, [channel][tap]: nine 16-byte loads (c0 is a multiple of 8)
struct DwWeights {
  bf16x8 v[9];
  __device__ __forceinline__ void load(const bf16* __restrict__ w, int c0) {
#pragma unroll
    for (int i = 0; i < 9; i++) v[i] = *(const bf16x8*)(w + c0 * 9 + i * 8);
  }
  __device__ __forceinline__ float at(int j, int tap) const { return (float)v[(j * 9 + tap) >> 3][(j * 9 + tap) & 7]; }
};

__global__ __launch_bounds__(256) void depthwise_fwd_kernel(const bf16* __restrict__ x, const bf16* __restrict__ w,
                                                            const bf16* __restrict__ gain, const bf16* __restrict__ shift,
                                                            bf16* __restrict__ z, bf16* __restrict__ y, DwGeom g,
                                                            long long total) {
  const int c8n = g.C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int c0 = (int)(i % c8n) * 8;
    const long long pix = i / c8n;
    const int wo = (int)(pix % g.Wo), ho = (int)((pix / g.Wo) % g.Ho);
    const long long b = pix / ((long long)g.Wo * g.Ho);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    DwWeights wt;
    wt.load(w, c0);
#pragma unroll
    for (int ky = 0; ky < 3; ky++) {
      const int h = ho * g.stride + ky - 1;
      if ((unsigned)h >= (unsigned)g.H) continue;
#pragma unroll
      for (int kx = 0; kx < 3; kx++) {
        const int ww = wo * g.stride + kx - 1;
        if ((unsigned)ww >= (unsigned)g.W) continue;
        const bf16x8 v = *(const bf16x8*)(x + ((b * g.H + h) * g.W + ww) * g.C + c0);
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] += (float)v[j] * wt.at(j, ky * 3 + kx);
      }
    }
    const bf16x8 gn = *(const bf16x8*)(gain + c0), sh = *(const bf16x8*)(shift + c0);
    bf16x8 zr, yr;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      zr[j] = (bf16)acc[j];
      yr[j] = (bf16)fminf(fmaxf((float)zr[j] * (float)gn[j] + (float)sh[j], 0.f), 6.f);
    }
    if (z) *(bf16x8*)(z + pix * g.C + c0) = zr;
    *(bf16x8*)(y + pix * g.C + c0) = yr;
  }
}

__global__ __launch_bounds__(256) void depthwise_dx_kernel(const bf16* __restrict__ d, const bf16* __restrict__ w,
                                                           const bf16* __restrict__ add, const bf16* __restrict__ mask,
                                                           bf16* __restrict__ out, DwGeom g, long long total) {
  const int c8n = g.C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int c0 = (int)(i % c8n) * 8;
    const long long pix = i / c8n;
    const int ww = (int)(pix % g.W), h = (int)((pix / g.W) % g.H);
    const long long b = pix / ((long long)g.W * g.H);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    DwWeights wt;
    wt.load(w, c0);
#pragma unroll
    for (int ky = 0; ky < 3; ky++) {
      const int hn = h + 1 - ky;                 // = ho * stride
      if (hn < 0 || hn % g.stride) continue;
      const int ho = hn / g.stride;
      if (ho >= g.Ho) continue;
#pragma unroll
      for (int kx = 0; kx < 3; kx++) {
        const int wn = ww + 1 - kx;
        if (wn < 0 || wn % g.stride) continue;
        const int wo = wn / g.stride;
        if (wo >= g.Wo) continue;
        const bf16x8 v = *(const bf16x8*)(d + ((b * g.Ho + ho) * g.Wo + wo) * g.C + c0);
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] += (float)v[j] * wt.at(j, ky * 3 + kx);
      }
    }
    if (add) {
      const bf16x8 v = *(const bf16x8*)(add + pix * g.C + c0);
#pragma unroll
      for (int j = 0; j < 8; j++) acc[j] += (float)v[j];
    }
    bf16x8 r;
    if (mask) {
      const bf16x8 mk = *(const bf16x8*)(mask + pix * g.C + c0);
#pragma unroll
      for (int j = 0; j < 8; j++) r[j] = ((float)mk[j] > 0.f && (float)mk[j] < 6.f) ? (bf16)acc[j] : (bf16)0.f;
    } else {
#pragma unroll
      for (int j = 0; j < 8; j++) r[j] = (bf16)acc[j];
    }
    *(bf16x8*)(out + pix * g.C + c0) = r;
  }
}

// Weight gradient, first stage: worker r (one thread per 8 channels) adds d * x over the output pixels
// r, r + R, r + 2R, ... in that order and writes its 72 sums to part[r][c * 9 + tap]; a column sum over the
// R rows finishes the reduction in a fixed order.
__global__ __launch_bounds__(256) void depthwise_dw_kernel(const bf16* __restrict__ d, const bf16* __restrict__ x,
                                                           float* __restrict__ part, DwGeom g, int R, long long total) {
  const int c8n = g.C >> 3;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c0 = (int)(i % c8n) * 8;
  const int r = (int)(i / c8n);
  const long long pixels = (long long)g.B * g.Ho * g.Wo;
  float acc[9][8];
#pragma unroll
  for (int t = 0; t < 9; t++)
#pragma unroll
    for (int j = 0; j < 8; j++) acc[t][j] = 0.f;
  for (long long pix = r; pix < pixels; pix += R) {
    const int wo = (int)(pix % g.Wo), ho = (int)((pix / g.Wo) % g.Ho);
    const long long b = pix / ((long long)g.Wo * g.Ho);
    const bf16x8 dv = *(const bf16x8*)(d + pix * g.C + c0);
#pragma unroll
    for (int ky = 0; ky < 3; ky++) {
      const int h = ho * g.stride + ky - 1;
      if ((unsigned)h >= (unsigned)g.H) continue;
#pragma unroll
      for (int kx = 0; kx < 3; kx++) {
        const int ww = wo * g.stride + kx - 1;
        if ((unsigned)ww >= (unsigned)g.W) continue;
        const bf16x8 v = *(const bf16x8*)(x + ((b * g.H + h) * g.W + ww) * g.C + c0);
#pragma unroll
        for (int j = 0; j < 8; j++) acc[ky * 3 + kx][j] += (float)dv[j] * (float)v[j];
      }
    }
  }
  float* o = part + (long long)r * g.C * 9 + c0 * 9;
#pragma unroll
  for (int j = 0; j < 8; j++)
#pragma unroll
    for (int t = 0; t < 9; t++) o[j * 9 + t] = acc[t][j];
}

// out = max(z + bias, 0) from an fp32 matrix [rows][N] (a split product's reduced sum); N % 4 == 0
__global__ __launch_bounds__(256) void bias_relu_rows_kernel(const float4* __restrict__ z, const bf16* __restrict__ bias,
                                                             bf16* __restrict__ out, int n4, long long total) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int c = (int)(i % n4) * 4;
    const float4 v = z[i];
    const bf16x4 b = *(const bf16x4*)(bias + c);
    bf16x4 r;
    r[0] = (bf16)fmaxf(v.x + (float)b[0], 0.f);
    r[1] = (bf16)fmaxf(v.y + (float)b[1], 0.f);
    r[2] = (bf16)fmaxf(v.z + (float)b[2], 0.f);
    r[3] = (bf16)fmaxf(v.w + (float)b[3], 0.f);
    *(bf16x4*)(out + i * 4) = r;
  }
}

// ---------------------------------------------------------------------------------------------
// stem: y = relu(z*g + b) evaluated in fp32 from the fp32 convolution output, 3x3 / stride 2 /
// pad 1 max pooling with the first maximum in (ky, kx) order; and its backward in gather form
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const float* __restrict__ z, const bf16* __restrict__ gain,
                                                          const bf16* __restrict__ shift, bf16* __restrict__ out,
                                                          uint8_t* __restrict__ arg, int B, int H, int W, int C, int Ho,
                                                          int Wo, long long total) {
  const int c8n = C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int c8 = (int)(i % c8n);
    const long long pix = i / c8n;
    const int ow = (int)(pix % Wo), oh = (int)((pix / Wo) % Ho), b = (int)(pix / ((long long)Wo * Ho));
    const bf16x8 g = *(const bf16x8*)(gain + c8 * 8), s = *(const bf16x8*)(shift + c8 * 8);
    float best[8];
    int bi[8];
#pragma unroll
    for (int j = 0; j < 8; j++) { best[j] = -INFINITY; bi[j] = 0; }
    for (int ky = 0; ky < 3; ky++) {
      const int h = oh * 2 - 1 + ky;
      if (h < 0 || h >= H) continue;
      for (int kx = 0; kx < 3; kx++) {
        const int w = ow * 2 - 1 + kx;
        if (w < 0 || w >= W) continue;
        const float* p = z + (((long long)b * H + h) * W + w) * C + c8 * 8;
        const float4 a = *(const float4*)p, bb = *(const float4*)(p + 4);
        const float v[8] = {a.x, a.y, a.z, a.w, bb.x, bb.y, bb.z, bb.w};
#pragma unroll
        for (int j = 0; j < 8; j++) {
          const float y = fmaxf(v[j] * (float)g[j] + (float)s[j], 0.f);
          if (y > best[j]) { best[j] = y; bi[j] = ky * 3 + kx; }
        }
      }
    }
    bf16x8 r;
    uint64_t packed = 0;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      r[j] = (bf16)best[j];
      packed |= (uint64_t)bi[j] << (8 * j);
    }
    *(bf16x8*)(out + pix * C + c8 * 8) = r;
    *(uint64_t*)(arg + pix * C + c8 * 8) = packed;
  }
}

// dx[b][h][w][c] = sum over the pooling windows that contain (h, w) and chose it of d, times (y > 0)
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const bf16* __restrict__ d, const uint8_t* __restrict__ arg,
                                                          const bf16* __restrict__ y, bf16* __restrict__ out, int B,
                                                          int H, int W, int C, int Ho, int Wo, long long total) {
  const int c8n = C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int c8 = (int)(i % c8n);
    const long long pix = i / c8n;
    const int w = (int)(pix % W), h = (int)((pix / W) % H), b = (int)(pix / ((long long)W * H));
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; j++) acc[j] = 0.f;
    for (int ky = 0; ky < 3; ky++) {
      const int hh = h + 1 - ky;
      if (hh < 0 || (hh & 1)) continue;
      const int oh = hh >> 1;
      if (oh >= Ho) continue;
      for (int kx = 0; kx < 3; kx++) {
        const int ww = w + 1 - kx;
        if (ww < 0 || (ww & 1)) continue;
        const int ow = ww >> 1;
        if (ow >= Wo) continue;
        const long long o = (((long long)b * Ho + oh) * Wo + ow) * C + c8 * 8;
        const bf16x8 v = *(const bf16x8*)(d + o);
        const uint64_t a = *(const uint64_t*)(arg + o);
#pragma unroll
        for (int j = 0; j < 8; j++)
          if ((int)((a >> (8 * j)) & 0xff) == ky * 3 + kx) acc[j] += (float)v[j];
      }
    }
    const bf16x8 yy = *(const bf16x8*)(y + pix * C + c8 * 8);
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; j++) r[j] = (float)yy[j] > 0.f ? (bf16)acc[j] : (bf16)0.f;
    *(bf16x8*)(out + pix * C + c8 * 8) = r;
  }
}

// 2x2 / stride 2 max pooling (plain convolution stacks): first maximum in (dy, dx) order
__global__ __launch_bounds__(256) void maxpool2_fwd_kernel(const bf16* __restrict__ y, bf16* __restrict__ out,
                                                           uint8_t* __restrict__ arg, int H, int W, int C, long long total) {
  const int c8n = C >> 3, Ho = H >> 1, Wo = W >> 1;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int c8 = (int)(i % c8n);
    const long long pix = i / c8n;
    const int ow = (int)(pix % Wo), oh = (int)((pix / Wo) % Ho);
    const long long b = pix / ((long long)Wo * Ho);
    float best[8];
    int bi[8];
#pragma unroll
    for (int j = 0; j < 8; j++) { best[j] = -INFINITY; bi[j] = 0; }
#pragma unroll
    for (int t = 0; t < 4; t++) {
      const bf16x8 v = *(const bf16x8*)(y + ((b * H + oh * 2 + (t >> 1)) * W + ow * 2 + (t & 1)) * C + c8 * 8);
#pragma unroll
      for (int j = 0; j < 8; j++)
        if ((float)v[j] > best[j]) { best[j] = (float)v[j]; bi[j] = t; }
    }
    bf16x8 r;
    uint64_t packed = 0;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      r[j] = (bf16)best[j];
      packed |= (uint64_t)bi[j] << (8 * j);
    }
    *(bf16x8*)(out + pix * C + c8 * 8) = r;
    *(uint64_t*)(arg + pix * C + c8 * 8) = packed;
  }
}

__global__ __launch_bounds__(256) void maxpool2_bwd_kernel(const bf16* __restrict__ d, const uint8_t* __restrict__ arg,
                                                           const bf16* __restrict__ y, bf16* __restrict__ out, int H, int W,
                                                           int C, long long total) {
  const int c8n = C >> 3, Ho = H >> 1, Wo = W >> 1;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int c8 = (int)(i % c8n);
    const long long pix = i / c8n;
    const int w = (int)(pix % W), h = (int)((pix / W) % H);
    const long long b = pix / ((long long)W * H);
    const long long o = ((b * Ho + (h >> 1)) * Wo + (w >> 1)) * C + c8 * 8;
    const bf16x8 dv = *(const bf16x8*)(d + o), yy = *(const bf16x8*)(y + pix * C + c8 * 8);
    const uint64_t a = *(const uint64_t*)(arg + o);
    const int tap = (h & 1) * 2 + (w & 1);
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; j++)
      r[j] = ((int)((a >> (8 * j)) & 0xff) == tap && (float)yy[j] > 0.f) ? dv[j] : (bf16)0.f;
    *(bf16x8*)(out + pix * C + c8 * 8) = r;
  }
}

// ---------------------------------------------------------------------------------------------
// global average pooling and its backward (+ the ReLU closing the last block)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const bf16* __restrict__ x, bf16* __restrict__ p, int B, int HW,
                                                          int C) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * C) return;
  const int b = i / C, c = i % C;
  float s = 0.f;
  for (int t = 0; t < HW; t++) s += (float)x[((long long)b * HW + t) * C + c];
  p[i] = (bf16)(s / (float)HW);
}

__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const bf16* __restrict__ dp, const bf16* __restrict__ y,
                                                          bf16* __restrict__ out, int HW, int C, long long n8, float hi) {
  const int c8n = C >> 3;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (long long)gridDim.x * blockDim.x) {
    const int c8 = (int)(i % c8n);
    const long long b = i / ((long long)c8n * HW);
    const bf16x8 v = *(const bf16x8*)(dp + b * C + c8 * 8), yy = *(const bf16x8*)(y + i * 8);
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; j++) r[j] = ((float)yy[j] > 0.f && (float)yy[j] < hi) ? (bf16)((float)v[j] / (float)HW) : (bf16)0.f;
    *(bf16x8*)(out + i * 8) = r;
  }
}

// rows of K elements -> rows of Kc >= K elements, tail zero (bf16); and back (fp32)
__global__ void pad_rows_kernel(const bf16* __restrict__ in, bf16* __restrict__ out, int rows, int K, int Kc) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * Kc) return;
  const int r = i / Kc, k = i % Kc;
  out[i] = k < K ? in[r * K + k] : (bf16)0.f;
}
__global__ void strip_rows_kernel(const float* __restrict__ in, float* __restrict__ out, int rows, int K, int Kc) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * K) return;
  out[i] = in[(i / K) * Kc + i % K];
}

// Operands of the stem convolution (7x7, stride 2, zero padding 3, at most 4 input channels) in the form its
// gathered GEMM reads.  Image: [B][H][W][C] -> [B][Hp][Wp][4] with pixel (h, w) at (h + 3, w + 3) and zeros elsewhere,
// one thread per padded pixel (8 bytes).  Weight: [O][7][7][C] -> [O][8][8][4], zero outside the 7x7xC window.
// Weight gradient: float [O][8][8][4] -> [O][7][7][C].
__global__ void stem_pad_image_kernel(const bf16* __restrict__ x, bf16* __restrict__ out, int H, int W, int C, int Hp, int Wp,
                                      long long total) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int wp = (int)(i % Wp), hp = (int)((i / Wp) % Hp);
  const long long b = i / ((long long)Wp * Hp);
  const int h = hp - 3, w = wp - 3;
  bf16x4 v = {(bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f};
  if ((unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) {
    const bf16* src = x + ((b * H + h) * W + w) * C;
    for (int c = 0; c < C; c++) v[c] = src[c];
  }
  *(bf16x4*)(out + i * 4) = v;
}
__global__ void stem_pack_weight_kernel(const bf16* __restrict__ w, bf16* __restrict__ out, int O, int C) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;   // index into out: (o, ky, kx, c)
  if (i >= O * 256) return;
  const int c = i & 3, kx = (i >> 2) & 7, ky = (i >> 5) & 7, o = i >> 8;
  out[i] = (ky < 7 && kx < 7 && c < C) ? w[((o * 7 + ky) * 7 + kx) * C + c] : (bf16)0.f;
}
__global__ void stem_unpack_dw_kernel(const float* __restrict__ in, float* __restrict__ out, int O, int C) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;   // index into out: (o, ky, kx, c)
  if (i >= O * 49 * C) return;
  const int c = i % C, kx = (i / C) % 7, ky = (i / (7 * C)) % 7, o = i / (49 * C);
  out[i] = in[o * 256 + ky * 32 + kx * 4 + c];
}

// out[c][8 - tap][o] = w[o][tap][c]: the weight of the convolution that carries a 3x3 convolution's output
// gradient back to its input (taps mirrored, channel roles exchanged)
__global__ void flip3x3_kernel(const bf16* __restrict__ w, bf16* __restrict__ out, int O, int C) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;   // index into out: (c, tap', o)
  if (i >= O * 9 * C) return;
  const int o = i % O, tp = (i / O) % 9, c = i / (9 * O);
  out[i] = w[((long long)o * 9 + (8 - tp)) * C + c];
}

inline unsigned grid_for(long long total) {
  long long b = (total + 255) / 256;
  return (unsigned)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

bool geom_ok(const ConvGeom& g) {
  if (g.B < 1 || g.H < 1 || g.W < 1 || g.C < 1 || g.k < 1 || g.stride < 1 || g.pad < 0 || g.Ho < 1 || g.Wo < 1) return false;
  if (g.Ho != (g.H + 2 * g.pad - g.k) / g.stride + 1 || g.Wo != (g.W + 2 * g.pad - g.k) / g.stride + 1) return false;
  if (g.Kc < g.k * g.k * g.C || (g.Kc & 7)) return false;
  return true;
}

}  // namespace

hipError_t im2col(const bf16* x, bf16* cols, const ConvGeom& g, hipStream_t s) {
  if (!geom_ok(g) || !al16(x) || !al16(cols)) return hipErrorInvalidValue;
  const long long M = (long long)g.B * g.Ho * g.Wo;
  if ((g.C & 7) == 0 && g.Kc == g.k * g.k * g.C) {
    const long long total = M * g.k * g.k * (g.C >> 3);
    hipLaunchKernelGGL(im2col_vec_kernel, dim3(grid_for(total)), dim3(256), 0, s, x, cols, g, total);
  } else {
    const long long total = M * (g.Kc >> 3);
    hipLaunchKernelGGL(im2col_any_kernel, dim3(grid_for(total)), dim3(256), 0, s, x, cols, g, total);
  }
  return hipGetLastError();
}

hipError_t col2im(const void* dcols, bool dcols_f32, const bf16* add, const bf16* mask, bf16* out, const ConvGeom& g,
                  hipStream_t s) {
  if (!geom_ok(g) || (g.C & 7) || g.Kc != g.k * g.k * g.C) return hipErrorInvalidValue;
  if (!al16(dcols) || !al16(out) || (add && !al16(add)) || (mask && !al16(mask))) return hipErrorInvalidValue;
  const long long total = (long long)g.B * g.H * g.W * (g.C >> 3);
  if (dcols_f32)
    hipLaunchKernelGGL(col2im_kernel<float>, dim3(grid_for(total)), dim3(256), 0, s, (const float*)dcols, add, mask, out, g, total);
  else
    hipLaunchKernelGGL(col2im_kernel<bf16>, dim3(grid_for(total)), dim3(256), 0, s, (const bf16*)dcols, add, mask, out, g, total);
  return hipGetLastError();
}

hipError_t affine_act(const bf16* z1, const float* z1_f32, const bf16* g1, const bf16* b1, const bf16* z2,
                      const bf16* g2, const bf16* b2, bool relu, bf16* out, long long rows, int C, hipStream_t s) {
  if (rows < 1 || C < 8 || (C & 7) || (!z1 && !z1_f32) || !g1 || !b1 || (g2 && !b2) || (g2 && !z2)) return hipErrorInvalidValue;
  if ((z1 && !al16(z1)) || (z1_f32 && !al16(z1_f32)) || !al16(g1) || !al16(b1) || (z2 && !al16(z2)) ||
      (g2 && (!al16(g2) || !al16(b2))) || !al16(out))
    return hipErrorInvalidValue;
  const long long n8 = rows * (C >> 3);
  if (z1_f32)
    hipLaunchKernelGGL((affine_kernel<true>), dim3(grid_for(n8)), dim3(256), 0, s, z1, z1_f32, g1, b1, z2, g2, b2,
                       relu ? 1 : 0, out, n8, C);
  else
    hipLaunchKernelGGL((affine_kernel<false>), dim3(grid_for(n8)), dim3(256), 0, s, z1, z1_f32, g1, b1, z2, g2, b2,
                       relu ? 1 : 0, out, n8, C);
  return hipGetLastError();
}

hipError_t scale_cols(const bf16* d, const bf16* gain, bf16* out, long long rows, int C, hipStream_t s) {
  if (rows < 1 || C < 8 || (C & 7) || !al16(d) || !al16(gain) || !al16(out)) return hipErrorInvalidValue;
  const long long n8 = rows * (C >> 3);
  hipLaunchKernelGGL(scale_cols_kernel, dim3(grid_for(n8)), dim3(256), 0, s, d, gain, out, n8, C);
  return hipGetLastError();
}

hipError_t bias_relu_rows(const float* z, const bf16* bias, bf16* out, int rows, int N, hipStream_t s) {
  if (rows < 1 || N < 4 || (N & 3) || !al16(z) || !bias || (reinterpret_cast<uintptr_t>(bias) & 7) || (reinterpret_cast<uintptr_t>(out) & 7))
    return hipErrorInvalidValue;
  const long long total = (long long)rows * (N >> 2);
  hipLaunchKernelGGL(bias_relu_rows_kernel, dim3(grid_for(total)), dim3(256), 0, s, (const float4*)z, bias, out, N >> 2, total);
  return hipGetLastError();
}

hipError_t add_mask(const bf16* a, const bf16* b, const bf16* mask, bf16* out, long long n, hipStream_t s, float mask_hi) {
  if (n < 8 || (n & 7) || !a || (!mask && !b) || !al16(a) || (b && !al16(b)) || (mask && !al16(mask)) || !al16(out))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(add_mask_kernel, dim3(grid_for(n >> 3)), dim3(256), 0, s, a, b, mask, out, n >> 3, mask_hi);
  return hipGetLastError();
}

namespace {
bool dw_geom(DwGeom& g, int B, int H, int W, int C, int stride) {
  if (B < 1 || H < 1 || W < 1 || C < 8 || (C & 7) || (stride != 1 && stride != 2)) return false;
  g.B = B; g.H = H; g.W = W; g.C = C; g.stride = stride;
  g.Ho = (H - 1) / stride + 1;
  g.Wo = (W - 1) / stride + 1;
  return true;
}
}  // namespace

hipError_t depthwise3x3_fwd(const bf16* x, const bf16* w, const bf16* gain, const bf16* shift, bf16* z, bf16* y, int B, int H,
                            int W, int C, int stride, hipStream_t s) {
  DwGeom g;
  if (!dw_geom(g, B, H, W, C, stride) || !al16(x) || !al16(w) || !al16(gain) || !al16(shift) || (z && !al16(z)) || !al16(y))
    return hipErrorInvalidValue;
  const long long total = (long long)B * g.Ho * g.Wo * (C >> 3);
  hipLaunchKernelGGL(depthwise_fwd_kernel, dim3(grid_for(total)), dim3(256), 0, s, x, w, gain, shift, z, y, g, total);
  return hipGetLastError();
}

hipError_t depthwise3x3_dx(const bf16* d, const bf16* w, const bf16* add, const bf16* relu6_y, bf16* out, int B, int H, int W,
                           int C, int stride, hipStream_t s) {
  DwGeom g;
  if (!dw_geom(g, B, H, W, C, stride) || !al16(d) || !al16(w) || (add && !al16(add)) || (relu6_y && !al16(relu6_y)) || !al16(out))
    return hipErrorInvalidValue;
  const long long total = (long long)B * H * W * (C >> 3);
  hipLaunchKernelGGL(depthwise_dx_kernel, dim3(grid_for(total)), dim3(256), 0, s, d, w, add, relu6_y, out, g, total);
  return hipGetLastError();
}

int depthwise3x3_dw_rows(int B, int H, int W, int C, int stride) {
  const long long pixels = (long long)B * ((H - 1) / stride + 1) * ((W - 1) / stride + 1);
  long long r = 65536 / (C >> 3);
  if (r < 64) r = 64;
  if (r > pixels) r = pixels;
  return (int)r;
}

hipError_t depthwise3x3_dw(const bf16* d, const bf16* x, float* part, int B, int H, int W, int C, int stride, hipStream_t s) {
  DwGeom g;
  if (!dw_geom(g, B, H, W, C, stride) || !al16(d) || !al16(x) || !al16(part)) return hipErrorInvalidValue;
  const int R = depthwise3x3_dw_rows(B, H, W, C, stride);
  const long long total = (long long)R * (C >> 3);
  hipLaunchKernelGGL(depthwise_dw_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, d, x, part, g, R, total);
  return hipGetLastError();
}

hipError_t maxpool3x3s2_fwd(const float* z, const bf16* gain, const bf16* shift, bf16* out, uint8_t* arg, int B, int H,
                            int W, int C, hipStream_t s) {
  if (B < 1 || H < 1 || W < 1 || C < 8 || (C & 7) || !al16(z) || !al16(gain) || !al16(shift) || !al16(out) || !al16(arg))
    return hipErrorInvalidValue;
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  const long long total = (long long)B * Ho * Wo * (C >> 3);
  hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(grid_for(total)), dim3(256), 0, s, z, gain, shift, out, arg, B, H, W, C, Ho,
                     Wo, total);
  return hipGetLastError();
}

hipError_t maxpool3x3s2_bwd(const bf16* d, const uint8_t* arg, const bf16* y, bf16* out, int B, int H, int W, int C,
                            hipStream_t s) {
  if (B < 1 || H < 1 || W < 1 || C < 8 || (C & 7) || !al16(d) || !al16(arg) || !al16(y) || !al16(out))
    return hipErrorInvalidValue;
  const int Ho = (H - 1) / 2 + 1, Wo = (W - 1) / 2 + 1;
  const long long total = (long long)B * H * W * (C >> 3);
  hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(grid_for(total)), dim3(256), 0, s, d, arg, y, out, B, H, W, C, Ho, Wo,
                     total);
  return hipGetLastError();
}

hipError_t maxpool2x2_fwd(const bf16* y, bf16* out, uint8_t* arg, int B, int H, int W, int C, hipStream_t s) {
  if (B < 1 || H < 2 || W < 2 || (H & 1) || (W & 1) || C < 8 || (C & 7) || !al16(y) || !al16(out) || !al16(arg))
    return hipErrorInvalidValue;
  const long long total = (long long)B * (H >> 1) * (W >> 1) * (C >> 3);
  hipLaunchKernelGGL(maxpool2_fwd_kernel, dim3(grid_for(total)), dim3(256), 0, s, y, out, arg, H, W, C, total);
  return hipGetLastError();
}

hipError_t maxpool2x2_bwd(const bf16* d, const uint8_t* arg, const bf16* y, bf16* out, int B, int H, int W, int C,
                          hipStream_t s) {
  if (B < 1 || H < 2 || W < 2 || (H & 1) || (W & 1) || C < 8 || (C & 7) || !al16(d) || !al16(arg) || !al16(y) || !al16(out))
    return hipErrorInvalidValue;
  const long long total = (long long)B * H * W * (C >> 3);
  hipLaunchKernelGGL(maxpool2_bwd_kernel, dim3(grid_for(total)), dim3(256), 0, s, d, arg, y, out, H, W, C, total);
  return hipGetLastError();
}

hipError_t avgpool_fwd(const bf16* x, bf16* p, int B, int HW, int C, hipStream_t s) {
  if (B < 1 || HW < 1 || C < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(avgpool_fwd_kernel, dim3((B * C + 255) / 256), dim3(256), 0, s, x, p, B, HW, C);
  return hipGetLastError();
}

hipError_t avgpool_bwd_relu(const bf16* dp, const bf16* y, bf16* out, int B, int HW, int C, hipStream_t s, float mask_hi) {
  if (B < 1 || HW < 1 || C < 8 || (C & 7) || !al16(dp) || !al16(y) || !al16(out)) return hipErrorInvalidValue;
  const long long n8 = (long long)B * HW * (C >> 3);
  hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(grid_for(n8)), dim3(256), 0, s, dp, y, out, HW, C, n8, mask_hi);
  return hipGetLastError();
}

hipError_t pad_rows(const bf16* in, bf16* out, int rows, int K, int Kc, hipStream_t s) {
  if (rows < 1 || K < 1 || Kc < K) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pad_rows_kernel, dim3((rows * Kc + 255) / 256), dim3(256), 0, s, in, out, rows, K, Kc);
  return hipGetLastError();
}

hipError_t flip3x3(const bf16* w, bf16* out, int O, int C, hipStream_t s) {
  if (O < 1 || C < 1 || (long long)O * 9 * C > 0x7fffffffll) return hipErrorInvalidValue;
  hipLaunchKernelGGL(flip3x3_kernel, dim3((O * 9 * C + 255) / 256), dim3(256), 0, s, w, out, O, C);
  return hipGetLastError();
}

hipError_t stem_pad_image(const bf16* x, bf16* out, int B, int H, int W, int C, int Hp, int Wp, hipStream_t s) {
  if (B < 1 || H < 1 || W < 1 || C < 1 || C > 4 || Hp < H + 3 || Wp < W + 3 || !al16(out)) return hipErrorInvalidValue;
  const long long total = (long long)B * Hp * Wp;
  if (total > 0x7fffffffll * 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stem_pad_image_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x, out, H, W, C, Hp, Wp, total);
  return hipGetLastError();
}

hipError_t stem_pack_weight(const bf16* w, bf16* out, int O, int C, hipStream_t s) {
  if (O < 1 || C < 1 || C > 4 || O > (1 << 20)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stem_pack_weight_kernel, dim3(O), dim3(256), 0, s, w, out, O, C);
  return hipGetLastError();
}

hipError_t stem_unpack_dw(const float* in, float* out, int O, int C, hipStream_t s) {
  if (O < 1 || C < 1 || C > 4 || O > (1 << 20)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stem_unpack_dw_kernel, dim3((O * 49 * C + 255) / 256), dim3(256), 0, s, in, out, O, C);
  return hipGetLastError();
}

hipError_t strip_rows(const float* in, float* out, int rows, int K, int Kc, hipStream_t s) {
  if (rows < 1 || K < 1 || Kc < K) return hipErrorInvalidValue;
  hipLaunchKernelGGL(strip_rows_kernel, dim3((rows * K + 255) / 256), dim3(256), 0, s, in, out, rows, K, Kc);
  return hipGetLastError();
}

}  // namespace et
