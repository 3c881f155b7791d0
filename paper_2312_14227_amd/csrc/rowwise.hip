// HBM-bound kernels of the training step: LayerNorm forward/backward, softmax forward/backward,
// cross-entropy, column and batch reductions (bias / LayerNorm gain and shift / embedding
// gradients, Sections 5.1 and 5.2), embedding assembly.  One 64-lane wave owns one row in the
// row-wise kernels; reductions inside a wave use cross-lane shuffles, all sums have a fixed
// order so results are bit-reproducible.
#include "kernels.h"

namespace et {
namespace {

constexpr int WAVE = 64;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------------
// LayerNorm forward: out = (h - mean) * rstd * gain + shift, statistics in fp32 (two passes)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const float* __restrict__ h, long long in_stride,
                                                            const bf16* __restrict__ gain,
                                                            const bf16* __restrict__ shift, float eps,
                                                            bf16* __restrict__ out, float* __restrict__ mean,
                                                            float* __restrict__ rstd, int rows, int D) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float4* x = (const float4*)(h + (long long)row * in_stride);
  const int n4 = D >> 2;
  float s = 0.f;
  for (int i = lane; i < n4; i += WAVE) {
    const float4 v = x[i];
    s += (v.x + v.y) + (v.z + v.w);
  }
  const float mu = wave_sum(s) / (float)D;
  float q = 0.f;
  for (int i = lane; i < n4; i += WAVE) {
    const float4 v = x[i];
    const float a = v.x - mu, b = v.y - mu, c = v.z - mu, d = v.w - mu;
    q += (a * a + b * b) + (c * c + d * d);
  }
  const float rs = 1.f / sqrtf(wave_sum(q) / (float)D + eps);
  if (lane == 0) {
    mean[row] = mu;
    rstd[row] = rs;
  }
  bf16x4* o = (bf16x4*)(out + (long long)row * D);
  const bf16x4* g4 = (const bf16x4*)gain;
  const bf16x4* b4 = (const bf16x4*)shift;
  for (int i = lane; i < n4; i += WAVE) {
    const float4 v = x[i];
    const bf16x4 g = g4[i], b = b4[i];
    bf16x4 r;
    r[0] = (bf16)((v.x - mu) * rs * (float)g[0] + (float)b[0]);
    r[1] = (bf16)((v.y - mu) * rs * (float)g[1] + (float)b[1]);
    r[2] = (bf16)((v.z - mu) * rs * (float)g[2] + (float)b[2]);
    r[3] = (bf16)((v.w - mu) * rs * (float)g[3] + (float)b[3]);
    o[i] = r;
  }
}

// The same for rows of V * 256 elements: the row stays in registers (V float4 per lane, all loads in flight at
// once) instead of being read three times; sums in the same order, so both kernels give the same bits.
template <int V>
__global__ __launch_bounds__(256) void layernorm_fwd_regs_kernel(const float* __restrict__ h, long long in_stride,
                                                                 const bf16* __restrict__ gain,
                                                                 const bf16* __restrict__ shift, float eps,
                                                                 bf16* __restrict__ out, float* __restrict__ mean,
                                                                 float* __restrict__ rstd, int rows) {
  constexpr int D = V * 256;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float4* x = (const float4*)(h + (long long)row * in_stride);
  float4 v[V];
#pragma unroll
  for (int j = 0; j < V; j++) v[j] = x[lane + j * WAVE];
  bf16x4 g[V], b[V];
#pragma unroll
  for (int j = 0; j < V; j++) {
    g[j] = ((const bf16x4*)gain)[lane + j * WAVE];
    b[j] = ((const bf16x4*)shift)[lane + j * WAVE];
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < V; j++) s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
  const float mu = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < V; j++) {
    const float a = v[j].x - mu, bb = v[j].y - mu, c = v[j].z - mu, d = v[j].w - mu;
    q += (a * a + bb * bb) + (c * c + d * d);
  }
  const float rs = 1.f / sqrtf(wave_sum(q) / (float)D + eps);
  if (lane == 0) {
    mean[row] = mu;
    rstd[row] = rs;
  }
  bf16x4* o = (bf16x4*)(out + (long long)row * D);
#pragma unroll
  for (int j = 0; j < V; j++) {
    bf16x4 r;
    r[0] = (bf16)((v[j].x - mu) * rs * (float)g[j][0] + (float)b[j][0]);
    r[1] = (bf16)((v[j].y - mu) * rs * (float)g[j][1] + (float)b[j][1]);
    r[2] = (bf16)((v[j].z - mu) * rs * (float)g[j][2] + (float)b[j][2]);
    r[3] = (bf16)((v[j].w - mu) * rs * (float)g[j][3] + (float)b[j][3]);
    o[lane + j * WAVE] = r;
  }
}

// ---------------------------------------------------------------------------------------------
// LayerNorm input gradient (+ residual branch): with xhat = (h-mean)*rstd, t = d*gain,
//   dh = skip + rstd * (t - mean(t) - xhat * mean(t*xhat))
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void layernorm_bwd_dx_kernel(const bf16* __restrict__ d, const float* __restrict__ h,
                                                               long long in_stride, const float* __restrict__ mean,
                                                               const float* __restrict__ rstd,
                                                               const bf16* __restrict__ gain,
                                                               const float* __restrict__ skip, float* __restrict__ dh,
                                                               bf16* __restrict__ dh16, long long out_stride, int rows,
                                                               int D) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float4* x = (const float4*)(h + (long long)row * in_stride);
  const bf16x4* d4 = (const bf16x4*)(d + (long long)row * D);
  const bf16x4* g4 = (const bf16x4*)gain;
  const int n4 = D >> 2;
  const float mu = mean[row], rs = rstd[row];
  float s1 = 0.f, s2 = 0.f;
  for (int i = lane; i < n4; i += WAVE) {
    const float4 v = x[i];
    const bf16x4 dv = d4[i], g = g4[i];
    const float t0 = (float)dv[0] * (float)g[0], t1 = (float)dv[1] * (float)g[1];
    const float t2 = (float)dv[2] * (float)g[2], t3 = (float)dv[3] * (float)g[3];
    s1 += (t0 + t1) + (t2 + t3);
    s2 += (t0 * ((v.x - mu) * rs) + t1 * ((v.y - mu) * rs)) + (t2 * ((v.z - mu) * rs) + t3 * ((v.w - mu) * rs));
  }
  const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
  const float4* sk = skip ? (const float4*)(skip + (long long)row * out_stride) : nullptr;
  float4* o = (float4*)(dh + (long long)row * out_stride);
  bf16x4* o16 = dh16 ? (bf16x4*)(dh16 + (long long)row * out_stride) : nullptr;
  for (int i = lane; i < n4; i += WAVE) {
    const float4 v = x[i];
    const bf16x4 dv = d4[i], g = g4[i];
    float4 r;
    r.x = rs * ((float)dv[0] * (float)g[0] - m1 - (v.x - mu) * rs * m2);
    r.y = rs * ((float)dv[1] * (float)g[1] - m1 - (v.y - mu) * rs * m2);
    r.z = rs * ((float)dv[2] * (float)g[2] - m1 - (v.z - mu) * rs * m2);
    r.w = rs * ((float)dv[3] * (float)g[3] - m1 - (v.w - mu) * rs * m2);
    if (sk) {
      const float4 k = sk[i];
      r.x += k.x; r.y += k.y; r.z += k.z; r.w += k.w;
    }
    o[i] = r;
    if (o16) {
      bf16x4 q;
      q[0] = (bf16)r.x; q[1] = (bf16)r.y; q[2] = (bf16)r.z; q[3] = (bf16)r.w;
      o16[i] = q;
    }
  }
}

// The same for rows of V * 256 elements, held in registers between the two passes (same sums, same order)
template <int V>
__global__ __launch_bounds__(256) void layernorm_bwd_dx_regs_kernel(const bf16* __restrict__ d, const float* __restrict__ h,
                                                                    long long in_stride, const float* __restrict__ mean,
                                                                    const float* __restrict__ rstd,
                                                                    const bf16* __restrict__ gain,
                                                                    const float* __restrict__ skip, float* __restrict__ dh,
                                                                    bf16* __restrict__ dh16, long long out_stride, int rows) {
  constexpr int D = V * 256;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float4* x = (const float4*)(h + (long long)row * in_stride);
  const bf16x4* d4 = (const bf16x4*)(d + (long long)row * D);
  const float4* sk = skip ? (const float4*)(skip + (long long)row * out_stride) : nullptr;
  float4 v[V], k[V];
  bf16x4 dv[V], g[V];
#pragma unroll
  for (int j = 0; j < V; j++) {
    v[j] = x[lane + j * WAVE];
    dv[j] = d4[lane + j * WAVE];
    g[j] = ((const bf16x4*)gain)[lane + j * WAVE];
    if (sk) k[j] = sk[lane + j * WAVE];
  }
  const float mu = mean[row], rs = rstd[row];
  float t[V][4];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int j = 0; j < V; j++) {
#pragma unroll
    for (int e = 0; e < 4; e++) t[j][e] = (float)dv[j][e] * (float)g[j][e];
    s1 += (t[j][0] + t[j][1]) + (t[j][2] + t[j][3]);
    s2 += (t[j][0] * ((v[j].x - mu) * rs) + t[j][1] * ((v[j].y - mu) * rs)) +
          (t[j][2] * ((v[j].z - mu) * rs) + t[j][3] * ((v[j].w - mu) * rs));
  }
  const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
  float4* o = (float4*)(dh + (long long)row * out_stride);
  bf16x4* o16 = dh16 ? (bf16x4*)(dh16 + (long long)row * out_stride) : nullptr;
#pragma unroll
  for (int j = 0; j < V; j++) {
    float4 r;
    r.x = rs * (t[j][0] - m1 - (v[j].x - mu) * rs * m2);
    r.y = rs * (t[j][1] - m1 - (v[j].y - mu) * rs * m2);
    r.z = rs * (t[j][2] - m1 - (v[j].z - mu) * rs * m2);
    r.w = rs * (t[j][3] - m1 - (v[j].w - mu) * rs * m2);
    if (sk) {
      r.x += k[j].x; r.y += k[j].y; r.z += k[j].z; r.w += k[j].w;
    }
    o[lane + j * WAVE] = r;
    if (o16) {
      bf16x4 q;
      q[0] = (bf16)r.x; q[1] = (bf16)r.y; q[2] = (bf16)r.z; q[3] = (bf16)r.w;
      o16[lane + j * WAVE] = q;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// column sums, stage 1: a block of 8 column-threads (8 columns each) x 32 row-threads sums
// cs_rows() rows of 64 columns; stage 2 adds the row-chunk partials in ascending order
// ---------------------------------------------------------------------------------------------
constexpr int CS_COLS = 64;
// rows per chunk: about 2048 workgroups per launch (a multiple of 32 rows, 64 to 1024), so that a tall narrow
// matrix and a short wide one both fill the chip; the same function sizes the partial buffer
__host__ __device__ inline int cs_rows(int rows, int cols) {
  const int col_blocks = (cols + CS_COLS - 1) / CS_COLS;
  const int chunks_wanted = 2048 / col_blocks > 0 ? 2048 / col_blocks : 1;
  int per = ((rows + chunks_wanted - 1) / chunks_wanted + 31) & ~31;
  return per < 64 ? 64 : (per > 1024 ? 1024 : per);
}

template <bool F32IN, bool XHAT>
__global__ __launch_bounds__(256) void colsum_stage1(const bf16* __restrict__ d16, const float* __restrict__ d32,
                                                     long long d_stride, const float* __restrict__ h,
                                                     long long h_stride, const float* __restrict__ mean,
                                                     const float* __restrict__ rstd, float* __restrict__ partials,
                                                     int rows, int cols) {
  __shared__ float red[32][CS_COLS + 1];
  const int cx = threadIdx.x & 7, ry = threadIdx.x >> 3;
  const int c0 = blockIdx.x * CS_COLS + cx * 8;
  const int chunk_rows = cs_rows(rows, cols);
  const int r_begin = blockIdx.y * chunk_rows, r_end = min(rows, r_begin + chunk_rows);
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; j++) acc[j] = 0.f;
  if (c0 < cols) {
    for (int r = r_begin + ry; r < r_end; r += 32) {
      float v[8];
      if (F32IN) {
        const float4 a = *(const float4*)(d32 + (long long)r * d_stride + c0);
        const float4 b = *(const float4*)(d32 + (long long)r * d_stride + c0 + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
      } else {
        const bf16x8 a = *(const bf16x8*)(d16 + (long long)r * d_stride + c0);
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = (float)a[j];
      }
      if (XHAT) {
        const float mu = mean[r], rs = rstd[r];
        const float4 a = *(const float4*)(h + (long long)r * h_stride + c0);
        const float4 b = *(const float4*)(h + (long long)r * h_stride + c0 + 4);
        v[0] *= (a.x - mu) * rs; v[1] *= (a.y - mu) * rs; v[2] *= (a.z - mu) * rs; v[3] *= (a.w - mu) * rs;
        v[4] *= (b.x - mu) * rs; v[5] *= (b.y - mu) * rs; v[6] *= (b.z - mu) * rs; v[7] *= (b.w - mu) * rs;
      }
#pragma unroll
      for (int j = 0; j < 8; j++) acc[j] += v[j];
    }
  }
#pragma unroll
  for (int j = 0; j < 8; j++) red[ry][cx * 8 + j] = acc[j];
  __syncthreads();
  if (threadIdx.x < CS_COLS) {
    const int c = blockIdx.x * CS_COLS + threadIdx.x;
    if (c < cols) {
      float s = red[0][threadIdx.x];
#pragma unroll
      for (int k = 1; k < 32; k++) s += red[k][threadIdx.x];
      partials[(long long)blockIdx.y * cols + c] = s;
    }
  }
}

// same reduction with an element-wise multiplier: out[c] = sum_r d[r][c] * z[r][c]
template <bool Z32>
__global__ __launch_bounds__(256) void colsum_mul_stage1(const bf16* __restrict__ d, const bf16* __restrict__ z16,
                                                         const float* __restrict__ z32, float* __restrict__ partials,
                                                         int rows, int cols) {
  __shared__ float red[32][CS_COLS + 1];
  const int cx = threadIdx.x & 7, ry = threadIdx.x >> 3;
  const int c0 = blockIdx.x * CS_COLS + cx * 8;
  const int chunk_rows = cs_rows(rows, cols);
  const int r_begin = blockIdx.y * chunk_rows, r_end = min(rows, r_begin + chunk_rows);
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; j++) acc[j] = 0.f;
  if (c0 < cols) {
    for (int r = r_begin + ry; r < r_end; r += 32) {
      const bf16x8 a = *(const bf16x8*)(d + (long long)r * cols + c0);
      if (Z32) {
        const float4 p = *(const float4*)(z32 + (long long)r * cols + c0);
        const float4 q = *(const float4*)(z32 + (long long)r * cols + c0 + 4);
        acc[0] += (float)a[0] * p.x; acc[1] += (float)a[1] * p.y; acc[2] += (float)a[2] * p.z; acc[3] += (float)a[3] * p.w;
        acc[4] += (float)a[4] * q.x; acc[5] += (float)a[5] * q.y; acc[6] += (float)a[6] * q.z; acc[7] += (float)a[7] * q.w;
      } else {
        const bf16x8 b = *(const bf16x8*)(z16 + (long long)r * cols + c0);
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] += (float)a[j] * (float)b[j];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; j++) red[ry][cx * 8 + j] = acc[j];
  __syncthreads();
  if (threadIdx.x < CS_COLS) {
    const int c = blockIdx.x * CS_COLS + threadIdx.x;
    if (c < cols) {
      float s = red[0][threadIdx.x];
#pragma unroll
      for (int k = 1; k < 32; k++) s += red[k][threadIdx.x];
      partials[(long long)blockIdx.y * cols + c] = s;
    }
  }
}

// both of the above from one read of d: partials [chunks][cols] of the plain sums, followed by [chunks][cols] of
// the sums with the multiplier; chunking and summation order as in the separate kernels, so the results are the same
template <bool Z32>
__global__ __launch_bounds__(256) void colsum_pair_stage1(const bf16* __restrict__ d, const bf16* __restrict__ z16,
                                                          const float* __restrict__ z32, float* __restrict__ partials,
                                                          int rows, int cols) {
  __shared__ float red[2][32][CS_COLS + 1];
  const int cx = threadIdx.x & 7, ry = threadIdx.x >> 3;
  const int c0 = blockIdx.x * CS_COLS + cx * 8;
  const int chunk_rows = cs_rows(rows, cols);
  const int r_begin = blockIdx.y * chunk_rows, r_end = min(rows, r_begin + chunk_rows);
  float acc[8], accz[8];
#pragma unroll
  for (int j = 0; j < 8; j++) acc[j] = accz[j] = 0.f;
  if (c0 < cols) {
    for (int r = r_begin + ry; r < r_end; r += 32) {
      const bf16x8 a = *(const bf16x8*)(d + (long long)r * cols + c0);
      float zz[8];
      if (Z32) {
        const float4 p = *(const float4*)(z32 + (long long)r * cols + c0);
        const float4 q = *(const float4*)(z32 + (long long)r * cols + c0 + 4);
        zz[0] = p.x; zz[1] = p.y; zz[2] = p.z; zz[3] = p.w; zz[4] = q.x; zz[5] = q.y; zz[6] = q.z; zz[7] = q.w;
      } else {
        const bf16x8 b = *(const bf16x8*)(z16 + (long long)r * cols + c0);
#pragma unroll
        for (int j = 0; j < 8; j++) zz[j] = (float)b[j];
      }
#pragma unroll
      for (int j = 0; j < 8; j++) {
        acc[j] += (float)a[j];
        accz[j] += (float)a[j] * zz[j];
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; j++) {
    red[0][ry][cx * 8 + j] = acc[j];
    red[1][ry][cx * 8 + j] = accz[j];
  }
  __syncthreads();
  if (threadIdx.x < 2 * CS_COLS) {
    const int which = threadIdx.x / CS_COLS, cl = threadIdx.x % CS_COLS;
    const int c = blockIdx.x * CS_COLS + cl;
    if (c < cols) {
      float s = red[which][0][cl];
#pragma unroll
      for (int k = 1; k < 32; k++) s += red[which][k][cl];
      partials[((long long)which * gridDim.y + blockIdx.y) * cols + c] = s;
    }
  }
}

// stage 2: 16 threads per column each add every 16th row-chunk partial, then the 16 sums are added
// in ascending order (a long serial loop per column would be bound by load latency)
constexpr int S2_PARTS = 16, S2_COLS = 16;
__global__ __launch_bounds__(256) void colsum_stage2(const float* __restrict__ partials, float* __restrict__ out,
                                                     int chunks, int cols) {
  __shared__ float red[S2_PARTS][S2_COLS + 1];
  const int cx = threadIdx.x % S2_COLS, part = threadIdx.x / S2_COLS;
  const int c = blockIdx.x * S2_COLS + cx;
  float s = 0.f;
  if (c < cols) {
#pragma unroll 4
    for (int k = part; k < chunks; k += S2_PARTS) s += partials[(long long)k * cols + c];
  }
  red[part][cx] = s;
  __syncthreads();
  if (threadIdx.x < S2_COLS && c < cols) {
    float t = red[0][cx];
#pragma unroll
    for (int q = 1; q < S2_PARTS; q++) t += red[q][cx];
    out[c] = t;
  }
}

// stage 2 of the pair: columns [0, cols) finish the plain sums into out0, columns [cols, 2 cols) the others into out1
__global__ __launch_bounds__(256) void colsum_pair_stage2(const float* __restrict__ partials, float* __restrict__ out0,
                                                          float* __restrict__ out1, int chunks, int cols) {
  __shared__ float red[S2_PARTS][S2_COLS + 1];
  const int cx = threadIdx.x % S2_COLS, part = threadIdx.x / S2_COLS;
  const int c2 = blockIdx.x * S2_COLS + cx;
  const int which = c2 >= cols ? 1 : 0, c = c2 - which * cols;
  const float* src = partials + (long long)which * chunks * cols;
  float s = 0.f;
  if (c2 < 2 * cols) {
#pragma unroll 4
    for (int k = part; k < chunks; k += S2_PARTS) s += src[(long long)k * cols + c];
  }
  red[part][cx] = s;
  __syncthreads();
  if (threadIdx.x < S2_COLS && c2 < 2 * cols) {
    float t = red[0][cx];
#pragma unroll
    for (int q = 1; q < S2_PARTS; q++) t += red[q][cx];
    (which ? out1 : out0)[c] = t;
  }
}

__global__ void batchsum_kernel(const float* __restrict__ d, float* __restrict__ out, int B, long long batch_stride,
                                int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = d[i];
  for (int b = 1; b < B; b++) s += d[(long long)b * batch_stride + i];
  out[i] = s;
}

// ---------------------------------------------------------------------------------------------
// softmax rows (attention probabilities) and its backward
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void softmax_rows_kernel(const float* __restrict__ s, bf16* __restrict__ p, int rows,
                                                           int cols, int ld) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* x = s + (long long)row * ld;
  bf16* o = p + (long long)row * ld;
  float mx = -INFINITY;
  for (int i = lane; i < cols; i += WAVE) mx = fmaxf(mx, x[i]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int i = lane; i < cols; i += WAVE) sum += __expf(x[i] - mx);
  const float inv = 1.f / wave_sum(sum);
  for (int i = lane; i < ld; i += WAVE) o[i] = (bf16)(i < cols ? __expf(x[i] - mx) * inv : 0.f);
}

__global__ __launch_bounds__(256) void softmax_bwd_rows_kernel(const float* __restrict__ dp, const bf16* __restrict__ p,
                                                               bf16* __restrict__ ds, float scale, int rows, int cols,
                                                               int ld) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* g = dp + (long long)row * ld;
  const bf16* pr = p + (long long)row * ld;
  bf16* o = ds + (long long)row * ld;
  float dot = 0.f;
  for (int i = lane; i < cols; i += WAVE) dot += g[i] * (float)pr[i];
  dot = wave_sum(dot);
  for (int i = lane; i < ld; i += WAVE) o[i] = (bf16)(i < cols ? scale * (float)pr[i] * (g[i] - dot) : 0.f);
}

// ---------------------------------------------------------------------------------------------
// mean softmax cross-entropy and its gradient: one wave per row (4 rows per block) writes the
// gradient and the row's loss term; a second one-wave kernel adds the terms in ascending order
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void xent_rows_kernel(const float* __restrict__ logits, const int32_t* __restrict__ y,
                                                        int B, int C, float* __restrict__ row_loss,
                                                        float* __restrict__ dl, bf16* __restrict__ dl16, int ld16) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= B) return;
  const float invB = 1.f / (float)B;
  const float* x = logits + (long long)r * C;
  float mx = -INFINITY;
  for (int i = lane; i < C; i += WAVE) mx = fmaxf(mx, x[i]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int i = lane; i < C; i += WAVE) sum += expf(x[i] - mx);
  sum = wave_sum(sum);
  const float lse = logf(sum) + mx;
  const int label = y[r];
  if (lane == 0) row_loss[r] = lse - x[label];
  for (int i = lane; i < ld16; i += WAVE) {
    float gval = 0.f;
    if (i < C) {
      gval = (expf(x[i] - lse) - (i == label ? 1.f : 0.f)) * invB;
      dl[(long long)r * C + i] = gval;
    }
    if (dl16) dl16[(long long)r * ld16 + i] = (bf16)gval;
  }
}

__global__ __launch_bounds__(64) void xent_loss_kernel(const float* __restrict__ row_loss, int B, float* __restrict__ loss) {
  if (threadIdx.x != 0) return;
  float acc = 0.f;
  for (int r = 0; r < B; r++) acc += row_loss[r];
  *loss = acc / (float)B;
}

// ---------------------------------------------------------------------------------------------
// embedding assembly, CLS-row drop, fill, cast
// ---------------------------------------------------------------------------------------------
__global__ void embed_assemble_kernel(const float* __restrict__ e, const bf16* __restrict__ cls,
                                      const bf16* __restrict__ pos, float* __restrict__ h0, int B, int T, int D) {
  const long long i4 = blockIdx.x * (long long)blockDim.x + threadIdx.x;
  const int d4 = D >> 2;
  if (i4 >= (long long)B * T * d4) return;
  const int c = (int)(i4 % d4) * 4;
  const long long bt = i4 / d4;
  const int t = (int)(bt % T);
  const long long b = bt / T;
  const bf16x4 pv = *(const bf16x4*)(pos + (long long)t * D + c);
  float4 r;
  if (t == 0) {
    const bf16x4 cv = *(const bf16x4*)(cls + c);
    r = make_float4((float)cv[0], (float)cv[1], (float)cv[2], (float)cv[3]);
  } else {
    r = *(const float4*)(e + (b * (T - 1) + (t - 1)) * D + c);
  }
  r.x += (float)pv[0]; r.y += (float)pv[1]; r.z += (float)pv[2]; r.w += (float)pv[3];
  *(float4*)(h0 + bt * D + c) = r;
}

__global__ void gather_patch_rows_kernel(const float* __restrict__ d, bf16* __restrict__ out, int B, int T, int D) {
  const long long i4 = blockIdx.x * (long long)blockDim.x + threadIdx.x;
  const int d4 = D >> 2;
  if (i4 >= (long long)B * (T - 1) * d4) return;
  const int c = (int)(i4 % d4) * 4;
  const long long bp = i4 / d4;
  const int p = (int)(bp % (T - 1));
  const long long b = bp / (T - 1);
  const float4 v = *(const float4*)(d + (b * T + p + 1) * D + c);
  bf16x4 q;
  q[0] = (bf16)v.x; q[1] = (bf16)v.y; q[2] = (bf16)v.z; q[3] = (bf16)v.w;
  *(bf16x4*)(out + bp * D + c) = q;
}

__global__ void fill_zero_kernel(uint4* __restrict__ p, size_t n16, unsigned char* __restrict__ tail, size_t ntail) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
  if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

__global__ void cast_bf16_kernel(const float* __restrict__ in, bf16* __restrict__ out, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += stride) out[i] = (bf16)in[i];
}

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool al8(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 7) == 0; }

}  // namespace

hipError_t layernorm_fwd(const float* h, long long in_stride, const bf16* gain, const bf16* shift, float eps, bf16* out,
                         float* mean, float* rstd, int rows, int D, hipStream_t s) {
  if (rows <= 0 || D <= 0 || (D & 3) || (in_stride & 3) || !al16(h) || !al8(gain) || !al8(shift) || !al8(out))
    return hipErrorInvalidValue;
  const dim3 grid((rows + 3) / 4), block(256);
  switch ((D & 255) ? 0 : D / 256) {
#define ET_LN_REGS(V) \
    case V: hipLaunchKernelGGL(layernorm_fwd_regs_kernel<V>, grid, block, 0, s, h, in_stride, gain, shift, eps, out, mean, rstd, rows); break;
    ET_LN_REGS(1) ET_LN_REGS(2) ET_LN_REGS(3) ET_LN_REGS(4) ET_LN_REGS(5) ET_LN_REGS(6) ET_LN_REGS(8)
#undef ET_LN_REGS
    default:
      hipLaunchKernelGGL(layernorm_fwd_kernel, grid, block, 0, s, h, in_stride, gain, shift, eps, out, mean, rstd, rows, D);
  }
  return hipGetLastError();
}

hipError_t layernorm_bwd_dx(const bf16* d, const float* h, long long in_stride, const float* mean, const float* rstd,
                            const bf16* gain, const float* skip, float* dh, bf16* dh16, long long out_stride, int rows,
                            int D, hipStream_t s) {
  if (rows <= 0 || D <= 0 || (D & 3) || (in_stride & 3) || (out_stride & 3) || !al16(h) || !al8(d) || !al8(gain) ||
      !al16(dh) || (skip && !al16(skip)) || (dh16 && !al8(dh16)))
    return hipErrorInvalidValue;
  const dim3 grid((rows + 3) / 4), block(256);
  switch ((D & 255) ? 0 : D / 256) {
#define ET_LN_REGS(V) \
    case V: hipLaunchKernelGGL(layernorm_bwd_dx_regs_kernel<V>, grid, block, 0, s, d, h, in_stride, mean, rstd, gain, skip, dh, dh16, out_stride, rows); break;
    ET_LN_REGS(1) ET_LN_REGS(2) ET_LN_REGS(3) ET_LN_REGS(4) ET_LN_REGS(5) ET_LN_REGS(6)
#undef ET_LN_REGS
    default:
      hipLaunchKernelGGL(layernorm_bwd_dx_kernel, grid, block, 0, s, d, h, in_stride, mean, rstd, gain, skip, dh, dh16, out_stride, rows, D);
  }
  return hipGetLastError();
}

size_t colsum_partial_elems(int rows, int cols) {
  const int per = cs_rows(rows, cols);
  return (size_t)((rows + per - 1) / per) * cols;
}

hipError_t colsum(const bf16* d, const float* d_f32, long long d_stride, const float* h, long long h_stride,
                  const float* mean, const float* rstd, float* out, float* partials, int rows, int cols,
                  hipStream_t s) {
  if (rows <= 0 || cols <= 0 || (cols & 7) || (d_stride & 7) || (h && (h_stride & 3)) || (!d && !d_f32) || !partials)
    return hipErrorInvalidValue;
  if ((d && !al16(d)) || (d_f32 && !al16(d_f32)) || (h && !al16(h))) return hipErrorInvalidValue;
  const int chunks = (rows + cs_rows(rows, cols) - 1) / cs_rows(rows, cols);
  dim3 grid((cols + CS_COLS - 1) / CS_COLS, chunks), block(256);
  if (d_f32) {
    if (h)
      hipLaunchKernelGGL((colsum_stage1<true, true>), grid, block, 0, s, d, d_f32, d_stride, h, h_stride, mean, rstd,
                         partials, rows, cols);
    else
      hipLaunchKernelGGL((colsum_stage1<true, false>), grid, block, 0, s, d, d_f32, d_stride, h, h_stride, mean, rstd,
                         partials, rows, cols);
  } else {
    if (h)
      hipLaunchKernelGGL((colsum_stage1<false, true>), grid, block, 0, s, d, d_f32, d_stride, h, h_stride, mean, rstd,
                         partials, rows, cols);
    else
      hipLaunchKernelGGL((colsum_stage1<false, false>), grid, block, 0, s, d, d_f32, d_stride, h, h_stride, mean, rstd,
                         partials, rows, cols);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_stage2, dim3((cols + S2_COLS - 1) / S2_COLS), dim3(256), 0, s, partials, out, chunks, cols);
  return hipGetLastError();
}

hipError_t colsum_mul(const bf16* d, const bf16* z, const float* z_f32, float* out, float* partials, int rows, int cols,
                      hipStream_t s) {
  if (rows <= 0 || cols <= 0 || (cols & 7) || !d || (!z && !z_f32) || !partials) return hipErrorInvalidValue;
  if (!al16(d) || (z && !al16(z)) || (z_f32 && !al16(z_f32))) return hipErrorInvalidValue;
  const int chunks = (rows + cs_rows(rows, cols) - 1) / cs_rows(rows, cols);
  dim3 grid((cols + CS_COLS - 1) / CS_COLS, chunks), block(256);
  if (z_f32)
    hipLaunchKernelGGL((colsum_mul_stage1<true>), grid, block, 0, s, d, z, z_f32, partials, rows, cols);
  else
    hipLaunchKernelGGL((colsum_mul_stage1<false>), grid, block, 0, s, d, z, z_f32, partials, rows, cols);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_stage2, dim3((cols + S2_COLS - 1) / S2_COLS), dim3(256), 0, s, partials, out, chunks, cols);
  return hipGetLastError();
}

hipError_t colsum_pair(const bf16* d, const bf16* z, const float* z_f32, float* out_sum, float* out_mul, float* partials,
                       int rows, int cols, hipStream_t s) {
  if (rows <= 0 || cols <= 0 || (cols & 7) || !d || (!z && !z_f32) || !partials || !out_sum || !out_mul) return hipErrorInvalidValue;
  if (!al16(d) || (z && !al16(z)) || (z_f32 && !al16(z_f32))) return hipErrorInvalidValue;
  const int chunks = (rows + cs_rows(rows, cols) - 1) / cs_rows(rows, cols);
  dim3 grid((cols + CS_COLS - 1) / CS_COLS, chunks), block(256);
  if (z_f32)
    hipLaunchKernelGGL((colsum_pair_stage1<true>), grid, block, 0, s, d, z, z_f32, partials, rows, cols);
  else
    hipLaunchKernelGGL((colsum_pair_stage1<false>), grid, block, 0, s, d, z, z_f32, partials, rows, cols);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_pair_stage2, dim3((2 * cols + S2_COLS - 1) / S2_COLS), dim3(256), 0, s, partials, out_sum, out_mul,
                     chunks, cols);
  return hipGetLastError();
}

hipError_t batchsum(const float* d, float* out, int B, long long batch_stride, int n, hipStream_t s) {
  if (B <= 0 || n <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(batchsum_kernel, dim3((n + 255) / 256), dim3(256), 0, s, d, out, B, batch_stride, n);
  return hipGetLastError();
}

hipError_t softmax_rows(const float* sc, bf16* p, int rows, int cols, int ld, hipStream_t s) {
  if (rows <= 0 || cols <= 0 || ld < cols) return hipErrorInvalidValue;
  hipLaunchKernelGGL(softmax_rows_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, sc, p, rows, cols, ld);
  return hipGetLastError();
}

hipError_t softmax_bwd_rows(const float* dp, const bf16* p, bf16* ds, float scale, int rows, int cols, int ld,
                            hipStream_t s) {
  if (rows <= 0 || cols <= 0 || ld < cols) return hipErrorInvalidValue;
  hipLaunchKernelGGL(softmax_bwd_rows_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, dp, p, ds, scale, rows, cols, ld);
  return hipGetLastError();
}

hipError_t xent(const float* logits, const int32_t* y, int B, int C, float* loss, float* dlogits, bf16* dlogits_bf16,
                int ld16, hipStream_t s) {
  if (B <= 0 || C <= 0 || ld16 < C) return hipErrorInvalidValue;
  float* row_loss = loss + 64;
  hipLaunchKernelGGL(xent_rows_kernel, dim3((B + 3) / 4), dim3(256), 0, s, logits, y, B, C, row_loss, dlogits,
                     dlogits_bf16, ld16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(xent_loss_kernel, dim3(1), dim3(64), 0, s, row_loss, B, loss);
  return hipGetLastError();
}

hipError_t embed_assemble(const float* e, const bf16* cls, const bf16* pos, float* h0, int B, int T, int D,
                          hipStream_t s) {
  if ((D & 3) || !al16(e) || !al8(cls) || !al8(pos) || !al16(h0)) return hipErrorInvalidValue;
  const long long n = (long long)B * T * (D / 4);
  hipLaunchKernelGGL(embed_assemble_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, e, cls, pos, h0, B, T, D);
  return hipGetLastError();
}

hipError_t gather_patch_rows(const float* d, bf16* out, int B, int T, int D, hipStream_t s) {
  if ((D & 3) || !al16(d) || !al8(out)) return hipErrorInvalidValue;
  const long long n = (long long)B * (T - 1) * (D / 4);
  hipLaunchKernelGGL(gather_patch_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, d, out, B, T, D);
  return hipGetLastError();
}

hipError_t fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (!al16(p)) return hipErrorInvalidValue;
  if (bytes == 0) return hipSuccess;
  const size_t n16 = bytes / 16, ntail = bytes % 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)p, n16,
                     (unsigned char*)p + n16 * 16, ntail);
  return hipGetLastError();
}

hipError_t cast_bf16(const float* in, bf16* out, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, in, out, n);
  return hipGetLastError();
}

}  // namespace et
