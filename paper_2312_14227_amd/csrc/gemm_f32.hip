// fp32 GEMM with plain FMA arithmetic for the fp32 MLP workload (true fp32 products and sums, so
// that gradients agree with the fp64 reference to 1e-5).  Same operand convention as the bf16
// kernel: D[i][j] = sum_k A(i,k) B(j,k), either operand optionally stored reduction-index-slow.
// 64 x 64 tile per 256-thread workgroup, 4 x 4 outputs per thread, K in slices of 16 through LDS.
#include "kernels.h"

namespace et {
namespace {

constexpr int TS = 64, KS = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32Desc g) {
  __shared__ float sa[KS][TS + 1];
  __shared__ float sb[KS][TS + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < g.K; k0 += KS) {
    // each thread stages 4 elements of each operand slice
#pragma unroll
    for (int p = 0; p < 4; p++) {
      const int e = threadIdx.x + p * 256;
      int r, k;
      if (g.a_t) { k = e / TS; r = e % TS; } else { r = e / KS; k = e % KS; }
      const int gi = m0 + r, gk = k0 + k;
      float v = 0.f;
      if (gi < g.M && gk < g.K) v = g.a_t ? g.A[(long long)gk * g.lda + gi] : g.A[(long long)gi * g.lda + gk];
      sa[k][r] = v;
      if (g.b_t) { k = e / TS; r = e % TS; } else { r = e / KS; k = e % KS; }
      const int gj = n0 + r;
      const int gk2 = k0 + k;
      v = 0.f;
      if (gj < g.N && gk2 < g.K) v = g.b_t ? g.B[(long long)gk2 * g.ldb + gj] : g.B[(long long)gj * g.ldb + gk2];
      sb[k][r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KS; k++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = sa[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) b[j] = sb[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int row = m0 + ty * 4 + i;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int col = n0 + tx * 4 + j;
      if (col >= g.N) continue;
      float v = acc[i][j];
      const long long ci = (long long)row * g.ldc + col;
      if (g.relu_out) v = fmaxf(v, 0.f);
      if (g.mask) v = g.mask[ci] > 0.f ? v : 0.f;
      g.C[ci] = v;
    }
  }
}

}  // namespace

hipError_t gemm_f32(const GemmF32Desc& d, hipStream_t s) {
  if (!d.A || !d.B || !d.C || d.M <= 0 || d.N <= 0 || d.K <= 0 || d.ldc < d.N) return hipErrorInvalidValue;
  if ((!d.a_t && d.lda < d.K) || (d.a_t && d.lda < d.M) || (!d.b_t && d.ldb < d.K) || (d.b_t && d.ldb < d.N))
    return hipErrorInvalidValue;
  dim3 grid((d.N + TS - 1) / TS, (d.M + TS - 1) / TS), block(256);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, s, d);
  return hipGetLastError();
}

}  // namespace et
