// Kernel-level entry points for tests and tuning.
#include "et_debug.h"

#include "et.h"
#include "kernels.h"

extern "C" int et_debug_gemm_bf16(const void* A, const void* B, void* C, int M, int N, int K, int lda, int ldb, int ldc,
                                  int a_t, int b_t, int c_f32, float alpha, const void* bias, const float* residual,
                                  int split_k, float* partials, int tile, void* stream) {
  et::GemmDesc g;
  g.A = (const et::bf16*)A; g.B = (const et::bf16*)B; g.C = C;
  g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.a_t = a_t != 0; g.b_t = b_t != 0; g.c_f32 = c_f32 != 0; g.alpha = alpha;
  g.bias = (const et::bf16*)bias; g.residual = residual; g.ldr = N;
  g.split_k = split_k < 1 ? 1 : split_k; g.partials = partials; g.tile = tile;
  const hipError_t e = et::gemm_bf16(g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}
