// Kernel-level entry points for tests and tuning.
#include "et_debug.h"

#include "et.h"
#include "kernels.h"

extern "C" int et_debug_gemm_bf16(const void* A, const void* B, void* C, int M, int N, int K, int lda, int ldb, int ldc,
                                  int a_t, int b_t, int c_f32, float alpha, const void* bias, const float* residual,
                                  int split_k, float* partials, int tile, int epilogue, void* aux, void* stream) {
  et::GemmDesc g;
  g.A = (const et::bf16*)A; g.B = (const et::bf16*)B; g.C = C;
  g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.a_t = a_t != 0; g.b_t = b_t != 0; g.c_f32 = c_f32 != 0; g.alpha = alpha;
  g.bias = (const et::bf16*)bias; g.residual = residual; g.ldr = ldc;
  g.split_k = split_k < 1 ? 1 : split_k; g.partials = partials; g.tile = tile;
  if (epilogue < 0 || epilogue > 3 || (epilogue != 0 && epilogue != 3 && !aux)) return ET_EINVAL;
  if (epilogue == 1) { g.mode = et::EPI_GELU_FWD; g.C2 = (et::bf16*)aux; }
  if (epilogue == 2) { g.mode = et::EPI_GELU_BWD; g.U = (const et::bf16*)aux; }
  if (epilogue == 3) g.mode = et::EPI_GELU_ONLY;
  const hipError_t e = et::gemm_bf16(g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

extern "C" int et_debug_conv3x3(const void* x, const void* w, void* out, int batch, int H, int W, int C, int N,
                                const void* bias, const void* U, int mode, int tile, void* stream) {
  et::GemmDesc g;
  g.A = (const et::bf16*)x; g.B = (const et::bf16*)w; g.C = out;
  g.M = batch * H * W; g.N = N; g.K = 9 * C; g.lda = 9 * C; g.ldb = 9 * C; g.ldc = N;
  g.conv_h = H; g.conv_w = W; g.conv_c = C; g.tile = tile;
  if (mode == 1) { g.mode = et::EPI_BIAS_RELU; g.bias = (const et::bf16*)bias; }
  if (mode == 2) { g.mode = et::EPI_RELU_MASK; g.U = (const et::bf16*)U; }
  if (batch < 1 || H < 1 || W < 1 || (long long)batch * H * W > 0x7fffffffll) return ET_EINVAL;
  const hipError_t e = et::gemm_bf16(g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

extern "C" int et_debug_conv3x3_split(const void* x, const void* w, void* out, void* z_out, int batch, int H, int W, int C, int N,
                                      const void* bias, const void* gain, const void* U, int mode, int split_k, float* partials,
                                      int tile, void* stream) {
  if (batch < 1 || H < 1 || W < 1 || (long long)batch * H * W > 0x7fffffffll) return ET_EINVAL;
  et::GemmDesc g;
  g.A = (const et::bf16*)x; g.B = (const et::bf16*)w; g.C = out;
  g.M = batch * H * W; g.N = N; g.K = 9 * C; g.lda = 9 * C; g.ldb = 9 * C; g.ldc = N;
  g.conv_h = H; g.conv_w = W; g.conv_c = C; g.tile = tile;
  if (mode == 1) { g.mode = et::EPI_BIAS_RELU; g.bias = (const et::bf16*)bias; }
  if (mode == 2) { g.mode = et::EPI_RELU_MASK; g.U = (const et::bf16*)U; }
  if (mode == 3) {
    g.mode = et::EPI_AFFINE_RELU; g.bias = (const et::bf16*)bias; g.gain = (const et::bf16*)gain;
    g.C = z_out; g.C2 = (et::bf16*)out; g.act_hi = 6.f;
  }
  g.split_k = split_k; g.partials = partials;
  if (split_k == 0) { et::gemm_bf16_plan_conv(g.M, g.N, g.K, &g.tile, &g.split_k); }
  const hipError_t e = et::gemm_bf16(g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

extern "C" int et_debug_conv3x3_dw(const void* x, const void* d, float* dw, int batch, int H, int W, int C, int N,
                                   int split_k, float* partials, int tile, void* stream) {
  if (batch < 1 || H < 1 || W < 1 || (long long)batch * H * W > 0x7fffffffll) return ET_EINVAL;
  et::GemmDesc g;
  g.A = (const et::bf16*)d; g.a_t = true; g.lda = N;
  g.B = (const et::bf16*)x; g.b_t = true; g.ldb = 9 * C;
  g.M = N; g.N = 9 * C; g.K = batch * H * W;
  g.C = dw; g.ldc = 9 * C; g.c_f32 = true;
  g.conv_h = H; g.conv_w = W; g.conv_c = C; g.tile = tile;
  g.split_k = split_k < 1 ? 1 : split_k; g.partials = partials;
  if (split_k == 0) et::gemm_bf16_plan_conv_dw(g.M, g.N, g.K, &g.tile, &g.split_k);
  const hipError_t e = et::gemm_bf16(g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

extern "C" int et_debug_conv_gathered(int op, const void* x, const void* w_or_d, void* out, int batch, int H, int W, int C, int N,
                                      int taps, int stride, int split_k, float* partials, int tile, void* stream) {
  if (batch < 1 || H < 1 || W < 1 || (taps != 1 && taps != 3) || (stride != 1 && stride != 2)) return ET_EINVAL;
  const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
  if ((long long)batch * Ho * Wo > 0x7fffffffll) return ET_EINVAL;
  const int kk = taps * taps * C, rows = batch * Ho * Wo;
  et::GemmDesc g;
  g.conv_h = H; g.conv_w = W; g.conv_c = C; g.conv_taps = taps; g.conv_stride = stride; g.tile = tile;
  g.split_k = split_k < 1 ? 1 : split_k; g.partials = partials;
  if (op == 0) {
    g.A = (const et::bf16*)x; g.B = (const et::bf16*)w_or_d; g.C = out;
    g.M = rows; g.N = N; g.K = kk; g.lda = kk; g.ldb = kk; g.ldc = N;
    if (split_k == 0) et::gemm_bf16_plan_conv(g.M, g.N, g.K, &g.tile, &g.split_k);
  } else if (op == 1) {
    g.A = (const et::bf16*)w_or_d; g.a_t = true; g.lda = N;
    g.B = (const et::bf16*)x; g.b_t = true; g.ldb = kk;
    g.M = N; g.N = kk; g.K = rows; g.C = out; g.ldc = kk; g.c_f32 = true;
    if (split_k == 0) et::gemm_bf16_plan_conv_dw(g.M, g.N, g.K, &g.tile, &g.split_k);
  } else {
    return ET_EINVAL;
  }
  const hipError_t e = et::gemm_bf16(g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

namespace {
struct StemPlan { int Ho, Wo, Hp, Wp, split; size_t off_w, off_dw, off_part, bytes; };
bool stem_plan(int batch, int H, int W, int C, int N, StemPlan* p) {
  if (batch < 1 || H < 1 || W < 1 || C < 1 || C > 4 || N < 8 || (N & 7)) return false;
  p->Ho = (H - 1) / 2 + 1; p->Wo = (W - 1) / 2 + 1;
  p->Hp = 2 * (p->Ho - 1) + 8; p->Wp = 2 * (p->Wo - 1) + 8;
  if (p->Hp > 4095 || p->Wp > 4095 || (long long)batch * p->Ho * p->Wo > 0x7fffffffll) return false;
  int tile;
  et::gemm_bf16_plan_conv_dw(N, 256, batch * p->Ho * p->Wo, &tile, &p->split);
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  p->off_w = up((size_t)batch * p->Hp * p->Wp * 4 * 2);
  p->off_dw = p->off_w + up((size_t)N * 256 * 2);
  p->off_part = p->off_dw + up((size_t)N * 256 * 4);
  p->bytes = p->off_part + up(et::gemm_bf16_partial_elems(N, 256, p->split) * 4 + 256);
  return true;
}
}  // namespace

extern "C" size_t et_debug_stem_ws_bytes(int batch, int H, int W, int C, int N) {
  StemPlan p;
  return stem_plan(batch, H, W, C, N, &p) ? p.bytes : 0;
}

extern "C" int et_debug_stem(int op, const void* x, const void* w_or_d, float* out, void* ws, int batch, int H, int W, int C,
                             int N, void* stream) {
  StemPlan p;
  if (!x || !w_or_d || !out || !ws || !stem_plan(batch, H, W, C, N, &p)) return ET_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  et::bf16* xpad = (et::bf16*)ws;
  et::bf16* w8 = (et::bf16*)((char*)ws + p.off_w);
  float* dw8 = (float*)((char*)ws + p.off_dw);
  hipError_t e = et::stem_pad_image((const et::bf16*)x, xpad, batch, H, W, C, p.Hp, p.Wp, s);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? ET_EINVAL : ET_EHIP;
  et::GemmDesc g;
  g.conv_h = p.Hp; g.conv_w = p.Wp; g.conv_c = 4; g.conv_taps = 7; g.conv_stride = 2; g.c_f32 = true;
  const int rows = batch * p.Ho * p.Wo;
  if (op == 0) {
    e = et::stem_pack_weight((const et::bf16*)w_or_d, w8, N, C, s);
    if (e != hipSuccess) return ET_EHIP;
    g.A = xpad; g.B = w8; g.C = out; g.M = rows; g.N = N; g.K = 256; g.lda = 256; g.ldb = 256; g.ldc = N;
    e = et::gemm_bf16(g, s);
  } else if (op == 1) {
    g.A = (const et::bf16*)w_or_d; g.a_t = true; g.lda = N; g.B = xpad; g.b_t = true; g.ldb = 256;
    g.M = N; g.N = 256; g.K = rows; g.C = dw8; g.ldc = 256;
    g.split_k = p.split; g.partials = (float*)((char*)ws + p.off_part);
    e = et::gemm_bf16(g, s);
    if (e == hipSuccess) e = et::stem_unpack_dw(dw8, out, N, C, s);
  } else {
    return ET_EINVAL;
  }
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

extern "C" size_t et_debug_depthwise3x3_ws_floats(int batch, int H, int W, int C, int stride) {
  if (batch < 1 || H < 1 || W < 1 || C < 8 || (C & 7) || (stride != 1 && stride != 2)) return 0;
  const int R = et::depthwise3x3_dw_rows(batch, H, W, C, stride);
  return (size_t)R * C * 9 + et::colsum_partial_elems(R, C * 9) + 64;
}

extern "C" int et_debug_depthwise3x3(int op, const void* a, const void* b, const void* gain, const void* shift, void* out0,
                                     void* out1, float* ws, int batch, int H, int W, int C, int stride, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  typedef const et::bf16* P;
  hipError_t e;
  if (op == 0) {
    e = et::depthwise3x3_fwd((P)a, (P)b, (P)gain, (P)shift, (et::bf16*)out0, (et::bf16*)out1, batch, H, W, C, stride, s);
  } else if (op == 1) {
    e = et::depthwise3x3_dx((P)a, (P)b, (P)gain, (P)shift, (et::bf16*)out0, batch, H, W, C, stride, s);
  } else if (op == 2) {
    if (!ws || et_debug_depthwise3x3_ws_floats(batch, H, W, C, stride) == 0) return ET_EINVAL;
    const int R = et::depthwise3x3_dw_rows(batch, H, W, C, stride);
    e = et::depthwise3x3_dw((P)a, (P)b, ws, batch, H, W, C, stride, s);
    if (e == hipSuccess)
      e = et::colsum(nullptr, ws, C * 9, nullptr, 0, nullptr, nullptr, (float*)out0, ws + (size_t)R * C * 9, R, C * 9, s);
  } else {
    return ET_EINVAL;
  }
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

extern "C" int et_debug_attention(int op, const void* qkv, void* out, float* lse, const void* dout, void* dqkv, int B, int T,
                                  int H, void* stream) {
  if (!qkv || !out || !lse || B < 1 || H < 1 || !et::attention_fused_supported(T, 64)) return ET_EINVAL;
  if ((reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(lse) |
       reinterpret_cast<uintptr_t>(dout) | reinterpret_cast<uintptr_t>(dqkv)) & 15)
    return ET_EINVAL;
  hipError_t e;
  if (op == 0) {
    e = et::attention_fwd((const et::bf16*)qkv, (et::bf16*)out, lse, B, T, H, 64, 0.125f, (hipStream_t)stream);
  } else if (op == 1) {
    if (!dout || !dqkv) return ET_EINVAL;
    e = et::attention_bwd((const et::bf16*)qkv, (const et::bf16*)out, (const et::bf16*)dout, lse, (et::bf16*)dqkv, B, T, H, 64,
                          0.125f, (hipStream_t)stream);
  } else {
    return ET_EINVAL;
  }
  if (e == hipErrorInvalidValue) return ET_EINVAL;
  return e == hipSuccess ? ET_OK : ET_EHIP;
}

namespace {
typedef unsigned dbg_u32x4 __attribute__((ext_vector_type(4)));
// plain streaming copy: a workgroup moves 16 KiB at a time, four 16-byte vectors per thread in flight, non-temporal
// accesses (every byte is touched once)
__global__ __launch_bounds__(256) void et_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const dbg_u32x4* s = (const dbg_u32x4*)src;
  dbg_u32x4* d = (dbg_u32x4*)dst;
  constexpr int U = 4;
  const size_t stride = (size_t)gridDim.x * 256 * U;
  for (size_t i0 = (size_t)blockIdx.x * 256 * U + threadIdx.x; i0 < n16; i0 += stride) {
    dbg_u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
      const size_t i = i0 + 256 * u;
      v[u] = __builtin_nontemporal_load(s + (i < n16 ? i : n16 - 1));
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
      const size_t i = i0 + 256 * u;
      if (i < n16) __builtin_nontemporal_store(v[u], d + i);
    }
  }
}
}  // namespace

namespace {
typedef et::bf16 dbg_bf16x8 __attribute__((ext_vector_type(8)));
typedef float dbg_f32x16 __attribute__((ext_vector_type(16)));
// Nothing but matrix instructions: every wave keeps four independent accumulators going, so the matrix pipe of its
// SIMD never waits for a result.  What this loop sustains is what the chip gives a GEMM at the clock it holds under
// an all-CU MFMA load.
__global__ __launch_bounds__(512) void mfma_peak_kernel(float* __restrict__ out, int iters) {
  // operands with the bit patterns of random values of either sign (what a matrix unit draws, and with it the clock the
  // chip holds, depends on how many operand bits toggle), four different pairs in turn
  unsigned h = (threadIdx.x + 1u) * 2654435761u + blockIdx.x * 40503u;
  dbg_bf16x8 a[4], b[4];
#pragma unroll
  for (int v = 0; v < 4; v++)
#pragma unroll
    for (int e = 0; e < 8; e++) {
      h = h * 1664525u + 1013904223u;
      a[v][e] = (et::bf16)(((float)(h >> 8) * (1.f / 8388608.f) - 1.f) * 0.05f);
      h = h * 1664525u + 1013904223u;
      b[v][e] = (et::bf16)(((float)(h >> 8) * (1.f / 8388608.f) - 1.f) * 0.05f);
    }
  dbg_f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[j][r] = 0.f;
  for (int it = 0; it < iters; it += 4) {   // (iters is a multiple of 4)
#pragma unroll
    for (int u = 0; u < 4; u++)
#pragma unroll
      for (int j = 0; j < 4; j++) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + u) & 3], acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; j++)
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc[j][r];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}
}  // namespace

extern "C" int et_debug_mfma_peak(float* out, int workgroups, int iters, void* stream) {
  if (!out || workgroups < 1 || workgroups > (1 << 20) || iters < 4 || (iters & 3) || iters > (1 << 24)) return ET_EINVAL;
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, out, iters);
  return hipGetLastError() == hipSuccess ? ET_OK : ET_EHIP;
}

extern "C" int et_debug_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15) || ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15))
    return ET_EINVAL;
  if (bytes == 0) return ET_OK;
  hipLaunchKernelGGL(et_copy_kernel, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst,
                     bytes / 16);
  return hipGetLastError() == hipSuccess ? ET_OK : ET_EHIP;
}
