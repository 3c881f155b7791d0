/* et_debug.h - kernel-level entry points for tests and tuning.  Not needed to run the training
 * step; they expose single kernels of the library so that each can be checked in isolation. */
#ifndef ET_DEBUG_H_
#define ET_DEBUG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* bf16 MFMA GEMM used for the forward product, the error-gradient passing and the weight
 * gradient (Section 5.1):  C[i][j] = alpha * sum_k A(i,k) * B(j,k) + bias[j] + residual[i][j]
 *   A(i,k) = a_t ? A[k*lda + i] : A[i*lda + k],   B(j,k) = b_t ? B[k*ldb + j] : B[j*ldb + k].
 * All pointers are device pointers; A, B, bias (nullable) bf16; residual (nullable) fp32 [M][ldc];
 * C is fp32 if c_f32 else bf16, leading dimension ldc.  split_k > 1 needs c_f32, ldc == N and
 * `partials` with M*N*split_k floats.  A residual needs c_f32 and a_t = b_t = 0.  tile: 0 =
 * automatic, otherwise a tile id of the library (1, 3: register-staged 128x128, 128x64; 5, 7:
 * direct-to-LDS 256x256, 256x128; 11, 13, 15, 17, 19, 21: the two-group tiles 256x256, 256x192, 256x128, 512x64,
 * 128x256, 64x512).  epilogue: 0 the plain one above; 1 GELU forward, with u = the value above: bf16 C = gelu'(u) and
 * a second bf16 output aux [M][ldc] = gelu(u); 2 GELU backward: bf16 C = value * aux, aux bf16 [M][ldc] the stored
 * gelu'(u) (b_t = 1 only); 3 bf16 C = gelu(u), aux unused.  stream: hipStream_t.
 * Returns 0, or -1 for a rejected argument, -3 for a HIP error. */
int et_debug_gemm_bf16(const void* A, const void* B, void* C, int M, int N, int K, int lda, int ldb, int ldc,
                       int a_t, int b_t, int c_f32, float alpha, const void* bias, const float* residual,
                       int split_k, float* partials, int tile, int epilogue, void* aux, void* stream);

/* 3x3 / stride 1 / zero padding 1 convolution as an implicit GEMM (the im2col matrix of Section 5.1's
 * convolution kernels is never written): out[b][h][w][n] = sum over (ky, kx, c) of
 * x[b][h+ky-1][w+kx-1][c] * w[n][ky][kx][c].  x bf16 NHWC [batch][H][W][C], C a multiple of 64; w bf16
 * [N][3][3][C]; out bf16 [batch*H*W][N], N a multiple of 4.  mode 0: plain; 1: out = max(v + bias[n], 0);
 * 2: out = U > 0 ? v : 0 with U bf16 shaped like out.  tile: 0 = automatic, or 11, 13, 15, 17 for the
 * 256x256, 256x192, 256x128, 512x64 tiles.  Device pointers, 16-byte aligned.  Returns 0, -1, -3 as above. */
int et_debug_conv3x3(const void* x, const void* w, void* out, int batch, int H, int W, int C, int N,
                     const void* bias, const void* U, int mode, int tile, void* stream);

/* The same convolution with its reduction over (tap, channel) split into split_k ranges (layers with few
 * pixels): fp32 parts go to `partials` (batch*H*W * N * split_k floats), a second kernel adds them in
 * ascending order and applies the epilogue.  mode 0, 1, 2 as above; 3: z_out (nullable) = the convolution
 * rounded to bf16, out = min(max(z * gain[n] + bias[n], 0), 6).  split_k = 0 lets the library plan tile and
 * split (then `partials` must hold 18 such copies).  N a multiple of 4. */
int et_debug_conv3x3_split(const void* x, const void* w, void* out, void* z_out, int batch, int H, int W, int C, int N,
                           const void* bias, const void* gain, const void* U, int mode, int split_k, float* partials, int tile,
                           void* stream);

/* Weight gradient of that convolution as an implicit GEMM: dw[n][ky][kx][c] = sum over pixels (b, h, w) of
 * d[b][h][w][n] * x[b][h+ky-1][w+kx-1][c].  x bf16 NHWC, C a multiple of 8; d bf16 [batch*H*W][N], N a multiple of 8;
 * dw fp32 [N][9 C]; batch*H*W a multiple of 64; H, W < 4096.  split_k > 1 reduces over that many pixel ranges
 * through `partials` (N * 9 C * split_k floats); split_k = 0 lets the library plan tile and split (then `partials`
 * must hold 256 such copies).  tile: 0 = automatic, or 11, 13, 19, 21 for the 256x256, 256x192, 128x256, 64x512
 * tiles.  Returns 0, -1, -3 as above. */
int et_debug_conv3x3_dw(const void* x, const void* d, float* dw, int batch, int H, int W, int C, int N, int split_k,
                        float* partials, int tile, void* stream);

/* The gathered (implicit im2col) convolution products in general form: taps = 3 (zero padding 1) or 1 (no padding),
 * stride 1 or 2, Ho = (H - 1) / stride + 1, Wo likewise.  x bf16 NHWC [batch][H][W][C].
 *   op 0 forward: w_or_d = weights bf16 [N][taps][taps][C], C a multiple of 64; out bf16 [batch*Ho*Wo][N];
 *   op 1 weight gradient: w_or_d = d bf16 [batch*Ho*Wo][N]; out fp32 [N][taps*taps*C]; C a multiple of 8,
 *     batch*Ho*Wo a multiple of 64.
 * split_k, partials, tile as in the two 3x3 entries above (split_k = 0 plans tile and split).  Returns 0, -1, -3. */
int et_debug_conv_gathered(int op, const void* x, const void* w_or_d, void* out, int batch, int H, int W, int C, int N,
                           int taps, int stride, int split_k, float* partials, int tile, void* stream);

/* Stem convolution (7x7, stride 2, zero padding 3, C <= 4 input channels) as a gathered GEMM over a padded copy of
 * the image.  x bf16 NHWC [batch][H][W][C]; Ho = (H - 1) / 2 + 1, Wo likewise; N a multiple of 8.
 *   op 0 forward: w_or_d = weights bf16 [N][7][7][C]; out fp32 [batch*Ho*Wo][N];
 *   op 1 weight gradient: w_or_d = d bf16 [batch*Ho*Wo][N]; out fp32 [N][7][7][C]; batch*Ho*Wo a multiple of 64.
 * ws = device scratch of et_debug_stem_ws_bytes(..) bytes (0 = arguments out of range), 256-byte aligned.
 * Returns 0, -1, -3. */
size_t et_debug_stem_ws_bytes(int batch, int H, int W, int C, int N);
int et_debug_stem(int op, const void* x, const void* w_or_d, float* out, void* ws, int batch, int H, int W, int C, int N,
                  void* stream);

/* 3x3 depthwise convolution kernels (zero padding 1, stride 1 or 2; NHWC bf16, C a multiple of 8; weights bf16
 * [C][9]; Ho = (H - 1) / stride + 1, Wo likewise).  op selects the kernel:
 *   0 forward: a = x [batch][H][W][C], b = weights, gain, shift [C]; out0 (nullable) = z, the convolution rounded to
 *     bf16; out1 = y = min(max(z * gain + shift, 0), 6), both [batch][Ho][Wo][C];
 *   1 input gradient: a = d [batch][Ho][Wo][C], b = weights, `gain` = an addend (nullable) and `shift` = a stored
 *     ReLU6 activation (nullable), both [batch][H][W][C]; out0 = (adjoint applied to d + addend) where 0 < activation < 6;
 *   2 weight gradient: a = d, b = x; out0 = fp32 [C][9]; ws = device scratch of et_debug_depthwise3x3_ws_floats(..) floats.
 * Device pointers, 16-byte aligned.  Returns 0, -1, -3 as above. */
size_t et_debug_depthwise3x3_ws_floats(int batch, int H, int W, int C, int stride);
int et_debug_depthwise3x3(int op, const void* a, const void* b, const void* gain, const void* shift, void* out0, void* out1,
                          float* ws, int batch, int H, int W, int C, int stride, void* stream);

/* Fused attention core of one layer for sequences of at most 224 tokens and head size 64 (Section 5.4 counts the
 * attention operations among the layers without weights; their backward time is charged to the tensor whose
 * gradient passing needs them).  qkv bf16 [B][T][3 D], D = 64 H, holding Q | K | V of every token; scale = 1/sqrt(64).
 *   op 0 forward: out bf16 [B][T][D] = softmax(Q K^T * scale) V per (batch, head); lse fp32 [B][H][T] = log-sum-exp
 *     of each query's scaled scores;
 *   op 1 backward: given out and lse of the forward pass and dout bf16 [B][T][D], dqkv bf16 [B][T][3 D] = gradients
 *     w.r.t. Q | K | V.
 * Device pointers, 16-byte aligned.  Returns 0, -1 (T > 224, bad sizes or pointers), -3 as above. */
int et_debug_attention(int op, const void* qkv, void* out, float* lse, const void* dout, void* dqkv, int B, int T, int H,
                       void* stream);

/* Device address and element count (bf16) of an activation the last forward pass of a bound context stored,
 * so that a test can check one layer at a time against the layer's definition applied to the stored input.
 * ET_VGG: "conv<i>.in" [batch][H][W][Cin], "conv<i>.y" (after bias + ReLU), "fc<j>.in" [batch][features];
 * ET_RESNET: "stem.y" (after affine + ReLU, before pooling), "pooled", per block in forward order "blk<i>.x"
 * (block input), "blk<i>.y1", "blk<i>.y2" (after the first / second convolution's affine + ReLU), "blk<i>.y";
 * ET_MOBILENET: "stem.y", "b<i>.x" (block input), "b<i>.y_exp" (after the expansion's ReLU6; the block input
 * when the block has no expansion), "b<i>.y_dw", "b<i>.y" (block output), "last.y".
 * Returns 0, -1 for an unknown name or model kind, -5 before the first forward pass. */
struct et_ctx;
int et_debug_activation(const struct et_ctx* ctx, const char* name, const void** dev, size_t* numel);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; 16-byte aligned device
 * pointers).  Used to calibrate hardware traffic counters against a known size. */
int et_debug_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Measurement support: a loop of nothing but bf16 matrix instructions (v_mfma_f32_32x32x16_bf16, four independent
 * accumulators per wave), `workgroups` workgroups of 8 waves, `iters` iterations each (a multiple of 4): workgroups * 8 * iters * 4
 * instructions of 32 768 floating-point operations.  What it sustains is the matrix rate the chip holds under an
 * all-CU load.  out: device, workgroups * 512 floats (written so that the loop is not optimised away).  Returns 0, -1, -3. */
int et_debug_mfma_peak(float* out, int workgroups, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ET_DEBUG_H_ */
