// Internal launch interface of the HIP kernels (gfx950).  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace et {

typedef __bf16 bf16;

// ------------------------------------------------------------------------------------------
// bf16 MFMA GEMM:  D[i][j] = alpha * sum_k A(i,k) * B(j,k)   (fp32 accumulation)
//   A(i,k) = a_t ? A[k*lda + i] : A[i*lda + k]      (a_t: the reduction index is the slow one)
//   B(j,k) = b_t ? B[k*ldb + j] : B[j*ldb + k]
// so forward (X W^T) is (a_t,b_t) = (0,0), input gradient (dY W) is (0,1) and weight gradient
// (dY^T X) is (1,1).  Requirements (checked on the host): 16-byte aligned bases, lda/ldb multiples
// of 8, ldc and the C batch strides multiples of 4; an operand that is not transposed must have
// finite data up to K rounded up to 8 in every row (the tail is multiplied by zeros or must itself
// be zero).  Only the (layout, epilogue) pairs the training step uses are built: a residual needs
// fp32 output and (0,0); GELU forward needs (0,0), GELU backward (0,1), split-K (1,1).
// ------------------------------------------------------------------------------------------
enum EpiMode : int {
  EPI_PLAIN = 0,     // C = v
  EPI_GELU_FWD = 1,  // C = gelu'(v) (bf16, kept for the backward pass), C2 = gelu(v) (bf16)
  EPI_GELU_BWD = 2,  // C = v * U, U = the stored gelu'(u)
  EPI_AFFINE_RELU = 3,  // C = z = v (bf16), C2 = max(z * gain[j] + bias[j], 0) (bf16), z as rounded to bf16
  EPI_BIAS_RELU = 6,    // C = max(v + bias, 0) (bf16)
  EPI_RELU_MASK = 7,    // C = U > 0 ? v : 0 (bf16): gradient through a ReLU whose output U was stored
  EPI_GELU_ONLY = 5,    // C = gelu(v) (bf16): the forward of a layer whose backward will not run
  EPI_AFFINE_ADD_RELU = 4,  // C = z, C2 = max(z * gain + bias + U * gain2 + bias2, 0); gain2 null: + U
};

struct GemmDesc {
  const bf16* A = nullptr;
  const bf16* B = nullptr;
  int M = 0, N = 0, K = 0;
  int lda = 0, ldb = 0;
  bool a_t = false, b_t = false;
  // batching: blockIdx.z = outer * z_inner + inner; offsets in elements
  int z_outer = 1, z_inner = 1;
  long long sAo = 0, sAi = 0, sBo = 0, sBi = 0, sCo = 0, sCi = 0;
  // split-K (weight gradients): > 1 writes fp32 partials to `partials` and reduces them in a
  // fixed order with a second kernel; batching must then be off
  int split_k = 1;
  float* partials = nullptr;
  // epilogue: v = alpha * acc + bias[j] + residual[i][j]
  float alpha = 1.f;
  const bf16* bias = nullptr;      // per output column
  const bf16* gain = nullptr;      // EPI_AFFINE_RELU / EPI_AFFINE_ADD_RELU, per output column
  const bf16* gain2 = nullptr;     // EPI_AFFINE_ADD_RELU (nullable, then bias2 is ignored too)
  const bf16* bias2 = nullptr;
  const float* residual = nullptr; // fp32 [M][ldr]
  int ldr = 0;
  int mode = EPI_PLAIN;
  // the AFFINE modes' activation is a clamp to [act_lo, act_hi] (defaults: ReLU; 0, 6: ReLU6; -inf, +inf: none);
  // EPI_RELU_MASK passes where 0 < U < mask_hi
  float act_lo = 0.f, act_hi = __builtin_inff(), mask_hi = __builtin_inff();
  void* C = nullptr;               // bf16 or fp32 [M][ldc]; may be null for the AFFINE modes (z not kept)
  int ldc = 0;
  bool c_f32 = false;
  bf16* C2 = nullptr;              // EPI_GELU_FWD
  const bf16* U = nullptr;         // EPI_GELU_BWD, EPI_AFFINE_ADD_RELU, EPI_RELU_MASK: same leading dimension as C
  // implicit convolution (conv_c > 0), 3x3 with zero padding 1 (conv_taps = 3) or 1x1 (conv_taps = 1), stride
  // conv_stride (1 or 2): A is the NHWC activation [batch, conv_h, conv_w, conv_c] itself, standing for its im2col
  // matrix [M = batch Ho Wo][K = taps^2 conv_c] (column (tap, c); Ho = (conv_h - 1) / stride + 1); conv_c must be a
  // multiple of 64; row-major operands, no batching; split_k > 1 (with `partials`, ldc == N, bf16 outputs, not with
  // the ADD / GELU modes) reduces in a second kernel that also applies the epilogue.
  // With a_t and b_t (weight gradient): B is the activation standing for [K = batch Ho Wo output pixels]
  // [N = taps^2 conv_c]; conv_c % 8 == 0, K a multiple of 64, fp32 output, split allowed
  int conv_h = 0, conv_w = 0, conv_c = 0, conv_taps = 3, conv_stride = 1;
  int tile = 0;                    // 0 = choose by shape; else a TileId (tuning/tests)
};

// returns hipSuccess, or hipErrorInvalidValue when a requirement above is violated
// *launches (nullable) receives the number of kernels launched (1, or 2 with split-K)
hipError_t gemm_bf16(const GemmDesc& d, hipStream_t s, int* launches = nullptr);
// fp32 partial elements needed for a split-K call
size_t gemm_bf16_partial_elems(int M, int N, int split_k);
// tile and split for a weight gradient [M][N] reduced over K rows (a cost model over tile shapes
// and split counts); pass both on in GemmDesc::tile and GemmDesc::split_k
void gemm_bf16_plan_split(int M, int N, int K, int* tile, int* split_k);
// the same for the implicit forward / gradient-passing 3x3 convolution [M pixels][N channels], K = 9 input channels:
// layers with few pixels split the reduction, and a second kernel sums the parts and applies the epilogue
void gemm_bf16_plan_conv(int M, int N, int K, int* tile, int* split_k);
// the same for the implicit weight gradient of a 3x3 convolution (M output channels, N = 9 input channels, K pixels)
void gemm_bf16_plan_conv_dw(int M, int N, int K, int* tile, int* split_k);

// ------------------------------------------------------------------------------------------
// fp32 GEMM (true fp32 FMA), same operand convention, for the fp32 MLP workload
//   relu_out: C = max(v, 0);  mask: C = v * (mask[i][j] > 0)  (ReLU backward, ldmask = ldc)
// ------------------------------------------------------------------------------------------
struct GemmF32Desc {
  const float* A = nullptr;
  const float* B = nullptr;
  float* C = nullptr;
  int M = 0, N = 0, K = 0, lda = 0, ldb = 0, ldc = 0;
  bool a_t = false, b_t = false;
  bool relu_out = false;
  const float* mask = nullptr;
};
hipError_t gemm_f32(const GemmF32Desc& d, hipStream_t s);

// ------------------------------------------------------------------------------------------
// row-wise and reduction kernels (HBM bound)
// ------------------------------------------------------------------------------------------
// LayerNorm forward over rows of an fp32 matrix; in_stride = elements between consecutive rows
hipError_t layernorm_fwd(const float* h, long long in_stride, const bf16* gain, const bf16* shift, float eps,
                         bf16* out, float* mean, float* rstd, int rows, int D, hipStream_t s);
// LayerNorm input gradient: dh = skip + LN'(d); writes fp32 and a bf16 copy.  skip may be null.
// out_stride lets the result be scattered (final LayerNorm on CLS rows); skip uses out_stride too.
hipError_t layernorm_bwd_dx(const bf16* d, const float* h, long long in_stride, const float* mean, const float* rstd,
                            const bf16* gain, const float* skip, float* dh, bf16* dh_bf16, long long out_stride,
                            int rows, int D, hipStream_t s);
// column sums over rows: out[c] = sum_r d[r][c] * (h ? (h[r][c]-mean[r])*rstd[r] : 1)
//   d is bf16 (d_f32 == nullptr) or fp32; two deterministic stages through `partials`
hipError_t colsum(const bf16* d, const float* d_f32, long long d_stride, const float* h, long long h_stride,
                  const float* mean, const float* rstd, float* out, float* partials, int rows, int cols,
                  hipStream_t s);
size_t colsum_partial_elems(int rows, int cols);
// sum over the batch: out[t][c] = sum_b d[b][t][c]   (t < T_out; fp32 in/out)
hipError_t batchsum(const float* d, float* out, int B, long long batch_stride, int n, hipStream_t s);

// softmax over the first `cols` entries of each fp32 row (ld elements apart); bf16 result, tail zeroed
hipError_t softmax_rows(const float* s, bf16* p, int rows, int cols, int ld, hipStream_t stream);
// dS = scale * P * (dP - sum(dP*P)); bf16 result, tail zeroed
hipError_t softmax_bwd_rows(const float* dp, const bf16* p, bf16* ds, float scale, int rows, int cols, int ld,
                            hipStream_t stream);

// fused attention core (tokens <= 224, head size 64), one workgroup per (batch, head):
//   forward: out[b][t][h*64+d] = softmax(Q K^T * scale) V, lse[b][h][t] = log-sum-exp of the scaled scores
//   backward: dqkv (same layout as qkv) from dout, recomputing the probabilities from lse; `out` is the stored
//   forward output (rowsum(P * dP) = dout . out)
bool attention_fused_supported(int T, int head_dim);
hipError_t attention_fwd(const bf16* qkv, bf16* out, float* lse, int B, int T, int H, int head_dim, float scale,
                         hipStream_t s);
hipError_t attention_bwd(const bf16* qkv, const bf16* out, const bf16* dout, const float* lse, bf16* dqkv, int B, int T, int H,
                         int head_dim, float scale, hipStream_t s);

// mean softmax cross-entropy: dlogits fp32 and (if not null) a bf16 copy [B][ld16], zero padded; `loss` points to
// 64 + B floats: the loss in element 0, the per-row terms from element 64 on (two launches)
hipError_t xent(const float* logits, const int32_t* y, int B, int C, float* loss, float* dlogits, bf16* dlogits_bf16,
                int ld16, hipStream_t s);

// ViT embedding: h0[b][0] = cls + pos[0]; h0[b][t] = e[b][t-1] + pos[t]  (e fp32 [B*(T-1)][D])
hipError_t embed_assemble(const float* e, const bf16* cls, const bf16* pos, float* h0, int B, int T, int D, hipStream_t s);
// drop the CLS rows: out[b*(T-1)+t-1] = bf16(d[b][t]) for t >= 1
hipError_t gather_patch_rows(const float* d, bf16* out, int B, int T, int D, hipStream_t s);
// fill with zeros (a kernel, so that it may be captured in a graph)
hipError_t fill_zero(void* p, size_t bytes, hipStream_t s);
// fp32 -> bf16
hipError_t cast_bf16(const float* in, bf16* out, size_t n, hipStream_t s);

// ------------------------------------------------------------------------------------------
// convolutional workload: NHWC bf16 activations, a convolution is a GEMM over an im2col matrix
// ------------------------------------------------------------------------------------------
struct ConvGeom {
  int B, H, W, C;      // input [B][H][W][C]
  int k, stride, pad;  // square kernel
  int Ho, Wo;          // output size, (H + 2 pad - k) / stride + 1
  int Kc;              // row length of the column matrix: k*k*C rounded up to a multiple of 8
};
// cols[B*Ho*Wo][Kc], column order (ky, kx, c); out-of-image taps and the row tail are zero
hipError_t im2col(const bf16* x, bf16* cols, const ConvGeom& g, hipStream_t s);
// out[B][H][W][C] = (adjoint of im2col applied to dcols  + add) * (mask > 0); add, mask nullable; C % 8 == 0;
// dcols is float32 [B*Ho*Wo][Kc] (dcols_f32) or bf16; the taps are added in float32, the result is rounded once
hipError_t col2im(const void* dcols, bool dcols_f32, const bf16* add, const bf16* mask, bf16* out, const ConvGeom& g,
                  hipStream_t s);
// folded BatchNorm: out = act(z1*g1 + b1 + t), t = z2*g2 + b2 (g2 given), z2 (g2 null) or 0 (z2 null);
// z1 is bf16, or fp32 when z1_f32 is given; rows x C, C % 8 == 0
hipError_t affine_act(const bf16* z1, const float* z1_f32, const bf16* g1, const bf16* b1, const bf16* z2,
                      const bf16* g2, const bf16* b2, bool relu, bf16* out, long long rows, int C, hipStream_t s);
// out[r][c] = d[r][c] * gain[c]
hipError_t scale_cols(const bf16* d, const bf16* gain, bf16* out, long long rows, int C, hipStream_t s);
// out = (a + b) * (mask > 0), n elements (n % 8 == 0); b nullable; out may alias a or b
hipError_t add_mask(const bf16* a, const bf16* b, const bf16* mask, bf16* out, long long n, hipStream_t s,
                    float mask_hi = __builtin_inff());
// stem pooling: y = relu(z*gain + shift) in fp32, then 3x3 / stride 2 / pad 1 maximum, first maximum in
// (ky, kx) order; arg holds the chosen tap (one byte per output element)
hipError_t maxpool3x3s2_fwd(const float* z, const bf16* gain, const bf16* shift, bf16* out, uint8_t* arg, int B, int H,
                            int W, int C, hipStream_t s);
// out[B][H][W][C] = (d routed back to the chosen taps) * (y > 0)
hipError_t maxpool3x3s2_bwd(const bf16* d, const uint8_t* arg, const bf16* y, bf16* out, int B, int H, int W, int C,
                            hipStream_t s);
// p[b][c] = mean over the HW positions; backward: out[b][t][c] = dp[b][c] / HW * (y[b][t][c] > 0)
hipError_t avgpool_fwd(const bf16* x, bf16* p, int B, int HW, int C, hipStream_t s);
hipError_t avgpool_bwd_relu(const bf16* dp, const bf16* y, bf16* out, int B, int HW, int C, hipStream_t s,
                            float mask_hi = __builtin_inff());
// 2x2 / stride 2 max pooling of y [B][H][W][C] (H, W even), first maximum in (dy, dx) order; arg: one byte per output
hipError_t maxpool2x2_fwd(const bf16* y, bf16* out, uint8_t* arg, int B, int H, int W, int C, hipStream_t s);
// out[B][H][W][C] = (d routed back to the chosen tap of its window) * (y > 0)
hipError_t maxpool2x2_bwd(const bf16* d, const uint8_t* arg, const bf16* y, bf16* out, int B, int H, int W, int C,
                          hipStream_t s);
// rows of K elements <-> rows of Kc >= K elements (zero tail)
// 3x3 depthwise convolution, zero padding 1, stride 1 or 2, NHWC, C % 8 == 0, weights [C][9] (bf16):
//   fwd: z (nullable: not kept) = the convolution, rounded; y = clamp(z * gain + shift, 0, 6)
//   dx:  out[B][H][W][C] = (adjoint applied to d [B][Ho][Wo][C] + add) * (0 < relu6_y < 6); add, relu6_y nullable
//   dw:  part[R][C * 9] fp32 partial sums over R = depthwise3x3_dw_rows(..) interleaved pixel subsets; their
//        column sum (colsum over R rows) is the gradient [C][9]
hipError_t depthwise3x3_fwd(const bf16* x, const bf16* w, const bf16* gain, const bf16* shift, bf16* z, bf16* y, int B, int H,
                            int W, int C, int stride, hipStream_t s);
hipError_t depthwise3x3_dx(const bf16* d, const bf16* w, const bf16* add, const bf16* relu6_y, bf16* out, int B, int H, int W,
                           int C, int stride, hipStream_t s);
int depthwise3x3_dw_rows(int B, int H, int W, int C, int stride);
hipError_t depthwise3x3_dw(const bf16* d, const bf16* x, float* part, int B, int H, int W, int C, int stride, hipStream_t s);
// out[rows][N] (bf16) = max(z[rows][N] + bias[N], 0), z fp32; N % 4 == 0
hipError_t bias_relu_rows(const float* z, const bf16* bias, bf16* out, int rows, int N, hipStream_t s);
// out[C][3][3][O] = w[O][3][3][C] with mirrored taps: the weight of the 3x3 convolution that maps an output
// gradient to the input gradient
hipError_t flip3x3(const bf16* w, bf16* out, int O, int C, hipStream_t s);
hipError_t pad_rows(const bf16* in, bf16* out, int rows, int K, int Kc, hipStream_t s);
hipError_t strip_rows(const float* in, float* out, int rows, int K, int Kc, hipStream_t s);
// operands of the stem convolution (7x7 / stride 2 / zero padding 3, C <= 4 input channels) for its gathered GEMM:
// the image padded to [B][Hp][Wp][4] (pixel (h, w) at (h + 3, w + 3)), the weight widened to [O][8][8][4], and the
// float32 weight gradient [O][8][8][4] brought back to [O][7][7][C]
hipError_t stem_pad_image(const bf16* x, bf16* out, int B, int H, int W, int C, int Hp, int Wp, hipStream_t s);
hipError_t stem_pack_weight(const bf16* w, bf16* out, int O, int C, hipStream_t s);
hipError_t stem_unpack_dw(const float* in, float* out, int O, int C, hipStream_t s);
// out[c] = sum_r d[r][c] * z[r][c]   (z bf16, or fp32 when z_f32 is given); same two stages as colsum
hipError_t colsum_mul(const bf16* d, const bf16* z, const float* z_f32, float* out, float* partials, int rows, int cols,
                      hipStream_t s);
// both sums from one read of d: out_sum[c] = sum_r d[r][c], out_mul[c] = sum_r d[r][c] * z[r][c], each identical to
// what colsum / colsum_mul give; partials must hold 2 * colsum_partial_elems(rows, cols) floats
hipError_t colsum_pair(const bf16* d, const bf16* z, const float* z_f32, float* out_sum, float* out_mul, float* partials,
                       int rows, int cols, hipStream_t s);

// ------------------------------------------------------------------------------------------
// importance (Eq. 2) and masked optimizer update over a table of tensors
// ------------------------------------------------------------------------------------------
struct TensorSeg {       // one chunk of one tensor
  const float* g;        // gradient
  const void* w;         // current weights (bf16 or fp32)
  const void* w_snap;    // snapshot
  uint32_t n;            // elements in this chunk
  uint32_t tensor;       // tensor index
};
// stage 1: one block per segment -> partial[seg]; stage 2: per tensor, fixed-order sum -> double
// metric 0: sum g (w_snap - w) (Eq. 2); 1: sum |w|; 2: sum |g| (w_snap is not read for 1 and 2)
hipError_t importance_reduce(const TensorSeg* segs_dev, int n_segs, const uint32_t* seg_begin_dev, int n_tensors,
                             bool bf16_weights, double* partial_dev, double* out_dev, hipStream_t s, int metric = 0);

struct UpdateSeg {
  const float* g;
  void* w;        // model weights (bf16 or fp32)
  float* master;  // fp32 master weights (bf16 models), else null
  float* m;
  float* v;       // Adam only
  uint32_t n;
  uint32_t tensor;
};
struct OptParams {
  int kind;       // 0 Adam, 1 SGDW
  float lr, beta1, beta2, eps, momentum, wd;
  float bc1, bc2; // 1 - beta1^t, 1 - beta2^t
  int dry;        // 1: compute, then store the values that were loaded (timing without side effects)
};
// segs_dev lists the chunks of ALL tensors, selected_dev the indices of the n_selected chunks that belong to
// selected tensors: one workgroup per listed chunk, nothing else is touched
hipError_t masked_update(const UpdateSeg* segs_dev, const uint32_t* selected_dev, int n_selected, bool bf16_weights,
                         OptParams p, hipStream_t s);

}  // namespace et
