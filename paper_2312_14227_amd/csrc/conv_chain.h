// Convolution units shared by the convolutional chains: a convolution is a GEMM over the rows of
// an im2col matrix (a 1x1 stride-1 convolution reads the activation itself): forward cols * W^T,
// dw() d^T * cols (split over the rows), dy() d * W followed by the gather-form adjoint of im2col.
// A 3x3 convolution of stride 1 or 2 (and a strided 1x1 one) with channel counts in multiples of 64 never
// writes that matrix: the forward product and dw() gather its rows from the activation inside the GEMM; dy()
// of a stride-1 3x3 convolution is the same kind of convolution of the output gradient with the mirrored
// weight, dy() of the strided ones goes through a float32 column gradient and the adjoint of im2col.
#pragma once
#include "context.h"

namespace et_exec {

// launch of an HBM-bound kernel of this workload: counted, and timed as kernel class 7 with its
// algorithmic bytes (operands read once, results written once)
#define ET_KB(n, bytes, expr)              \
  do {                                     \
    KernelTimer kt__(c, 7, (double)(bytes)); \
    ET_K(n, expr);                         \
  } while (0)

// The per-channel pieces of a folded-BN affine y = z * gain + shift (tensors tg = gain, tg + 1 = shift) on the
// gradient d [M][C] of y: dw(shift) = column sum of d, dw(gain) = column sum of d * z (z bf16, or float32 z32),
// dy(gain): dout = d * gain.  With gain and shift both selected one kernel reads d once for both sums (same
// summation order as the separate kernels, so a tensor's gradient does not depend on its neighbour's selection);
// the profile shares that kernel's time evenly between the two tensors.  dy_used = false skips dy(gain) although
// the chain passes the tensor: a projection shortcut's scaled gradient has no reader when its weight is not selected
// and nothing in front of the block is (the time model then charges a few microseconds that are not spent).
inline int affine_back(et_ctx* c, const uint8_t* mask, int jstar, int tg, const bf16* d, const bf16* z, const float* z32,
                       bf16* dout, long long M, int C, bool dy_used = true) {
  float* cp = c->colsum_partials;
  hipStream_t s = c->stream;
  const double zb = z32 ? 4.0 : 2.0;
  if (mask[tg] && mask[tg + 1]) {
    Region r(c, PH_DW, tg + 1, tg);
    ET_KB(2, (2.0 + zb) * M * C, et::colsum_pair(d, z, z32, c->grad[tg + 1], c->grad[tg], cp, (int)M, C, s));
  } else if (mask[tg + 1]) {
    Region r(c, PH_DW, tg + 1);
    ET_KB(2, 2.0 * M * C, et::colsum(d, nullptr, C, nullptr, 0, nullptr, nullptr, c->grad[tg + 1], cp, (int)M, C, s));
  } else if (mask[tg]) {
    Region r(c, PH_DW, tg);
    ET_KB(2, (2.0 + zb) * M * C, et::colsum_mul(d, z, z32, c->grad[tg], cp, (int)M, C, s));
  }
  if (tg > jstar && dy_used) {
    Region r(c, PH_DY, tg);
    ET_KB(1, 4.0 * M * C, et::scale_cols(d, (const bf16*)c->w[tg], dout, M, C, s));
  }
  return ET_OK;
}

inline et::ConvGeom geom(const et_ctx* c, const ConvUnit& u) {
  et::ConvGeom g;
  g.B = c->desc.batch; g.H = u.H; g.W = u.W; g.C = u.Cin; g.k = u.k; g.stride = u.stride; g.pad = (u.k - 1) / 2;
  g.Ho = u.Ho; g.Wo = u.Wo; g.Kc = u.Kc;
  return g;
}

inline void init_unit(ConvUnit& u, int t, int H, int W, int Cin, int Cout, int k, int stride) {
  u.t = t; u.H = H; u.W = W; u.Cin = Cin; u.Cout = Cout; u.k = k; u.stride = stride;
  const int pad = (k - 1) / 2;
  u.Ho = (H + 2 * pad - k) / stride + 1;
  u.Wo = (W + 2 * pad - k) / stride + 1;
  u.Kc = round8(k * k * Cin);
  u.in = nullptr; u.cols = nullptr; u.z = nullptr; u.y = nullptr;
}

inline size_t rows_of(const et_ctx* c, const ConvUnit& u) { return (size_t)c->desc.batch * u.Ho * u.Wo; }
inline bool needs_cols(const ConvUnit& u) { return u.k > 1 || u.stride > 1; }
// which of the three products of a unit run as implicit GEMMs
// (3x3 of stride 1 or 2 and strided 1x1 convolutions gather their rows inside the GEMM)
inline bool gathered_kind(const ConvUnit& u) { return (u.k == 3 && (u.stride == 1 || u.stride == 2)) || (u.k == 1 && u.stride == 2); }
inline bool implicit_fwd(const ConvUnit& u) { return gathered_kind(u) && (u.Cin % 64) == 0; }
inline bool implicit_dy(const ConvUnit& u) { return u.k == 3 && u.stride == 1 && (u.Cout % 64) == 0 && (u.Cin % 8) == 0; }
inline bool implicit_dw(const et_ctx* c, const ConvUnit& u) {
  return gathered_kind(u) && (u.Cin % 8) == 0 && ((size_t)c->desc.batch * u.Ho * u.Wo) % 64 == 0 && u.H < 4096 && u.W < 4096;
}
// tile and split of a unit's implicit forward (or, with the channel roles exchanged, gradient-passing) product
inline void plan_implicit(et_ctx* c, et::GemmDesc& g) {
  et::gemm_bf16_plan_conv(g.M, g.N, g.K, &g.tile, &g.split_k);
  g.partials = c->gemm_partials;
  if (et::gemm_bf16_partial_elems(g.M, g.N, g.split_k) > c->gemm_partial_elems) g.split_k = 1;
}
inline size_t conv_split_partials(const et_ctx* c, const ConvUnit& u) {
  size_t n = 0;
  int tile, split;
  const int M = (int)rows_of(c, u);
  if (implicit_fwd(u)) {
    et::gemm_bf16_plan_conv(M, u.Cout, u.k * u.k * u.Cin, &tile, &split);
    n = std::max(n, et::gemm_bf16_partial_elems(M, u.Cout, split));
  }
  if (implicit_dy(u)) {
    et::gemm_bf16_plan_conv(M, u.Cin, 9 * u.Cout, &tile, &split);
    n = std::max(n, et::gemm_bf16_partial_elems(M, u.Cin, split));
  }
  return n;
}
// fp32 partial elements of a unit's weight gradient with the split its plan chooses
inline size_t conv_dw_partials(const et_ctx* c, const ConvUnit& u) {
  const int M = (int)rows_of(c, u);
  int tile, split;
  if (implicit_dw(c, u)) {
    et::gemm_bf16_plan_conv_dw(u.Cout, u.k * u.k * u.Cin, M, &tile, &split);
    return et::gemm_bf16_partial_elems(u.Cout, u.k * u.k * u.Cin, split);
  }
  return et::gemm_bf16_partial_elems(u.Cout, u.Kc, split_for(u.Cout, u.Kc, M));
}

// z = cols(in) * Wm^T; with gain/shift the GEMM epilogue also writes y = max(z * gain + shift, 0)
inline int conv_forward(et_ctx* c, const ConvUnit& u, const bf16* in, const bf16* Wm, void* z, bool z_f32,
                 const bf16* gain = nullptr, const bf16* shift = nullptr, bf16* y = nullptr, const bf16* branch = nullptr,
                 const bf16* gain2 = nullptr, const bf16* shift2 = nullptr) {
  const bf16* A = in;
  if (needs_cols(u) && !implicit_fwd(u)) {
    ET_KB(1, 2.0 * ((double)c->desc.batch * u.H * u.W * u.Cin + (double)rows_of(c, u) * u.Kc),
          et::im2col(in, u.cols, geom(c, u), c->stream));
    A = u.cols;
  }
  et::GemmDesc g = linear_fwd(A, Wm, nullptr, (int)rows_of(c, u), u.Cout, u.Kc);
  if (implicit_fwd(u)) { g.conv_h = u.H; g.conv_w = u.W; g.conv_c = u.Cin; g.conv_taps = u.k; g.conv_stride = u.stride; }
  g.C = z; g.c_f32 = z_f32;
  if (gain) {
    g.mode = et::EPI_AFFINE_RELU; g.gain = gain; g.bias = shift; g.C2 = y;
    if (branch) {   // the other branch of a block end, inside the same ReLU
      g.mode = et::EPI_AFFINE_ADD_RELU; g.U = branch; g.gain2 = gain2; g.bias2 = shift2;
    }
  }
  if (implicit_fwd(u) && !z_f32 && !branch) plan_implicit(c, g);
  ET_G(g);
  return ET_OK;
}

inline int conv_dw(et_ctx* c, const ConvUnit& u, const bf16* in, const bf16* d, float* dW) {
  if (implicit_dw(c, u)) {   // B operand: the activation standing for its im2col matrix
    et::GemmDesc g;
    const int kk = u.k * u.k * u.Cin;
    g.A = d; g.a_t = true; g.lda = u.Cout; g.B = in; g.b_t = true; g.ldb = kk;
    g.M = u.Cout; g.N = kk; g.K = (int)rows_of(c, u);
    g.C = dW; g.ldc = kk; g.c_f32 = true;
    g.conv_h = u.H; g.conv_w = u.W; g.conv_c = u.Cin; g.conv_taps = u.k; g.conv_stride = u.stride;
    et::gemm_bf16_plan_conv_dw(g.M, g.N, g.K, &g.tile, &g.split_k);
    g.partials = c->gemm_partials;
    if (et::gemm_bf16_partial_elems(g.M, g.N, g.split_k) > c->gemm_partial_elems) g.split_k = 1;
    ET_G(g);
    return ET_OK;
  }
  if (implicit_fwd(u)) {     // the im2col matrix exists only here, in the shared column buffer
    ET_KB(1, 2.0 * ((double)c->desc.batch * u.H * u.W * u.Cin + (double)rows_of(c, u) * u.Kc),
          et::im2col(in, c->rdcols, geom(c, u), c->stream));
    ET_G(linear_dw(c, d, u.Cout, c->rdcols, u.Kc, dW, (int)rows_of(c, u), u.Cout, u.Kc));
    return ET_OK;
  }
  const bf16* A = needs_cols(u) ? u.cols : in;
  ET_G(linear_dw(c, d, u.Cout, A, u.Kc, dW, (int)rows_of(c, u), u.Cout, u.Kc));
  return ET_OK;
}

// Gradient of the column matrix: dcols[M][Kc] = d[M][Cout] * Wm[Cout][Kc].  For a 1x1 convolution this is the
// input gradient itself, stored as bf16 like every tensor handed from one operation to the next.  For a larger
// kernel it is an intermediate whose shifted copies the adjoint of im2col has yet to add: it stays float32, so
// that the input gradient is rounded once, after the sum, as in the implicit-GEMM form of the same operation.
inline bool dcols_f32(const ConvUnit& u) { return u.k > 1; }
inline size_t dcols_bytes(const et_ctx* c, const ConvUnit& u) { return rows_of(c, u) * u.Kc * (dcols_f32(u) ? 4 : 2); }
inline int conv_dcols(et_ctx* c, const ConvUnit& u, const bf16* d, const bf16* Wm, void* dcols) {
  et::GemmDesc g = linear_dx(d, Wm, (int)rows_of(c, u), u.Cout, u.Kc);
  g.C = dcols;
  g.c_f32 = dcols_f32(u);
  ET_G(g);
  return ET_OK;
}


// dy() of a 3x3 / stride 1 unit as an implicit GEMM: out = (convolution of d with the mirrored weight), times
// the ReLU mask (relu_y > 0) if given; c->wflip receives the mirrored weight [Cin][3][3][Cout]
inline int conv_dy_implicit(et_ctx* c, const ConvUnit& u, const bf16* d, const bf16* W, const bf16* relu_y, bf16* out) {
  ET_K(1, et::flip3x3(W, c->wflip, u.Cout, u.Cin, c->stream));
  et::GemmDesc g = linear_fwd(d, c->wflip, nullptr, (int)rows_of(c, u), u.Cin, 9 * u.Cout);
  g.conv_h = u.H; g.conv_w = u.W; g.conv_c = u.Cout;
  g.C = out;
  if (relu_y) { g.mode = et::EPI_RELU_MASK; g.U = relu_y; }
  plan_implicit(c, g);
  ET_G(g);
  return ET_OK;
}

}  // namespace et_exec
