// Convolution units shared by the convolutional chains: a convolution is a GEMM over the rows of
// an im2col matrix kept from the forward pass (a 1x1 stride-1 convolution reads the activation
// itself): forward cols * W^T, dw() d^T * cols (split over the rows), dy() d * W followed by the
// gather-form adjoint of im2col.
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

// z = cols(in) * Wm^T; with gain/shift the GEMM epilogue also writes y = max(z * gain + shift, 0)
inline int conv_forward(et_ctx* c, const ConvUnit& u, const bf16* in, const bf16* Wm, void* z, bool z_f32,
                 const bf16* gain = nullptr, const bf16* shift = nullptr, bf16* y = nullptr, const bf16* branch = nullptr,
                 const bf16* gain2 = nullptr, const bf16* shift2 = nullptr) {
  const bf16* A = in;
  if (needs_cols(u)) {
    ET_KB(1, 2.0 * ((double)c->desc.batch * u.H * u.W * u.Cin + (double)rows_of(c, u) * u.Kc),
          et::im2col(in, u.cols, geom(c, u), c->stream));
    A = u.cols;
  }
  et::GemmDesc g = linear_fwd(A, Wm, nullptr, (int)rows_of(c, u), u.Cout, u.Kc);
  g.C = z; g.c_f32 = z_f32;
  if (gain) {
    g.mode = et::EPI_AFFINE_RELU; g.gain = gain; g.bias = shift; g.C2 = y;
    if (branch) {   // the other branch of a block end, inside the same ReLU
      g.mode = et::EPI_AFFINE_ADD_RELU; g.U = branch; g.gain2 = gain2; g.bias2 = shift2;
    }
  }
  ET_G(g);
  return ET_OK;
}

inline int conv_dw(et_ctx* c, const ConvUnit& u, const bf16* in, const bf16* d, float* dW) {
  const bf16* A = needs_cols(u) ? u.cols : in;
  ET_G(linear_dw(c, d, u.Cout, A, u.Kc, dW, (int)rows_of(c, u), u.Cout, u.Kc));
  return ET_OK;
}

// gradient of the column matrix: dcols[M][Kc] = d[M][Cout] * Wm[Cout][Kc]
inline int conv_dcols(et_ctx* c, const ConvUnit& u, const bf16* d, const bf16* Wm, bf16* dcols) {
  et::GemmDesc g = linear_dx(d, Wm, (int)rows_of(c, u), u.Cout, u.Kc);
  g.C = dcols;
  ET_G(g);
  return ET_OK;
}


}  // namespace et_exec
