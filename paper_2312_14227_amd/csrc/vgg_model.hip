// Plain convolution stack (VGG family) on the tensor-level chain (Sections 2.3 and 5).  Every
// convolution and linear layer is two tensors, Kernel and Bias (Section 5.1).  The backward pass
// carries the gradient w.r.t. the pre-activation of the layer being visited: a bias's dw() is
// its column sum and its dy() the identity (t_dy = 0); a kernel's dw() is d^T * (layer input)
// and its dy() passes d to the layer input and on through the operations without weights in
// front of it (ReLU, 2x2 max pooling, flattening) to the pre-activation of the previous layer.
//
// Bias and ReLU are the epilogue of the layer's GEMM, applied to the unrounded sum; the
// pre-activation itself is never stored (the ReLU mask is read from the stored activation).
//
// A convolution whose input channels come in multiples of 64 runs as an implicit GEMM: the
// forward product gathers the im2col rows from the activation, and dy() is the same kind of
// convolution of the output gradient with the mirrored weight, its epilogue applying the ReLU
// mask of the previous layer; dw() gathers the same rows as the B operand of d^T * cols, reduced
// over the pixels.  The im2col matrix of such a layer is never written.  Other convolutions (the
// first one) keep the matrix from the forward pass and pass the gradient through d * W and the
// adjoint of im2col.
#include "conv_chain.h"

namespace {

// weight matrix of convolution i as the GEMM reads it (the first one is padded to 16-byte rows)
inline const bf16* conv_matrix(const et_ctx* c, size_t i) {
  const ConvUnit& u = c->vconv[i];
  return u.Kc == 9 * u.Cin ? (const bf16*)c->w[u.t] : c->stem_w8;
}

// A hidden linear layer on a small batch is one row of output tiles streaming the whole weight
// matrix: split over the input features so that every CU streams a part, then reduce, add the
// bias and apply the ReLU (the same single rounding as the fused epilogue).
inline int fc_split(int batch, int out, int in) {
  if (batch > 128) return 1;
  int tile, split;
  et::gemm_bf16_plan_split(batch, out, in, &tile, &split);
  return split;
}

}  // namespace

int build_vgg(et_ctx* c) {
  const et_model_desc& d = c->desc;
  if (d.dtype != ET_BF16 || d.batch < 1 || d.in_ch < 1 || d.n_stages < 1 || d.n_stages > ET_MAX_STAGES) return ET_EINVAL;
  if (d.n_layers < 0 || d.n_layers > ET_MAX_MLP_LAYERS || d.classes < 8 || (d.classes % 8)) return ET_EINVAL;
  if (d.image < (1 << d.n_stages) || (d.image % (1 << d.n_stages))) return ET_EINVAL;
  for (int s = 0; s < d.n_stages; s++)
    if (d.stage_blocks[s] < 1 || d.planes[s] < 8 || (d.planes[s] % 8)) return ET_EINVAL;
  for (int j = 0; j < d.n_layers; j++)
    if (d.dims[j] < 8 || (d.dims[j] % 8)) return ET_EINVAL;
  auto add = [&](const std::string& n, size_t numel) { c->tensors.push_back({n, numel, ET_BF16}); };
  const size_t B = d.batch, b16 = sizeof(bf16), f32 = sizeof(float);

  int H = d.image, Cin = d.in_ch, t = 0;
  for (int s = 0; s < d.n_stages; s++) {
    for (int k = 0; k < d.stage_blocks[s]; k++) {
      ConvUnit u;
      init_unit(u, t, H, H, Cin, d.planes[s], 3, 1);
      const std::string pre = "conv" + std::to_string(c->vconv.size()) + ".";
      add(pre + "W", (size_t)u.Cout * 9 * Cin);
      add(pre + "b", u.Cout);
      c->vconv.push_back(u);
      c->vstage.push_back(s);
      Cin = u.Cout;
      t += 2;
    }
    H /= 2;
  }
  const int feat = H * H * Cin, n_fc = d.n_layers + 1;
  c->vdims.assign(1, feat);
  for (int j = 0; j < d.n_layers; j++) c->vdims.push_back(d.dims[j]);
  c->vdims.push_back(d.classes);
  for (int j = 0; j < n_fc; j++) {
    add("fc" + std::to_string(j) + ".W", (size_t)c->vdims[j + 1] * c->vdims[j]);
    add("fc" + std::to_string(j) + ".b", c->vdims[j + 1]);
  }

  // ---- workspace
  size_t max_act = 0, max_cols = 0, max_cs = 0, pe = 0, max_flip = 8, dcols_b = 16;
  c->vpool.assign(d.n_stages, nullptr);
  c->varg.assign(d.n_stages, nullptr);
  for (size_t i = 0; i < c->vconv.size(); i++) {
    ConvUnit& u = c->vconv[i];
    const size_t M = rows_of(c, u);
    if (!implicit_fwd(u)) reserve(c, &u.cols, b16 * M * u.Kc);
    if (implicit_dy(u)) max_flip = std::max(max_flip, (size_t)u.Cout * 9 * u.Cin);
    reserve(c, &u.y, b16 * M * u.Cout);
    max_act = std::max(max_act, std::max(M * u.Cout, M * round8(u.Cin)));
    if (!implicit_dw(c, u) || !implicit_dy(u)) max_cols = std::max(max_cols, M * u.Kc);
    if (i > 0 && !implicit_dy(u)) dcols_b = std::max(dcols_b, dcols_bytes(c, u));   // conv0 passes nothing on
    max_cs = std::max(max_cs, et::colsum_partial_elems((int)M, u.Cout));
    pe = std::max(pe, std::max(conv_dw_partials(c, u), conv_split_partials(c, u)));
    const bool last_of_stage = i + 1 == c->vconv.size() || c->vstage[i + 1] != c->vstage[i];
    if (last_of_stage) {
      reserve(c, &c->vpool[c->vstage[i]], b16 * (M / 4) * u.Cout);
      reserve(c, &c->varg[c->vstage[i]], (M / 4) * u.Cout);
    }
  }
  {
    const ConvUnit& u = c->vconv[0];
    reserve(c, &c->stem_w8, b16 * (size_t)u.Cout * u.Kc);
    reserve(c, &c->stem_dw8, f32 * (size_t)u.Cout * u.Kc);
  }
  c->vact.assign(n_fc, nullptr);   // vact[0]: the last pooled output (set by the forward pass)
  for (int j = 1; j < n_fc; j++) reserve(c, &c->vact[j], b16 * B * c->vdims[j]);
  size_t max_fc = 8;
  for (int j = 0; j + 1 < n_fc; j++) {
    const int sp = fc_split(d.batch, c->vdims[j + 1], c->vdims[j]);
    if (sp > 1) {
      max_fc = std::max(max_fc, B * (size_t)c->vdims[j + 1]);
      pe = std::max(pe, et::gemm_bf16_partial_elems(d.batch, c->vdims[j + 1], sp));
    }
  }
  reserve(c, &c->fc_z32, f32 * max_fc);
  for (int j = 0; j < n_fc; j++) {
    max_act = std::max(max_act, B * (size_t)std::max(c->vdims[j], c->vdims[j + 1]));
    max_cs = std::max(max_cs, et::colsum_partial_elems((int)B, c->vdims[j + 1]));
    pe = std::max(pe, et::gemm_bf16_partial_elems(c->vdims[j + 1], c->vdims[j], split_for(c->vdims[j + 1], c->vdims[j], (int)B)));
  }
  const int C = d.classes;
  reserve(c, &c->logits, f32 * B * C);
  reserve(c, &c->dlogits, f32 * B * C);
  reserve(c, &c->dl16, b16 * B * C);
  reserve(c, &c->loss, 256 + sizeof(float) * (size_t)d.batch);
  for (int i = 0; i < 3; i++) reserve(c, &c->rd[i], b16 * max_act);
  reserve(c, &c->rdcols, std::max(b16 * std::max<size_t>(max_cols, 8), dcols_b));
  reserve(c, &c->wflip, b16 * max_flip);
  c->gemm_partial_elems = pe;
  reserve(c, &c->gemm_partials, f32 * std::max<size_t>(pe, 64));
  reserve(c, &c->colsum_partials, f32 * std::max<size_t>(max_cs, 64));
  // every matrix dimension and element count below is handled as int by the GEMM
  if (max_act > 0x7fffffffull || max_cols > 0x7fffffffull) return ET_EINVAL;
  return ET_OK;
}

int vgg_forward(et_ctx* c, const void* x, const int32_t* y) {
  const et_model_desc& d = c->desc;
  Region r(c, PH_FWD, -1);
  hipStream_t s = c->stream;
  auto Wt = [&](int i) { return (const bf16*)c->w[i]; };
  const int B = d.batch;
  const bf16* h = (const bf16*)x;
  for (size_t i = 0; i < c->vconv.size(); i++) {
    ConvUnit& u = c->vconv[i];
    const size_t M = rows_of(c, u);
    u.in = h;
    if (u.Kc != 9 * u.Cin) ET_K(1, et::pad_rows(Wt(u.t), c->stem_w8, u.Cout, 9 * u.Cin, u.Kc, s));
    et::GemmDesc g = linear_fwd(u.cols, conv_matrix(c, i), Wt(u.t + 1), (int)M, u.Cout, u.Kc);
    g.mode = et::EPI_BIAS_RELU; g.C = u.y;
    if (implicit_fwd(u)) {
      g.A = h; g.conv_h = u.H; g.conv_w = u.W; g.conv_c = u.Cin;
      plan_implicit(c, g);
    } else {
      ET_KB(1, 2.0 * ((double)M * u.Cin + (double)M * u.Kc), et::im2col(h, u.cols, geom(c, u), s));
    }
    ET_G(g);
    h = u.y;
    if (i + 1 == c->vconv.size() || c->vstage[i + 1] != c->vstage[i]) {
      const int st = c->vstage[i];
      ET_KB(1, 2.0 * M * u.Cout + 3.0 * (M / 4) * u.Cout, et::maxpool2x2_fwd(u.y, c->vpool[st], c->varg[st], B, u.Ho, u.Wo, u.Cout, s));
      h = c->vpool[st];
    }
  }
  c->vact[0] = const_cast<bf16*>(h);   // flattened in (h, w, c) order: the pooled tensor as it lies in memory
  const int n_fc = (int)c->vdims.size() - 1, t_fc = 2 * (int)c->vconv.size();
  for (int j = 0; j < n_fc; j++) {
    et::GemmDesc g = linear_fwd(c->vact[j], Wt(t_fc + 2 * j), Wt(t_fc + 2 * j + 1), B, c->vdims[j + 1], c->vdims[j]);
    const int sp = j + 1 < n_fc ? fc_split(B, c->vdims[j + 1], c->vdims[j]) : 1;
    if (sp > 1 && et::gemm_bf16_partial_elems(B, c->vdims[j + 1], sp) <= c->gemm_partial_elems) {
      g.bias = nullptr; g.C = c->fc_z32; g.c_f32 = true; g.split_k = sp; g.partials = c->gemm_partials;
      ET_G(g);
      ET_K(1, et::bias_relu_rows(c->fc_z32, Wt(t_fc + 2 * j + 1), c->vact[j + 1], B, c->vdims[j + 1], s));
      continue;
    }
    if (j + 1 < n_fc) {
      g.mode = et::EPI_BIAS_RELU; g.C = c->vact[j + 1];
    } else {
      g.C = c->logits; g.c_f32 = true;
    }
    ET_G(g);
  }
  ET_K(2, et::xent(c->logits, y, B, d.classes, c->loss, c->dlogits, c->dl16, d.classes, s));
  return ET_OK;
}

int vgg_backward(et_ctx* c, const void* x, const uint8_t* mask) {
  const et_model_desc& md = c->desc;
  const int N = (int)c->tensors.size(), B = md.batch;
  int jstar = -1;
  for (int j = 0; j < N; j++)
    if (mask[j]) { jstar = j; break; }
  if (jstar < 0) return ET_OK;
  auto Wt = [&](int i) { return (const bf16*)c->w[i]; };
  auto sel = [&](int j) { return mask[j] != 0; };
  auto pass = [&](int j) { return j > jstar; };
  hipStream_t s = c->stream;
  float* cp = c->colsum_partials;
  const int n_fc = (int)c->vdims.size() - 1, n_conv = (int)c->vconv.size(), t_fc = 2 * n_conv;
  int rc;

  // d: gradient w.r.t. the pre-activation of the layer being visited (bf16), ping-pong in rd[0..1]
  const bf16* dcur = nullptr;
  int slot = 0;
  auto next_buf = [&]() { slot ^= 1; return c->rd[slot]; };

  // ---- linear layers, output side first
  for (int j = n_fc - 1; j >= 0; j--) {
    const int tw = t_fc + 2 * j, in = c->vdims[j], out = c->vdims[j + 1];
    const bool last = j == n_fc - 1;
    const bf16* dmat = last ? c->dl16 : dcur;   // the matrix products read the bf16 copy of the logit gradient
    if (jstar > tw + 1) return ET_OK;
    if (sel(tw + 1)) {
      Region r(c, PH_DW, tw + 1);
      if (last) ET_K(2, et::colsum(nullptr, c->dlogits, out, nullptr, 0, nullptr, nullptr, c->grad[tw + 1], cp, B, out, s));
      else ET_K(2, et::colsum(dcur, nullptr, out, nullptr, 0, nullptr, nullptr, c->grad[tw + 1], cp, B, out, s));
    }
    if (sel(tw)) {
      Region r(c, PH_DW, tw);
      ET_G(linear_dw(c, dmat, out, c->vact[j], in, c->grad[tw], B, out, in));
    }
    if (pass(tw)) {
      Region r(c, PH_DY, tw);
      et::GemmDesc g = linear_dx(dmat, Wt(tw), B, out, in);
      g.C = c->rd[2];
      ET_G(g);
      bf16* dn = next_buf();
      if (j > 0) {   // ReLU of the previous linear layer
        ET_KB(1, 6.0 * B * in, et::add_mask(c->rd[2], nullptr, c->vact[j], dn, (long long)B * in, s));
      } else {       // un-flatten, last max pooling, ReLU of the last convolution
        const ConvUnit& u = c->vconv[n_conv - 1];
        const double n = (double)rows_of(c, u) * u.Cout;
        ET_KB(1, 3.0 * n / 4 + 4.0 * n, et::maxpool2x2_bwd(c->rd[2], c->varg[c->vstage[n_conv - 1]], u.y, dn, B, u.Ho, u.Wo, u.Cout, s));
      }
      dcur = dn;
    }
  }

  // ---- convolutions
  for (int i = n_conv - 1; i >= 0; i--) {
    const ConvUnit& u = c->vconv[i];
    const int t = u.t;
    if (jstar > t + 1) return ET_OK;
    const long long M = (long long)rows_of(c, u);
    if (sel(t + 1)) {
      Region r(c, PH_DW, t + 1);
      ET_KB(2, 2.0 * M * u.Cout, et::colsum(dcur, nullptr, u.Cout, nullptr, 0, nullptr, nullptr, c->grad[t + 1], cp, (int)M, u.Cout, s));
    }
    if (sel(t)) {
      Region r(c, PH_DW, t);
      if (u.Kc == 9 * u.Cin) {
        if ((rc = conv_dw(c, u, u.in, dcur, c->grad[t])) != ET_OK) return rc;
      } else {
        if ((rc = conv_dw(c, u, u.in, dcur, c->stem_dw8)) != ET_OK) return rc;
        ET_K(1, et::strip_rows(c->stem_dw8, c->grad[t], u.Cout, 9 * u.Cin, u.Kc, s));
      }
    }
    if (pass(t)) {   // i > 0 here: tensor 0 is never passed
      Region r(c, PH_DY, t);
      const ConvUnit& p = c->vconv[i - 1];
      bf16* dn = next_buf();
      const double nin = (double)M * u.Cin;
      const bool same_stage = c->vstage[i - 1] == c->vstage[i];
      if (implicit_dy(u)) {
        // input gradient = 3x3 convolution of d with the mirrored weight [Cin][3][3][Cout]
        if ((rc = conv_dy_implicit(c, u, dcur, Wt(t), same_stage ? p.y : nullptr, same_stage ? dn : c->rd[2])) != ET_OK) return rc;
        if (!same_stage)
          ET_KB(1, 3.0 * nin + 16.0 * nin, et::maxpool2x2_bwd(c->rd[2], c->varg[c->vstage[i - 1]], p.y, dn, B, p.Ho, p.Wo, p.Cout, s));
        dcur = dn;
        continue;
      }
      if ((rc = conv_dcols(c, u, dcur, conv_matrix(c, i), c->rdcols)) != ET_OK) return rc;
      if (same_stage) {
        ET_KB(1, (dcols_f32(u) ? 4.0 : 2.0) * M * u.Kc + 4.0 * nin, et::col2im(c->rdcols, dcols_f32(u), nullptr, p.y, dn, geom(c, u), s));
      } else {       // a pooling layer sits in between
        ET_KB(1, (dcols_f32(u) ? 4.0 : 2.0) * M * u.Kc + 2.0 * nin, et::col2im(c->rdcols, dcols_f32(u), nullptr, nullptr, c->rd[2], geom(c, u), s));
        ET_KB(1, 3.0 * nin + 16.0 * nin, et::maxpool2x2_bwd(c->rd[2], c->varg[c->vstage[i - 1]], p.y, dn, B, p.Ho, p.Wo, p.Cout, s));
      }
      dcur = dn;
    }
  }
  (void)x;
  return ET_OK;
}
