// Inverted-residual network (MobileNetV2 family) on the tensor-level chain (Sections 2.3 and 5).
// Every convolution is followed by a folded BatchNorm (per-channel affine), so it contributes
// the tensors W, g, b; per block the chain is [exp.W, exp.g, exp.b,] dw.W, dw.g, dw.b, proj.W,
// proj.g, proj.b.  ReLU6 follows the stem, the expansion, the depthwise and the last
// convolution; the projection ends without an activation and a stride-1 block of equal widths
// adds its input to its output.  From the output side the gradient of such a block's output
// enters the projection's affine and is also kept (rdsum) until dy() of the block's first
// weight, where it joins the gradient that came through the main branch.
//
// The 1x1 convolutions are GEMMs over the activation rows, with the affine and the activation
// (or the shortcut sum) as the epilogue; the depthwise convolutions have no reduction over
// channels to feed a matrix unit and are direct HBM-bound kernels (8 channels per thread).
#include "conv_chain.h"

namespace {

constexpr float kInf = __builtin_inff();

inline size_t rows_in(const et_ctx* c, const MbBlockBufs& b) { return (size_t)c->desc.batch * b.H * b.W; }
inline size_t rows_out(const et_ctx* c, const MbBlockBufs& b) { return (size_t)c->desc.batch * b.Ho * b.Wo; }

// y = clamp(z * gain + shift [+ branch], lo, hi) with z = X * W^T as the GEMM's epilogue
int pointwise_forward(et_ctx* c, const bf16* X, const bf16* W, int M, int N, int K, bf16* z, const bf16* gain,
                      const bf16* shift, bf16* y, float lo, float hi, const bf16* branch = nullptr) {
  et::GemmDesc g = linear_fwd(X, W, nullptr, M, N, K);
  g.C = z;
  g.mode = et::EPI_AFFINE_RELU; g.gain = gain; g.bias = shift; g.C2 = y; g.act_lo = lo; g.act_hi = hi;
  if (branch) { g.mode = et::EPI_AFFINE_ADD_RELU; g.U = branch; }
  ET_G(g);
  return ET_OK;
}

}  // namespace

int build_mobilenet(et_ctx* c) {
  const et_model_desc& d = c->desc;
  auto mult8 = [](int v) { return v >= 8 && (v % 8) == 0; };
  if (d.dtype != ET_BF16 || d.batch < 1 || d.image < 2 || d.in_ch < 1 || d.n_stages < 1 || d.n_stages > ET_MAX_STAGES)
    return ET_EINVAL;
  if (!mult8(d.stem) || !mult8(d.last) || !mult8(d.classes)) return ET_EINVAL;
  for (int s = 0; s < d.n_stages; s++)
    if (d.stage_blocks[s] < 1 || !mult8(d.planes[s]) || d.expand[s] < 1 || (d.strides[s] != 1 && d.strides[s] != 2))
      return ET_EINVAL;
  auto add = [&](const std::string& n, size_t numel) { c->tensors.push_back({n, numel, ET_BF16}); };
  const size_t B = d.batch, b16 = sizeof(bf16), f32 = sizeof(float);

  init_unit(c->stem, 0, d.image, d.image, d.in_ch, d.stem, 3, 2);
  add("stem.W", (size_t)d.stem * 9 * d.in_ch); add("stem.g", d.stem); add("stem.b", d.stem);
  int H = c->stem.Ho, W = c->stem.Wo, Cin = d.stem, t = 3, bi = 0;
  for (int s = 0; s < d.n_stages; s++)
    for (int k = 0; k < d.stage_blocks[s]; k++, bi++) {
      MbBlockBufs b = {};
      b.Cin = Cin; b.hid = Cin * d.expand[s]; b.Cout = d.planes[s]; b.stride = k == 0 ? d.strides[s] : 1;
      b.H = H; b.W = W; b.Ho = (H - 1) / b.stride + 1; b.Wo = (W - 1) / b.stride + 1;
      b.expand = d.expand[s] != 1; b.shortcut = b.stride == 1 && Cin == b.Cout;
      b.t = t;
      const std::string pre = "b" + std::to_string(bi) + ".";
      if (b.expand) {
        add(pre + "exp.W", (size_t)b.hid * Cin); add(pre + "exp.g", b.hid); add(pre + "exp.b", b.hid);
        t += 3;
      }
      b.t_dw = t;
      add(pre + "dw.W", (size_t)b.hid * 9); add(pre + "dw.g", b.hid); add(pre + "dw.b", b.hid);
      add(pre + "proj.W", (size_t)b.Cout * b.hid); add(pre + "proj.g", b.Cout); add(pre + "proj.b", b.Cout);
      t += 6;
      c->mblk.push_back(b);
      H = b.Ho; W = b.Wo; Cin = b.Cout;
    }
  init_unit(c->mlast, t, H, W, Cin, d.last, 1, 1);
  add("last.W", (size_t)d.last * Cin); add("last.g", d.last); add("last.b", d.last);
  const int C = d.classes;
  add("head.W", (size_t)C * d.last); add("head.b", C);

  // ---- workspace
  size_t max_act = 0, max_cs = 0, pe = 0, max_dwp = 64;
  auto act = [&](size_t rows, size_t ch) {
    max_act = std::max(max_act, rows * ch);
    max_cs = std::max(max_cs, 2 * et::colsum_partial_elems((int)rows, (int)ch));   // (gain and shift sums in one launch)
  };
  auto wgrad = [&](int out, int in, size_t rows) {
    pe = std::max(pe, et::gemm_bf16_partial_elems(out, in, split_for(out, in, (int)rows)));
  };
  {
    ConvUnit& u = c->stem;
    const size_t M = rows_of(c, u);
    reserve(c, &u.cols, b16 * M * u.Kc);
    reserve(c, &u.z, b16 * M * u.Cout);
    reserve(c, &u.y, b16 * M * u.Cout);
    reserve(c, &c->stem_w8, b16 * (size_t)u.Cout * u.Kc);
    reserve(c, &c->stem_dw8, f32 * (size_t)u.Cout * u.Kc);
    act(M, u.Cout);
    wgrad(u.Cout, u.Kc, M);
  }
  for (MbBlockBufs& b : c->mblk) {
    const size_t Mi = rows_in(c, b), Mo = rows_out(c, b);
    if (b.expand) {
      reserve(c, &b.z_exp, b16 * Mi * b.hid);
      reserve(c, &b.y_exp, b16 * Mi * b.hid);
      act(Mi, b.hid);
      wgrad(b.hid, b.Cin, Mi);
    }
    reserve(c, &b.z_dw, b16 * Mo * b.hid);
    reserve(c, &b.y_dw, b16 * Mo * b.hid);
    reserve(c, &b.z_proj, b16 * Mo * b.Cout);
    reserve(c, &b.y, b16 * Mo * b.Cout);
    act(Mo, b.hid);
    act(Mo, b.Cout);
    act(Mi, b.Cin);
    wgrad(b.Cout, b.hid, Mo);
    const int R = et::depthwise3x3_dw_rows(d.batch, b.H, b.W, b.hid, b.stride);
    max_dwp = std::max(max_dwp, (size_t)R * b.hid * 9);
    max_cs = std::max(max_cs, et::colsum_partial_elems(R, b.hid * 9));
  }
  {
    ConvUnit& u = c->mlast;
    const size_t M = rows_of(c, u);
    reserve(c, &u.z, b16 * M * u.Cout);
    reserve(c, &u.y, b16 * M * u.Cout);
    act(M, u.Cout);
    wgrad(u.Cout, u.Cin, M);
  }
  reserve(c, &c->zc, b16 * B * d.last);
  reserve(c, &c->logits, f32 * B * C);
  reserve(c, &c->dlogits, f32 * B * C);
  reserve(c, &c->dl16, b16 * B * C);
  reserve(c, &c->loss, 256 + sizeof(float) * (size_t)d.batch);
  reserve(c, &c->dz, b16 * B * d.last);
  max_cs = std::max(max_cs, et::colsum_partial_elems((int)B, C));
  wgrad(C, d.last, B);
  for (int i = 0; i < 3; i++) reserve(c, &c->rd[i], b16 * max_act);
  reserve(c, &c->rdsum, b16 * max_act);
  reserve(c, &c->dw_part, f32 * max_dwp);
  c->gemm_partial_elems = pe;
  reserve(c, &c->gemm_partials, f32 * std::max<size_t>(pe, 64));
  reserve(c, &c->colsum_partials, f32 * std::max<size_t>(max_cs, 64));
  // every matrix dimension and element count below is handled as int by the GEMM
  if (max_act > 0x7fffffffull || rows_of(c, c->stem) * c->stem.Kc > 0x7fffffffull || max_dwp > 0x7fffffffull) return ET_EINVAL;
  return ET_OK;
}

int mobilenet_forward(et_ctx* c, const void* x, const int32_t* y, const uint8_t* mask) {
  const et_model_desc& d = c->desc;
  Region r(c, PH_FWD, -1);
  hipStream_t s = c->stream;
  auto Wt = [&](int i) { return (const bf16*)c->w[i]; };
  // a convolution's output z is read again only by the gradient of its gain
  auto keep = [&](bf16* z, int gain_index) -> bf16* { return (!mask || mask[gain_index]) ? z : nullptr; };
  const int B = d.batch;
  int rc;
  {  // stem: 3x3 / stride 2 convolution over the im2col matrix (rows padded to 16 bytes), affine, ReLU6
    ConvUnit& u = c->stem;
    const size_t M = rows_of(c, u);
    ET_K(1, et::pad_rows(Wt(0), c->stem_w8, u.Cout, 9 * u.Cin, u.Kc, s));
    ET_KB(1, 2.0 * ((double)B * u.H * u.W * u.Cin + (double)M * u.Kc), et::im2col((const bf16*)x, u.cols, geom(c, u), s));
    if ((rc = pointwise_forward(c, u.cols, c->stem_w8, (int)M, u.Cout, u.Kc, keep(u.z, 1), Wt(1), Wt(2), u.y, 0.f, 6.f)) != ET_OK)
      return rc;
  }
  const bf16* h = c->stem.y;
  for (MbBlockBufs& b : c->mblk) {
    const int t = b.t, td = b.t_dw;
    const size_t Mi = rows_in(c, b), Mo = rows_out(c, b);
    b.x = h;
    const bf16* a = h;
    if (b.expand) {
      if ((rc = pointwise_forward(c, h, Wt(t), (int)Mi, b.hid, b.Cin, keep(b.z_exp, t + 1), Wt(t + 1), Wt(t + 2), b.y_exp, 0.f, 6.f)) != ET_OK)
        return rc;
      a = b.y_exp;
    }
    ET_KB(1, 2.0 * ((double)Mi * b.hid + 2.0 * Mo * b.hid),
          et::depthwise3x3_fwd(a, Wt(td), Wt(td + 1), Wt(td + 2), keep(b.z_dw, td + 1), b.y_dw, B, b.H, b.W, b.hid, b.stride, s));
    // projection: affine without activation, plus the block input where the shortcut exists
    if ((rc = pointwise_forward(c, b.y_dw, Wt(td + 3), (int)Mo, b.Cout, b.hid, keep(b.z_proj, td + 4), Wt(td + 4), Wt(td + 5), b.y,
                                -kInf, kInf, b.shortcut ? h : nullptr)) != ET_OK)
      return rc;
    h = b.y;
  }
  {
    ConvUnit& u = c->mlast;
    const int t = u.t;
    if ((rc = pointwise_forward(c, h, Wt(t), (int)rows_of(c, u), u.Cout, u.Cin, keep(u.z, t + 1), Wt(t + 1), Wt(t + 2), u.y, 0.f, 6.f)) != ET_OK)
      return rc;
    ET_KB(1, 2.0 * rows_of(c, u) * u.Cout, et::avgpool_fwd(u.y, c->zc, B, u.Ho * u.Wo, u.Cout, s));
    et::GemmDesc g = linear_fwd(c->zc, Wt(t + 3), Wt(t + 4), B, d.classes, u.Cout);
    g.C = c->logits; g.c_f32 = true;
    ET_G(g);
  }
  ET_K(2, et::xent(c->logits, y, B, d.classes, c->loss, c->dlogits, c->dl16, d.classes, s));
  return ET_OK;
}

int mobilenet_backward(et_ctx* c, const void* x, const uint8_t* mask) {
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

  auto affine_back = [&](int tg, const bf16* dsrc, const bf16* z, bf16* dout, long long M, int C) -> int {
    return et_exec::affine_back(c, mask, jstar, tg, dsrc, z, nullptr, dout, M, C);
  };
  int rc;

  // ---- head and the last convolution
  const ConvUnit& ul = c->mlast;
  const int tl = ul.t, Cl = ul.Cout, C = md.classes, HWl = ul.Ho * ul.Wo;
  const long long Ml = (long long)rows_of(c, ul);
  if (sel(tl + 4)) {
    Region r(c, PH_DW, tl + 4);
    ET_K(2, et::colsum(nullptr, c->dlogits, C, nullptr, 0, nullptr, nullptr, c->grad[tl + 4], cp, B, C, s));
  }
  if (sel(tl + 3)) {
    Region r(c, PH_DW, tl + 3);
    ET_G(linear_dw(c, c->dl16, C, c->zc, Cl, c->grad[tl + 3], B, C, Cl));
  }
  if (!pass(tl + 3)) return ET_OK;
  {  // through the head matrix, the average pooling and the ReLU6 of the last convolution
    Region r(c, PH_DY, tl + 3);
    et::GemmDesc g = linear_dx(c->dl16, Wt(tl + 3), B, C, Cl);
    g.C = c->dz;
    ET_G(g);
    ET_KB(1, 4.0 * Ml * Cl, et::avgpool_bwd_relu(c->dz, ul.y, c->rd[1], B, HWl, Cl, s, 6.f));
  }
  if ((rc = affine_back(tl + 1, c->rd[1], ul.z, c->rd[0], Ml, Cl)) != ET_OK) return rc;
  if (jstar > tl) return ET_OK;
  const bf16* last_in = c->mblk.back().y;
  if (sel(tl)) {
    Region r(c, PH_DW, tl);
    ET_G(linear_dw(c, c->rd[0], Cl, last_in, ul.Cin, c->grad[tl], (int)Ml, Cl, ul.Cin));
  }
  if (!pass(tl)) return ET_OK;
  {  // the block output in front of it has no activation
    Region r(c, PH_DY, tl);
    et::GemmDesc g = linear_dx(c->rd[0], Wt(tl), (int)Ml, Cl, ul.Cin);
    g.C = c->rdsum;
    ET_G(g);
  }

  // ---- blocks, output side first; on entry rdsum holds the gradient of the block output
  for (int bi = (int)c->mblk.size() - 1; bi >= 0; bi--) {
    const MbBlockBufs& b = c->mblk[bi];
    const int t = b.t, td = b.t_dw;
    if (jstar > td + 5) return ET_OK;
    const long long Mi = (long long)rows_in(c, b), Mo = (long long)rows_out(c, b);
    const bf16* stem_y = bi == 0 ? c->stem.y : nullptr;   // ReLU6 of the stem sits in front of the first block
    // projection
    if ((rc = affine_back(td + 4, c->rdsum, b.z_proj, c->rd[0], Mo, b.Cout)) != ET_OK) return rc;
    if (jstar > td + 3) return ET_OK;
    if (sel(td + 3)) {
      Region r(c, PH_DW, td + 3);
      ET_G(linear_dw(c, c->rd[0], b.Cout, b.y_dw, b.hid, c->grad[td + 3], (int)Mo, b.Cout, b.hid));
    }
    if (!pass(td + 3)) return ET_OK;
    {  // through the projection matrix and the ReLU6 after the depthwise convolution
      Region r(c, PH_DY, td + 3);
      et::GemmDesc g = linear_dx(c->rd[0], Wt(td + 3), (int)Mo, b.Cout, b.hid);
      g.C = c->rd[1];
      ET_G(g);
      ET_KB(1, 6.0 * Mo * b.hid, et::add_mask(c->rd[1], nullptr, b.y_dw, c->rd[1], Mo * b.hid, s, 6.f));
    }
    // depthwise convolution
    if ((rc = affine_back(td + 1, c->rd[1], b.z_dw, c->rd[0], Mo, b.hid)) != ET_OK) return rc;
    if (jstar > td) return ET_OK;
    const bf16* dw_in = b.expand ? b.y_exp : b.x;
    if (sel(td)) {
      Region r(c, PH_DW, td);
      const int R = et::depthwise3x3_dw_rows(B, b.H, b.W, b.hid, b.stride);
      ET_KB(1, 2.0 * (Mo + Mi) * b.hid + 4.0 * R * b.hid * 9, et::depthwise3x3_dw(c->rd[0], dw_in, c->dw_part, B, b.H, b.W, b.hid, b.stride, s));
      ET_KB(2, 4.0 * R * b.hid * 9, et::colsum(nullptr, c->dw_part, b.hid * 9, nullptr, 0, nullptr, nullptr, c->grad[td], cp, R, b.hid * 9, s));
    }
    if (!pass(td)) return ET_OK;
    if (!b.expand) {
      // the depthwise convolution is the block's first weight: its input gradient meets the shortcut here
      Region r(c, PH_DY, td);
      ET_KB(1, 2.0 * (Mo + Mi * (b.shortcut ? 3.0 : 2.0)) * b.hid,
            et::depthwise3x3_dx(c->rd[0], Wt(td), b.shortcut ? c->rdsum : nullptr, stem_y, c->rdsum, B, b.H, b.W, b.hid, b.stride, s));
      continue;
    }
    {  // through the depthwise convolution and the ReLU6 after the expansion
      Region r(c, PH_DY, td);
      ET_KB(1, 2.0 * (Mo + 2.0 * Mi) * b.hid, et::depthwise3x3_dx(c->rd[0], Wt(td), nullptr, b.y_exp, c->rd[1], B, b.H, b.W, b.hid, b.stride, s));
    }
    // expansion
    if ((rc = affine_back(t + 1, c->rd[1], b.z_exp, c->rd[0], Mi, b.hid)) != ET_OK) return rc;
    if (jstar > t) return ET_OK;
    if (sel(t)) {
      Region r(c, PH_DW, t);
      ET_G(linear_dw(c, c->rd[0], b.hid, b.x, b.Cin, c->grad[t], (int)Mi, b.hid, b.Cin));
    }
    if (!pass(t)) return ET_OK;
    {  // through the expansion matrix to the block input, where the shortcut's gradient joins
      Region r(c, PH_DY, t);
      et::GemmDesc g = linear_dx(c->rd[0], Wt(t), (int)Mi, b.hid, b.Cin);
      const bool fix = b.shortcut || stem_y;
      g.C = fix ? c->rd[2] : c->rdsum;
      ET_G(g);
      if (fix)
        ET_KB(1, (b.shortcut ? 8.0 : 6.0) * Mi * b.Cin,
              et::add_mask(c->rd[2], b.shortcut ? c->rdsum : nullptr, stem_y, c->rdsum, Mi * b.Cin, s, 6.f));
    }
  }

  // ---- stem: rdsum holds the gradient of its activation's input side (after the ReLU6 mask)
  {
    const ConvUnit& u = c->stem;
    const long long M = (long long)rows_of(c, u);
    if ((rc = affine_back(1, c->rdsum, u.z, c->rd[0], M, u.Cout)) != ET_OK) return rc;
    if (sel(0)) {
      Region r(c, PH_DW, 0);
      ET_G(linear_dw(c, c->rd[0], u.Cout, u.cols, u.Kc, c->stem_dw8, (int)M, u.Cout, u.Kc));
      ET_K(1, et::strip_rows(c->stem_dw8, c->grad[0], u.Cout, 9 * u.Cin, u.Kc, s));
    }
  }
  (void)x;
  return ET_OK;
}
