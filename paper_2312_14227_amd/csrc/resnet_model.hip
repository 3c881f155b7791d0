// Bottleneck residual CNN on the tensor-level chain (Sections 2.3 and 5).  A branched network is
// unrolled by execution order: per block c1.W, c1.g, c1.b, c2.*, c3.*, then the projection
// shortcut sc.W, sc.g, sc.b.  From the output side the shortcut tensors of a block are therefore
// visited first; they work on the gradient of the block's pre-ReLU sum.  Passing the gradient
// through the shortcut convolution to the block input is needed exactly when something before
// the block is selected, so it belongs to dy(c1.W), where the two branches meet.  BatchNorm is
// folded into a per-channel affine, so a gain's dw() is a column sum of d * (convolution output)
// and a shift's dw() a column sum of d.
//
// A convolution is a GEMM over the rows of an im2col matrix kept from the forward pass (a 1x1
// stride-1 convolution reads the activation itself): forward cols * W^T, dw() d^T * cols (split
// over the rows), dy() d * W followed by the gather-form adjoint of im2col fused with the branch
// sum and the ReLU mask.  The 3x3 convolutions, the strided 1x1 ones and the stem run as implicit
// GEMMs instead (the matrix is gathered from the activation inside the kernel; dy() of a stride-1
// 3x3 convolution is a convolution with the mirrored weight whose epilogue applies the ReLU mask).
// The stem's convolution output stays fp32 so that the max-pooling argmax is decided on unrounded
// values.
#include "conv_chain.h"

// The stem (7x7, stride 2) runs as a gathered GEMM over a padded copy of the image when the image has at most four
// channels and the output pixels come in whole slices of 64 (the weight gradient reduces over them).
static bool stem_gathered(const et_ctx* c) {
  const ConvUnit& u = c->stem;
  return u.k == 7 && u.stride == 2 && u.Cin <= 4 && rows_of(c, u) % 64 == 0 && c->stem_hp >= u.H + 3 && c->stem_wp >= u.W + 3 &&
         c->stem_hp <= 4095 && c->stem_wp <= 4095;
}

int build_resnet(et_ctx* c) {
  const et_model_desc& d = c->desc;
  if (d.dtype != ET_BF16 || d.batch < 1 || d.image < 4 || d.in_ch < 1 || d.n_stages < 1 || d.n_stages > ET_MAX_STAGES)
    return ET_EINVAL;
  if (d.stem < 8 || (d.stem % 8) || d.classes < 8 || (d.classes % 8)) return ET_EINVAL;
  int n_blocks = 0;
  for (int s = 0; s < d.n_stages; s++) {
    if (d.stage_blocks[s] < 1 || d.planes[s] < 8 || (d.planes[s] % 8)) return ET_EINVAL;
    n_blocks += d.stage_blocks[s];
  }
  auto add = [&](const std::string& n, size_t numel) { c->tensors.push_back({n, numel, ET_BF16}); };
  const size_t B = d.batch, b16 = sizeof(bf16), f32 = sizeof(float);

  init_unit(c->stem, 0, d.image, d.image, d.in_ch, d.stem, 7, 2);
  add("stem.W", (size_t)d.stem * 49 * d.in_ch); add("stem.g", d.stem); add("stem.b", d.stem);
  const int Hs = c->stem.Ho, Ws = c->stem.Wo;
  int H = (Hs - 1) / 2 + 1, W = (Ws - 1) / 2 + 1, Cin = d.stem;   // after max pooling
  if (H < 1 || W < 1) return ET_EINVAL;

  c->rblk.assign(n_blocks, ResBlockBufs());
  int bi = 0, t = 3;
  for (int s = 0; s < d.n_stages; s++)
    for (int k = 0; k < d.stage_blocks[s]; k++, bi++) {
      ResBlockBufs& b = c->rblk[bi];
      const int p = d.planes[s], stride = (k == 0 && s > 0) ? 2 : 1;
      b.t = t; b.proj = k == 0; b.x = nullptr; b.y = nullptr;
      const std::string pre = "s" + std::to_string(s) + "b" + std::to_string(k) + ".";
      init_unit(b.c1, t, H, W, Cin, p, 1, 1);
      init_unit(b.c2, t + 3, H, W, p, p, 3, stride);
      init_unit(b.c3, t + 6, b.c2.Ho, b.c2.Wo, p, 4 * p, 1, 1);
      add(pre + "c1.W", (size_t)p * Cin); add(pre + "c1.g", p); add(pre + "c1.b", p);
      add(pre + "c2.W", (size_t)p * 9 * p); add(pre + "c2.g", p); add(pre + "c2.b", p);
      add(pre + "c3.W", (size_t)4 * p * p); add(pre + "c3.g", 4 * p); add(pre + "c3.b", 4 * p);
      t += 9;
      if (b.proj) {
        init_unit(b.sc, t, H, W, Cin, 4 * p, 1, stride);
        add(pre + "sc.W", (size_t)4 * p * Cin); add(pre + "sc.g", 4 * p); add(pre + "sc.b", 4 * p);
        t += 3;
      } else if (Cin != 4 * p || stride != 1) {
        return ET_EINVAL;
      }
      H = b.c2.Ho; W = b.c2.Wo; Cin = 4 * p;
    }
  if (!c->rblk[0].proj) return ET_EINVAL;
  const int Cf = Cin, C = d.classes, C8 = round8(d.classes);
  add("head.W", (size_t)C * Cf); add("head.b", C);

  // ---- workspace
  size_t max_act = 0, max_cols = 0, max_cs = 0, pe = 0, max_flip = 8, dcols_b = 16;
  auto act = [&](size_t rows, size_t ch) {
    max_act = std::max(max_act, rows * ch);
    max_cs = std::max(max_cs, 2 * et::colsum_partial_elems((int)rows, (int)ch));   // (gain and shift sums in one launch)
  };
  auto wg = [&](const ConvUnit& u) {
    const int M = (int)rows_of(c, u);
    pe = std::max(pe, std::max(conv_dw_partials(c, u), conv_split_partials(c, u)));
    max_cols = std::max(max_cols, (size_t)M * u.Kc);   // the column matrix of any unit fits rdcols,
    dcols_b = std::max(dcols_b, dcols_bytes(c, u));     // and so does its column gradient
    if (implicit_dy(u)) max_flip = std::max(max_flip, (size_t)u.Cout * 9 * u.Cin);
  };
  auto unit = [&](ConvUnit& u, bool with_y) {
    const size_t M = rows_of(c, u);
    if (needs_cols(u) && !implicit_fwd(u)) reserve(c, &u.cols, b16 * M * u.Kc);
    reserve(c, &u.z, b16 * M * u.Cout);
    if (with_y) reserve(c, &u.y, b16 * M * u.Cout);
    act(M, u.Cout);
    wg(u);
  };
  {
    ConvUnit& u = c->stem;
    const size_t M = rows_of(c, u);
    // With at most 4 input channels the stem reads a padded copy of the image through the gathered GEMM (window
    // widened to 8 x 8 x 4 = 256 columns) instead of an im2col matrix; the weight gradient needs whole slices of 64 pixels.
    c->stem_hp = 2 * (u.Ho - 1) + 8;
    c->stem_wp = 2 * (u.Wo - 1) + 8;
    const bool gathered = stem_gathered(c);
    const size_t Kw = gathered ? 256 : (size_t)u.Kc;
    if (gathered) reserve(c, &c->stem_xpad, b16 * B * c->stem_hp * c->stem_wp * 4);
    else reserve(c, &u.cols, b16 * M * u.Kc);
    reserve(c, &c->stem_z32, f32 * M * u.Cout);
    reserve(c, &c->pool_y, b16 * M * u.Cout);
    reserve(c, &c->stem_w8, b16 * (size_t)u.Cout * Kw);
    reserve(c, &c->stem_dw8, f32 * (size_t)u.Cout * Kw);
    act(M, u.Cout);
    if (gathered) {
      int tile, split;
      et::gemm_bf16_plan_conv_dw(u.Cout, 256, (int)M, &tile, &split);
      pe = std::max(pe, et::gemm_bf16_partial_elems(u.Cout, 256, split));
    } else {
      pe = std::max(pe, et::gemm_bf16_partial_elems(u.Cout, u.Kc, split_for(u.Cout, u.Kc, (int)M)));
    }
    const size_t Mp = B * c->rblk[0].c1.H * c->rblk[0].c1.W;
    reserve(c, &c->pooled, b16 * Mp * u.Cout);
    reserve(c, &c->pool_arg, Mp * u.Cout);
    act(Mp, u.Cout);
  }
  for (ResBlockBufs& b : c->rblk) {
    unit(b.c1, true);
    unit(b.c2, true);
    unit(b.c3, false);
    if (b.proj) unit(b.sc, false);
    reserve(c, &b.y, b16 * rows_of(c, b.c3) * b.c3.Cout);
  }
  reserve(c, &c->zc, b16 * B * Cf);
  reserve(c, &c->logits, f32 * B * C);
  reserve(c, &c->dlogits, f32 * B * C);
  reserve(c, &c->dl16, b16 * B * C8);
  reserve(c, &c->loss, 256 + sizeof(float) * (size_t)d.batch);
  reserve(c, &c->dz, b16 * B * Cf);
  max_cs = std::max(max_cs, et::colsum_partial_elems((int)B, C));
  pe = std::max(pe, et::gemm_bf16_partial_elems(C, Cf, split_for(C, Cf, (int)B)));
  for (int i = 0; i < 2; i++) reserve(c, &c->rd[i], b16 * max_act);
  reserve(c, &c->rdsum, b16 * max_act);
  reserve(c, &c->rdsc, b16 * max_act);
  reserve(c, &c->rdcols, std::max(b16 * std::max<size_t>(max_cols, 8), dcols_b));
  reserve(c, &c->wflip, b16 * max_flip);
  c->gemm_partial_elems = pe;
  reserve(c, &c->gemm_partials, f32 * std::max<size_t>(pe, 64));
  reserve(c, &c->colsum_partials, f32 * std::max<size_t>(max_cs, 64));
  // every matrix dimension and element count below is handled as int by the GEMM
  if (max_act > 0x7fffffffull || max_cols > 0x7fffffffull || rows_of(c, c->stem) * c->stem.Kc > 0x7fffffffull)
    return ET_EINVAL;
  return ET_OK;
}

int resnet_forward(et_ctx* c, const void* x, const int32_t* y, const uint8_t* mask) {
  const et_model_desc& d = c->desc;
  Region r(c, PH_FWD, -1);
  hipStream_t s = c->stream;
  auto Wt = [&](int i) { return (const bf16*)c->w[i]; };
  const int B = d.batch;
  {  // stem: convolution (fp32 result), affine + ReLU, max pooling
    const ConvUnit& u = c->stem;
    if (stem_gathered(c)) {
      ET_K(1, et::stem_pack_weight(Wt(0), c->stem_w8, u.Cout, u.Cin, s));
      ET_KB(1, 2.0 * B * ((double)u.H * u.W * u.Cin + (double)c->stem_hp * c->stem_wp * 4),
            et::stem_pad_image((const bf16*)x, c->stem_xpad, B, u.H, u.W, u.Cin, c->stem_hp, c->stem_wp, s));
      et::GemmDesc g = linear_fwd(c->stem_xpad, c->stem_w8, nullptr, (int)rows_of(c, u), u.Cout, 256);
      g.conv_h = c->stem_hp; g.conv_w = c->stem_wp; g.conv_c = 4; g.conv_taps = 7; g.conv_stride = 2;
      g.C = c->stem_z32; g.c_f32 = true;
      ET_G(g);
    } else {
      ET_K(1, et::pad_rows(Wt(0), c->stem_w8, u.Cout, 49 * u.Cin, u.Kc, s));
      int rc = conv_forward(c, u, (const bf16*)x, c->stem_w8, c->stem_z32, true);
      if (rc != ET_OK) return rc;
    }
    const double n = (double)rows_of(c, u) * u.Cout, np = (double)B * c->rblk[0].c1.H * c->rblk[0].c1.W * u.Cout;
    ET_KB(1, 6.0 * n, et::affine_act(nullptr, c->stem_z32, Wt(1), Wt(2), nullptr, nullptr, nullptr, true, c->pool_y,
                                     (long long)rows_of(c, u), u.Cout, s));
    ET_KB(1, 4.0 * n + 3.0 * np,
          et::maxpool3x3s2_fwd(c->stem_z32, Wt(1), Wt(2), c->pooled, c->pool_arg, B, u.Ho, u.Wo, u.Cout, s));
  }
  const bf16* h = c->pooled;
  // a convolution's output z is read again only by the gradient of its gain
  auto keep = [&](bf16* z, int gain_index) -> bf16* { return (!mask || mask[gain_index]) ? z : nullptr; };
  for (ResBlockBufs& b : c->rblk) {
    const int t = b.t;
    b.x = h;
    // c1, c2: the affine + ReLU is the epilogue of the convolution's GEMM (z is kept for the gain's gradient)
    int rc = conv_forward(c, b.c1, h, Wt(t), keep(b.c1.z, t + 1), false, Wt(t + 1), Wt(t + 2), b.c1.y);
    if (rc != ET_OK) return rc;
    rc = conv_forward(c, b.c2, b.c1.y, Wt(t + 3), keep(b.c2.z, t + 4), false, Wt(t + 4), Wt(t + 5), b.c2.y);
    if (rc != ET_OK) return rc;
    // block end: y = max(c3.z * g + b + shortcut, 0) is the epilogue of c3's GEMM; the projection
    // shortcut's convolution runs first
    if (b.proj) {
      rc = conv_forward(c, b.sc, h, Wt(t + 9), b.sc.z, false);
      if (rc != ET_OK) return rc;
      rc = conv_forward(c, b.c3, b.c2.y, Wt(t + 6), keep(b.c3.z, t + 7), false, Wt(t + 7), Wt(t + 8), b.y, b.sc.z, Wt(t + 10), Wt(t + 11));
    } else {
      rc = conv_forward(c, b.c3, b.c2.y, Wt(t + 6), keep(b.c3.z, t + 7), false, Wt(t + 7), Wt(t + 8), b.y, h);
    }
    if (rc != ET_OK) return rc;
    h = b.y;
  }
  const ResBlockBufs& last = c->rblk.back();
  const int Cf = last.c3.Cout, N = (int)c->tensors.size();
  ET_KB(1, 2.0 * B * last.c3.Ho * last.c3.Wo * Cf, et::avgpool_fwd(h, c->zc, B, last.c3.Ho * last.c3.Wo, Cf, s));
  {
    et::GemmDesc g = linear_fwd(c->zc, Wt(N - 2), Wt(N - 1), B, d.classes, Cf);
    g.C = c->logits; g.c_f32 = true;
    ET_G(g);
  }
  ET_K(2, et::xent(c->logits, y, B, d.classes, c->loss, c->dlogits, c->dl16, round8(d.classes), s));
  return ET_OK;
}

int resnet_backward(et_ctx* c, const void* x, const uint8_t* mask) {
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
  int rc;

  // ---- head
  const ResBlockBufs& last = c->rblk.back();
  const int Cf = last.c3.Cout, C = md.classes, C8 = round8(md.classes), HWf = last.c3.Ho * last.c3.Wo;
  if (sel(N - 1)) {
    Region r(c, PH_DW, N - 1);
    ET_K(2, et::colsum(nullptr, c->dlogits, C, nullptr, 0, nullptr, nullptr, c->grad[N - 1], cp, B, C, s));
  }
  if (sel(N - 2)) {
    Region r(c, PH_DW, N - 2);
    ET_G(linear_dw(c, c->dl16, C8, c->zc, Cf, c->grad[N - 2], B, C, Cf));
  }
  if (pass(N - 2)) {  // through the head matrix, the average pooling and the ReLU closing the last block
    Region r(c, PH_DY, N - 2);
    et::GemmDesc g = linear_dx(c->dl16, Wt(N - 2), B, C, Cf);
    g.lda = C8; g.C = c->dz;
    ET_G(g);
    ET_KB(1, 4.0 * B * HWf * Cf, et::avgpool_bwd_relu(c->dz, last.y, c->rdsum, B, HWf, Cf, s));
  }

  // ---- blocks, output side first.  On entry rdsum holds the gradient of the block's pre-ReLU sum.
  for (int bi = (int)c->rblk.size() - 1; bi >= 0; bi--) {
    const ResBlockBufs& b = c->rblk[bi];
    const int t = b.t;
    if (jstar > t + (b.proj ? 11 : 8)) break;
    const long long M3 = (long long)rows_of(c, b.c3), M2 = (long long)rows_of(c, b.c2), M1 = (long long)rows_of(c, b.c1);
    if (b.proj) {
      if ((rc = affine_back(c, mask, jstar, t + 10, c->rdsum, b.sc.z, nullptr, c->rdsc, M3, b.sc.Cout, sel(t + 9) || pass(t))) != ET_OK)
        return rc;
      if (sel(t + 9)) {
        Region r(c, PH_DW, t + 9);
        if ((rc = conv_dw(c, b.sc, b.x, c->rdsc, c->grad[t + 9])) != ET_OK) return rc;
      }
    }
    // main branch: c3
    if ((rc = affine_back(c, mask, jstar, t + 7, c->rdsum, b.c3.z, nullptr, c->rd[0], M3, b.c3.Cout)) != ET_OK) return rc;
    if (sel(t + 6)) {
      Region r(c, PH_DW, t + 6);
      if ((rc = conv_dw(c, b.c3, b.c2.y, c->rd[0], c->grad[t + 6])) != ET_OK) return rc;
    }
    if (pass(t + 6)) {  // through the 1x1 convolution and the ReLU after c2
      Region r(c, PH_DY, t + 6);
      if ((rc = conv_dcols(c, b.c3, c->rd[0], Wt(t + 6), c->rd[1])) != ET_OK) return rc;
      ET_KB(1, 6.0 * M2 * b.c2.Cout, et::add_mask(c->rd[1], nullptr, b.c2.y, c->rd[1], M2 * b.c2.Cout, s));
    }
    // c2
    if ((rc = affine_back(c, mask, jstar, t + 4, c->rd[1], b.c2.z, nullptr, c->rd[0], M2, b.c2.Cout)) != ET_OK) return rc;
    if (sel(t + 3)) {
      Region r(c, PH_DW, t + 3);
      if ((rc = conv_dw(c, b.c2, b.c1.y, c->rd[0], c->grad[t + 3])) != ET_OK) return rc;
    }
    if (pass(t + 3)) {  // through the 3x3 convolution and the ReLU after c1
      Region r(c, PH_DY, t + 3);
      if (implicit_dy(b.c2)) {
        if ((rc = conv_dy_implicit(c, b.c2, c->rd[0], Wt(t + 3), b.c1.y, c->rd[1])) != ET_OK) return rc;
      } else {
        if ((rc = conv_dcols(c, b.c2, c->rd[0], Wt(t + 3), c->rdcols)) != ET_OK) return rc;
        ET_KB(1, (dcols_f32(b.c2) ? 4.0 : 2.0) * M2 * b.c2.Kc + 4.0 * M1 * b.c1.Cout, et::col2im(c->rdcols, dcols_f32(b.c2), nullptr, b.c1.y, c->rd[1], geom(c, b.c2), s));
      }
    }
    // c1
    if ((rc = affine_back(c, mask, jstar, t + 1, c->rd[1], b.c1.z, nullptr, c->rd[0], M1, b.c1.Cout)) != ET_OK) return rc;
    if (sel(t)) {
      Region r(c, PH_DW, t);
      if ((rc = conv_dw(c, b.c1, b.x, c->rd[0], c->grad[t])) != ET_OK) return rc;
    }
    if (pass(t)) {
      // through c1, joined by the shortcut branch (through the shortcut convolution, or the
      // identity), then through the ReLU closing the previous block -- or, for the first block,
      // the max pooling and the stem's ReLU
      Region r(c, PH_DY, t);
      if ((rc = conv_dcols(c, b.c1, c->rd[0], Wt(t), c->rd[1])) != ET_OK) return rc;
      const bf16* prev_y = bi > 0 ? c->rblk[bi - 1].y : nullptr;
      if (b.proj) {
        if ((rc = conv_dcols(c, b.sc, c->rdsc, Wt(t + 9), c->rdcols)) != ET_OK) return rc;
        ET_KB(1, 2.0 * M3 * b.sc.Kc + (prev_y ? 6.0 : 4.0) * M1 * b.c1.Cin,
              et::col2im(c->rdcols, dcols_f32(b.sc), c->rd[1], prev_y, prev_y ? c->rdsum : c->rd[0], geom(c, b.sc), s));
      } else {
        ET_KB(1, 8.0 * M1 * b.c1.Cin, et::add_mask(c->rd[1], c->rdsum, prev_y, c->rdsum, M1 * b.c1.Cin, s));
      }
      if (!prev_y) {
        const ConvUnit& u = c->stem;
        ET_KB(1, 3.0 * M1 * b.c1.Cin + 4.0 * B * u.Ho * u.Wo * u.Cout,
              et::maxpool3x3s2_bwd(c->rd[0], c->pool_arg, c->pool_y, c->rdsum, B, u.Ho, u.Wo, u.Cout, s));
      }
    }
  }

  // ---- stem
  if (jstar <= 2) {
    const ConvUnit& u = c->stem;
    const long long M = (long long)rows_of(c, u);
    if ((rc = affine_back(c, mask, jstar, 1, c->rdsum, nullptr, c->stem_z32, c->rd[0], M, u.Cout)) != ET_OK) return rc;
    if (sel(0)) {
      Region r(c, PH_DW, 0);
      if (stem_gathered(c)) {   // B operand: the padded image standing for [pixel][8 x 8 x 4]
        et::GemmDesc g;
        g.A = c->rd[0]; g.a_t = true; g.lda = u.Cout; g.B = c->stem_xpad; g.b_t = true; g.ldb = 256;
        g.M = u.Cout; g.N = 256; g.K = (int)M;
        g.C = c->stem_dw8; g.ldc = 256; g.c_f32 = true;
        g.conv_h = c->stem_hp; g.conv_w = c->stem_wp; g.conv_c = 4; g.conv_taps = 7; g.conv_stride = 2;
        et::gemm_bf16_plan_conv_dw(g.M, g.N, g.K, &g.tile, &g.split_k);
        g.partials = c->gemm_partials;
        if (et::gemm_bf16_partial_elems(g.M, g.N, g.split_k) > c->gemm_partial_elems) g.split_k = 1;
        ET_G(g);
        ET_K(1, et::stem_unpack_dw(c->stem_dw8, c->grad[0], u.Cout, u.Cin, s));
      } else {
        ET_G(linear_dw(c, c->rd[0], u.Cout, u.cols, u.Kc, c->stem_dw8, (int)M, u.Cout, u.Kc));
        ET_K(1, et::strip_rows(c->stem_dw8, c->grad[0], u.Cout, 49 * u.Cin, u.Kc, s));
      }
    }
  }
  (void)x;
  return ET_OK;
}
