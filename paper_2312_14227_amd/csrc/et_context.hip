// Step executor behind the C ABI: the static operation chain of a model, the workspace plan, the
// masked backward pass on the tensor-level chain (Sections 2.2, 2.3 and 5), the in-place timing
// profiler (Section 5), the importance evaluation (Eq. 2) and the masked optimizer update.
//
// The backward pass is the loop of the tensor-level time model:
//     for j = N-1 .. j*:   if M[j]: dw(j);    if j > j*: dy(j)
// with j* the input-most selected tensor.  dw(j) and dy(j) are separate kernel launches, so the
// time of a masked step is the sum of the times of the launched pieces, which is exactly what the
// selector's time model assumes.  Backward kernels of operations without weights (ReLU, GELU, the
// attention core, residual additions) sit in the dy() of the tensor that has to be passed for them
// to be needed; a LayerNorm's input-gradient kernel sits in dy(gain).
#include "context.h"

namespace {

// -----------------------------------------------------------------------------------------------
// model construction
// -----------------------------------------------------------------------------------------------
int build_mlp(et_ctx* c) {
  const et_model_desc& d = c->desc;
  if (d.n_layers < 1 || d.n_layers > ET_MAX_MLP_LAYERS || d.dtype != ET_F32 || d.batch < 1) return ET_EINVAL;
  for (int i = 0; i <= d.n_layers; i++)
    if (d.dims[i] < 1) return ET_EINVAL;
  for (int i = 0; i < d.n_layers; i++)
    c->tensors.push_back({"fc" + std::to_string(i) + ".W", (size_t)d.dims[i + 1] * d.dims[i], ET_F32});
  const int B = d.batch, C = d.dims[d.n_layers];
  int maxdim = 0;
  for (int i = 0; i <= d.n_layers; i++) maxdim = std::max(maxdim, d.dims[i]);
  c->act.assign(d.n_layers, nullptr);
  for (int i = 1; i < d.n_layers; i++) reserve(c, &c->act[i], sizeof(float) * B * d.dims[i]);
  reserve(c, &c->logits, sizeof(float) * B * C);
  reserve(c, &c->dlogits, sizeof(float) * B * C);
  reserve(c, &c->loss, 256 + sizeof(float) * (size_t)d.batch);
  reserve(c, &c->dbuf[0], sizeof(float) * B * maxdim);
  reserve(c, &c->dbuf[1], sizeof(float) * B * maxdim);
  return ET_OK;
}

int build_vit(et_ctx* c) {
  const et_model_desc& d = c->desc;
  if (d.dtype != ET_BF16 || d.batch < 1 || d.tokens < 2 || d.blocks < 1 || d.heads < 1) return ET_EINVAL;
  if (d.width < 8 || d.patch_dim < 8 || d.mlp < 8 || d.classes < 8) return ET_EINVAL;
  if ((d.width % 8) || (d.patch_dim % 8) || (d.mlp % 8) || (d.classes % 8) || (d.width % d.heads) ||
      ((d.width / d.heads) % 8))
    return ET_EINVAL;
  if (!(d.ln_eps > 0.f)) return ET_EINVAL;
  const size_t D = d.width, F = d.mlp, P = d.patch_dim, T = d.tokens, C = d.classes;
  auto add = [&](const std::string& n, size_t numel) { c->tensors.push_back({n, numel, ET_BF16}); };
  add("patch.W", D * P); add("patch.b", D); add("cls", D); add("pos", T * D);
  for (int l = 0; l < d.blocks; l++) {
    const std::string p = "blk" + std::to_string(l) + ".";
    add(p + "ln1.g", D); add(p + "ln1.b", D); add(p + "qkv.W", 3 * D * D); add(p + "qkv.b", 3 * D);
    add(p + "proj.W", D * D); add(p + "proj.b", D); add(p + "ln2.g", D); add(p + "ln2.b", D);
    add(p + "fc1.W", F * D); add(p + "fc1.b", F); add(p + "fc2.W", D * F); add(p + "fc2.b", D);
  }
  add("lnf.g", D); add("lnf.b", D); add("head.W", C * D); add("head.b", C);

  const size_t B = d.batch, M = B * T, H = d.heads, ldT = round8(d.tokens), C8 = round8(d.classes);
  const size_t f32 = sizeof(float), b16 = sizeof(bf16);
  reserve(c, &c->e, f32 * B * (T - 1) * D);
  c->blk.assign(d.blocks, VitBlockBufs());
  for (int l = 0; l < d.blocks; l++) {
    VitBlockBufs& b = c->blk[l];
    reserve(c, &b.h_in, f32 * M * D);
    reserve(c, &b.h_mid, f32 * M * D);
    reserve(c, &b.mean1, f32 * M); reserve(c, &b.rstd1, f32 * M);
    reserve(c, &b.mean2, f32 * M); reserve(c, &b.rstd2, f32 * M);
    reserve(c, &b.a1, b16 * M * D);
    reserve(c, &b.qkv, b16 * M * 3 * D);
    reserve(c, &b.p, b16 * B * H * T * ldT);
    reserve(c, &b.lse, f32 * B * H * T);
    reserve(c, &b.o, b16 * M * D);
    reserve(c, &b.a2, b16 * M * D);
    reserve(c, &b.u, b16 * M * F);
    reserve(c, &b.ga, b16 * M * F);
  }
  reserve(c, &c->h_out, f32 * M * D);
  reserve(c, &c->s_f32, f32 * B * H * T * ldT);
  reserve(c, &c->meanf, f32 * B); reserve(c, &c->rstdf, f32 * B);
  reserve(c, &c->zc, b16 * B * D);
  reserve(c, &c->logits, f32 * B * C);
  reserve(c, &c->dlogits, f32 * B * C);
  reserve(c, &c->dl16, b16 * B * C8);
  reserve(c, &c->loss, 256 + sizeof(float) * (size_t)d.batch);
  reserve(c, &c->dz, b16 * B * D);
  reserve(c, &c->dh, f32 * M * D);
  reserve(c, &c->dh16, b16 * M * D);
  reserve(c, &c->da, b16 * M * D);
  reserve(c, &c->du, b16 * M * F);
  reserve(c, &c->dattn, b16 * M * D);
  reserve(c, &c->dqkv, b16 * M * 3 * D);
  reserve(c, &c->ds, b16 * B * H * T * ldT);
  reserve(c, &c->de, b16 * B * (T - 1) * D);
  // split-K partials: the largest weight gradient
  size_t pe = 0;
  auto wg = [&](size_t Mo, size_t No, size_t K) {
    pe = std::max(pe, et::gemm_bf16_partial_elems((int)Mo, (int)No, split_for((int)Mo, (int)No, (int)K)));
  };
  wg(3 * D, D, M); wg(D, D, M); wg(F, D, M); wg(D, F, M); wg(D, P, B * (T - 1)); wg(C, D, B);
  c->gemm_partial_elems = pe;
  reserve(c, &c->gemm_partials, f32 * std::max<size_t>(pe, 64));
  reserve(c, &c->colsum_partials, f32 * et::colsum_partial_elems((int)M, (int)std::max(3 * D, F)));
  return ET_OK;
}

void build_tables_plan(et_ctx* c) {
  const size_t N = c->tensors.size();
  c->seg_begin.assign(N + 1, 0);
  for (size_t i = 0; i < N; i++)
    c->seg_begin[i + 1] = c->seg_begin[i] + (uint32_t)((c->tensors[i].numel + SEG_ELEMS - 1) / SEG_ELEMS);
  c->n_segs = c->seg_begin[N];
  reserve(c, &c->imp_segs_dev, sizeof(et::TensorSeg) * c->n_segs);
  reserve(c, &c->upd_segs_dev, sizeof(et::UpdateSeg) * c->n_segs);
  reserve(c, &c->upd_selected_dev, sizeof(uint32_t) * c->n_segs);
  reserve(c, &c->seg_begin_dev, sizeof(uint32_t) * (N + 1));
  reserve(c, &c->imp_partial_dev, sizeof(double) * c->n_segs);
  reserve(c, &c->imp_out_dev, sizeof(double) * N);
}

// -----------------------------------------------------------------------------------------------
// MLP forward / backward
// -----------------------------------------------------------------------------------------------
int mlp_forward(et_ctx* c, const void* x, const int32_t* y) {
  const et_model_desc& d = c->desc;
  Region r(c, PH_FWD, -1);
  const int B = d.batch, L = d.n_layers;
  for (int i = 0; i < L; i++) {
    et::GemmF32Desc g;
    g.A = i == 0 ? (const float*)x : c->act[i];
    g.B = (const float*)c->w[i];
    g.C = i + 1 < L ? c->act[i + 1] : c->logits;
    g.M = B; g.N = d.dims[i + 1]; g.K = d.dims[i];
    g.lda = g.K; g.ldb = g.K; g.ldc = g.N;
    g.relu_out = i + 1 < L;
    ET_K(1, et::gemm_f32(g, c->stream));
  }
  ET_K(2, et::xent(c->logits, y, B, d.dims[L], c->loss, c->dlogits, nullptr, d.dims[L], c->stream));
  return ET_OK;
}

int mlp_backward(et_ctx* c, const void* x, const uint8_t* mask) {
  const et_model_desc& d = c->desc;
  const int B = d.batch, L = d.n_layers;
  int jstar = -1;
  for (int j = 0; j < L; j++)
    if (mask[j]) { jstar = j; break; }
  if (jstar < 0) return ET_OK;
  const float* dcur = c->dlogits;
  int flip = 0;
  for (int j = L - 1; j >= jstar; j--) {
    const int out = d.dims[j + 1], in = d.dims[j];
    if (mask[j]) {
      Region r(c, PH_DW, j);
      et::GemmF32Desc g;                      // dW[out][in] = sum_b d[b][out] a[b][in]
      g.A = dcur; g.a_t = true; g.lda = out;
      g.B = j == 0 ? (const float*)x : c->act[j]; g.b_t = true; g.ldb = in;
      g.C = c->grad[j]; g.M = out; g.N = in; g.K = B; g.ldc = in;
      ET_K(1, et::gemm_f32(g, c->stream));
    }
    if (j > jstar) {
      Region r(c, PH_DY, j);
      et::GemmF32Desc g;                      // d'[b][in] = (sum_o d[b][o] W[o][in]) * (a[b][in] > 0)
      g.A = dcur; g.lda = out;
      g.B = (const float*)c->w[j]; g.b_t = true; g.ldb = in;
      g.C = c->dbuf[flip]; g.M = B; g.N = in; g.K = out; g.ldc = in;
      g.mask = c->act[j];
      ET_K(1, et::gemm_f32(g, c->stream));
      dcur = c->dbuf[flip];
      flip ^= 1;
    }
  }
  return ET_OK;
}

// -----------------------------------------------------------------------------------------------
// ViT forward / backward
// -----------------------------------------------------------------------------------------------
struct VitDims {
  int B, T, D, H, dh, F, P, C, L, M, ldT, C8;
  float scale;
};

VitDims vit_dims(const et_model_desc& d) {
  VitDims v;
  v.B = d.batch; v.T = d.tokens; v.D = d.width; v.H = d.heads; v.dh = d.width / d.heads; v.F = d.mlp;
  v.P = d.patch_dim; v.C = d.classes; v.L = d.blocks; v.M = d.batch * d.tokens; v.ldT = round8(d.tokens);
  v.C8 = round8(d.classes);
  v.scale = 1.f / std::sqrt((float)v.dh);
  return v;
}

int vit_forward(et_ctx* c, const void* x, const int32_t* y, const uint8_t* mask) {
  const VitDims v = vit_dims(c->desc);
  // input-most selected tensor: gelu'(u) of a block is read only when the gradient is passed through its fc2
  int jstar = -1;
  if (mask) {
    jstar = (int)c->tensors.size();
    for (int j = 0; j < (int)c->tensors.size(); j++)
      if (mask[j]) { jstar = j; break; }
  }
  Region r(c, PH_FWD, -1);
  auto W = [&](int i) { return (const bf16*)c->w[i]; };
  {
    et::GemmDesc g = linear_fwd((const bf16*)x, W(0), W(1), v.B * (v.T - 1), v.D, v.P);
    g.C = c->e; g.c_f32 = true;
    ET_G(g);
  }
  ET_K(1, et::embed_assemble(c->e, W(2), W(3), c->blk[0].h_in, v.B, v.T, v.D, c->stream));
  for (int l = 0; l < v.L; l++) {
    VitBlockBufs& b = c->blk[l];
    const int t0 = 4 + 12 * l;
    float* h_next = l + 1 < v.L ? c->blk[l + 1].h_in : c->h_out;
    ET_K(1, et::layernorm_fwd(b.h_in, v.D, W(t0 + 0), W(t0 + 1), c->desc.ln_eps, b.a1, b.mean1, b.rstd1, v.M, v.D,
                              c->stream));
    {
      et::GemmDesc g = linear_fwd(b.a1, W(t0 + 2), W(t0 + 3), v.M, 3 * v.D, v.D);
      g.C = b.qkv;
      ET_G(g);
    }
    if (et::attention_fused_supported(v.T, v.dh)) {
      KernelTimer kt(c, 5, 4.0 * v.B * v.H * (double)v.T * v.T * v.dh);
      ET_K(1, et::attention_fwd(b.qkv, b.o, b.lse, v.B, v.T, v.H, v.dh, v.scale, c->stream));
    } else {
      {  // S = scale * Q K^T per (batch, head)
        et::GemmDesc g;
        g.A = b.qkv; g.lda = 3 * v.D; g.B = b.qkv + v.D; g.ldb = 3 * v.D; g.M = v.T; g.N = v.T; g.K = v.dh;
        g.z_outer = v.B; g.z_inner = v.H;
        g.sAo = (long long)v.T * 3 * v.D; g.sAi = v.dh; g.sBo = g.sAo; g.sBi = v.dh;
        g.C = c->s_f32; g.c_f32 = true; g.ldc = v.ldT; g.sCo = (long long)v.H * v.T * v.ldT; g.sCi = (long long)v.T * v.ldT;
        g.alpha = v.scale;
        ET_G(g);
      }
      ET_K(1, et::softmax_rows(c->s_f32, b.p, v.B * v.H * v.T, v.T, v.ldT, c->stream));
      {  // O = P V
        et::GemmDesc g;
        g.A = b.p; g.lda = v.ldT; g.B = b.qkv + 2 * v.D; g.b_t = true; g.ldb = 3 * v.D; g.M = v.T; g.N = v.dh; g.K = v.T;
        g.z_outer = v.B; g.z_inner = v.H;
        g.sAo = (long long)v.H * v.T * v.ldT; g.sAi = (long long)v.T * v.ldT; g.sBo = (long long)v.T * 3 * v.D; g.sBi = v.dh;
        g.C = b.o; g.ldc = v.D; g.sCo = (long long)v.T * v.D; g.sCi = v.dh;
        ET_G(g);
      }
    }
    {
      et::GemmDesc g = linear_fwd(b.o, W(t0 + 4), W(t0 + 5), v.M, v.D, v.D);
      g.residual = b.h_in; g.ldr = v.D; g.C = b.h_mid; g.c_f32 = true;
      ET_G(g);
    }
    ET_K(1, et::layernorm_fwd(b.h_mid, v.D, W(t0 + 6), W(t0 + 7), c->desc.ln_eps, b.a2, b.mean2, b.rstd2, v.M, v.D,
                              c->stream));
    {
      et::GemmDesc g = linear_fwd(b.a2, W(t0 + 8), W(t0 + 9), v.M, v.F, v.D);
      if (t0 + 10 > jstar) {   // also when mask is null (jstar = -1)
        g.mode = et::EPI_GELU_FWD; g.C = b.u; g.C2 = b.ga;
      } else {
        g.mode = et::EPI_GELU_ONLY; g.C = b.ga;
      }
      ET_G(g);
    }
    {
      et::GemmDesc g = linear_fwd(b.ga, W(t0 + 10), W(t0 + 11), v.M, v.D, v.F);
      g.residual = b.h_mid; g.ldr = v.D; g.C = h_next; g.c_f32 = true;
      ET_G(g);
    }
  }
  const int N = (int)c->tensors.size();
  ET_K(1, et::layernorm_fwd(c->h_out, (long long)v.T * v.D, W(N - 4), W(N - 3), c->desc.ln_eps, c->zc, c->meanf,
                            c->rstdf, v.B, v.D, c->stream));
  {
    et::GemmDesc g = linear_fwd(c->zc, W(N - 2), W(N - 1), v.B, v.C, v.D);
    g.C = c->logits; g.c_f32 = true;
    ET_G(g);
  }
  ET_K(2, et::xent(c->logits, y, v.B, v.C, c->loss, c->dlogits, c->dl16, v.C8, c->stream));
  return ET_OK;
}

int vit_attention_backward(et_ctx* c, const VitDims& v, VitBlockBufs& b) {
  if (et::attention_fused_supported(v.T, v.dh)) {
    KernelTimer kt(c, 6, 8.0 * v.B * v.H * (double)v.T * v.T * v.dh);
    ET_K(1, et::attention_bwd(b.qkv, b.o, c->dattn, b.lse, c->dqkv, v.B, v.T, v.H, v.dh, v.scale, c->stream));
    return ET_OK;
  }
  const long long sQo = (long long)v.T * 3 * v.D, sPo = (long long)v.H * v.T * v.ldT, sPi = (long long)v.T * v.ldT;
  const long long sOo = (long long)v.T * v.D;
  auto batched = [&](et::GemmDesc& g) { g.z_outer = v.B; g.z_inner = v.H; };
  {  // dV[s][d] = sum_t P[t][s] dO[t][d]
    et::GemmDesc g;
    g.A = b.p; g.a_t = true; g.lda = v.ldT; g.sAo = sPo; g.sAi = sPi;
    g.B = c->dattn; g.b_t = true; g.ldb = v.D; g.sBo = sOo; g.sBi = v.dh;
    g.M = v.T; g.N = v.dh; g.K = v.T; batched(g);
    g.C = c->dqkv + 2 * v.D; g.ldc = 3 * v.D; g.sCo = sQo; g.sCi = v.dh;
    ET_G(g);
  }
  {  // dP = dO V^T
    et::GemmDesc g;
    g.A = c->dattn; g.lda = v.D; g.sAo = sOo; g.sAi = v.dh;
    g.B = b.qkv + 2 * v.D; g.ldb = 3 * v.D; g.sBo = sQo; g.sBi = v.dh;
    g.M = v.T; g.N = v.T; g.K = v.dh; batched(g);
    g.C = c->s_f32; g.c_f32 = true; g.ldc = v.ldT; g.sCo = sPo; g.sCi = sPi;
    ET_G(g);
  }
  ET_K(1, et::softmax_bwd_rows(c->s_f32, b.p, c->ds, v.scale, v.B * v.H * v.T, v.T, v.ldT, c->stream));
  {  // dQ = dS K   (the 1/sqrt(dh) factor is already in dS)
    et::GemmDesc g;
    g.A = c->ds; g.lda = v.ldT; g.sAo = sPo; g.sAi = sPi;
    g.B = b.qkv + v.D; g.b_t = true; g.ldb = 3 * v.D; g.sBo = sQo; g.sBi = v.dh;
    g.M = v.T; g.N = v.dh; g.K = v.T; batched(g);
    g.C = c->dqkv; g.ldc = 3 * v.D; g.sCo = sQo; g.sCi = v.dh;
    ET_G(g);
  }
  {  // dK[s][d] = sum_t dS[t][s] Q[t][d]
    et::GemmDesc g;
    g.A = c->ds; g.a_t = true; g.lda = v.ldT; g.sAo = sPo; g.sAi = sPi;
    g.B = b.qkv; g.b_t = true; g.ldb = 3 * v.D; g.sBo = sQo; g.sBi = v.dh;
    g.M = v.T; g.N = v.dh; g.K = v.T; batched(g);
    g.C = c->dqkv + v.D; g.ldc = 3 * v.D; g.sCo = sQo; g.sCi = v.dh;
    ET_G(g);
  }
  return ET_OK;
}

int vit_backward(et_ctx* c, const void* x, const uint8_t* mask) {
  const VitDims v = vit_dims(c->desc);
  const int N = (int)c->tensors.size();
  int jstar = -1;
  for (int j = 0; j < N; j++)
    if (mask[j]) { jstar = j; break; }
  if (jstar < 0) return ET_OK;
  auto W = [&](int i) { return (const bf16*)c->w[i]; };
  auto sel = [&](int j) { return mask[j] != 0; };
  auto pass = [&](int j) { return j > jstar; };
  hipStream_t s = c->stream;
  float* cp = c->colsum_partials;

  // ---- head and final LayerNorm (CLS rows)
  if (sel(N - 1)) {
    Region r(c, PH_DW, N - 1);
    ET_K(2, et::colsum(nullptr, c->dlogits, v.C, nullptr, 0, nullptr, nullptr, c->grad[N - 1], cp, v.B, v.C, s));
  }
  if (sel(N - 2)) {
    Region r(c, PH_DW, N - 2);
    ET_G(linear_dw(c, c->dl16, v.C8, c->zc, v.D, c->grad[N - 2], v.B, v.C, v.D));
  }
  if (pass(N - 2)) {
    Region r(c, PH_DY, N - 2);
    et::GemmDesc g = linear_dx(c->dl16, W(N - 2), v.B, v.C, v.D);
    g.lda = v.C8; g.C = c->dz;
    ET_G(g);
  }
  if (sel(N - 3)) {
    Region r(c, PH_DW, N - 3);
    ET_K(2, et::colsum(c->dz, nullptr, v.D, nullptr, 0, nullptr, nullptr, c->grad[N - 3], cp, v.B, v.D, s));
  }
  if (sel(N - 4)) {
    Region r(c, PH_DW, N - 4);
    ET_K(2, et::colsum(c->dz, nullptr, v.D, c->h_out, (long long)v.T * v.D, c->meanf, c->rstdf, c->grad[N - 4], cp,
                       v.B, v.D, s));
  }
  if (pass(N - 4)) {
    Region r(c, PH_DY, N - 4);
    ET_K(1, et::fill_zero(c->dh, sizeof(float) * (size_t)v.M * v.D, s));
    ET_K(1, et::fill_zero(c->dh16, sizeof(bf16) * (size_t)v.M * v.D, s));
    ET_K(1, et::layernorm_bwd_dx(c->dz, c->h_out, (long long)v.T * v.D, c->meanf, c->rstdf, W(N - 4), nullptr, c->dh,
                                 c->dh16, (long long)v.T * v.D, v.B, v.D, s));
  }

  // ---- blocks, output side first
  for (int l = v.L - 1; l >= 0; l--) {
    VitBlockBufs& b = c->blk[l];
    const int t0 = 4 + 12 * l;
    if (jstar > t0 + 11) break;
    if (sel(t0 + 11)) {
      Region r(c, PH_DW, t0 + 11);
      ET_K(2, et::colsum(nullptr, c->dh, v.D, nullptr, 0, nullptr, nullptr, c->grad[t0 + 11], cp, v.M, v.D, s));
    }
    if (sel(t0 + 10)) {
      Region r(c, PH_DW, t0 + 10);
      ET_G(linear_dw(c, c->dh16, v.D, b.ga, v.F, c->grad[t0 + 10], v.M, v.D, v.F));
    }
    if (pass(t0 + 10)) {  // through fc2.W, then through the GELU (b.u holds gelu'(pre-activation))
      Region r(c, PH_DY, t0 + 10);
      et::GemmDesc g = linear_dx(c->dh16, W(t0 + 10), v.M, v.D, v.F);
      g.mode = et::EPI_GELU_BWD; g.U = b.u; g.C = c->du;
      ET_G(g);
    }
    if (sel(t0 + 9)) {
      Region r(c, PH_DW, t0 + 9);
      ET_K(2, et::colsum(c->du, nullptr, v.F, nullptr, 0, nullptr, nullptr, c->grad[t0 + 9], cp, v.M, v.F, s));
    }
    if (sel(t0 + 8)) {
      Region r(c, PH_DW, t0 + 8);
      ET_G(linear_dw(c, c->du, v.F, b.a2, v.D, c->grad[t0 + 8], v.M, v.F, v.D));
    }
    if (pass(t0 + 8)) {
      Region r(c, PH_DY, t0 + 8);
      et::GemmDesc g = linear_dx(c->du, W(t0 + 8), v.M, v.F, v.D);
      g.C = c->da;
      ET_G(g);
    }
    if (sel(t0 + 7)) {
      Region r(c, PH_DW, t0 + 7);
      ET_K(2, et::colsum(c->da, nullptr, v.D, nullptr, 0, nullptr, nullptr, c->grad[t0 + 7], cp, v.M, v.D, s));
    }
    if (sel(t0 + 6)) {
      Region r(c, PH_DW, t0 + 6);
      ET_K(2, et::colsum(c->da, nullptr, v.D, b.h_mid, v.D, b.mean2, b.rstd2, c->grad[t0 + 6], cp, v.M, v.D, s));
    }
    if (pass(t0 + 6)) {  // LayerNorm input gradient joined by the residual branch
      Region r(c, PH_DY, t0 + 6);
      ET_K(1, et::layernorm_bwd_dx(c->da, b.h_mid, v.D, b.mean2, b.rstd2, W(t0 + 6), c->dh, c->dh, c->dh16, v.D, v.M,
                                   v.D, s));
    }
    if (sel(t0 + 5)) {
      Region r(c, PH_DW, t0 + 5);
      ET_K(2, et::colsum(nullptr, c->dh, v.D, nullptr, 0, nullptr, nullptr, c->grad[t0 + 5], cp, v.M, v.D, s));
    }
    if (sel(t0 + 4)) {
      Region r(c, PH_DW, t0 + 4);
      ET_G(linear_dw(c, c->dh16, v.D, b.o, v.D, c->grad[t0 + 4], v.M, v.D, v.D));
    }
    if (pass(t0 + 4)) {  // through proj.W, then through the attention core
      Region r(c, PH_DY, t0 + 4);
      et::GemmDesc g = linear_dx(c->dh16, W(t0 + 4), v.M, v.D, v.D);
      g.C = c->dattn;
      ET_G(g);
      int rc = vit_attention_backward(c, v, b);
      if (rc != ET_OK) return rc;
    }
    if (sel(t0 + 3)) {
      Region r(c, PH_DW, t0 + 3);
      ET_K(2, et::colsum(c->dqkv, nullptr, 3 * v.D, nullptr, 0, nullptr, nullptr, c->grad[t0 + 3], cp, v.M, 3 * v.D, s));
    }
    if (sel(t0 + 2)) {
      Region r(c, PH_DW, t0 + 2);
      ET_G(linear_dw(c, c->dqkv, 3 * v.D, b.a1, v.D, c->grad[t0 + 2], v.M, 3 * v.D, v.D));
    }
    if (pass(t0 + 2)) {
      Region r(c, PH_DY, t0 + 2);
      et::GemmDesc g = linear_dx(c->dqkv, W(t0 + 2), v.M, 3 * v.D, v.D);
      g.C = c->da;
      ET_G(g);
    }
    if (sel(t0 + 1)) {
      Region r(c, PH_DW, t0 + 1);
      ET_K(2, et::colsum(c->da, nullptr, v.D, nullptr, 0, nullptr, nullptr, c->grad[t0 + 1], cp, v.M, v.D, s));
    }
    if (sel(t0 + 0)) {
      Region r(c, PH_DW, t0 + 0);
      ET_K(2, et::colsum(c->da, nullptr, v.D, b.h_in, v.D, b.mean1, b.rstd1, c->grad[t0 + 0], cp, v.M, v.D, s));
    }
    if (pass(t0 + 0)) {
      Region r(c, PH_DY, t0 + 0);
      ET_K(1, et::layernorm_bwd_dx(c->da, b.h_in, v.D, b.mean1, b.rstd1, W(t0 + 0), c->dh, c->dh, c->dh16, v.D, v.M,
                                   v.D, s));
    }
  }

  // ---- embedding: pos, cls, patch.b, patch.W
  if (jstar <= 3) {
    if (sel(3)) {
      Region r(c, PH_DW, 3);
      ET_K(1, et::batchsum(c->dh, c->grad[3], v.B, (long long)v.T * v.D, v.T * v.D, s));
    }
    if (sel(2)) {
      Region r(c, PH_DW, 2);
      ET_K(1, et::batchsum(c->dh, c->grad[2], v.B, (long long)v.T * v.D, v.D, s));
    }
    if (pass(2)) {  // past the CLS token: keep the patch rows
      Region r(c, PH_DY, 2);
      ET_K(1, et::gather_patch_rows(c->dh, c->de, v.B, v.T, v.D, s));
    }
    if (sel(1)) {
      Region r(c, PH_DW, 1);
      ET_K(2, et::colsum(c->de, nullptr, v.D, nullptr, 0, nullptr, nullptr, c->grad[1], cp, v.B * (v.T - 1), v.D, s));
    }
    if (sel(0)) {
      Region r(c, PH_DW, 0);
      ET_G(linear_dw(c, c->de, v.D, (const bf16*)x, v.P, c->grad[0], v.B * (v.T - 1), v.D, v.P));
    }
  }
  return ET_OK;
}

// mask (nullable = keep everything): tensors that only the backward pass reads (the GELU derivative,
// a convolution's output ahead of its affine) are stored only if the masked backward pass will read them
int run_forward(et_ctx* c, const void* x, const int32_t* y, const uint8_t* mask = nullptr) {
  c->cur_phase = PH_FWD;
  if (c->desc.kind == ET_RESNET) return resnet_forward(c, x, y, mask);
  if (c->desc.kind == ET_VGG) return vgg_forward(c, x, y);
  if (c->desc.kind == ET_MOBILENET) return mobilenet_forward(c, x, y, mask);
  return c->desc.kind == ET_MLP ? mlp_forward(c, x, y) : vit_forward(c, x, y, mask);
}
int run_backward(et_ctx* c, const void* x, const uint8_t* mask) {
  c->cur_phase = PH_DW;
  if (c->desc.kind == ET_RESNET) return resnet_backward(c, x, mask);
  if (c->desc.kind == ET_VGG) return vgg_backward(c, x, mask);
  if (c->desc.kind == ET_MOBILENET) return mobilenet_backward(c, x, mask);
  return c->desc.kind == ET_MLP ? mlp_backward(c, x, mask) : vit_backward(c, x, mask);
}

int run_update(et_ctx* c, const uint8_t* mask, const et_opt* opt, bool dry) {
  const size_t N = c->tensors.size();
  if (c->state.empty()) return ET_ESTATE;
  if (opt->kind != ET_ADAM && opt->kind != ET_SGDW) return ET_EINVAL;
  if (opt->kind == ET_ADAM && opt->step < 1) return ET_EINVAL;
  // the chunks of the selected tensors, listed on the device; rebuilt only when the mask changes
  std::vector<uint8_t> norm(N);
  for (size_t i = 0; i < N; i++) norm[i] = mask[i] ? 1 : 0;
  if (c->upd_mask != norm) {
    c->upd_mask = norm;
    c->upd_selected.clear();
    for (size_t i = 0; i < N; i++)
      if (mask[i])
        for (uint32_t sg = c->seg_begin[i]; sg < c->seg_begin[i + 1]; sg++) c->upd_selected.push_back(sg);
    if (!c->upd_selected.empty())
      ET_HIP(hipMemcpyAsync(c->upd_selected_dev, c->upd_selected.data(), sizeof(uint32_t) * c->upd_selected.size(),
                            hipMemcpyHostToDevice, c->stream));
  }
  if (c->upd_selected.empty()) return ET_OK;
  et::OptParams p;
  p.kind = opt->kind == ET_ADAM ? 0 : 1;
  p.lr = opt->lr; p.beta1 = opt->beta1; p.beta2 = opt->beta2; p.eps = opt->eps; p.momentum = opt->momentum; p.wd = opt->wd;
  p.bc1 = (float)(1.0 - std::pow((double)opt->beta1, (double)opt->step));
  p.bc2 = (float)(1.0 - std::pow((double)opt->beta2, (double)opt->step));
  p.dry = dry ? 1 : 0;
  c->cur_phase = PH_UPD;
  Region r(c, PH_UPD, -1);
  double sel_elems = 0.0;
  for (size_t i = 0; i < N; i++)
    if (mask[i]) sel_elems += (double)c->tensors[i].numel;
  // bytes per selected element: read g + fp32 weight + moments, write fp32 weight + moments (+ bf16 copy)
  const double per_elem = (opt->kind == ET_ADAM ? 28.0 : 20.0) + (c->bf16_model ? 2.0 : 0.0);
  KernelTimer kt(c, 4, sel_elems * per_elem);
  ET_K(1, et::masked_update(c->upd_segs_dev, c->upd_selected_dev, (int)c->upd_selected.size(), c->bf16_model, p, c->stream));
  return ET_OK;
}

bool valid_mask_args(const et_ctx* c, const void* x, const int32_t* y) { return c && c->bound && x && y; }

}  // namespace

// -------------------------------------------------------------------------------------------------
// C ABI
// -------------------------------------------------------------------------------------------------
extern "C" {

const char* et_strerror(int status) {
  switch (status) {
    case ET_OK: return "ok";
    case ET_INFEASIBLE: return "budget below the forward time: empty mask";
    case ET_EINVAL: return "invalid argument";
    case ET_ENOMEM: return "out of memory or workspace too small";
    case ET_EHIP: return "HIP runtime error";
    case ET_ENAN: return "importance is NaN or infinite";
    case ET_ESTATE: return "buffers not bound";
    default: return "unknown status";
  }
}

const char* et_last_hip_error(const et_ctx* c) { return c ? hipGetErrorString(c->hip_err) : "no context"; }

int et_create(const et_model_desc* desc, void* hip_stream, et_ctx** out) {
  if (!desc || !out) return ET_EINVAL;
  *out = nullptr;
  et_ctx* c = new (std::nothrow) et_ctx();
  if (!c) return ET_ENOMEM;
  int rc;
  try {
    c->desc = *desc;
    c->stream = (hipStream_t)hip_stream;
    c->bf16_model = desc->dtype == ET_BF16;
    if (desc->kind == ET_MLP) rc = build_mlp(c);
    else if (desc->kind == ET_VIT) rc = build_vit(c);
    else if (desc->kind == ET_RESNET) rc = build_resnet(c);
    else if (desc->kind == ET_VGG) rc = build_vgg(c);
    else if (desc->kind == ET_MOBILENET) rc = build_mobilenet(c);
    else rc = ET_EINVAL;
    if (rc == ET_OK) {
      c->state_slots = c->bf16_model ? 3 : 2;
      build_tables_plan(c);
    }
  } catch (const std::bad_alloc&) {
    rc = ET_ENOMEM;
  }
  if (rc != ET_OK) {
    delete c;
    return rc;
  }
  *out = c;
  return ET_OK;
}

int et_destroy(et_ctx* c) {
  if (!c) return ET_EINVAL;
  for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->kevent_pool) (void)hipEventDestroy(e);
  delete c;
  return ET_OK;
}

int et_num_tensors(const et_ctx* c, int32_t* n) {
  if (!c || !n) return ET_EINVAL;
  *n = (int32_t)c->tensors.size();
  return ET_OK;
}

int et_tensor_info(const et_ctx* c, int32_t i, size_t* numel, int32_t* dtype, const char** name) {
  if (!c || i < 0 || (size_t)i >= c->tensors.size()) return ET_EINVAL;
  if (numel) *numel = c->tensors[i].numel;
  if (dtype) *dtype = c->tensors[i].dtype;
  if (name) *name = c->tensors[i].name.c_str();
  return ET_OK;
}

size_t et_workspace_bytes(const et_ctx* c) { return c ? c->ws_bytes : 0; }

int et_state_slots(const et_ctx* c, int32_t* k) {
  if (!c || !k) return ET_EINVAL;
  *k = c->state_slots;
  return ET_OK;
}

int et_bind(et_ctx* c, void* const* w_dev, void* const* opt_state_dev, void* const* grad_dev, void* workspace_dev,
            size_t workspace_bytes) {
  if (!c || !w_dev || !grad_dev || !workspace_dev) return ET_EINVAL;
  if (workspace_bytes < c->ws_bytes) return ET_ENOMEM;
  if (reinterpret_cast<uintptr_t>(workspace_dev) & 255) return ET_EINVAL;
  const size_t N = c->tensors.size();
  const int k = c->state_slots;
  for (size_t i = 0; i < N; i++) {
    if (!w_dev[i] || !grad_dev[i]) return ET_EINVAL;
    if ((reinterpret_cast<uintptr_t>(w_dev[i]) | reinterpret_cast<uintptr_t>(grad_dev[i])) & 15) return ET_EINVAL;
    if (opt_state_dev)
      for (int s = 0; s < k; s++)
        if (!opt_state_dev[i * k + s] || (reinterpret_cast<uintptr_t>(opt_state_dev[i * k + s]) & 15)) return ET_EINVAL;
  }
  try {
    c->bound = false;
    c->upd_mask.clear();          // the device list of selected chunks lives in the (new) workspace
    c->upd_selected.clear();
    c->w.assign(w_dev, w_dev + N);
    c->grad.resize(N);
    for (size_t i = 0; i < N; i++) c->grad[i] = (float*)grad_dev[i];
    c->state.clear();
    if (opt_state_dev) {
      c->state.resize(N * k);
      for (size_t i = 0; i < N * k; i++) c->state[i] = (float*)opt_state_dev[i];
    }
    c->ws = (unsigned char*)workspace_dev;
    for (auto& pr : c->plan) *pr.first = c->ws + pr.second;
    // static tables
    c->upd_segs_host.assign(c->n_segs, et::UpdateSeg());
    c->imp_segs_host.assign(c->n_segs, et::TensorSeg());
    const size_t wsize = c->bf16_model ? sizeof(bf16) : sizeof(float);
    for (size_t i = 0; i < N; i++) {
      for (uint32_t sg = c->seg_begin[i]; sg < c->seg_begin[i + 1]; sg++) {
        const size_t off = (size_t)(sg - c->seg_begin[i]) * SEG_ELEMS;
        const uint32_t n = (uint32_t)std::min<size_t>(SEG_ELEMS, c->tensors[i].numel - off);
        et::UpdateSeg& u = c->upd_segs_host[sg];
        u.g = c->grad[i] + off;
        u.w = (unsigned char*)c->w[i] + off * wsize;
        u.n = n;
        u.tensor = (uint32_t)i;
        u.master = u.m = u.v = nullptr;
        if (opt_state_dev) {
          if (c->bf16_model) {
            u.master = c->state[i * k + 0] + off; u.m = c->state[i * k + 1] + off; u.v = c->state[i * k + 2] + off;
          } else {
            u.m = c->state[i * k + 0] + off; u.v = c->state[i * k + 1] + off;
          }
        }
        et::TensorSeg& t = c->imp_segs_host[sg];
        t.g = u.g; t.w = u.w; t.w_snap = nullptr; t.n = n; t.tensor = (uint32_t)i;
      }
    }
  } catch (const std::bad_alloc&) {
    return ET_ENOMEM;
  }
  ET_HIP(et::fill_zero(c->ws, c->ws_bytes, c->stream));
  ET_HIP(hipMemcpyAsync(c->upd_segs_dev, c->upd_segs_host.data(), sizeof(et::UpdateSeg) * c->n_segs,
                        hipMemcpyHostToDevice, c->stream));
  ET_HIP(hipMemcpyAsync(c->seg_begin_dev, c->seg_begin.data(), sizeof(uint32_t) * (N + 1), hipMemcpyHostToDevice,
                        c->stream));
  ET_HIP(hipStreamSynchronize(c->stream));
  c->bound = true;
  return ET_OK;
}

int et_train_step(et_ctx* c, const void* x_dev, const int32_t* y_dev, const uint8_t* mask_host, const et_opt* opt,
                  float* loss_host) {
  if (!c || !x_dev || !y_dev || !mask_host) return ET_EINVAL;
  if (!c->bound) return ET_ESTATE;
  if (reinterpret_cast<uintptr_t>(x_dev) & 15) return ET_EINVAL;
  c->launches[0] = c->launches[1] = c->launches[2] = c->launches[3] = 0;
  int rc = run_forward(c, x_dev, y_dev, mask_host);
  if (rc != ET_OK) return rc;
  rc = run_backward(c, x_dev, mask_host);
  if (rc != ET_OK) return rc;
  if (opt) {
    rc = run_update(c, mask_host, opt, false);
    if (rc != ET_OK) return rc;
  }
  if (loss_host) {
    ET_HIP(hipMemcpyAsync(loss_host, c->loss, sizeof(float), hipMemcpyDeviceToHost, c->stream));
    ET_HIP(hipStreamSynchronize(c->stream));
  }
  return ET_OK;
}

int et_last_launch_counts(const et_ctx* c, int32_t* forward, int32_t* backward, int32_t* update) {
  if (!c) return ET_EINVAL;
  if (forward) *forward = c->launches[PH_FWD];
  if (backward) *backward = c->launches[PH_DW] + c->launches[PH_DY];
  if (update) *update = c->launches[PH_UPD];
  return ET_OK;
}

int et_debug_activation(const et_ctx* c, const char* name, const void** dev, size_t* numel) {
  if (!c || !name || !dev || !numel || !c->bound) return ET_EINVAL;
  const std::string n(name);
  const size_t B = c->desc.batch;
  *dev = nullptr;
  *numel = 0;
  auto give = [&](const void* p, size_t count) { *dev = p; *numel = count; return p ? ET_OK : ET_ESTATE; };
  if (c->desc.kind == ET_VGG) {
    for (size_t i = 0; i < c->vconv.size(); i++) {
      const ConvUnit& u = c->vconv[i];
      const std::string pre = "conv" + std::to_string(i);
      if (n == pre + ".in") return give(u.in, B * u.H * u.W * u.Cin);
      if (n == pre + ".y") return give(u.y, B * u.Ho * u.Wo * u.Cout);
    }
    for (size_t j = 0; j < c->vact.size(); j++)
      if (n == "fc" + std::to_string(j) + ".in") return give(c->vact[j], B * c->vdims[j]);
  } else if (c->desc.kind == ET_RESNET) {
    const ConvUnit& st = c->stem;
    if (n == "stem.y") return give(c->pool_y, B * st.Ho * st.Wo * st.Cout);
    if (n == "pooled") return give(c->pooled, B * c->rblk[0].c1.H * c->rblk[0].c1.W * st.Cout);
    for (size_t i = 0; i < c->rblk.size(); i++) {
      const ResBlockBufs& b = c->rblk[i];
      const std::string pre = "blk" + std::to_string(i);
      if (n == pre + ".x") return give(b.x, B * b.c1.H * b.c1.W * b.c1.Cin);
      if (n == pre + ".y1") return give(b.c1.y, B * b.c1.Ho * b.c1.Wo * b.c1.Cout);
      if (n == pre + ".y2") return give(b.c2.y, B * b.c2.Ho * b.c2.Wo * b.c2.Cout);
      if (n == pre + ".y") return give(b.y, B * b.c3.Ho * b.c3.Wo * b.c3.Cout);
    }
  } else if (c->desc.kind == ET_MOBILENET) {
    if (n == "stem.y") return give(c->stem.y, B * c->stem.Ho * c->stem.Wo * c->stem.Cout);
    if (n == "last.y") return give(c->mlast.y, B * c->mlast.Ho * c->mlast.Wo * c->mlast.Cout);
    for (size_t i = 0; i < c->mblk.size(); i++) {
      const MbBlockBufs& b = c->mblk[i];
      const std::string pre = "b" + std::to_string(i);
      if (n == pre + ".x") return give(b.x, B * b.H * b.W * b.Cin);
      if (n == pre + ".y_exp") return give(b.expand ? b.y_exp : b.x, B * b.H * b.W * b.hid);
      if (n == pre + ".y_dw") return give(b.y_dw, B * b.Ho * b.Wo * b.hid);
      if (n == pre + ".y") return give(b.y, B * b.Ho * b.Wo * b.Cout);
    }
  }
  return ET_EINVAL;
}

int et_kernel_timing(et_ctx* c, int32_t enable) {
  if (!c) return ET_EINVAL;
  ET_HIP(hipStreamSynchronize(c->stream));
  c->ktiming = enable != 0;
  c->krecs.clear();
  c->kcal.clear();
  c->kevents_used = 0;
  if (c->ktiming) {
    // what an event pair measures with nothing between its events (the hand-over between two commands)
    for (int i = 0; i < 33; i++) {
      KernelRecord r;
      r.cls = -1;
      r.work = 0.0;
      for (hipEvent_t* ev : {&r.e0, &r.e1}) {
        if (c->kevents_used == c->kevent_pool.size()) {
          hipEvent_t e;
          ET_HIP(hipEventCreate(&e));
          c->kevent_pool.push_back(e);
        }
        *ev = c->kevent_pool[c->kevents_used++];
      }
      ET_HIP(hipEventRecord(r.e0, c->stream));
      ET_HIP(hipEventRecord(r.e1, c->stream));
      c->kcal.push_back(r);
    }
  }
  return ET_OK;
}

int et_kernel_timing_overhead(et_ctx* c, double* ns_per_pair) {
  if (!c || !ns_per_pair) return ET_EINVAL;
  if (c->kcal.empty()) return ET_ESTATE;
  ET_HIP(hipStreamSynchronize(c->stream));
  std::vector<double> t;
  for (const KernelRecord& r : c->kcal) {
    float ms = 0.f;
    ET_HIP(hipEventElapsedTime(&ms, r.e0, r.e1));
    t.push_back((double)ms * 1e6);
  }
  std::sort(t.begin(), t.end());
  *ns_per_pair = t[t.size() / 2];
  return ET_OK;
}

int et_kernel_timing_read(et_ctx* c, int32_t kernel_class, uint64_t* launches, double* total_ns, double* work) {
  if (!c || kernel_class < 0 || kernel_class >= ET_NUM_KERNEL_CLASSES) return ET_EINVAL;
  ET_HIP(hipStreamSynchronize(c->stream));
  uint64_t n = 0;
  double ns = 0.0, w = 0.0;
  for (const KernelRecord& r : c->krecs) {
    if (r.cls != kernel_class) continue;
    float ms = 0.f;
    ET_HIP(hipEventElapsedTime(&ms, r.e0, r.e1));
    n++;
    ns += (double)ms * 1e6;
    w += r.work;
  }
  if (launches) *launches = n;
  if (total_ns) *total_ns = ns;
  if (work) *work = w;
  return ET_OK;
}

namespace {
// full backward pass, then one segmented reduction of g * (snapshot - w) over all tensors;
// master: both are float32 (snapshot of, and current, master weights)
int importance_impl(et_ctx* c, const void* x_dev, const int32_t* y_dev, void* const* snapshot_dev,
                    double* importance_host, bool master, int metric = 0) {
  if (!c || !importance_host || metric < 0 || metric > 2) return ET_EINVAL;
  if (metric != 1 && (!x_dev || !y_dev)) return ET_EINVAL;   // the weight magnitude needs no pass over data
  if (metric == 0 && !snapshot_dev) return ET_EINVAL;
  if (!c->bound) return ET_ESTATE;
  if (master && !c->bf16_model) return ET_EINVAL;
  if (master && c->state.empty()) return ET_ESTATE;
  const size_t N = c->tensors.size();
  const bool bf16_w = c->bf16_model && !master;
  const size_t wsize = bf16_w ? sizeof(bf16) : sizeof(float);
  if (metric == 0)
    for (size_t i = 0; i < N; i++)
      if (!snapshot_dev[i] || (reinterpret_cast<uintptr_t>(snapshot_dev[i]) & 15)) return ET_EINVAL;
  std::vector<uint8_t> ones(N, 1);
  c->launches[0] = c->launches[1] = c->launches[2] = c->launches[3] = 0;
  if (metric != 1) {
    int rc = run_forward(c, x_dev, y_dev);
    if (rc != ET_OK) return rc;
    rc = run_backward(c, x_dev, ones.data());
    if (rc != ET_OK) return rc;
  }
  const int k = c->state_slots;
  for (size_t i = 0; i < N; i++)
    for (uint32_t sg = c->seg_begin[i]; sg < c->seg_begin[i + 1]; sg++) {
      const size_t off = (size_t)(sg - c->seg_begin[i]) * SEG_ELEMS;
      et::TensorSeg& t = c->imp_segs_host[sg];
      t.w = master ? (const void*)(c->state[i * k] + off) : (const void*)((const unsigned char*)c->w[i] + off * wsize);
      t.w_snap = metric == 0 ? (const unsigned char*)snapshot_dev[i] + off * wsize : t.w;
    }
  ET_HIP(hipMemcpyAsync(c->imp_segs_dev, c->imp_segs_host.data(), sizeof(et::TensorSeg) * c->n_segs,
                        hipMemcpyHostToDevice, c->stream));
  c->cur_phase = PH_DW;
  double imp_bytes = 0.0;
  for (size_t i = 0; i < N; i++) imp_bytes += (double)c->tensors[i].numel * (metric == 0 ? 4.0 + 2.0 * wsize : (metric == 1 ? (double)wsize : 4.0));
  {
    KernelTimer kt(c, 3, imp_bytes);
    ET_K(2, et::importance_reduce(c->imp_segs_dev, (int)c->n_segs, c->seg_begin_dev, (int)N, bf16_w, c->imp_partial_dev,
                                  c->imp_out_dev, c->stream, metric));
  }
  ET_HIP(hipMemcpyAsync(importance_host, c->imp_out_dev, sizeof(double) * N, hipMemcpyDeviceToHost, c->stream));
  ET_HIP(hipStreamSynchronize(c->stream));
  return ET_OK;
}
}  // namespace

int et_importance(et_ctx* c, const void* x_dev, const int32_t* y_dev, void* const* w_snapshot_dev,
                  double* importance_host) {
  return importance_impl(c, x_dev, y_dev, w_snapshot_dev, importance_host, false);
}

int et_importance_master(et_ctx* c, const void* x_dev, const int32_t* y_dev, void* const* w_snapshot_f32_dev,
                         double* importance_host) {
  return importance_impl(c, x_dev, y_dev, w_snapshot_f32_dev, importance_host, true);
}

int et_tensor_metric(et_ctx* c, const void* x_dev, const int32_t* y_dev, int32_t metric, double* metric_host) {
  if (metric != ET_METRIC_WEIGHT_L1 && metric != ET_METRIC_GRAD_L1) return ET_EINVAL;
  return importance_impl(c, x_dev, y_dev, nullptr, metric_host, false, metric);
}

int et_profile(et_ctx* c, const void* x_dev, const int32_t* y_dev, int32_t warmup, int32_t reps, uint64_t* t_fwd_ns,
               uint64_t* t_dw_ns, uint64_t* t_dy_ns) {
  if (!c || !x_dev || !y_dev || !t_fwd_ns || !t_dw_ns || !t_dy_ns || warmup < 0 || reps < 1) return ET_EINVAL;
  if (!c->bound) return ET_ESTATE;
  const size_t N = c->tensors.size();
  std::vector<uint8_t> ones(N, 1);
  et_opt opt;
  std::memset(&opt, 0, sizeof(opt));
  opt.kind = c->bf16_model ? ET_ADAM : ET_SGDW;
  opt.lr = 1e-4f; opt.beta1 = 0.9f; opt.beta2 = 0.999f; opt.eps = 1e-8f; opt.momentum = 0.9f; opt.wd = 5e-4f; opt.step = 1;
  const bool with_update = !c->state.empty();
  // per rep: forward time, per tensor dw / dy, update
  std::vector<std::vector<double>> fwd(1), dw(N), dy(N), upd(1);
  for (int it = 0; it < warmup + reps; it++) {
    const bool timed = it >= warmup;
    c->profiling = timed;
    c->scopes.clear();
    c->events_used = 0;
    int rc = run_forward(c, x_dev, y_dev);
    if (rc == ET_OK) rc = run_backward(c, x_dev, ones.data());
    if (rc == ET_OK && with_update) rc = run_update(c, ones.data(), &opt, true);
    c->profiling = false;
    if (rc != ET_OK) return rc;
    ET_HIP(hipStreamSynchronize(c->stream));
    if (c->hip_err != hipSuccess) return ET_EHIP;
    if (!timed) continue;
    // the same iteration without regions, timed as a whole: the instrumented one is slower by the
    // measurement's own overhead, which is taken off the regions in equal parts (a region never
    // loses more than half of what it measured)
    hipEvent_t p0, p1;
    ET_HIP(get_event(c, &p0));
    ET_HIP(get_event(c, &p1));
    ET_HIP(hipEventRecord(p0, c->stream));
    rc = run_forward(c, x_dev, y_dev);
    if (rc == ET_OK) rc = run_backward(c, x_dev, ones.data());
    if (rc == ET_OK && with_update) rc = run_update(c, ones.data(), &opt, true);
    if (rc != ET_OK) return rc;
    ET_HIP(hipEventRecord(p1, c->stream));
    ET_HIP(hipStreamSynchronize(c->stream));
    if (c->hip_err != hipSuccess) return ET_EHIP;
    float plain_ms = 0.f;
    ET_HIP(hipEventElapsedTime(&plain_ms, p0, p1));
    double instrumented = 0.0;
    for (const Scope& sc : c->scopes) {
      float ms = 0.f;
      ET_HIP(hipEventElapsedTime(&ms, sc.e0, sc.e1));
      instrumented += (double)ms * 1e6;
    }
    const double overhead = c->scopes.empty() ? 0.0 : std::max(0.0, (instrumented - (double)plain_ms * 1e6) / (double)c->scopes.size());
    std::vector<double> sdw(N, 0.0), sdy(N, 0.0);
    double sf = 0.0, su = 0.0;
    for (const Scope& sc : c->scopes) {
      float ms = 0.f;
      ET_HIP(hipEventElapsedTime(&ms, sc.e0, sc.e1));
      double ns = (double)ms * 1e6;
      ns -= std::min(overhead, 0.5 * ns);
      if (sc.phase == PH_FWD) sf += ns;
      else if (sc.phase == PH_UPD) su += ns;
      else if (sc.phase == PH_DW && sc.tensor2 >= 0) { sdw[sc.tensor] += 0.5 * ns; sdw[sc.tensor2] += 0.5 * ns; }
      else if (sc.phase == PH_DW) sdw[sc.tensor] += ns;
      else sdy[sc.tensor] += ns;
    }
    fwd[0].push_back(sf);
    upd[0].push_back(su);
    for (size_t i = 0; i < N; i++) { dw[i].push_back(sdw[i]); dy[i].push_back(sdy[i]); }
  }
  auto median = [](std::vector<double>& v) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    return n % 2 ? v[n / 2] : 0.5 * (v[n / 2 - 1] + v[n / 2]);
  };
  *t_fwd_ns = (uint64_t)std::llround(median(fwd[0]));
  const double upd_ns = median(upd[0]);
  double total_elems = 0.0;
  for (size_t i = 0; i < N; i++) total_elems += (double)c->tensors[i].numel;
  for (size_t i = 0; i < N; i++) {
    // the update is one launch over all selected tensors: a tensor's share is its share of the bytes
    const double share = upd_ns * (double)c->tensors[i].numel / total_elems;
    t_dw_ns[i] = (uint64_t)std::llround(median(dw[i]) + share);
    t_dy_ns[i] = (uint64_t)std::llround(median(dy[i]));
  }
  return ET_OK;
}

}  // extern "C"
