// Shared state of the step executor: the context behind the C ABI, the workspace planner, the
// timed regions of the profiler (Section 5) and the GEMM launch helpers used by the per-model
// forward / backward chains.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "et.h"
#include "kernels.h"

using et::bf16;

namespace et_exec {

constexpr uint32_t SEG_ELEMS = 16384;  // elements per chunk of the importance / update tables

enum Phase { PH_FWD = 0, PH_DW = 1, PH_DY = 2, PH_UPD = 3 };

struct TensorInfo {
  std::string name;
  size_t numel;
  int32_t dtype;
};

struct Scope {  // one timed region of the profile (tensor2 >= 0: its time is shared evenly by two tensors)
  int phase, tensor, tensor2;
  hipEvent_t e0, e1;
};

struct KernelRecord {  // one timed kernel launch (measurement support)
  int cls;
  double work;
  hipEvent_t e0, e1;
};

struct VitBlockBufs {
  float *h_in, *h_mid, *mean1, *rstd1, *mean2, *rstd2, *lse;
  bf16 *a1, *qkv, *p, *o, *a2, *u, *ga;
};

// activations kept by one convolution + affine (+ReLU) unit of the ResNet
struct ConvUnit {
  int t;                      // tensor index of the convolution weight (gain t+1, shift t+2)
  int H, W, Cin, Ho, Wo, Cout, k, stride, Kc;   // Kc: padded column count of the im2col matrix
  const bf16* in;             // input activation [B,H,W,Cin]
  bf16* cols;                 // im2col matrix [B*Ho*Wo][Kc] (null: the input itself is the matrix)
  bf16* z;                    // convolution output [B*Ho*Wo][Cout]
  bf16* y;                    // after affine (+ReLU); for the last unit of a block: the block output
};
struct ResBlockBufs {
  int t;
  bool proj;
  ConvUnit c1, c2, c3, sc;
  const bf16* x;              // block input
  bf16* y;                    // block output (after the closing ReLU)
};

// activations kept by one inverted-residual block (MobileNetV2 family)
struct MbBlockBufs {
  int t, t_dw;                 // tensor index of the block's first weight and of its depthwise weight
  int Cin, hid, Cout, stride, H, W, Ho, Wo;
  bool expand, shortcut;
  const bf16* x;               // block input [B,H,W,Cin]
  bf16 *z_exp, *y_exp;         // expansion: convolution output, after affine + ReLU6   [B,H,W,hid]
  bf16 *z_dw, *y_dw;           // depthwise: the same                                   [B,Ho,Wo,hid]
  bf16 *z_proj, *y;            // projection output and the block output                [B,Ho,Wo,Cout]
};

}  // namespace et_exec
using namespace et_exec;

struct et_ctx {
  et_model_desc desc;
  hipStream_t stream = nullptr;
  std::vector<TensorInfo> tensors;
  int32_t state_slots = 0;
  bool bf16_model = false;

  // workspace plan (offsets in bytes)
  size_t ws_bytes = 0;
  std::vector<std::pair<void**, size_t>> plan;  // (where to store the pointer, offset)

  // bound buffers
  bool bound = false;
  std::vector<void*> w;
  std::vector<float*> grad;
  std::vector<float*> state;
  unsigned char* ws = nullptr;

  // MLP buffers
  std::vector<float*> act;  // act[i]: input of layer i (act[0] is x itself, not in the workspace)
  float *logits = nullptr, *dlogits = nullptr, *loss = nullptr, *dbuf[2] = {nullptr, nullptr};

  // ViT buffers
  std::vector<VitBlockBufs> blk;
  float *e = nullptr, *h_out = nullptr, *s_f32 = nullptr, *meanf = nullptr, *rstdf = nullptr, *dh = nullptr;
  bf16 *zc = nullptr, *dl16 = nullptr, *dz = nullptr, *dh16 = nullptr, *da = nullptr, *du = nullptr, *dattn = nullptr,
       *dqkv = nullptr, *ds = nullptr, *de = nullptr;
  float *gemm_partials = nullptr, *colsum_partials = nullptr;
  size_t gemm_partial_elems = 0;

  // ResNet buffers
  ConvUnit stem;
  std::vector<ResBlockBufs> rblk;
  bf16 *stem_w8 = nullptr, *pool_y = nullptr, *pooled = nullptr, *rd[3] = {nullptr, nullptr, nullptr}, *rdsum = nullptr,
       *rdsc = nullptr, *rdcols = nullptr;
  uint8_t* pool_arg = nullptr;
  float *stem_dw8 = nullptr, *stem_z32 = nullptr;
  bf16* stem_xpad = nullptr;   // ResNet stem as a gathered GEMM: the image padded to 4 channels and by the window
  int stem_hp = 0, stem_wp = 0;

  // plain convolution stack (VGG family): one unit per convolution (y: after bias + ReLU),
  // per stage the pooled output and the chosen taps, the inputs of the linear layers
  std::vector<ConvUnit> vconv;
  std::vector<int> vstage;
  std::vector<bf16*> vpool;
  std::vector<uint8_t*> varg;
  std::vector<bf16*> vact;
  std::vector<int> vdims;           // vdims[j] -> vdims[j+1]: linear layer j
  bf16* wflip = nullptr;            // mirrored weight of the convolution whose dy() is running
  float* fc_z32 = nullptr;          // reduced sum of a linear layer's split forward product

  // inverted-residual network: blocks; the stem and the last convolution are ConvUnits (`stem`, `mlast`)
  std::vector<MbBlockBufs> mblk;
  ConvUnit mlast;
  float* dw_part = nullptr;         // partial sums of a depthwise weight gradient

  // tables for importance / update
  std::vector<uint32_t> seg_begin;  // [N+1]
  uint32_t n_segs = 0;
  et::TensorSeg* imp_segs_dev = nullptr;
  et::UpdateSeg* upd_segs_dev = nullptr;
  uint32_t* seg_begin_dev = nullptr;
  uint32_t* upd_selected_dev = nullptr;   // indices of the chunks of the tensors selected by upd_mask
  std::vector<uint32_t> upd_selected;
  std::vector<uint8_t> upd_mask;          // the mask upd_selected_dev was built for
  double *imp_partial_dev = nullptr, *imp_out_dev = nullptr;
  std::vector<et::UpdateSeg> upd_segs_host;
  std::vector<et::TensorSeg> imp_segs_host;

  // launch accounting and profiling
  int32_t launches[4] = {0, 0, 0, 0};
  int cur_phase = PH_FWD;
  bool profiling = false;
  std::vector<Scope> scopes;
  std::vector<hipEvent_t> event_pool;
  size_t events_used = 0;
  hipError_t hip_err = hipSuccess;

  // per-kernel-class timing
  bool ktiming = false;
  std::vector<KernelRecord> kcal;   // event pairs with nothing between them, recorded when timing is enabled
  std::vector<KernelRecord> krecs;
  std::vector<hipEvent_t> kevent_pool;
  size_t kevents_used = 0;
};

namespace et_exec {

#define ET_HIP(expr)                       \
  do {                                     \
    hipError_t e__ = (expr);               \
    if (e__ != hipSuccess) {               \
      c->hip_err = e__;                    \
      return ET_EHIP;                      \
    }                                      \
  } while (0)

// kernel launch through a wrapper that returns hipError_t; counts the launches
#define ET_K(n, expr)                      \
  do {                                     \
    hipError_t e__ = (expr);               \
    if (e__ != hipSuccess) {               \
      c->hip_err = e__;                    \
      return ET_EHIP;                      \
    }                                      \
    c->launches[c->cur_phase] += (n);      \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int round8(int v) { return (v + 7) & ~7; }

template <typename T>
inline void reserve(et_ctx* c, T** where, size_t bytes) {
  c->plan.emplace_back(reinterpret_cast<void**>(where), c->ws_bytes);
  c->ws_bytes += align_up(bytes, 256);
}

inline hipError_t get_event(et_ctx* c, hipEvent_t* ev) {
  if (c->events_used == c->event_pool.size()) {
    hipEvent_t e;
    hipError_t r = hipEventCreate(&e);
    if (r != hipSuccess) return r;
    c->event_pool.push_back(e);
  }
  *ev = c->event_pool[c->events_used++];
  return hipSuccess;
}

// timed region: events are recorded only while profiling
struct Region {
  et_ctx* c;
  bool on;
  size_t idx = 0;
  Region(et_ctx* ctx, int phase, int tensor, int tensor2 = -1) : c(ctx), on(ctx->profiling) {
    c->cur_phase = phase;
    if (!on) return;
    Scope s;
    s.phase = phase;
    s.tensor = tensor;
    s.tensor2 = tensor2;
    if (get_event(c, &s.e0) != hipSuccess || get_event(c, &s.e1) != hipSuccess) {
      on = false;
      c->hip_err = hipErrorOutOfMemory;
      return;
    }
    (void)hipEventRecord(s.e0, c->stream);
    idx = c->scopes.size();
    c->scopes.push_back(s);
  }
  ~Region() {
    if (on) (void)hipEventRecord(c->scopes[idx].e1, c->stream);
  }
};

// split of the reduction dimension for a weight gradient [Mo][No] reduced over K rows
inline int split_for(int Mo, int No, int K) {
  int tile, split;
  et::gemm_bf16_plan_split(Mo, No, K, &tile, &split);
  return split;
}

// Y[M][N] = X[M][K] W[N][K]^T (+ bias) ...
inline et::GemmDesc linear_fwd(const bf16* X, const bf16* W, const bf16* bias, int M, int N, int K) {
  et::GemmDesc g;
  g.A = X; g.lda = K; g.B = W; g.ldb = K; g.M = M; g.N = N; g.K = K; g.bias = bias; g.ldc = N;
  return g;
}
// dX[M][K] = dY[M][N] W[N][K]
inline et::GemmDesc linear_dx(const bf16* dY, const bf16* W, int M, int N, int K) {
  et::GemmDesc g;
  g.A = dY; g.lda = N; g.B = W; g.b_t = true; g.ldb = K; g.M = M; g.N = K; g.K = N; g.ldc = K;
  return g;
}
// dW[N][K] = dY[M][N]^T X[M][K], fp32, split over the rows
inline et::GemmDesc linear_dw(et_ctx* c, const bf16* dY, int ldy, const bf16* X, int ldx, float* dW, int M, int N, int K) {
  et::GemmDesc g;
  g.A = dY; g.a_t = true; g.lda = ldy; g.B = X; g.b_t = true; g.ldb = ldx; g.M = N; g.N = K; g.K = M;
  g.C = dW; g.ldc = K; g.c_f32 = true;
  et::gemm_bf16_plan_split(N, K, M, &g.tile, &g.split_k);
  g.partials = c->gemm_partials;
  if (et::gemm_bf16_partial_elems(N, K, g.split_k) > c->gemm_partial_elems) { g.split_k = 1; g.tile = 0; }
  return g;
}

// bracket a launch with events while per-kernel timing is on
struct KernelTimer {
  et_ctx* c;
  bool on = false;
  size_t idx = 0;
  KernelTimer(et_ctx* ctx, int cls, double work) : c(ctx) {
    if (!c->ktiming) return;
    KernelRecord r;
    r.cls = cls;
    r.work = work;
    for (hipEvent_t* ev : {&r.e0, &r.e1}) {
      if (c->kevents_used == c->kevent_pool.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { c->hip_err = hipErrorOutOfMemory; return; }
        c->kevent_pool.push_back(e);
      }
      *ev = c->kevent_pool[c->kevents_used++];
    }
    (void)hipEventRecord(r.e0, c->stream);
    idx = c->krecs.size();
    c->krecs.push_back(r);
    on = true;
  }
  ~KernelTimer() {
    if (on) (void)hipEventRecord(c->krecs[idx].e1, c->stream);
  }
};

inline int launch_gemm(et_ctx* c, const et::GemmDesc& g) {
  int n = 0;
  const int cls = g.a_t ? 2 : (g.b_t ? 1 : 0);
  KernelTimer kt(c, cls, 2.0 * g.M * g.N * (double)g.K * g.z_outer * g.z_inner);
  hipError_t e = et::gemm_bf16(g, c->stream, &n);
  if (e != hipSuccess) { c->hip_err = e; return ET_EHIP; }
  c->launches[c->cur_phase] += n;
  return ET_OK;
}
#define ET_G(g)                            \
  do {                                     \
    int r__ = launch_gemm(c, (g));         \
    if (r__ != ET_OK) return r__;          \
  } while (0)

}  // namespace et_exec

// per-model chains (each in its own file)
int build_resnet(et_ctx* c);
// mask (nullable = keep everything): the forward pass stores a backward-only tensor only if the
// masked backward pass will read it
int resnet_forward(et_ctx* c, const void* x, const int32_t* y, const uint8_t* mask);
int resnet_backward(et_ctx* c, const void* x, const uint8_t* mask);
int build_mobilenet(et_ctx* c);
int mobilenet_forward(et_ctx* c, const void* x, const int32_t* y, const uint8_t* mask);
int mobilenet_backward(et_ctx* c, const void* x, const uint8_t* mask);
int build_vgg(et_ctx* c);
int vgg_forward(et_ctx* c, const void* x, const int32_t* y);
int vgg_backward(et_ctx* c, const void* x, const uint8_t* mask);
