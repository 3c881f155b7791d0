// Host side of the bf16 MFMA GEMM: argument checks, tile choice, split-K reduction.
#include <algorithm>

#include "gemm_bf16_kernels.h"

namespace et {
namespace {

// out[i] = sum_z part[z][i], z ascending: the same order on every run
__global__ void splitk_reduce_kernel(const float4* __restrict__ part, float4* __restrict__ out, size_t n4, int splits) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= n4) return;
  float4 s = part[i];
  for (int z = 1; z < splits; z++) {
    const float4 p = part[(size_t)z * n4 + i];
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  out[i] = s;
}

// many chunks, few outputs: 16 lanes share one output vector, lane g adds the chunks g, g + 16, ... in
// order, then the 16 sums are added in lane order (through LDS): again the same order on every run
__global__ __launch_bounds__(256) void splitk_reduce_wide_kernel(const float4* __restrict__ part, float4* __restrict__ out,
                                                                 size_t n4, int splits) {
  __shared__ float4 sh[16][16];
  const int o = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const size_t i = blockIdx.x * (size_t)16 + o;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n4)
    for (int z = grp; z < splits; z += 16) {
      const float4 p = part[(size_t)z * n4 + i];
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
  sh[grp][o] = s;
  __syncthreads();
  if (grp == 0 && i < n4) {
    float4 t = sh[0][o];
    for (int k = 1; k < 16; k++) {
      const float4 p = sh[k][o];
      t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
    }
    out[i] = t;
  }
}

// Split implicit convolution: out = epilogue(sum_z part[z]), z ascending.  mode: 0 bf16 copy, 1 max(v + bias, 0),
// 2 0 < U < mask_hi ? v : 0, 3 z = bf16(v) (kept if zout), y = clamp(z * gain + bias, lo, hi)
struct ReduceEpi {
  const float4* part;
  size_t n4;
  int splits, N, mode;
  const bf16* bias;
  const bf16* gain;
  const bf16* U;
  bf16* out;
  bf16* zout;
  float lo, hi, mask_hi;
};

__global__ __launch_bounds__(256) void splitk_reduce_epilogue_kernel(ReduceEpi e) {
  typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= e.n4) return;
  float4 s = e.part[i];
  for (int z = 1; z < e.splits; z++) {
    const float4 p = e.part[(size_t)z * e.n4 + i];
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  float v[4] = {s.x, s.y, s.z, s.w};
  const int col = (int)((i * 4) % (size_t)e.N);
  bf16x4 o;
  if (e.mode == 1) {
    const bf16x4 b = *(const bf16x4*)(e.bias + col);
#pragma unroll
    for (int j = 0; j < 4; j++) o[j] = (bf16)fmaxf(v[j] + (float)b[j], 0.f);
  } else if (e.mode == 2) {
    const bf16x4 u = ((const bf16x4*)e.U)[i];
#pragma unroll
    for (int j = 0; j < 4; j++) o[j] = ((float)u[j] > 0.f && (float)u[j] < e.mask_hi) ? (bf16)v[j] : (bf16)0.f;
  } else if (e.mode == 3) {
    const bf16x4 g = *(const bf16x4*)(e.gain + col), b = *(const bf16x4*)(e.bias + col);
    bf16x4 z;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      z[j] = (bf16)v[j];
      o[j] = (bf16)fminf(fmaxf((float)z[j] * (float)g[j] + (float)b[j], e.lo), e.hi);
    }
    if (e.zout) ((bf16x4*)e.zout)[i] = z;
  } else {
#pragma unroll
    for (int j = 0; j < 4; j++) o[j] = (bf16)v[j];
  }
  ((bf16x4*)e.out)[i] = o;
}

enum TileId : int { T_AUTO = 0, T_128x128 = 1, T_128x64 = 3, T_DMA_256x256 = 5, T_DMA_256x128 = 7, T_PP_256x256 = 11, T_PP_256x192 = 13,
              T_PP_256x128 = 15, T_PP_512x64 = 17, T_PP_128x256 = 19, T_PP_64x512 = 21 };

// number of compute units of the current device (256 on an MI355X), looked up once per device; a multiple of 8
// (one share per XCD) as the resident kernels' unit order assumes whenever a workgroup takes a second unit
int compute_units() {
  static int cus[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
    cus[dev] = n & ~7;
  }
  return cus[dev];
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Cost model behind the tile and split choice for large problems (seconds, one launch):
//   rounds of workgroups over the 256 CUs x time of one workgroup at the rate a CU sustains with
//   that tile (measured on the ViT shapes: about 3.3 TFLOP/s per CU with the 256x256 two-group
//   tile, 3.0 with 256x192), plus, for a split reduction, writing and re-reading the fp32 partials.
struct Plan { int tile, split; double cost; };

struct TileRate { int tile, bm, bn; double rate; };

Plan plan_tiles(int M, int N, int K, bool may_split, const TileRate* cand, int n_cand) {
  Plan best = {T_AUTO, 1, 1e30};
  const int slices = (K + gemm::PBK - 1) / gemm::PBK;
  const int max_split = may_split ? std::max(1, std::min(256, slices / 4)) : 1;
  for (int ci = 0; ci < n_cand; ci++) {
    const TileRate& c = cand[ci];
    const long long tiles = (long long)((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
    for (int s = 1; s <= max_split; s++) {
      const int per = (slices + s - 1) / s;
      const int chunks = (slices + per - 1) / per;
      if (chunks != s) continue;   // this split leaves empty chunks: the same work as a smaller one
      const long long rounds = (tiles * s + 255) / 256;
      double t = rounds * (2.0 * c.bm * c.bn * per * gemm::PBK / c.rate);
      if (s > 1) t += (2.0 * s + 1.0) * M * N * 4.0 / 3.5e12 + 4e-6;   // partial traffic and one more launch
      if (t < best.cost) best = {c.tile, s, t};
    }
  }
  return best;
}

Plan plan_large(int M, int N, int K, bool may_split) {
  static const TileRate cand[2] = {{T_PP_256x256, 256, 256, 3.3e12}, {T_PP_256x192, 256, 192, 3.0e12}};
  return plan_tiles(M, N, K, may_split, cand, 2);
}

// weight gradient of a convolution, [M = output channels][N = 9 input channels] reduced over the pixels:
// few output channels take the tiles that are narrow in M (rates measured on the VGG16 shapes)
Plan plan_conv_dw(int M, int N, int K) {
  static const TileRate cand[4] = {{T_PP_256x256, 256, 256, 3.3e12}, {T_PP_256x192, 256, 192, 3.0e12},
                                   {T_PP_128x256, 128, 256, 2.4e12}, {T_PP_64x512, 64, 512, 2.0e12}};
  return plan_tiles(M, N, K, true, cand, 4);
}

// implicit convolution (forward, gradient passing): the same cost model over the four tiles, with the rates a
// CU sustains on the VGG16 layer shapes (the shifted rows of the nine taps hit in the L2, so the wide tiles
// run faster here than on a stored matrix)
int choose_conv_tile(const GemmDesc& d) {
  if (d.tile == T_PP_256x256 || d.tile == T_PP_256x192 || d.tile == T_PP_256x128 || d.tile == T_PP_512x64) return d.tile;
  static const TileRate cand[4] = {{T_PP_256x256, 256, 256, 4.5e12}, {T_PP_256x192, 256, 192, 4.0e12},
                                   {T_PP_256x128, 256, 128, 3.3e12}, {T_PP_512x64, 512, 64, 2.6e12}};
  return plan_tiles(d.M, d.N, d.K, false, cand, 4).tile;
}

int choose_tile(const GemmDesc& d, int k_per_block) {
  const bool dma_ok = (d.K % gemm::DBK) == 0 && (k_per_block % gemm::DBK) == 0;
  const bool pp_ok = (d.K % gemm::PBK) == 0 && (k_per_block % gemm::PBK) == 0;
  if (d.tile == T_PP_256x256 || d.tile == T_PP_256x192) return pp_ok ? d.tile : (dma_ok ? T_DMA_256x256 : T_128x128);
  if (d.tile == T_PP_256x128 || d.tile == T_PP_512x64 || d.tile == T_PP_128x256 || d.tile == T_PP_64x512) return pp_ok ? d.tile : T_128x128;
  if (d.tile == T_DMA_256x256 || d.tile == T_DMA_256x128) return dma_ok ? d.tile : T_128x128;
  if (d.tile != T_AUTO) return d.tile;
  if (d.N <= 64 || d.K <= 64) return T_128x64;   // one K slice: a stream over the rows, more workgroups in flight win
  // large problems: a two-group tile where K comes in slices of 64 (4-20 % faster than either
  // direct-to-LDS tile on every forward, passing and gradient product of the ViT shapes), else
  // the direct-to-LDS tile with slices of 32
  // too few 256x256 tiles to fill the 256 CUs: products of more than 8 GFLOP (a ViT-L layer at batch 32) take the
  // 256x128 two-group tile (13 % faster there than 256x192), smaller ones (late ResNet / MobileNet stages: a few
  // thousand rows) the register-staged tiles, several workgroups per CU, which are up to twice as fast there
  const long long big_tiles = (long long)((d.M + 255) / 256) * ((d.N + 255) / 256) * d.z_outer * d.z_inner;
  if (d.M >= 512 && d.N >= 256 && big_tiles < 128 && d.mode != EPI_GELU_FWD && d.mode != EPI_GELU_BWD && d.mode != EPI_GELU_ONLY) {
    if (pp_ok && k_per_block >= 4 * gemm::PBK && 2.0 * d.M * d.N * (double)k_per_block >= 8e9 && d.z_outer * d.z_inner == 1)
      return T_PP_256x128;
    return (long long)((d.M + 127) / 128) * ((d.N + 127) / 128) >= 256 ? T_128x128 : T_128x64;
  }
  if (d.M >= 512 && d.N >= 256) {
    // (the GELU forward epilogues, 20 instructions per element, cost a 256x256 tile as much as half its main loop;
    // two 256x128 direct-to-LDS workgroups per CU that overlap one's epilogue with the other's MFMAs run no
    // faster than the resident two-group tile: 101.7 against 101.3 us for the ViT-B fc1 product)
    if (pp_ok && k_per_block >= 4 * gemm::PBK) return plan_large(d.M, d.N, k_per_block, false).tile;
    if (dma_ok && k_per_block >= 4 * gemm::DBK) return d.N >= 2560 ? T_DMA_256x128 : T_DMA_256x256;
  }
  return T_128x128;
}

}  // namespace

size_t gemm_bf16_partial_elems(int M, int N, int split_k) { return split_k > 1 ? (size_t)M * N * split_k : 0; }

void gemm_bf16_plan_conv(int M, int N, int K, int* tile, int* split_k) {
  static const TileRate cand[4] = {{T_PP_256x256, 256, 256, 4.5e12}, {T_PP_256x192, 256, 192, 4.0e12},
                                   {T_PP_256x128, 256, 128, 3.3e12}, {T_PP_512x64, 512, 64, 2.6e12}};
  const Plan pl = plan_tiles(M, N, K, (N & 3) == 0, cand, 4);
  *tile = pl.tile;
  *split_k = pl.split;
}

void gemm_bf16_plan_conv_dw(int M, int N, int K, int* tile, int* split_k) {
  const Plan pl = plan_conv_dw(M, N, K);
  *tile = pl.tile;
  *split_k = pl.split;
}

void gemm_bf16_plan_split(int M, int N, int K, int* tile, int* split_k) {
  *tile = T_AUTO;
  *split_k = 1;
  if (M >= 256 && N >= 256 && (K % gemm::PBK) == 0 && K >= 4 * gemm::PBK) {
    const Plan pl = plan_large(M, N, K, true);
    *tile = pl.tile;
    *split_k = pl.split;
  } else if (M >= 256 && N >= 256 && (K % gemm::DBK) == 0 && K >= 128 * gemm::DBK) {
    // a long reduction whose length is a multiple of 32 but not of 64 (ViT-L at batch 32: 6 304 rows) takes the
    // direct-to-LDS tiles; unsplit, its 16-64 tiles of 256x256 would leave most CUs idle.  Measured on those shapes:
    // about 256 units in all, at most 8 chunks (4096x1024: 98 -> 71 us with 4 chunks; 1024x1024: 70 -> 31 us with 8).
    // Shorter reductions (1 568 rows: the last ResNet-50 stage) are better off with the rule below.
    const int tiles = ((M + 255) / 256) * ((N + 255) / 256);
    *split_k = std::max(1, std::min(8, 256 / tiles));
    *tile = tiles >= 32 ? T_DMA_256x256 : T_DMA_256x128;
  } else {   // small outputs: as many chunks as keep the CUs busy, each at least 4 slices
    const int tiles = ((M + 127) / 128) * ((N + 127) / 128);
    const int slices = (K + gemm::SBK - 1) / gemm::SBK;
    *split_k = std::max(1, std::min(std::min(256 / std::max(tiles, 1), std::max(1, slices / 4)), 256));
  }
}

hipError_t gemm_bf16(const GemmDesc& d, hipStream_t s, int* launches) {
  if (launches) *launches = 0;
  const bool c_optional = d.mode == EPI_AFFINE_RELU || d.mode == EPI_AFFINE_ADD_RELU;
  if (!d.A || !d.B || (!d.C && !c_optional) || d.M <= 0 || d.N <= 0 || d.K <= 0) return hipErrorInvalidValue;
  if (!aligned(d.A, 16) || !aligned(d.B, 16) || !aligned(d.C, 16) || (d.lda & 7) || (d.ldb & 7)) return hipErrorInvalidValue;
  if ((d.sAo | d.sAi | d.sBo | d.sBi) & 7) return hipErrorInvalidValue;
  if ((d.sCo | d.sCi) & 3) return hipErrorInvalidValue;
  if (d.z_outer < 1 || d.z_inner < 1) return hipErrorInvalidValue;
  // rows must be long enough for the 16-byte loads of the contiguous index
  if (!d.a_t && d.conv_c <= 0 && d.lda < ((d.K + 7) & ~7)) return hipErrorInvalidValue;
  if (!d.b_t && d.ldb < ((d.K + 7) & ~7)) return hipErrorInvalidValue;
  if (d.a_t && d.lda < ((d.M + 7) & ~7)) return hipErrorInvalidValue;
  if (d.b_t && !(d.conv_c > 0 && d.a_t) && d.ldb < ((d.N + 7) & ~7)) return hipErrorInvalidValue;
  if (d.bias && !aligned(d.bias, 8)) return hipErrorInvalidValue;
  const bool conv = d.conv_c > 0;
  const bool conv_dw = conv && d.a_t && d.b_t;
  const int taps2 = d.conv_taps * d.conv_taps;
  int conv_ho = 0, conv_wo = 0;
  const bool stem = conv && d.conv_taps == 7;
  if (stem) {   // padded image [.., conv_h, conv_w, 4]; the window is widened to 8 x 8
    if (d.conv_c != 4 || d.conv_stride != 2 || d.conv_h < 8 || d.conv_w < 8 || (d.conv_w & 1) || d.conv_h > 4095 || d.conv_w > 4095 ||
        d.z_outer != 1 || d.z_inner != 1)
      return hipErrorInvalidValue;
    conv_ho = (d.conv_h - 8) / 2 + 1;
    conv_wo = (d.conv_w - 8) / 2 + 1;
    if (conv_dw ? (d.N != 256 || (d.K % (conv_ho * conv_wo)) || (d.K % gemm::PBK) || !d.c_f32)
                : (d.K != 256 || (d.M % (conv_ho * conv_wo)) || d.a_t || d.b_t || d.split_k > 1 || d.mode != EPI_PLAIN || !d.c_f32 ||
                   d.residual))
      return hipErrorInvalidValue;
  } else if (conv) {
    if ((d.conv_taps != 1 && d.conv_taps != 3) || (d.conv_stride != 1 && d.conv_stride != 2) || d.conv_h < 1 || d.conv_w < 1 ||
        d.conv_h > 4095 || d.conv_w > 4095)
      return hipErrorInvalidValue;
    conv_ho = (d.conv_h - 1) / d.conv_stride + 1;
    conv_wo = (d.conv_w - 1) / d.conv_stride + 1;
  }
  if (stem) {
  } else if (conv_dw) {   // B is the activation; the reduction runs over the output pixels
    if ((d.conv_c & 7) || d.N != taps2 * d.conv_c || (d.K % (conv_ho * conv_wo)) || (d.K % gemm::PBK) || d.z_outer != 1 ||
        d.z_inner != 1 || !d.c_f32)
      return hipErrorInvalidValue;
  } else if (conv) {
    if ((d.conv_c % gemm::PBK) || d.K != taps2 * d.conv_c || (d.M % (conv_ho * conv_wo)) || d.a_t || d.b_t || d.z_outer != 1 ||
        d.z_inner != 1)
      return hipErrorInvalidValue;
    // a split reduction finishes in a second kernel that applies the epilogue: outputs without padding
    if (d.split_k > 1 && (!d.partials || !aligned(d.partials, 16) || d.ldc != d.N || (d.N & 3) || d.c_f32 || d.residual ||
                          d.alpha != 1.f || d.mode == EPI_AFFINE_ADD_RELU || d.mode == EPI_GELU_FWD || d.mode == EPI_GELU_BWD ||
                          d.mode == EPI_GELU_ONLY || (d.mode == EPI_PLAIN && d.bias)))
      return hipErrorInvalidValue;
    if (d.split_k > 1 && ((d.mode == EPI_AFFINE_RELU && (!d.C2 || !d.gain || !d.bias || !aligned(d.C2, 8) || !aligned(d.gain, 8))) ||
                          (d.mode == EPI_RELU_MASK && (!d.U || !aligned(d.U, 8))) || (d.mode == EPI_BIAS_RELU && !d.bias)))
      return hipErrorInvalidValue;
  }
  const bool conv_split = conv && !conv_dw && d.split_k > 1;
  if (d.residual && (d.ldr < d.N || (d.ldr & 3) || !aligned(d.residual, 16))) return hipErrorInvalidValue;

  gemm::Params p;
  p.A = d.A; p.B = d.B; p.M = d.M; p.N = d.N; p.K = d.K; p.lda = d.lda; p.ldb = d.ldb;
  p.z_inner = d.z_inner;
  p.sAo = d.sAo; p.sAi = d.sAi; p.sBo = d.sBo; p.sBi = d.sBi; p.sCo = d.sCo; p.sCi = d.sCi;
  p.split_k = 1; p.k_chunk = 0;
  p.alpha = d.alpha; p.bias = d.bias; p.gain = d.gain; p.gain2 = d.gain2; p.bias2 = d.bias2; p.residual = d.residual; p.ldr = d.ldr;
  p.C = d.C; p.ldc = d.ldc; p.C2 = d.C2; p.U = d.U;
  p.cH = d.conv_h; p.cW = d.conv_w; p.cC = d.conv_c;
  p.cT = stem ? 8 : d.conv_taps; p.cS = d.conv_stride; p.cHo = conv_ho; p.cWo = conv_wo;
  p.act_lo = d.act_lo; p.act_hi = d.act_hi; p.mask_hi = d.mask_hi;
  int zdim = d.z_outer * d.z_inner;
  int epi;
  int k_per_block = d.K;
  if (d.split_k > 1) {
    if (!conv_split && (zdim != 1 || !d.partials || !d.c_f32 || d.bias || d.residual || d.mode != EPI_PLAIN || d.alpha != 1.f ||
                        d.ldc != d.N || (d.N & 3) || !aligned(d.partials, 16)))
      return hipErrorInvalidValue;
    const int slices = (d.K + gemm::SBK - 1) / gemm::SBK;
    const int per = (slices + d.split_k - 1) / d.split_k;
    p.k_chunk = per * gemm::SBK;
    p.split_k = (slices + per - 1) / per;  // no empty chunks
    k_per_block = p.k_chunk;
  }
  if (p.split_k > 1) {
    p.C = d.partials;
    zdim = p.split_k;
    epi = gemm::E_PARTIAL;
  } else {
    p.split_k = 1;
    if (d.ldc < d.N || (d.ldc & 3)) return hipErrorInvalidValue;
    if (d.mode == EPI_GELU_FWD) {
      if (!d.C2 || d.c_f32 || d.residual || !aligned(d.C2, 8)) return hipErrorInvalidValue;
      epi = gemm::E_GELU_FWD;
    } else if (d.mode == EPI_BIAS_RELU) {
      if (d.c_f32 || d.residual || d.a_t || d.b_t) return hipErrorInvalidValue;
      epi = gemm::E_BIAS_RELU;
    } else if (d.mode == EPI_GELU_ONLY) {
      if (d.c_f32 || d.residual || d.a_t || d.b_t) return hipErrorInvalidValue;
      epi = gemm::E_GELU_ONLY;
    } else if (d.mode == EPI_AFFINE_RELU) {
      if (!d.C2 || !d.gain || !d.bias || d.c_f32 || d.residual || d.a_t || d.b_t || !aligned(d.C2, 8)) return hipErrorInvalidValue;
      epi = gemm::E_AFFINE;
    } else if (d.mode == EPI_AFFINE_ADD_RELU) {
      if (!d.C2 || !d.gain || !d.bias || !d.U || (d.gain2 && !d.bias2) || d.c_f32 || d.residual || d.a_t || d.b_t ||
          !aligned(d.C2, 8) || !aligned(d.U, 8))
        return hipErrorInvalidValue;
      epi = gemm::E_AFFINE_ADD;
    } else if (d.mode == EPI_RELU_MASK) {
      if (!d.U || d.c_f32 || d.residual || d.bias || !aligned(d.U, 8)) return hipErrorInvalidValue;
      epi = gemm::E_RELU_MASK;
    } else if (d.mode == EPI_GELU_BWD) {
      if (!d.U || d.c_f32 || d.residual || d.bias || !aligned(d.U, 8)) return hipErrorInvalidValue;
      epi = gemm::E_GELU_BWD;
    } else if (d.c_f32) {
      epi = d.residual ? gemm::E_F32_RES : gemm::E_F32;
    } else {
      if (d.residual) return hipErrorInvalidValue;
      epi = gemm::E_BF16;
    }
  }
  int BM, BN;
  gemm::LaunchFn fn;
  const bool conv_general = conv && !(d.conv_taps == 3 && d.conv_stride == 1);   // geometry as launch arguments
  bool resident = true;   // the two-group kernels keep one workgroup per CU that walks over the tiles
  if (conv_dw) {
    int tile = d.tile;
    if (tile != T_PP_256x256 && tile != T_PP_256x192 && tile != T_PP_128x256 && tile != T_PP_64x512)
      tile = plan_conv_dw(d.M, d.N, k_per_block).tile;
    switch (tile) {
      case T_PP_64x512: BM = 64; BN = 512; fn = gemm::pp_convdw_64x512(epi, conv_general); break;
      case T_PP_128x256: BM = 128; BN = 256; fn = gemm::pp_convdw_128x256(epi, conv_general); break;
      case T_PP_256x192: BM = 256; BN = 192; fn = gemm::pp_convdw_256x192(epi, conv_general); break;
      default: BM = 256; BN = 256; fn = gemm::pp_convdw_256x256(epi, conv_general); break;
    }
  } else if (stem) {   // few output channels, fp32 result
    BM = 512; BN = 64; fn = gemm::pp_conv_512x64(epi, conv_general);
  } else if (conv) {
    switch (choose_conv_tile(d)) {
      case T_PP_512x64: BM = 512; BN = 64; fn = gemm::pp_conv_512x64(epi, conv_general); break;
      case T_PP_256x128: BM = 256; BN = 128; fn = gemm::pp_conv_256x128(epi, conv_general); break;
      case T_PP_256x192: BM = 256; BN = 192; fn = gemm::pp_conv_256x192(epi, conv_general); break;
      default: BM = 256; BN = 256; fn = gemm::pp_conv_256x256(epi, conv_general); break;
    }
  } else
  switch (choose_tile(d, k_per_block)) {
    case T_PP_64x512: BM = 64; BN = 512; fn = gemm::pp_64x512(d.a_t, d.b_t, epi); break;
    case T_PP_128x256: BM = 128; BN = 256; fn = gemm::pp_128x256(d.a_t, d.b_t, epi); break;
    case T_PP_512x64: BM = 512; BN = 64; fn = gemm::pp_512x64(d.a_t, d.b_t, epi); break;
    case T_PP_256x128: BM = 256; BN = 128; fn = gemm::pp_256x128(d.a_t, d.b_t, epi); break;
    case T_128x64: BM = 128; BN = 64; fn = gemm::staged_128x64(d.a_t, d.b_t, epi); resident = false; break;
    case T_DMA_256x256: BM = 256; BN = 256; fn = gemm::dma_256x256(d.a_t, d.b_t, epi); resident = false; break;
    case T_DMA_256x128: BM = 256; BN = 128; fn = gemm::dma_256x128(d.a_t, d.b_t, epi); resident = false; break;
    case T_PP_256x192: BM = 256; BN = 192; fn = gemm::pp_256x192(d.a_t, d.b_t, epi); break;
    case T_PP_256x256: BM = 256; BN = 256; fn = gemm::pp_256x256(d.a_t, d.b_t, epi); break;
    default: BM = 128; BN = 128; fn = gemm::staged_128x128(d.a_t, d.b_t, epi); resident = false; break;
  }
  if (!fn) return hipErrorInvalidValue;  // this (layout, epilogue) pair is not part of the training step
  const int tiles = ((d.M + BM - 1) / BM) * ((d.N + BN - 1) / BN);
  if ((long long)tiles * zdim >= (1ll << 23)) return hipErrorInvalidValue;   // (the resident kernels' unit arithmetic)
  p.units = tiles * zdim;
  // resident kernels: every workgroup takes the same number of units (600 tiles run as 200 workgroups of 3 rather than
  // 256 of 2 or 3: the launch takes 3 tile times either way, and the CUs left idle lower the load the others run under)
  int resident_grid = p.units;
  const int cus = compute_units();
  if (resident_grid > cus) {
    const int rounds = (p.units + cus - 1) / cus;
    resident_grid = std::min(cus, ((p.units + rounds - 1) / rounds + 7) & ~7);
  }
  hipError_t e = resident ? fn(p, dim3(resident_grid, 1, 1), s) : fn(p, dim3(tiles, 1, zdim), s);
  if (e != hipSuccess) return e;
  if (launches) *launches = 1;
  if (p.split_k > 1 && conv_split) {
    ReduceEpi r;
    r.part = (const float4*)d.partials; r.n4 = (size_t)d.M * d.N / 4; r.splits = p.split_k; r.N = d.N;
    r.mode = d.mode == EPI_BIAS_RELU ? 1 : d.mode == EPI_RELU_MASK ? 2 : d.mode == EPI_AFFINE_RELU ? 3 : 0;
    r.bias = d.bias; r.gain = d.gain; r.U = d.U;
    r.out = d.mode == EPI_AFFINE_RELU ? d.C2 : (bf16*)d.C;
    r.zout = d.mode == EPI_AFFINE_RELU ? (bf16*)d.C : nullptr;
    r.lo = d.act_lo; r.hi = d.act_hi; r.mask_hi = d.mask_hi;
    hipLaunchKernelGGL(splitk_reduce_epilogue_kernel, dim3((unsigned)((r.n4 + 255) / 256)), dim3(256), 0, s, r);
    e = hipGetLastError();
    if (launches) *launches = 2;
  } else if (p.split_k > 1) {
    const size_t n4 = (size_t)d.M * d.N / 4;
    if (p.split_k > 32)
      hipLaunchKernelGGL(splitk_reduce_wide_kernel, dim3((unsigned)((n4 + 15) / 16)), dim3(256), 0, s,
                         (const float4*)d.partials, (float4*)d.C, n4, p.split_k);
    else
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                         (const float4*)d.partials, (float4*)d.C, n4, p.split_k);
    e = hipGetLastError();
    if (launches) *launches = 2;
  }
  return e;
}

}  // namespace et
