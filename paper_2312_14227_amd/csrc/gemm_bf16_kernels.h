// bf16 MFMA GEMM kernels for gfx950: D[i][j] = alpha * sum_k A(i,k) B(j,k), fp32 accumulation.
//
// The dense contractions of the training step (Section 5.1: forward product, error-gradient
// passing T1, weight gradient T3) all reduce to this form with either operand optionally stored
// with the reduction index as the slow one:
//   forward   Y  = X  W^T : A = X  [M][K],  B = W [N][K]                          (a_t = 0, b_t = 0)
//   passing   dX = dY W   : A = dY [M][N'], B = W [N'][K'] read as B(j=k', k=n')  (b_t = 1)
//   gradient  dW = dY^T X : A = dY [M'][N'] read as A(i=n', k=m), B = X likewise  (a_t = b_t = 1)
//
// Common design: one workgroup computes a BM x BN tile with v_mfma_f32_32x32x16_bf16; 64-lane
// waves in a WGM x WGN grid each own a (BM/WGM) x (BN/WGN) sub-tile.
//   - operand with contiguous reduction index: the LDS tile keeps rows of k values, 16-byte chunks
//     XOR-swizzled with the row so that the ds_read_b128 of 16 consecutive rows cover all 64 banks
//     (measured: 237 B/clk/CU against 124 with an 8-row swizzle); a lane reads its 8 consecutive
//     k values directly;
//   - operand with the reduction index slow ("transposed"): LDS keeps the global layout
//     [k-rows][tile rows] and the lanes fetch their 2 x 4 k values with ds_read_b64_tr_b16, the
//     LDS transpose read of gfx950: in every group of 16 lanes, lane 4c+a supplies the address of
//     4 consecutive elements of k-row c, and lane i receives element i of k-rows 0..3.
// Three main loops share this:
//   gemm_staged_kernel: K slices of 64 through two LDS buffers, the global loads of slice t+1 are
//     issued into registers before the MFMAs of slice t (small tiles, several workgroups per CU;
//     any K, with a predicated last slice);
//   gemm_dma_kernel: K slices of 32 loaded with global_load_lds_dwordx4 straight into a ring of
//     LDS stages, several slices in flight (large tiles; K a multiple of 32);
//   gemm_pp_kernel: K slices of 64 through registers into two LDS stages, the eight waves in two
//     groups that alternate between MFMAs and memory work (256x256 tile; K a multiple of 64).
// Rows beyond the matrix edge are clamped to valid addresses (their products are never stored).
// Epilogue: every wave passes its accumulators through a private LDS area, 32 rows at a time, so
// that each lane ends up with 4 consecutive columns of one row: bias, residual, GELU and the
// stores then work on 8- and 16-byte vectors and whole 128-byte lines.
// Workgroup ids are remapped so that consecutive tiles run on the same XCD (ids are dealt
// round-robin over the 8 XCDs, each with its own L2), in groups of 8 tile rows.
#pragma once
#include <type_traits>

#include "kernels.h"

namespace et {
namespace gemm {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int NUM_XCD = 8;

// compile-time epilogues
enum Epi : int {
  E_F32 = 0,        // C fp32 = alpha*v + bias
  E_F32_RES = 1,    // C fp32 = alpha*v + bias + residual
  E_BF16 = 2,       // C bf16 = alpha*v + bias
  E_GELU_FWD = 3,   // with u = v + bias: C bf16 = gelu'(u) (kept for the backward pass), C2 bf16 = gelu(u)
  E_GELU_BWD = 4,   // C bf16 = v * U, U = the stored gelu'(u)
  E_PARTIAL = 5,    // split-K partial: C fp32 [z][M][N] = v
  E_AFFINE = 6,     // C bf16 = z = v, C2 bf16 = max(z * gain[j] + bias[j], 0) with z as rounded to bf16
  E_BIAS_RELU = 9,  // C bf16 = max(alpha*v + bias, 0)
  E_RELU_MASK = 10, // C bf16 = U > 0 ? v : 0 (gradient through a ReLU whose output U was stored)
  E_GELU_ONLY = 8,  // C bf16 = gelu(v + bias) (forward of a block whose backward will not run)
  E_AFFINE_ADD = 7, // as E_AFFINE with a second branch inside the ReLU: + U * gain2[j] + bias2[j] (or + U if gain2 is null)
};

struct Params {
  const bf16* A;
  const bf16* B;
  int M, N, K;
  int lda, ldb;
  int z_inner;
  long long sAo, sAi, sBo, sBi, sCo, sCi;
  int split_k, k_chunk;  // split_k > 1: chunk z of the reduction is [z*k_chunk, (z+1)*k_chunk)
  float alpha;
  const bf16* bias;
  const bf16* gain;      // E_AFFINE, E_AFFINE_ADD: per output column
  const bf16* gain2;     // E_AFFINE_ADD (nullable), with bias2
  const bf16* bias2;
  const float* residual;
  int ldr;
  void* C;
  int ldc;
  bf16* C2;
  const bf16* U;
  float act_lo, act_hi;  // E_AFFINE, E_AFFINE_ADD: the activation is a clamp to [act_lo, act_hi] (0, +inf: ReLU; 0, 6: ReLU6; -inf, +inf: none)
  float mask_hi;         // E_RELU_MASK passes where 0 < U < mask_hi
  int cH, cW, cC;        // implicit 3x3 convolution (gemm_pp_kernel<.., CONV>): input height, width, channels
  int no_store;          // tuning aids: 1 run the main loop, store nothing; 2 also issue no loads; 4 all tiles load the same panels
};

// GELU (exact erf form) and its derivative from one exponential: with x = u / sqrt(2),
//   erf(|x|) = 1 - (a1 t + .. + a5 t^5) exp(-x^2),  t = 1 / (1 + p |x|)   (Abramowitz-Stegun 7.1.26,
//   absolute error < 1.5e-7, far below the bf16 rounding of the results)
//   gelu(u) = u Phi(u),  gelu'(u) = Phi(u) + u exp(-u^2/2) / sqrt(2 pi),  Phi(u) = (1 + erf(x)) / 2
// (t from the hardware reciprocal, 1 ulp: a correctly rounded division costs eleven instructions here)
__device__ __forceinline__ void gelu_both(float u, float& g, float& dg) {
  // constants folded: p / sqrt(2) for t, -log2(e) / 2 for exp(-x^2) = 2^(-u^2 log2(e) / 2)
  const float t = __builtin_amdgcn_rcpf(fmaf(0.23164189f, fabsf(u), 1.f));
  const float e = __builtin_amdgcn_exp2f(u * u * -0.72134752f);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float phi = fmaf(0.5f, copysignf(fmaf(-poly, e, 1.f), u), 0.5f);
  g = u * phi;
  dg = fmaf(u * e, 0.39894228040143268f, phi);
}

__device__ __forceinline__ float gelu_only(float u) {
  const float t = __builtin_amdgcn_rcpf(fmaf(0.23164189f, fabsf(u), 1.f));
  const float e = __builtin_amdgcn_exp2f(u * u * -0.72134752f);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  return u * fmaf(0.5f, copysignf(fmaf(-poly, e, 1.f), u), 0.5f);
}

__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

// tile coordinates of this workgroup and its index z along the grid's third dimension (batch or reduction chunk).
// Workgroups are dealt to the 8 XCDs (one L2 each) round-robin in launch order, x fastest; the mapping below undoes
// that so that an XCD works on consecutive tiles, which share operand panels.  In a split reduction only the tiles
// of ONE chunk share anything, so there the unit of the dealing is (chunk, tile): an XCD gets a run of consecutive
// tiles of one chunk (then of the next) instead of the same few tiles of every chunk.
template <int BM, int BN>
__device__ __forceinline__ void tile_coords(const Params& g, int& m0, int& n0, int& z) {
  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (g.M + BM - 1) / BM;
  const int nt = tiles_m * tiles_n;     // = gridDim.x
  int t;
  if (g.split_k > 1) {
    const int total = nt * g.split_k;   // gridDim.z = split_k
    const int w = blockIdx.z * nt + blockIdx.x;
    const int xcd = w % NUM_XCD, idx = w / NUM_XCD;
    const int per = total / NUM_XCD, rem = total % NUM_XCD;
    const int u = xcd * per + (xcd < rem ? xcd : rem) + idx;
    z = u / nt;
    t = u % nt;
  } else {
    const int w = blockIdx.x;
    const int xcd = w % NUM_XCD, idx = w / NUM_XCD;
    const int per = nt / NUM_XCD, rem = nt % NUM_XCD;
    t = xcd * per + (xcd < rem ? xcd : rem) + idx;  // undo the round-robin XCD dealing
    z = blockIdx.z;
  }
  constexpr int GROUP = 8;                                   // 8 tile rows, walked column by column
  const int gsz = GROUP * tiles_n;
  const int grp = t / gsz, in = t % gsz;
  const int first = grp * GROUP;
  const int gm = min(tiles_m - first, GROUP);
  m0 = (first + in % gm) * BM;
  n0 = (in / gm) * BN;
}

// batch / split-K bookkeeping
__device__ __forceinline__ void batch_offsets(const Params& g, int z, const bf16*& A, const bf16*& B, long long& c_off,
                                              int& k_begin, int& k_end) {
  A = g.A;
  B = g.B;
  k_begin = 0;
  k_end = g.K;
  if (g.split_k > 1) {
    k_begin = z * g.k_chunk;
    k_end = min(g.K, k_begin + g.k_chunk);
    c_off = (long long)z * g.M * g.N;
  } else {
    const int zo = z / g.z_inner, zi = z % g.z_inner;
    A += zo * g.sAo + zi * g.sAi;
    B += zo * g.sBo + zi * g.sBi;
    c_off = zo * g.sCo + zi * g.sCi;
  }
}

// -------------------------------------------------------------------------------------------------
// Epilogue of one wave.  acc[mi][ni][r] holds element (mi*32 + (r/4)*8 + (lane/32)*4 + r%4,
// ni*32 + lane%32) of the wave's TM x TN sub-tile whose top-left corner is (row0, col0).
// `stage` is this wave's private LDS area of 32 * TN floats.
// -------------------------------------------------------------------------------------------------
template <int EPI, int MI, int NI>
__device__ __forceinline__ void wave_epilogue(const Params& g, f32x16 (&acc)[MI][NI], float* stage, int row0, int col0,
                                              long long c_off, int lane) {
  constexpr int TN = NI * 32;
  constexpr int CPL = TN / 4;    // lanes per row when reading back 4 columns each
  constexpr int RPI = 64 / CPL;  // rows covered by one wave-wide read
  const int l32 = lane & 31, khalf = lane >> 5;
  const int c4 = (lane % CPL) * 4, rsub = lane / CPL;
  const int col = col0 + c4;
  // (when 64 is not a multiple of CPL the last lanes of the wave have no row of their own)
  const bool col_any = col < g.N && rsub < RPI, col_full = col + 3 < g.N;
  const int ld = EPI == E_PARTIAL ? g.N : g.ldc;
  float bias[4] = {0.f, 0.f, 0.f, 0.f};
  float gain[4] = {1.f, 1.f, 1.f, 1.f};
  float gain2[4] = {1.f, 1.f, 1.f, 1.f}, bias2[4] = {0.f, 0.f, 0.f, 0.f};
  if ((EPI == E_AFFINE || EPI == E_AFFINE_ADD) && col_any) {
    for (int j = 0; j < 4 && col + j < g.N; j++) gain[j] = (float)g.gain[col + j];
    if (EPI == E_AFFINE_ADD && g.gain2)
      for (int j = 0; j < 4 && col + j < g.N; j++) {
        gain2[j] = (float)g.gain2[col + j];
        bias2[j] = (float)g.bias2[col + j];
      }
  }
  if (EPI != E_PARTIAL && EPI != E_GELU_BWD && EPI != E_RELU_MASK && g.bias && col_any) {
    if (col_full) {
      const bf16x4 b = *(const bf16x4*)(g.bias + col);
#pragma unroll
      for (int j = 0; j < 4; j++) bias[j] = (float)b[j];
    } else {
      for (int j = 0; j < 4 && col + j < g.N; j++) bias[j] = (float)g.bias[col + j];
    }
  }
  constexpr bool HAS_RES = EPI == E_F32_RES;
  constexpr bool HAS_U = EPI == E_GELU_BWD || EPI == E_AFFINE_ADD || EPI == E_RELU_MASK;
#pragma unroll
  for (int mi = 0; mi < MI; mi++) {
    // the second operands of this 32-row block are requested before the accumulators go through
    // LDS, all at once: one memory latency per block instead of one per row group
    float4 pre_res[HAS_RES ? 32 / RPI : 1];
    bf16x4 pre_u[HAS_U ? 32 / RPI : 1];
    if (HAS_RES || HAS_U) {
#pragma unroll
      for (int it = 0; it < 32 / RPI; it++) {
        const int row = row0 + mi * 32 + min(it * RPI + rsub, 31);
        if (row < g.M && col_any && col_full) {
          if (HAS_RES) pre_res[it] = *(const float4*)(g.residual + (long long)row * g.ldr + col);
          if (HAS_U) pre_u[it] = *(const bf16x4*)(g.U + c_off + (long long)row * ld + col);
        }
      }
    }
#pragma unroll
    for (int ni = 0; ni < NI; ni++)
#pragma unroll
      for (int r = 0; r < 16; r++) stage[((r >> 2) * 8 + khalf * 4 + (r & 3)) * TN + ni * 32 + l32] = acc[mi][ni][r];
    // the same wave reads back: LDS operations of one wave complete in order
#pragma unroll
    for (int it = 0; it < 32 / RPI; it++) {
      const int rr = min(it * RPI + rsub, 31);
      const float4 raw = *(const float4*)(stage + rr * TN + c4);
      const int row = row0 + mi * 32 + rr;
      if (row >= g.M || !col_any) continue;
      float v[4] = {raw.x, raw.y, raw.z, raw.w};
      const long long ci = c_off + (long long)row * ld + col;
      if (EPI == E_AFFINE || EPI == E_AFFINE_ADD) {
#pragma unroll
        for (int j = 0; j < 4; j++) v[j] *= g.alpha;
      } else if (EPI != E_PARTIAL) {
#pragma unroll
        for (int j = 0; j < 4; j++) v[j] = v[j] * g.alpha + bias[j];
      }
      if (col_full) {
        if (EPI == E_F32_RES) {
          const float4 rs = pre_res[HAS_RES ? it : 0];
          v[0] += rs.x; v[1] += rs.y; v[2] += rs.z; v[3] += rs.w;
        }
        if (EPI == E_GELU_BWD) {
          const bf16x4 u = pre_u[HAS_U ? it : 0];
#pragma unroll
          for (int j = 0; j < 4; j++) v[j] *= (float)u[j];
        }
        if (EPI == E_RELU_MASK) {
          const bf16x4 u = pre_u[HAS_U ? it : 0];
#pragma unroll
          for (int j = 0; j < 4; j++) v[j] = ((float)u[j] > 0.f && (float)u[j] < g.mask_hi) ? v[j] : 0.f;
        }
        if (EPI == E_F32 || EPI == E_F32_RES || EPI == E_PARTIAL) {
          *(float4*)((float*)g.C + ci) = make_float4(v[0], v[1], v[2], v[3]);
        } else if (EPI == E_GELU_FWD) {
          bf16x4 o, o2;
#pragma unroll
          for (int j = 0; j < 4; j++) {
            float gv, dgv;
            gelu_both(v[j], gv, dgv);
            o[j] = (bf16)dgv;
            o2[j] = (bf16)gv;
          }
          *(bf16x4*)((bf16*)g.C + ci) = o;
          *(bf16x4*)(g.C2 + ci) = o2;
        } else if (EPI == E_GELU_ONLY) {
          bf16x4 o;
#pragma unroll
          for (int j = 0; j < 4; j++) o[j] = (bf16)gelu_only(v[j]);
          *(bf16x4*)((bf16*)g.C + ci) = o;
        } else if (EPI == E_BIAS_RELU) {
          bf16x4 o;
#pragma unroll
          for (int j = 0; j < 4; j++) o[j] = (bf16)fmaxf(v[j], 0.f);
          *(bf16x4*)((bf16*)g.C + ci) = o;
        } else if (EPI == E_AFFINE) {
          bf16x4 o, o2;
#pragma unroll
          for (int j = 0; j < 4; j++) {
            o[j] = (bf16)v[j];
            o2[j] = (bf16)fminf(fmaxf((float)o[j] * gain[j] + bias[j], g.act_lo), g.act_hi);
          }
          if (g.C) *(bf16x4*)((bf16*)g.C + ci) = o;   // z is kept only if the gain's gradient will be computed
          *(bf16x4*)(g.C2 + ci) = o2;
        } else if (EPI == E_AFFINE_ADD) {
          const bf16x4 u = pre_u[HAS_U ? it : 0];
          bf16x4 o, o2;
#pragma unroll
          for (int j = 0; j < 4; j++) {
            o[j] = (bf16)v[j];
            o2[j] = (bf16)fminf(fmaxf(((float)o[j] * gain[j] + bias[j]) + ((float)u[j] * gain2[j] + bias2[j]), g.act_lo), g.act_hi);
          }
          if (g.C) *(bf16x4*)((bf16*)g.C + ci) = o;
          *(bf16x4*)(g.C2 + ci) = o2;
        } else {
          bf16x4 o;
#pragma unroll
          for (int j = 0; j < 4; j++) o[j] = (bf16)v[j];
          *(bf16x4*)((bf16*)g.C + ci) = o;
        }
      } else {  // ragged right edge: element by element
        for (int j = 0; j < 4 && col + j < g.N; j++) {
          float x = v[j];
          if (EPI == E_GELU_ONLY) {
            ((bf16*)g.C)[ci + j] = (bf16)gelu_only(x);
            continue;
          }
          if (EPI == E_BIAS_RELU) {
            ((bf16*)g.C)[ci + j] = (bf16)fmaxf(x, 0.f);
            continue;
          }
          if (EPI == E_F32_RES) x += g.residual[(long long)row * g.ldr + col + j];
          if (EPI == E_GELU_BWD) x *= (float)g.U[ci + j];
          if (EPI == E_RELU_MASK) x = ((float)g.U[ci + j] > 0.f && (float)g.U[ci + j] < g.mask_hi) ? x : 0.f;
          if (EPI == E_F32 || EPI == E_F32_RES || EPI == E_PARTIAL) {
            ((float*)g.C)[ci + j] = x;
          } else if (EPI == E_GELU_FWD) {
            float gv, dgv;
            gelu_both(x, gv, dgv);
            ((bf16*)g.C)[ci + j] = (bf16)dgv;
            g.C2[ci + j] = (bf16)gv;
          } else if (EPI == E_AFFINE) {
            const bf16 z = (bf16)x;
            if (g.C) ((bf16*)g.C)[ci + j] = z;
            g.C2[ci + j] = (bf16)fminf(fmaxf((float)z * gain[j] + bias[j], g.act_lo), g.act_hi);
          } else if (EPI == E_AFFINE_ADD) {
            const bf16 z = (bf16)x;
            if (g.C) ((bf16*)g.C)[ci + j] = z;
            g.C2[ci + j] = (bf16)fminf(fmaxf(((float)z * gain[j] + bias[j]) + ((float)g.U[ci + j] * gain2[j] + bias2[j]), g.act_lo), g.act_hi);
          } else {
            ((bf16*)g.C)[ci + j] = (bf16)x;
          }
        }
      }
    }
  }
}

// =================================================================================================
// register-staged kernel: K slices of 64, two LDS buffers
// =================================================================================================
constexpr int SBK = 64;

template <int ROWS, bool T>
struct StagedLds {
  static constexpr int PITCH = T ? (ROWS * 2 + 32) : (SBK * 2);   // transposed: k-rows padded by 32 B
  static constexpr int BYTES = T ? (SBK * PITCH) : (ROWS * PITCH);
};

template <int BM, int BN, int WGM, int WGN, bool AT, bool BT, int EPI>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_staged_kernel(Params g) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int TM = BM / WGM, TN = BN / WGN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int A_VECS = BM * SBK / 8 / NT, B_VECS = BN * SBK / 8 / NT;
  static_assert(A_VECS * NT * 8 == BM * SBK && B_VECS * NT * 8 == BN * SBK, "tile/threads mismatch");
  typedef StagedLds<BM, AT> LA;
  typedef StagedLds<BN, BT> LB;
  constexpr int STAGE = LA::BYTES + LB::BYTES;
  constexpr int EPI_BYTES = WGM * WGN * 32 * TN * 4;
  constexpr int SMEM = 2 * STAGE > EPI_BYTES ? 2 * STAGE : EPI_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WGN, wave_n = wave % WGN;
  int m0, n0, z;
  tile_coords<BM, BN>(g, m0, n0, z);
  const bf16* A;
  const bf16* B;
  long long c_off;
  int k_begin, k_end;
  batch_offsets(g, z, A, B, c_off, k_begin, k_end);
  const int k_end_pad = min((g.K + 7) & ~7, ((k_end + 7) & ~7));
  const int nk = (k_end - k_begin + SBK - 1) / SBK;

  // per-thread source pointers of its 16-byte pieces (slice 0); rows/columns clamped into the matrix
  const bf16* pa[A_VECS];
  const bf16* pb[B_VECS];
  int ka[A_VECS], kb[B_VECS];  // k index (within a slice) each piece starts at
#pragma unroll
  for (int p = 0; p < A_VECS; p++) {
    const int v = tid + p * NT;
    if (!AT) {
      const int row = v >> 3, kc = v & 7;
      ka[p] = kc * 8;
      pa[p] = A + (long long)min(m0 + row, g.M - 1) * g.lda + k_begin + kc * 8;
    } else {
      const int kr = v / (BM / 8), ic = v % (BM / 8);
      int gi = m0 + ic * 8;
      if (gi + 8 > ((g.M + 7) & ~7)) gi = 0;
      ka[p] = kr;
      pa[p] = A + (long long)(k_begin + kr) * g.lda + gi;
    }
  }
#pragma unroll
  for (int p = 0; p < B_VECS; p++) {
    const int v = tid + p * NT;
    if (!BT) {
      const int row = v >> 3, kc = v & 7;
      kb[p] = kc * 8;
      pb[p] = B + (long long)min(n0 + row, g.N - 1) * g.ldb + k_begin + kc * 8;
    } else {
      const int kr = v / (BN / 8), jc = v % (BN / 8);
      int gj = n0 + jc * 8;
      if (gj + 8 > ((g.N + 7) & ~7)) gj = 0;
      kb[p] = kr;
      pb[p] = B + (long long)(k_begin + kr) * g.ldb + gj;
    }
  }
  const long long a_step = AT ? (long long)SBK * g.lda : SBK;
  const long long b_step = BT ? (long long)SBK * g.ldb : SBK;

  uint4 ra[A_VECS], rb[B_VECS];
  // full slices need no predicate; the last slice of a ragged K zero-fills beyond the end
  auto load_global = [&](int kt) {
    const int k0 = k_begin + kt * SBK;
    const bool full = k0 + SBK <= k_end;
#pragma unroll
    for (int p = 0; p < A_VECS; p++) {
      const bool ok = full || (k0 + ka[p] < (AT ? k_end : k_end_pad));
      ra[p] = ok ? *(const uint4*)pa[p] : make_uint4(0, 0, 0, 0);
      pa[p] += a_step;
    }
#pragma unroll
    for (int p = 0; p < B_VECS; p++) {
      const bool ok = full || (k0 + kb[p] < (BT ? k_end : k_end_pad));
      rb[p] = ok ? *(const uint4*)pb[p] : make_uint4(0, 0, 0, 0);
      pb[p] += b_step;
    }
  };

  auto store_lds = [&](int buf) {
    unsigned char* sa = smem + buf * STAGE;
    unsigned char* sb = sa + LA::BYTES;
#pragma unroll
    for (int p = 0; p < A_VECS; p++) {
      const int v = tid + p * NT;
      int off;
      if (!AT) {
        const int row = v >> 3, kc = v & 7;
        off = row * LA::PITCH + ((kc ^ ((row >> 1) & 7)) << 4);
      } else {
        const int kr = v / (BM / 8), ic = v % (BM / 8);
        off = kr * LA::PITCH + (ic << 4);
      }
      *(uint4*)(sa + off) = ra[p];
    }
#pragma unroll
    for (int p = 0; p < B_VECS; p++) {
      const int v = tid + p * NT;
      int off;
      if (!BT) {
        const int row = v >> 3, kc = v & 7;
        off = row * LB::PITCH + ((kc ^ ((row >> 1) & 7)) << 4);
      } else {
        const int kr = v / (BN / 8), jc = v % (BN / 8);
        off = kr * LB::PITCH + (jc << 4);
      }
      *(uint4*)(sb + off) = rb[p];
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; mi++)
#pragma unroll
    for (int ni = 0; ni < NI; ni++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mi][ni][r] = 0.f;

  const int l32 = lane & 31, khalf = lane >> 5;          // direct: row, which 8 of the 16 k
  const int grp = lane >> 4, r16 = lane & 15;            // transposed: 16-lane groups
  const int tr_col = (grp & 1) * 16 + 4 * (r16 & 3);     // first of the 4 elements addressed
  const int tr_krow = (grp >> 1) * 8 + (r16 >> 2);       // k-row addressed (first read)

  auto compute = [&](int buf) {
    const unsigned char* sa = smem + buf * STAGE;
    const unsigned char* sb = sa + LA::BYTES;
#pragma unroll
    for (int ks = 0; ks < SBK / 16; ks++) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int mi = 0; mi < MI; mi++) {
        const int rbase = wave_m * TM + mi * 32;
        if (!AT) {
          const int row = rbase + l32, chunk = ks * 2 + khalf;
          af[mi] = *(const bf16x8*)(sa + row * LA::PITCH + ((chunk ^ ((row >> 1) & 7)) << 4));
        } else {
          const unsigned char* p = sa + (ks * 16 + tr_krow) * LA::PITCH + (rbase + tr_col) * 2;
          bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * LA::PITCH);
          af[mi] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
      }
#pragma unroll
      for (int ni = 0; ni < NI; ni++) {
        const int rbase = wave_n * TN + ni * 32;
        if (!BT) {
          const int row = rbase + l32, chunk = ks * 2 + khalf;
          bfr[ni] = *(const bf16x8*)(sb + row * LB::PITCH + ((chunk ^ ((row >> 1) & 7)) << 4));
        } else {
          const unsigned char* p = sb + (ks * 16 + tr_krow) * LB::PITCH + (rbase + tr_col) * 2;
          bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * LB::PITCH);
          bfr[ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
      }
#pragma unroll
      for (int mi = 0; mi < MI; mi++)
#pragma unroll
        for (int ni = 0; ni < NI; ni++)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
    }
  };

  if (nk > 0) {
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt++) {
      if (kt + 1 < nk) load_global(kt + 1);
      compute(kt & 1);
      if (kt + 1 < nk) store_lds((kt + 1) & 1);
      __syncthreads();
    }
  }
  if (g.no_store) return;
  wave_epilogue<EPI, MI, NI>(g, acc, (float*)smem + wave * 32 * TN, m0 + wave_m * TM, n0 + wave_n * TN, c_off, lane);
}

// =================================================================================================
// direct-to-LDS kernel: K slices of 32, ring of LDS stages filled by global_load_lds_dwordx4
// =================================================================================================
// Each lane's 16 bytes of a wave-wide load land at (load's LDS base) + 16 * lane, so the bank
// swizzle is applied on the global side: the lane computes which 16-byte piece belongs at its
// fixed LDS position.
//   - operand with contiguous reduction index: position = row * 4 + (chunk ^ ((row >> 2) & 3))
//     (rows of 64 B, four to a 256-byte bank line; 16 consecutive rows of one chunk column fall
//     into distinct banks);
//   - transposed operand: [32 k-rows][tile rows]; 16-byte chunk j of k-row k sits at
//     j ^ ((k & 3) << 1), so the 4 k-rows touched by one ds_read_b64_tr_b16 use distinct banks.
// The loads go through inline assembly and are waited for with explicit s_waitcnt vmcnt(n): the
// compiler would otherwise wait for ALL outstanding loads before any LDS read.
constexpr int DBK = 32;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// workgroup barrier that the compiler may not move memory operations across (no fence: the
// explicit vmcnt waits order the LDS writes of the direct loads)
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}

template <int BM, int BN, int WGM, int WGN, int RING, bool AT, bool BT, int EPI>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_dma_kernel(Params g) {
  constexpr int NW = WGM * WGN;
  constexpr int TM = BM / WGM, TN = BN / WGN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int A_BYTES = BM * DBK * 2, B_BYTES = BN * DBK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LOADS = BM / 16 / NW, B_LOADS = BN / 16 / NW;  // wave-wide 1 KiB loads per wave and slice
  constexpr int LOADS = A_LOADS + B_LOADS;
  static_assert(A_LOADS * 16 * NW == BM && B_LOADS * 16 * NW == BN, "tile/waves mismatch");
  static_assert(RING >= 3 && RING * STAGE <= 160 * 1024, "LDS ring too large");
  static_assert(NW * 32 * TN * 4 <= RING * STAGE, "epilogue staging does not fit");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[RING * STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WGN, wave_n = wave % WGN;
  int m0, n0, z;
  tile_coords<BM, BN>(g, m0, n0, z);
  if (g.no_store & 4) { m0 = 0; n0 = 0; }
  const bf16* A;
  const bf16* B;
  long long c_off;
  int k_begin, k_end;
  batch_offsets(g, z, A, B, c_off, k_begin, k_end);
  const int nk = (k_end - k_begin) / DBK;

  // per-lane global source of each of this wave's loads (slice 0)
  const bf16* ga[A_LOADS];
  const bf16* gb[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; i++) {
    const int q = wave * A_LOADS + i;  // which 1 KiB piece of the A stage
    if (!AT) {
      const int row = q * 16 + (lane >> 2);
      const int chunk = (lane & 3) ^ ((row >> 2) & 3);
      ga[i] = A + (long long)min(m0 + row, g.M - 1) * g.lda + k_begin + chunk * 8;
    } else {
      constexpr int CR = BM / 8;  // 16-byte chunks per k-row
      const int pos = q * 64 + lane;
      const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << 1);
      int gi = m0 + j * 8;
      if (gi + 8 > ((g.M + 7) & ~7)) gi = 0;
      ga[i] = A + (long long)(k_begin + k) * g.lda + gi;
    }
  }
#pragma unroll
  for (int i = 0; i < B_LOADS; i++) {
    const int q = wave * B_LOADS + i;
    if (!BT) {
      const int row = q * 16 + (lane >> 2);
      const int chunk = (lane & 3) ^ ((row >> 2) & 3);
      gb[i] = B + (long long)min(n0 + row, g.N - 1) * g.ldb + k_begin + chunk * 8;
    } else {
      constexpr int CR = BN / 8;
      const int pos = q * 64 + lane;
      const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << 1);
      int gj = n0 + j * 8;
      if (gj + 8 > ((g.N + 7) & ~7)) gj = 0;
      gb[i] = B + (long long)(k_begin + k) * g.ldb + gj;
    }
  }
  const long long a_step = AT ? (long long)DBK * g.lda : DBK;
  const long long b_step = BT ? (long long)DBK * g.ldb : DBK;
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;

  auto issue = [&](int stage) {
    if (g.no_store & 2) return;
    const unsigned sa = __builtin_amdgcn_readfirstlane(lds0 + stage * STAGE + wave * A_LOADS * 1024);
    const unsigned sb = __builtin_amdgcn_readfirstlane(lds0 + stage * STAGE + A_BYTES + wave * B_LOADS * 1024);
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      dma16(ga[i], sa + i * 1024);
      ga[i] += a_step;
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      dma16(gb[i], sb + i * 1024);
      gb[i] += b_step;
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; mi++)
#pragma unroll
    for (int ni = 0; ni < NI; ni++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mi][ni][r] = 0.f;

  const int l32 = lane & 31, khalf = lane >> 5;
  const int grp16 = lane >> 4, r16 = lane & 15;
  const int tr_col = (grp16 & 1) * 16 + 4 * (r16 & 3);
  const int tr_krow = (grp16 >> 1) * 8 + (r16 >> 2);
  const int tr_swz = (r16 >> 2) << 1;  // (k & 3) << 1, the same for both halves of the 8 k values

  auto load_a = [&](const unsigned char* sa, int ks, int mi) -> bf16x8 {
    const int rbase = wave_m * TM + mi * 32;
    if (!AT) {
      const int row = rbase + l32, chunk = ks * 2 + khalf;
      return *(const bf16x8*)(sa + row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4));
    } else {
      const int col = rbase + tr_col;
      const unsigned char* p = sa + (ks * 16 + tr_krow) * (BM * 2) + (((col >> 3) ^ tr_swz) << 4) + ((col >> 2) & 1) * 8;
      bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * (BM * 2));
      return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  auto load_b = [&](const unsigned char* sb, int ks, int ni) -> bf16x8 {
    const int rbase = wave_n * TN + ni * 32;
    if (!BT) {
      const int row = rbase + l32, chunk = ks * 2 + khalf;
      return *(const bf16x8*)(sb + row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4));
    } else {
      const int col = rbase + tr_col;
      const unsigned char* p = sb + (ks * 16 + tr_krow) * (BN * 2) + (((col >> 3) ^ tr_swz) << 4) + ((col >> 2) & 1) * 8;
      bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * (BN * 2));
      return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };

  // Software pipeline.  The fragments of the first half (16 of the 32 k) of slice t+1 are read
  // from LDS while the second half of slice t is multiplied, and the wait + barrier that makes
  // slice t+1 visible sits between the two halves, so LDS latency and the barrier overlap MFMAs.
  //   iteration t:  read F1(t) | mfma F0(t) | wait slice t+1, barrier | issue loads of slice
  //                 t+RING-1 into the stage of slice t-1 | read F0(t+1) | mfma F1(t)
  // At the barrier of iteration t every wave has issued the MFMAs of F0(t), hence finished all
  // reads of slice t-1: its stage may be overwritten.
  auto load_frags = [&](const unsigned char* sa, int ks, bf16x8 (&af)[MI], bf16x8 (&bfr)[NI]) {
    const unsigned char* sb = sa + A_BYTES;
#pragma unroll
    for (int mi = 0; mi < MI; mi++) af[mi] = load_a(sa, ks, mi);
#pragma unroll
    for (int ni = 0; ni < NI; ni++) bfr[ni] = load_b(sb, ks, ni);
  };
  auto mma = [&](bf16x8 (&af)[MI], bf16x8 (&bfr)[NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; mi++)
#pragma unroll
      for (int ni = 0; ni < NI; ni++)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
  };
  // wait until slice `s` has landed: slices s+1 .. min(s + RING - 3, nk - 1) may stay in flight
  auto wait_slice = [&](int sl) {
    const int younger = min(RING - 3, nk - 1 - sl);
    if (RING >= 5 && younger >= 2) wait_vmcnt<2 * LOADS>();
    else if (RING >= 4 && younger >= 1) wait_vmcnt<LOADS>();
    else wait_vmcnt<0>();
  };

  bf16x8 a0[MI], b0[NI], a1[MI], b1[NI];
#pragma unroll
  for (int sl = 0; sl < RING - 2; sl++)
    if (sl < nk) issue(sl);
  if (nk > 0) {
    wait_slice(0);
    block_barrier();
    if (RING - 2 < nk) issue(RING - 2);
    load_frags(smem, 0, a0, b0);
  }
  for (int kt = 0; kt < nk; kt++) {
    const unsigned char* sa = smem + (kt % RING) * STAGE;
    load_frags(sa, 1, a1, b1);
    mma(a0, b0);
    if (kt + 1 < nk) wait_slice(kt + 1);
    block_barrier();
    if (kt + RING - 1 < nk) issue((kt + RING - 1) % RING);
    if (kt + 1 < nk) load_frags(smem + ((kt + 1) % RING) * STAGE, 0, a0, b0);
    mma(a1, b1);
  }
  if (g.no_store & 7) return;
  __syncthreads();  // every wave is done with the stages before they are reused for the epilogue
  wave_epilogue<EPI, MI, NI>(g, acc, (float*)smem + wave * 32 * TN, m0 + wave_m * TM, n0 + wave_n * TN, c_off, lane);
}

// =================================================================================================
// two-group kernel: K slices of 64 through registers into two LDS stages
// =================================================================================================
// Measured on this chip: a wave-wide load whose lanes cover 16 rows x 64 B costs 18 ns per CU
// when every CU loads, one that covers 8 rows x 128 B (whole cache lines) 10 ns; with slices of 32
// the operand loads of a 256x256 tile take longer than its MFMAs.  This kernel therefore loads
// slices of 64 (128-byte row pieces), and since two 64 KiB stages are all that fits in LDS, the
// third buffer of the pipeline is the register file: a slice is loaded into registers one slice
// period before it is written to the stage that has just been read for the last time.
//
// Schedule.  The 8 waves form two groups with one wave on each SIMD; in every barrier interval
// one group multiplies half a slice (16 MFMAs) while the other does its memory work, then they
// swap, so the matrix pipe of a SIMD always has a wave with operands in registers:
//   group 0:  M(0,0) | C(0,0) | M(0,1) | C(0,1) | M(1,0) | ...
//   group 1:         | M(0,0) | C(0,0) | M(0,1) | C(0,1) | ...
// M(t,h): write this wave's A (h=0) or B (h=1) pieces of slice t+1 from registers to stage
// (t+1)%2, start the global loads of the same pieces of slice t+2 into those registers, read the
// fragments of half h of slice t from stage t%2.  Stage (t+1)%2 held slice t-1, last read in
// interval 4t-1; it is written in intervals 4t..4t+3 and first read in interval 4t+4.  Loads and
// stores past the last slice are not skipped but repeat the last slice into a dead stage, which
// keeps the loop free of branches.  Every wave executes the same number of barriers: group 1 one
// extra before the loop, group 0 one extra after it.
constexpr int PBK = 64;

//
// CONV = 1: the A operand is the im2col matrix of a 3x3 / stride 1 / zero padding 1 convolution
// that is never written: row m is output pixel m of an NHWC activation [.., cH, cW, cC] (g.A),
// column (tap, c) is input channel c at the pixel shifted by the tap.  cC is a multiple of 64, so
// a K slice is 64 channels of one tap: the same 128-byte row pieces as in a stored matrix, read
// from the shifted pixel, or replaced by zeros outside the image.
// CONV = 2 (weight gradient, AT = BT = true): the B operand [pixel][(tap, c)] is that same matrix,
// gathered from the activation g.B; the reduction runs over the pixels, 64 per slice, and each
// 16-byte piece (8 channels of one tap, fixed for a lane) comes from the pixel shifted by its tap.
template <int BM, int BN, int WGM, int WGN, bool AT, bool BT, int EPI, int CONV = 0>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_pp_kernel(Params g) {
  constexpr int NW = WGM * WGN;
  constexpr int TM = BM / WGM, TN = BN / WGN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int A_BYTES = BM * PBK * 2, B_BYTES = BN * PBK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW;  // wave-wide 1 KiB pieces per wave and slice
  static_assert(NW == 8, "two groups of four waves");
  // transposed operands ([64 k-rows][tile width] in LDS, read with ds_read_b64_tr_b16): the 16-byte chunks of a k-row
  // are XORed with (k & 3) << TSH.  Sixteen lanes read 32 bytes of each of four k-rows; with rows of 256 or 512
  // bytes (a multiple of the 256-byte bank span) a shift of 2 spreads the two 16-lane groups that share a clock
  // over all 64 banks, where a shift of 1 would put them on the same 32; widths that are not a multiple of 128
  // elements (192) keep the shift of 1, their rows being offset by half a bank span anyway.
  constexpr int TSH_A = (BM % 128 == 0) ? 2 : 1, TSH_B = (BN % 128 == 0) ? 2 : 1;
  static_assert(A_LOADS * 1024 * NW == A_BYTES && B_LOADS * 1024 * NW == B_BYTES, "tile/waves mismatch");
  constexpr int EPI_BYTES = NW * 32 * TN * 4;
  constexpr int SMEM = 2 * STAGE > EPI_BYTES ? 2 * STAGE : EPI_BYTES;
  static_assert(SMEM <= 160 * 1024, "LDS");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WGN, wave_n = wave % WGN;
  int m0, n0, z;
  tile_coords<BM, BN>(g, m0, n0, z);
  if (g.no_store & 4) { m0 = 0; n0 = 0; }
  const bf16* A;
  const bf16* B;
  long long c_off;
  int k_begin, k_end;
  batch_offsets(g, z, A, B, c_off, k_begin, k_end);
  const int nk = (k_end - k_begin) / PBK;

  // per-lane global source and LDS destination (within a stage) of each of this wave's pieces
  const bf16* ga[A_LOADS];
  const bf16* gb[B_LOADS];
  int la[A_LOADS], lb[B_LOADS];
  static_assert(CONV != 1 || (!AT && !BT), "implicit convolution, forward: row-major operands");
  static_assert(CONV != 2 || (AT && BT), "implicit convolution, weight gradient: both operands reduce over rows");
  int coh[CONV == 1 ? A_LOADS : 1], cow[CONV == 1 ? A_LOADS : 1];   // CONV 1: output pixel (h, w) of each piece's row
#pragma unroll
  for (int i = 0; i < A_LOADS; i++) {
    const int q = wave * A_LOADS + i;
    if (CONV == 1) {  // centre tap of the row's pixel
      const int row = q * 8 + (lane >> 3), chunk = lane & 7;
      const int m = min(m0 + row, g.M - 1);
      cow[i] = m % g.cW;
      coh[i] = (m / g.cW) % g.cH;
      ga[i] = A + (long long)m * g.cC + chunk * 8;
      la[i] = row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
    } else if (!AT) {  // 8 rows x 128 B; 16-byte chunk c of row r sits at chunk position c ^ ((r >> 1) & 7)
      const int row = q * 8 + (lane >> 3), chunk = lane & 7;
      ga[i] = A + (long long)min(m0 + row, g.M - 1) * g.lda + k_begin + chunk * 8;
      la[i] = row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
    } else {    // [64 k-rows][BM]; chunk j of k-row k sits at chunk position j ^ ((k & 3) << TSH_A)
      constexpr int CR = BM / 8;
      const int pos = q * 64 + lane;
      const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << TSH_A);
      int gi = m0 + j * 8;
      if (gi + 8 > ((g.M + 7) & ~7)) gi = 0;
      ga[i] = A + (long long)(k_begin + k) * g.lda + gi;
      la[i] = pos * 16;
    }
  }
  // CONV 2: per piece, (dy + 1) << 26 | (dx + 1) << 24 | h << 12 | w for its tap and the pixel (h, w) of its k-row
  // (cH, cW < 4096), and the tap's element offset
  int bpix[CONV == 2 ? B_LOADS : 1], boff[CONV == 2 ? B_LOADS : 1];
#pragma unroll
  for (int i = 0; i < B_LOADS; i++) {
    const int q = wave * B_LOADS + i;
    if (CONV == 2) {
      constexpr int CR = BN / 8;
      const int pos = q * 64 + lane;
      const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << TSH_B);
      int gj = n0 + j * 8;
      if (gj + 8 > g.N) gj = 0;                 // N = 9 cC is a multiple of 8
      const int tap = gj / g.cC, ch = gj % g.cC;
      const int dy = tap / 3 - 1, dx = tap % 3 - 1;
      const int pix = k_begin + k;
      bpix[i] = ((dy + 1) << 26) | ((dx + 1) << 24) | (((pix / g.cW) % g.cH) << 12) | (pix % g.cW);
      boff[i] = (dy * g.cW + dx) * g.cC;
      gb[i] = B + (long long)pix * g.cC + ch;   // centre tap
      lb[i] = A_BYTES + pos * 16;
    } else if (!BT) {
      const int row = q * 8 + (lane >> 3), chunk = lane & 7;
      gb[i] = B + (long long)min(n0 + row, g.N - 1) * g.ldb + k_begin + chunk * 8;
      lb[i] = A_BYTES + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
    } else {
      constexpr int CR = BN / 8;
      const int pos = q * 64 + lane;
      const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << TSH_B);
      int gj = n0 + j * 8;
      if (gj + 8 > ((g.N + 7) & ~7)) gj = 0;
      gb[i] = B + (long long)(k_begin + k) * g.ldb + gj;
      lb[i] = A_BYTES + pos * 16;
    }
  }
  const long long a_step = AT ? (long long)PBK * g.lda : PBK;
  const long long b_step = CONV == 2 ? (long long)PBK * g.cC : (BT ? (long long)PBK * g.ldb : PBK);
  // CONV 2: a slice moves every piece 64 pixels on: (h, w) advance by (64 / cW, 64 % cW) with carries
  const int b_sw = CONV == 2 ? PBK % g.cW : 0, b_sh = CONV == 2 ? (PBK / g.cW) % g.cH : 0;

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; mi++)
#pragma unroll
    for (int ni = 0; ni < NI; ni++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mi][ni][r] = 0.f;

  const int l32 = lane & 31, khalf = lane >> 5;
  const int grp16 = lane >> 4, r16 = lane & 15;
  const int tr_col = (grp16 & 1) * 16 + 4 * (r16 & 3);
  const int tr_krow = (grp16 >> 1) * 8 + (r16 >> 2);
  const int tr_row = r16 >> 2;   // k & 3 of the lane's k-row, the same for both halves of the 8 k values

  // fragment of k-step ks (16 k values, 0..3) of the slice in stage `st`
  auto load_a = [&](const unsigned char* st, int ks, int mi) -> bf16x8 {
    const int rbase = wave_m * TM + mi * 32;
    if (!AT) {
      const int row = rbase + l32, chunk = ks * 2 + khalf;
      return *(const bf16x8*)(st + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
    } else {
      const int col = rbase + tr_col;
      const unsigned char* p = st + (ks * 16 + tr_krow) * (BM * 2) + (((col >> 3) ^ (tr_row << TSH_A)) << 4) + ((col >> 2) & 1) * 8;
      bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * (BM * 2));
      return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  auto load_b = [&](const unsigned char* st, int ks, int ni) -> bf16x8 {
    const unsigned char* sb = st + A_BYTES;
    const int rbase = wave_n * TN + ni * 32;
    if (!BT) {
      const int row = rbase + l32, chunk = ks * 2 + khalf;
      return *(const bf16x8*)(sb + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
    } else {
      const int col = rbase + tr_col;
      const unsigned char* p = sb + (ks * 16 + tr_krow) * (BN * 2) + (((col >> 3) ^ (tr_row << TSH_B)) << 4) + ((col >> 2) & 1) * 8;
      bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + 4 * (BN * 2));
      return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  auto load_frags = [&](const unsigned char* st, int ks, bf16x8 (&af)[MI], bf16x8 (&bfr)[NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; mi++) af[mi] = load_a(st, ks, mi);
#pragma unroll
    for (int ni = 0; ni < NI; ni++) bfr[ni] = load_b(st, ks, ni);
  };
  auto mma = [&](bf16x8 (&af)[MI], bf16x8 (&bfr)[NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; mi++)
#pragma unroll
      for (int ni = 0; ni < NI; ni++)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
  };

  u32x4 ra[A_LOADS], rb[B_LOADS];
  // CONV: tap (dy, dx) and channel offset of the next slice to load (uniform), the element offset
  // of that slice from the centre tap, and per lane one bit per piece: "the registers hold data"
  // (as opposed to a pixel outside the image, stored as zeros)
  // (a split reduction starts at column k_begin = (tap, channel offset) of the matrix)
  int c_dy = -1, c_dx = -1, c_sub = 0;
  if (CONV == 1) {
    const int tap0 = k_begin / g.cC;
    c_sub = k_begin % g.cC;
    c_dy = tap0 / 3 - 1;
    c_dx = tap0 % 3 - 1;
  }
  long long c_off_a = CONV == 1 ? (long long)(c_dy * g.cW + c_dx) * g.cC + c_sub : 0;
  unsigned c_ok = 0;
  auto conv_load = [&](int i) {
    const bool ok = (unsigned)(coh[CONV == 1 ? i : 0] + c_dy) < (unsigned)g.cH && (unsigned)(cow[CONV == 1 ? i : 0] + c_dx) < (unsigned)g.cW;
    ra[i] = *(const u32x4*)(ga[i] + (ok ? c_off_a : 0));
    c_ok = ok ? (c_ok | (1u << i)) : (c_ok & ~(1u << i));
  };
  auto conv_advance = [&](bool advance) {
    if (!advance) return;
    c_sub += PBK;
    if (c_sub == g.cC) {
      c_sub = 0;
      if (++c_dx == 2) { c_dx = -1; c_dy++; }
    }
    c_off_a = (long long)(c_dy * g.cW + c_dx) * g.cC + c_sub;
  };
  // pointers always address a valid slice: they stop advancing at the last one
  auto load_a_regs = [&](bool advance) {
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      if (CONV == 1) {
        conv_load(i);
      } else {
        ra[i] = *(const u32x4*)ga[i];
        ga[i] += advance ? a_step : 0;
      }
    }
    if (CONV == 1) conv_advance(advance);
  };
  unsigned b_ok = 0;   // CONV 2: per lane one bit per piece, "the registers hold data"
  auto conv_load_b = [&](int i, bool advance) {
    const int k = CONV == 2 ? i : 0;
    const int dy = (bpix[k] >> 26) - 1, dx = ((bpix[k] >> 24) & 3) - 1;
    int h = (bpix[k] >> 12) & 4095, w = bpix[k] & 4095;
    const bool ok = (unsigned)(h + dy) < (unsigned)g.cH && (unsigned)(w + dx) < (unsigned)g.cW;
    rb[i] = *(const u32x4*)(gb[i] + (ok ? boff[k] : 0));
    b_ok = ok ? (b_ok | (1u << i)) : (b_ok & ~(1u << i));
    if (advance) {
      gb[i] += b_step;
      w += b_sw;
      h += b_sh;
      if (w >= g.cW) { w -= g.cW; h++; }
      if (h >= g.cH) h -= g.cH;
      bpix[k] = (bpix[k] & ~0xffffff) | (h << 12) | w;
    }
  };
  auto load_b_regs = [&](bool advance) {
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      if (CONV == 2) {
        conv_load_b(i, advance);
      } else {
        rb[i] = *(const u32x4*)gb[i];
        gb[i] += advance ? b_step : 0;
      }
    }
  };
  auto store_a = [&](unsigned char* st) {
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      if (CONV == 1) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        *(u32x4*)(st + la[i]) = ((c_ok >> i) & 1u) ? ra[i] : zero;
      } else {
        *(u32x4*)(st + la[i]) = ra[i];
      }
    }
  };
  auto store_b = [&](unsigned char* st) {
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      if (CONV == 2) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        *(u32x4*)(st + lb[i]) = ((b_ok >> i) & 1u) ? rb[i] : zero;
      } else {
        *(u32x4*)(st + lb[i]) = rb[i];
      }
    }
  };

  const int group = wave >> 2;
  bf16x8 a0[MI], b0[NI], a1[MI], b1[NI];
  // prologue: slice 0 into stage 0, slice 1 (or slice 0 again) into the registers
  if (CONV == 0) {
    // both slices are requested before the first is stored: one memory latency instead of two
    u32x4 ra0[A_LOADS], rb0[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      ra0[i] = *(const u32x4*)ga[i];
      ga[i] += nk > 1 ? a_step : 0;
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      rb0[i] = *(const u32x4*)gb[i];
      gb[i] += nk > 1 ? b_step : 0;
    }
    load_a_regs(nk > 2);
    load_b_regs(nk > 2);
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) *(u32x4*)(smem + la[i]) = ra0[i];
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) *(u32x4*)(smem + lb[i]) = rb0[i];
  } else {
    load_a_regs(nk > 1);
    load_b_regs(nk > 1);
    store_a(smem);
    store_b(smem);
    load_a_regs(nk > 2);
    load_b_regs(nk > 2);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  block_barrier();
  if (group == 1) block_barrier();
  // one C phase: the MFMAs of two k-steps with this wave's global loads of one operand spread
  // evenly between them, so that the loads of the four SIMDs reach
  // the texture addresser evenly instead of in a burst that would stall the issuing waves
  constexpr int P = MI * NI * 2;   // MFMAs of one C phase
  // load j is issued in the middle of its share of the phase's MFMAs (staggering the four SIMDs
  // against each other as well was measured and is slower)
  {
    constexpr int S = 2;
    auto c_phase = [&](auto loads_tag, auto&& load_one) {
      constexpr int L = decltype(loads_tag)::value;
      __builtin_amdgcn_s_setprio(1);
      int n = 0;
#pragma unroll
      for (int half = 0; half < 2; half++)
#pragma unroll
        for (int mi = 0; mi < MI; mi++)
#pragma unroll
          for (int ni = 0; ni < NI; ni++) {
            acc[mi][ni] = half == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[mi], b0[ni], acc[mi][ni], 0, 0, 0)
                                    : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[mi], b1[ni], acc[mi][ni], 0, 0, 0);
            n++;
#pragma unroll
            for (int j = 0; j < L; j++)
              if (n == 1 + (4 * j * P + S * P) / (4 * L)) {
                __builtin_amdgcn_sched_barrier(0);
                load_one(j);
                __builtin_amdgcn_sched_barrier(0);
              }
          }
      __builtin_amdgcn_s_setprio(0);
      block_barrier();
    };
    for (int kt = 0; kt < nk; kt++) {
      unsigned char* cur = smem + (kt & 1) * STAGE;
      unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE;
      const bool adv = kt + 3 < nk;   // the registers are reloaded with slice min(kt + 2, nk - 1)
      store_a(nxt);
      load_frags(cur, 0, a0, b0);
      load_frags(cur, 1, a1, b1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      block_barrier();
      c_phase(std::integral_constant<int, A_LOADS>(), [&](int i) {
        if (CONV == 1) {
          conv_load(i);
          if (i == A_LOADS - 1) conv_advance(adv);
        } else {
          ra[i] = *(const u32x4*)ga[i];
          ga[i] += adv ? a_step : 0;
        }
      });
      store_b(nxt);
      load_frags(cur, 2, a0, b0);
      load_frags(cur, 3, a1, b1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      block_barrier();
      c_phase(std::integral_constant<int, B_LOADS>(), [&](int i) {
        if (CONV == 2) {
          conv_load_b(i, adv);
        } else {
          rb[i] = *(const u32x4*)gb[i];
          gb[i] += adv ? b_step : 0;
        }
      });
    }
  }
  if (group == 0) block_barrier();
  if (g.no_store & 7) return;
  __syncthreads();  // every wave is done with the stages before they are reused for the epilogue
  wave_epilogue<EPI, MI, NI>(g, acc, (float*)smem + wave * 32 * TN, m0 + wave_m * TM, n0 + wave_n * TN, c_off, lane);
}

// host side: pick the instantiation for (layout, epilogue); returns false if that pair is not built
typedef hipError_t (*LaunchFn)(const Params&, dim3 grid, hipStream_t);
LaunchFn staged_128x128(bool a_t, bool b_t, int epi);
LaunchFn staged_128x64(bool a_t, bool b_t, int epi);
LaunchFn dma_256x256(bool a_t, bool b_t, int epi);
LaunchFn dma_256x128(bool a_t, bool b_t, int epi);
LaunchFn pp_256x256(bool a_t, bool b_t, int epi);
LaunchFn pp_256x192(bool a_t, bool b_t, int epi);
LaunchFn pp_256x128(bool a_t, bool b_t, int epi);
LaunchFn pp_512x64(bool a_t, bool b_t, int epi);
// implicit 3x3 convolution (A gathered from the activation), row-major operands
LaunchFn pp_conv_256x256(int epi);
LaunchFn pp_conv_256x192(int epi);
LaunchFn pp_conv_256x128(int epi);
LaunchFn pp_conv_512x64(int epi);
// tiles for weight gradients with few output rows, and the implicit weight gradient of a 3x3 convolution
LaunchFn pp_128x256(bool a_t, bool b_t, int epi);
LaunchFn pp_64x512(bool a_t, bool b_t, int epi);
LaunchFn pp_convdw_256x256(int epi);
LaunchFn pp_convdw_256x192(int epi);
LaunchFn pp_convdw_128x256(int epi);
LaunchFn pp_convdw_64x512(int epi);

}  // namespace gemm
}  // namespace et
