// bf16 MFMA GEMM for gfx950: D[i][j] = alpha * sum_k A(i,k) B(j,k), fp32 accumulation.
//
// The dense contractions of the training step (Section 5.1: forward product, error-gradient
// passing T1, weight-gradient T3) all reduce to this form with either operand optionally stored
// with the reduction index as the slow one:
//   forward   Y  = X  W^T : A = X  [M][K],  B = W [N][K]            (a_t = 0, b_t = 0)
//   passing   dX = dY W   : A = dY [M][N'], B = W [N'][K'] read as B(j=k', k=n')  (b_t = 1)
//   gradient  dW = dY^T X : A = dY [M'][N'] read as A(i=n', k=m), B = X likewise   (a_t = b_t = 1)
//
// Design: one workgroup computes a BM x BN tile with v_mfma_f32_32x32x16_bf16; 64-lane waves in a
// WGM x WGN grid each own a (BM/WGM) x (BN/WGN) sub-tile.  K is consumed in slices of 64 through
// two LDS buffers: the global loads of slice t+1 are issued into registers before the MFMAs of
// slice t and written to the other buffer afterwards (one barrier per slice).
//   - operand with contiguous reduction index: LDS rows of 64 bf16 (128 B), the 16-byte chunk
//     index XOR-swizzled with the row so that the ds_read_b128 of 8 consecutive rows hit
//     distinct banks; a lane reads its 8 consecutive k values directly;
//   - operand with the reduction index slow ("transposed"): LDS keeps the global layout
//     [64 k-rows][tile rows] (row pitch padded by 32 B) and the lanes fetch their 2 x 4 k values
//     with ds_read_b64_tr_b16, the LDS transpose read of gfx950: in every group of 16 lanes,
//     lane 4c+a supplies the address of 4 consecutive elements of k-row c, and lane i receives
//     element i of k-rows 0..3.
// Workgroup ids are remapped so that consecutive tiles run on the same XCD (ids are dealt
// round-robin over the 8 XCDs, each with its own L2).
#include "kernels.h"

namespace et {
namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;
constexpr int NUM_XCD = 8;

struct Params {
  const bf16* A;
  const bf16* B;
  int M, N, K;
  int lda, ldb;
  int z_inner;
  long long sAo, sAi, sBo, sBi, sCo, sCi;
  int split_k, k_chunk;  // split_k > 1: blockIdx.z picks [z*k_chunk, (z+1)*k_chunk)
  float alpha;
  const bf16* bias;
  const float* residual;
  int ldr;
  int mode;
  void* C;
  int ldc;
  int c_f32;
  bf16* C2;
  const bf16* U;
};

__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.f + erff(u * 0.70710678118654752f)) + u * __expf(-0.5f * u * u) * 0.39894228040143268f;
}

__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

template <int ROWS, bool T>
struct OperandLds {
  // bytes of one K slice of an operand tile with ROWS rows
  static constexpr int PITCH = T ? (ROWS * 2 + 32) : (BK * 2);
  static constexpr int BYTES = T ? (BK * PITCH) : (ROWS * PITCH);
};

template <int BM, int BN, int WGM, int WGN, bool AT, bool BT>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(Params g) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int TM = BM / WGM, TN = BN / WGN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int A_VECS = BM * BK / 8 / NT, B_VECS = BN * BK / 8 / NT;
  static_assert(A_VECS * NT * 8 == BM * BK && B_VECS * NT * 8 == BN * BK, "tile/threads mismatch");
  typedef OperandLds<BM, AT> LA;
  typedef OperandLds<BN, BT> LB;
  constexpr int STAGE = LA::BYTES + LB::BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WGN, wave_n = wave % WGN;

  // ---- which tile: undo the round-robin XCD dealing, then n fastest
  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (g.M + BM - 1) / BM;
  const int nt = tiles_m * tiles_n;
  int t;
  {
    const int w = blockIdx.x;
    const int xcd = w % NUM_XCD, idx = w / NUM_XCD;
    const int per = nt / NUM_XCD, rem = nt % NUM_XCD;
    t = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int m0 = (t / tiles_n) * BM, n0 = (t % tiles_n) * BN;

  // ---- batch / split-K
  const int z = blockIdx.z;
  const bf16* __restrict__ A = g.A;
  const bf16* __restrict__ B = g.B;
  long long c_off = 0;
  int k_begin = 0, k_end = g.K;
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
  const int k_end_pad = min((g.K + 7) & ~7, k_begin + (g.split_k > 1 ? g.k_chunk : ((g.K + 7) & ~7)));
  const int nk = (k_end - k_begin + BK - 1) / BK;
  const int M8 = (g.M + 7) & ~7, N8 = (g.N + 7) & ~7;

  uint4 ra[A_VECS], rb[B_VECS];

  auto load_global = [&](int kt) {
    const int k0 = k_begin + kt * BK;
#pragma unroll
    for (int p = 0; p < A_VECS; p++) {
      const int v = tid + p * NT;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (!AT) {
        const int row = v >> 3, kc = v & 7;
        const int gi = m0 + row, gk = k0 + kc * 8;
        if (gi < g.M && gk < k_end_pad) val = *(const uint4*)(A + (long long)gi * g.lda + gk);
      } else {
        const int kr = v / (BM / 8), ic = v % (BM / 8);
        const int gk = k0 + kr, gi = m0 + ic * 8;
        if (gk < k_end && gi < M8) val = *(const uint4*)(A + (long long)gk * g.lda + gi);
      }
      ra[p] = val;
    }
#pragma unroll
    for (int p = 0; p < B_VECS; p++) {
      const int v = tid + p * NT;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (!BT) {
        const int row = v >> 3, kc = v & 7;
        const int gj = n0 + row, gk = k0 + kc * 8;
        if (gj < g.N && gk < k_end_pad) val = *(const uint4*)(B + (long long)gj * g.ldb + gk);
      } else {
        const int kr = v / (BN / 8), jc = v % (BN / 8);
        const int gk = k0 + kr, gj = n0 + jc * 8;
        if (gk < k_end && gj < N8) val = *(const uint4*)(B + (long long)gk * g.ldb + gj);
      }
      rb[p] = val;
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
        off = row * LA::PITCH + ((kc ^ (row & 7)) << 4);
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
        off = row * LB::PITCH + ((kc ^ (row & 7)) << 4);
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

  // lane geometry for the two kinds of LDS reads
  const int l32 = lane & 31, khalf = lane >> 5;                     // direct: row, which 8 of the 16 k
  const int grp = lane >> 4, r16 = lane & 15;                       // transposed: 16-lane groups
  const int tr_col = (grp & 1) * 16 + 4 * (r16 & 3);                // first of the 4 elements addressed
  const int tr_krow = (grp >> 1) * 8 + (r16 >> 2);                  // k-row addressed (first read)

  auto compute = [&](int buf) {
    const unsigned char* sa = smem + buf * STAGE;
    const unsigned char* sb = sa + LA::BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ks++) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int mi = 0; mi < MI; mi++) {
        const int rbase = wave_m * TM + mi * 32;
        if (!AT) {
          const int row = rbase + l32, chunk = ks * 2 + khalf;
          af[mi] = *(const bf16x8*)(sa + row * LA::PITCH + ((chunk ^ (row & 7)) << 4));
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
          bfr[ni] = *(const bf16x8*)(sb + row * LB::PITCH + ((chunk ^ (row & 7)) << 4));
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

  // ---- epilogue.  acc[mi][ni][r] is element (row, col) =
  //      (mi*32 + (r/4)*8 + (lane/32)*4 + r%4,  ni*32 + lane%32) of the wave's sub-tile
  const bool partial = g.split_k > 1;
#pragma unroll
  for (int ni = 0; ni < NI; ni++) {
    const int col = n0 + wave_n * TN + ni * 32 + l32;
    if (col >= g.N) continue;
    float bias = 0.f;
    if (!partial && g.bias) bias = (float)g.bias[col];
#pragma unroll
    for (int mi = 0; mi < MI; mi++) {
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int row = m0 + wave_m * TM + mi * 32 + (r >> 2) * 8 + khalf * 4 + (r & 3);
        if (row >= g.M) continue;
        float v = acc[mi][ni][r];
        if (partial) {
          ((float*)g.C)[c_off + (long long)row * g.N + col] = v;
          continue;
        }
        v = v * g.alpha + bias;
        if (g.residual) v += g.residual[(long long)row * g.ldr + col];
        const long long ci = c_off + (long long)row * g.ldc + col;
        if (g.mode == EPI_GELU_BWD) v *= gelu_grad_f((float)g.U[ci]);
        if (g.c_f32)
          ((float*)g.C)[ci] = v;
        else
          ((bf16*)g.C)[ci] = (bf16)v;
        if (g.mode == EPI_GELU_FWD) g.C2[ci] = (bf16)gelu_f(v);
      }
    }
  }
}

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

enum TileId : int { T_AUTO = 0, T_128x128 = 1, T_128x64 = 3 };

template <int BM, int BN, int WGM, int WGN>
hipError_t launch_layout(const Params& p, const GemmDesc& d, int zdim, hipStream_t s) {
  const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  dim3 grid(tiles, 1, zdim), block(WGM * WGN * 64);
  if (!d.a_t && !d.b_t)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, false, false>), grid, block, 0, s, p);
  else if (!d.a_t && d.b_t)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, false, true>), grid, block, 0, s, p);
  else if (d.a_t && d.b_t)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, true, true>), grid, block, 0, s, p);
  else
    return hipErrorInvalidValue;  // (a_t, !b_t) is not used by the training step
  return hipGetLastError();
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int choose_tile(const GemmDesc& d) {
  if (d.tile != T_AUTO) return d.tile;
  return d.N <= 64 ? T_128x64 : T_128x128;
}

}  // namespace

size_t gemm_bf16_partial_elems(int M, int N, int split_k) { return split_k > 1 ? (size_t)M * N * split_k : 0; }

hipError_t gemm_bf16(const GemmDesc& d, hipStream_t s, int* launches) {
  if (launches) *launches = 0;
  if (!d.A || !d.B || !d.C || d.M <= 0 || d.N <= 0 || d.K <= 0) return hipErrorInvalidValue;
  if (!aligned16(d.A) || !aligned16(d.B) || (d.lda & 7) || (d.ldb & 7)) return hipErrorInvalidValue;
  if ((d.sAo | d.sAi | d.sBo | d.sBi) & 7) return hipErrorInvalidValue;
  if (d.z_outer < 1 || d.z_inner < 1) return hipErrorInvalidValue;
  // rows must be long enough for the 16-byte loads of the contiguous index
  if (!d.a_t && d.lda < ((d.K + 7) & ~7)) return hipErrorInvalidValue;
  if (!d.b_t && d.ldb < ((d.K + 7) & ~7)) return hipErrorInvalidValue;
  if (d.a_t && d.lda < ((d.M + 7) & ~7)) return hipErrorInvalidValue;
  if (d.b_t && d.ldb < ((d.N + 7) & ~7)) return hipErrorInvalidValue;
  if (d.mode == EPI_GELU_FWD && (!d.C2 || d.c_f32)) return hipErrorInvalidValue;
  if (d.mode == EPI_GELU_BWD && !d.U) return hipErrorInvalidValue;
  if (d.residual && d.ldr < d.N) return hipErrorInvalidValue;
  Params p;
  p.A = d.A; p.B = d.B; p.M = d.M; p.N = d.N; p.K = d.K; p.lda = d.lda; p.ldb = d.ldb;
  p.z_inner = d.z_inner;
  p.sAo = d.sAo; p.sAi = d.sAi; p.sBo = d.sBo; p.sBi = d.sBi; p.sCo = d.sCo; p.sCi = d.sCi;
  p.split_k = 1; p.k_chunk = 0;
  p.alpha = d.alpha; p.bias = d.bias; p.residual = d.residual; p.ldr = d.ldr; p.mode = d.mode;
  p.C = d.C; p.ldc = d.ldc; p.c_f32 = d.c_f32 ? 1 : 0; p.C2 = d.C2; p.U = d.U;
  int zdim = d.z_outer * d.z_inner;
  if (d.split_k > 1) {
    if (zdim != 1 || !d.partials || !d.c_f32 || d.bias || d.residual || d.mode != EPI_PLAIN || d.alpha != 1.f ||
        d.ldc != d.N || (((size_t)d.M * d.N) & 3))
      return hipErrorInvalidValue;
    const int slices = (d.K + BK - 1) / BK;
    const int per = (slices + d.split_k - 1) / d.split_k;
    p.k_chunk = per * BK;
    p.split_k = (slices + per - 1) / per;  // no empty chunks
    if (p.split_k > 1) {
      p.C = d.partials;
      zdim = p.split_k;
    } else {
      p.split_k = 1;
    }
  } else if (d.ldc < d.N) {
    return hipErrorInvalidValue;
  }
  hipError_t e;
  switch (choose_tile(d)) {
    case T_128x64: e = launch_layout<128, 64, 2, 2>(p, d, zdim, s); break;
    default: e = launch_layout<128, 128, 2, 2>(p, d, zdim, s); break;
  }
  if (e != hipSuccess) return e;
  if (launches) *launches = 1;
  if (d.split_k > 1) {
    const size_t n4 = (size_t)d.M * d.N / 4;
    if (p.split_k > 1) {
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                         (const float4*)d.partials, (float4*)d.C, n4, p.split_k);
      e = hipGetLastError();
      if (launches) *launches = 2;
    }
  }
  return e;
}

}  // namespace et
