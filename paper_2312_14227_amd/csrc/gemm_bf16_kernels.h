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
  int units;             // gemm_pp_kernel: tiles x (batch entries or reduction chunks), the work its resident workgroups loop over
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
  int cH, cW, cC;        // implicit convolution (gemm_pp_kernel<.., CONV>): input height, width, channels;
  int cT, cS, cHo, cWo;  // taps per side (3, or 1 for a strided 1x1), stride, output height and width
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

// The same for a resident workgroup that loops over units of work (gemm_pp_kernel): unit w = blockIdx.x + round *
// gridDim.x runs on XCD w % 8 in every round (the grid is a multiple of 8 whenever there is a second round), and the
// units of one XCD are consecutive (chunk or batch entry, tile) pairs in the walk above.
// Quotient and remainder of 0 <= u < 2^23 by d >= 1 through a float reciprocal (exact after one correction step:
// the float product is off by less than one unit).  The kernels divide by the same few divisors for every unit.
__device__ __forceinline__ void divmod_small(int u, int d, float rcp_d, int& q, int& r) {
  q = (int)((float)u * rcp_d);
  r = u - q * d;
  if (r < 0) { q--; r += d; }
  if (r >= d) { q++; r -= d; }
}

template <int BM, int BN>
__device__ __forceinline__ void unit_coords(const Params& g, int w, int& m0, int& n0, int& z) {
  const int tiles_n = (g.N + BN - 1) / BN;
  const int tiles_m = (g.M + BM - 1) / BM;
  const int nt = tiles_m * tiles_n;
  const int xcd = w % NUM_XCD, idx = w / NUM_XCD;
  const int per = g.units / NUM_XCD, rem = g.units % NUM_XCD;
  const int u = xcd * per + (xcd < rem ? xcd : rem) + idx;
  int t;
  divmod_small(u, nt, 1.0f / (float)nt, z, t);
  constexpr int GROUP = 8;
  const int gsz = GROUP * tiles_n;
  int grp, in;
  divmod_small(t, gsz, 1.0f / (float)gsz, grp, in);
  const int first = grp * GROUP;
  const int gm = min(tiles_m - first, GROUP);
  int qn, rm;
  divmod_small(in, gm, 1.0f / (float)gm, qn, rm);   // gm <= 8
  m0 = (first + rm) * BM;
  n0 = qn * BN;
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
// Epilogue of one wave.  The kernels multiply with the operands exchanged (MFMA of the B fragment by the A
// fragment), so a lane owns ROWS: acc[mi][ni][r] holds element
//   (mi*32 + lane%32,  ni*32 + (r/4)*8 + (lane/32)*4 + r%4)
// of the wave's TM x TN sub-tile whose top-left corner is (row0, col0): four consecutive columns per register
// quadruple.  The sub-tile goes through the wave's private LDS area 32 rows at a time and comes back with
// consecutive lanes on consecutive columns of a row, so that global stores (and the row-major second operands)
// are whole 128-byte lines:
//   - bf16 outputs that need only per-column parameters (bias, folded-BN gain and shift) are finished in the
//     registers (bias, GELU, affine + clamp), packed to bf16 and staged with 8-byte LDS writes, read back and
//     stored 16 bytes per lane (two staged outputs for GELU forward and the affine pair);
//   - everything else (fp32 outputs, residual, a second operand U) is staged as fp32 with 16-byte LDS writes and
//     finished after the read-back, 4 columns per lane.
// Row pitches are padded (8 bytes for bf16 rows, 16 for fp32 rows) so that the 32 rows written by one
// instruction fall into distinct banks.  `mid(mi)` is called before every 32-row block but the first: the
// accumulators of the blocks before it have been stored and their registers are free (a resident kernel
// requests the first slices of its next tile there).
// -------------------------------------------------------------------------------------------------
struct NoMid {
  __device__ __forceinline__ void operator()(int) const {}
};
template <int TN>
constexpr int epi_wave_bytes() { return 32 * (TN + 4) * 4; }   // fp32 rows of TN + 4; two bf16 areas of rows of 2 TN + 8 bytes

template <int EPI>
constexpr bool epi_pre() {
  return EPI == E_BF16 || EPI == E_GELU_FWD || EPI == E_GELU_ONLY || EPI == E_BIAS_RELU || EPI == E_AFFINE;
}

// FULL: the wave's whole sub-tile lies inside the matrix and every store address is 16-byte aligned: no per-lane
// bounds checks, no ragged paths (all but the last row and column of tiles take this variant).
template <int EPI, int MI, int NI, bool FULL, typename Mid>
__device__ __forceinline__ void wave_epilogue_impl(const Params& g, f32x16 (&acc)[MI][NI], unsigned char* stage, int row0, int col0,
                                                   long long c_off, int lane, Mid&& mid) {
  constexpr int TN = NI * 32;
  const int l32 = lane & 31, khalf = lane >> 5;
  const int ld = EPI == E_PARTIAL ? g.N : g.ldc;
  if constexpr (epi_pre<EPI>()) {
    constexpr bool TWO = EPI == E_GELU_FWD || EPI == E_AFFINE;
    constexpr int PITCH = TN * 2 + 8;                 // bytes per staged bf16 row
    constexpr int AREA = 32 * PITCH;
    static_assert(2 * AREA <= epi_wave_bytes<TN>(), "staging area");
    constexpr int V = (64 % (TN / 8) == 0) ? 8 : 4;   // columns per lane when reading back (16 or 8 bytes)
    constexpr int CPL = TN / V;                       // lanes per row
    constexpr int RPI = 64 / CPL;                     // rows covered by one wave-wide read
    constexpr int ITERS = (32 + RPI - 1) / RPI;
    typedef bf16 bf16xv __attribute__((ext_vector_type(V)));
    // per-column parameters of this lane's column quadruples
    bf16x4 bias_q[NI][4], gain_q[EPI == E_AFFINE ? NI : 1][4];
    const bool has_bias = g.bias != nullptr;
#pragma unroll
    for (int ni = 0; ni < NI; ni++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int col = col0 + ni * 32 + q * 8 + khalf * 4;
        bf16x4 b, gn;
#pragma unroll
        for (int j = 0; j < 4; j++) { b[j] = (bf16)0.f; gn[j] = (bf16)1.f; }
        if (FULL || col + 3 < g.N) {
          if (has_bias) b = *(const bf16x4*)(g.bias + col);
          if (EPI == E_AFFINE) gn = *(const bf16x4*)(g.gain + col);
        } else {
          for (int j = 0; j < 4 && col + j < g.N; j++) {
            if (has_bias) b[j] = g.bias[col + j];
            if (EPI == E_AFFINE) gn[j] = g.gain[col + j];
          }
        }
        bias_q[ni][q] = b;
        if (EPI == E_AFFINE) gain_q[ni][q] = gn;
      }
    // read-back coordinates: V columns of one row per lane
    const int cv = (lane % CPL) * V, rsub = lane / CPL;
    const int colr = col0 + cv;
    const bool lane_on = rsub < RPI && (FULL || colr < g.N);
    const bool wide = FULL || (colr + V - 1 < g.N && (ld & 7) == 0 && (c_off & 7) == 0 && ((uintptr_t)g.C & 15) == 0 &&
                               (!TWO || ((uintptr_t)g.C2 & 15) == 0));
    const bool keep_c = !(EPI == E_AFFINE) || g.C != nullptr;    // z is kept only if the gain's gradient will be computed
    long long ci = c_off + (long long)(row0 + rsub) * ld + colr;  // element index of this lane's piece, first row group
    const long long ci_step = (long long)RPI * ld;
#pragma unroll
    for (int mi = 0; mi < MI; mi++) {
      if (mi > 0) mid(mi);
#pragma unroll
      for (int ni = 0; ni < NI; ni++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          bf16x4 o, o2;
#pragma unroll
          for (int j = 0; j < 4; j++) {
            const float a = acc[mi][ni][q * 4 + j];
            if (EPI == E_AFFINE) {
              o[j] = (bf16)(a * g.alpha);
              o2[j] = (bf16)fminf(fmaxf((float)o[j] * (float)gain_q[EPI == E_AFFINE ? ni : 0][q][j] + (float)bias_q[ni][q][j], g.act_lo), g.act_hi);
            } else {
              const float v = a * g.alpha + (float)bias_q[ni][q][j];
              if (EPI == E_GELU_FWD) {
                float gv, dgv;
                gelu_both(v, gv, dgv);
                o[j] = (bf16)dgv;
                o2[j] = (bf16)gv;
              } else if (EPI == E_GELU_ONLY) {
                o[j] = (bf16)gelu_only(v);
              } else if (EPI == E_BIAS_RELU) {
                o[j] = (bf16)fmaxf(v, 0.f);
              } else {
                o[j] = (bf16)v;
              }
            }
          }
          unsigned char* p = stage + l32 * PITCH + (ni * 32 + q * 8 + khalf * 4) * 2;
          *(bf16x4*)p = o;
          if (TWO) *(bf16x4*)(p + AREA) = o2;
        }
      // the same wave reads back: LDS operations of one wave complete in order
      bf16xv rd[ITERS], rd2[TWO ? ITERS : 1];
#pragma unroll
      for (int it = 0; it < ITERS; it++) {
        const unsigned char* p = stage + min(it * RPI + rsub, 31) * PITCH + cv * 2;
        rd[it] = *(const bf16xv*)p;
        if (TWO) rd2[TWO ? it : 0] = *(const bf16xv*)(p + AREA);
      }
      if (lane_on) {
#pragma unroll
        for (int it = 0; it < ITERS; it++, ci += ci_step) {
          const int rr = it * RPI + rsub;
          if ((32 % RPI != 0 && rr >= 32) || (!FULL && row0 + mi * 32 + rr >= g.M)) continue;
          if (wide) {
            if (keep_c) *(bf16xv*)((bf16*)g.C + ci) = rd[it];
            if (TWO) *(bf16xv*)(g.C2 + ci) = rd2[TWO ? it : 0];
          } else {
            for (int j = 0; j < V && colr + j < g.N; j++) {
              if (keep_c) ((bf16*)g.C)[ci + j] = rd[it][j];
              if (TWO) g.C2[ci + j] = rd2[TWO ? it : 0][j];
            }
          }
        }
        ci += (32 - ITERS * RPI) * (long long)ld;   // (zero when RPI divides 32)
      }
    }
  } else {
    constexpr int PITCH = TN + 4;    // floats per staged row
    float* stf = (float*)stage;
    constexpr int CPL = TN / 4;      // lanes per row when reading back 4 columns each
    constexpr int RPI = 64 / CPL;    // rows covered by one wave-wide read
    constexpr int ITERS = (32 + RPI - 1) / RPI;
    const int c4 = (lane % CPL) * 4, rsub = lane / CPL;
    const int col = col0 + c4;
    // (when 64 is not a multiple of CPL the last lanes of the wave have no row of their own)
    const bool col_any = (FULL || col < g.N) && rsub < RPI, col_full = FULL || col + 3 < g.N;
    float bias[4] = {0.f, 0.f, 0.f, 0.f};
    float gain[4] = {1.f, 1.f, 1.f, 1.f};
    float gain2[4] = {1.f, 1.f, 1.f, 1.f}, bias2[4] = {0.f, 0.f, 0.f, 0.f};
    if (EPI == E_AFFINE_ADD && col_any) {
      for (int j = 0; j < 4 && col + j < g.N; j++) gain[j] = (float)g.gain[col + j];
      if (g.gain2)
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
    long long ci0 = c_off + (long long)(row0 + rsub) * ld + col;               // this lane's piece, first row group
    long long ri0 = HAS_RES ? (long long)(row0 + rsub) * g.ldr + col : 0;      // the same in the residual
    const long long ci_step = (long long)RPI * ld, ri_step = HAS_RES ? (long long)RPI * g.ldr : 0;
#pragma unroll
    for (int mi = 0; mi < MI; mi++) {
      if (mi > 0) mid(mi);
      // the second operands of this 32-row block are requested before the accumulators go through
      // LDS, all at once: one memory latency per block instead of one per row group
      float4 pre_res[HAS_RES ? ITERS : 1];
      bf16x4 pre_u[HAS_U ? ITERS : 1];
      if ((HAS_RES || HAS_U) && col_any && col_full) {
        long long ci = ci0, ri = ri0;
#pragma unroll
        for (int it = 0; it < ITERS; it++, ci += ci_step, ri += ri_step) {
          const int rr = it * RPI + rsub;
          if ((32 % RPI != 0 && rr >= 32) || (!FULL && row0 + mi * 32 + rr >= g.M)) continue;
          if (HAS_RES) pre_res[HAS_RES ? it : 0] = *(const float4*)(g.residual + ri);
          if (HAS_U) pre_u[HAS_U ? it : 0] = *(const bf16x4*)(g.U + ci);
        }
      }
#pragma unroll
      for (int ni = 0; ni < NI; ni++)
#pragma unroll
        for (int q = 0; q < 4; q++)
          *(float4*)(stf + l32 * PITCH + ni * 32 + q * 8 + khalf * 4) =
              make_float4(acc[mi][ni][q * 4], acc[mi][ni][q * 4 + 1], acc[mi][ni][q * 4 + 2], acc[mi][ni][q * 4 + 3]);
      // the same wave reads back: LDS operations of one wave complete in order
      float4 rd[ITERS];
#pragma unroll
      for (int it = 0; it < ITERS; it++) rd[it] = *(const float4*)(stf + min(it * RPI + rsub, 31) * PITCH + c4);
      if (col_any) {
        long long ci = ci0;
#pragma unroll
        for (int it = 0; it < ITERS; it++, ci += ci_step) {
          const int rr = it * RPI + rsub;
          if ((32 % RPI != 0 && rr >= 32) || (!FULL && row0 + mi * 32 + rr >= g.M)) continue;
          const float4 raw = rd[it];
          float v[4] = {raw.x, raw.y, raw.z, raw.w};
          if (EPI == E_AFFINE_ADD) {
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
            const long long ri = (long long)(row0 + mi * 32 + rr) * g.ldr + col;
            for (int j = 0; j < 4 && col + j < g.N; j++) {
              float x = v[j];
              if (EPI == E_F32_RES) x += g.residual[ri + j];
              if (EPI == E_GELU_BWD) x *= (float)g.U[ci + j];
              if (EPI == E_RELU_MASK) x = ((float)g.U[ci + j] > 0.f && (float)g.U[ci + j] < g.mask_hi) ? x : 0.f;
              if (EPI == E_F32 || EPI == E_F32_RES || EPI == E_PARTIAL) {
                ((float*)g.C)[ci + j] = x;
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
      ci0 += 32 * (long long)ld;
      ri0 += HAS_RES ? 32 * (long long)g.ldr : 0;
    }
  }
}

template <int EPI, int MI, int NI, typename Mid = NoMid>
__device__ __forceinline__ void wave_epilogue(const Params& g, f32x16 (&acc)[MI][NI], unsigned char* stage, int row0, int col0,
                                              long long c_off, int lane, Mid&& mid = NoMid()) {
  constexpr int TN = NI * 32;
  const int ld = EPI == E_PARTIAL ? g.N : g.ldc;
  // uniform over the wave: the whole sub-tile inside the matrix, every vector access aligned
  bool full = row0 + MI * 32 <= g.M && col0 + TN <= g.N;
  if (epi_pre<EPI>())
    full = full && (ld & 7) == 0 && (c_off & 7) == 0 && ((uintptr_t)g.C & 15) == 0 && ((uintptr_t)g.C2 & 15) == 0;
  if (full)
    wave_epilogue_impl<EPI, MI, NI, true>(g, acc, stage, row0, col0, c_off, lane, mid);
  else
    wave_epilogue_impl<EPI, MI, NI, false>(g, acc, stage, row0, col0, c_off, lane, mid);
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
  constexpr int EPI_BYTES = WGM * WGN * epi_wave_bytes<TN>();
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
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], af[mi], acc[mi][ni], 0, 0, 0);
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
  wave_epilogue<EPI, MI, NI>(g, acc, smem + wave * epi_wave_bytes<TN>(), m0 + wave_m * TM, n0 + wave_n * TN, c_off, lane);
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
  static_assert(NW * epi_wave_bytes<TN>() <= RING * STAGE, "epilogue staging does not fit");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[RING * STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WGN, wave_n = wave % WGN;
  int m0, n0, z;
  tile_coords<BM, BN>(g, m0, n0, z);
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
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], af[mi], acc[mi][ni], 0, 0, 0);
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
  __syncthreads();  // every wave is done with the stages before they are reused for the epilogue
  wave_epilogue<EPI, MI, NI>(g, acc, smem + wave * epi_wave_bytes<TN>(), m0 + wave_m * TM, n0 + wave_n * TN, c_off, lane);
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
// CONV = 1: the A operand is the im2col matrix of a 3x3 / zero padding 1 convolution of stride 1 or 2 (or of a
// strided 1x1 convolution) that is never written: row m is output pixel m, column (tap, c) is input channel c of
// the NHWC activation [.., cH, cW, cC] (g.A) at the pixel that tap reads.  cC is a multiple of 64, so a K slice
// is 64 channels of one tap: the same 128-byte row pieces as in a stored matrix, read from the shifted pixel,
// or replaced by zeros outside the image.
// CONV = 2 (weight gradient, AT = BT = true): the B operand [output pixel][(tap, c)] is that same matrix,
// gathered from the activation g.B; the reduction runs over the output pixels, 64 per slice, and each
// 16-byte piece (8 channels of one tap, fixed for a lane) comes from the input pixel its tap reads.
// GEN = false compiles the geometry of the common case in (3x3, stride 1: output size = input size); GEN = true takes
// taps, stride and output size from the launch arguments (stride 2, 1x1 taps, the stem form below).
// Stem form of both (cT == 8: a 7x7 / stride 2 / zero padding 3 convolution of an image with at most 4 channels):
// the activation is the image padded to 4 channels and by 3 pixels at the top and left (zeros up to cH x cW with
// cW even), the window is widened to 8 x 8 with zero weights, so K = 8 * 8 * 4 = 256 and a K slice is two window
// rows of 64 contiguous bytes each, 16-byte aligned, that never leave the padded image: no validity test.
template <int BM, int BN, int WGM, int WGN, bool AT, bool BT, int EPI, int CONV = 0, bool GEN = false>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_pp_kernel(Params g) {
  // convolution geometry: compile-time constants for the common 3x3 / stride 1 form, launch arguments for the general one
  const int cS = GEN ? g.cS : 1, cT = GEN ? g.cT : 3, cHo = GEN ? g.cHo : g.cH, cWo = GEN ? g.cWo : g.cW;
  const bool stem = GEN && g.cT == 8;
  const int ssh = cS >> 1;   // the stride (1 or 2) as a shift
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
  constexpr int EPI_BYTES = NW * epi_wave_bytes<TN>();
  constexpr int SMEM = 2 * STAGE > EPI_BYTES ? 2 * STAGE : EPI_BYTES;
  static_assert(SMEM <= 160 * 1024, "LDS");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WGN, wave_n = wave % WGN;
  static_assert(CONV != 1 || (!AT && !BT), "implicit convolution, forward: row-major operands");
  static_assert(CONV != 2 || (AT && BT), "implicit convolution, weight gradient: both operands reduce over rows");

  // ---- state of the unit of work (tile, and batch entry or reduction chunk) being computed
  int m0, n0, z;
  const bf16* A;
  const bf16* B;
  long long c_off;
  int k_begin, k_end, nk;
  // per-lane global source of each of this wave's pieces; CONV 1: output pixel (h, w) of each piece's row;
  // CONV 2: per piece, (dy + 1) << 26 | (dx + 1) << 24 | h << 12 | w for its tap and the pixel (h, w) of its k-row
  // (cH, cW < 4096), and the tap's element offset
  const bf16* ga[A_LOADS];
  const bf16* gb[B_LOADS];
  int coh[CONV == 1 ? A_LOADS : 1], cow[CONV == 1 ? A_LOADS : 1];
  int bpix[CONV == 2 ? B_LOADS : 1], boff[CONV == 2 ? B_LOADS : 1];
  // CONV 1: tap (dy, dx) and channel offset of the next slice to load (uniform), the element offset of that
  // slice from the centre tap (a split reduction starts at column k_begin = (tap, channel offset) of the matrix)
  int c_dy = -1, c_dx = -1, c_sub = 0;
  long long c_off_a = 0;

  // LDS destination (within a stage) of each piece: the same for every unit
  int la[A_LOADS], lb[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; i++) {
    const int q = wave * A_LOADS + i;
    if (CONV == 1 || !AT) {  // 8 rows x 128 B; 16-byte chunk c of row r sits at chunk position c ^ ((r >> 1) & 7)
      const int row = q * 8 + (lane >> 3), chunk = lane & 7;
      la[i] = row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
    } else {                 // [64 k-rows][BM]; chunk j of k-row k sits at chunk position j ^ ((k & 3) << TSH_A)
      la[i] = (q * 64 + lane) * 16;
    }
  }
#pragma unroll
  for (int i = 0; i < B_LOADS; i++) {
    const int q = wave * B_LOADS + i;
    if (CONV != 2 && !BT) {
      const int row = q * 8 + (lane >> 3), chunk = lane & 7;
      lb[i] = A_BYTES + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
    } else {
      lb[i] = A_BYTES + (q * 64 + lane) * 16;
    }
  }

  auto setup = [&](int w) {
    // (lane-dependent values of the address computation come from an opaque copy of the thread index: they are
    // recomputed per unit instead of occupying registers throughout the main loop)
    int s_tid = tid;
    asm volatile("" : "+v"(s_tid));
    const int lane = s_tid & 63, wave = s_tid >> 6;
    unit_coords<BM, BN>(g, w, m0, n0, z);
    batch_offsets(g, z, A, B, c_off, k_begin, k_end);
    nk = (k_end - k_begin) / PBK;
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      const int q = wave * A_LOADS + i;
      if (CONV == 1) {  // centre tap of the row's pixel
        const int row = q * 8 + (lane >> 3), chunk = lane & 7;
        const int m = min(m0 + row, g.M - 1);
        const int wo = m % cWo, t = m / cWo, ho = t % cHo, img = t / cHo;
        cow[CONV == 1 ? i : 0] = wo * cS;           // input coordinates of the centre tap
        coh[CONV == 1 ? i : 0] = ho * cS;
        ga[i] = A + ((long long)(img * g.cH + ho * cS) * g.cW + wo * cS) * g.cC + chunk * 8;
        if (stem) {   // stem form: chunk = (row of the pair, pixel pair); nothing lies outside the padded image
          cow[CONV == 1 ? i : 0] = 0;
          coh[CONV == 1 ? i : 0] = 0;
          ga[i] = A + ((long long)(img * g.cH + ho * 2 + (chunk >> 2)) * g.cW + wo * 2) * 4 + (chunk & 3) * 8;
        }
      } else if (!AT) {
        const int row = q * 8 + (lane >> 3), chunk = lane & 7;
        ga[i] = A + (long long)min(m0 + row, g.M - 1) * g.lda + k_begin + chunk * 8;
      } else {
        constexpr int CR = BM / 8;
        const int pos = q * 64 + lane;
        const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << TSH_A);
        int gi = m0 + j * 8;
        if (gi + 8 > ((g.M + 7) & ~7)) gi = 0;
        ga[i] = A + (long long)(k_begin + k) * g.lda + gi;
      }
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      const int q = wave * B_LOADS + i;
      if (CONV == 2) {
        constexpr int CR = BN / 8;
        const int pos = q * 64 + lane;
        const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << TSH_B);
        int gj = n0 + j * 8;
        if (gj + 8 > g.N) gj = 0;                 // N = 9 cC is a multiple of 8
        const int tap = gj / g.cC;
        int ch = gj % g.cC;
        int dy = tap / cT - (cT >> 1), dx = tap % cT - (cT >> 1);
        int off = (dy * g.cW + dx) * g.cC;
        if (stem) {   // stem form: column = (row 0..7, pixel pair 0..3, 8 values), always inside the padded image
          off = ((gj >> 5) * g.cW) * 4 + ((gj >> 3) & 3) * 8;
          dy = dx = ch = 0;
        }
        const int pix = k_begin + k;               // output pixel of this k-row
        const int wo = pix % cWo, t = pix / cWo, ho = t % cHo, img = t / cHo;
        bpix[CONV == 2 ? i : 0] = ((dy + 1) << 26) | ((dx + 1) << 24) | (ho << 12) | wo;
        boff[CONV == 2 ? i : 0] = off;
        gb[i] = B + ((long long)(img * g.cH + ho * cS) * g.cW + wo * cS) * g.cC + ch;   // centre tap
      } else if (!BT) {
        const int row = q * 8 + (lane >> 3), chunk = lane & 7;
        gb[i] = B + (long long)min(n0 + row, g.N - 1) * g.ldb + k_begin + chunk * 8;
      } else {
        constexpr int CR = BN / 8;
        const int pos = q * 64 + lane;
        const int k = pos / CR, j = (pos % CR) ^ ((k & 3) << TSH_B);
        int gj = n0 + j * 8;
        if (gj + 8 > ((g.N + 7) & ~7)) gj = 0;
        gb[i] = B + (long long)(k_begin + k) * g.ldb + gj;
      }
    }
    if (CONV == 1) {
      const int tap0 = k_begin / g.cC;
      c_sub = k_begin % g.cC;
      c_dy = tap0 / cT - (cT >> 1);
      c_dx = tap0 % cT - (cT >> 1);
      c_off_a = (long long)(c_dy * g.cW + c_dx) * g.cC + c_sub;
      if (stem) {   // stem form: a slice is two rows of the 8 x 8 window
        c_sub = c_dy = c_dx = 0;
        c_off_a = (long long)(k_begin / PBK) * 2 * g.cW * 4;
      }
    }
  };
  const long long a_step = AT ? (long long)PBK * g.lda : PBK;
  const long long b_step = BT ? (long long)PBK * g.ldb : PBK;
  // CONV 2: a slice moves every piece 64 output pixels on: (image, ho, wo) advance by (64 / (cHo cWo), (64 / cWo) % cHo,
  // 64 % cWo) with carries, and the input pointer follows by the corresponding number of input pixels
  const int b_sw = CONV == 2 ? PBK % cWo : 0, b_sh = CONV == 2 ? (PBK / cWo) % cHo : 0,
            b_sb = CONV == 2 ? PBK / (cWo * cHo) : 0;
  // element distance of that move without carries, and what a carry out of a row / out of an image adds
  const int b_d0 = CONV == 2 ? ((b_sb * g.cH + (b_sh << ssh)) * g.cW + (b_sw << ssh)) * g.cC : 0;
  const int b_dw = CONV == 2 ? ((g.cW - cWo) << ssh) * g.cC : 0, b_dh = CONV == 2 ? (g.cH - (cHo << ssh)) * g.cW * g.cC : 0;

  f32x16 acc[MI][NI];

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

  u32x4 ra[A_LOADS], rb[B_LOADS];
  // per lane one bit per piece: "the registers hold data" (as opposed to a pixel outside the image, stored as zeros)
  unsigned c_ok = 0;
  auto conv_load = [&](int i) {
    const bool ok = (unsigned)(coh[CONV == 1 ? i : 0] + c_dy) < (unsigned)g.cH && (unsigned)(cow[CONV == 1 ? i : 0] + c_dx) < (unsigned)g.cW;
    ra[i] = *(const u32x4*)(ga[i] + (ok ? c_off_a : 0));
    c_ok = ok ? (c_ok | (1u << i)) : (c_ok & ~(1u << i));
  };
  auto conv_advance = [&](bool advance) {
    if (!advance) return;
    if (stem) {
      c_off_a += 2 * g.cW * 4;
      return;
    }
    c_sub += PBK;
    if (c_sub == g.cC) {
      c_sub = 0;
      if (++c_dx > (cT >> 1)) { c_dx = -(cT >> 1); c_dy++; }
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
    const bool ok = (unsigned)((h << ssh) + dy) < (unsigned)g.cH && (unsigned)((w << ssh) + dx) < (unsigned)g.cW;
    rb[i] = *(const u32x4*)(gb[i] + (ok ? boff[k] : 0));
    b_ok = ok ? (b_ok | (1u << i)) : (b_ok & ~(1u << i));
    if (advance) {
      int delta = b_d0;
      w += b_sw;
      h += b_sh;
      if (w >= cWo) { w -= cWo; h++; delta += b_dw; }
      if (h >= cHo) { h -= cHo; delta += b_dh; }
      gb[i] += delta;
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
  // Start of a unit, plain product: slices 0 and 1 are both requested before the first is stored (one memory
  // latency instead of two), and, from the second unit on, before the epilogue of the unit just finished: the
  // loads travel while the accumulators pass through LDS and the stores of that tile drain.
  u32x4 ra0[CONV == 0 ? A_LOADS : 1], rb0[CONV == 0 ? B_LOADS : 1];
  auto first_loads = [&]() {
#pragma unroll
    for (int i = 0; i < A_LOADS; i++) {
      ra0[CONV == 0 ? i : 0] = *(const u32x4*)ga[i];
      ga[i] += nk > 1 ? a_step : 0;
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; i++) {
      rb0[CONV == 0 ? i : 0] = *(const u32x4*)gb[i];
      gb[i] += nk > 1 ? b_step : 0;
    }
  };
  auto second_loads = [&]() {
    load_a_regs(nk > 2);
    load_b_regs(nk > 2);
  };
  // barrier between phases that exchange data through LDS only: the wave's own LDS operations are complete,
  // outstanding global loads and stores are left in flight (a __syncthreads would wait for them too)
  auto lds_barrier = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    block_barrier();
  };
  // one C phase: the MFMAs of two k-steps with this wave's global loads of one operand spread
  // evenly between them, so that the loads of the four SIMDs reach
  // the texture addresser evenly instead of in a burst that would stall the issuing waves
  constexpr int P = MI * NI * 2;   // MFMAs of one C phase
  // load j is issued in the middle of its share of the phase's MFMAs (staggering the four SIMDs
  // against each other as well was measured and is slower)
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
          acc[mi][ni] = half == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b0[ni], a0[mi], acc[mi][ni], 0, 0, 0)
                                  : __builtin_amdgcn_mfma_f32_32x32x16_bf16(b1[ni], a1[mi], acc[mi][ni], 0, 0, 0);
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

  // The workgroup stays resident and walks over units w = blockIdx.x, + gridDim.x, ...: the launch cost of a
  // workgroup is paid once, and the stores of a tile drain while the next tile's first slices arrive.
  int w = blockIdx.x;
  setup(w);
  if (CONV == 0) { first_loads(); second_loads(); }
  for (;;) {
#pragma unroll
    for (int mi = 0; mi < MI; mi++)
#pragma unroll
      for (int ni = 0; ni < NI; ni++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[mi][ni][r] = 0.f;
    // slice 0 into stage 0, slice 1 (or slice 0 again) into the registers
    if (CONV == 0) {
#pragma unroll
      for (int i = 0; i < A_LOADS; i++) *(u32x4*)(smem + la[i]) = ra0[CONV == 0 ? i : 0];
#pragma unroll
      for (int i = 0; i < B_LOADS; i++) *(u32x4*)(smem + lb[i]) = rb0[CONV == 0 ? i : 0];
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
    if (group == 0) block_barrier();
    // where this tile goes; then the next unit's coordinates and first loads, ahead of the epilogue
    const int m0e = m0, n0e = n0;
    const long long e_off = c_off;
    const int w_next = w + (int)gridDim.x;
    const bool more = w_next < g.units;
    lds_barrier();    // every wave is done with the stages before they are reused for the epilogue
    // The next unit's coordinates and its first slice are requested from inside the epilogue, once half of the
    // accumulator registers are free: the loads travel while the second half is stored.  (After the last unit
    // the same unit's first slice is requested once more and dropped: an unconditional request leaves no path on
    // which the registers of the previous request would have to survive the main loop.)
    // (not where the epilogue needs the registers itself: prefetched residual rows, two sets of per-column parameters)
    constexpr bool MID_PREFETCH = CONV == 0 && MI > 1 && EPI != E_F32_RES && EPI != E_AFFINE;
    auto mid = [&](int mi) {
      if (MID_PREFETCH && mi == (MI + 1) / 2) {   // slice 0, once half of the accumulators are stored
        setup(more ? w_next : w);
        first_loads();
      }
      if (MID_PREFETCH && mi == MI - 1) second_loads();   // slice 1 before the last block
    };
    // (the epilogue's own lane-dependent values are derived from an opaque copy of the thread index, so that they
    // are computed here and not kept in registers across the main loop of every unit)
    int e_tid = tid;
    asm volatile("" : "+v"(e_tid));
    const int e_lane = e_tid & 63, e_wave = e_tid >> 6;
    wave_epilogue<EPI, MI, NI>(g, acc, smem + e_wave * epi_wave_bytes<TN>(), m0e + (e_wave / WGN) * TM, n0e + (e_wave % WGN) * TN, e_off,
                               e_lane, mid);
    if (!more) break;
    w = w_next;
    if (!MID_PREFETCH) {
      setup(w_next);
      if (CONV == 0) { first_loads(); second_loads(); }
    }
    lds_barrier();    // and done with the epilogue's staging area before the next unit's first slice is stored
  }
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
LaunchFn pp_conv_256x256(int epi, bool general);
LaunchFn pp_conv_256x192(int epi, bool general);
LaunchFn pp_conv_256x128(int epi, bool general);
LaunchFn pp_conv_512x64(int epi, bool general);
// tiles for weight gradients with few output rows, and the implicit weight gradient of a 3x3 convolution
LaunchFn pp_128x256(bool a_t, bool b_t, int epi);
LaunchFn pp_64x512(bool a_t, bool b_t, int epi);
LaunchFn pp_convdw_256x256(int epi, bool general);
LaunchFn pp_convdw_256x192(int epi, bool general);
LaunchFn pp_convdw_128x256(int epi, bool general);
LaunchFn pp_convdw_64x512(int epi, bool general);

}  // namespace gemm
}  // namespace et
