// Fused attention core for short sequences (tokens <= 224, head size 64): forward
// O = softmax(Q K^T / sqrt(d)) V and its backward (dQ, dK, dV), one workgroup per (batch, head).
// These are the "attention operations" the paper counts among the non-trainable layers (Section
// 5.4): they hold no weights, their backward time is charged to the tensor whose passing needs it.
//
// Everything of one head fits on chip: K and V (forward) or Q, K, V, dO (backward) are staged in
// LDS once, rows beyond the sequence zero-filled; the score matrix never goes to memory.
//
// Register layout trick.  v_mfma_f32_32x32x16_bf16 returns a 32x32 tile with lane l holding
// column l%32 and rows (r/4)*8 + (l/32)*4 + r%4 (r = 0..15).  Scores are computed TRANSPOSED,
// S^T = K Q^T, so a lane holds ONE query (l%32) and 16 keys per 32-key tile: the softmax over keys
// is an in-lane loop plus one exchange with lane l^32.  The same registers, converted to bf16, are
// exactly an MFMA A operand (row = query l%32, 8 reduction slots per lane) for P V, with the
// reduction slots meaning keys (e/4)*8 + (l/32)*4 + e%4 of a 16-key group; the matching B operand
// (V with the same key order, one column d per lane) is what two ds_read_b64_tr_b16 deliver from
// V stored [key][d].  No shuffle or LDS round trip between the two matrix products.
// The backward pass uses the mirrored trick (S = Q K^T, a lane holds one key) for dK and dV, and takes
// rowsum(P * dP) of a query from the stored forward output: it equals dO . O.
#include "kernels.h"

#include <type_traits>

namespace et {
namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int DH = 64;
constexpr int NWAVES = 8, NTHREADS = NWAVES * 64;
// LDS rows are the 128 bytes of 64 bf16 without padding; the 16-byte chunk c of row r sits at chunk position
// c ^ swz(r).  Every tile is read two ways and both must spread over the 64 banks:
//   - row-major fragments (ds_read_b128, 16 consecutive rows x one chunk per 16 lanes): rows alternate between the
//     two 128-byte halves of the 256-byte bank span, so the 8 even rows of a group need 8 different positions;
//   - transposing fragments (ds_read_b64_tr_b16, 4 consecutive rows x 64 contiguous bytes per 32 lanes): rows
//     r and r + 2 share a half, so their 64-byte pieces must land in different quarters.
// swz(r) = bit 1 of r as the high bit, bits 2..3 of r as the low bits, does both (a plain (r >> 1) & 7 leaves the
// transposing reads two-way conflicted, as did padded rows of 160 bytes: 41-45 % conflict cycles measured).
constexpr int PITCH = 128;
__device__ __forceinline__ int swz(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

// rows [0, T) of NM [T][64] bf16 matrices (row stride ld[m] elements) into LDS rows of PITCH bytes; rows
// [T, TP) are zero-filled.  All loads are issued before the first store, so the matrices arrive
// after one memory latency instead of one per 16-byte piece.
template <int TP, int NM>
__device__ __forceinline__ void stage_rows(unsigned char* const (&dst)[NM], const bf16* const (&src)[NM],
                                           const long long (&ld)[NM], int T, int tid) {
  constexpr int PER = (TP * 8 + NTHREADS - 1) / NTHREADS;
  uint4 val[NM][PER];
#pragma unroll
  for (int m = 0; m < NM; m++)
#pragma unroll
    for (int i = 0; i < PER; i++) {
      const int v = tid + i * NTHREADS, row = v >> 3, c = v & 7;
      val[m][i] = make_uint4(0, 0, 0, 0);
      if (row < T) val[m][i] = *(const uint4*)(src[m] + (long long)row * ld[m] + c * 8);
    }
#pragma unroll
  for (int m = 0; m < NM; m++)
#pragma unroll
    for (int i = 0; i < PER; i++) {
      const int v = tid + i * NTHREADS, row = v >> 3, c = v & 7;
      if (v < TP * 8) *(uint4*)(dst[m] + row * PITCH + ((c ^ swz(row)) << 4)) = val[m][i];
    }
}

// A- or B-operand fragment of rows [row0, row0+32) for reduction slice ks (16 of the 64 columns):
// lane l gets row row0 + l%32, columns ks*16 + (l/32)*8 .. +7
__device__ __forceinline__ bf16x8 frag_direct(const unsigned char* m, int row0, int ks, int lane) {
  const int row = row0 + (lane & 31);
  return *(const bf16x8*)(m + row * PITCH + (((ks * 2 + (lane >> 5)) ^ swz(row)) << 4));
}

// B-operand fragment for a reduction over ROWS of a matrix stored [row][64]: lane l gets column
// col0 + l%32 and the 8 rows  row0 + (e/4)*8 + (l/32)*4 + e%4  (e = 0..7)
__device__ __forceinline__ bf16x8 frag_rows_tr(const unsigned char* m, int row0, int col0, int lane) {
  const int g = lane >> 4, r16 = lane & 15;
  // (rows r and r + 8 differ in bit 3, which is bit 1 of swz: the second address is computed on its own)
  const int row = row0 + (g >> 1) * 4 + (r16 >> 2);
  const int byte = (col0 + (g & 1) * 16 + 4 * (r16 & 3)) * 2;      // 8-byte piece inside the logical row
  const int chunk = byte >> 4, half = byte & 8;
  const unsigned char* p = m + row * PITCH + ((chunk ^ swz(row)) << 4) + half;
  const unsigned char* p8 = m + (row + 8) * PITCH + ((chunk ^ swz(row + 8)) << 4) + half;
  const bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p8);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// element r of an MFMA result tile: row offset inside the 32x32 tile
__device__ __forceinline__ int tile_row(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }

// Store a 32 x 64 result tile (lane = row l%32, registers t[dt][a*4 + e] = column dt*32 + a*8 + (l/32)*4 + e), times
// `mul`, as bf16 rows of `ld` elements starting at `base` (row 0 of the tile), rows >= `rows` left out.  Straight
// from the registers a store instruction would put 16 bytes into each of 32 rows (8-byte pieces of two lanes);
// written that way the 19 MB of a ViT-B forward output cost 6 us.  The tile goes through a wave-private 4 KiB LDS
// area instead (16-byte chunks XORed with (row >> 1) & 7: even and odd rows lie in different halves of the 256-byte
// bank span, so 16 consecutive rows of one column are spread over all 64 banks) and
// leaves as whole 128-byte rows, 8 lanes x 16 bytes each.  LDS instructions of one wave execute in order, so no
// barrier is needed between the writes and the reads, nor between two tiles through the same area.
constexpr int STORE_AREA = 32 * 128;
__device__ __forceinline__ void store_tile(unsigned char* area, const f32x16 (&t)[2], float mul, bf16* base, long long ld,
                                           int rows, int lane) {
  asm volatile("" : "+v"(lane));   // (addresses below are computed here, not kept live through the caller's main loop)
  const int l32 = lane & 31, khalf = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < 2; dt++)
#pragma unroll
    for (int a = 0; a < 4; a++) {
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; e++) v[e] = (bf16)(t[dt][a * 4 + e] * mul);
      *(bf16x4*)(area + l32 * 128 + (((dt * 4 + a) ^ ((l32 >> 1) & 7)) << 4) + khalf * 8) = v;
    }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int row = i * 8 + (lane >> 3), chunk = lane & 7;
    const bf16x8 v = *(const bf16x8*)(area + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
    if (row < rows) *(bf16x8*)(base + row * ld + chunk * 8) = v;
  }
}

// -------------------------------------------------------------------------------------------------
// forward
// -------------------------------------------------------------------------------------------------
// One resident workgroup per CU walks over (batch, head) items.  K and V of an item are brought into one of two LDS
// buffers by direct-to-LDS loads (no registers), issued while the previous item is computed, so the memory latency
// of an item is paid once per workgroup, not once per item.  A lane's 16 bytes of a wave-wide direct load land at
// (base in M0) + 16 * lane: the bank swizzle is therefore applied on the global side (the lane at chunk position p
// of row r fetches chunk p ^ swz(r)).  Rows beyond the sequence repeat the last row: their keys are masked with
// -inf, and a probability of zero times a finite V row adds nothing.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}

template <int KT>
__global__ __launch_bounds__(NTHREADS) void attention_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ out,
                                                                 float* __restrict__ lse, int T, int H, float scale, int items) {
  constexpr int TP = KT * 32;
  constexpr int MAT = TP * PITCH;                       // one matrix: a multiple of 1 KiB
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * 2 * MAT + NWAVES * STORE_AREA];   // [buffer][K, V], store areas
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int D = H * DH;
  const long long ld = 3LL * D;
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  const int l32 = lane & 31, khalf = lane >> 5;
  // exp(scale * x) = 2^(c x): the scale is folded into the exponent, scores stay as the MFMA leaves them
  const float c = scale * 1.44269504088896341f;

  // the KT * 8 one-KiB pieces (8 rows each) of an item's K and V are dealt to the 8 waves, KT each
  // (lane-dependent address pieces come from an opaque copy of the thread index, so that they are recomputed per item
  // instead of staying in registers through the matrix products)
  auto issue = [&](int item, int buf) {
    int t_ = tid;
    asm volatile("" : "+v"(t_));
    const int lane = t_ & 63, wave = t_ >> 6;
    const int b = item / H, h = item % H;
    const bf16* kbase = qkv + (long long)b * T * ld + h * DH + D;
#pragma unroll
    for (int i = 0; i < KT; i++) {
      const int p = wave * KT + i, m = p / (KT * 4), rp = p % (KT * 4);
      const int row = rp * 8 + (lane >> 3), pos = lane & 7;
      const bf16* src = kbase + m * D + (long long)min(row, T - 1) * ld + ((pos ^ swz(row)) << 3);
      dma16(src, __builtin_amdgcn_readfirstlane(lds0 + (buf * 2 + m) * MAT + rp * 1024));
    }
  };
  // Q fragments of an item for this wave's query tile, straight from memory (B operand: row = query, 8 consecutive d)
  auto load_q = [&](int item, bf16x8 (&qf)[4]) {
    int t_ = tid;
    asm volatile("" : "+v"(t_));
    const int l32 = t_ & 31, khalf = (t_ >> 5) & 1, wave = t_ >> 6;
    const int b = item / H, h = item % H;
    const bf16* q = qkv + (long long)b * T * ld + h * DH;
    const int qrow = min(wave * 32 + l32, T - 1);
#pragma unroll
    for (int ks = 0; ks < 4; ks++) qf[ks] = *(const bf16x8*)(q + (long long)qrow * ld + ks * 16 + khalf * 8);
  };

  int item = blockIdx.x;
  if (item >= items) return;
  bf16x8 qf[4];
  load_q(item, qf);
  issue(item, 0);
  for (int buf = 0; item < items; item += gridDim.x, buf ^= 1) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's pieces of the item have landed
    asm volatile("s_barrier" ::: "memory");            // ... and everyone's; the other buffer is no longer read
    const int next = item + gridDim.x;
    if (next < items) issue(next, buf ^ 1);
    const unsigned char* sk = smem + (buf * 2) * MAT;
    const unsigned char* sv = sk + MAT;
    if (wave < KT) {
      const int qt = wave;
      const int b = item / H, h = item % H;
      // S^T tiles (unscaled), all kept in registers: lane holds query l%32 and keys kt*32 + tile_row(r)
      f32x16 st[KT];
#pragma unroll
      for (int kt = 0; kt < KT; kt++) {
#pragma unroll
        for (int r = 0; r < 16; r++) st[kt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ks++)
          st[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct(sk, kt * 32, ks, lane), qf[ks], st[kt], 0, 0, 0);
      }
      // (the Q fragments are no longer needed: their registers take the next item's, which arrive under the rest of
      // this item's work)
      if (next < items) load_q(next, qf);
      // only the last tile has keys beyond T
#pragma unroll
      for (int r = 0; r < 16; r++) st[KT - 1][r] = (KT - 1) * 32 + tile_row(r, lane) < T ? st[KT - 1][r] : -INFINITY;
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < KT; kt++)
#pragma unroll
        for (int r = 0; r < 16; r++) mx = fmaxf(mx, st[kt][r]);
      const float M = fmaxf(mx, __shfl_xor(mx, 32, 64));   // finite: key 0 is never masked
      const float mc = -M * c;

      // O^T = V^T exp(scale (S - M))^T with unnormalised probabilities, which are already an MFMA operand (query
      // l%32, 8 keys per lane); the result tile has lane = query as well, so the sum of a query's probabilities,
      // collected on the way, divides its own registers afterwards
      float sum = 0.f;
      f32x16 o[2];
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[dt][r] = 0.f;
#pragma unroll
      for (int kt = 0; kt < KT; kt++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
          bf16x8 pf;
#pragma unroll
          for (int e = 0; e < 8; e++) {
            const float p = __builtin_amdgcn_exp2f(fmaf(st[kt][j * 8 + e], c, mc));
            sum += p;
            pf[e] = (bf16)p;
          }
#pragma unroll
          for (int dt = 0; dt < 2; dt++)
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_tr(sv, kt * 32 + j * 16, dt * 32, lane), pf, o[dt], 0, 0, 0);
        }
      const float S = sum + __shfl_xor(sum, 32, 64);
      const float inv = 1.f / S;
      const int row = qt * 32 + l32;
      if (khalf == 0 && row < T) lse[((long long)b * H + h) * T + row] = M * scale + logf(S);
      // result tile: lane holds query l%32 and d = dt*32 + tile_row(r); it is a lane's own sum that divides its registers
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[dt][r] *= inv;
      store_tile(smem + 2 * 2 * MAT + wave * STORE_AREA, o, 1.f, out + ((long long)b * T + qt * 32) * D + h * DH, D, T - qt * 32, lane);
    }
    if (wave >= KT && next < items) load_q(next, qf);   // (a wave without a query tile: keeps the loop uniform)
  }
}

// -------------------------------------------------------------------------------------------------
// backward: dS = P * (dP - rowsum(P*dP)) / sqrt(d);  dQ = dS K,  dK = dS^T Q,  dV = P^T dO
// -------------------------------------------------------------------------------------------------
template <int KT>
__global__ __launch_bounds__(NTHREADS) void attention_bwd_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ out,
                                                            const bf16* __restrict__ dout, const float* __restrict__ lse,
                                                            bf16* __restrict__ dqkv, int T, int H, float scale) {
  constexpr int TP = KT * 32;
  __shared__ __attribute__((aligned(16))) unsigned char sq[TP * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned char sk[TP * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned char sv[TP * PITCH];
  __shared__ __attribute__((aligned(16))) unsigned char sdo[TP * PITCH];
  __shared__ __attribute__((aligned(16))) float s_lse[TP];
  __shared__ __attribute__((aligned(16))) float s_dot[TP];  // rowsum(P * dP) per query
  __shared__ __attribute__((aligned(16))) unsigned char s_store[NWAVES * STORE_AREA];   // per wave: rows on their way out
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int D = H * DH;
  const long long ld = 3LL * D;
  const bf16* q = qkv + (long long)b * T * ld + h * DH;
  {
    unsigned char* const dst[4] = {sq, sk, sv, sdo};
    const bf16* const src[4] = {q, q + D, q + 2 * D, dout + (long long)b * T * D + h * DH};
    const long long lds[4] = {ld, ld, ld, (long long)D};
    stage_rows<TP, 4>(dst, src, lds, T, tid);
  }
  // exp(scale * s - lse) = 2^(c s - lse log2(e)): both factors are folded in here; padded queries get
  // lse = +inf, so their probabilities vanish.  Padded keys need no mask: their K and V rows are zero, so they
  // add nothing to dQ, and their own dK / dV rows are never stored.
  const float c = scale * 1.44269504088896341f;
  for (int i = tid; i < TP; i += NTHREADS) s_lse[i] = i < T ? lse[((long long)b * H + h) * T + i] * 1.44269504088896341f : INFINITY;
  __syncthreads();

  const int l32 = lane & 31, khalf = lane >> 5;

  // ---- pass A: a wave owns 32 queries (one per lane pair).  rowsum(P * dP) of a query equals dO . O (O = P V is
  // the stored forward output), so it needs no sweep over the keys of its own; then dQ^T = K^T dS^T, whose
  // result tile has lane = query again (the factor 1/sqrt(d) of dS is applied once at the end)
  for (int qt = wave; qt < KT; qt += NWAVES) {
    bf16x8 qf[4], dof[4];
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      qf[ks] = frag_direct(sq, qt * 32, ks, lane);
      dof[ks] = frag_direct(sdo, qt * 32, ks, lane);
    }
    const float my_lse = s_lse[qt * 32 + l32];
    float dot = 0.f;
    {
      const int qrow = min(qt * 32 + l32, T - 1);
      const bf16* orow = out + ((long long)b * T + qrow) * D + h * DH;
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        const bf16x8 of = *(const bf16x8*)(orow + ks * 16 + khalf * 8);
#pragma unroll
        for (int e = 0; e < 8; e++) dot += (float)of[e] * (float)dof[ks][e];
      }
      dot += __shfl_xor(dot, 32, 64);
      if (khalf == 0) s_dot[qt * 32 + l32] = dot;
    }
    f32x16 dq[2];
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) dq[dt][r] = 0.f;
#pragma unroll 1
    for (int kt = 0; kt < KT; kt++) {
      f32x16 st, dp;
#pragma unroll
      for (int r = 0; r < 16; r++) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct(sk, kt * 32, ks, lane), qf[ks], st, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct(sv, kt * 32, ks, lane), dof[ks], dp, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < 2; j++) {
        bf16x8 dsf;
#pragma unroll
        for (int e = 0; e < 8; e++) {
          const int r = j * 8 + e;
          const float p = __builtin_amdgcn_exp2f(fmaf(st[r], c, -my_lse));
          dsf[e] = (bf16)(p * (dp[r] - dot));
        }
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_tr(sk, kt * 32 + j * 16, dt * 32, lane), dsf, dq[dt], 0, 0, 0);
      }
    }
    store_tile(s_store + wave * STORE_AREA, dq, scale, dqkv + ((long long)b * T + qt * 32) * ld + h * DH, ld, T - qt * 32, lane);
  }
  __syncthreads();

  // ---- pass B: a wave owns 32 keys (one per lane pair): S = Q K^T tiles with lane = key; dV^T = dO^T P and
  // dK^T = Q^T dS keep lane = key in their result tiles
  for (int kt = wave; kt < KT; kt += NWAVES) {
    bf16x8 kf[4], vf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      kf[ks] = frag_direct(sk, kt * 32, ks, lane);
      vf[ks] = frag_direct(sv, kt * 32, ks, lane);
    }
    f32x16 dk[2], dv[2];
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }
#pragma unroll 1
    for (int qt = 0; qt < KT; qt++) {
      f32x16 st, dp;
#pragma unroll
      for (int r = 0; r < 16; r++) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct(sq, qt * 32, ks, lane), kf[ks], st, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_direct(sdo, qt * 32, ks, lane), vf[ks], dp, 0, 0, 0);
      }
      // rows of the tile are queries qt*32 + tile_row(r): their lse / dot come in groups of 4
      float pr[16], ds[16];
#pragma unroll
      for (int a = 0; a < 4; a++) {
        const float4 l4 = *(const float4*)(s_lse + qt * 32 + a * 8 + khalf * 4);
        const float4 d4 = *(const float4*)(s_dot + qt * 32 + a * 8 + khalf * 4);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const int r = a * 4 + e;
          const float p = __builtin_amdgcn_exp2f(fmaf(st[r], c, -lv[e]));
          pr[r] = p;
          ds[r] = p * (dp[r] - dv4[e]);
        }
      }
#pragma unroll
      for (int j = 0; j < 2; j++) {
        bf16x8 pf, dsf;
#pragma unroll
        for (int e = 0; e < 8; e++) { pf[e] = (bf16)pr[j * 8 + e]; dsf[e] = (bf16)ds[j * 8 + e]; }
#pragma unroll
        for (int dt = 0; dt < 2; dt++) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_tr(sdo, qt * 32 + j * 16, dt * 32, lane), pf, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows_tr(sq, qt * 32 + j * 16, dt * 32, lane), dsf, dk[dt], 0, 0, 0);
        }
      }
    }
    bf16* drow0 = dqkv + ((long long)b * T + kt * 32) * ld + h * DH;
    store_tile(s_store + wave * STORE_AREA, dk, scale, drow0 + D, ld, T - kt * 32, lane);
    store_tile(s_store + wave * STORE_AREA, dv, 1.f, drow0 + 2 * D, ld, T - kt * 32, lane);
  }
}

template <int KT>
hipError_t launch_fwd(const bf16* qkv, bf16* out, float* lse, int B, int T, int H, float scale, hipStream_t s) {
  // one resident workgroup per CU (two LDS buffers of K and V each); fewer when there are fewer items
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  const int items = B * H;
  hipLaunchKernelGGL((attention_fwd_kernel<KT>), dim3(items < cus ? items : cus), dim3(NTHREADS), 0, s, qkv, out, lse, T, H, scale, items);
  return hipGetLastError();
}
template <int KT>
hipError_t launch_bwd(const bf16* qkv, const bf16* out, const bf16* dout, const float* lse, bf16* dqkv, int B, int T, int H,
                      float scale, hipStream_t s) {
  hipLaunchKernelGGL((attention_bwd_kernel<KT>), dim3(B * H), dim3(NTHREADS), 0, s, qkv, out, dout, lse, dqkv, T, H, scale);
  return hipGetLastError();
}

}  // namespace

bool attention_fused_supported(int T, int head_dim) { return head_dim == DH && T >= 1 && T <= 224; }

hipError_t attention_fwd(const bf16* qkv, bf16* out, float* lse, int B, int T, int H, int head_dim, float scale,
                         hipStream_t s) {
  if (!attention_fused_supported(T, head_dim) || B < 1 || H < 1) return hipErrorInvalidValue;
  switch ((T + 31) / 32) {
    case 1: return launch_fwd<1>(qkv, out, lse, B, T, H, scale, s);
    case 2: return launch_fwd<2>(qkv, out, lse, B, T, H, scale, s);
    case 3: return launch_fwd<3>(qkv, out, lse, B, T, H, scale, s);
    case 4: return launch_fwd<4>(qkv, out, lse, B, T, H, scale, s);
    case 5: return launch_fwd<5>(qkv, out, lse, B, T, H, scale, s);
    case 6: return launch_fwd<6>(qkv, out, lse, B, T, H, scale, s);
    default: return launch_fwd<7>(qkv, out, lse, B, T, H, scale, s);
  }
}

hipError_t attention_bwd(const bf16* qkv, const bf16* out, const bf16* dout, const float* lse, bf16* dqkv, int B, int T, int H,
                         int head_dim, float scale, hipStream_t s) {
  if (!attention_fused_supported(T, head_dim) || B < 1 || H < 1 || !out) return hipErrorInvalidValue;
  switch ((T + 31) / 32) {
    case 1: return launch_bwd<1>(qkv, out, dout, lse, dqkv, B, T, H, scale, s);
    case 2: return launch_bwd<2>(qkv, out, dout, lse, dqkv, B, T, H, scale, s);
    case 3: return launch_bwd<3>(qkv, out, dout, lse, dqkv, B, T, H, scale, s);
    case 4: return launch_bwd<4>(qkv, out, dout, lse, dqkv, B, T, H, scale, s);
    case 5: return launch_bwd<5>(qkv, out, dout, lse, dqkv, B, T, H, scale, s);
    case 6: return launch_bwd<6>(qkv, out, dout, lse, dqkv, B, T, H, scale, s);
    default: return launch_bwd<7>(qkv, out, dout, lse, dqkv, B, T, H, scale, s);
  }
}

}  // namespace et
