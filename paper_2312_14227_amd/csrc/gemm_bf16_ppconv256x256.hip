// Instantiations of the two-group bf16 GEMM kernel for one tile shape (see gemm_bf16_kernels.h):
// the plain product and the implicit 3x3 convolution (forward / gradient passing, weight gradient).
#include "gemm_bf16_kernels.h"

namespace et {
namespace gemm {
namespace {

template <bool AT, bool BT, int E, int CONV, bool GEN = false>
hipError_t launch(const Params& p, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((gemm_pp_kernel<256, 256, 2, 4, AT, BT, E, CONV, GEN>), grid, dim3(512), 0, s, p);
  return hipGetLastError();
}

}  // namespace

LaunchFn pp_conv_256x256(int epi, bool general) {
  // (general: stride 2, 1x1 taps or the stem form, geometry from the launch arguments; the epilogues those layers use)
  if (general) {
    if (epi == E_BF16) return launch<false, false, E_BF16, 1, true>;
    if (epi == E_F32) return launch<false, false, E_F32, 1, true>;
    if (epi == E_AFFINE) return launch<false, false, E_AFFINE, 1, true>;
    if (epi == E_PARTIAL) return launch<false, false, E_PARTIAL, 1, true>;
    return nullptr;
  }
#define ET_PICK(E) \
  if (epi == E) return launch<false, false, E, 1>;
  ET_PICK(E_BF16)
  ET_PICK(E_BIAS_RELU)
  ET_PICK(E_AFFINE)
  ET_PICK(E_RELU_MASK)
  ET_PICK(E_PARTIAL)
#undef ET_PICK
  return nullptr;
}

LaunchFn pp_convdw_256x256(int epi, bool general) {
  if (general) {
    if (epi == E_F32) return launch<true, true, E_F32, 2, true>;
    if (epi == E_PARTIAL) return launch<true, true, E_PARTIAL, 2, true>;
    return nullptr;
  }
  if (epi == E_F32) return launch<true, true, E_F32, 2>;
  if (epi == E_PARTIAL) return launch<true, true, E_PARTIAL, 2>;
  return nullptr;
}

}  // namespace gemm
}  // namespace et
