// Instantiations of the two-group bf16 GEMM kernel for one tile shape (see gemm_bf16_kernels.h):
// the plain product and the implicit 3x3 convolution (forward / gradient passing, weight gradient).
#include "gemm_bf16_kernels.h"

namespace et {
namespace gemm {
namespace {

template <bool AT, bool BT, int E, int CONV, bool GEN = false>
hipError_t launch(const Params& p, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((gemm_pp_kernel<512, 64, 8, 1, AT, BT, E, CONV, GEN>), grid, dim3(512), 0, s, p);
  return hipGetLastError();
}

}  // namespace

LaunchFn pp_512x64(bool a_t, bool b_t, int epi) {
#define ET_PICK(AT, BT, E) \
  if (a_t == AT && b_t == BT && epi == E) return launch<AT, BT, E, 0>;
  ET_PICK(false, false, E_F32)
  ET_PICK(false, false, E_F32_RES)
  ET_PICK(false, false, E_BF16)
  ET_PICK(false, false, E_BIAS_RELU)
  ET_PICK(false, false, E_AFFINE)
  ET_PICK(false, false, E_AFFINE_ADD)
  ET_PICK(false, true, E_F32)
  ET_PICK(false, true, E_BF16)
  ET_PICK(true, true, E_F32)
  ET_PICK(true, true, E_BF16)
  ET_PICK(true, true, E_PARTIAL)
#undef ET_PICK
  return nullptr;
}

LaunchFn pp_conv_512x64(int epi, bool general) {
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

}  // namespace gemm
}  // namespace et
