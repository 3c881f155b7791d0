// Instantiations of the two-group bf16 GEMM kernel for one tile shape (see gemm_bf16_kernels.h):
// the plain product and the implicit 3x3 convolution (forward / gradient passing, weight gradient).
#include "gemm_bf16_kernels.h"

namespace et {
namespace gemm {
namespace {

template <bool AT, bool BT, int E, int CONV>
hipError_t launch(const Params& p, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((gemm_pp_kernel<256, 256, 2, 4, AT, BT, E, CONV>), grid, dim3(512), 0, s, p);
  return hipGetLastError();
}

}  // namespace

LaunchFn pp_conv_256x256(int epi) {
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

LaunchFn pp_convdw_256x256(int epi) {
  if (epi == E_F32) return launch<true, true, E_F32, 2>;
  if (epi == E_PARTIAL) return launch<true, true, E_PARTIAL, 2>;
  return nullptr;
}

}  // namespace gemm
}  // namespace et
