// Instantiations of the bf16 GEMM kernels for one tile shape (see gemm_bf16_kernels.h).
#include "gemm_bf16_kernels.h"

namespace et {
namespace gemm {
namespace {

template <bool AT, bool BT, int E>
hipError_t launch(const Params& p, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((gemm_staged_kernel<128, 128, 2, 2, AT, BT, E>), grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace

LaunchFn staged_128x128(bool a_t, bool b_t, int epi) {
#define ET_PICK(AT, BT, E) \
  if (a_t == AT && b_t == BT && epi == E) return launch<AT, BT, E>;
  ET_PICK(false, false, E_F32)
  ET_PICK(false, false, E_F32_RES)
  ET_PICK(false, false, E_PARTIAL)
  ET_PICK(false, false, E_BF16)
  ET_PICK(false, false, E_GELU_FWD)
  ET_PICK(false, false, E_GELU_ONLY)
  ET_PICK(false, false, E_BIAS_RELU)
  ET_PICK(false, false, E_AFFINE)
  ET_PICK(false, false, E_AFFINE_ADD)
  ET_PICK(false, true, E_F32)
  ET_PICK(false, true, E_BF16)
  ET_PICK(false, true, E_GELU_BWD)
  ET_PICK(true, true, E_F32)
  ET_PICK(true, true, E_BF16)
  ET_PICK(true, true, E_PARTIAL)
#undef ET_PICK
  return nullptr;
}

}  // namespace gemm
}  // namespace et
