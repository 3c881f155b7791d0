// Instantiations of the two-group bf16 GEMM kernel for one tile shape (see gemm_bf16_kernels.h):
// the plain product and the implicit 3x3 convolution (forward / gradient passing, weight gradient).
#include "gemm_bf16_kernels.h"

namespace et {
namespace gemm {
namespace {

template <bool AT, bool BT, int E, int CONV, bool GEN = false>
hipError_t launch(const Params& p, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((gemm_pp_kernel<128, 256, 2, 4, AT, BT, E, CONV, GEN>), grid, dim3(512), 0, s, p);
  return hipGetLastError();
}

}  // namespace

LaunchFn pp_128x256(bool a_t, bool b_t, int epi) {
#define ET_PICK(AT, BT, E) \
  if (a_t == AT && b_t == BT && epi == E) return launch<AT, BT, E, 0>;
  ET_PICK(true, true, E_F32)
  ET_PICK(true, true, E_BF16)
  ET_PICK(true, true, E_PARTIAL)
#undef ET_PICK
  return nullptr;
}

LaunchFn pp_convdw_128x256(int epi, bool general) {
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
