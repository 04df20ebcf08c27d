// Instantiations of the register-staged tiled kernel with the window-row-segment gather (small-channel
// NHWC layers of 16-bit types, e.g. a 3-channel stem).
#include "igemm_kernel.hpp"

namespace sc {

template <int DT>
static LaunchFn pick(int bm, int bn) {
  if (bm == 128 && bn == 64) return igemm_launch<DT, 128, 64, 2, 2, 2, 4>;
  if (bm == 64 && bn == 128) return igemm_launch<DT, 64, 128, 2, 2, 2, 4>;
  if (bm == 64 && bn == 64) return igemm_launch<DT, 64, 64, 2, 2, 2, 4>;
  if (bm == 128 && bn == 32) return igemm_launch<DT, 128, 32, 4, 1, 2, 4>;
  if (bm == 32 && bn == 128) return igemm_launch<DT, 32, 128, 1, 4, 2, 4>;
  return nullptr;
}

LaunchFn rowseg_kernel(int dtype, int bm, int bn) {
  if (dtype == kBF16) return pick<kBF16>(bm, bn);
  if (dtype == kF16) return pick<kF16>(bm, bn);
  return nullptr;
}

}  // namespace sc
