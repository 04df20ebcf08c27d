// Instantiations of the slab form of the tiled kernel (16-bit operands, float accumulate).
#include "igemm_slab_kernel.hpp"

namespace sc {

template <int DT>
static LaunchFn pick_slab(int bm, bool splitk) {
  if (bm == 256) return splitk ? igemm_slab_launch<DT, 256, 4, 2, true> : igemm_slab_launch<DT, 256, 4, 2, false>;   // eight wavefronts
  if (bm == 128) return splitk ? igemm_slab_launch<DT, 128, 2, 2, true> : igemm_slab_launch<DT, 128, 2, 2, false>;
  return nullptr;
}

LaunchFn slab_kernel(int dtype, int bm, bool splitk) {
  if (dtype == kBF16) return pick_slab<kBF16>(bm, splitk);
  if (dtype == kF16) return pick_slab<kF16>(bm, splitk);
  return nullptr;
}

}  // namespace sc
