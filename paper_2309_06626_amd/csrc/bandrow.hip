// Instantiations of the band kernel of small-channel layers (16-bit operands, float accumulate).
#include "bandrow_kernel.hpp"

namespace sc {

template <int DT>
static RowBandLaunchFn pick(int mi, int kh, int gpw) {
  if (mi != 1 && mi != 2) return nullptr;
  // the 7x7 window of three channels (ResNet stems): 21 groups, unrolled
  if (kh == 7 && gpw == 3) return mi == 1 ? bandrow_launch<DT, 1, 7, 3> : bandrow_launch<DT, 2, 7, 3>;
  return mi == 1 ? bandrow_launch<DT, 1, 0, 0> : bandrow_launch<DT, 2, 0, 0>;
}

RowBandLaunchFn bandrow_kernel_for(int dtype, int mi, int kh, int gpw) {
  if (dtype == kBF16) return pick<kBF16>(mi, kh, gpw);
  if (dtype == kF16) return pick<kF16>(mi, kh, gpw);
  return nullptr;
}

}  // namespace sc
