// Instantiations of the band kernel of small-channel layers (16-bit operands, float accumulate).
#include "bandrow_kernel.hpp"

namespace sc {

RowBandLaunchFn bandrow_kernel_for(int dtype, int mi) {
  if (dtype == kBF16) return mi == 1 ? bandrow_launch<kBF16, 1> : mi == 2 ? bandrow_launch<kBF16, 2> : nullptr;
  if (dtype == kF16) return mi == 1 ? bandrow_launch<kF16, 1> : mi == 2 ? bandrow_launch<kF16, 2> : nullptr;
  return nullptr;
}

}  // namespace sc
