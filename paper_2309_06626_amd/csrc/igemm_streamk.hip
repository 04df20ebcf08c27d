// Instantiations of the stream-K tiled kernel (16-bit operands, float accumulate).
#include "igemm_streamk_kernel.hpp"

namespace sc {

template <int DT>
static LaunchFn pick_streamk(int bm, int bn) {
  if (bm == 128 && bn == 128) return igemm_streamk_launch<DT, 128, 128, 2, 2, 3>;
  if (bm == 64 && bn == 128) return igemm_streamk_launch<DT, 64, 128, 2, 2, 3>;
  if (bm == 128 && bn == 64) return igemm_streamk_launch<DT, 128, 64, 2, 2, 3>;
  if (bm == 64 && bn == 64) return igemm_streamk_launch<DT, 64, 64, 2, 2, 3>;
  return nullptr;
}

LaunchFn streamk_kernel(int dtype, int bm, int bn) {
  if (dtype == kBF16) return pick_streamk<kBF16>(bm, bn);
  if (dtype == kF16) return pick_streamk<kF16>(bm, bn);
  return nullptr;
}

}  // namespace sc
