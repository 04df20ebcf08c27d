// Instantiations of the buffer-load tiled kernel (16-bit operands, float accumulate).
#include "igemm_buf_kernel.hpp"

namespace sc {

// ring of two tiles for layers with at most two K tiles (less LDS, more workgroups per CU)
template <int DT>
static LaunchFn pick_shallow(int bm, int bn) {
  if (bm == 128 && bn == 64) return igemm_buf_launch<DT, 128, 64, 2, 2, 2>;
  if (bm == 96 && bn == 128) return igemm_buf_launch<DT, 96, 128, 1, 4, 2>;
  if (bm == 64 && bn == 128) return igemm_buf_launch<DT, 64, 128, 2, 2, 2>;
  if (bm == 64 && bn == 64) return igemm_buf_launch<DT, 64, 64, 2, 2, 2>;
  if (bm == 128 && bn == 32) return igemm_buf_launch<DT, 128, 32, 4, 1, 2>;
  if (bm == 32 && bn == 128) return igemm_buf_launch<DT, 32, 128, 1, 4, 2>;
  return nullptr;
}

template <int DT>
static LaunchFn pick(int bm, int bn) {
  if (bm == 256 && bn == 128) return igemm_buf_launch<DT, 256, 128, 4, 2, 3>;   // eight wavefronts
  if (bm == 128 && bn == 256) return igemm_buf_launch<DT, 128, 256, 2, 4, 3>;   // eight wavefronts
  if (bm == 128 && bn == 128) return igemm_buf_launch<DT, 128, 128, 2, 4, 3>;   // eight wavefronts
  if (bm == 128 && bn == 64) return igemm_buf_launch<DT, 128, 64, 2, 2, 3>;
  if (bm == 96 && bn == 128) return igemm_buf_launch<DT, 96, 128, 1, 4, 3>;
  if (bm == 64 && bn == 128) return igemm_buf_launch<DT, 64, 128, 2, 2, 3>;
  if (bm == 64 && bn == 64) return igemm_buf_launch<DT, 64, 64, 2, 2, 3>;
  if (bm == 128 && bn == 32) return igemm_buf_launch<DT, 128, 32, 4, 1, 3>;
  if (bm == 32 && bn == 128) return igemm_buf_launch<DT, 32, 128, 1, 4, 3>;
  return nullptr;
}

template <int DT>
static LaunchFn pick_splitk(int bm, int bn) {
  if (bm == 256 && bn == 128) return igemm_buf_launch<DT, 256, 128, 4, 2, 3, true>;
  if (bm == 128 && bn == 256) return igemm_buf_launch<DT, 128, 256, 2, 4, 3, true>;
  if (bm == 128 && bn == 128) return igemm_buf_launch<DT, 128, 128, 2, 4, 3, true>;
  if (bm == 96 && bn == 128) return igemm_buf_launch<DT, 96, 128, 1, 4, 3, true>;
  if (bm == 64 && bn == 128) return igemm_buf_launch<DT, 64, 128, 2, 2, 3, true>;
  return nullptr;
}

LaunchFn buf_splitk_kernel(int dtype, int bm, int bn) {
  if (dtype == kBF16) return pick_splitk<kBF16>(bm, bn);
  if (dtype == kF16) return pick_splitk<kF16>(bm, bn);
  return nullptr;
}

LaunchFn buf_kernel(int dtype, int bm, int bn, bool shallow) {
  if (dtype == kBF16) return shallow ? pick_shallow<kBF16>(bm, bn) : pick<kBF16>(bm, bn);
  if (dtype == kF16) return shallow ? pick_shallow<kF16>(bm, bn) : pick<kF16>(bm, bn);
  return nullptr;
}

}  // namespace sc
