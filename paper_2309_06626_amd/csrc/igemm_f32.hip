// Instantiations of the fused masked-convolution kernel for f32 operands (float accumulate).
#include "band_kernel.hpp"
#include "igemm_kernel.hpp"

namespace sc {

static const KernelEntry g_table[] = {
    SC_KERNEL_ENTRY(kF32, 256, 128, 2, 2, 2, 3),
    SC_KERNEL_ENTRY(kF32, 128, 256, 2, 2, 2, 3),
    SC_KERNEL_ENTRY(kF32, 128, 128, 2, 2, 3, 3),
    SC_KERNEL_ENTRY(kF32, 256, 64, 4, 1, 2, 3),
    SC_KERNEL_ENTRY(kF32, 128, 64, 2, 2, 4, 3),
    SC_KERNEL_ENTRY(kF32, 64, 128, 2, 2, 4, 3),
    SC_KERNEL_ENTRY(kF32, 64, 64, 2, 2, 4, 3),
    SC_KERNEL_ENTRY(kF32, 96, 128, 1, 4, 2, 3),
    SC_KERNEL_ENTRY(kF32, 128, 32, 4, 1, 4, 3),
    SC_KERNEL_ENTRY(kF32, 32, 128, 1, 4, 4, 3),
};

const KernelEntry* kernels_f32(int* count) {
  *count = (int)(sizeof(g_table) / sizeof(g_table[0]));
  return g_table;
}

static const BandTable g_band = SC_BAND_TABLE(kF32);
const BandTable* band_f32() { return &g_band; }

}  // namespace sc
