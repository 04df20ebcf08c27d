// Instantiations of the fused masked-convolution kernel for f16 operands (float accumulate).
#include "band_kernel.hpp"
#include "bandstream_kernel.hpp"
#include "igemm_kernel.hpp"

namespace sc {

static const KernelEntry g_table[] = {
    SC_KERNEL_ENTRY(kF16, 256, 128, 2, 2, 2, 3),
    SC_KERNEL_ENTRY(kF16, 128, 256, 2, 2, 2, 3),
    SC_KERNEL_ENTRY_SPLITK(kF16, 128, 128, 2, 2, 3, 3, 4),
    SC_KERNEL_ENTRY(kF16, 256, 64, 4, 1, 2, 3),
    SC_KERNEL_ENTRY_SPLITK(kF16, 128, 64, 2, 2, 4, 3, 6),
    SC_KERNEL_ENTRY_SPLITK(kF16, 64, 128, 2, 2, 4, 3, 6),
    SC_KERNEL_ENTRY_SPLITK(kF16, 64, 64, 2, 2, 4, 3, 8),
    SC_KERNEL_ENTRY(kF16, 96, 128, 1, 4, 2, 3),
    SC_KERNEL_ENTRY(kF16, 128, 32, 4, 1, 4, 3),
    SC_KERNEL_ENTRY(kF16, 32, 128, 1, 4, 4, 3),
};

const KernelEntry* kernels_f16(int* count) {
  *count = (int)(sizeof(g_table) / sizeof(g_table[0]));
  return g_table;
}

static const BandTable g_band = SC_BAND_TABLE(kF16);
const BandTable* band_f16() { return &g_band; }
static const BandStreamTable g_stream = SC_BANDSTREAM_TABLE(kF16);
const BandStreamTable* bandstream_f16() { return &g_stream; }

}  // namespace sc
