// Instantiations of the tap-pipelined band kernel (16-bit operands, float accumulate).
#include "bandtap_kernel.hpp"

namespace sc {

static const BandTapTable g_tap_bf16 = SC_BANDTAP_TABLE(kBF16);
const BandTapTable* bandtap_bf16() { return &g_tap_bf16; }
static const BandTapTable g_tap_f16 = SC_BANDTAP_TABLE(kF16);
const BandTapTable* bandtap_f16() { return &g_tap_f16; }

}  // namespace sc
