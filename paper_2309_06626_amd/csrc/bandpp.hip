// Instantiations of the alternating-group band kernel (16-bit operands, float accumulate).
#include "bandpp_kernel.hpp"

namespace sc {

static const BandPPTable g_pp_bf16 = SC_BANDPP_TABLE(kBF16);
const BandPPTable* bandpp_bf16() { return &g_pp_bf16; }
static const BandPPTable g_pp_f16 = SC_BANDPP_TABLE(kF16);
const BandPPTable* bandpp_f16() { return &g_pp_f16; }

}  // namespace sc
