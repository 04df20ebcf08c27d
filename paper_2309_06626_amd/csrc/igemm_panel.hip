// Instantiations of the row-panel kernel (16-bit operands, float accumulate).
#include "igemm_panel_kernel.hpp"

namespace sc {

LaunchFn panel_bf16() { return igemm_panel_launch<kBF16, kPanelBM, kPanelBN, 2, 2>; }
LaunchFn panel_f16() { return igemm_panel_launch<kF16, kPanelBM, kPanelBN, 2, 2>; }

}  // namespace sc
