// The slice-product kernel for one mode (real product, double-double sum).
#include "product_kernel.h"

namespace ozimmu {

hipError_t launch_product_dd(const GemmArgs& g, int s, hipStream_t st) { return launch_product_mode<kModeDD>(g, s, st); }

}  // namespace ozimmu
