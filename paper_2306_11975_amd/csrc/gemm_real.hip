// The slice-product kernel for one mode (real product, FP64 sum).
#include "product_kernel.h"

namespace ozimmu {

hipError_t launch_product_real(const GemmArgs& g, int s, hipStream_t st) { return launch_product_mode<kModeReal>(g, s, st); }

}  // namespace ozimmu
