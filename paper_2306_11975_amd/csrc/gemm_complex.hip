// The slice-product kernel for one mode (the four real products of a complex one per workgroup).
#include "product_kernel.h"

namespace ozimmu {

hipError_t launch_product_complex(const GemmArgs& g, int s, hipStream_t st) { return launch_product_mode<kModeComplex>(g, s, st); }

}  // namespace ozimmu
