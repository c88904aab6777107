// Dispatch of the slice-product kernel (product_kernel.h) by mode; the modes are compiled in
// translation units of their own (gemm_real.hip, gemm_dd.hip, gemm_complex.hip) so that they build in parallel.
#include "ozimmu_internal.h"

namespace ozimmu {

hipError_t launch_product_real(const GemmArgs& g, int s, hipStream_t st);
hipError_t launch_product_dd(const GemmArgs& g, int s, hipStream_t st);
hipError_t launch_product_complex(const GemmArgs& g, int s, hipStream_t st);

hipError_t launch_slice_gemm(const GemmArgs& args, int s, int mode, hipStream_t st) {
    if (args.tiles_m * args.tiles_n == 0 || args.t_end <= args.t_begin) return hipSuccess;
    switch (mode) {
        case 0: return launch_product_real(args, s, st);
        case 1: return launch_product_dd(args, s, st);
        case 2: return args.block_steps == 0 ? launch_product_complex(args, s, st) : hipErrorInvalidValue;
    }
    return hipErrorInvalidValue;
}

}  // namespace ozimmu
