// Down projection, per-block-regime kernels with two weight blocks per wavefront
// (tile_kernel_mixed<2, ...>).  A translation unit of its own: these are the largest kernels of
// the library and compile in parallel with the rest.
#include "ffn_kernels.hpp"

namespace moe {

hipError_t launch_down_mixed_wide_nt(const GemmArgs& a, int max_blocks, hipStream_t s) {
    return launch_tile_mixed<2, false, true, true>(a, max_blocks, s);
}

hipError_t launch_down_mixed_wide(const GemmArgs& a, int max_blocks, hipStream_t s) {
    return launch_tile_mixed<2, false, true, false>(a, max_blocks, s);
}

}  // namespace moe
