// The decode kernel instantiated for the row-major 8-bit base of bd_linear_multitenant_q8 (see linear_decode_tiled_kernel.h).
#include "linear_decode_tiled_kernel.h"

namespace bd {

hipError_t launch_linear_decode_rowmajor_q8(const TiledArgs& args, int n_jobs, hipStream_t st) {
    return launch_tiled_t<true, true>(args, n_jobs, st);
}

}  // namespace bd
