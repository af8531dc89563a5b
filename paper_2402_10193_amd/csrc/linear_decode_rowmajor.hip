// The decode kernel instantiated for the row-major tensors of bd_linear_multitenant (see linear_decode_tiled_kernel.h).
#include "linear_decode_tiled_kernel.h"

namespace bd {

hipError_t launch_linear_decode_rowmajor(const TiledArgs& args, int n_jobs, hipStream_t st) {
    return launch_tiled_t<false, true>(args, n_jobs, st);
}

}  // namespace bd
