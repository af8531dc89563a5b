// The tiled decode kernel instantiated for the fp16 base (see linear_decode_tiled_kernel.h).
#include "linear_decode_tiled_kernel.h"

namespace bd {

hipError_t launch_linear_decode_tiled(const TiledArgs& args, int n_jobs, hipStream_t st) {
    return launch_tiled_t<false>(args, n_jobs, st);
}

}  // namespace bd
