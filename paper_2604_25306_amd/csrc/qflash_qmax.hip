// The quantised-maximum variant of the forward pass (NOT Algorithm 1 as printed: the reference level
// of the integer softmax is the running maximum rounded up to a whole octave, so that past
// accumulators are rescaled by exact shifts; see process_tile).  Same kernels, same launch
// geometry, instantiated with QMAX in a translation unit of their own.
#include "qflash_resident.h"

int qflash_launch_fwd_qmax(const QflashKernelArgs& a, int d, int kv_tile, size_t lds, int lds_limit, int threads, void* stream) {
    return launch_shape<true>(a, d, kv_tile, lds, lds_limit, threads, (hipStream_t)stream);
}
