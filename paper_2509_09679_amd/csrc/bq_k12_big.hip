// Instantiations of the specialised transform kernels for quantiser groups of more than 128 channels, up to one
// scale per row (per-token quantisation): n = 256 .. 8192.
#include "bq_k12_kernel.h"

namespace bq {

hipError_t launch_k12_big_dtype(Mode mode, const K12Args &A, int bits, unsigned grid, int dtype, bool virt, bool wide,
                                hipStream_t stream)
{
    if (wide) return launch_k12_dtype<false, true, true>(mode, A, bits, grid, dtype, stream);
    if (virt) return launch_k12_dtype<true, false, true>(mode, A, bits, grid, dtype, stream);
    return launch_k12_dtype<false, false, true>(mode, A, bits, grid, dtype, stream);
}

}  // namespace bq
