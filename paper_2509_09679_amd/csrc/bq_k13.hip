// n = 8192 instantiations of the specialised transform kernels (1024 threads, both halves of a row side by side).
#include "bq_k12_kernel.h"

namespace bq {

hipError_t launch_k13_dtype(Mode mode, const K12Args &A, int bits, unsigned grid, int dtype, hipStream_t stream)
{
    return launch_k12_dtype<false, true>(mode, A, bits, grid, dtype, stream);
}

}  // namespace bq
