// Measurement helpers (not part of the method): a plain streaming copy and a float32 FMA issue-rate loop, so
// that a benchmark can quote what this GPU delivers for the two roofs next to the published peaks.
#include "bq_internal.h"

namespace bq {

// 16 bytes per lane and access, persistent grid, everything coalesced
__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t count)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) dst[i] = src[i];
}

// The read side alone: every lane XORs what it loads and stores the result once at the end (16 bytes per thread).
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ sink, size_t count)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
        const uint4 v = src[i];
        acc.x ^= v.x;
        acc.y ^= v.y;
        acc.z ^= v.z;
        acc.w ^= v.w;
    }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

// Persistent grids of the two streaming probes, swept on 2 GiB (256 threads per workgroup): the copy is fastest with
// three workgroups per compute unit (768: 5.55 TB/s; 1024 and 1280 alike, 2048 and more 4.5 .. 4.7, 512 4.9), the read
// with eight (2048: 6.45 TB/s; 1024: 6.3).
constexpr unsigned kProbeCopyGrid = 768, kProbeReadGrid = 2048;

constexpr int kProbeChains = 16;  // independent accumulators per lane: no FMA waits for another

// Every lane runs kProbeChains independent chains of `iters` float32 FMAs (plain v_fma_f32 / v_fmac_f32: this
// library is compiled without packed float32 instructions).  The sum of the chains is stored so that nothing
// is optimised away.
__global__ __launch_bounds__(256) void probe_fma_kernel(float *out, int iters, float a, float b)
{
    float acc[kProbeChains];
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c) acc[c] = (float)(threadIdx.x + c);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kProbeChains; ++c) acc[c] = __builtin_fmaf(acc[c], a, b);
    }
    float sum = 0.0f;
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c) sum += acc[c];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

constexpr int kProbeFmaBlocks = 4096, kProbeFmaThreads = 256;

}  // namespace bq

extern "C" {

bq_status bq_probe_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return BQ_ERR_NULL;
    if (((uintptr_t)src & 15) || ((uintptr_t)dst & 15) || (bytes & 15)) return BQ_ERR_ALIGN;
    if (bytes == 0) return BQ_OK;
    const size_t count = bytes / 16;
    const size_t want = (count + 255) / 256;
    const unsigned grid = (unsigned)(want < bq::kProbeCopyGrid ? want : bq::kProbeCopyGrid);
    hipLaunchKernelGGL(bq::probe_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst, count);
    return hipGetLastError() == hipSuccess ? BQ_OK : BQ_ERR_HIP;
}

size_t bq_probe_read_sink_bytes(void) { return (size_t)bq::kProbeReadGrid * 256 * 16; }

bq_status bq_probe_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (!src || !sink) return BQ_ERR_NULL;
    if (((uintptr_t)src & 15) || ((uintptr_t)sink & 15) || (bytes & 15)) return BQ_ERR_ALIGN;
    // every thread of the fixed grid stores its 16 bytes, whatever the size
    hipLaunchKernelGGL(bq::probe_read_kernel, dim3(bq::kProbeReadGrid), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src,
                       (uint4 *)sink, bytes / 16);
    return hipGetLastError() == hipSuccess ? BQ_OK : BQ_ERR_HIP;
}

size_t bq_probe_fma_out_floats(void) { return (size_t)bq::kProbeFmaBlocks * bq::kProbeFmaThreads; }

int64_t bq_probe_fma(float *out, int32_t iters, void *stream)
{
    if (!out || iters < 1) return -1;
    hipLaunchKernelGGL(bq::probe_fma_kernel, dim3(bq::kProbeFmaBlocks), dim3(bq::kProbeFmaThreads), 0, (hipStream_t)stream, out,
                       (int)iters, 0.999f, 0.001f);
    if (hipGetLastError() != hipSuccess) return -1;
    return (int64_t)bq::kProbeFmaBlocks * bq::kProbeFmaThreads * bq::kProbeChains * (int64_t)iters;
}

}  // extern "C"
