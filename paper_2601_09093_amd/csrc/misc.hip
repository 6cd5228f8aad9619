// Error names, version, and the plain copy kernel used to calibrate profiler byte counters.
#include "common.h"

namespace step {
namespace {

__global__ __launch_bounds__(256) void copy16(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace step

extern "C" const char *step_strerror(int code)
{
    switch (code) {
        case STEP_OK: return "STEP_OK";
        case STEP_EINVAL: return "STEP_EINVAL: bad dimension, null or misaligned pointer";
        case STEP_EWORKSPACE: return "STEP_EWORKSPACE: workspace missing, misaligned or too small";
        case STEP_ELAUNCH: return "STEP_ELAUNCH: kernel launch refused by the HIP runtime";
        case STEP_EPAGE: return "STEP_EPAGE: block-table entry outside the page pool";
        case STEP_ELEN: return "STEP_ELEN: sequence length negative or beyond the block-table row";
        case STEP_EINDEX: return "STEP_EINDEX: boundary row or trace index out of range";
        case STEP_ENAN: return "STEP_ENAN: NaN score on a live trace";
        case STEP_EREFCOUNT: return "STEP_EREFCOUNT: released page had refcount <= 0";
        case STEP_EKLIVE: return "STEP_EKLIVE: k exceeds the number of live traces";
        case STEP_EPLAN: return "STEP_EPLAN: the workspace holds no attention plan made for these dims";
    }
    return "unknown libstep error";
}

extern "C" const char *step_version(void) { return "0.1"; }

extern "C" int step_calib_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || bytes % 16 || !step::aligned(dst, 16) || !step::aligned(src, 16)) return STEP_EINVAL;
    if (bytes == 0) return STEP_OK;
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(step::copy16, dim3((unsigned)blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<uint4 *>(dst), reinterpret_cast<const uint4 *>(src), n);
    return step::launch_status();
}
