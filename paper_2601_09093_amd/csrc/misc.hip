// Error names, version, and the plain copy kernel used to calibrate profiler byte counters.
#include "common.h"

namespace step {
namespace {

__global__ __launch_bounds__(256) void copy16(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// Bare tile-read probe: wave (w, g) reads the K and V tiles (4096 bytes each) of KV head g of the pages
// ids[w * pages_per_wave .. +pages_per_wave), two pages in flight, and folds them into a word nobody needs.
// PATTERN 0: 1 KB contiguous per load instruction (the dot2 kernel's loads); 1: the matrix-core operand
// pattern (K: 16 rows x 64 bytes, V: 4 rows x 256 bytes per instruction).  NT: non-temporal loads.
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
// (occupancy of exactly one wave per SIMD, like the streaming kernels it stands in for)
template <int PATTERN, bool NT>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 1))) void read_probe(const u32x4 *__restrict__ kp, const u32x4 *__restrict__ vp,
                                                 const int32_t *__restrict__ ids, int pages_per_wave, int Hkv, int NP,
                                                 u32 *sink)
{
    const int lane = threadIdx.x, c = lane & 15, gr = lane >> 4;
    const int g = blockIdx.x % Hkv, w = blockIdx.x / Hkv;
    const int32_t *b = ids + (size_t)w * pages_per_wave;
    u32x4 acc = {0, 0, 0, 0};
    u32x4 k[2][4], v[2][4];
    auto load = [&](int slot, int pg) {
        const int page = b[pg];
        const size_t tile = ((size_t)((u32)page < (u32)NP ? page : 0) * Hkv + g) * 256;  // in 16-byte units
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            size_t ko, vo;
            if constexpr (PATTERN == 0) { ko = tile + j * 64 + lane; vo = ko; }
            else { ko = tile + c * 16 + j * 4 + gr; vo = tile + (4 * gr + j) * 16 + c; }
            if constexpr (NT) {
                k[slot][j] = __builtin_nontemporal_load(kp + ko);
                v[slot][j] = __builtin_nontemporal_load(vp + vo);
            } else {
                k[slot][j] = kp[ko];
                v[slot][j] = vp[vo];
            }
        }
    };
    load(0, 0);
    load(1, pages_per_wave > 1 ? 1 : 0);
    for (int pg = 0; pg < pages_per_wave; pg += 2) {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
#pragma unroll
            for (int j = 0; j < 4; ++j) acc ^= k[d][j] ^ v[d][j];
            if (pg + 2 + d < pages_per_wave) load(d, pg + 2 + d);
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1;
}

}  // namespace

Profile &profile()
{
    static Profile p;
    return p;
}

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
        case STEP_EPLAN: return "STEP_EPLAN: the workspace holds no shared-prefix lengths made for these dims (step_attn_plan)";
        case STEP_EFREELIST: return "STEP_EFREELIST: the workspace holds no free list for this pool, or it does not match the refcounts";
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
    step::launch_kernel(step::kKernCopy, step::copy16, dim3((unsigned)blocks), dim3(256),
                        reinterpret_cast<hipStream_t>(stream), reinterpret_cast<uint4 *>(dst),
                        reinterpret_cast<const uint4 *>(src), n);
    return step::launch_status();
}

extern "C" int step_read_probe(const void *k_pages, const void *v_pages, const int32_t *page_ids, int32_t waves,
                               int32_t pages_per_wave, int32_t Hkv, int32_t NP, int32_t pattern, int32_t nontemporal,
                               uint32_t *sink, void *stream)
{
    if (!k_pages || !v_pages || !page_ids || !sink || waves <= 0 || pages_per_wave <= 0 || Hkv <= 0 || NP <= 0)
        return STEP_EINVAL;
    if (!step::aligned(k_pages, 16) || !step::aligned(v_pages, 16) || (pattern != 0 && pattern != 1)) return STEP_EINVAL;
    typedef step::u32x4 V;
    void (*kernel)(const V *, const V *, const int32_t *, int, int, int, step::u32 *) =
        pattern == 0 ? (nontemporal ? step::read_probe<0, true> : step::read_probe<0, false>)
                     : (nontemporal ? step::read_probe<1, true> : step::read_probe<1, false>);
    step::launch_kernel(step::kKernReadProbe, kernel, dim3((unsigned)waves * Hkv), dim3(64),
                        reinterpret_cast<hipStream_t>(stream), reinterpret_cast<const V *>(k_pages),
                        reinterpret_cast<const V *>(v_pages), page_ids, pages_per_wave, Hkv, NP, sink);
    return step::launch_status();
}

extern "C" const char *step_profile_kernel_name(int id)
{
    static const char *const names[step::kKernCount] = {
        "attn_front", "attn_plan_blocks", "attn_partial", "attn_merge", "score_hidden", "score_finish", "prune_fused",
        "prune_select", "prune_release", "prune_compact", "reserve_pages", "freelist", "append_kv", "weighted_vote", "calib_copy",
        "read_probe"};
    return (id >= 0 && id < step::kKernCount) ? names[id] : "unknown";
}

extern "C" int step_profile_begin(int cap)
{
    step::Profile &p = step::profile();
    if (cap <= 0 || p.ev) return STEP_EINVAL;
    p.ev = new hipEvent_t[2 * (size_t)cap];
    p.ids = new int32_t[(size_t)cap];
    for (int i = 0; i < 2 * cap; ++i)
        if (hipEventCreate(&p.ev[i]) != hipSuccess) return STEP_ELAUNCH;
    p.cap = cap;
    p.used = 0;
    return STEP_OK;
}

extern "C" int step_profile_end(int32_t *kernel_ids, float *ms, int cap)
{
    step::Profile &p = step::profile();
    if (!p.ev || !ms || !kernel_ids || cap < p.used) return -STEP_EINVAL;
    const int n = p.used;
    for (int i = 0; i < n; ++i) {
        (void)hipEventSynchronize(p.ev[2 * i + 1]);
        if (hipEventElapsedTime(&ms[i], p.ev[2 * i], p.ev[2 * i + 1]) != hipSuccess) ms[i] = -1.f;
        kernel_ids[i] = p.ids[i];
    }
    for (int i = 0; i < 2 * p.cap; ++i) (void)hipEventDestroy(p.ev[i]);
    delete[] p.ev;
    delete[] p.ids;
    p = step::Profile();
    return n;
}
