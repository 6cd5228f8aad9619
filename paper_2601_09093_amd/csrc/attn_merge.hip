// attn_merge: stage 2 of paged_decode_attn.
#include "attn_common.h"

namespace step {
namespace attn {
namespace {

// ---------------------------------------------------------------------------------------------
// stage 2: out[i][h][:] = sum_c 2^(m_c - M) acc_c / sum_c 2^(m_c - M) l_c, rounded to bf16
// ---------------------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(64) void attn_merge(const AttnArgs a)
{
    constexpr int DPT = D / 64;
    const int lane = threadIdx.x;
    const int i = blockIdx.x / a.Hq, h = blockIdx.x % a.Hq;
    const int g = h / G, hh = h % G;
    uint16_t *orow = a.out + ((size_t)i * a.Hq + h) * D;
    // the trace's partials: parts_b sub-chunks of its block's shared prefix (slots p * N + i), then cnt2
    // consecutive private-page records from first2
    const int nb = pages_of(a.seq_lens[i], a.MAXB);
    int parts, sc;
    prefix_split(a, clamp_shared(a, a.blk_shared[i / a.TB], nb), parts, sc);
    const int f2 = a.first2[i], c2 = a.cnt2[i];
    int nch = nb > 0 ? parts + c2 : 0;
    if (nch > 0 && (c2 < 0 || f2 < a.priv_base || (long long)f2 + c2 > (long long)a.priv_base + a.N + a.Wh)) {
        if (lane == 0) report(a.status, STEP_EPLAN);
        nch = 0;
    }
    auto slot_of = [&](int ch) { return (size_t)(ch < parts ? a.prefix_base + ch * a.N + i : f2 + (ch - parts)) * a.Hkv + g; };

    float o[DPT];
#pragma unroll
    for (int t = 0; t < DPT; ++t) o[t] = 0.f;
    float M = kMinusBig, den = 0.f;
    // 64 pieces at a time: lane p holds (m, l) of piece base + p, the wave agrees on the maximum,
    // then the piece accumulators are added with four loads in flight
    for (int base = 0; base < nch; base += 64) {
        const int cnt = min(64, nch - base);
        float mp = kMinusBig, lp = 0.f;
        if (lane < cnt) {
            const float *ml = a.part_ml + slot_of(base + lane) * (G * 2) + hh * 2;
            mp = ml[0];
            lp = ml[1];
        }
        float Mn = wave_max(mp);
        Mn = fmaxf(Mn, M);
        const float resc = __builtin_amdgcn_exp2f(M - Mn);
        M = Mn;
        den *= resc;
#pragma unroll
        for (int t = 0; t < DPT; ++t) o[t] *= resc;
        const float fp = __builtin_amdgcn_exp2f(mp - M);  // 0 for lanes without a piece
        den += wave_sum(fp * lp);
        int p = 0;
        for (; p + 3 < cnt; p += 4) {
            float v[4][DPT], f[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float *pa = a.part_acc + slot_of(base + p + u) * (G * D) + hh * D;
                f[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fp), p + u));  // (p is the same in every lane)
#pragma unroll
                for (int t = 0; t < DPT; ++t) v[u][t] = pa[lane * DPT + t];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int t = 0; t < DPT; ++t) o[t] = fmaf(f[u], v[u][t], o[t]);
        }
        for (; p < cnt; ++p) {
            const float *pa = a.part_acc + slot_of(base + p) * (G * D) + hh * D;
            const float f = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fp), p));
#pragma unroll
            for (int t = 0; t < DPT; ++t) o[t] = fmaf(f, pa[lane * DPT + t], o[t]);
        }
    }
    const float inv = den > 0.f ? 1.0f / den : 0.f;
    if constexpr (DPT == 2) {
        const u32 w = f32_to_bf16_bits(o[0] * inv) | (f32_to_bf16_bits(o[1] * inv) << 16);
        reinterpret_cast<u32 *>(orow)[lane] = w;
    } else {
        orow[lane] = (uint16_t)f32_to_bf16_bits(o[0] * inv);
    }
}

}  // namespace

void launch_merge(const AttnArgs &a, int D, hipStream_t s)
{
    const dim3 grid((u32)(a.N * a.Hq));
    const int key = D * 16 + a.Hq / a.Hkv;
    switch (key) {
        case 64 * 16 + 1: launch_kernel(kKernMerge, attn_merge<64, 1>, grid, dim3(64), s, a); break;
        case 64 * 16 + 2: launch_kernel(kKernMerge, attn_merge<64, 2>, grid, dim3(64), s, a); break;
        case 64 * 16 + 4: launch_kernel(kKernMerge, attn_merge<64, 4>, grid, dim3(64), s, a); break;
        case 64 * 16 + 8: launch_kernel(kKernMerge, attn_merge<64, 8>, grid, dim3(64), s, a); break;
        case 128 * 16 + 1: launch_kernel(kKernMerge, attn_merge<128, 1>, grid, dim3(64), s, a); break;
        case 128 * 16 + 2: launch_kernel(kKernMerge, attn_merge<128, 2>, grid, dim3(64), s, a); break;
        case 128 * 16 + 4: launch_kernel(kKernMerge, attn_merge<128, 4>, grid, dim3(64), s, a); break;
        case 128 * 16 + 8: launch_kernel(kKernMerge, attn_merge<128, 8>, grid, dim3(64), s, a); break;
    }
}

}  // namespace attn
}  // namespace step
