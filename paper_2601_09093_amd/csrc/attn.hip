// paged_decode_attn: split-K (flash-decoding) grouped-query decode attention over a paged bf16
// KV cache -- the attention inside NextToken(t) of Algorithm 1 (the paper gives no formula; this
// is softmax(q K^T scale) V for the newest token of every live trace).
//
// Stage 1 (attn_partial): one 64-lane wavefront per work item (trace i, KV head g, chunk of CP
//   pages).  A (page, head) tile is P*D bf16 contiguous; the wave reads it with 16-byte loads,
//   lane l taking bytes [j*1024 + 16 l, +16) of the tile on load j, so every load instruction
//   covers 1 KB of consecutive addresses.  A row of D values therefore lives in LPR = D/8
//   neighbouring lanes and each group of LPR lanes ("row group" r) sees the tokens r, r+TPI, ...
//   of every page: TPI = 64/LPR independent online-softmax streams per wave, which never talk
//   to each other inside the page loop and are merged once at the end of the item.
//   The G query heads of the group share every K and V register.
// Stage 2 (attn_merge): per (trace, query head) combine the chunk partials (m, l, acc) and round
//   to bf16.
#include "common.h"

namespace step {
namespace {

constexpr float kMinusBig = -1.0e30f;  // finite "no token seen yet" running max (keeps exp2 NaN-free)

struct AttnArgs {
    const uint16_t *q, *k_pages, *v_pages;
    const int32_t *block_tables, *seq_lens;
    float *part_acc;  // [N*Hkv*maxchunks][G][D]
    float *part_ml;   // [N*Hkv*maxchunks][G][2]  (running max in log2 units, sum of weights)
    uint16_t *out;
    int32_t *status;
    int N, Hq, Hkv, MAXB, NP, CP, maxchunks;
    float scale_log2;  // scale * log2(e)
};

template <int BIT>
__device__ __forceinline__ float partner(float v)
{
    if constexpr (BIT == 3) return dpp<kDppRowMirror>(v);
    else if constexpr (BIT == 2) return dpp<kDppHalfMirror>(v);
    else if constexpr (BIT == 1) return dpp<kDppXor2>(v);
    else return dpp<kDppXor1>(v);
}

// One stage of the transposing reduction: lanes whose bit BIT of c differ pair up, each keeps the
// half of its NCUR values whose index has that bit equal to its own and adds the partner's copy.
template <int BIT, int NCUR, int NV>
__device__ __forceinline__ void bfly_stage(float (&val)[NV], int c)
{
    const bool up = (c >> BIT) & 1;
#pragma unroll
    for (int t = 0; t < NCUR / 2; ++t) {
        const float lo = val[t], hi = val[t + NCUR / 2];
        const float keep = up ? hi : lo;
        const float send = up ? lo : hi;
        val[t] = keep + partner<BIT>(send);
    }
}

template <int D, int G>
__global__ __launch_bounds__(64) void attn_partial(const AttnArgs a)
{
    constexpr int LPR = D / 8;            // lanes per token row
    constexpr int TPI = 64 / LPR;         // token rows per load instruction
    constexpr int IPP = kPageTokens / TPI;  // load instructions per (page, head) tile
    constexpr int NV = IPP * G;           // logits per lane per page before reduction
    constexpr bool FAST = (NV == LPR);    // transposing reduction leaves exactly one logit per lane
    __shared__ float pbuf[64];

    const int lane = threadIdx.x;
    const int r = lane / LPR, c = lane % LPR;

    u32 bid = blockIdx.x;
    const int g = bid % a.Hkv;
    bid /= a.Hkv;
    const int i = bid % a.N;
    const int ch = bid / a.N;

    const int L = a.seq_lens[i];
    if (L <= 0 || (long long)L > (long long)a.MAXB * kPageTokens) {
        if (L != 0 && ch == 0 && g == 0 && lane == 0) report(a.status, STEP_ELEN);
        return;
    }
    const int nb = (L + kPageTokens - 1) / kPageTokens;
    const int first = ch * a.CP;
    if (first >= nb) return;
    const int end = min(nb, first + a.CP);

    uint4 qv[G];
#pragma unroll
    for (int h = 0; h < G; ++h)
        qv[h] = *reinterpret_cast<const uint4 *>(a.q + ((size_t)i * a.Hq + (size_t)g * G + h) * D + c * 8);

    float m[G], acc[G][8];
    float lrep[G];             // !FAST: sum of weights per head, replicated over the row's lanes
    float m_own = kMinusBig;   // FAST: running max / weight sum of this lane's own head c % G
    float l_own = 0.f;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = kMinusBig;
        lrep[h] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
    }

    const int32_t *bt = a.block_tables + (size_t)i * a.MAXB;
    const size_t tile_elems = (size_t)kPageTokens * D;

    auto load_tile = [&](int page, uint4 (&k)[IPP], uint4 (&v)[IPP]) {
        const size_t off = ((size_t)page * a.Hkv + g) * tile_elems;
        const uint4 *kt = reinterpret_cast<const uint4 *>(a.k_pages + off);
        const uint4 *vt = reinterpret_cast<const uint4 *>(a.v_pages + off);
#pragma unroll
        for (int j = 0; j < IPP; ++j) k[j] = kt[j * 64 + lane];
#pragma unroll
        for (int j = 0; j < IPP; ++j) v[j] = vt[j * 64 + lane];
    };

    auto process = [&](uint4 (&k)[IPP], uint4 (&v)[IPP], int ntok) {
        if (ntok < kPageTokens) {  // last page of the trace: slots >= ntok hold garbage (maybe NaN)
#pragma unroll
            for (int j = 0; j < IPP; ++j)
                if (j * TPI + r >= ntok) {
                    k[j] = make_uint4(0, 0, 0, 0);
                    v[j] = make_uint4(0, 0, 0, 0);
                }
        }
        float val[NV];
#pragma unroll
        for (int j = 0; j < IPP; ++j)
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float s = dot2_bf16(k[j].x, qv[h].x, 0.f);
                s = dot2_bf16(k[j].y, qv[h].y, s);
                s = dot2_bf16(k[j].z, qv[h].z, s);
                s = dot2_bf16(k[j].w, qv[h].w, s);
                val[j * G + h] = s;
            }
        float pv[NV];
        if constexpr (FAST) {
            if constexpr (LPR == 16) bfly_stage<3, 16, NV>(val, c);
            if constexpr (LPR >= 8) bfly_stage<2, 8, NV>(val, c);
            bfly_stage<1, 4, NV>(val, c);
            bfly_stage<0, 2, NV>(val, c);
            // this lane now owns the logit of (slot (c/G)*TPI + r, head c % G)
            float x = val[0] * a.scale_log2;
            if (ntok < kPageTokens && (c / G) * TPI + r >= ntok) x = -INFINITY;
            float mx = x;
            if constexpr (LPR == 16) {
                mx = fmaxf(mx, dpp<kDppRowRor4>(mx));
                mx = fmaxf(mx, dpp<kDppRowRor8>(mx));
            } else {
                mx = fmaxf(mx, __shfl_xor(mx, 4));
            }
            const float m_new = fmaxf(m_own, mx);
            if (__any(m_new > m_own)) {
                float mq[G];
                mq[0] = fmaxf(m[0], dpp<STEP_DPP_QUAD_BCAST(0)>(mx));
                mq[1] = fmaxf(m[1], dpp<STEP_DPP_QUAD_BCAST(1)>(mx));
                mq[2] = fmaxf(m[2], dpp<STEP_DPP_QUAD_BCAST(2)>(mx));
                mq[3] = fmaxf(m[3], dpp<STEP_DPP_QUAD_BCAST(3)>(mx));
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float alpha = __builtin_amdgcn_exp2f(m[h] - mq[h]);
                    m[h] = mq[h];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
                }
                l_own *= __builtin_amdgcn_exp2f(m_own - m_new);
                m_own = m_new;
            }
            const float p = __builtin_amdgcn_exp2f(x - m_own);
            l_own += p;
            // every lane of the row group needs all NV weights of the group: exchange through LDS
            pbuf[lane] = p;
            __builtin_amdgcn_wave_barrier();
            const float4 *pb = reinterpret_cast<const float4 *>(pbuf + r * LPR);
#pragma unroll
            for (int t = 0; t < NV / 4; ++t) {
                const float4 f = pb[t];
                pv[4 * t + 0] = f.x; pv[4 * t + 1] = f.y; pv[4 * t + 2] = f.z; pv[4 * t + 3] = f.w;
            }
            __builtin_amdgcn_wave_barrier();
        } else {
            // plain all-reduce over the row's lanes: every lane ends with all NV logits of its rows
#pragma unroll
            for (int v0 = 0; v0 < NV; ++v0) {
                float s = val[v0];
#pragma unroll
                for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
                s *= a.scale_log2;
                if (ntok < kPageTokens && (v0 / G) * TPI + r >= ntok) s = -INFINITY;
                val[v0] = s;
            }
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float mx = val[h];
#pragma unroll
                for (int j = 1; j < IPP; ++j) mx = fmaxf(mx, val[j * G + h]);
                const float m_new = fmaxf(m[h], mx);
                const float alpha = __builtin_amdgcn_exp2f(m[h] - m_new);
                m[h] = m_new;
                lrep[h] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
#pragma unroll
                for (int j = 0; j < IPP; ++j) {
                    const float p = __builtin_amdgcn_exp2f(val[j * G + h] - m_new);
                    pv[j * G + h] = p;
                    lrep[h] += p;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < IPP; ++j) {
            const u32 w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            float vf[8];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                vf[2 * t] = bf16_lo(w[t]);
                vf[2 * t + 1] = bf16_hi(w[t]);
            }
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float pw = pv[j * G + h];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(pw, vf[e], acc[h][e]);
            }
        }
    };

    auto ntok_of = [&](int pg) { return pg == nb - 1 ? L - pg * kPageTokens : kPageTokens; };
    auto page_ok = [&](int page) { return (u32)page < (u32)a.NP; };

    uint4 ka[IPP], va[IPP], kb[IPP], vb[IPP];
    int pa = bt[first];
    bool oka = page_ok(pa);
    if (oka) load_tile(pa, ka, va);
    bool bad_page = !oka;
    for (int pg = first; pg < end; pg += 2) {
        bool okb = false;
        if (pg + 1 < end) {
            const int pb = bt[pg + 1];
            okb = page_ok(pb);
            bad_page |= !okb;
            if (okb) load_tile(pb, kb, vb);
        }
        if (oka) process(ka, va, ntok_of(pg));
        oka = false;
        if (pg + 2 < end) {
            pa = bt[pg + 2];
            oka = page_ok(pa);
            bad_page |= !oka;
            if (oka) load_tile(pa, ka, va);
        }
        if (okb) process(kb, vb, ntok_of(pg + 1));
    }
    if (bad_page && lane == 0) report(a.status, STEP_EPAGE);

    // ---- merge the TPI row-group streams of this wave, write the item's partial ----
    float lh[G];
    if constexpr (FAST) {
        float ls = l_own;
        if constexpr (LPR == 16) {
            ls += dpp<kDppRowRor4>(ls);
            ls += dpp<kDppRowRor8>(ls);
        } else {
            ls += __shfl_xor(ls, 4);
        }
        lh[0] = dpp<STEP_DPP_QUAD_BCAST(0)>(ls);
        lh[1] = dpp<STEP_DPP_QUAD_BCAST(1)>(ls);
        lh[2] = dpp<STEP_DPP_QUAD_BCAST(2)>(ls);
        lh[3] = dpp<STEP_DPP_QUAD_BCAST(3)>(ls);
    } else {
#pragma unroll
        for (int h = 0; h < G; ++h) lh[h] = lrep[h];
    }
    const size_t item = ((size_t)i * a.Hkv + g) * a.maxchunks + ch;
    float *pacc = a.part_acc + item * (G * D);
    float *pml = a.part_ml + item * (G * 2);
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float M = m[h];
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
        const float f = __builtin_amdgcn_exp2f(m[h] - M);
        float l = lh[h] * f;
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) l += __shfl_xor(l, off);
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = acc[h][e] * f;
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off);
            o[e] = x;
        }
        if (r == 0) {
            float4 *dst = reinterpret_cast<float4 *>(pacc + h * D + c * 8);
            dst[0] = make_float4(o[0], o[1], o[2], o[3]);
            dst[1] = make_float4(o[4], o[5], o[6], o[7]);
            if (c == 0) {
                pml[h * 2 + 0] = M;
                pml[h * 2 + 1] = l;
            }
        }
    }
}

// out[i][h][:] = sum_c 2^(m_c - M) acc_c / sum_c 2^(m_c - M) l_c, rounded to bf16.
template <int D, int G>
__global__ __launch_bounds__(64) void attn_merge(const AttnArgs a)
{
    constexpr int DPT = D / 64;
    const int lane = threadIdx.x;
    const int i = blockIdx.x / a.Hq, h = blockIdx.x % a.Hq;
    const int g = h / G, hh = h % G;
    uint16_t *orow = a.out + ((size_t)i * a.Hq + h) * D;
    const int L = a.seq_lens[i];
    float o[DPT];
#pragma unroll
    for (int t = 0; t < DPT; ++t) o[t] = 0.f;
    float den = 0.f;
    if (L > 0 && (long long)L <= (long long)a.MAXB * kPageTokens) {
        const int nb = (L + kPageTokens - 1) / kPageTokens;
        const int nch = (nb + a.CP - 1) / a.CP;
        const size_t item0 = ((size_t)i * a.Hkv + g) * a.maxchunks;
        float M = kMinusBig;
        for (int ch = 0; ch < nch; ++ch) M = fmaxf(M, a.part_ml[(item0 + ch) * (G * 2) + hh * 2]);
        for (int ch = 0; ch < nch; ++ch) {
            const float *ml = a.part_ml + (item0 + ch) * (G * 2) + hh * 2;
            const float f = __builtin_amdgcn_exp2f(ml[0] - M);
            den += f * ml[1];
            const float *pa = a.part_acc + (item0 + ch) * (G * D) + hh * D;
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

int chunk_pages_for(const step_attn_dims *d)
{
    static const int env = [] {
        const char *s = getenv("STEP_ATTN_CHUNK_PAGES");
        return s ? atoi(s) : 0;
    }();
    if (env > 0) return env;
    (void)d;
    return 32;
}

bool dims_ok(const step_attn_dims *d)
{
    if (!d) return false;
    if (d->N < 0 || d->Hq <= 0 || d->Hkv <= 0 || d->MAXB < 0 || d->NP < 0) return false;
    if (d->P != kPageTokens || (d->D != 64 && d->D != 128)) return false;
    if (d->Hq % d->Hkv) return false;
    const int G = d->Hq / d->Hkv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return false;
    if ((long long)d->N * d->Hq > (1ll << 30)) return false;
    return true;
}

template <int D, int G>
int launch(const AttnArgs &a, hipStream_t s)
{
    const long long items = (long long)a.N * a.Hkv * a.maxchunks;
    if (items > 0x7fffffffll) return STEP_EINVAL;
    if (items > 0) hipLaunchKernelGGL((attn_partial<D, G>), dim3((u32)items), dim3(64), 0, s, a);
    hipLaunchKernelGGL((attn_merge<D, G>), dim3((u32)(a.N * a.Hq)), dim3(64), 0, s, a);
    return launch_status();
}

}  // namespace
}  // namespace step

using namespace step;

extern "C" size_t step_attn_workspace_bytes(const step_attn_dims *d)
{
    if (!dims_ok(d)) return 0;
    const int CP = chunk_pages_for(d);
    const size_t maxchunks = ((size_t)d->MAXB + CP - 1) / CP;
    const size_t items = (size_t)d->N * d->Hkv * maxchunks;
    const size_t G = d->Hq / d->Hkv;
    size_t acc = items * G * d->D * sizeof(float);
    acc = (acc + 255) & ~(size_t)255;
    const size_t ml = items * G * 2 * sizeof(float);
    return acc + ((ml + 255) & ~(size_t)255) + 256;
}

extern "C" int paged_decode_attn(const step_attn_dims *d, const uint16_t *q, const uint16_t *k_pages,
                                 const uint16_t *v_pages, const int32_t *block_tables, const int32_t *seq_lens,
                                 uint16_t *out, void *workspace, size_t workspace_bytes, int32_t *status,
                                 void *stream)
{
    if (!dims_ok(d)) return STEP_EINVAL;
    if (d->N == 0) return STEP_OK;
    if (!q || !k_pages || !v_pages || !block_tables || !seq_lens || !out) return STEP_EINVAL;
    if (!aligned(q, 16) || !aligned(k_pages, 16) || !aligned(v_pages, 16) || !aligned(out, 4)) return STEP_EINVAL;
    const size_t need = step_attn_workspace_bytes(d);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < need) return STEP_EWORKSPACE;

    AttnArgs a;
    a.q = q; a.k_pages = k_pages; a.v_pages = v_pages;
    a.block_tables = block_tables; a.seq_lens = seq_lens;
    a.out = out; a.status = status;
    a.N = d->N; a.Hq = d->Hq; a.Hkv = d->Hkv; a.MAXB = d->MAXB; a.NP = d->NP;
    a.CP = chunk_pages_for(d);
    a.maxchunks = (d->MAXB + a.CP - 1) / a.CP;
    a.scale_log2 = d->scale * 1.4426950408889634f;
    const size_t G = d->Hq / d->Hkv;
    size_t acc_bytes = (size_t)d->N * d->Hkv * a.maxchunks * G * d->D * sizeof(float);
    acc_bytes = (acc_bytes + 255) & ~(size_t)255;
    a.part_acc = reinterpret_cast<float *>(workspace);
    a.part_ml = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + acc_bytes);

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const int key = d->D * 16 + (int)G;
    switch (key) {
        case 64 * 16 + 1: return launch<64, 1>(a, s);
        case 64 * 16 + 2: return launch<64, 2>(a, s);
        case 64 * 16 + 4: return launch<64, 4>(a, s);
        case 64 * 16 + 8: return launch<64, 8>(a, s);
        case 128 * 16 + 1: return launch<128, 1>(a, s);
        case 128 * 16 + 2: return launch<128, 2>(a, s);
        case 128 * 16 + 4: return launch<128, 4>(a, s);
        case 128 * 16 + 8: return launch<128, 8>(a, s);
    }
    return STEP_EINVAL;
}
