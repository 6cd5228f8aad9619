// attn_partial_g4: stage 1 of paged_decode_attn for G = 4, D = 128 (bf16 dot2 on the vector ALUs).
#include "attn_common.h"

namespace step {
namespace attn {
namespace {

// ---------------------------------------------------------------------------------------------
// stage 1, G == 4 and D == 128 (the shape of all three models of the paper): persistent, software-pipelined.
//   phase A(page) : logits of the page (bf16 dot2), transposing reduction that leaves each lane
//                   with one (token, head) logit, running max, p = 2^(x - m), rounded to bf16 and
//                   packed in token pairs, handed to the row group through LDS.
//   phase B(page) : acc += P V with bf16 dot2 on (token pair) x (head), fp32 accumulation.
// A(page j+1) and B(page j) are independent and sit in ONE basic block, so the scheduler overlaps
// the cross-lane / LDS / exp latencies of A with the dot2 stream of B.  The rescale of acc by
// 2^(m_old - m_new), needed only when a page raises the running max, follows B.
// The weight sum l is accumulated from the same bf16-rounded weights that multiply V, so the result
// is an exact weighted average of V rows with weights perturbed by <= 2^-9 relative.
// ---------------------------------------------------------------------------------------------
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

// One wave per SIMD is part of the design (the work is cut into as many equal runs as there are SIMDs), so the
// kernel asks for an occupancy of exactly one: the hardware then cannot put two of its waves on one SIMD and
// leave another idle, which it otherwise sometimes did (seen as a 6 % longer kernel whenever the launch before
// it had left the workgroup dispatcher in a different state, and as 0.7 % on average).
template <int D>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_partial_g4(const AttnArgs a)
{
    constexpr int G = 4;
    constexpr int LPR = D / 8, TPI = 64 / LPR, IPP = kPageTokens / TPI, NV = IPP * G;
    static_assert(D == 128 && NV == LPR, "a row is 16 lanes wide: one logit per lane after the transposing reduction");
    constexpr int NPAIR = IPP / 2;  // token pairs per lane per page
    __shared__ u32 pbuf[2][64];
    __shared__ int P_s[kMaxPlanN + 1], base_s[kMaxPlanN + 1];

    const int lane = threadIdx.x;
    const int r = lane / LPR, c = lane % LPR;
    // gridDim == Wh * Hkv: wave (wh, g) serves KV head g only.  Consecutive workgroups land on
    // consecutive XCDs, so with Hkv == 8 every XCD streams (and caches) the tiles of one KV head.
    // The wave works out its own run of private pages (attn_common.h) and walks its records.
    const int g = blockIdx.x % a.Hkv;
    const int wh = blockIdx.x / a.Hkv;
    const WavePlan wp = plan_build(a, lane, P_s, base_s, blockIdx.x == 0);
    if (blockIdx.x == 0) publish_plan(a, wp, lane, P_s, base_s);
    RunWalker walk(a, wp, P_s, base_s, wh);
    if (!walk.more()) return;
    if (a.NP <= 0) {
        if (lane == 0) report(a.status, STEP_EPAGE);
        return;
    }

    const size_t tile_u4 = (size_t)kPageTokens * D / 8;  // uint4 units per (page, head) tile
    const uint4 *kbase = reinterpret_cast<const uint4 *>(a.k_pages);
    const uint4 *vbase = reinterpret_cast<const uint4 *>(a.v_pages);
    bool bad_page = false;
    auto tile_at = [&](int page) -> size_t {
        const bool ok = (u32)page < (u32)a.NP;
        bad_page |= !ok;
        return ((size_t)(ok ? page : 0) * a.Hkv + g) * tile_u4 + lane;
    };
    // KV tiles are read once and never again by this wave: non-temporal loads (streaming cache
    // policy) keep them from displacing each other in the caches; measured +10 % on a bare tile
    // stream, and the shared prompt tiles are still served from L2
    auto load4 = [&](const uint4 *base, size_t off, uint4 (&x)[IPP]) {
        typedef u32 u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int j = 0; j < IPP; ++j) {
            const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + off + j * 64));
            x[j] = make_uint4(t.x, t.y, t.z, t.w);
        }
    };

    uint4 qv[G];
    auto load_q = [&](int i) {
#pragma unroll
        for (int h = 0; h < G; ++h)
            qv[h] = *reinterpret_cast<const uint4 *>(a.q + ((size_t)i * a.Hq + (size_t)g * G + h) * D + c * 8);
    };

    float m[G], acc[G][8];
    float m_own, l_own, mx_pending;

    // The lanes of a row group exchange their weights through pbuf: lane l writes word l, the group's other
    // lanes read it (wave_lds_sync marks the exchange points).
    auto phaseA = [&](const uint4 (&k)[IPP], int slot, int ntok) {
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
        bfly_stage<3, 16, NV>(val, c);
        bfly_stage<2, 8, NV>(val, c);
        bfly_stage<1, 4, NV>(val, c);
        bfly_stage<0, 2, NV>(val, c);
        // this lane owns the logit of (slot (c/G)*TPI + r, head c % G); slots >= ntok are not tokens
        float x = val[0] * a.scale_log2;
        x = ((c / G) * TPI + r < ntok) ? x : -INFINITY;
        float mx = x;
        mx = max_nc(mx, dpp<kDppRowRor4>(mx));
        mx = max_nc(mx, dpp<kDppRowRor8>(mx));
        const float m_new = max_nc(m_own, mx);
        const float alpha_own = __builtin_amdgcn_exp2f(m_own - m_new);
        m_own = m_new;
        mx_pending = mx;
        const float p = __builtin_amdgcn_exp2f(x - m_new);
        // lane c + 4 of the row group holds the same head's weight for the next token row
        const float p_next = dpp<0x12C>(p);  // row_ror:12 = value of lane (c + 4) % 16
        const bf16x2 pk = {(__bf16)p, (__bf16)p_next};
        const u32 w = __builtin_bit_cast(u32, pk);
        l_own = fmaf(l_own, alpha_own, bf16_lo(w));
        wave_lds_sync();  // the reads of this slot two pages ago come first
        pbuf[slot][lane] = w;
        wave_lds_sync();  // the row group's reads of this slot come after
    };

    auto pv_pairs = [&](const uint4 (&v)[IPP], int slot) {
        const uint4 *pb = reinterpret_cast<const uint4 *>(&pbuf[slot][r * LPR]);
#pragma unroll
        for (int pr = 0; pr < NPAIR; ++pr) {
            const uint4 pp = pb[2 * pr];  // words 8 pr .. 8 pr + 3: heads 0..3 of token pair pr
            const u32 ph[4] = {pp.x, pp.y, pp.z, pp.w};
            const u32 w0[4] = {v[2 * pr].x, v[2 * pr].y, v[2 * pr].z, v[2 * pr].w};
            const u32 w1[4] = {v[2 * pr + 1].x, v[2 * pr + 1].y, v[2 * pr + 1].z, v[2 * pr + 1].w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const u32 lo = __builtin_amdgcn_perm(w1[t], w0[t], 0x05040100u);  // (row0[2t],   row1[2t])
                const u32 hi = __builtin_amdgcn_perm(w1[t], w0[t], 0x07060302u);  // (row0[2t+1], row1[2t+1])
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    acc[h][2 * t] = dot2_bf16(lo, ph[h], acc[h][2 * t]);
                    acc[h][2 * t + 1] = dot2_bf16(hi, ph[h], acc[h][2 * t + 1]);
                }
            }
        }
    };

    auto rescale = [&]() {
        float mq[G];
        mq[0] = max_nc(m[0], dpp<STEP_DPP_QUAD_BCAST(0)>(mx_pending));
        mq[1] = max_nc(m[1], dpp<STEP_DPP_QUAD_BCAST(1)>(mx_pending));
        mq[2] = max_nc(m[2], dpp<STEP_DPP_QUAD_BCAST(2)>(mx_pending));
        mq[3] = max_nc(m[3], dpp<STEP_DPP_QUAD_BCAST(3)>(mx_pending));
        const bool grow = (mq[0] > m[0]) | (mq[1] > m[1]) | (mq[2] > m[2]) | (mq[3] > m[3]);
        if (__any(grow)) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float alpha = __builtin_amdgcn_exp2f(m[h] - mq[h]);
                m[h] = mq[h];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
            }
        }
    };
    // rows past the trace's last token may hold anything (NaN included): clear them before they
    // meet a zero weight
    auto clear_tail = [&](uint4 (&v)[IPP], int ntok) {
#pragma unroll
        for (int jj = 0; jj < IPP; ++jj)
            if (jj * TPI + r >= ntok) v[jj] = make_uint4(0, 0, 0, 0);
    };

    uint4 k0[IPP], v0[IPP], k1[IPP], v1[IPP];
    Record rec = walk.take();
    {
        const int32_t *bt0 = a.block_tables + (size_t)rec.i * a.MAXB + rec.first;
        const size_t t0 = tile_at(scalar_read(bt0)), t1 = tile_at(scalar_read(bt0 + (rec.n > 1 ? 1 : 0)));
        load4(kbase, t0, k0);
        load4(vbase, t0, v0);
        load4(kbase, t1, k1);
        load4(vbase, t1, v1);
        load_q(rec.i);
    }

    for (;;) {
        const bool has_next = walk.more();
        // the next record and the ids of its first two pages are fetched now and consumed after this
        // record's pages
        const Record nrec = has_next ? walk.take() : rec;
        const int32_t *nbt = a.block_tables + (size_t)nrec.i * a.MAXB + nrec.first;
        const int npage0 = scalar_read(nbt), npage1 = scalar_read(nbt + (nrec.n > 1 ? 1 : 0));

        const int n = rec.n;
        const int32_t *bt = a.block_tables + (size_t)rec.i * a.MAXB + rec.first;
        // page ids are fetched one loop trip (two pages) ahead of the tile loads that need them; the
        // index is clamped so the pipeline can run past the end without a branch (the surplus load
        // re-reads the last tile, which is then not used)
        auto page_id = [&](int j) { return scalar_read(bt + min(j, n - 1)); };
        auto ntok_of = [&](int j) { return j == n - 1 ? rec.ntok : kPageTokens; };

        m_own = kMinusBig; l_own = 0.f; mx_pending = kMinusBig;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            m[h] = kMinusBig;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
        }

        int pid2 = page_id(2), pid3 = page_id(3);
        phaseA(k0, 0, ntok_of(0));
        rescale();
        int j = 0;
        for (; j + 2 <= n - 1; j += 2) {
            const size_t t2 = tile_at(pid2), t3 = tile_at(pid3);
            pid2 = page_id(j + 4);
            pid3 = page_id(j + 5);
            load4(kbase, t2, k0);
            phaseA(k1, 1, kPageTokens);
            pv_pairs(v0, 0);
            load4(vbase, t2, v0);
            rescale();
            load4(kbase, t3, k1);
            phaseA(k0, 0, ntok_of(j + 2));
            pv_pairs(v1, 1);
            load4(vbase, t3, v1);
            rescale();
        }
        if (j + 1 <= n - 1) {
            phaseA(k1, 1, ntok_of(j + 1));
            pv_pairs(v0, 0);
            rescale();
            clear_tail(v1, ntok_of(j + 1));
            pv_pairs(v1, 1);
        } else {
            clear_tail(v0, ntok_of(j));
            pv_pairs(v0, 0);
        }

        // all four tile buffers are dead: start the next record before reducing this one
        if (has_next) {
            const size_t t0 = tile_at(npage0), t1 = tile_at(npage1);
            load4(kbase, t0, k0);
            load4(vbase, t0, v0);
            load4(kbase, t1, k1);
            load4(vbase, t1, v1);
            load_q(nrec.i);
        }

        // ---- merge the TPI row-group streams of this wave, write the record's partial ----
        float ls = l_own;
        ls += dpp<kDppRowRor4>(ls);
        ls += dpp<kDppRowRor8>(ls);
        float lh[G];
        lh[0] = dpp<STEP_DPP_QUAD_BCAST(0)>(ls);
        lh[1] = dpp<STEP_DPP_QUAD_BCAST(1)>(ls);
        lh[2] = dpp<STEP_DPP_QUAD_BCAST(2)>(ls);
        lh[3] = dpp<STEP_DPP_QUAD_BCAST(3)>(ls);
        const size_t slot = (size_t)rec.slot * a.Hkv + g;
        float *pacc = a.part_acc + slot * (G * D);
        float *pml = a.part_ml + slot * (G * 2);
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float M = m[h];
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) M = max_nc(M, __shfl_xor(M, off));
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
        if (!has_next) break;
        rec = nrec;
    }
    if (bad_page && lane == 0) report(a.status, STEP_EPAGE);
}

}  // namespace

void launch_stream_g4(const AttnArgs &a, hipStream_t s)
{
    launch_kernel(kKernStage1, attn_partial_g4<128>, dim3((u32)(a.Wh * a.Hkv)), dim3(64), s, a);
}

// resident waves of the streaming kernel per compute unit, from the occupancy query (8 if it fails)
int stream_g4_waves_per_cu()
{
    int nblk = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nblk, attn_partial_g4<128>, 64, 0) != hipSuccess || nblk <= 0) nblk = 8;
    return nblk;
}

}  // namespace attn
}  // namespace step
