// Final stage of the verification attention: for each (sequence, node, query
// head) attend over the draft-tree segment (the node itself and its ancestors,
// tree decode of Algorithm 1) on the vector ALU, merge that with the split-KV
// partials of the context part by their log-sum-exp weights, normalise and store.
// Sixteen lanes per output row (a lane owns D / 16 adjacent channels), four query heads of
// one KV group per wavefront: they share the node, its root path and the draft K / V rows.
#include "internal.h"

namespace specpv {

// Sum over the 16 lanes of a DPP row, result in every lane of the row: lane ^ 1, lane ^ 2,
// then the mirrors inside 8 and 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_row(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_row<0xB1>(x);
    x += dpp_row<0x4E>(x);
    x += dpp_row<0x141>(x);
    x += dpp_row<0x140>(x);
    return x;
}

// CPL adjacent channels of one row, 16 bytes per memory instruction (rows are 16-byte aligned).
template <typename T, int CPL> struct Chan;
template <int CPL> struct Chan<float, CPL> {
    typedef float4 Raw[CPL / 4];
    static __device__ __forceinline__ void load(const void *p, int64_t i, Raw &r) {
#pragma unroll
        for (int x = 0; x < CPL / 4; ++x) r[x] = *(const float4 *)((const float *)p + i + 4 * x);
    }
    static __device__ __forceinline__ void unpack(const Raw &r, float *f) {
#pragma unroll
        for (int x = 0; x < CPL / 4; ++x) { f[4 * x] = r[x].x; f[4 * x + 1] = r[x].y; f[4 * x + 2] = r[x].z; f[4 * x + 3] = r[x].w; }
    }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, const float *f) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int x = 0; x < CPL / 4; ++x) {
            f32x4 v = {f[4 * x], f[4 * x + 1], f[4 * x + 2], f[4 * x + 3]};
            __builtin_nontemporal_store(v, (f32x4 *)((float *)p + i + 4 * x));
        }
    }
};
template <> struct Chan<bf16_t, 8> {
    typedef uint4 Raw;
    static __device__ __forceinline__ void load(const void *p, int64_t i, Raw &r) { r = *(const uint4 *)((const uint16_t *)p + i); }
    static __device__ __forceinline__ void unpack(const Raw &r, float *f) { Elem<bf16_t>::unpack(r, f); }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, const float *f) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        u32x4 v;
#pragma unroll
        for (int x = 0; x < 4; ++x) v[x] = float_to_bf16_bits(f[2 * x]) | ((uint32_t)float_to_bf16_bits(f[2 * x + 1]) << 16);
        __builtin_nontemporal_store(v, (u32x4 *)((uint16_t *)p + i));
    }
};
template <> struct Chan<bf16_t, 4> {
    typedef uint2 Raw;
    static __device__ __forceinline__ void load(const void *p, int64_t i, Raw &r) { r = *(const uint2 *)((const uint16_t *)p + i); }
    static __device__ __forceinline__ void unpack(const Raw &r, float *f) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, const float *f) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        u32x2 v;
#pragma unroll
        for (int x = 0; x < 2; ++x) v[x] = float_to_bf16_bits(f[2 * x]) | ((uint32_t)float_to_bf16_bits(f[2 * x + 1]) << 16);
        __builtin_nontemporal_store(v, (u32x2 *)((uint16_t *)p + i));
    }
};
// The lane's CPL fp32 values of a partial row (i: the row's first element + 4 * (lane & 15)), read
// once: streaming hint.  Rows of 128 are stored so that piece x of all 16 lanes is one dense run
// (partial_pos); the values come out in channel order.
template <int CPL> __device__ __forceinline__ void load_partial(const float *p, int64_t i, float *f)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int x = 0; x < CPL / 4; ++x) {
#ifndef SPECPV_PARTIAL_PLAIN
        const f32x4 v = __builtin_nontemporal_load((const f32x4 *)(p + i + 64 * x));
#else
        const f32x4 v = *(const f32x4 *)(p + i + 64 * x);
#endif
        f[4 * x] = v[0]; f[4 * x + 1] = v[1]; f[4 * x + 2] = v[2]; f[4 * x + 3] = v[3];
    }
}

// The same for the fp16 form of the partials: the lane's CPL channels (adjacent, in order) of a row of D
// halves whose first element has index i.
template <int CPL> __device__ __forceinline__ void load_partial_half(const float *p, int64_t i, int lane16, float *f)
{
    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
    const f16x4 *src = (const f16x4 *)((const _Float16 *)p + i + lane16 * CPL);
#pragma unroll
    for (int x = 0; x < CPL / 4; ++x) {
        const f16x4 v = __builtin_nontemporal_load(src + x);
        f[4 * x] = (float)v[0]; f[4 * x + 1] = (float)v[1]; f[4 * x + 2] = (float)v[2]; f[4 * x + 3] = (float)v[3];
    }
}

// NP: context partials fetched per round (the smallest of 2, 4, 8 that covers the split count keeps
// the registers, and with them the resident wavefronts of a batch, in proportion).
// MULTI: more splits than NP (the many splits of a full verification): rounds of NP, each round's
// reads requested before the previous round is merged.  Without it the split count is at most NP.
// NB: path nodes whose draft K / V rows are requested in the first go: 8 (a tree of candidates alone), or 24
// when partially verified tokens stand in front of the tree as keys (every candidate's path then starts with
// that whole chain; more registers, so only then).
// HALF: the partials' O rows are fp16 and normalised (see Partials); else fp32 sums.
#ifdef SPECPV_TIMELINE
#define SPECPV_CSTAMP(i)                                                                                     \
    do {                                                                                                     \
        if (part.timeline && threadIdx.x == 0)                                                               \
            part.timeline[(2048 + ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 16 + (i)] = \
                __builtin_amdgcn_s_memrealtime();                                                            \
    } while (0)
#else
#define SPECPV_CSTAMP(i) do {} while (0)
#endif

template <typename T, int D, int NP, bool MULTI, int NB, bool HALF>
__global__ __launch_bounds__(256) void combine_kernel(const int32_t *a_parent, const void *a_q, const float *a_po,
                                                    const float *a_pml, int a_M, int a_Hq, int a_G, int a_nsplit,
                                                    Shape s, Partials part, void *out, float *lse, float scale_log2)
{
    // the leading scalar arguments repeat what the first round of reads needs; they can be preloaded into registers
    s.parent = a_parent; s.q = a_q; s.M = a_M; s.Hq = a_Hq; s.G = a_G;
    part.o = const_cast<float *>(a_po); part.ml = const_cast<float *>(a_pml); part.nsplit = a_nsplit;
    SPECPV_CSTAMP(0);   // entry
    constexpr int CPL = D / 16;   // channels per lane: d = (lane & 15) * CPL + x
    typedef typename Chan<T, CPL>::Raw Raw;
    const int lane = threadIdx.x & 63;
    const int d0 = (lane & 15) * CPL;
    // x = XCD (workgroups go to the XCDs round-robin in linear order), y = node, z = bg / 8: the rows
    // of (sequence, KV head) bg are merged on XCD bg % 8, where the split kernel produced them
    const int bg = (int)blockIdx.z * 8 + (int)blockIdx.x;
    if (bg >= s.batch * s.Hkv) return;
    const int j = (int)blockIdx.y;
    const int b = bg / s.Hkv;
    // four query heads of the KV group per wavefront; a group size that is no multiple of four
    // leaves lanes that repeat the last head and store nothing
    const int g = bg - b * s.Hkv, hh = (int)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) * 4 + (lane >> 4);
    const bool live = hh < s.G;
    const int h = g * s.G + (live ? hh : s.G - 1);

    // ---- every read whose address is known from the arguments goes out first ----------
    // the tree has s.Mk nodes; query row j is node j + s.koff (the nodes in front are keys only)
    const int32_t *par = s.parent + (int64_t)b * s.Mk;
    const int par0 = lane < s.Mk ? par[lane] : -1;
    const int par1 = lane + 64 < s.Mk ? par[lane + 64] : -1;
    const int64_t qrow = (((int64_t)b * s.M + j) * s.Hq + h) * D;
    Raw qraw;
    Chan<T, CPL>::load(s.q, qrow + d0, qraw);
    const int64_t prow0 = (((int64_t)b * s.Hq + h) * part.nsplit) * s.M + j;
    // ... including the first NP context partials (all of them in the usual case); the 16 lanes
    // of a row all fetch the row's (m, l) pairs, so the merge below needs no cross-lane step
    struct Round { float2 ml[NP]; float po[NP][CPL]; };
    auto fetch = [&](int sp0, Round &r) {
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int64_t prow = prow0 + (int64_t)min(sp0 + u, part.nsplit - 1) * s.M;
            r.ml[u] = *(const float2 *)(part.ml + prow * 2);
            if (HALF) load_partial_half<CPL>(part.o, prow * D, lane & 15, r.po[u]);
            else load_partial<CPL>(part.o, prow * D + 4 * (lane & 15), r.po[u]);
        }
    };
    Round ra;
    fetch(0, ra);

    // ---- root path of node j as a bit set (wave-uniform walk over the parent registers) --
    unsigned long long anc_lo = 0ull, anc_hi = 0ull;
    {
        int a = j + s.koff;
        // (nodes below kctx are partially verified tokens that the context kernels have attended already)
        for (int guard = 0; a >= s.kctx && guard < s.Mk; ++guard) {
            if (a < 64) anc_lo |= 1ull << a; else anc_hi |= 1ull << (a - 64);
            const int pa = a < 64 ? __builtin_amdgcn_readlane(par0, a) : __builtin_amdgcn_readlane(par1, a - 64);
            a = pa < a ? pa : -1;   // a malformed parent[] (not strictly decreasing) ends the walk
        }
    }
    SPECPV_CSTAMP(1);   // parents in, root path walked
    // ---- second (and last) round of reads: draft K / V of the first 8 nodes of the path ----
    auto pop = [&]() -> int {
        int a = -1;
        if (anc_lo) { a = __builtin_ctzll(anc_lo); anc_lo &= anc_lo - 1; }
        else if (anc_hi) { a = 64 + __builtin_ctzll(anc_hi); anc_hi &= anc_hi - 1; }
        return a;
    };
    int a8[NB];
    Raw kd8[NB], vd8[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        a8[u] = pop();
        const int64_t drow = (((int64_t)b * s.Mk + max(a8[u], 0)) * s.Hkv + g) * D;
        Chan<T, CPL>::load(s.kd, drow + d0, kd8[u]);
        Chan<T, CPL>::load(s.vd, drow + d0, vd8[u]);
    }

    // ---- context partials, merged relative to their running maximum (first-round data) ----
    float m_ctx = -INFINITY, l_ctx = 0.f, o[CPL];
#pragma unroll
    for (int x = 0; x < CPL; ++x) o[x] = 0.f;
    auto merge = [&](int sp0, const Round &r) {
        float m_new = m_ctx;
#pragma unroll
        for (int u = 0; u < NP; ++u)
            if (sp0 + u < part.nsplit) m_new = fmaxf(m_new, r.ml[u].x);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m_ctx - m_use);   // 0 while nothing has been merged
        l_ctx *= alpha;
#pragma unroll
        for (int x = 0; x < CPL; ++x) o[x] *= alpha;
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const float w = (sp0 + u < part.nsplit && r.ml[u].y > 0.f) ? exp2f(r.ml[u].x - m_use) : 0.f;
            l_ctx = fmaf(r.ml[u].y, w, l_ctx);
            const float wo = HALF ? w * r.ml[u].y : w;   // a normalised partial weighs in with its l
#pragma unroll
            for (int x = 0; x < CPL; ++x) o[x] = fmaf(wo, r.po[u][x], o[x]);
        }
        m_ctx = m_new;
    };
    if (!MULTI) {
        merge(0, ra);
    } else {
        // two register sets in turn; a fetch and the merge in front of which it goes out stay in one
        // basic block, so that the merge waits for its own round only
        Round rb;
        for (int sp0 = 0;;) {
            if (sp0 + NP >= part.nsplit) { merge(sp0, ra); break; }
            fetch(sp0 + NP, rb);
            merge(sp0, ra);
            sp0 += NP;
            if (sp0 + NP >= part.nsplit) { merge(sp0, rb); break; }
            fetch(sp0 + NP, ra);
            merge(sp0, rb);
            sp0 += NP;
        }
    }

    SPECPV_CSTAMP(2);   // context partials in and merged
    // ---- draft-tree segment: the node itself and its ancestors --------------------------
    float qv[CPL];
    Chan<T, CPL>::unpack(qraw, qv);
    float m = -INFINITY, l = 0.f, od[CPL];
#pragma unroll
    for (int x = 0; x < CPL; ++x) od[x] = 0.f;
    // online softmax over four nodes (slots without a node have a[u] < 0 and weigh nothing)
    auto four = [&](const int *a, const Raw *kdv, const Raw *vdv) {
        float z[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float kf[CPL];
            Chan<T, CPL>::unpack(kdv[u], kf);
            float dot = 0.f;
#pragma unroll
            for (int x = 0; x < CPL; ++x) dot = fmaf(qv[x], kf[x], dot);
            z[u] = a[u] >= 0 ? row16_sum(dot) * scale_log2 : -INFINITY;
        }
        const float m_new = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), m);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m - m_use);
        l *= alpha;
#pragma unroll
        for (int x = 0; x < CPL; ++x) od[x] *= alpha;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float pe = exp2f(z[u] - m_use);   // 0 for the unused slots
            l += pe;
            float vf[CPL];
            Chan<T, CPL>::unpack(vdv[u], vf);
#pragma unroll
            for (int x = 0; x < CPL; ++x) od[x] = fmaf(pe, vf[x], od[x]);
        }
        m = m_new;
    };
    four(a8, kd8, vd8);
#pragma unroll
    for (int u = 4; u < NB; u += 4)
        if (a8[u] >= 0) four(a8 + u, kd8 + u, vd8 + u);
    while (anc_lo | anc_hi) {   // paths longer than 8 nodes (partially verified tokens in front of the tree): 8 per trip
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            a8[u] = pop();
            const int64_t drow = (((int64_t)b * s.Mk + max(a8[u], 0)) * s.Hkv + g) * D;
            Chan<T, CPL>::load(s.kd, drow + d0, kd8[u]);
            Chan<T, CPL>::load(s.vd, drow + d0, vd8[u]);
        }
        four(a8, kd8, vd8);
        if (a8[4] >= 0) four(a8 + 4, kd8 + 4, vd8 + 4);
    }

    SPECPV_CSTAMP(3);   // draft K / V rows in, tree segment done
    // ---- merge the two and store ---------------------------------------------------------
    const float m_all = fmaxf(m, m_ctx);
    const float wd = exp2f(m - m_all);
    const float wc = m_ctx == -INFINITY ? 0.f : exp2f(m_ctx - m_all);
    const float den = l * wd + l_ctx * wc;
    const float inv = 1.f / den;
    if (!live) return;
    float res[CPL];
#pragma unroll
    for (int x = 0; x < CPL; ++x) res[x] = (od[x] * wd + o[x] * wc) * inv;
    Chan<T, CPL>::store_stream(out, qrow + d0, res);
    if (lse && (lane & 15) == 0) lse[((int64_t)b * s.M + j) * s.Hq + h] = (m_all + log2f(den)) * kLn2;
    SPECPV_CSTAMP(4);   // stored (issued)
}

template <typename T, int D>
static void launch_combine_t(const Shape &s, Partials p, void *out, float *lse, hipStream_t st)
{
    dim3 grid(8, s.M, (s.batch * s.Hkv + 7) / 8), block(64 * ((s.G + 3) / 4));
    const float scale_log2 = kLog2e / sqrtf((float)s.D);
#define SPECPV_LAUNCH_K(NP, MULTI, NB, HALF)                                                                              \
    hipLaunchKernelGGL((combine_kernel<T, D, NP, MULTI, NB, HALF>), grid, block, 0, st, s.parent, s.q, (const float *)p.o, \
                       (const float *)p.ml, s.M, s.Hq, s.G, p.nsplit, s, p, out, lse, scale_log2)
#define SPECPV_LAUNCH_NP(NP, MULTI)                                                                                      \
    do {                                                                                                                \
        if (s.koff > s.kctx) { if (p.o_half) SPECPV_LAUNCH_K(NP, MULTI, 24, true); else SPECPV_LAUNCH_K(NP, MULTI, 24, false); } \
        else { if (p.o_half) SPECPV_LAUNCH_K(NP, MULTI, 8, true); else SPECPV_LAUNCH_K(NP, MULTI, 8, false); }           \
    } while (0)
    if (p.nsplit <= 2) SPECPV_LAUNCH_NP(2, false);
    else if (p.nsplit <= 4) SPECPV_LAUNCH_NP(4, false);
    else if (p.nsplit <= 8) SPECPV_LAUNCH_NP(8, false);
    else SPECPV_LAUNCH_NP(8, true);
#undef SPECPV_LAUNCH_NP
#undef SPECPV_LAUNCH_K
}

hipError_t launch_combine(const Shape &s, int dtype, Partials p, void *out, float *lse, hipStream_t st)
{
    if (dtype == SPECPV_BF16) {
        if (s.D == 128) launch_combine_t<bf16_t, 128>(s, p, out, lse, st); else launch_combine_t<bf16_t, 64>(s, p, out, lse, st);
    } else {
        if (s.D == 128) launch_combine_t<float, 128>(s, p, out, lse, st); else launch_combine_t<float, 64>(s, p, out, lse, st);
    }
    return hipGetLastError();
}

}  // namespace specpv
