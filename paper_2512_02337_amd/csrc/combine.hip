// Final stage of the verification attention: for each (sequence, node, query
// head) attend over the draft-tree segment (the node itself and its ancestors,
// tree decode of Algorithm 1) on the vector ALU, merge that with the split-KV
// partials of the context part by their log-sum-exp weights, normalise and store.
// One wavefront per output row; lanes own channels.
#include "internal.h"

namespace specpv {

// Whole-wavefront sum / max through DPP (no LDS round trips: this kernel is a chain of
// dependent reductions): lane ^ 1, lane ^ 2, then the mirrors inside 8 and 16 lanes leave
// every lane of a row of 16 with the row's result; row_bcast:15 adds the end of rows 0 and 2
// into rows 1 and 3, row_bcast:31 the end of row 1 into rows 2 and 3; lane 63 holds the
// total, which readlane hands back as a wavefront-uniform value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_get(float v, float fill)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_u(float x)
{
    x += dpp_get<0xB1, 0xf>(x, 0.f);
    x += dpp_get<0x4E, 0xf>(x, 0.f);
    x += dpp_get<0x141, 0xf>(x, 0.f);
    x += dpp_get<0x140, 0xf>(x, 0.f);
    x += dpp_get<0x142, 0xa>(x, 0.f);
    x += dpp_get<0x143, 0xc>(x, 0.f);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}
__device__ __forceinline__ float wave_max_u(float x)
{
    x = fmaxf(x, dpp_get<0xB1, 0xf>(x, -INFINITY));
    x = fmaxf(x, dpp_get<0x4E, 0xf>(x, -INFINITY));
    x = fmaxf(x, dpp_get<0x141, 0xf>(x, -INFINITY));
    x = fmaxf(x, dpp_get<0x140, 0xf>(x, -INFINITY));
    x = fmaxf(x, dpp_get<0x142, 0xa>(x, -INFINITY));
    x = fmaxf(x, dpp_get<0x143, 0xc>(x, -INFINITY));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// A lane's DPL adjacent channels of one row, one memory instruction each way (rows are 16-byte aligned).
typedef float cmb_f32x2 __attribute__((ext_vector_type(2)));
template <typename T, int DPL> struct Chan;
template <> struct Chan<float, 1> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float *f) { f[0] = ((const float *)p)[i]; }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, const float *f) { __builtin_nontemporal_store(f[0], (float *)p + i); }
};
template <> struct Chan<float, 2> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float *f) {
        const cmb_f32x2 v = *(const cmb_f32x2 *)((const float *)p + i);
        f[0] = v.x; f[1] = v.y;
    }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, const float *f) {
        cmb_f32x2 v; v.x = f[0]; v.y = f[1];
        __builtin_nontemporal_store(v, (cmb_f32x2 *)((float *)p + i));
    }
};
template <> struct Chan<bf16_t, 1> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float *f) { f[0] = bf16_bits_to_float(((const uint16_t *)p)[i]); }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, const float *f) { __builtin_nontemporal_store(float_to_bf16_bits(f[0]), (uint16_t *)p + i); }
};
template <> struct Chan<bf16_t, 2> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float *f) {
        const uint32_t w = *(const uint32_t *)((const uint16_t *)p + i);
        f[0] = __uint_as_float(w << 16); f[1] = __uint_as_float(w & 0xffff0000u);
    }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, const float *f) {
        const uint32_t w = float_to_bf16_bits(f[0]) | ((uint32_t)float_to_bf16_bits(f[1]) << 16);
        __builtin_nontemporal_store(w, (uint32_t *)((uint16_t *)p + i));
    }
};
template <int DPL> __device__ __forceinline__ void load_partial(const float *p, int64_t i, float *f)
{
    if constexpr (DPL == 2) {
        const cmb_f32x2 v = __builtin_nontemporal_load((const cmb_f32x2 *)(p + i));
        f[0] = v.x; f[1] = v.y;
    } else {
        f[0] = __builtin_nontemporal_load(p + i);
    }
}

// NP: context partials fetched per round (the smallest of 2, 4, 8 that covers the split count in
// one round keeps the registers, and with them the resident wavefronts of a batch, in proportion).
template <typename T, int D, int NP>
__global__ __launch_bounds__(1024) void combine_kernel(const int32_t *a_parent, const void *a_q, const float *a_po,
                                                     const float *a_pml, int a_M, int a_Hq, int a_G, int a_nsplit,
                                                     Shape s, Partials part, void *out, float *lse, float scale_log2)
{
    // the leading scalar arguments repeat what the first round of reads needs; they can be preloaded into registers
    s.parent = a_parent; s.q = a_q; s.M = a_M; s.Hq = a_Hq; s.G = a_G;
    part.o = const_cast<float *>(a_po); part.ml = const_cast<float *>(a_pml); part.nsplit = a_nsplit;
    constexpr int DPL = D / 64;   // channels per lane: d = lane * DPL + x
    const int lane = threadIdx.x & 63;
    const int d0 = lane * DPL;
    const int g = blockIdx.y, b = blockIdx.z, j = blockIdx.x;
    const int h = g * s.G + (int)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // one wavefront per query head of the KV group

    // ---- every read whose address is known from the arguments goes out first ----------
    const int32_t *par = s.parent + (int64_t)b * s.M;
    const int par0 = lane < s.M ? par[lane] : -1;
    const int par1 = lane + 64 < s.M ? par[lane + 64] : -1;
    const int64_t qrow = (((int64_t)b * s.M + j) * s.Hq + h) * D;
    float qv[DPL];
    Chan<T, DPL>::load(s.q, qrow + d0, qv);
    const int64_t prow0 = (((int64_t)b * s.Hq + h) * part.nsplit) * s.M + j;
    float2 mlv = make_float2(-INFINITY, 0.f);   // lane sp holds (m, l) of split sp
    if (lane < part.nsplit) mlv = *(const float2 *)(part.ml + (prow0 + (int64_t)lane * s.M) * 2);

    // ... including the first NP context partials (all of them in the usual case)
    float po[NP][DPL];
#pragma unroll
    for (int u = 0; u < NP; ++u) {
        const int sp = min(u, part.nsplit - 1);
        const int64_t prow = prow0 + (int64_t)sp * s.M;
        load_partial<DPL>(part.o, prow * D + d0, po[u]);
    }

    // ---- root path of node j as a bit set (wave-uniform walk over the parent registers) --
    unsigned long long anc_lo = 0ull, anc_hi = 0ull;
    {
        int a = j;
        for (int guard = 0; a >= 0 && guard < s.M; ++guard) {
            if (a < 64) anc_lo |= 1ull << a; else anc_hi |= 1ull << (a - 64);
            const int pa = a < 64 ? __builtin_amdgcn_readlane(par0, a) : __builtin_amdgcn_readlane(par1, a - 64);
            a = pa < a ? pa : -1;   // a malformed parent[] (not strictly decreasing) ends the walk
        }
    }
    // ---- second (and last) round of reads: draft K / V of the first 8 nodes of the path ----
    auto pop = [&]() -> int {
        int a = -1;
        if (anc_lo) { a = __builtin_ctzll(anc_lo); anc_lo &= anc_lo - 1; }
        else if (anc_hi) { a = 64 + __builtin_ctzll(anc_hi); anc_hi &= anc_hi - 1; }
        return a;
    };
    int a8[8];
    float kd8[8][DPL], vd8[8][DPL];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        a8[u] = pop();
        const int64_t drow = (((int64_t)b * s.M + max(a8[u], 0)) * s.Hkv + g) * D;
        Chan<T, DPL>::load(s.kd, drow + d0, kd8[u]);
        Chan<T, DPL>::load(s.vd, drow + d0, vd8[u]);
    }

    // ---- context partials, merged relative to their own maximum (first-round data) -------
    const float m_ctx = wave_max_u(mlv.x);
    const float m_ctx_use = m_ctx == -INFINITY ? 0.f : m_ctx;
    const float w_mine = mlv.y > 0.f ? exp2f(mlv.x - m_ctx_use) : 0.f;
    const float l_ctx = wave_sum_u(mlv.y * w_mine);
    float o[DPL];
#pragma unroll
    for (int x = 0; x < DPL; ++x) o[x] = 0.f;
#pragma unroll
    for (int u = 0; u < NP; ++u) {
        const float w = u < part.nsplit ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_mine), u)) : 0.f;
#pragma unroll
        for (int x = 0; x < DPL; ++x) o[x] = fmaf(w, po[u][x], o[x]);
    }
    for (int sp0 = NP; sp0 < part.nsplit; sp0 += NP) {
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int sp = min(sp0 + u, part.nsplit - 1);
            const int64_t prow = prow0 + (int64_t)sp * s.M;
            load_partial<DPL>(part.o, prow * D + d0, po[u]);
        }
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const float w = sp0 + u < part.nsplit ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_mine), sp0 + u)) : 0.f;
#pragma unroll
            for (int x = 0; x < DPL; ++x) o[x] = fmaf(w, po[u][x], o[x]);
        }
    }

    // ---- draft-tree segment: the node itself and its ancestors --------------------------
    float m = -INFINITY, l = 0.f, od[DPL];
#pragma unroll
    for (int x = 0; x < DPL; ++x) od[x] = 0.f;
    // online softmax over four nodes (slots without a node have a[u] < 0 and weigh nothing)
    auto four = [&](const int *a, float (*kdv)[DPL], float (*vdv)[DPL]) {
        float z[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float dot = 0.f;
#pragma unroll
            for (int x = 0; x < DPL; ++x) dot = fmaf(qv[x], kdv[u][x], dot);
            z[u] = a[u] >= 0 ? wave_sum_u(dot) * scale_log2 : -INFINITY;
        }
        const float m_new = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), m);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m - m_use);
        l *= alpha;
#pragma unroll
        for (int x = 0; x < DPL; ++x) od[x] *= alpha;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float pe = exp2f(z[u] - m_use);   // 0 for the unused slots
            l += pe;
#pragma unroll
            for (int x = 0; x < DPL; ++x) od[x] = fmaf(pe, vdv[u][x], od[x]);
        }
        m = m_new;
    };
    four(a8, kd8, vd8);
    if (a8[4] >= 0) four(a8 + 4, kd8 + 4, vd8 + 4);
    while (anc_lo | anc_hi) {   // paths longer than 8 nodes
        int a[4];
        float kdv[4][DPL], vdv[4][DPL];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a[u] = pop();
            const int64_t drow = (((int64_t)b * s.M + max(a[u], 0)) * s.Hkv + g) * D;
            Chan<T, DPL>::load(s.kd, drow + d0, kdv[u]);
            Chan<T, DPL>::load(s.vd, drow + d0, vdv[u]);
        }
        four(a, kdv, vdv);
    }

    // ---- merge the two and store ---------------------------------------------------------
    const float m_all = fmaxf(m, m_ctx);
    const float wd = exp2f(m - m_all);
    const float wc = m_ctx == -INFINITY ? 0.f : exp2f(m_ctx - m_all);
    const float den = l * wd + l_ctx * wc;
    const float inv = 1.f / den;
    float res[DPL];
#pragma unroll
    for (int x = 0; x < DPL; ++x) res[x] = (od[x] * wd + o[x] * wc) * inv;
    Chan<T, DPL>::store_stream(out, qrow + d0, res);
    if (lse && lane == 0) lse[((int64_t)b * s.M + j) * s.Hq + h] = (m_all + log2f(den)) * kLn2;
}

hipError_t launch_combine(const Shape &s, int dtype, Partials p, void *out, float *lse, hipStream_t st)
{
    dim3 grid(s.M, s.Hkv, s.batch), block(64 * s.G);
    const float scale_log2 = kLog2e / sqrtf((float)s.D);
#define SPECPV_LAUNCH_NP(T, DD, NP) \
    hipLaunchKernelGGL((combine_kernel<T, DD, NP>), grid, block, 0, st, s.parent, s.q, (const float *)p.o, (const float *)p.ml, s.M, s.Hq, s.G, p.nsplit, s, p, out, lse, scale_log2)
#define SPECPV_LAUNCH(T, DD) \
    do { \
        if (p.nsplit <= 2) SPECPV_LAUNCH_NP(T, DD, 2); \
        else if (p.nsplit <= 4) SPECPV_LAUNCH_NP(T, DD, 4); \
        else SPECPV_LAUNCH_NP(T, DD, 8); \
    } while (0)
    if (dtype == SPECPV_BF16) {
        if (s.D == 128) SPECPV_LAUNCH(bf16_t, 128); else SPECPV_LAUNCH(bf16_t, 64);
    } else {
        if (s.D == 128) SPECPV_LAUNCH(float, 128); else SPECPV_LAUNCH(float, 64);
    }
#undef SPECPV_LAUNCH
#undef SPECPV_LAUNCH_NP
    return hipGetLastError();
}

}  // namespace specpv
