// Final stage of the verification attention: for each (sequence, node, query
// head) attend over the draft-tree segment (the node itself and its ancestors,
// tree decode of Algorithm 1) on the vector ALU, merge that with the split-KV
// partials of the context part by their log-sum-exp weights, normalise and store.
// One wavefront per output row; lanes own channels.
#include "internal.h"

namespace specpv {

template <typename T, int D>
__global__ __launch_bounds__(64) void combine_kernel(Shape s, Partials part, void *out, float *lse,
                                                     float scale_log2)
{
    constexpr int DPL = D / 64;
    __shared__ int par[SPECPV_MAX_M];
    __shared__ int anc[SPECPV_MAX_M];
    __shared__ int n_anc_sh;
    const int lane = threadIdx.x;
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z, g = h / s.G;
    for (int x = lane; x < s.M; x += 64) par[x] = s.parent[(int64_t)b * s.M + x];
    __syncthreads();
    if (lane == 0) {
        // root path of node j; a malformed parent[] (not strictly decreasing) ends the walk
        int n = 0, a = j;
        while (a >= 0 && n < s.M) {
            anc[n++] = a;
            const int pa = par[a];
            a = (pa < a) ? pa : -1;
        }
        n_anc_sh = n;
    }
    __syncthreads();
    const int n_anc = n_anc_sh;

    float qv[DPL], o[DPL];
    const int64_t qrow = (((int64_t)b * s.M + j) * s.Hq + h) * D;
#pragma unroll
    for (int x = 0; x < DPL; ++x) { qv[x] = Elem<T>::load(s.q, qrow + lane + 64 * x); o[x] = 0.f; }
    float m = -INFINITY, l = 0.f;
    for (int n = 0; n < n_anc; ++n) {
        const int64_t drow = (((int64_t)b * s.M + anc[n]) * s.Hkv + g) * D;
        float dot = 0.f;
#pragma unroll
        for (int x = 0; x < DPL; ++x) dot = fmaf(qv[x], Elem<T>::load(s.kd, drow + lane + 64 * x), dot);
        const float z = wave_sum(dot) * scale_log2;
        const float m_new = fmaxf(m, z);
        const float alpha = exp2f(m - m_new), pe = exp2f(z - m_new);
        l = l * alpha + pe;
#pragma unroll
        for (int x = 0; x < DPL; ++x)
            o[x] = fmaf(pe, Elem<T>::load(s.vd, drow + lane + 64 * x), o[x] * alpha);
        m = m_new;
    }
    // merge with the context partials
    const int64_t prow0 = (((int64_t)b * s.Hq + h) * part.nsplit) * s.M + j;
    float m_all = m;
    for (int sp = 0; sp < part.nsplit; ++sp)
        m_all = fmaxf(m_all, part.ml[(prow0 + (int64_t)sp * s.M) * 2]);
    const float wd = exp2f(m - m_all);
    float den = l * wd;
#pragma unroll
    for (int x = 0; x < DPL; ++x) o[x] *= wd;
    for (int sp = 0; sp < part.nsplit; ++sp) {
        const int64_t prow = prow0 + (int64_t)sp * s.M;
        const float ms = part.ml[prow * 2], ls = part.ml[prow * 2 + 1];
        if (ls == 0.f) continue;  // split without valid tokens
        const float w = exp2f(ms - m_all);
        den = fmaf(ls, w, den);
#pragma unroll
        for (int x = 0; x < DPL; ++x) o[x] = fmaf(w, part.o[prow * D + lane + 64 * x], o[x]);
    }
    const float inv = 1.f / den;
#pragma unroll
    for (int x = 0; x < DPL; ++x) Elem<T>::store(out, qrow + lane + 64 * x, o[x] * inv);
    if (lse && lane == 0) lse[((int64_t)b * s.M + j) * s.Hq + h] = (m_all + log2f(den)) * kLn2;
}

hipError_t launch_combine(const Shape &s, int dtype, Partials p, void *out, float *lse, hipStream_t st)
{
    dim3 grid(s.M, s.Hq, s.batch), block(64);
    const float scale_log2 = kLog2e / sqrtf((float)s.D);
#define SPECPV_LAUNCH(T, DD) \
    hipLaunchKernelGGL((combine_kernel<T, DD>), grid, block, 0, st, s, p, out, lse, scale_log2)
    if (dtype == SPECPV_BF16) {
        if (s.D == 128) SPECPV_LAUNCH(bf16_t, 128); else SPECPV_LAUNCH(bf16_t, 64);
    } else {
        if (s.D == 128) SPECPV_LAUNCH(float, 128); else SPECPV_LAUNCH(float, 64);
    }
#undef SPECPV_LAUNCH
    return hipGetLastError();
}

}  // namespace specpv
