// Context part of the verification attention on the vector ALU, for any
// supported dtype and head dim (used for fp32 and for shapes the MFMA kernel does
// not take).  One wavefront per (query head, node, KV split): lanes own tokens for
// q.k, then own channels for p.v.  Writes split-KV partials; combine.hip merges
// them and adds the draft-tree segment.
#include "internal.h"

namespace specpv {

template <typename T, int D>
__global__ __launch_bounds__(64) void attn_ctx_generic_kernel(Shape s, const int32_t *sel_idx,
                                                              const int32_t *sel_count, int n_sel,
                                                              Partials part, float scale_log2)
{
    constexpr int E = Elem<T>::kPerVec;
    constexpr int DPL = D / 64;  // channels per lane in the p.v phase
    __shared__ float qs[D];
    __shared__ float ps[64];
    __shared__ int toks[64];
    const int lane = threadIdx.x;
    const int sp = blockIdx.x, j = blockIdx.y;
    const int b = blockIdx.z / s.Hq, h = blockIdx.z % s.Hq, g = h / s.G;
    const int L = s.ctx_len[b];
    int nb = L > 0 ? (L + s.B - 1) / s.B : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    const int32_t *sel = sel_idx ? sel_idx + ((int64_t)b * s.Hkv + g) * n_sel : nullptr;
    int cnt = nb;
    if (sel) cnt = max(0, min(sel_count[(int64_t)b * s.Hkv + g], n_sel));
    const int64_t T_virtual = (int64_t)cnt * s.B;
    const int64_t C = (T_virtual + 63) / 64;
    const int64_t c0 = C * sp / part.nsplit, c1 = C * (sp + 1) / part.nsplit;

    for (int d = lane; d < D; d += 64)
        qs[d] = Elem<T>::load(s.q, (((int64_t)b * s.M + j) * s.Hq + h) * D + d);
    __syncthreads();
    const T *kbase = (const T *)s.k + (int64_t)b * s.sb + (int64_t)g * s.sh;
    const T *vbase = (const T *)s.v + (int64_t)b * s.sb + (int64_t)g * s.sh;

    float m = -INFINITY, l = 0.f, o[DPL];
#pragma unroll
    for (int x = 0; x < DPL; ++x) o[x] = 0.f;

    for (int64_t c = c0; c < c1; ++c) {
        const int64_t p = c * 64 + lane;
        int tok = -1;
        if (p < T_virtual) {
            const int slot = (int)(p / s.B);
            const int blk = sel ? sel[slot] : slot;
            if (blk >= 0 && blk < nb) {
                tok = blk * s.B + (int)(p % s.B);
                if (tok >= L) tok = -1;
            }
        }
        float z = -INFINITY;
        if (tok >= 0) {
            const T *kr = kbase + (int64_t)tok * s.st;
            float dot = 0.f;
#pragma unroll 4
            for (int d0 = 0; d0 < D; d0 += E) {
                float f[E];
                Elem<T>::unpack(*(const uint4 *)(kr + d0), f);
#pragma unroll
                for (int e = 0; e < E; ++e) dot = fmaf(qs[d0 + e], f[e], dot);
            }
            z = dot * scale_log2;
        }
        const float m_new = fmaxf(m, wave_max(z));
        if (m_new == -INFINITY) continue;  // wave-uniform: nothing valid so far
        const float alpha = exp2f(m - m_new);
        const float pe = tok >= 0 ? exp2f(z - m_new) : 0.f;
        l = l * alpha + wave_sum(pe);
        m = m_new;
#pragma unroll
        for (int x = 0; x < DPL; ++x) o[x] *= alpha;
        ps[lane] = pe;
        toks[lane] = tok;
        __syncthreads();
        for (int t = 0; t < 64; ++t) {
            const int tk = toks[t];
            if (tk < 0) continue;
            const float pt = ps[t];
            const T *vr = vbase + (int64_t)tk * s.st;
#pragma unroll
            for (int x = 0; x < DPL; ++x) o[x] = fmaf(pt, Elem<T>::load(vr, lane + 64 * x), o[x]);
        }
        __syncthreads();
    }
    const int64_t row = (((int64_t)b * s.Hq + h) * part.nsplit + sp) * s.M + j;
#pragma unroll
    for (int x = 0; x < DPL; ++x) __builtin_nontemporal_store(o[x], part.o + row * D + partial_pos(lane + 64 * x, D));   // written once, read once by the combine
    if (lane == 0) { part.ml[row * 2] = m; part.ml[row * 2 + 1] = l; }
}

hipError_t launch_attn_ctx_generic(const Shape &s, int dtype, const int32_t *sel_idx,
                                   const int32_t *sel_count, int n_sel, Partials p, hipStream_t st)
{
    dim3 grid(p.nsplit, s.M, s.batch * s.Hq), block(64);
    const float scale_log2 = kLog2e / sqrtf((float)s.D);
#define SPECPV_LAUNCH(T, DD) \
    hipLaunchKernelGGL((attn_ctx_generic_kernel<T, DD>), grid, block, 0, st, s, sel_idx, sel_count, n_sel, p, scale_log2)
    if (dtype == SPECPV_BF16) {
        if (s.D == 128) SPECPV_LAUNCH(bf16_t, 128); else SPECPV_LAUNCH(bf16_t, 64);
    } else {
        if (s.D == 128) SPECPV_LAUNCH(float, 128); else SPECPV_LAUNCH(float, 64);
    }
#undef SPECPV_LAUNCH
    return hipGetLastError();
}

}  // namespace specpv
