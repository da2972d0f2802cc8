// Block key summaries (Section 3.2, eq. 1): element-wise max and min of the keys
// of each block.  Pure HBM streaming: one wavefront per (block, KV head), 16-byte
// loads, the lanes that share a channel group are folded with cross-lane shuffles.
#include "internal.h"
#ifndef SPECPV_SUM_UNR
#define SPECPV_SUM_UNR 16
#endif

namespace specpv {

// 16-byte read of data that is used once: keep it from displacing what the caches hold
__device__ __forceinline__ uint4 load_stream(const uint4 *p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void summarize_kernel(Shape s, int blk_begin, int blk_end,
                                                        void *kmax, void *kmin)
{
    constexpr int E = Elem<T>::kPerVec;   // elements per 16-byte load
    constexpr int LPR = D / E;            // lanes that cover one token row
    constexpr int RPP = 64 / LPR;         // token rows per wavefront pass
    static_assert(D % E == 0 && LPR <= 64 && 64 % LPR == 0, "head dim does not tile a wavefront");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = blockIdx.y, b = blockIdx.z;
    const int L = s.ctx_len[b];
    if (L <= 0) return;
    int nb = (L + s.B - 1) / s.B;
    if (nb > s.max_blocks) nb = s.max_blocks;
    const int end = (blk_end < 0 || blk_end > nb) ? nb : blk_end;
    const int i = blk_begin + blockIdx.x * 4 + wave;
    if (i >= end) return;
    const int t0 = i * s.B;
    const int t1 = min(t0 + s.B, L);
    const int c = lane % LPR, rsub = lane / LPR;
    const T *base = (const T *)s.k + (int64_t)b * s.sb + (int64_t)g * s.sh + c * E;
    float mx[E], mn[E];
#pragma unroll
    for (int e = 0; e < E; ++e) { mx[e] = -INFINITY; mn[e] = INFINITY; }
    // UNR independent 16-byte loads per lane in flight: the kernel is bound by the bytes it
    // keeps in flight against the memory latency
    constexpr int UNR = SPECPV_SUM_UNR;
    int t = t0 + rsub;
    for (; t + (UNR - 1) * RPP < t1; t += UNR * RPP) {
        uint4 u[UNR];
#pragma unroll
        for (int x = 0; x < UNR; ++x) u[x] = load_stream((const uint4 *)(base + (int64_t)(t + x * RPP) * s.st));
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            float f[E];
            Elem<T>::unpack(u[x], f);
#pragma unroll
            for (int e = 0; e < E; ++e) { mx[e] = fmaxf(mx[e], f[e]); mn[e] = fminf(mn[e], f[e]); }
        }
    }
    for (; t < t1; t += RPP) {
        const uint4 u = *(const uint4 *)(base + (int64_t)t * s.st);
        float f[E];
        Elem<T>::unpack(u, f);
#pragma unroll
        for (int e = 0; e < E; ++e) { mx[e] = fmaxf(mx[e], f[e]); mn[e] = fminf(mn[e], f[e]); }
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], off));
            mn[e] = fminf(mn[e], __shfl_xor(mn[e], off));
        }
    }
    if (rsub == 0) {
        const int64_t o = (((int64_t)b * s.Hkv + g) * s.max_blocks + i) * D + c * E;
        // one 16-byte store per array (o is a multiple of E elements)
        *(uint4 *)((T *)kmax + o) = Elem<T>::pack(mx);
        *(uint4 *)((T *)kmin + o) = Elem<T>::pack(mn);
    }
}

hipError_t launch_summarize(const Shape &s, int dtype, int blk_begin, int blk_end,
                            void *kmax, void *kmin, hipStream_t st)
{
    const int hi = (blk_end < 0 || blk_end > s.max_blocks) ? s.max_blocks : blk_end;
    if (hi <= blk_begin) return hipSuccess;
    dim3 grid((hi - blk_begin + 3) / 4, s.Hkv, s.batch), block(256);
#define SPECPV_LAUNCH(T, DD) \
    hipLaunchKernelGGL((summarize_kernel<T, DD>), grid, block, 0, st, s, blk_begin, blk_end, kmax, kmin)
    if (dtype == SPECPV_BF16) {
        if (s.D == 128) SPECPV_LAUNCH(bf16_t, 128); else SPECPV_LAUNCH(bf16_t, 64);
    } else {
        if (s.D == 128) SPECPV_LAUNCH(float, 128); else SPECPV_LAUNCH(float, 64);
    }
#undef SPECPV_LAUNCH
    return hipGetLastError();
}

}  // namespace specpv
