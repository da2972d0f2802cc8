// Block scoring (Section 3.2, eq. 2 and eq. 3) on the vector ALU for any dtype,
// and the per-(sequence, KV head) top-k selection of sink + retrieval + local
// blocks.  The MFMA scoring kernel for bf16 lives in score_mfma.hip.
#include "internal.h"
#include "topk.h"

namespace specpv {

// ---------------------------------------------------------------------------
// Generic scoring: one lane owns one block; the query rows are staged through
// LDS 32 at a time and broadcast to all lanes.  fp32 FMA, channels in ascending
// order, rows in ascending order, so a block's score does not depend on where
// the block sits in the grid.
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(64) void score_generic_kernel(Shape s, const void *kmax, const void *kmin,
                                                          int reduce, int last_node, int kind, float *scores)
{
    constexpr int RC = 32;  // query rows per LDS pass
    __shared__ float qs[RC][D];
    const int lane = threadIdx.x;
    const int g = blockIdx.y, b = blockIdx.z;
    const int L = s.ctx_len[b];
    int nb = L > 0 ? (L + s.B - 1) / s.B : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    if ((int)blockIdx.x * 64 >= nb) return;
    const int i = blockIdx.x * 64 + lane;
    const bool valid = i < nb;
    const int R = s.M * s.G;
    const int64_t so = (((int64_t)b * s.Hkv + g) * s.max_blocks + (valid ? i : 0)) * D;
    float acc_sum = 0.f, acc_max = -INFINITY;
    for (int r0 = 0; r0 < R; r0 += RC) {
        const int nrows = min(RC, R - r0);
        __syncthreads();
        for (int x = lane; x < RC * D; x += 64) {
            const int r = x / D, d = x % D;
            float val = 0.f;
            if (r < nrows) {
                const int j = (r0 + r) / s.G, hh = (r0 + r) % s.G;
                val = Elem<T>::load(s.q, (((int64_t)b * s.M + j) * s.Hq + g * s.G + hh) * D + d);
            }
            qs[r][d] = val;
        }
        __syncthreads();
        float am[RC], an[RC];
#pragma unroll
        for (int r = 0; r < RC; ++r) { am[r] = 0.f; an[r] = 0.f; }
        for (int d0 = 0; d0 < D; d0 += 8) {
            float kx[8], kn[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                kx[e] = Elem<T>::load(kmax, so + d0 + e);
                kn[e] = Elem<T>::load(kmin, so + d0 + e);
            }
            if (kind == SPECPV_SCORE_CHANNEL_BOUND) {
                // per channel the larger product: q * Kmax where q >= 0, q * Kmin where q < 0 (Kmax >= Kmin)
#pragma unroll
                for (int r = 0; r < RC; ++r) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float qv = qs[r][d0 + e];
                        am[r] = fmaf(qv, qv < 0.f ? kn[e] : kx[e], am[r]);
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < RC; ++r) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float qv = qs[r][d0 + e];
                        am[r] = fmaf(qv, kx[e], am[r]);
                        an[r] = fmaf(qv, kn[e], an[r]);
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            if (r < nrows) {
                const float sv = kind == SPECPV_SCORE_CHANNEL_BOUND ? am[r] : fmaxf(am[r], an[r]);
                if (reduce == SPECPV_REDUCE_MAX) acc_max = fmaxf(acc_max, sv);
                else if (reduce == SPECPV_REDUCE_MEAN) acc_sum += sv;
                else if ((r0 + r) / s.G == last_node) acc_sum += sv;
            }
        }
    }
    float out;
    if (reduce == SPECPV_REDUCE_MAX) out = acc_max;
    else if (reduce == SPECPV_REDUCE_MEAN) out = acc_sum / (float)R;
    else out = acc_sum / (float)s.G;
    if (valid) scores[((int64_t)b * s.Hkv + g) * s.max_blocks + i] = out;
}

static hipError_t launch_scores_generic(const Shape &s, int dtype, const void *kmax, const void *kmin,
                                 int reduce, int last_node, int kind, float *scores, hipStream_t st)
{
    dim3 grid((s.max_blocks + 63) / 64, s.Hkv, s.batch), block(64);
#define SPECPV_LAUNCH(T, DD) \
    hipLaunchKernelGGL((score_generic_kernel<T, DD>), grid, block, 0, st, s, kmax, kmin, reduce, last_node, kind, scores)
    if (dtype == SPECPV_BF16) {
        if (s.D == 128) SPECPV_LAUNCH(bf16_t, 128); else SPECPV_LAUNCH(bf16_t, 64);
    } else {
        if (s.D == 128) SPECPV_LAUNCH(float, 128); else SPECPV_LAUNCH(float, 64);
    }
#undef SPECPV_LAUNCH
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Selection.  One 256-thread workgroup per (sequence, KV head).
// Every candidate block gets the 64-bit key  (orderable(score) << 32) | ~index,
// so "larger key" means "higher fp32 score, then lower index", and keys are
// unique.  The k-th largest key is found by an MSB-first radix select (8 passes
// of 8 bits, LDS histogram); the kept set is then every candidate with key >=
// that threshold plus the sink and local blocks, written in ascending block
// order through a ballot / popcount compaction.
// ---------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long select_key(float score, int idx)
{
    if (score == 0.f) score = 0.f;  // -0 and +0 compare equal: give them one key
    uint32_t u = __float_as_uint(score);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)u << 32) | (unsigned long long)(0xffffffffu - (uint32_t)idx);
}

__global__ __launch_bounds__(256) void topk_kernel(const float *scores, const int32_t *ctx_len, int B,
                                                   int max_blocks, int Hkv, int ns, int nr, int k, int n_row,
                                                   int32_t *sel_idx, int32_t *sel_count)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t suffix[257];
    __shared__ unsigned long long sh_prefix;
    __shared__ int sh_krem;
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, b = blockIdx.y;
    const int n_sel = ns + k + nr;
    const int L = ctx_len[b];
    int nb = L > 0 ? (L + B - 1) / B : 0;
    if (nb > max_blocks) nb = max_blocks;
    const float *sc = scores + ((int64_t)b * Hkv + g) * max_blocks;
    int32_t *out = sel_idx + ((int64_t)b * Hkv + g) * n_row;   // n_row >= n_sel entries per row
    const bool all = nb <= n_sel;
    const int lo = ns, hi = nb - nr;
    unsigned long long thresh = ~0ull;
    bool any_topk = false;
    if (!all && k > 0) {   // here hi - lo > k
        any_topk = true;
        if (tid == 0) { sh_prefix = 0ull; sh_krem = k; }
        __syncthreads();
        for (int pass = 0; pass < 8; ++pass) {
            const int shift = 56 - 8 * pass;
            const unsigned long long prefix = sh_prefix;
            const int krem = sh_krem;
            hist[tid] = 0;
            __syncthreads();
            for (int i = lo + tid; i < hi; i += 256) {
                const unsigned long long key = select_key(sc[i], i);
                if (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)))
                    atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            // suffix[d] = number of matching keys whose digit is >= d
            suffix[tid] = hist[tid];
            if (tid == 0) suffix[256] = 0;
            __syncthreads();
            for (int off = 1; off < 256; off <<= 1) {
                const uint32_t add = (tid + off < 256) ? suffix[tid + off] : 0u;
                __syncthreads();
                suffix[tid] += add;
                __syncthreads();
            }
            if (suffix[tid] >= (uint32_t)krem && suffix[tid + 1] < (uint32_t)krem) {
                sh_prefix = prefix | ((unsigned long long)tid << shift);
                sh_krem = krem - (int)suffix[tid + 1];
            }
            __syncthreads();
        }
        thresh = sh_prefix;
    }
    int base = 0;
    for (int i0 = 0; i0 < nb; i0 += 256) {
        const int i = i0 + tid;
        bool keep = false;
        if (i < nb) {
            keep = all || i < lo || i >= hi;
            if (!keep && any_topk) keep = select_key(sc[i], i) >= thresh;
        }
        const unsigned long long bal = __ballot(keep);
        if (lane == 0) wave_tot[wave] = __popcll(bal);
        __syncthreads();
        int pos = base + __popcll(bal & ((1ull << lane) - 1ull));
        int tot = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) pos += wave_tot[w];
            tot += wave_tot[w];
        }
        if (keep && pos < n_sel) out[pos] = i;
        base += tot;
        __syncthreads();
    }
    if (base > n_sel) base = n_sel;
    for (int c = base + tid; c < n_row; c += 256) out[c] = -1;
    if (tid == 0) sel_count[(int64_t)b * Hkv + g] = base;
}

// Faster selection for lists of up to 256 * P blocks (P <= 16): see topk.h.
template <int P>
__global__ __launch_bounds__(256) void topk_fast_kernel(const float *scores, const int32_t *ctx_len, int B,
                                                        int max_blocks, int Hkv, TopkArgs a)
{
    __shared__ TopkLds lds;
    topk_fast_body<P, false>(lds, scores, ctx_len, B, max_blocks, Hkv, blockIdx.x, blockIdx.y, a);
}

bool score_mfma_supported(const Shape &s, int dtype);
hipError_t launch_scores_mfma(const Shape &s, const void *kmax, const void *kmin, int reduce,
                              int last_node, int kind, float *scores, const TopkArgs *sel,
                              unsigned long long *arrive, hipStream_t st);

hipError_t launch_scores(const Shape &s, int dtype, const void *kmax, const void *kmin,
                         int reduce, int last_node, int kind, float *scores, const TopkArgs *sel,
                         unsigned long long *arrive, hipStream_t st)
{
    if (score_mfma_supported(s, dtype))
        return launch_scores_mfma(s, kmax, kmin, reduce, last_node, kind, scores, sel, arrive, st);
    if (sel) return hipErrorInvalidValue;   // the caller asks score_select_supported() first
    return launch_scores_generic(s, dtype, kmax, kmin, reduce, last_node, kind, scores, st);
}

hipError_t launch_topk(const Shape &s, const float *scores, int ns, int nr, int k, int n_row,
                       int32_t *sel_idx, int32_t *sel_count, hipStream_t st)
{
    dim3 grid(s.Hkv, s.batch), block(256);
    const TopkArgs a{ns, nr, k, n_row, sel_idx, sel_count};
#define SPECPV_TOPK(KERN) \
    hipLaunchKernelGGL(KERN, grid, block, 0, st, scores, s.ctx_len, s.B, s.max_blocks, s.Hkv, a)
    if (s.max_blocks <= 256 * 4) SPECPV_TOPK(topk_fast_kernel<4>);
    else if (s.max_blocks <= 256 * 8) SPECPV_TOPK(topk_fast_kernel<8>);
    else if (s.max_blocks <= 256 * 16) SPECPV_TOPK(topk_fast_kernel<16>);
    else
        hipLaunchKernelGGL(topk_kernel, grid, block, 0, st, scores, s.ctx_len, s.B, s.max_blocks, s.Hkv, ns, nr, k, n_row,
                           sel_idx, sel_count);
#undef SPECPV_TOPK
    return hipGetLastError();
}

}  // namespace specpv
