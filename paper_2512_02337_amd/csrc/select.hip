// Block scoring (Section 3.2, eq. 2 and eq. 3) on the vector ALU for any dtype,
// and the per-(sequence, KV head) top-k selection of sink + retrieval + local
// blocks.  The MFMA scoring kernel for bf16 lives in score_mfma.hip.
#include "internal.h"

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

// Faster selection for lists of up to 256 * P blocks (P <= 16): thread t owns the P
// consecutive blocks t*P .. t*P+P-1 and keeps their scores in registers, so that
//   - the radix select reads memory once and only runs over the 32 score bits (4 passes of 8
//     bits; the histogram's suffix sums are one wavefront's work, without workgroup barriers);
//   - ties at the threshold score are broken towards the lower index by ranking the tied
//     blocks in index order (one workgroup-wide prefix sum) instead of four more radix passes;
//   - the ascending output comes from one more prefix sum over the per-thread keep counts.
__device__ __forceinline__ uint32_t score_bits(float score)
{
    if (score == 0.f) score = 0.f;  // -0 and +0 compare equal: give them one key
    const uint32_t u = __float_as_uint(score);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Wavefront scans and reductions through DPP (no LDS round trips).  row_shr:n shifts inside rows
// of 16 lanes (zeros come in), row_bcast:15 / row_bcast:31 carry the row totals on.
template <int CTRL, int ROW_MASK, bool ZERO_FILL>
__device__ __forceinline__ int dpp_i32(int v, int fill)
{
    return __builtin_amdgcn_update_dpp(fill, v, CTRL, ROW_MASK, 0xf, ZERO_FILL);
}
__device__ __forceinline__ int wave_inclusive_scan(int x)
{
    x += dpp_i32<0x111, 0xf, true>(x, 0);   // row_shr:1
    x += dpp_i32<0x112, 0xf, true>(x, 0);   // row_shr:2
    x += dpp_i32<0x114, 0xf, true>(x, 0);   // row_shr:4
    x += dpp_i32<0x118, 0xf, true>(x, 0);   // row_shr:8
    x += dpp_i32<0x142, 0xa, false>(x, 0);  // row_bcast:15 into rows 1 and 3
    x += dpp_i32<0x143, 0xc, false>(x, 0);  // row_bcast:31 into rows 2 and 3
    return x;
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x)
{
    x = min(x, (uint32_t)dpp_i32<0xB1, 0xf, false>((int)x, -1));
    x = min(x, (uint32_t)dpp_i32<0x4E, 0xf, false>((int)x, -1));
    x = min(x, (uint32_t)dpp_i32<0x141, 0xf, false>((int)x, -1));
    x = min(x, (uint32_t)dpp_i32<0x140, 0xf, false>((int)x, -1));
    x = min(x, (uint32_t)dpp_i32<0x142, 0xa, false>((int)x, -1));
    x = min(x, (uint32_t)dpp_i32<0x143, 0xc, false>((int)x, -1));
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x)
{
    x = max(x, (uint32_t)dpp_i32<0xB1, 0xf, false>((int)x, 0));
    x = max(x, (uint32_t)dpp_i32<0x4E, 0xf, false>((int)x, 0));
    x = max(x, (uint32_t)dpp_i32<0x141, 0xf, false>((int)x, 0));
    x = max(x, (uint32_t)dpp_i32<0x140, 0xf, false>((int)x, 0));
    x = max(x, (uint32_t)dpp_i32<0x142, 0xa, false>((int)x, 0));
    x = max(x, (uint32_t)dpp_i32<0x143, 0xc, false>((int)x, 0));
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

// exclusive prefix sum of v over the 256 threads (and the total), two barriers
__device__ __forceinline__ int block_exclusive_scan(int v, int *wave_tot, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int inc = wave_inclusive_scan(v);
    __syncthreads();   // wave_tot may still be read from a previous call
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int off = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (w < wave) off += wave_tot[w];
        total += wave_tot[w];
    }
    return off + inc - v;
}

template <int P>
__global__ __launch_bounds__(256) void topk_fast_kernel(const float *scores, const int32_t *ctx_len, int B,
                                                        int max_blocks, int Hkv, int ns, int nr, int k, int n_row,
                                                        int32_t *sel_idx, int32_t *sel_count)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_digit, sh_above;
    __shared__ uint32_t wave_min[4], wave_max_[4];
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, b = blockIdx.y;
    const int n_sel = ns + k + nr;
    const float *sc = scores + ((int64_t)b * Hkv + g) * max_blocks;
    int32_t *out = sel_idx + ((int64_t)b * Hkv + g) * n_row;   // n_row >= n_sel entries per row

    const int i0 = tid * P;
    // the scores are requested before the context length is known (any block below max_blocks
    // is readable), so the two cold reads overlap
    float raw[P];
#pragma unroll
    for (int j = 0; j < P; ++j) raw[j] = sc[min(i0 + j, max_blocks - 1)];
    const int L = ctx_len[b];
    int nb = L > 0 ? (L + B - 1) / B : 0;
    if (nb > max_blocks) nb = max_blocks;
    const bool all = nb <= n_sel;
    const int lo = ns, hi = nb - nr;          // candidates of the top-k: blocks lo .. hi-1
    const bool any_topk = !all && k > 0;      // then hi - lo > k
    uint32_t key[P];
    uint32_t cand = 0;                        // bit j: block i0 + j is a top-k candidate
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int i = i0 + j;
        const bool c = any_topk && i >= lo && i < hi;
        key[j] = c ? score_bits(raw[j]) : 0u;
        cand |= (c ? 1u : 0u) << j;
        if (c) { kmin = min(kmin, key[j]); kmax = max(kmax, key[j]); }
    }

    uint32_t prefix = 0;                      // threshold bits decided so far
    int krem = k;                             // how many of the keys that match prefix still belong to the top k
    if (any_topk) {
        // Smallest and largest key of the workgroup: the bits above the highest bit in which
        // they differ are common to all keys and need no pass.  Starting the digits right
        // there also spreads the first histogram over its bins (the leading bits of scores
        // of similar magnitude are all alike, and LDS atomics on one address serialise).
        kmin = wave_min_u32(kmin);
        kmax = wave_max_u32(kmax);
        if (lane == 0) { wave_min[wave] = kmin; wave_max_[wave] = kmax; }
        __syncthreads();
        kmin = min(min(wave_min[0], wave_min[1]), min(wave_min[2], wave_min[3]));
        kmax = max(max(wave_max_[0], wave_max_[1]), max(wave_max_[2], wave_max_[3]));
        const uint32_t diff = kmin ^ kmax;
        int top = diff ? 32 - __builtin_clz(diff) : 0;   // number of low bits that are not common to all keys
        prefix = top < 32 ? (kmax >> top) << top : 0u;
        while (top > 0) {
            const int width = top < 8 ? top : 8, shift = top - width;
            const uint32_t mask = (1u << width) - 1u;
            hist[tid] = 0;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < P; ++j)
                if (((cand >> j) & 1u) && (top >= 32 || (key[j] >> top) == (prefix >> top)))
                    atomicAdd(&hist[(key[j] >> shift) & mask], 1u);
            __syncthreads();
            if (wave == 0) {
                // lane l owns digits 4l .. 4l+3; suf[x] = number of matching keys with digit >= 4l + x
                const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
                // sum over the lanes above l = total - inclusive prefix of l
                const uint32_t mine = h0 + h1 + h2 + h3;
                const uint32_t pre = (uint32_t)wave_inclusive_scan((int)mine);
                const uint32_t all_keys = (uint32_t)__builtin_amdgcn_readlane((int)pre, 63);
                const uint32_t higher = all_keys - pre;              // keys with digit >= 4l + 4
                const uint32_t suf[5] = {higher + h3 + h2 + h1 + h0, higher + h3 + h2 + h1, higher + h3 + h2, higher + h3, higher};
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    if (suf[x] >= (uint32_t)krem && suf[x + 1] < (uint32_t)krem) {   // true for exactly one digit
                        sh_digit = (uint32_t)(4 * lane + x);
                        sh_above = suf[x + 1];
                    }
            }
            __syncthreads();
            prefix |= sh_digit << shift;
            krem -= (int)sh_above;
            top = shift;
        }
    }
    // prefix is the k-th largest score key; krem (>= 1) of the blocks that tie with it are kept,
    // lowest indices first
    uint32_t tie = 0;
#pragma unroll
    for (int j = 0; j < P; ++j)
        if (((cand >> j) & 1u) && key[j] == prefix) tie |= 1u << j;
    int tie_rank = 0, tie_total = 0;
    if (any_topk) tie_rank = block_exclusive_scan(__popc(tie), wave_tot, tie_total);
    uint32_t keep = 0;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int i = i0 + j;
        bool kp = false;
        if (i < nb) {
            kp = all || i < lo || i >= hi;
            if (!kp && ((cand >> j) & 1u)) {
                if (key[j] > prefix) kp = true;
                else if ((tie >> j) & 1u) { kp = tie_rank < krem; ++tie_rank; }
            }
        }
        keep |= (kp ? 1u : 0u) << j;
    }
    int total = 0;
    int pos = block_exclusive_scan(__popc(keep), wave_tot, total);
#pragma unroll
    for (int j = 0; j < P; ++j)
        if ((keep >> j) & 1u) {
            if (pos < n_sel) out[pos] = i0 + j;
            ++pos;
        }
    if (total > n_sel) total = n_sel;
    for (int c = total + tid; c < n_row; c += 256) out[c] = -1;
    if (tid == 0) sel_count[(int64_t)b * Hkv + g] = total;
}

bool score_mfma_supported(const Shape &s, int dtype);
hipError_t launch_scores_mfma(const Shape &s, const void *kmax, const void *kmin, int reduce,
                              int last_node, int kind, float *scores, hipStream_t st);

hipError_t launch_scores(const Shape &s, int dtype, const void *kmax, const void *kmin,
                         int reduce, int last_node, int kind, float *scores, hipStream_t st)
{
    if (score_mfma_supported(s, dtype))
        return launch_scores_mfma(s, kmax, kmin, reduce, last_node, kind, scores, st);
    return launch_scores_generic(s, dtype, kmax, kmin, reduce, last_node, kind, scores, st);
}

hipError_t launch_topk(const Shape &s, const float *scores, int ns, int nr, int k, int n_row,
                       int32_t *sel_idx, int32_t *sel_count, hipStream_t st)
{
    dim3 grid(s.Hkv, s.batch), block(256);
#define SPECPV_TOPK(KERN)                                                                        \
    hipLaunchKernelGGL(KERN, grid, block, 0, st, scores, s.ctx_len, s.B, s.max_blocks, s.Hkv, ns, nr, k, n_row, \
                       sel_idx, sel_count)
    if (s.max_blocks <= 256 * 4) SPECPV_TOPK(topk_fast_kernel<4>);
    else if (s.max_blocks <= 256 * 8) SPECPV_TOPK(topk_fast_kernel<8>);
    else if (s.max_blocks <= 256 * 16) SPECPV_TOPK(topk_fast_kernel<16>);
    else SPECPV_TOPK(topk_kernel);
#undef SPECPV_TOPK
    return hipGetLastError();
}

}  // namespace specpv
