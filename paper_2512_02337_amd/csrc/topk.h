// Selection of sink + retrieval + local blocks (Section 3.2) for lists of up to 256 * P blocks
// (P <= 16), as a device function: the selection kernel calls it, and so does the last workgroup
// of a (sequence, KV head) in the scoring kernel when the two run as one launch.
//
// The first 256 threads of the workgroup work: thread t owns the P consecutive blocks
// t*P .. t*P+P-1 and keeps their scores in registers, so that
//   - the radix select reads memory once and only runs over the score bits in which the
//     candidates differ (at most 4 passes of 8 bits, one barrier each);
//   - ties at the threshold score are broken towards the lower index by ranking the tied
//     blocks in index order instead of four more radix passes over the index bits;
//   - tie ranks and the ascending output positions come from one workgroup-wide prefix sum.
// Further threads of a larger workgroup own no blocks and only take part in the barriers.
#pragma once
#include "internal.h"

namespace specpv {

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

// Three histograms used in turn: pass p counts in histogram p % 3 and clears histogram (p + 1) % 3,
// which was last read two passes ago (before the previous barrier).  Entries 256 .. 319: one
// per lane, for the keys that are no longer in the race (never read).
struct TopkLds {
    __attribute__((aligned(16))) uint32_t hist[3][320];
    __attribute__((aligned(16))) uint32_t wave_min[4];
    __attribute__((aligned(16))) uint32_t wave_max[4];
    __attribute__((aligned(16))) uint32_t wave_tot[4];
};

// Every thread of the workgroup calls this (it holds workgroup barriers).  ACROSS: the scores
// were stored by other workgroups of the same launch with agent-scope stores and are read the
// same way, past the caches that are private to a part of the chip.
//
// What costs time here is the length of a wavefront's chain of dependent instructions and the
// number of barriers, not the arithmetic: a pass of the radix select is one round of LDS atomics,
// ONE barrier, and a suffix scan of the histogram that every wavefront does for itself; ties and
// output positions come from ONE more workgroup-wide prefix sum.
template <int P, bool ACROSS>
__device__ __forceinline__ void topk_fast_body(TopkLds &lds, const float *scores, const int32_t *ctx_len, int B,
                                               int max_blocks, int Hkv, int g, int b, const TopkArgs &a)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ns = a.ns, nr = a.nr, k = a.k, n_row = a.n_row;
    const int n_sel = ns + k + nr;
    const float *sc = scores + ((int64_t)b * Hkv + g) * max_blocks;
    int32_t *out = a.sel_idx + ((int64_t)b * Hkv + g) * n_row;

    const int i0 = tid * P;   // threads past 256 start behind the last block: they keep nothing
    // the scores are requested before the context length is known (any block below max_blocks
    // is readable), so the two cold reads overlap
    float raw[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const float *p = sc + min(i0 + j, max_blocks - 1);
        if (ACROSS)
            raw[j] = __uint_as_float(__hip_atomic_load((const uint32_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        else
            raw[j] = *p;
    }
    if (tid < 256) { lds.hist[0][tid] = 0; lds.hist[1][tid] = 0; }   // ahead of the first barrier below
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
    uint32_t live = cand;                     // bit j: key j matches the threshold in all bits decided so far
    if (any_topk) {
        // Smallest and largest key of the workgroup: the bits above the highest bit in which
        // they differ are common to all keys and need no pass.
        kmin = wave_min_u32(kmin);
        kmax = wave_max_u32(kmax);
        if (lane == 0 && wave < 4) { lds.wave_min[wave] = kmin; lds.wave_max[wave] = kmax; }
        __syncthreads();
        {
            const uint4 mn = *(const uint4 *)lds.wave_min, mx = *(const uint4 *)lds.wave_max;
            kmin = min(min(mn.x, mn.y), min(mn.z, mn.w));
            kmax = max(max(mx.x, mx.y), max(mx.z, mx.w));
        }
        const uint32_t diff = kmin ^ kmax;
        int top = diff ? 32 - __builtin_clz(diff) : 0;   // number of low bits that are not common to all keys
        prefix = top < 32 ? (kmax >> top) << top : 0u;
        int cur = 0;
        while (top > 0) {
            const int width = top < 8 ? top : 8, shift = top - width;
            const uint32_t mask = (1u << width) - 1u;
            const int nxt = cur == 2 ? 0 : cur + 1;
            if (tid < 256) lds.hist[nxt][tid] = 0;
            uint32_t dig[P];
#pragma unroll
            for (int j = 0; j < P; ++j) dig[j] = (key[j] >> shift) & mask;
            if (wave < 4) {
                // no branch per key: a key that is out of the race counts in its lane's own spare entry
#pragma unroll
                for (int j = 0; j < P; ++j)
                    atomicAdd(&lds.hist[cur][((live >> j) & 1u) ? dig[j] : 256u + (uint32_t)lane], 1u);
            }
            __syncthreads();
            // Every wavefront for itself: lane l owns digits 4l .. 4l+3; suf[x] = number of live keys with
            // digit >= 4l + x.  Exactly one (lane, x) has suf[x] >= krem > suf[x + 1]: that digit is the
            // threshold's, and suf[x + 1] keys lie above it.
            const uint4 h = *(const uint4 *)&lds.hist[cur][4 * lane];
            const uint32_t mine = h.x + h.y + h.z + h.w;
            const uint32_t pre = (uint32_t)wave_inclusive_scan((int)mine);
            const uint32_t higher = (uint32_t)__builtin_amdgcn_readlane((int)pre, 63) - pre;   // keys with digit >= 4l + 4
            const uint32_t s3 = higher + h.w, s2 = s3 + h.z, s1 = s2 + h.y, s0 = s1 + h.x;
            const uint32_t kr = (uint32_t)krem;
            const bool mine_has = s0 >= kr && higher < kr;
            const int x = s3 >= kr ? 3 : (s2 >= kr ? 2 : (s1 >= kr ? 1 : 0));      // the largest x with suf[x] >= krem
            const uint32_t above = x == 3 ? higher : (x == 2 ? s3 : (x == 1 ? s2 : s1));
            const int owner = __builtin_ctzll(__ballot(mine_has));
            const uint32_t digit = (uint32_t)(4 * owner + __builtin_amdgcn_readlane(x, owner));
            krem -= __builtin_amdgcn_readlane((int)above, owner);
            prefix |= digit << shift;
#pragma unroll
            for (int j = 0; j < P; ++j)
                if (dig[j] != digit) live &= ~(1u << j);
            top = shift;
            cur = nxt;
        }
    }
    // prefix is the k-th largest score key; the keys still live are the ones that tie with it, and krem
    // (>= 1) of those are kept, lowest indices first.  One prefix sum carries two counts: blocks that are
    // kept whatever the ties (low half) and tied blocks (high half), both at most 4096.
    uint32_t sure = 0;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int i = i0 + j;
        const bool fixed = i < nb && (all || i < lo || i >= hi);
        const bool won = ((cand >> j) & 1u) && key[j] > prefix;
        sure |= ((fixed || won) ? 1u : 0u) << j;
    }
    const uint32_t tie = any_topk ? live : 0u;
    const uint32_t packed = (uint32_t)__popc(sure) | ((uint32_t)__popc(tie) << 16);
    const uint32_t inc = (uint32_t)wave_inclusive_scan((int)packed);
    if (lane == 63 && wave < 4) lds.wave_tot[wave] = inc;
    __syncthreads();
    uint32_t before = inc - packed, total = 0;
    {
        const uint4 wt = *(const uint4 *)lds.wave_tot;
        const uint32_t w[4] = {wt.x, wt.y, wt.z, wt.w};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (v < wave) before += w[v];
            total += w[v];
        }
    }
    const int kr = krem;
    int sure_before = (int)(before & 0xffffu), tie_before = (int)(before >> 16);
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const bool is_sure = (sure >> j) & 1u, is_tie = (tie >> j) & 1u;
        const int pos = sure_before + min(tie_before, kr);    // kept blocks in front of this one
        if ((is_sure || (is_tie && tie_before < kr)) && pos < n_sel) out[pos] = i0 + j;
        sure_before += is_sure ? 1 : 0;
        tie_before += is_tie ? 1 : 0;
    }
    int n_kept = (int)(total & 0xffffu) + min((int)(total >> 16), any_topk ? kr : 0);
    if (n_kept > n_sel) n_kept = n_sel;
    for (int c = n_kept + tid; c < n_row; c += blockDim.x) out[c] = -1;
    if (tid == 0) a.sel_count[(int64_t)b * Hkv + g] = n_kept;
}

}  // namespace specpv
