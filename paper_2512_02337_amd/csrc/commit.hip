// KV side of what follows a verify step (Section 3.2: the candidates' K/V wait in the buffer
// until verification has decided which of them survive; Section 3.3: a full verification
// moves the partially verified tokens into the cache).  Pure data
// movement of at most a few dozen rows per (sequence, KV head), then the block summaries
// (eq. 1) of the blocks that received tokens.
#include "internal.h"

namespace specpv {

constexpr int kCommitMaxRows = 128;   // pending + accepted rows one call moves per sequence (host-checked)

// One workgroup per (KV head, sequence); a row of D elements is D * sizeof(T) / 16 lanes.
// Every source row is read into registers before anything is written (the compaction of
// the buffer moves rows within one array).
// Several layers in one launch: blockIdx.z picks the layer's pointers from a table that travels
// with the kernel arguments.  All layers share one shape, one set of strides and the counters.
constexpr int kCommitLayers = 32;   // layers per launch
struct CommitLayers {
    void *k[kCommitLayers], *v[kCommitLayers], *buf_k[kCommitLayers], *buf_v[kCommitLayers];
    void *kmax[kCommitLayers], *kmin[kCommitLayers];
};

template <typename T, int D>
__global__ __launch_bounds__(256) void commit_copy_kernel(Shape s, CommitLayers lay, int P, int Mt,
                                                          const int32_t *n_pending, const int32_t *accepted,
                                                          const int32_t *n_accepted, int max_accept, int to_cache)
{
    T *const buf_k = (T *)lay.buf_k[blockIdx.z], *const buf_v = (T *)lay.buf_v[blockIdx.z];
    s.k = lay.k[blockIdx.z];
    s.v = lay.v[blockIdx.z];
    constexpr int LPR = D * (int)sizeof(T) / 16;   // lanes per row
    constexpr int RPP = 256 / LPR;                 // rows per pass
    constexpr int PASSES = (kCommitMaxRows + RPP - 1) / RPP;
    const int g = blockIdx.x, b = blockIdx.y;
    const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
    const int L = s.ctx_len[b];
    const int n = min(max(n_pending[b], 0), P);
    int a = min(max(n_accepted[b], 0), max_accept);
    int total = n + a;
    if (to_cache) total = min(total, max(0, s.max_blocks * s.B - L));   // the cache is full: the rest is dropped
    else total = min(total, P);
    const int64_t buf_rows = (int64_t)P + Mt;
    auto buf_row = [&](T *base, int row) -> uint4 * {
        return (uint4 *)(base + (((int64_t)b * buf_rows + row) * s.Hkv + g) * D) + c;
    };
    uint4 kr[PASSES], vr[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int i = p * RPP + r0;
        if (i < total) {
            int src;
            if (i < n) src = P - n + i;                             // pending token i (oldest first)
            else src = P + min(max(accepted[(int64_t)b * max_accept + (i - n)], 0), Mt - 1);   // accepted candidate
            kr[p] = *buf_row(buf_k, src);
            vr[p] = *buf_row(buf_v, src);
        }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int i = p * RPP + r0;
        if (i < total) {
            if (to_cache) {
                const int64_t off = (int64_t)b * s.sb + (int64_t)g * s.sh + (int64_t)(L + i) * s.st;
                *((uint4 *)((T *)s.k + off) + c) = kr[p];
                *((uint4 *)((T *)s.v + off) + c) = vr[p];
            } else {
                *buf_row(buf_k, P - total + i) = kr[p];
                *buf_row(buf_v, P - total + i) = vr[p];
            }
        }
    }
}

// One thread per sequence, after the copies: the new lengths (the old committed length goes to
// old_len for the summary update).
__global__ void commit_update_kernel(Shape s, int P, int32_t *ctx_len, int32_t *n_pending,
                                     const int32_t *n_accepted, int max_accept, int to_cache, int32_t *old_len,
                                     int32_t *dropped)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= s.batch) return;
    const int L = ctx_len[b];
    const int n = min(max(n_pending[b], 0), P);
    const int a = min(max(n_accepted[b], 0), max_accept);
    old_len[b] = L;
    int stored;
    if (to_cache) {
        stored = min(n + a, max(0, s.max_blocks * s.B - L));
        ctx_len[b] = L + stored;
        n_pending[b] = 0;
    } else {
        stored = min(n + a, P);
        n_pending[b] = stored;
    }
    if (dropped) {
        dropped[2 * b] = n + a - stored;   // tokens that found no room
        dropped[2 * b + 1] = 0;            // list entries that found no room: commit_extend_lists_kernel
    }
}

// After a commit to the cache (Section 3.3: the committed tokens stay part of the partial cache):
// every block that holds one of the tokens old_len .. new length - 1 joins the kept-block list of
// each KV head, behind the entries it has, unless the block is listed already (the ragged last
// block of the local window).  One wavefront per (KV head, sequence, layer).
struct CommitLists {
    int32_t *idx[kCommitLayers], *cnt[kCommitLayers];
};
__global__ __launch_bounds__(64) void commit_extend_lists_kernel(Shape s, CommitLists ls, int n_sel,
                                                                 const int32_t *old_len, int32_t *dropped)
{
    const int g = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int L = s.ctx_len[b], L0 = old_len[b];
    if (L <= L0) return;
    int32_t *row = ls.idx[blockIdx.z] + ((int64_t)b * s.Hkv + g) * n_sel;
    int32_t *cntp = ls.cnt[blockIdx.z] + (int64_t)b * s.Hkv + g;
    const int cnt0 = min(max(*cntp, 0), n_sel);
    const int first = L0 / s.B, last = (L - 1) / s.B;
    int cnt = cnt0, missed = 0;
    for (int blk = first; blk <= last; ++blk) {
        bool here = false;
        for (int i = lane; i < cnt0; i += 64) here |= row[i] == blk;
        if (__any(here)) continue;
        if (cnt < n_sel) { if (lane == 0) row[cnt] = blk; ++cnt; }
        else ++missed;
    }
    if (lane == 0) {
        *cntp = cnt;
        if (missed && dropped) atomicMax(&dropped[2 * b + 1], missed);
    }
}

// eq. 1 for the blocks old_len / B .. (new length - 1) / B of every sequence: one wavefront per
// (block, KV head), lanes over 16-byte pieces of a row, rows strided over the lane groups.
template <typename T, int D>
__global__ __launch_bounds__(64) void summarize_tail_kernel(Shape s, CommitLayers lay, const int32_t *old_len)
{
    constexpr int E = Elem<T>::kPerVec;
    constexpr int LPR = D / E;
    constexpr int RPP = 64 / LPR;
    const int layer = blockIdx.z / s.batch;
    const int lane = threadIdx.x, g = blockIdx.y, b = blockIdx.z - layer * s.batch;
    void *const kmax = lay.kmax[layer], *const kmin = lay.kmin[layer];
    s.k = lay.k[layer];
    const int L = s.ctx_len[b], L0 = old_len[b];
    if (L <= L0) return;
    const int i = L0 / s.B + blockIdx.x;
    if (i >= s.max_blocks || (int64_t)i * s.B >= L) return;
    const int t0 = i * s.B, t1 = min(t0 + s.B, L);
    const int c = lane % LPR, rsub = lane / LPR;
    const T *base = (const T *)s.k + (int64_t)b * s.sb + (int64_t)g * s.sh + c * E;
    float mx[E], mn[E];
#pragma unroll
    for (int e = 0; e < E; ++e) { mx[e] = -INFINITY; mn[e] = INFINITY; }
    for (int t = t0 + rsub; t < t1; t += RPP) {
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
        *(uint4 *)((T *)kmax + o) = Elem<T>::pack(mx);
        *(uint4 *)((T *)kmin + o) = Elem<T>::pack(mn);
    }
}

// layers: n_layers entries each of k, v (the caches), buf_k, buf_v (the buffers) and, for a commit to
// the cache, kmax, kmin (or all NULL).  s carries the shape, the strides and ctx_len (shared).
hipError_t launch_commit(const Shape &s, int dtype, int n_layers, void *const *k, void *const *v,
                         void *const *buf_k, void *const *buf_v, int P, int Mt,
                         int32_t *n_pending, const int32_t *accepted, const int32_t *n_accepted,
                         int max_accept, int to_cache, void *const *kmax, void *const *kmin,
                         const specpv_lists *lists, int32_t *dropped, int32_t *old_len, hipStream_t st)
{
    if (P + max_accept > kCommitMaxRows) return hipErrorInvalidValue;
    const bool summaries = to_cache && kmax && kmin && kmax[0] && kmin[0];
    // the copies of every layer read the counters, so all of them go before the update
    for (int l0 = 0; l0 < n_layers; l0 += kCommitLayers) {
        const int nl = n_layers - l0 < kCommitLayers ? n_layers - l0 : kCommitLayers;
        CommitLayers lay = {};
        for (int l = 0; l < nl; ++l) {
            lay.k[l] = k[l0 + l]; lay.v[l] = v[l0 + l];
            lay.buf_k[l] = buf_k[l0 + l]; lay.buf_v[l] = buf_v[l0 + l];
        }
        const dim3 grid(s.Hkv, s.batch, nl);
#define SPECPV_COPY(T, DD)                                                                             \
    hipLaunchKernelGGL((commit_copy_kernel<T, DD>), grid, dim3(256), 0, st, s, lay, P, Mt,              \
                       n_pending, accepted, n_accepted, max_accept, to_cache)
        if (dtype == SPECPV_BF16) {
            if (s.D == 128) SPECPV_COPY(bf16_t, 128); else SPECPV_COPY(bf16_t, 64);
        } else {
            if (s.D == 128) SPECPV_COPY(float, 128); else SPECPV_COPY(float, 64);
        }
#undef SPECPV_COPY
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(commit_update_kernel, dim3((s.batch + 63) / 64), dim3(64), 0, st, s, P,
                       (int32_t *)s.ctx_len, n_pending, n_accepted, max_accept, to_cache, old_len, dropped);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (to_cache && lists) {
        for (int l0 = 0; l0 < n_layers; l0 += kCommitLayers) {
            const int nl = n_layers - l0 < kCommitLayers ? n_layers - l0 : kCommitLayers;
            CommitLists ls = {};
            for (int l = 0; l < nl; ++l) { ls.idx[l] = lists[l0 + l].sel_idx; ls.cnt[l] = lists[l0 + l].sel_count; }
            hipLaunchKernelGGL(commit_extend_lists_kernel, dim3(s.Hkv, s.batch, nl), dim3(64), 0, st, s, ls,
                               lists[0].n_sel, old_len, dropped);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    if (!summaries) return hipSuccess;
    // blocks that can have received one of at most P + max_accept tokens
    const int touched = (P + max_accept + s.B - 1) / s.B + 1;
    for (int l0 = 0; l0 < n_layers; l0 += kCommitLayers) {
        const int nl = n_layers - l0 < kCommitLayers ? n_layers - l0 : kCommitLayers;
        CommitLayers lay = {};
        for (int l = 0; l < nl; ++l) { lay.k[l] = k[l0 + l]; lay.kmax[l] = kmax[l0 + l]; lay.kmin[l] = kmin[l0 + l]; }
        const dim3 g2(touched, s.Hkv, s.batch * nl);
#define SPECPV_SUM(T, DD) hipLaunchKernelGGL((summarize_tail_kernel<T, DD>), g2, dim3(64), 0, st, s, lay, old_len)
        if (dtype == SPECPV_BF16) {
            if (s.D == 128) SPECPV_SUM(bf16_t, 128); else SPECPV_SUM(bf16_t, 64);
        } else {
            if (s.D == 128) SPECPV_SUM(float, 128); else SPECPV_SUM(float, 64);
        }
#undef SPECPV_SUM
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace specpv

namespace specpv {

// Gathered (physically contiguous) partial cache, Section 3.2: one workgroup per (list slot,
// KV head, sequence) copies one block of K and of V with 16-byte accesses, all of a thread's
// reads issued before its writes.
// 16-byte copies with the streaming hint (every byte is read once and written once)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const void *p)
{
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_t *)p));
}
__device__ __forceinline__ void stream_store16(void *p, uint4 v)
{
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4_t, v), (u32x4_t *)p);
}

template <typename T, int D>
__global__ __launch_bounds__(256) void gather_blocks_kernel(Shape s, const int32_t *sel_idx, const int32_t *sel_count,
                                                            int n_sel, T *out_k, T *out_v, int32_t *out_len)
{
    constexpr int E = Elem<T>::kPerVec;
    constexpr int LPR = D / E;
    constexpr int RPP = 256 / LPR;
    const int slot = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int L = s.ctx_len[b];
    int nb = L > 0 ? (L + s.B - 1) / s.B : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    const int cnt = max(0, min(sel_count[(int64_t)b * s.Hkv + g], n_sel));
    const int blk = slot < cnt ? sel_idx[((int64_t)b * s.Hkv + g) * n_sel + slot] : -1;
    const bool valid = blk >= 0 && blk < nb;
    const int c = threadIdx.x % LPR, rsub = threadIdx.x / LPR;
    const int64_t src0 = (int64_t)b * s.sb + (int64_t)g * s.sh + c * E;
    const int64_t dst0 = (((int64_t)b * s.Hkv + g) * n_sel + slot) * s.B * D + c * E;
    for (int r0 = 0; r0 < s.B; r0 += 4 * RPP) {
        uint4 kk[4], vv[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int r = r0 + x * RPP + rsub, t = blk * s.B + r;
            kk[x] = make_uint4(0, 0, 0, 0);
            vv[x] = kk[x];
            if (valid && r < s.B && t < L) {
                kk[x] = stream_load16((const T *)s.k + src0 + (int64_t)t * s.st);
                vv[x] = stream_load16((const T *)s.v + src0 + (int64_t)t * s.st);
            }
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int r = r0 + x * RPP + rsub;
            if (r < s.B) {
                stream_store16(out_k + dst0 + (int64_t)r * D, kk[x]);
                stream_store16(out_v + dst0 + (int64_t)r * D, vv[x]);
            }
        }
    }
    if (out_len && threadIdx.x == 0 && valid) {
        const int rows = slot * s.B + min(s.B, L - blk * s.B);   // token rows up to and including this block
        atomicMax(&out_len[b], rows);
    }
}

__global__ void zero_i32_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_gather(const Shape &s, int dtype, const int32_t *sel_idx, const int32_t *sel_count, int n_sel,
                         void *out_k, void *out_v, int32_t *out_len, hipStream_t st)
{
    const dim3 grid(n_sel, s.Hkv, s.batch);
    if (grid.z > 65535u || grid.y > 65535u) return hipErrorInvalidConfiguration;   // before anything is enqueued
    if (out_len) hipLaunchKernelGGL(zero_i32_kernel, dim3((s.batch + 63) / 64), dim3(64), 0, st, out_len, s.batch);
#define SPECPV_GATHER(T, DD) \
    hipLaunchKernelGGL((gather_blocks_kernel<T, DD>), grid, dim3(256), 0, st, s, sel_idx, sel_count, n_sel, (T *)out_k, (T *)out_v, out_len)
    if (dtype == SPECPV_BF16) {
        if (s.D == 128) SPECPV_GATHER(bf16_t, 128); else SPECPV_GATHER(bf16_t, 64);
    } else {
        if (s.D == 128) SPECPV_GATHER(float, 128); else SPECPV_GATHER(float, 64);
    }
#undef SPECPV_GATHER
    return hipGetLastError();
}

}  // namespace specpv
