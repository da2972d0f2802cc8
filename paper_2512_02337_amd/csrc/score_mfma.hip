// Block scoring (Section 3.2, eq. 2 and eq. 3; optionally the channel-wise bound) on the matrix
// cores for bf16, head dim 128.
//
// Per KV head the scores are max(Q . Kmax^T, Q . Kmin^T) reduced over the M*G query rows:
// two [rows x 128] x [128 x blocks] products.  A workgroup owns a tile of 32 blocks and
// spreads the query rows over its wavefronts, 32 rows at a time: a wavefront holds the two
// 32 x 128 summary tiles as MFMA B operands (lane = block) and its query rows as A operand
// (lane = row), so each lane ends up with 16 rows of ONE block; the element-wise max of the
// two accumulators and the reduction over rows (mean / max / rows of one node) are
// lane-local.  All reads of a wavefront are issued at once (one round trip); the
// wavefronts' partial results meet in LDS.  The sum order is the same for every block, so
// identical blocks get bit-identical scores wherever they sit.
//
// The same launch can do the selection as well: every workgroup of a (sequence, KV head)
// counts itself in when its scores are stored, and the one that finds itself last runs the
// top-k over the scores of all of them (no workgroup waits for another).
#include "internal.h"
#include "topk.h"
#include <type_traits>

namespace specpv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kScoreMaxWaves = 16;

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *glb_void_ptr;

// Eight 16-byte LDS reads and the wait for them, in assembly: the compiler would put a wait for every LDS-DMA
// in flight in front of an LDS read of its own, and, short of registers, schedules one read per matrix
// instruction.  OFF: a constant byte offset, added by the instructions themselves (16 bits).
template <int OFF>
__device__ __forceinline__ void lds_read8(const uint32_t (&a)[8], uint4 (&k)[8])
{
    static_assert(OFF >= 0 && OFF < 65536, "the offset field has 16 bits");
    asm volatile(
        "ds_read_b128 %0, %8 offset:%16\n\t"
        "ds_read_b128 %1, %9 offset:%16\n\t"
        "ds_read_b128 %2, %10 offset:%16\n\t"
        "ds_read_b128 %3, %11 offset:%16\n\t"
        "ds_read_b128 %4, %12 offset:%16\n\t"
        "ds_read_b128 %5, %13 offset:%16\n\t"
        "ds_read_b128 %6, %14 offset:%16\n\t"
        "ds_read_b128 %7, %15 offset:%16\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(k[0]), "=&v"(k[1]), "=&v"(k[2]), "=&v"(k[3]), "=&v"(k[4]), "=&v"(k[5]), "=&v"(k[6]), "=&v"(k[7])
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]), "n"(OFF)
        : "memory");
}

// BOUND: the channel-wise bound instead of eq. 2.  Per channel the larger product is q * Kmax
// where q >= 0 and q * Kmin where q < 0 (Kmax >= Kmin), so the bound is the sum of two inner
// products as well: max(q, 0) . Kmax + min(q, 0) . Kmin, accumulated into one tile.
// TILES tiles of 32 blocks per workgroup: the query rows are fetched once for all of them (for
// batches, where the workgroups are many and the repeated query reads are most of the traffic).
// ACROSS: the scores are read by another workgroup of this launch: agent-scope stores, which go
// past the caches that are private to a part of the chip.
template <bool BOUND, int TILES, bool ACROSS>
__device__ __forceinline__ void score_tiles(const Shape &s, const uint16_t *__restrict__ kmax,
                                            const uint16_t *__restrict__ kmin, int reduce, int last_node,
                                            float *__restrict__ scores)
{
    // the two summary tiles of this workgroup's 32 blocks: row-major, 256 B per block, the
    // 16-byte pieces of row t stored at piece index p ^ (t & 15) so that the operand reads
    // below (16 lanes per cycle, same piece, different rows) spread over all 64 banks
    __shared__ __attribute__((aligned(1024))) char tile[2 * TILES][8192];   // [tile][Kmax | Kmin]
    __shared__ float red[kScoreMaxWaves][64 * TILES];
    const int lane = threadIdx.x & 63, W = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, kg = lane >> 5;
    const int g = blockIdx.y, b = blockIdx.z;
    const int i0 = blockIdx.x * 32 * TILES;
    const int R = s.M * s.G;
    const int L = s.ctx_len[b];   // one sequence: only needed at the very end, its latency overlaps with everything else
    int nb = L > 0 ? (L + s.B - 1) / s.B : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    // in a batch the grid covers the longest sequence: workgroups past the end of a shorter one leave
    // at once (there the wait for the length is cheaper than their reads)
    if (s.batch > 1 && i0 >= nb) return;   // (only out of this function: the workgroup still counts itself in)

    // Summary rows go from memory straight into LDS (16 DMA operations of 1 KiB shared by the
    // wavefronts; operation d brings rows 4*(d&7) .. +3 of Kmax (d < 8) or Kmin, one 256-byte
    // row per 16 lanes).  Rows past the end of the arrays repeat the last row; their scores
    // are never stored.
    {
        const int r4 = lane >> 4, pos = lane & 15;
        const int64_t arr_row0 = ((int64_t)b * s.Hkv + g) * s.max_blocks;
        for (int d = wave; d < 16 * TILES; d += W) {
            const int i = d & 7, row = 4 * i + r4, t = d >> 4;
            const int blk = min(i0 + 32 * t + row, s.max_blocks - 1);
            const char *src = (const char *)((d & 8) ? kmin : kmax) + ((arr_row0 + blk) * 128) * 2 + 16 * (pos ^ (row & 15));
            __builtin_amdgcn_global_load_lds((glb_void_ptr)src, (lds_void_ptr)(tile[d >> 3] + i * 1024), 16, 0, 2);   // streaming hint: read once
        }
    }

    float acc[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) acc[t] = reduce == SPECPV_REDUCE_MAX ? -INFINITY : 0.f;
    const uint16_t *q = (const uint16_t *)s.q;
    bool landed = false;
    // query rows r0 .. r0+31 as A operand: lane = row (every wavefront has at least one such block)
    for (int r0 = wave * 32; r0 < R; r0 += W * 32) {
        const int r = min(r0 + n, R - 1);
        const int j = r / s.G, hh = r - j * s.G;
        const uint16_t *qrow = q + (((int64_t)b * s.M + j) * s.Hq + g * s.G + hh) * 128 + kg * 8;
        uint4 qa[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qa[ks] = *(const uint4 *)(qrow + ks * 16);
        if (!landed) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's DMA operations (and query rows) are in
            __syncthreads();                      // ... and so are everybody else's
            landed = true;
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            // summary tiles as B operands: lane = block, channels 16*ks + 8*kg .. +8
            const char *bxp = tile[2 * t] + n * 256, *bnp = tile[2 * t + 1] + n * 256;
            bf16x8 bx[8], bn[8];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const int off = (32 * ks + 16 * kg) ^ (16 * (n & 15));
                bx[ks] = __builtin_bit_cast(bf16x8, *(const uint4 *)(bxp + off));
                bn[ks] = __builtin_bit_cast(bf16x8, *(const uint4 *)(bnp + off));
            }
            f32x16 sx, sn;
#pragma unroll
            for (int x = 0; x < 16; ++x) { sx[x] = 0.f; sn[x] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                if (BOUND) {
                    // split the packed bf16 pairs by sign: 0xffff in the halves whose sign bit is set
                    uint4 neg, pos;
                    const uint32_t w[4] = {qa[ks].x, qa[ks].y, qa[ks].z, qa[ks].w};
                    uint32_t pw[4], nw[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t m = ((w[e] >> 15) & 0x00010001u) * 0xffffu;
                        nw[e] = w[e] & m;
                        pw[e] = w[e] & ~m;
                    }
                    pos = make_uint4(pw[0], pw[1], pw[2], pw[3]);
                    neg = make_uint4(nw[0], nw[1], nw[2], nw[3]);
                    sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pos), bx[ks], sx, 0, 0, 0);
                    sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, neg), bn[ks], sx, 0, 0, 0);
                } else {
                    const bf16x8 a = __builtin_bit_cast(bf16x8, qa[ks]);
                    sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bx[ks], sx, 0, 0, 0);
                    sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bn[ks], sn, 0, 0, 0);
                }
            }
            // accumulator slot x holds row r0 + (x>>2)*8 + kg*4 + (x&3) of this lane's block
            if (reduce != SPECPV_REDUCE_LAST && r0 + 32 <= R) {
                // all 32 rows count (every wavefront but the one with the ragged end): no per-row tests; the
                // same order of operations as below
                if (reduce == SPECPV_REDUCE_MAX) {
#pragma unroll
                    for (int x = 0; x < 16; ++x) acc[t] = fmaxf(acc[t], BOUND ? sx[x] : fmaxf(sx[x], sn[x]));
                } else {
#pragma unroll
                    for (int x = 0; x < 16; ++x) acc[t] += BOUND ? sx[x] : fmaxf(sx[x], sn[x]);
                }
            } else {
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int row = r0 + (x >> 2) * 8 + kg * 4 + (x & 3);
                    const float sv = BOUND ? sx[x] : fmaxf(sx[x], sn[x]);
                    if (reduce == SPECPV_REDUCE_MAX) {
                        if (row < R) acc[t] = fmaxf(acc[t], sv);
                    } else if (reduce == SPECPV_REDUCE_MEAN) {
                        if (row < R) acc[t] += sv;
                    } else {
                        if (row < R && row / s.G == last_node) acc[t] += sv;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < TILES; ++t) red[wave][64 * t + lane] = acc[t];
    __syncthreads();
    if (wave >= TILES) return;
    // wavefront t finishes tile t
    const int t = wave;
    float a = red[0][64 * t + lane];
    for (int w = 1; w < W; ++w) {
        const float o = red[w][64 * t + lane];
        a = reduce == SPECPV_REDUCE_MAX ? fmaxf(a, o) : a + o;
    }
    const float other = __shfl_xor(a, 32);
    float out;
    if (reduce == SPECPV_REDUCE_MAX) out = fmaxf(a, other);
    else if (reduce == SPECPV_REDUCE_MEAN) out = (a + other) / (float)R;
    else out = (a + other) / (float)s.G;
    const int blk = i0 + 32 * t + n;
    if (kg == 0 && blk < nb) {
        float *dst = scores + ((int64_t)b * s.Hkv + g) * s.max_blocks + blk;
        if (ACROSS) __hip_atomic_store((uint32_t *)dst, __float_as_uint(out), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else *dst = out;
    }
}

// The same for batches, query-stationary: a workgroup whose wavefronts hold all the query rows (one block of 32 each)
// takes STG stages of TILES tiles (32 * TILES * STG consecutive blocks).  All stages are requested at once -- the
// tiles fill the LDS; the cross-wavefront sums reuse it at the end -- so the query rows are fetched once per
// 32 * TILES * STG blocks and a workgroup pays one round trip.  The operand reads of a tile are batched in assembly
// (lds_read8): left to the compiler they were issued one pair per matrix instruction, each waiting for the last.
template <bool BOUND, int TILES, int STG, bool ACROSS>
__device__ __forceinline__ void score_tiles_staged(const Shape &s, const uint16_t *__restrict__ kmax,
                                                   const uint16_t *__restrict__ kmin, int reduce, int last_node,
                                                   float *__restrict__ scores)
{
    constexpr int TOT = TILES * STG;
    __shared__ __attribute__((aligned(1024))) char tile[STG][2 * TILES][8192];   // [stage][tile][Kmax | Kmin], swizzled as above
    static_assert(sizeof(tile) >= sizeof(float) * kScoreMaxWaves * 64 * TOT, "the partial sums reuse the tiles' memory");
    float (*red)[64 * TOT] = (float (*)[64 * TOT])&tile[0][0][0];
    const int lane = threadIdx.x & 63, W = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, kg = lane >> 5;
    const int g = blockIdx.y, b = blockIdx.z;
    const int i0 = blockIdx.x * 32 * TOT;
    const int R = s.M * s.G;   // <= 32 W (host-checked): wavefront w owns rows 32 w .. 32 w + 31
    const int L = s.ctx_len[b];
    int nb = L > 0 ? (L + s.B - 1) / s.B : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    // stages that hold blocks of this sequence (a batch's grid covers the longest one); at least one
    const int lim = s.batch > 1 ? nb : s.max_blocks;
    if (i0 >= lim) return;   // (only out of this function: the workgroup still counts itself in)
    const int n_st = min(STG, (lim - i0 + 32 * TILES - 1) / (32 * TILES));

    const int r4 = lane >> 4, pos = lane & 15;
    const int64_t arr_row0 = ((int64_t)b * s.Hkv + g) * s.max_blocks;
    auto issue = [&](int st) {
        for (int d = wave; d < 16 * TILES; d += W) {
            const int i = d & 7, row = 4 * i + r4, t = d >> 4;
            const int blk = min(i0 + 32 * (st * TILES + t) + row, s.max_blocks - 1);
            const char *src = (const char *)((d & 8) ? kmin : kmax) + ((arr_row0 + blk) * 128) * 2 + 16 * (pos ^ (row & 15));
            __builtin_amdgcn_global_load_lds((glb_void_ptr)src, (lds_void_ptr)(tile[st][d >> 3] + i * 1024), 16, 0, 2);
        }
    };
    issue(0);
    const int r0 = wave * 32;
    uint4 qa[8];
    {
        const int r = min(r0 + n, R - 1);
        const int j = r / s.G, hh = r - j * s.G;
        const uint16_t *qrow = (const uint16_t *)s.q + (((int64_t)b * s.M + j) * s.Hq + g * s.G + hh) * 128 + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qa[ks] = *(const uint4 *)(qrow + ks * 16);
    }
    for (int st = 1; st < n_st; ++st) issue(st);

    float acc[TOT];
#pragma unroll
    for (int t = 0; t < TOT; ++t) acc[t] = reduce == SPECPV_REDUCE_MAX ? -INFINITY : 0.f;
    // One wait for all of it and one barrier (measured against a wait and a barrier per stage, the later stages
    // landing under the arithmetic of the earlier ones: 21.8 against 22.9 us on the ragged batch of four at G = 5).
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's DMA operations and query rows are in
    __syncthreads();                      // ... and so are everybody else's
#pragma unroll
    for (int st = 0; st < STG; ++st) {
        if (st < n_st) {
            uint32_t ka[8];   // this lane's operand pieces of a tile's block n: k-step ks at (32 ks + 16 kg) ^ 16 (n & 15)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                ka[ks] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)tile[st][0] + (uint32_t)(n * 256) +
                         (uint32_t)((32 * ks + 16 * kg) ^ (16 * (n & 15)));
            auto one_tile = [&](auto tc) __attribute__((always_inline)) {
                constexpr int t = decltype(tc)::value;
                uint4 bxr[8], bnr[8];
                lds_read8<(2 * t) * 8192>(ka, bxr);
                lds_read8<(2 * t + 1) * 8192>(ka, bnr);
                bf16x8 bx[8], bn[8];
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    bx[ks] = __builtin_bit_cast(bf16x8, bxr[ks]);
                    bn[ks] = __builtin_bit_cast(bf16x8, bnr[ks]);
                }
                f32x16 sx, sn;
#pragma unroll
                for (int x = 0; x < 16; ++x) { sx[x] = 0.f; sn[x] = 0.f; }
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 a = __builtin_bit_cast(bf16x8, qa[ks]);
                    if (BOUND) {
                        // (see score_tiles) the packed bf16 pairs split by sign
                        const uint32_t w[4] = {qa[ks].x, qa[ks].y, qa[ks].z, qa[ks].w};
                        uint32_t pw[4], nw[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint32_t m = ((w[e] >> 15) & 0x00010001u) * 0xffffu;
                            nw[e] = w[e] & m;
                            pw[e] = w[e] & ~m;
                        }
                        sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3])), bx[ks], sx, 0, 0, 0);
                        sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, make_uint4(nw[0], nw[1], nw[2], nw[3])), bn[ks], sx, 0, 0, 0);
                    } else {
                        sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bx[ks], sx, 0, 0, 0);
                        sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bn[ks], sn, 0, 0, 0);
                    }
                }
                float &ac = acc[st * TILES + t];
                if (reduce != SPECPV_REDUCE_LAST && r0 + 32 <= R) {   // all 32 rows count: no per-row tests, same order
                    if (reduce == SPECPV_REDUCE_MAX) {
#pragma unroll
                        for (int x = 0; x < 16; ++x) ac = fmaxf(ac, BOUND ? sx[x] : fmaxf(sx[x], sn[x]));
                    } else {
#pragma unroll
                        for (int x = 0; x < 16; ++x) ac += BOUND ? sx[x] : fmaxf(sx[x], sn[x]);
                    }
                } else {
#pragma unroll
                    for (int x = 0; x < 16; ++x) {
                        const int row = r0 + (x >> 2) * 8 + kg * 4 + (x & 3);
                        const float sv = BOUND ? sx[x] : fmaxf(sx[x], sn[x]);
                        if (reduce == SPECPV_REDUCE_MAX) {
                            if (row < R) ac = fmaxf(ac, sv);
                        } else if (reduce == SPECPV_REDUCE_MEAN) {
                            if (row < R) ac += sv;
                        } else {
                            if (row < R && row / s.G == last_node) ac += sv;
                        }
                    }
                }
            };
            one_tile(std::integral_constant<int, 0>{});
            if constexpr (TILES > 1) one_tile(std::integral_constant<int, 1>{});
            if constexpr (TILES > 2) { one_tile(std::integral_constant<int, 2>{}); one_tile(std::integral_constant<int, 3>{}); }
            static_assert(TILES == 1 || TILES == 2 || TILES == 4, "tiles per stage");
        }
    }
    __syncthreads();   // every wavefront is done with the tiles: their memory takes the partial sums
#pragma unroll
    for (int t = 0; t < TOT; ++t) red[wave][64 * t + lane] = acc[t];
    __syncthreads();
    for (int t = wave; t < TOT; t += W) {
        float a = red[0][64 * t + lane];
        for (int w = 1; w < W; ++w) {
            const float o = red[w][64 * t + lane];
            a = reduce == SPECPV_REDUCE_MAX ? fmaxf(a, o) : a + o;
        }
        const float other = __shfl_xor(a, 32);
        float out;
        if (reduce == SPECPV_REDUCE_MAX) out = fmaxf(a, other);
        else if (reduce == SPECPV_REDUCE_MEAN) out = (a + other) / (float)R;
        else out = (a + other) / (float)s.G;
        const int blk = i0 + 32 * t + n;
        if (kg == 0 && blk < nb) {
            float *dst = scores + ((int64_t)b * s.Hkv + g) * s.max_blocks + blk;
            if (ACROSS) __hip_atomic_store((uint32_t *)dst, __float_as_uint(out), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else *dst = out;
        }
    }
}

// P = 0: scores only.  P = 4, 8, 16: scores, then the selection over lists of up to 256 * P blocks
// by the last workgroup of each (sequence, KV head) to get here (workgroups of at least 256 threads).
// Arrival is counted on two levels, because agent-scope atomics on one address are executed one
// after the other (64 workgroups on one word: + 4.4 us; 8 + 8: + 0.9 us): the workgroups of a
// (sequence, KV head) are dealt to eight groups by blockIdx.x % 8, the last of a group counts
// the group in on the pair's own word.  Pair p = b * Hkv + g owns the words arrive[(9 p + i) * wstride],
// i = 0 for the pair, 1 + j for group j; all are zero before the launch, and whoever finds a count
// complete sets it back to zero.
// WMAX: the most wavefronts a launch of this instantiation has (fewer leave the compiler more registers: at
// ten it keeps a tile's sixteen operand reads ahead of the matrix instructions instead of one read per instruction).
template <bool BOUND, int TILES, int P, int STG = 1, int WMAX = kScoreMaxWaves>
__global__ __launch_bounds__(64 * WMAX) void score_mfma_kernel(Shape s, const uint16_t *__restrict__ kmax,
                                                                         const uint16_t *__restrict__ kmin, int reduce,
                                                                         int last_node, float *__restrict__ scores,
                                                                         TopkArgs a, unsigned long long *arrive, int wstride)
{
    if constexpr (STG > 1) score_tiles_staged<BOUND, TILES, STG, P != 0>(s, kmax, kmin, reduce, last_node, scores);
    else score_tiles<BOUND, TILES, P != 0>(s, kmax, kmin, reduce, last_node, scores);
    if constexpr (P != 0) {
        __shared__ TopkLds lds;
        __shared__ int is_last;
        const int g = blockIdx.y, b = blockIdx.z;
        // A store is counted as done (vmcnt) when it has been acknowledged at the scope it was issued
        // with; the counters below are only touched after that, and the last workgroup only reads the
        // scores after it has seen the full counts: no further fence is needed.
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's score stores are out
        __syncthreads();                      // ... and so are everybody else's
        if (threadIdx.x == 0) {
            unsigned long long *pair = arrive + ((int64_t)b * s.Hkv + g) * 9 * wstride;
            const int j = blockIdx.x & 7;
            unsigned long long *group = pair + (int64_t)(1 + j) * wstride;
            const unsigned long long n_j = (gridDim.x - j + 7) >> 3;     // workgroups with blockIdx.x % 8 == j
            const unsigned long long n_groups = gridDim.x < 8 ? gridDim.x : 8;
            bool last = false;
            if (__hip_atomic_fetch_add(group, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1ull == n_j) {
                __hip_atomic_store(group, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (__hip_atomic_fetch_add(pair, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1ull == n_groups) {
                    __hip_atomic_store(pair, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    last = true;
                }
            }
            is_last = last ? 1 : 0;
        }
        __syncthreads();
        if (!is_last) return;
        topk_fast_body<P, true>(lds, scores, s.ctx_len, s.B, s.max_blocks, s.Hkv, g, b, a);
    }
}

bool score_mfma_supported(const Shape &s, int dtype) { return dtype == SPECPV_BF16 && s.D == 128; }

bool score_select_supported(const Shape &s, int dtype)
{
    // the selection needs 256 threads, lists of at most 4096 blocks and nine arrival words per (sequence, KV head)
    const int row_tiles = (s.M * s.G + 31) / 32;
    return score_mfma_supported(s, dtype) && row_tiles >= 4 && s.max_blocks <= 256 * 16 &&
           (size_t)s.batch * s.Hkv * 9 * sizeof(unsigned long long) <= kArriveBytes;
}

// sel != nullptr: the selection runs in the same launch (score_select_supported(s, dtype) holds and
// arrive points to zeroed words)
hipError_t launch_scores_mfma(const Shape &s, const void *kmax, const void *kmin, int reduce,
                              int last_node, int kind, float *scores, const TopkArgs *sel,
                              unsigned long long *arrive, hipStream_t st)
{
    // one wavefront per block of 32 query rows; T tiles per workgroup need T wavefronts to finish them
    const int row_tiles = (s.M * s.G + 31) / 32;
    const int tiles1 = (s.max_blocks + 31) / 32;
    // two or four tiles per workgroup where the workgroups are many (measured: at one 128K sequence,
    // 512 workgroups, 10.3 us with two tiles against 9.6 with one; at four sequences, 2048
    // workgroups, 46 us with one tile, 33 with two, 29 with four)
    const int64_t wgs1 = (int64_t)tiles1 * s.Hkv * s.batch, cus = device_cu_count();
    const int T = (row_tiles >= 4 && wgs1 >= 8 * cus) ? 4 : ((row_tiles >= 2 && wgs1 >= 4 * cus) ? 2 : 1);
    // ... and where they are many and the query rows are 9 or 10 blocks of 32 (G = 5 with 60 nodes: one block per
    // wavefront, and few enough wavefronts for 168 registers each), four stages of two tiles with the query rows
    // held over them (measured, scoring + selection per call: ragged batch of four at G = 5 30.0 against 34.4 us,
    // eight sequences of 64K at G = 5 30.5 against 36.3; at G = 4, eight blocks of rows, 16 x 32K: 27.9 against
    // 27.1, so those stay with four tiles).  eq.-2 scores only: the channel-wise bound splits the query operands by
    // sign and has no registers to hold them.
    const bool staged = T == 4 && row_tiles >= 9 && row_tiles <= 10 && kind != SPECPV_SCORE_CHANNEL_BOUND;
    const int per_wg = staged ? 8 : T;
    dim3 grid((tiles1 + per_wg - 1) / per_wg, s.Hkv, s.batch), block(64 * (row_tiles < kScoreMaxWaves ? row_tiles : kScoreMaxWaves));
    const int P = !sel ? 0 : (s.max_blocks <= 256 * 4 ? 4 : (s.max_blocks <= 256 * 8 ? 8 : 16));
    const TopkArgs a = sel ? *sel : TopkArgs{0, 0, 0, 0, nullptr, nullptr};
    // every arrival word on a 128-byte line of its own where the region is large enough for that
    const int wstride = (size_t)s.batch * s.Hkv * 9 * 128 <= kArriveBytes ? 16 : 1;
#define SPECPV_LAUNCH(BOUND, TILES, PP) \
    hipLaunchKernelGGL((score_mfma_kernel<BOUND, TILES, PP>), grid, block, 0, st, s, (const uint16_t *)kmax, \
                       (const uint16_t *)kmin, reduce, last_node, scores, a, arrive, wstride)
#define SPECPV_LAUNCH_P(BOUND, TILES) \
    do { if (P == 0) SPECPV_LAUNCH(BOUND, TILES, 0); else if (P == 4) SPECPV_LAUNCH(BOUND, TILES, 4); \
         else if (P == 8) SPECPV_LAUNCH(BOUND, TILES, 8); else SPECPV_LAUNCH(BOUND, TILES, 16); } while (0)
#define SPECPV_LAUNCH_S(BOUND, PP) \
    hipLaunchKernelGGL((score_mfma_kernel<BOUND, 2, PP, 4, 10>), grid, block, 0, st, s, (const uint16_t *)kmax, \
                       (const uint16_t *)kmin, reduce, last_node, scores, a, arrive, wstride)
#define SPECPV_LAUNCH_SP(BOUND) \
    do { if (P == 0) SPECPV_LAUNCH_S(BOUND, 0); else if (P == 4) SPECPV_LAUNCH_S(BOUND, 4); \
         else if (P == 8) SPECPV_LAUNCH_S(BOUND, 8); else SPECPV_LAUNCH_S(BOUND, 16); } while (0)
    if (staged) {
        SPECPV_LAUNCH_SP(false);
    } else if (kind == SPECPV_SCORE_CHANNEL_BOUND) {
        if (T == 4) SPECPV_LAUNCH_P(true, 4); else if (T == 2) SPECPV_LAUNCH_P(true, 2); else SPECPV_LAUNCH_P(true, 1);
    } else {
        if (T == 4) SPECPV_LAUNCH_P(false, 4); else if (T == 2) SPECPV_LAUNCH_P(false, 2); else SPECPV_LAUNCH_P(false, 1);
    }
#undef SPECPV_LAUNCH_SP
#undef SPECPV_LAUNCH_S
#undef SPECPV_LAUNCH_P
#undef SPECPV_LAUNCH
    return hipGetLastError();
}

}  // namespace specpv
