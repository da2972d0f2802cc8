// Block scoring (Section 3.2, eq. 2 and eq. 3) on the matrix cores for bf16, head dim 128.
//
// Per KV head the scores are max(Q . Kmax^T, Q . Kmin^T) reduced over the M*G query rows:
// two [rows x 128] x [128 x blocks] products.  One wavefront owns a tile of 32 blocks: it
// keeps the two 32 x 128 summary tiles in registers as MFMA B operands (lane = block) and
// walks over the query rows 32 at a time (MFMA A operand, lane = row), so each lane ends up
// with 16 rows of ONE block; the element-wise max of the two accumulators and the reduction
// over rows (mean / max / rows of one node) are lane-local, with a single exchange between
// lane and lane ^ 32 at the end.  The sum order is the same for every block, so identical
// blocks get bit-identical scores wherever they sit.
#include "internal.h"

namespace specpv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__global__ __launch_bounds__(256) void score_mfma_kernel(Shape s, const uint16_t *__restrict__ kmax,
                                                         const uint16_t *__restrict__ kmin, int reduce,
                                                         int last_node, float *__restrict__ scores)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, kg = lane >> 5;
    const int g = blockIdx.y, b = blockIdx.z;
    const int L = s.ctx_len[b];
    int nb = L > 0 ? (L + s.B - 1) / s.B : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    const int tile = blockIdx.x * 4 + wave;
    const int i0 = tile * 32;
    if (i0 >= nb) return;
    const int blk = min(i0 + n, nb - 1);   // lanes past the end repeat the last block; not stored
    const int R = s.M * s.G;

    // summary tiles as B operands: lane = block, channels 16*ks + 8*kg .. +8
    const int64_t srow = (((int64_t)b * s.Hkv + g) * s.max_blocks + blk) * 128 + kg * 8;
    bf16x8 bx[8], bn[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        bx[ks] = __builtin_bit_cast(bf16x8, *(const uint4 *)(kmax + srow + ks * 16));
        bn[ks] = __builtin_bit_cast(bf16x8, *(const uint4 *)(kmin + srow + ks * 16));
    }

    float acc = reduce == SPECPV_REDUCE_MAX ? -INFINITY : 0.f;
    const uint16_t *q = (const uint16_t *)s.q;
    // query rows r0 .. r0+31 as A operand: lane = row; the next tile's rows are requested
    // while the current tile is multiplied
    auto load_rows = [&](int r0, uint4 (&dst)[8]) {
        const int r = min(r0 + n, R - 1);
        const int j = r / s.G, hh = r - j * s.G;
        const uint16_t *qrow = q + (((int64_t)b * s.M + j) * s.Hq + g * s.G + hh) * 128 + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) dst[ks] = *(const uint4 *)(qrow + ks * 16);
    };
    auto row_tile = [&](int r0, const uint4 (&qa)[8]) {
        f32x16 sx, sn;
#pragma unroll
        for (int x = 0; x < 16; ++x) { sx[x] = 0.f; sn[x] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, qa[ks]);
            sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bx[ks], sx, 0, 0, 0);
            sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bn[ks], sn, 0, 0, 0);
        }
        // accumulator slot x holds row r0 + (x>>2)*8 + kg*4 + (x&3) of this lane's block
#pragma unroll
        for (int x = 0; x < 16; ++x) {
            const int row = r0 + (x >> 2) * 8 + kg * 4 + (x & 3);
            const float sv = fmaxf(sx[x], sn[x]);
            if (reduce == SPECPV_REDUCE_MAX) {
                if (row < R) acc = fmaxf(acc, sv);
            } else if (reduce == SPECPV_REDUCE_MEAN) {
                if (row < R) acc += sv;
            } else {
                if (row < R && row / s.G == last_node) acc += sv;
            }
        }
    };
    uint4 qa[8], qb[8];
    load_rows(0, qa);
    for (int r0 = 0; r0 < R; r0 += 64) {
        if (r0 + 32 < R) load_rows(r0 + 32, qb);
        row_tile(r0, qa);
        if (r0 + 32 < R) {
            if (r0 + 64 < R) load_rows(r0 + 64, qa);
            row_tile(r0 + 32, qb);
        }
    }
    const float other = __shfl_xor(acc, 32);
    float out;
    if (reduce == SPECPV_REDUCE_MAX) out = fmaxf(acc, other);
    else if (reduce == SPECPV_REDUCE_MEAN) out = (acc + other) / (float)R;
    else out = (acc + other) / (float)s.G;
    if (kg == 0 && i0 + n < nb) scores[((int64_t)b * s.Hkv + g) * s.max_blocks + i0 + n] = out;
}

bool score_mfma_supported(const Shape &s, int dtype) { return dtype == SPECPV_BF16 && s.D == 128; }

hipError_t launch_scores_mfma(const Shape &s, const void *kmax, const void *kmin, int reduce,
                              int last_node, float *scores, hipStream_t st)
{
    const int tiles = (s.max_blocks + 31) / 32;
    dim3 grid((tiles + 3) / 4, s.Hkv, s.batch), block(256);
    hipLaunchKernelGGL(score_mfma_kernel, grid, block, 0, st, s, (const uint16_t *)kmax, (const uint16_t *)kmin,
                       reduce, last_node, scores);
    return hipGetLastError();
}

}  // namespace specpv
