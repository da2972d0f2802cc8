// Context part of the verification attention on the matrix cores, for bf16 with
// head dim 128 (Section 3.2: the draft tree attends over the kept blocks as one KV
// segment; with all blocks kept this is the full verification of Section 3.3).
//
// Work decomposition.  A workgroup (4 wavefronts) owns one query head, one tile of
// up to 64 tree nodes and one KV split; inside it every wavefront owns the whole
// row tile and a contiguous range of 32-token chunks, so K and V go from global
// memory straight into MFMA operand registers -- nothing is gathered and no LDS is
// used in the main loop.  The G query heads of a KV head that read the same split
// are placed on one XCD, next to each other in dispatch order, so that the split's
// K/V bytes come from HBM once and from that XCD's L2 afterwards.
//
// Per chunk (v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//   S^T = K . Q^T     tokens are the M index, query rows the N index, so each
//                     lane holds 16 tokens of ONE query row: running max, sum and
//                     rescale are lane-local (one cross-lane exchange with lane^32);
//   O^T += V^T . P^T  the S^T accumulator, converted to bf16, already has the
//                     B-operand layout; V is loaded as 4 channels x 8 tokens per
//                     lane and transposed in registers with byte permutes.
// The contraction index may be permuted freely as long as both operands agree,
// which is what makes the register layouts line up.
//
// Epilogue: the four wavefronts merge their (O, m, l) through LDS and write one
// split-KV partial per (head, split, node); combine.hip finishes.
#include "internal.h"

namespace specpv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kOPitch = 132;  // floats per staged output row (128 + 4: conflict-free 16-byte writes)

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &u) { return __builtin_bit_cast(bf16x8, u); }

// lo16(a) | lo16(b) << 16   and   hi16(a) | hi16(b) << 16
__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

struct ChunkRegs {
    uint4 kf[8];     // K rows as A operand: token = lane & 31, channels 16*ks + 8*(lane >> 5) .. +8
    uint2 vr[2][8];  // V: for k-step ks2, slot e: token tt(ks2, e, lane >> 5), channels 4*(lane & 31) .. +4
    uint32_t vmask;  // bit t: token t of the chunk exists
};

template <int NRB, bool ALIGNED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_ctx_mfma_kernel(Shape s, const int32_t *sel_idx, const int32_t *sel_count, int n_sel,
                          Partials part, float scale_log2, int n_units, int GR)
{
    extern __shared__ float lds[];
    constexpr int ROWS = NRB * 32;
    float *ms = lds;                 // [4][ROWS]
    float *ls = lds + 4 * ROWS;      // [4][ROWS]
    float *obuf = lds + 8 * ROWS;    // [4][ROWS][kOPitch]

    // ---- which piece of work is this workgroup -------------------------------------
    const int id = blockIdx.x;
    const int xcd = id & 7, qd = id >> 3;
    const int r = qd % GR, u = (qd / GR) * 8 + xcd;
    if (u >= n_units) return;
    const int sp = u % part.nsplit;
    const int g = (u / part.nsplit) % s.Hkv;
    const int b = u / (part.nsplit * s.Hkv);
    const int hh = r % s.G, rt = r / s.G;
    const int h = g * s.G + hh;
    const int m0 = rt * 64;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, kg = lane >> 5;

    const int L = s.ctx_len[b];
    int nb = L > 0 ? (L + s.B - 1) / s.B : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    const int32_t *sel = sel_idx ? sel_idx + ((int64_t)b * s.Hkv + g) * n_sel : nullptr;
    int cnt = nb;
    if (sel) cnt = max(0, min(sel_count[(int64_t)b * s.Hkv + g], n_sel));
    const int64_t T = nb > 0 ? (int64_t)cnt * s.B : 0;
    const int C = (int)((T + 31) / 32);
    const int W = part.nsplit * 4, wsid = sp * 4 + wave;
    const int c0 = (int)((int64_t)C * wsid / W), c1 = (int)((int64_t)C * (wsid + 1) / W);

    const uint16_t *kbase = (const uint16_t *)s.k + (int64_t)b * s.sb + (int64_t)g * s.sh;
    const uint16_t *vbase = (const uint16_t *)s.v + (int64_t)b * s.sb + (int64_t)g * s.sh;

    // ---- Q fragments (B operand of S^T = K . Q^T): row = lane & 31 ------------------
    bf16x8 qf[NRB][8];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int j = m0 + rb * 32 + n;
        const uint16_t *qrow = (const uint16_t *)s.q + (((int64_t)b * s.M + min(j, s.M - 1)) * s.Hq + h) * 128 + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 x = *(const uint4 *)(qrow + ks * 16);
            if (j >= s.M) x = make_uint4(0, 0, 0, 0);
            qf[rb][ks] = as_bf16x8(x);
        }
    }

    f32x16 O[NRB][4];
    float m_run[NRB], l_run[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[rb][j][i] = 0.f;
    }

    // token row of lane's token t = lane & 31 in chunk c, or -1
    auto lookup = [&](int c) -> int {
        if (c >= c1) return -1;
        const int64_t p = (int64_t)c * 32 + n;
        if (p >= T) return -1;
        const int slot = (int)(p / s.B);
        const int blk = sel ? sel[slot] : slot;
        if (blk < 0 || blk >= nb) return -1;
        const int tok = blk * s.B + (int)(p - (int64_t)slot * s.B);
        return tok < L ? tok : -1;
    };

    auto issue = [&](ChunkRegs &cr, int tok) {
        const uint32_t vm = (uint32_t)__ballot(tok >= 0);
        cr.vmask = vm;
        const int tk = tok >= 0 ? tok : 0;  // L > 0 here, row 0 exists: masked out later
        const uint16_t *kr = kbase + (int64_t)tk * s.st + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) cr.kf[ks] = *(const uint4 *)(kr + ks * 16);
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int tt = 16 * ks2 + 8 * (e >> 2) + 4 * kg + (e & 3);
                int tv;
                if (ALIGNED) tv = min(__builtin_amdgcn_readfirstlane(tk) + tt, L - 1);  // 32 consecutive rows of one block
                else tv = __shfl(tk, tt);
                cr.vr[ks2][e] = *(const uint2 *)(vbase + (int64_t)tv * s.st + n * 4);
            }
    };

    auto compute = [&](const ChunkRegs &cr) {
        f32x16 S[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int i = 0; i < 16; ++i) S[rb][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
                S[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(cr.kf[ks]), qf[rb][ks], S[rb], 0, 0, 0);
        const bool full = cr.vmask == 0xffffffffu;
        uint4 pf[NRB][2];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (!full) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int tt = (i >> 2) * 8 + kg * 4 + (i & 3);
                    if (!((cr.vmask >> tt) & 1u)) S[rb][i] = -INFINITY;
                }
            }
            float mx = S[rb][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[rb][i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[rb], mx * scale_log2);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_use);
            float p[16], lsum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[i] = __builtin_amdgcn_exp2f(fmaf(S[rb][i], scale_log2, -m_use));
                lsum += p[i];
            }
            l_run[rb] = fmaf(l_run[rb], alpha, lsum);
            m_run[rb] = m_new;
            pf[rb][0] = make_uint4(pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]),
                                   pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7]));
            pf[rb][1] = make_uint4(pack_bf16x2(p[8], p[9]), pack_bf16x2(p[10], p[11]),
                                   pack_bf16x2(p[12], p[13]), pack_bf16x2(p[14], p[15]));
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 16; ++i) O[rb][j][i] *= alpha;
            }
        }
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
            // 8 tokens x 4 channels  ->  4 channels x 8 tokens
            uint4 vt[4];
            const uint2 *v = cr.vr[ks2];
            vt[0] = make_uint4(pack_lo(v[0].x, v[1].x), pack_lo(v[2].x, v[3].x), pack_lo(v[4].x, v[5].x), pack_lo(v[6].x, v[7].x));
            vt[1] = make_uint4(pack_hi(v[0].x, v[1].x), pack_hi(v[2].x, v[3].x), pack_hi(v[4].x, v[5].x), pack_hi(v[6].x, v[7].x));
            vt[2] = make_uint4(pack_lo(v[0].y, v[1].y), pack_lo(v[2].y, v[3].y), pack_lo(v[4].y, v[5].y), pack_lo(v[6].y, v[7].y));
            vt[3] = make_uint4(pack_hi(v[0].y, v[1].y), pack_hi(v[2].y, v[3].y), pack_hi(v[4].y, v[5].y), pack_hi(v[6].y, v[7].y));
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb)
                    O[rb][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vt[j]), as_bf16x8(pf[rb][ks2]), O[rb][j], 0, 0, 0);
        }
    };

    // ---- main loop: loads of chunk c+1 are in flight while chunk c is computed -------
    if (c0 < c1) {
        ChunkRegs ra, rb2;
        issue(ra, lookup(c0));
        int tok_next = lookup(c0 + 1);
        for (int c = c0; c < c1; c += 2) {
            if (c + 1 < c1) issue(rb2, tok_next);
            tok_next = lookup(c + 2);
            compute(ra);
            if (c + 1 < c1) {
                if (c + 2 < c1) issue(ra, tok_next);
                tok_next = lookup(c + 3);
                compute(rb2);
            }
        }
    }

    // ---- merge the four wavefronts ---------------------------------------------------
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        l_run[rb] += __shfl_xor(l_run[rb], 32);
        if (kg == 0) {
            ms[wave * ROWS + rb * 32 + n] = m_run[rb];
            ls[wave * ROWS + rb * 32 + n] = l_run[rb];
        }
    }
    __syncthreads();
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int row = rb * 32 + n;
        float mg = fmaxf(fmaxf(ms[row], ms[ROWS + row]), fmaxf(ms[2 * ROWS + row], ms[3 * ROWS + row]));
        const float m_use = mg == -INFINITY ? 0.f : mg;
        const float a = __builtin_amdgcn_exp2f(m_run[rb] - m_use);
        float *dst = obuf + ((size_t)wave * ROWS + row) * kOPitch;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int mi = (i >> 2) * 8 + kg * 4 + (i & 3);
            *(float4 *)(dst + 4 * mi) = make_float4(O[rb][0][i] * a, O[rb][1][i] * a, O[rb][2][i] * a, O[rb][3][i] * a);
        }
    }
    __syncthreads();
    constexpr int RPW = ROWS / 4;  // rows each wavefront finishes
    const int64_t prow0 = (((int64_t)b * s.Hq + h) * part.nsplit + sp) * s.M;
    for (int rr = 0; rr < RPW; ++rr) {
        const int row = wave * RPW + rr;
        const int j = m0 + row;
        if (j >= s.M) break;
        float2 acc = make_float2(0.f, 0.f);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float2 x = *(const float2 *)(obuf + ((size_t)w * ROWS + row) * kOPitch + 2 * lane);
            acc.x += x.x; acc.y += x.y;
        }
        *(float2 *)(part.o + (prow0 + j) * 128 + 2 * lane) = acc;
    }
    if (lane < RPW) {
        const int row = wave * RPW + lane;
        const int j = m0 + row;
        if (j < s.M) {
            const float mg = fmaxf(fmaxf(ms[row], ms[ROWS + row]), fmaxf(ms[2 * ROWS + row], ms[3 * ROWS + row]));
            const float m_use = mg == -INFINITY ? 0.f : mg;
            float lt = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) lt += ls[w * ROWS + row] * __builtin_amdgcn_exp2f(ms[w * ROWS + row] - m_use);
            part.ml[(prow0 + j) * 2] = mg;
            part.ml[(prow0 + j) * 2 + 1] = lt;
        }
    }
}

bool attn_ctx_mfma_supported(const Shape &s, int dtype)
{
    return dtype == SPECPV_BF16 && s.D == 128 && s.st % 8 == 0;
}

hipError_t launch_attn_ctx_mfma(const Shape &s, const int32_t *sel_idx, const int32_t *sel_count,
                                int n_sel, Partials p, hipStream_t st)
{
    const int row_tiles = (s.M + 63) / 64;
    const int GR = s.G * row_tiles;
    const int n_units = s.batch * s.Hkv * p.nsplit;
    const int grid = ((n_units + 7) / 8) * 8 * GR;
    const float scale_log2 = kLog2e / sqrtf(128.f);
    const bool nrb1 = s.M <= 32;
    const bool aligned = s.B % 32 == 0;
    const int rows = nrb1 ? 32 : 64;
    const size_t lds = (size_t)(8 * rows + 4 * rows * kOPitch) * sizeof(float);
#define SPECPV_LAUNCH(NRB, AL)                                                                         \
    do {                                                                                               \
        static bool attr_set = false;                                                                  \
        auto kern = attn_ctx_mfma_kernel<NRB, AL>;                                                     \
        if (!attr_set) {                                                                               \
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (e != hipSuccess) return e;                                                             \
            attr_set = true;                                                                           \
        }                                                                                              \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, s, sel_idx, sel_count, n_sel, p,      \
                           scale_log2, n_units, GR);                                                   \
    } while (0)
    if (nrb1) { if (aligned) SPECPV_LAUNCH(1, true); else SPECPV_LAUNCH(1, false); }
    else      { if (aligned) SPECPV_LAUNCH(2, true); else SPECPV_LAUNCH(2, false); }
#undef SPECPV_LAUNCH
    return hipGetLastError();
}

}  // namespace specpv
