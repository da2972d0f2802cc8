// Context part of the verification attention on the matrix cores, for bf16 with
// head dim 128 (Section 3.2: the draft tree attends over the kept blocks as one KV
// segment; with all blocks kept this is the full verification of Section 3.3).
//
// Work decomposition.  A workgroup (8 wavefronts, two per SIMD) owns one query head,
// one tile of up to 64 tree nodes and one KV split; inside it four pairs of
// wavefronts each own a contiguous range of 32-token chunks, the two wavefronts of
// a pair taking 32 rows of the tile each.  Nothing is gathered: K and V rows go
// from their place in the cache straight into a small per-pair LDS ring by LDS-DMA
// (global_load_lds), two chunks ahead of the arithmetic, and from there into MFMA
// operand registers.  The G query heads of a KV head that read the same split are
// placed on one XCD, next to each other in dispatch order, so that the split's K/V
// bytes come from HBM once and from that XCD's L2 afterwards.
//
// Per chunk (v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//   S^T = K . Q^T     tokens are the M index, query rows the N index, so each
//                     lane holds 16 tokens of ONE query row: max, sum and rescale
//                     are lane-local (one exchange with lane ^ 32);
//   O^T += V^T . P^T  the S^T accumulator, converted to bf16, already has the
//                     B-operand layout; V comes out of LDS transposed (8 tokens
//                     of one channel per lane) through ds_read_b64_tr_b16.
// The contraction index may be permuted freely as long as both operands agree,
// which is what makes the register layouts line up.
//
// The reference maximum of a row is only moved when the true maximum runs more than
// 2^8 ahead of it, so rescaling the accumulators is rare.
//
// Epilogue: the four token groups merge their (O, m, l) through LDS and write one
// split-KV partial per (head, split, node); combine.hip finishes.
//
// attn_ctx_mfma_kernel (above description) is used when a wavefront has only a few chunks to go
// through (the partial verification over a 4K-token cache); attn_ctx_mfma_group_kernel, further
// down, when it has many (full verification of a long context): there a workgroup serves all
// query heads of a KV head.
#include "internal.h"

namespace specpv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *glb_void_ptr;

constexpr int kOPitch = 132;         // floats per staged output row (128 + 4: conflict-free 16-byte writes)
// One 32-token chunk in LDS: 8 KiB of K (row-major, 16-byte pieces XOR-swizzled by row & 7) and
// the V rows in 8 pieces of 4 rows (tokens i, i+8, i+16, i+24 in piece i), 1088 bytes apart, for
// the transposing LDS reads (see lds_read_v).
constexpr int kVPiecePitch = 1088;
constexpr int kStageBytes = 8192 + 8 * kVPiecePitch;
constexpr int kStages = 2;           // ring depth per wavefront pair (eight-wavefront kernel)
constexpr int kRingBytes = 4 * kStages * kStageBytes;
// Cache policy of the K / V requests: 2 = the streaming hint (nt).  K / V rows are used once per
// workgroup; with the hint the requests are served faster, and the sharing of a KV head's rows
// between its query heads' workgroups through L2 is unaffected (same fetch counters).
constexpr int kKvAux = 2;
constexpr float kRescaleSlack = 8.f; // the reference max may lag the true max by 2^8

// Exact n / d for 0 <= n < 2^31 with a host-prepared multiplier (no integer divide
// on the GPU: one takes about forty vector instructions).
struct FastDiv {
    uint32_t mul, shift, d;
    __device__ __forceinline__ uint32_t div(uint32_t n) const { return d == 1 ? n : (__umulhi(n, mul) >> shift); }
};
static FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;                       // l = ceil(log2 d)
    if (d <= 1) { f.mul = 0; f.shift = 0; return f; }
    f.mul = (uint32_t)(((1ull << (31 + l)) + d - 1) / d);   // ceil(2^(31+l) / d) <= 2^32 - 1 for d >= 2
    f.shift = l - 1;
    return f;
}

struct MfmaArgs {
    const int32_t *sel_idx, *sel_count;
    int n_sel;
    float scale_log2;
    int n_units, row_tiles, n_bg;
    int rph, n_row_blocks;   // group kernel: 32-row blocks per query head, and per KV group (G * rph)
    FastDiv div_nsplit, div_hkv, div_B, div_W;
};

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &u) { return __builtin_bit_cast(bf16x8, u); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}
// acc + lo(p) + hi(p) for a packed bf16 pair
__device__ __forceinline__ float add_bf16x2(uint32_t p, float acc)
{
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p), ones, acc, false);
}

// 16 bytes per lane from global memory straight into LDS (no registers involved):
// lane l of the wavefront lands at lds_dst + 16*l.
__device__ __forceinline__ void dma16(const char *gsrc, char *lds_dst)
{
    __builtin_amdgcn_global_load_lds((glb_void_ptr)gsrc, (lds_void_ptr)lds_dst, 16, 0, kKvAux);
}

// Four such operations 1 KiB apart on both sides: gbase is wavefront-uniform, the per-lane
// byte offsets alternate between off_even (operations 0, 2) and off_odd (1, 3).  The
// immediate offset of the instruction is added to the global and to the LDS address.
__device__ __forceinline__ void dma16x4(const char *gbase, uint32_t off_even, uint32_t off_odd, char *lds_dst)
{
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + off_even), (lds_void_ptr)lds_dst, 16, 0, kKvAux);
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + off_odd), (lds_void_ptr)lds_dst, 16, 1024, kKvAux);
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + off_even), (lds_void_ptr)lds_dst, 16, 2048, kKvAux);
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + off_odd), (lds_void_ptr)lds_dst, 16, 3072, kKvAux);
}

// The LDS reads of staged K / V are written in assembly so that the compiler does not
// put a full vector-memory wait in front of them (it cannot tell which in-flight
// LDS-DMA a read depends on); the waits are placed by hand instead.
template <int OFF>
__device__ __forceinline__ void lds_read_k(const uint32_t (&a)[8], uint4 (&k)[8])
{
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

// The same with four address registers: the operand piece of k-step ks + 4 lies 128 bytes
// behind that of k-step ks (the swizzle only touches the address bits below).
__device__ __forceinline__ void lds_read_k4(const uint32_t (&a)[4], uint4 (&k)[8])
{
    asm volatile(
        "ds_read_b128 %0, %8\n\t"
        "ds_read_b128 %1, %9\n\t"
        "ds_read_b128 %2, %10\n\t"
        "ds_read_b128 %3, %11\n\t"
        "ds_read_b128 %4, %8 offset:128\n\t"
        "ds_read_b128 %5, %9 offset:128\n\t"
        "ds_read_b128 %6, %10 offset:128\n\t"
        "ds_read_b128 %7, %11 offset:128\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(k[0]), "=&v"(k[1]), "=&v"(k[2]), "=&v"(k[3]), "=&v"(k[4]), "=&v"(k[5]), "=&v"(k[6]), "=&v"(k[7])
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3])
        : "memory");
}

// V operands (A operand of O^T += V^T . P^T: per lane 8 tokens of ONE channel) through the
// transposing LDS read ds_read_b64_tr_b16.  Inside a group of 16 lanes, lane s reads 8 bytes
// (4 channels) and receives, as lane 4a + c, element c of what lanes a, a+4, a+8, a+12 read.
// With lane s reading token (s >> 2) of a token quad and channels 4 * (s & 3) .. +3 of a
// 16-channel group, every lane ends up with the four tokens of the quad for channel
// (lane & 15) of the group: lane m = lane & 31 holds channel 32j + m of tile j, its k-group the
// tokens 16*ks2 + 8*hf + 4*kg + 0..3.  The four rows of a quad sit in four different V pieces,
// 1088 bytes apart, i.e. 64 bytes apart modulo the bank cycle: no bank conflicts.
// v[(ks2 * 4 + j) * 2 + hf]; addr = piece (4*kg + (s >> 2)), byte 32 * (group & 1) + 8 * (s & 3).
__device__ __forceinline__ void lds_read_v(uint32_t addr, uint2 (&v)[16])
{
    asm volatile(
        "ds_read_b64_tr_b16 %0, %16 offset:0\n\t"
        "ds_read_b64_tr_b16 %1, %16 offset:256\n\t"
        "ds_read_b64_tr_b16 %2, %16 offset:64\n\t"
        "ds_read_b64_tr_b16 %3, %16 offset:320\n\t"
        "ds_read_b64_tr_b16 %4, %16 offset:128\n\t"
        "ds_read_b64_tr_b16 %5, %16 offset:384\n\t"
        "ds_read_b64_tr_b16 %6, %16 offset:192\n\t"
        "ds_read_b64_tr_b16 %7, %16 offset:448\n\t"
        "ds_read_b64_tr_b16 %8, %16 offset:512\n\t"
        "ds_read_b64_tr_b16 %9, %16 offset:768\n\t"
        "ds_read_b64_tr_b16 %10, %16 offset:576\n\t"
        "ds_read_b64_tr_b16 %11, %16 offset:832\n\t"
        "ds_read_b64_tr_b16 %12, %16 offset:640\n\t"
        "ds_read_b64_tr_b16 %13, %16 offset:896\n\t"
        "ds_read_b64_tr_b16 %14, %16 offset:704\n\t"
        "ds_read_b64_tr_b16 %15, %16 offset:960\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7]),
          "=&v"(v[8]), "=&v"(v[9]), "=&v"(v[10]), "=&v"(v[11]), "=&v"(v[12]), "=&v"(v[13]), "=&v"(v[14]), "=&v"(v[15])
        : "v"(addr)
        : "memory");
}

// The split-KV partials are written once here and read once by the combine kernel, which runs on
// other CUs (and mostly other XCDs): stored with the streaming hint they do not linger in this
// XCD's L2 as dirty lines that the end of the kernel has to write back (measured: 3.6 % of the
// partial-verify step).
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_partial(float *p, float2 v)
{
    f32x2 x = {v.x, v.y};
#ifndef SPECPV_PARTIAL_PLAIN
    __builtin_nontemporal_store(x, (f32x2 *)p);
#else
    *(f32x2 *)p = x;
#endif
}

// max / sum over the two half-wavefronts (lane and lane ^ 32)
__device__ __forceinline__ float max_xor32(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor32(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}


// grid: x = r * 8 + xcd   (r = query head within the group + G * row tile),  y = unit / 8
// with unit = ((b * Hkv + g) * nsplit + split).  Workgroups are handed to the 8 XCDs
// round-robin in linear order and gridDim.x is a multiple of 8, so a unit (and the G
// query heads that share its K/V bytes) stays on XCD unit % 8.
//
// Workgroup = 8 wavefronts = 4 token groups x 2 row blocks.  Wavefronts tg and tg + 4
// sit on the same SIMD, work on the same chunks (rows 0..31 and 32..63 of the tile)
// and share one LDS ring; the first of the pair requests the K rows, the second the V
// rows.  Two workgroup barriers per chunk order "DMA landed -> both read" and "both
// read -> stage may be refilled".  Every wavefront runs the same number of iterations
// (the largest chunk count in the workgroup), so the barriers always match up.
template <bool ALIGNED>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_ctx_mfma_kernel(Shape s, Partials part, MfmaArgs a)
{
    extern __shared__ char lds_raw[];
    float *ms = (float *)lds_raw;            // [4 token groups][64 rows]
    float *ls = ms + 4 * 64;                 // [4][64]
    char *ring = lds_raw + 2048;             // [4 pairs][kStages][K 8 KiB | V 8 KiB]
    float *obuf = (float *)(lds_raw + 2048); // [4][64][kOPitch], reuses the ring after the main loop

    // ---- which piece of work is this workgroup -------------------------------------
    const int xcd = blockIdx.x & 7, r = blockIdx.x >> 3;
    const int bgh = (int)a.div_nsplit.div(blockIdx.y);
    const int sp = (int)blockIdx.y - bgh * part.nsplit;
    const int bg = bgh * 8 + xcd;
    if (bg >= a.n_bg) return;
    const int b = (int)a.div_hkv.div((uint32_t)bg);
    const int g = bg - b * s.Hkv;
    const int rt = r >= s.G ? 1 : 0;          // at most two row tiles (M <= 128)
    const int hh = r - rt * s.G;
    const int h = g * s.G + hh;
    const int m0 = rt * 64;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tg = wave & 3, rb = wave >> 2;
    const int n = lane & 31, kg = lane >> 5;

    // Everything whose address only depends on the kernel arguments is requested up
    // front, so that the cold-miss latencies of these small reads overlap: context
    // length, list length, the kept-block ids this wavefront will most likely need
    // (assuming a full list), and the query rows.
    const int32_t *sel = a.sel_idx ? a.sel_idx + (int64_t)bg * a.n_sel : nullptr;
    const int W = part.nsplit * 4, wsid = sp * 4 + tg;
    const uint32_t Bu = (uint32_t)s.B;
    const int L = s.ctx_len[b];
    const int cnt_raw = sel ? a.sel_count[bg] : 0;
    // chunks of a list that precede the share of token group w; shares differ by at most one
    auto first_chunk = [&](uint32_t chunks, int w) -> int {
        const uint32_t base = a.div_W.div(chunks), rem = chunks - base * (uint32_t)W;
        return (int)((uint32_t)w * base + min((uint32_t)w, rem));
    };
    // lane t: the kept-block id that chunk t of this wavefront falls into, if the list is full
    // (its length is not known yet; the usual case)
    uint32_t spec_C = 0u;
    int spec_blk = -1;
    if (ALIGNED && sel) {
        spec_C = ((uint32_t)a.n_sel * Bu + 31u) >> 5;
        const uint32_t slot = a.div_B.div((uint32_t)(first_chunk(spec_C, wsid) + lane) * 32u);
        spec_blk = slot < (uint32_t)a.n_sel ? sel[slot] : -1;
    }
    uint4 qraw[8];
    {
        const int j = min(m0 + rb * 32 + n, s.M - 1);   // rows past M repeat row M-1; never stored
        const uint16_t *qrow = (const uint16_t *)s.q + (((int64_t)b * s.M + j) * s.Hq + h) * 128 + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qraw[ks] = *(const uint4 *)(qrow + ks * 16);
    }

    int nb = L > 0 ? (int)a.div_B.div((uint32_t)(L + s.B - 1)) : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    int cnt = nb;
    if (sel) cnt = max(0, min(cnt_raw, a.n_sel));
    const uint32_t T = nb > 0 ? (uint32_t)cnt * Bu : 0u;   // host guarantees max_blocks * B <= 2^30
    const uint32_t C = (T + 31u) >> 5;
    const int c0 = first_chunk(C, wsid), c1 = first_chunk(C, wsid + 1);
    const int nch = c1 - c0;
    const int nch_max = first_chunk(C, sp * 4 + 1) - first_chunk(C, sp * 4);   // token group 0 has the most

    // uniform slab bases; per-lane byte offsets inside a slab fit 32 bits (host-checked)
    const char *kb = (const char *)s.k + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const char *vb = (const char *)s.v + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const uint32_t st2 = (uint32_t)s.st * 2u;   // bytes per token row step

    char *my_ring = ring + tg * (kStages * kStageBytes);
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)my_ring;
    // K tile in LDS: row-major, 256 B per token, the 16-byte pieces of row t stored at
    // piece index (p ^ (t & 7)) so that the operand reads below (32 lanes, same piece,
    // different rows) spread over all banks.  Operand piece of k-step ks: 2*ks + kg.
    uint32_t kread[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
        kread[ks] = ring_addr + (uint32_t)n * 256u + (((uint32_t)(32 * ks + 16 * kg)) ^ (16u * ((uint32_t)n & 7u)));
    const uint32_t vread = ring_addr + 8192u + (uint32_t)(4 * kg + ((lane & 15) >> 2)) * kVPiecePitch +
                           32u * (uint32_t)((lane >> 4) & 1) + 8u * (uint32_t)(lane & 3);   // + stage * kStageBytes

    // ---- chunk -> token rows ------------------------------------------------------------
    // ALIGNED (B % 32 == 0): a chunk lies inside one block, so its 32 rows are consecutive.  The
    // first rows of the next 64 chunks of this wavefront sit in a register (lane t: chunk
    // row_base + t) and are picked with readlane.  Encoding: r >= 0: all 32 rows r .. r+31 are
    // valid tokens (the common case, handled without any further test); -1: no valid token;
    // -2 - r: rows from r on, cut off by the context length.
    int row_base = 0, row0vec = -1;
    auto encode_row = [&](int blk, uint32_t p0, uint32_t slot) -> int {
        if (blk < 0 || blk >= nb) return -1;
        const int r = blk * s.B + (int)(p0 - slot * Bu);
        return r >= L ? -1 : (r + 32 > L ? -2 - r : r);
    };
    auto fill_rows = [&](int cb) {
        row_base = cb;
        int r = -1;
        if (cb + lane < nch) {
            const uint32_t p0 = (uint32_t)(c0 + cb + lane) * 32u;   // < T: the slot below is < cnt
            const uint32_t slot = a.div_B.div(p0);
            r = encode_row(sel ? sel[slot] : (int)slot, p0, slot);
        }
        row0vec = r;
        // wait for the list entries here, inside the rare branch, so that the common path that
        // joins behind it carries no pending load (and no wait on the DMA prefetch)
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    };
    // general case: this lane's token (t = lane & 31) of chunk ci, or -1
    auto lane_row = [&](int ci) -> int {
        const uint32_t p = (uint32_t)(c0 + ci) * 32u + (uint32_t)n;
        if (p >= T) return -1;
        const uint32_t slot = a.div_B.div(p);
        const int blk = sel ? sel[slot] : (int)slot;
        if (blk < 0 || blk >= nb) return -1;
        const int tok = blk * s.B + (int)(p - slot * Bu);
        return tok < L ? tok : -1;
    };

    uint32_t vmask_st[kStages];   // validity bits of the chunk this wavefront last requested rows for, per stage

    // Request this wavefront's half of chunk ci: 8 DMA operations of 1 KiB (one 256-byte row per
    // 16 lanes).  rb == 0: the K rows, operation i brings rows 4i .. 4i+3, pieces swizzled by
    // row & 7.  rb == 1: the V rows, operation i brings rows i, i+8, i+16, i+24 into piece i.
    const int r4 = lane >> 4, pos = lane & 15;
    const uint32_t sw_even = 16u * (uint32_t)(pos ^ r4), sw_odd = sw_even ^ 64u, vsw = 16u * (uint32_t)pos;
    const uint32_t lane_row_off = (uint32_t)r4 * st2;
    auto issue = [&](int ci) {
        const int stg = ci & (kStages - 1);
        char *dst = my_ring + stg * kStageBytes;
        char *dstv = dst + 8192;
        int tok;
        if (ALIGNED) {
            if (ci - row_base >= 64) fill_rows(ci);
            const int r0 = __builtin_amdgcn_readlane(row0vec, ci - row_base);
            if (r0 >= 0) {
                vmask_st[stg] = 0xffffffffu;
                const size_t row0 = (size_t)((uint32_t)r0 * st2);   // fits 32 bits (host-checked)
                if (st2 == 256u) {
                    // rows are 256 bytes apart (the usual head-major cache): the instruction's
                    // immediate offset, added to the global and to the LDS address, covers the step
                    // between consecutive operations (K: 1 KiB on both sides; V: 256 bytes, with the
                    // LDS base adjusted for the rest of the piece pitch)
                    if (rb == 0) {
                        dma16x4(kb + row0, lane_row_off + sw_even, lane_row_off + sw_odd, dst);
                        dma16x4(kb + row0 + 4096, lane_row_off + sw_even, lane_row_off + sw_odd, dst + 4096);
                    } else {
                        const char *vsrc = vb + row0 + ((uint32_t)r4 * 2048u + vsw);
#define SPECPV_VOP(i) __builtin_amdgcn_global_load_lds((glb_void_ptr)vsrc, (lds_void_ptr)(dstv + (i) * (kVPiecePitch - 256)), 16, (i) * 256, kKvAux)
                        SPECPV_VOP(0); SPECPV_VOP(1); SPECPV_VOP(2); SPECPV_VOP(3);
                        SPECPV_VOP(4); SPECPV_VOP(5); SPECPV_VOP(6); SPECPV_VOP(7);
#undef SPECPV_VOP
                    }
                } else if (rb == 0) {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        dma16(kb + row0 + (size_t)(4 * i) * st2 + (lane_row_off + ((i & 1) ? sw_odd : sw_even)), dst + i * 1024);
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        dma16(vb + row0 + (size_t)(8 * r4 + i) * st2 + vsw, dstv + i * kVPiecePitch);
                }
                return;
            }
            const int rr = -2 - r0;   // r0 == -1 gives -1
            tok = (rr >= 0 && rr + n < L) ? rr + n : -1;
        } else {
            tok = lane_row(ci);
        }
        const uint32_t vm = (uint32_t)__ballot(tok >= 0);
        const uint32_t tk = tok >= 0 ? (uint32_t)tok : 0u;   // row 0 exists (L > 0); masked later
        vmask_st[stg] = vm;
        if (rb == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 4 * i + r4) * st2;
                dma16(kb + (tv + ((i & 1) ? sw_odd : sw_even)), dst + i * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 8 * r4 + i) * st2;
                dma16(vb + (tv + vsw), dstv + i * kVPiecePitch);
            }
        }
    };

    // ---- Q fragments (B operand of S^T = K . Q^T): row = lane & 31 ------------------
    bf16x8 qf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = as_bf16x8(qraw[ks]);
    if (ALIGNED && nch > 0) {
        if (sel && C == spec_C) {   // the usual case: the speculative ids are the right ones
            const uint32_t p0 = (uint32_t)(c0 + lane) * 32u;
            row0vec = lane < nch ? encode_row(spec_blk, p0, a.div_B.div(p0)) : -1;
        } else {
            fill_rows(0);
        }
    }
    // every load above has been consumed here: from now on the only vector-memory
    // operations of this wavefront in flight are its own DMA groups (8 operations each)
    // (as an instruction the compiler knows, not inline assembly: otherwise it assumes that the
    // loads of the prologue may still be in flight at the loop header and waits for vmcnt(0),
    // i.e. for the prefetch just issued, at the first use of Q in every iteration)
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), expcnt and lgkmcnt untouched
    asm volatile("" ::: "memory");

    f32x16 O[4];
    float m_ref = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[j][i] = 0.f;

    // ---- main loop ---------------------------------------------------------------------
    if (nch > 0) issue(0);
    if (nch > 1) issue(1);
    for (int i = 0; i < nch_max; ++i) {
        const bool active = i < nch;
        const int stg = i & 1;
        // own half of chunk i has landed (the only younger group is chunk i+1's)
        if (i + 1 < nch) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();          // ... and so has the partner's half
        uint4 kf[8];
        uint2 v[16];
        const uint32_t vmask = vmask_st[stg];
        if (active) {
            if (stg) lds_read_k<kStageBytes>(kread, kf); else lds_read_k<0>(kread, kf);
            lds_read_v(vread + stg * kStageBytes, v);
        }
        __builtin_amdgcn_s_barrier();          // both wavefronts of the pair hold chunk i in registers
        if (i + 2 < nch) issue(i + 2);
        if (!active) continue;

        f32x16 S;
#pragma unroll
        for (int x = 0; x < 16; ++x) S[x] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), qf[ks], S, 0, 0, 0);

        if (vmask != 0xffffffffu) {
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int tt = (x >> 2) * 8 + kg * 4 + (x & 3);
                if (!((vmask >> tt) & 1u)) S[x] = -INFINITY;
            }
        }
        float mx = fmaxf(S[0], S[1]);
#pragma unroll
        for (int x = 2; x < 16; x += 2) mx = fmaxf(fmaxf(mx, S[x]), S[x + 1]);
        mx = max_xor32(mx) * a.scale_log2;
        // the reference max only moves when the true max gets more than 2^slack ahead
        if (__any(mx > m_ref + kRescaleSlack)) {
            const float m_new = mx > m_ref + kRescaleSlack ? mx : m_ref;
            const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_ref - m_new);
            m_ref = m_new;
            l_run *= alpha;
            if (__any(alpha != 1.f && l_run != 0.f)) {   // nothing to rescale while O is still zero
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int x = 0; x < 16; ++x) O[j][x] *= alpha;
            }
        }
        const float m_use = m_ref == -INFINITY ? 0.f : m_ref;
        uint32_t pk[8];
        float lsum = 0.f;
#pragma unroll
        for (int x = 0; x < 16; x += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(S[x], a.scale_log2, -m_use));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(S[x + 1], a.scale_log2, -m_use));
            pk[x >> 1] = pack_bf16x2(p0, p1);
            lsum = add_bf16x2(pk[x >> 1], lsum);   // the sum runs over the rounded weights the MFMA sees
        }
        l_run += lsum;
        const uint4 pf0 = make_uint4(pk[0], pk[1], pk[2], pk[3]), pf1 = make_uint4(pk[4], pk[5], pk[6], pk[7]);
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint2 lo = v[(ks2 * 4 + j) * 2], hi = v[(ks2 * 4 + j) * 2 + 1];
                O[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y)),
                                                               as_bf16x8(ks2 ? pf1 : pf0), O[j], 0, 0, 0);
            }
    }
    __syncthreads();   // every wavefront is done with the rings: the epilogue reuses that LDS

    // ---- merge the four token groups ---------------------------------------------------
    {
        l_run = sum_xor32(l_run);
        const int row = rb * 32 + n;
        if (kg == 0) {
            ms[tg * 64 + row] = m_ref;
            ls[tg * 64 + row] = l_run;
        }
        // accumulator element 4q + x of tile j is channel 32j + 8q + 4kg + x of this lane's row
        float *dst = obuf + ((size_t)tg * 64 + row) * kOPitch;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4 *)(dst + 32 * j + 8 * q + 4 * kg) = make_float4(O[j][4 * q], O[j][4 * q + 1], O[j][4 * q + 2], O[j][4 * q + 3]);
    }
    __syncthreads();
    constexpr int RPW = 8;  // rows each wavefront finishes
    const int64_t prow0 = ((int64_t)(b * s.Hq + h) * part.nsplit + sp) * s.M;
    // weights of the four token groups for the rows this wavefront finishes (lane -> row)
    float wgt[4], m_row = -INFINITY, l_row = 0.f;
    {
        const int row = wave * RPW + (lane & (RPW - 1));
        float mw[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) { mw[w] = ms[w * 64 + row]; m_row = fmaxf(m_row, mw[w]); }
        const float m_use = m_row == -INFINITY ? 0.f : m_row;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            wgt[w] = __builtin_amdgcn_exp2f(mw[w] - m_use);   // 0 for a token group without valid tokens
            l_row = fmaf(ls[w * 64 + row], wgt[w], l_row);
        }
    }
    {
        float2 acc[RPW];
#pragma unroll
        for (int uu = 0; uu < RPW; ++uu) {
            const int row = wave * RPW + uu;
            acc[uu] = make_float2(0.f, 0.f);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float ww = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wgt[w]), uu));   // uniform: no LDS shuffle
                const float2 x = *(const float2 *)(obuf + ((size_t)w * 64 + row) * kOPitch + partial_chan(2 * lane, 128));
                acc[uu].x = fmaf(ww, x.x, acc[uu].x);
                acc[uu].y = fmaf(ww, x.y, acc[uu].y);
            }
        }
#pragma unroll
        for (int uu = 0; uu < RPW; ++uu) {
            const int j = m0 + wave * RPW + uu;
            if (j < s.M) store_partial(part.o + (prow0 + j) * 128 + 2 * lane, acc[uu]);   // positions 2 lane, 2 lane + 1 of the stored order
        }
    }
    if (lane < RPW) {
        const int j = m0 + wave * RPW + lane;
        if (j < s.M) *(float2 *)(part.ml + (prow0 + j) * 2) = make_float2(m_row, l_row);
    }
}

// ---- group variant: the query heads of a KV head in one workgroup --------------------------
// For long token ranges.  The G x ceil(M / 32) blocks of 32 query rows that share a KV head are
// dealt to workgroups of up to 8 wavefronts, one row block per wavefront (G = 4, M <= 64: one
// workgroup of 8; G = 5: two workgroups of 5).  A workgroup owns (sequence, KV head, its row
// blocks, KV split) and walks the split's chunks once for all of them: its W wavefronts share
// ONE ring of four stages and each brings its share of a chunk's 16 DMA operations, so every
// K / V byte is requested from memory exactly once per workgroup, whatever the caches do.
// Chunks are requested three ahead of the arithmetic (measured: two is slightly slower, four
// and six are no faster).  One workgroup barrier per chunk: past the barrier of chunk i every
// part of chunk i has landed, and every wavefront has finished reading chunk i - 1, whose stage
// is the one that chunk i + 3 is then requested into.
// A wavefront keeps its rows to itself over the whole split, so the epilogue has nothing to
// merge: it only turns the accumulators into row-major partials.
constexpr int kGroupStages = 4;   // a power of two
constexpr int kGroupAhead = 3;    // <= kGroupStages - 1

template <bool ALIGNED, int W>   // W wavefronts per workgroup: 2, 4, 6 or 8
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_ctx_mfma_group_kernel(Shape s, Partials part, MfmaArgs a)
{
    extern __shared__ char lds_raw[];
    char *ring = lds_raw;                  // [kGroupStages][K 8 KiB | V 8 pieces of 1088 B]
    float *obuf = (float *)lds_raw;        // [W wavefronts][32 rows][kOPitch], reuses the ring after the main loop

    const int xcd = blockIdx.x & 7, wg_part = blockIdx.x >> 3;
    const int u = blockIdx.y * 8 + xcd;
    if (u >= a.n_units) return;
    const int bg = (int)a.div_nsplit.div((uint32_t)u);
    const int sp = u - bg * part.nsplit;
    const int b = (int)a.div_hkv.div((uint32_t)bg);
    const int g = bg - b * s.Hkv;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // this wavefront's row block: head hh of the KV group, rows m0 .. m0 + 31 of the tree.  A
    // workgroup may have a wavefront too many (row block counts that do not divide): it brings
    // its share of the chunks and keeps the barriers, but computes and stores nothing.
    const int rbx = wg_part * W + wave;
    const bool live = rbx < a.n_row_blocks;
    const int rbx_c = live ? rbx : a.n_row_blocks - 1;
    const int hh = rbx_c / a.rph;
    const int m0 = (rbx_c - hh * a.rph) * 32;
    const int h = g * s.G + hh;
    const bool second = wave >= 4;            // the second wavefront of its SIMD (wavefronts w and w + 4 share one)
    const int n = lane & 31, kg = lane >> 5;

    const int32_t *sel = a.sel_idx ? a.sel_idx + (int64_t)bg * a.n_sel : nullptr;
    const int NS = part.nsplit;               // div_W divides by the number of splits here
    const uint32_t Bu = (uint32_t)s.B;
    const int L = s.ctx_len[b];
    const int cnt_raw = sel ? a.sel_count[bg] : 0;
    auto first_chunk = [&](uint32_t chunks, int w) -> int {
        const uint32_t base = a.div_W.div(chunks), rem = chunks - base * (uint32_t)NS;
        return (int)((uint32_t)w * base + min((uint32_t)w, rem));
    };
    uint4 qraw[8];
    {
        const int j = min(m0 + n, s.M - 1);   // rows past M repeat row M-1; never stored
        const uint16_t *qrow = (const uint16_t *)s.q + (((int64_t)b * s.M + j) * s.Hq + h) * 128 + kg * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qraw[ks] = *(const uint4 *)(qrow + ks * 16);
    }

    int nb = L > 0 ? (int)a.div_B.div((uint32_t)(L + s.B - 1)) : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    int cnt = nb;
    if (sel) cnt = max(0, min(cnt_raw, a.n_sel));
    const uint32_t T = nb > 0 ? (uint32_t)cnt * Bu : 0u;
    const uint32_t C = (T + 31u) >> 5;
    const int c0 = first_chunk(C, sp), c1 = first_chunk(C, sp + 1);
    const int nch = c1 - c0;                  // the same for all wavefronts: the barriers match up

    const char *kb = (const char *)s.k + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const char *vb = (const char *)s.v + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const uint32_t st2 = (uint32_t)s.st * 2u;

    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)ring;
    uint32_t kread[4];   // + stage * kStageBytes; k-step ks + 4 is 128 bytes behind k-step ks
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        kread[ks] = ring_addr + (uint32_t)n * 256u + (((uint32_t)(32 * ks + 16 * kg)) ^ (16u * ((uint32_t)n & 7u)));
    const uint32_t vread = ring_addr + 8192u + (uint32_t)(4 * kg + ((lane & 15) >> 2)) * kVPiecePitch +
                           32u * (uint32_t)((lane >> 4) & 1) + 8u * (uint32_t)(lane & 3);   // + stage * kStageBytes

    // ---- chunk -> token rows ------------------------------------------------------------
    // ALIGNED (B % 32 == 0): a chunk lies inside one block, so its 32 rows are consecutive.  The
    // first rows of the next 64 chunks sit in a register (lane t: chunk row_base + t) and are
    // picked with readlane.  Encoding: r >= 0: all 32 rows r .. r+31 are valid tokens (the common
    // case, handled without any further test); -1: no valid token; -2 - r: rows from r on, cut
    // off by the context length.
    int row_base = 0, row0vec = -1;
    auto fill_rows = [&](int cb) {
        row_base = cb;
        int r = -1;
        if (cb + lane < nch) {
            const uint32_t p0 = (uint32_t)(c0 + cb + lane) * 32u;   // < T: the slot below is < cnt
            const uint32_t slot = a.div_B.div(p0);
            const int blk = sel ? sel[slot] : (int)slot;
            if (blk >= 0 && blk < nb) {
                r = blk * s.B + (int)(p0 - slot * Bu);
                if (r >= L) r = -1;
                else if (r + 32 > L) r = -2 - r;
            }
        }
        row0vec = r;
        // wait for the list entries here, inside the rare branch, so that the common path that
        // joins behind it carries no pending load (and no wait on the DMA prefetch)
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    };
    // general case: this lane's token (t = lane & 31) of chunk ci, or -1
    auto lane_row = [&](int ci) -> int {
        const uint32_t p = (uint32_t)(c0 + ci) * 32u + (uint32_t)n;
        if (p >= T) return -1;
        const uint32_t slot = a.div_B.div(p);
        const int blk = sel ? sel[slot] : (int)slot;
        if (blk < 0 || blk >= nb) return -1;
        const int tok = blk * s.B + (int)(p - slot * Bu);
        return tok < L ? tok : -1;
    };

    // Request this wavefront's operations of chunk ci into stage stg (1 KiB each, one 256-byte row
    // per 16 lanes).  A chunk is 16 operations: K operation i (0 .. 7) brings rows 4i .. 4i+3, pieces
    // swizzled by row & 7; V operation i brings rows i, i+8, i+16, i+24 into piece i.  Wavefront w
    // takes operations w, w + W, w + 2W, ...  Returns the validity bits of the chunk's 32 tokens.
    // Everything that depends on the wavefront is folded into a few registers up front, so that
    // the common path is straight-line code.
    constexpr int NOPS = (16 + W - 1) / W;
    const int n_ops = (16 - wave + W - 1) / W;       // NOPS or NOPS - 1
    const int r4 = lane >> 4, pos = lane & 15;
    const uint32_t sw_even = 16u * (uint32_t)(pos ^ r4), sw_odd = sw_even ^ 64u, vsw = 16u * (uint32_t)pos;
    const char *src_lane[NOPS];   // per operation: source of this lane relative to the chunk's first row
    int dst_off[NOPS];            // ... and where it lands in the stage
#pragma unroll
    for (int t = 0; t < NOPS; ++t) {
        const int o = min(wave + W * t, 15), i = o & 7;
        if (o < 8) {
            src_lane[t] = kb + ((uint32_t)(4 * i + r4) * st2 + ((i & 1) ? sw_odd : sw_even));
            dst_off[t] = i * 1024;
        } else {
            src_lane[t] = vb + ((uint32_t)(8 * r4 + i) * st2 + vsw);
            dst_off[t] = 8192 + i * kVPiecePitch;
        }
    }
    auto issue = [&](int ci, int stg) -> uint32_t {
        char *dst = ring + stg * kStageBytes;
        int tok;
        if (ALIGNED) {
            if (ci - row_base >= 64) fill_rows(ci);
            const int r0 = __builtin_amdgcn_readlane(row0vec, ci - row_base);
            if (r0 >= 0) {
                const uint32_t row_off = (uint32_t)r0 * st2;   // fits 32 bits (host-checked)
#pragma unroll
                for (int t = 0; t < NOPS; ++t)
                    if (16 % W == 0 || t < NOPS - 1 || n_ops == NOPS)
                        __builtin_amdgcn_global_load_lds((glb_void_ptr)(src_lane[t] + row_off), (lds_void_ptr)(dst + dst_off[t]), 16, 0, kKvAux);
                return 0xffffffffu;
            }
            const int rr = -2 - r0;   // r0 == -1 gives -1
            tok = (rr >= 0 && rr + n < L) ? rr + n : -1;
        } else {
            tok = lane_row(ci);
        }
        const uint32_t vm = (uint32_t)__ballot(tok >= 0);
        const uint32_t tk = tok >= 0 ? (uint32_t)tok : 0u;   // row 0 exists (L > 0); masked later
#pragma unroll
        for (int t = 0; t < NOPS; ++t) {
            if (16 % W != 0 && t == NOPS - 1 && n_ops != NOPS) continue;
            const int o = wave + W * t, i = o & 7;
            if (o < 8) {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 4 * i + r4) * st2;
                dma16(kb + (tv + ((i & 1) ? sw_odd : sw_even)), dst + dst_off[t]);
            } else {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 8 * r4 + i) * st2;
                dma16(vb + (tv + vsw), dst + dst_off[t]);
            }
        }
        return vm;
    };

    bf16x8 qf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = as_bf16x8(qraw[ks]);
    if (ALIGNED && nch > 0) fill_rows(0);
    // from here on only this wavefront's DMA groups (n_ops operations each) are in flight (an
    // instruction the compiler knows, see attn_ctx_mfma_kernel)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");

    f32x16 O[4];
    float m_ref = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[j][i] = 0.f;

    // validity bits of the chunks in the ring: lane t holds those of stage t
    uint32_t vmv = 0u;
    for (int c = 0; c < kGroupAhead && c < nch; ++c) {
        const uint32_t vm = issue(c, c);
        vmv = lane == c ? vm : vmv;
    }
    // The barrier puts all eight wavefronts at the same point once per chunk; if they then all did
    // the same thing, they would queue for the LDS, then for the matrix cores, then for the vector
    // ALU.  So the two wavefronts of a SIMD (w and w + 4) run half a chunk apart: the second one
    // keeps P and V of its chunk in registers and does the O^T += V^T . P^T products after the next
    // barrier, while the first one reads its operands from LDS.
    uint2 v[16];
    uint4 pf0 = make_uint4(0u, 0u, 0u, 0u), pf1 = pf0;
    auto pv = [&]() {
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint2 lo = v[(ks2 * 4 + j) * 2], hi = v[(ks2 * 4 + j) * 2 + 1];
                O[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y)),
                                                               as_bf16x8(ks2 ? pf1 : pf0), O[j], 0, 0, 0);
            }
    };
    for (int i = 0; i < nch; ++i) {
        // own part of chunk i has landed: kGroupAhead - 1 younger groups of n_ops operations may
        // stay in flight (towards the end of the range there are fewer: wait for all, they are due anyway)
        if (i + kGroupAhead - 1 >= nch) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (n_ops == NOPS) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NOPS * (kGroupAhead - 1)) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NOPS - 1) * (kGroupAhead - 1)) : "memory");
        __builtin_amdgcn_s_barrier();   // ... and so have the others'; chunk i-1 has been read by all
        if (i + kGroupAhead < nch) {
            const int is = (i + kGroupAhead) & (kGroupStages - 1);
            const uint32_t vm = issue(i + kGroupAhead, is);
            vmv = lane == is ? vm : vmv;
        }
        const int rs = i & (kGroupStages - 1);
        const uint32_t vmask = (uint32_t)__builtin_amdgcn_readlane((int)vmv, rs);
        if (!live) continue;
        if (second && i > 0) pv();   // chunk i - 1, before its V registers are overwritten
        uint4 kf[8];
        {
            const uint32_t soff = (uint32_t)rs * kStageBytes;
            const uint32_t ka[4] = {kread[0] + soff, kread[1] + soff, kread[2] + soff, kread[3] + soff};
            lds_read_k4(ka, kf);
        }
        lds_read_v(vread + (uint32_t)rs * kStageBytes, v);
        f32x16 S;
#pragma unroll
        for (int x = 0; x < 16; ++x) S[x] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), qf[ks], S, 0, 0, 0);

        if (vmask != 0xffffffffu) {
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                const int tt = (x >> 2) * 8 + kg * 4 + (x & 3);
                if (!((vmask >> tt) & 1u)) S[x] = -INFINITY;
            }
        }
        float mx = fmaxf(S[0], S[1]);
#pragma unroll
        for (int x = 2; x < 16; x += 2) mx = fmaxf(fmaxf(mx, S[x]), S[x + 1]);
        mx = max_xor32(mx) * a.scale_log2;
        // the reference max only moves when the true max gets more than 2^slack ahead
        if (__any(mx > m_ref + kRescaleSlack)) {
            const float m_new = mx > m_ref + kRescaleSlack ? mx : m_ref;
            const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_ref - m_new);
            m_ref = m_new;
            l_run *= alpha;
            if (__any(alpha != 1.f && l_run != 0.f)) {   // nothing to rescale while O is still zero
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int x = 0; x < 16; ++x) O[j][x] *= alpha;
            }
        }
        const float m_use = m_ref == -INFINITY ? 0.f : m_ref;
        uint32_t pk[8];
        float lsum = 0.f;
#pragma unroll
        for (int x = 0; x < 16; x += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(S[x], a.scale_log2, -m_use));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(S[x + 1], a.scale_log2, -m_use));
            pk[x >> 1] = pack_bf16x2(p0, p1);
            lsum = add_bf16x2(pk[x >> 1], lsum);   // the sum runs over the rounded weights the MFMA sees
        }
        l_run += lsum;
        pf0 = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        pf1 = make_uint4(pk[4], pk[5], pk[6], pk[7]);
        if (!second) pv();
    }
    if (second && live && nch > 0) pv();
    __syncthreads();   // every wavefront is done with the ring: the epilogue reuses that LDS
    if (!live) return;

    // ---- one partial per (head, split, node): accumulators -> row-major through LDS ------
    l_run = sum_xor32(l_run);
    const int64_t prow0 = ((int64_t)(b * s.Hq + h) * part.nsplit + sp) * s.M;
    {
        // accumulator element 4q + x of tile j is channel 32j + 8q + 4kg + x of this lane's row
        float *dst = obuf + ((size_t)wave * 32 + n) * kOPitch;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4 *)(dst + 32 * j + 8 * q + 4 * kg) = make_float4(O[j][4 * q], O[j][4 * q + 1], O[j][4 * q + 2], O[j][4 * q + 3]);
    }
    // a wavefront reads back only what it wrote itself: no barrier
    const int jrow0 = m0;
#pragma unroll 8
    for (int uu = 0; uu < 32; ++uu) {
        const float2 x = *(const float2 *)(obuf + ((size_t)wave * 32 + uu) * kOPitch + partial_chan(2 * lane, 128));
        if (jrow0 + uu < s.M) store_partial(part.o + (prow0 + jrow0 + uu) * 128 + 2 * lane, x);   // positions 2 lane, 2 lane + 1 of the stored order
    }
    if (kg == 0 && jrow0 + n < s.M) *(float2 *)(part.ml + (prow0 + jrow0 + n) * 2) = make_float2(m_ref, l_run);
}

bool attn_ctx_mfma_supported(const Shape &s, int dtype)
{
    // per-lane byte offsets inside one (sequence, KV head) slab are kept in 32 bits
    const int64_t span = ((int64_t)s.max_blocks * s.B + 64) * s.st * 2;
    return dtype == SPECPV_BF16 && s.D == 128 && s.st % 8 == 0 && span < ((int64_t)1 << 31);
}

// Row blocks of 32 query rows per KV group, and how the group kernel deals them to workgroups.
struct GroupLayout {
    int rph, n_row_blocks, parts, waves;
};
static GroupLayout group_layout(const Shape &s)
{
    GroupLayout g;
    g.rph = (s.M + 31) / 32;
    g.n_row_blocks = s.G * g.rph;
    g.parts = (g.n_row_blocks + 7) / 8;
    const int w = (g.n_row_blocks + g.parts - 1) / g.parts;   // 1 .. 8
    g.waves = w <= 2 ? 2 : (w <= 4 ? 4 : (w <= 6 ? 6 : 8));
    return g;
}
int attn_group_parts(const Shape &s) { return group_layout(s).parts; }

hipError_t launch_attn_ctx_mfma(const Shape &s, const int32_t *sel_idx, const int32_t *sel_count,
                                int n_sel, Partials p, int kind, hipStream_t st)
{
    if (kind != kAttnSplit && kind != kAttnGroup) return hipErrorInvalidValue;
    const GroupLayout gl = group_layout(s);
    MfmaArgs a;
    a.sel_idx = sel_idx;
    a.sel_count = sel_count;
    a.n_sel = n_sel;
    a.scale_log2 = kLog2e / sqrtf(128.f);
    a.row_tiles = (s.M + 63) / 64;
    a.rph = gl.rph;
    a.n_row_blocks = gl.n_row_blocks;
    a.n_units = s.batch * s.Hkv * p.nsplit;
    a.n_bg = s.batch * s.Hkv;
    a.div_nsplit = make_fastdiv((uint32_t)p.nsplit);
    a.div_hkv = make_fastdiv((uint32_t)s.Hkv);
    a.div_B = make_fastdiv((uint32_t)s.B);
    // token ranges per split: four (one per token group of a workgroup), or one in the group kernel
    a.div_W = make_fastdiv((uint32_t)p.nsplit * (kind == kAttnGroup ? 1u : 4u));
    const int GR = kind == kAttnGroup ? gl.parts : s.G * a.row_tiles;
    // group kernel: a unit (sequence, KV head, split) per 8 consecutive x; split kernel: (sequence, KV
    // head) bg on XCD bg % 8 with all its splits and query heads (y = (bg / 8) * nsplit + split)
    const dim3 grid(8 * GR, kind == kAttnGroup ? (a.n_units + 7) / 8 : ((a.n_bg + 7) / 8) * p.nsplit);
    if (grid.y > 65535u) return hipErrorInvalidConfiguration;
    const bool aligned = s.B % 32 == 0;
    const size_t lds_split = 2048 + (size_t)max(kRingBytes, 4 * 64 * kOPitch * (int)sizeof(float));
    const size_t lds_group = (size_t)max(kGroupStages * kStageBytes, gl.waves * 32 * kOPitch * (int)sizeof(float));
#define SPECPV_LAUNCH(KERN, THREADS, LDS)                                                              \
    do {                                                                                               \
        static PerDeviceOnce once;   /* one per kernel instantiation */                               \
        auto kern = KERN;                                                                              \
        const hipError_t e0 = once.run([&] {                                                           \
            return hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(LDS)); \
        });                                                                                            \
        if (e0 != hipSuccess) return e0;                                                               \
        hipLaunchKernelGGL(kern, grid, dim3(THREADS), LDS, st, s, p, a);                                \
    } while (0)
#define SPECPV_LAUNCH_GROUP(WW)                                                                        \
    do {                                                                                               \
        if (aligned) SPECPV_LAUNCH((attn_ctx_mfma_group_kernel<true, WW>), 64 * WW, lds_group);         \
        else SPECPV_LAUNCH((attn_ctx_mfma_group_kernel<false, WW>), 64 * WW, lds_group);                \
    } while (0)
    if (kind == kAttnGroup) {
        switch (gl.waves) {
        case 2: SPECPV_LAUNCH_GROUP(2); break;
        case 4: SPECPV_LAUNCH_GROUP(4); break;
        case 6: SPECPV_LAUNCH_GROUP(6); break;
        default: SPECPV_LAUNCH_GROUP(8); break;
        }
    } else {
        if (aligned) SPECPV_LAUNCH(attn_ctx_mfma_kernel<true>, 512, lds_split);
        else SPECPV_LAUNCH(attn_ctx_mfma_kernel<false>, 512, lds_split);
    }
#undef SPECPV_LAUNCH_GROUP
#undef SPECPV_LAUNCH
    return hipGetLastError();
}

}  // namespace specpv
