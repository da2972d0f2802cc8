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
#include <type_traits>

namespace specpv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *glb_void_ptr;

constexpr int kOPitch = 132;         // floats per staged output row (128 + 4: conflict-free 16-byte writes)
// One 32-token chunk in LDS: 8 KiB of K (row-major, 16-byte pieces XOR-swizzled by row & 15: the LDS has 64
// banks, so the 16 lanes that a 16-byte read serves per cycle must cover all 16 pieces of a 256-byte bank row;
// with row & 7 the operand reads ran at half the rate) and
// the V rows in 8 pieces of 4 rows (tokens i, i+8, i+16, i+24 in piece i), 1088 bytes apart, for
// the transposing LDS reads (see lds_read_v).
constexpr int kVPiecePitch = 1088;
constexpr int kStageBytes = 8192 + 8 * kVPiecePitch;
constexpr int kStages = 2;           // ring depth per wavefront pair (eight-wavefront kernel)
constexpr int kRingBytes = 4 * kStages * kStageBytes;
constexpr int kQStageBytes = 2 * 8 * 1024;   // the query rows of a workgroup's two row blocks as MFMA operands (eight-wavefront kernel)
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

// Four such operations 1 KiB apart on both sides (K rows 4 i .. 4 i + 3 for i = 0 .. 3, or 4 .. 7): gbase is
// wavefront-uniform, row_off the lane's row (lane / 16) in bytes, sw0 its piece 16 * ((lane & 15) ^ (lane / 16));
// operation i fetches the piece that the swizzle by row & 15 puts at the lane's place, sw0 ^ 64 i.  The
// immediate offset of the instruction is added to the global and to the LDS address.
__device__ __forceinline__ void dma16x4(const char *gbase, uint32_t row_off, uint32_t sw0, char *lds_dst)
{
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + (row_off + sw0)), (lds_void_ptr)lds_dst, 16, 0, kKvAux);
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + (row_off + (sw0 ^ 64u))), (lds_void_ptr)lds_dst, 16, 1024, kKvAux);
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + (row_off + (sw0 ^ 128u))), (lds_void_ptr)lds_dst, 16, 2048, kKvAux);
    __builtin_amdgcn_global_load_lds((glb_void_ptr)(gbase + (row_off + (sw0 ^ 192u))), (lds_void_ptr)lds_dst, 16, 3072, kKvAux);
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

// Four k-steps (half of a chunk's K operands).
template <int OFF> __device__ __forceinline__ void lds_read_k_half(const uint32_t (&a)[4], uint4 (&k)[4])
{
    asm volatile(
        "ds_read_b128 %0, %4 offset:%8\n\t"
        "ds_read_b128 %1, %5 offset:%8\n\t"
        "ds_read_b128 %2, %6 offset:%8\n\t"
        "ds_read_b128 %3, %7 offset:%8\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(k[0]), "=&v"(k[1]), "=&v"(k[2]), "=&v"(k[3])
        : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "n"(OFF)
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
// OFF: a constant byte offset (a ring stage), added by the instructions themselves.
template <int OFF = 0>
__device__ __forceinline__ void lds_read_v(uint32_t addr, uint2 (&v)[16])
{
    static_assert(OFF >= 0 && OFF + 960 < 65536, "the offset field has 16 bits");
    asm volatile(
        "ds_read_b64_tr_b16 %0, %16 offset:%17\n\t"
        "ds_read_b64_tr_b16 %1, %16 offset:%17+256\n\t"
        "ds_read_b64_tr_b16 %2, %16 offset:%17+64\n\t"
        "ds_read_b64_tr_b16 %3, %16 offset:%17+320\n\t"
        "ds_read_b64_tr_b16 %4, %16 offset:%17+128\n\t"
        "ds_read_b64_tr_b16 %5, %16 offset:%17+384\n\t"
        "ds_read_b64_tr_b16 %6, %16 offset:%17+192\n\t"
        "ds_read_b64_tr_b16 %7, %16 offset:%17+448\n\t"
        "ds_read_b64_tr_b16 %8, %16 offset:%17+512\n\t"
        "ds_read_b64_tr_b16 %9, %16 offset:%17+768\n\t"
        "ds_read_b64_tr_b16 %10, %16 offset:%17+576\n\t"
        "ds_read_b64_tr_b16 %11, %16 offset:%17+832\n\t"
        "ds_read_b64_tr_b16 %12, %16 offset:%17+640\n\t"
        "ds_read_b64_tr_b16 %13, %16 offset:%17+896\n\t"
        "ds_read_b64_tr_b16 %14, %16 offset:%17+704\n\t"
        "ds_read_b64_tr_b16 %15, %16 offset:%17+960\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7]),
          "=&v"(v[8]), "=&v"(v[9]), "=&v"(v[10]), "=&v"(v[11]), "=&v"(v[12]), "=&v"(v[13]), "=&v"(v[14]), "=&v"(v[15])
        : "v"(addr), "n"(OFF)
        : "memory");
}

// Half of that: the operands of token half ks2 (OFF = 512 ks2), v[j * 2 + hf].
template <int OFF> __device__ __forceinline__ void lds_read_v_half(uint32_t addr, uint2 (&v)[8])
{
    asm volatile(
        "ds_read_b64_tr_b16 %0, %8 offset:%9\n\t"
        "ds_read_b64_tr_b16 %1, %8 offset:%10\n\t"
        "ds_read_b64_tr_b16 %2, %8 offset:%11\n\t"
        "ds_read_b64_tr_b16 %3, %8 offset:%12\n\t"
        "ds_read_b64_tr_b16 %4, %8 offset:%13\n\t"
        "ds_read_b64_tr_b16 %5, %8 offset:%14\n\t"
        "ds_read_b64_tr_b16 %6, %8 offset:%15\n\t"
        "ds_read_b64_tr_b16 %7, %8 offset:%16\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
        : "v"(addr), "n"(OFF), "n"(OFF + 256), "n"(OFF + 64), "n"(OFF + 320), "n"(OFF + 128), "n"(OFF + 384), "n"(OFF + 192),
          "n"(OFF + 448)
        : "memory");
}

// The split-KV partials are written once here and read once by the combine kernel, which runs on
// other CUs (and mostly other XCDs): stored with the streaming hint they do not linger in this
// XCD's L2 as dirty lines that the end of the kernel has to write back (measured: 3.6 % of the
// partial-verify step).
// Two values of a split's normalised result as fp16 (clamped to fp16's range), one streaming 4-byte store.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_partial_half(float *row, int lane, float a, float b)
{
    const f16x2 hv = {(_Float16)__builtin_amdgcn_fmed3f(a, -65504.f, 65504.f), (_Float16)__builtin_amdgcn_fmed3f(b, -65504.f, 65504.f)};
    __builtin_nontemporal_store(__builtin_bit_cast(uint32_t, hv), (uint32_t *)row + lane);
}
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


__device__ __forceinline__ float max_xor16(float x)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor16(float x)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// Sum over the 16 lanes of a DPP row, result in every lane of the row: lane ^ 1, lane ^ 2, then the
// mirrors inside 8 and 16 lanes.
template <int CTRL> __device__ __forceinline__ float dpp_row_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_row_f32<0xB1>(x);
    x += dpp_row_f32<0x4E>(x);
    x += dpp_row_f32<0x141>(x);
    x += dpp_row_f32<0x140>(x);
    return x;
}
// max / sum over the 8 lanes 8 u .. 8 u + 7 (lane ^ 1, lane ^ 2, mirror inside 8)
__device__ __forceinline__ float oct_max(float x)
{
    x = fmaxf(x, dpp_row_f32<0xB1>(x));
    x = fmaxf(x, dpp_row_f32<0x4E>(x));
    x = fmaxf(x, dpp_row_f32<0x141>(x));
    return x;
}
__device__ __forceinline__ float oct_sum(float x)
{
    x += dpp_row_f32<0xB1>(x);
    x += dpp_row_f32<0x4E>(x);
    x += dpp_row_f32<0x141>(x);
    return x;
}
// The root path of tree node j as a bit set; par0 / par1 hold parent[lane] / parent[lane + 64].
// Everything is wave-uniform (scalar registers).
// Nodes below `stop` (partially verified tokens that the context kernels attend) end the walk.
__device__ __forceinline__ void root_path(int j, int n_nodes, int stop, int par0, int par1, unsigned long long &lo,
                                          unsigned long long &hi)
{
    int aa = j;
    for (int guard = 0; aa >= stop && guard < n_nodes; ++guard) {
        if (aa < 64) lo |= 1ull << aa; else hi |= 1ull << (aa - 64);
        const int pa = aa < 64 ? __builtin_amdgcn_readlane(par0, aa) : __builtin_amdgcn_readlane(par1, aa - 64);
        aa = pa < aa ? pa : -1;   // a malformed parent[] (not strictly decreasing) ends the walk
    }
}
// lowest node of the set (removed from it), or -1
__device__ __forceinline__ int pop_node(unsigned long long &lo, unsigned long long &hi)
{
    int aa = -1;
    if (lo) { aa = __builtin_ctzll(lo); lo &= lo - 1; }
    else if (hi) { aa = 64 + __builtin_ctzll(hi); hi &= hi - 1; }
    return aa;
}

// ---- eight-wavefront kernel: one query head, one tile of up to 64 nodes, one KV split ----------
// grid: x = r * 8 + xcd   (r = query head within the group + G * row tile),
//       y = (bg / 8) * nsplit + split   with bg = b * Hkv + g and xcd = bg % 8.
// Workgroups are handed to the 8 XCDs round-robin in linear order and gridDim.x is a multiple of
// 8, so a (sequence, KV head) stays on XCD bg % 8 with all its splits and query heads: the K/V
// bytes of a split come from HBM once and from that XCD's L2 for the other query heads, and the
// split-KV partials of a head meet in one L2.
//
// Workgroup = 8 wavefronts = 4 token groups x 2 row blocks.  Wavefronts tg and tg + 4
// sit on the same SIMD, work on the same chunks (rows 0..31 and 32..63 of the tile)
// and share one LDS ring; the first of the pair requests the K rows, the second the V
// rows.  Two workgroup barriers per chunk order "DMA landed -> both read" and "both
// read -> stage may be refilled".  Every wavefront runs the same number of iterations
// (the largest chunk count in the workgroup), so the barriers always match up.
//
// FUSED: the whole call in this one kernel.
//  * The draft-tree segment (a node attends itself and its ancestors, tree decode of Algorithm 1)
//    is one more partial per row, in slot `nctx` behind the context splits: the workgroup of
//    split sp computes it for the rows r = sp (mod nctx) of its tile on the vector ALU, one row
//    per wavefront, while its first K/V chunks are on their way.
//  * Partials are stored with ordinary stores (they stay in this XCD's L2), then the workgroup
//    adds itself to the tile's arrival word (one 64-bit atomic add: arrival count in the top byte,
//    7 bits of count per hardware XCC id below).  No workgroup ever waits for another one.
//  * The workgroup whose add completes the count merges the nctx + 1 partials of its tile by their
//    log-sum-exp weights, normalises, stores out / lse and zeroes the word.  It reads the
//    others' partials from L2, which is only right if they were written through the SAME L2: if
//    the XCC ids in the word say that any workgroup of the tile ran elsewhere (never seen; the
//    dispatcher's round-robin is not a documented guarantee), the last workgroup recomputes the
//    tile from scratch instead -- every split and the draft segment, merged in its own registers --
//    so the result never depends on where workgroups run.
constexpr int kXccBits = 7;
#ifdef SPECPV_TIMELINE
#define SPECPV_STAMP(i)                                                                                       \
    do {                                                                                                      \
        if (f.timeline && threadIdx.x == 0 && !REDO)                                                          \
            f.timeline[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 16 + (i)] = __builtin_amdgcn_s_memrealtime(); \
    } while (0)
// core clock against real time over a workgroup's life: cycles, 10 ns ticks and the number of chunks go to
// words 0 .. 2 of row ROW of the stamp buffer (the real-time counter runs at 100 MHz whatever the chip does,
// s_memtime counts core cycles)
#define SPECPV_CLOCKS_BEGIN const unsigned long long clk0_ = clock64(), rt0_ = __builtin_amdgcn_s_memrealtime()
#define SPECPV_CLOCKS_END(TL, ROW, NCH)                                                                       \
    do {                                                                                                      \
        if ((TL) && threadIdx.x == 0 && (size_t)(ROW) < 4096) {                                               \
            unsigned long long *t_ = (TL) + (size_t)(ROW) * 16;                                               \
            t_[0] = clock64() - clk0_;                                                                        \
            t_[1] = __builtin_amdgcn_s_memrealtime() - rt0_;                                                  \
            t_[2] = (unsigned long long)(NCH);                                                                \
        }                                                                                                     \
    } while (0)
#else
#define SPECPV_STAMP(i) do {} while (0)
#define SPECPV_CLOCKS_BEGIN do {} while (0)
#define SPECPV_CLOCKS_END(TL, ROW, NCH) do {} while (0)
#endif        // per-XCC arrival count (splits <= 64)

// One pass over the token ranges of split `sp0` of `ns_eff` splits.  REDO = false: the ordinary pass of
// a workgroup (ns_eff = nctx); returns true if this workgroup, the last of its tile, has to take the
// recompute route.  REDO = true: that route -- the pass runs as the only split of one (sp0 = 0, ns_eff = 1).
// Everything, the argument-dependent reads included, is done again in the second pass, so that it keeps
// no register of the first one alive.
// PEND: partially verified tokens may stand in front of the tree (s.kctx > 0); without it the kernel is the one
// that the headline shape runs, free of that path's registers and tests.
template <bool ALIGNED, bool FUSED, bool REDO, bool PEND>
__device__ __forceinline__ bool attn_ctx_pass(Shape s, Partials part, MfmaArgs a, FusedArgs f, const int nctx,
                                              const int sp0, const int ns_eff, char *lds_raw)
{
    float *ms = (float *)lds_raw;            // [4 token groups][64 rows]
    float *ls = ms + 4 * 64;                 // [4][64]
    char *ring = lds_raw + 2048;             // [4 pairs][kStages][K 8 KiB | V 8 KiB]
    float *obuf = (float *)(lds_raw + 2048); // [4][64][kOPitch], reuses the ring after the main loop
    constexpr bool redo = REDO;
    const int sp = sp0;
    SPECPV_CLOCKS_BEGIN;
    SPECPV_STAMP(0);   // entry

    // ---- which piece of work is this workgroup -------------------------------------
    const int xcd = blockIdx.x & 7, r = blockIdx.x >> 3;
    const int bgh = (int)a.div_nsplit.div(blockIdx.y);
    const int bg = bgh * 8 + xcd;
    if (bg >= a.n_bg) return false;
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
    // length, list length, the kept-block list (up to 256 entries, lane t: entries t, t + 64, ..),
    // the query rows, and for the draft segment the parents and this wavefront's first row.
    const int32_t *sel = a.sel_idx ? a.sel_idx + (int64_t)bg * a.n_sel : nullptr;
    const uint32_t Bu = (uint32_t)s.B;
    const int L = s.ctx_len[b];
    const int cnt_raw = sel ? a.sel_count[bg] : 0;
    const bool list_in_regs = ALIGNED && sel && a.n_sel <= 256;
    int idv[4] = {-1, -1, -1, -1};
    if (list_in_regs) {
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if (lane + 64 * x < a.n_sel) idv[x] = sel[lane + 64 * x];
    }
    // The query rows of a row block are the same for its four wavefronts (one per token group): each brings
    // a quarter of them (k-steps 2 tg, 2 tg + 1) straight into LDS, laid out as the operands are read
    // (k-step ks of row block rb: 1 KiB, lane l's 16 bytes at 16 l), and all four read the whole from there
    // once the requests have landed -- a quarter of the bytes through the CU's memory path in the phase
    // where the first K / V chunks are requested.
    char *qstage = lds_raw + 2048 + max(kRingBytes, 4 * 64 * kOPitch * (int)sizeof(float));
    {
        const int j = min(m0 + rb * 32 + n, s.M - 1);   // rows past M repeat row M-1; never stored
        const char *qrow = (const char *)((const uint16_t *)s.q + (((int64_t)b * s.M + j) * s.Hq + h) * 128 + kg * 8);
        char *dst = qstage + (rb * 8 + 2 * tg) * 1024;
        __builtin_amdgcn_global_load_lds((glb_void_ptr)(qrow + 64 * tg), (lds_void_ptr)dst, 16, 0, 0);   // a k-step is 16 channels: 32 bytes
        __builtin_amdgcn_global_load_lds((glb_void_ptr)(qrow + 64 * tg + 32), (lds_void_ptr)(dst + 1024), 16, 0, 0);
    }
    const int rows_tile = min(64, s.M - m0);            // >= 1
    int par0 = -1, par1 = -1;
    uint4 qd_first = make_uint4(0u, 0u, 0u, 0u);
    if (FUSED) {
        const int32_t *par = s.parent + (int64_t)b * s.Mk;
        if (lane < s.Mk) par0 = par[lane];
        if (lane + 64 < s.Mk) par1 = par[lane + 64];
        const int r0 = min(sp0 + ns_eff * wave, rows_tile - 1);
        qd_first = *(const uint4 *)((const uint16_t *)s.q + (((int64_t)b * s.M + m0 + r0) * s.Hq + h) * 128 + (lane & 15) * 8);
    }

    int nb = L > 0 ? (int)a.div_B.div((uint32_t)(L + s.B - 1)) : 0;
    if (nb > s.max_blocks) nb = s.max_blocks;
    int cnt = nb;
    if (sel) cnt = max(0, min(cnt_raw, a.n_sel));
    const uint32_t T = nb > 0 ? (uint32_t)cnt * Bu : 0u;   // host guarantees max_blocks * B <= 2^30
    // chunks of cache tokens, then the chunks of the partially verified tokens (the first kctx draft nodes: a
    // chain that every query node descends from, so all rows attend all of them, like cache tokens)
    const uint32_t C_ctx = (T + 31u) >> 5;
    const int kctx = PEND ? s.kctx : 0;
    const uint32_t C = C_ctx + (((uint32_t)kctx + 31u) >> 5);
    const char *kdb = (const char *)s.kd + (((int64_t)b * s.Mk) * s.Hkv + g) * 256;
    const char *vdb = (const char *)s.vd + (((int64_t)b * s.Mk) * s.Hkv + g) * 256;
    const uint32_t stp = (uint32_t)s.Hkv * 256u;   // bytes from one draft node's row to the next

    // uniform slab bases; per-lane byte offsets inside a slab fit 32 bits (host-checked)
    const char *kb = (const char *)s.k + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const char *vb = (const char *)s.v + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const uint32_t st2 = (uint32_t)s.st * 2u;   // bytes per token row step

    char *my_ring = ring + tg * (kStages * kStageBytes);
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)my_ring;
    // K tile in LDS: row-major, 256 B per token, the 16-byte pieces of row t stored at
    // piece index (p ^ (t & 15)) so that the operand reads below (16 lanes per cycle, same piece,
    // different rows) spread over all 64 banks.  Operand piece of k-step ks: 2*ks + kg.
    uint32_t kread[4];   // + stage * kStageBytes; k-step ks + 4: the address XOR 128 (rows and stages start 256-byte aligned)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        kread[ks] = ring_addr + (uint32_t)n * 256u + (((uint32_t)(32 * ks + 16 * kg)) ^ (16u * ((uint32_t)n & 15u)));
    const uint32_t vread = ring_addr + 8192u + (uint32_t)(4 * kg + ((lane & 15) >> 2)) * kVPiecePitch +
                           32u * (uint32_t)((lane >> 4) & 1) + 8u * (uint32_t)(lane & 3);   // + stage * kStageBytes

    bf16x8 qf[8];   // Q fragments (B operand of S^T = K . Q^T): row = lane & 31; read from LDS in front of the main loop

    const int r4 = lane >> 4, pos = lane & 15;
    const uint32_t sw0 = 16u * (uint32_t)(pos ^ r4), vsw = 16u * (uint32_t)pos;   // K row 4 i + r4: piece pos ^ ((4 i + r4) & 15) = sw0 ^ 64 (i & 3)
    const uint32_t lane_row_off = (uint32_t)r4 * st2;
    constexpr int RPW = 8;  // rows each wavefront finishes in the epilogue

    const int W = ns_eff * 4, wsid = sp * 4 + tg;
    // chunks of a list that precede the share of token group w; shares differ by at most one
    auto first_chunk = [&](uint32_t chunks, int w) -> int {
        const uint32_t base = redo ? (chunks >> 2) : a.div_W.div(chunks), rem = chunks - base * (uint32_t)W;
        return (int)((uint32_t)w * base + min((uint32_t)w, rem));
    };
    const int c0 = first_chunk(C, wsid), c1 = first_chunk(C, wsid + 1);
    const int nch = c1 - c0;
    const int nch_max = first_chunk(C, sp * 4 + 1) - first_chunk(C, sp * 4);   // token group 0 has the most
    if (!FUSED) SPECPV_STAMP(9);   // the scalar reads (lengths, list length) are in: the chunk counts are known

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
        if (cb + lane < nch && (uint32_t)(c0 + cb + lane) < C_ctx) {
            const uint32_t p0 = (uint32_t)(c0 + cb + lane) * 32u;   // < T: the slot below is < cnt
            const uint32_t slot = a.div_B.div(p0);
            r = encode_row(sel ? sel[slot] : (int)slot, p0, slot);
        }
        row0vec = r;
        // wait for the list entries here, inside the rare branch, so that the common path that
        // joins behind it carries no pending load (and no wait on the DMA prefetch)
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    };
    // the first 64 chunks: the list sits in registers (lane t: entries t, t + 64, ...), so this is a
    // cross-lane read and no second trip to memory
    auto fill_rows_first = [&]() {
        if (!list_in_regs) { fill_rows(0); return; }
        const uint32_t p0 = (uint32_t)(c0 + lane) * 32u;
        const uint32_t slot = a.div_B.div(p0);
        const int src = (int)(slot & 63u);
        const int e0 = __shfl(idv[0], src), e1 = __shfl(idv[1], src), e2 = __shfl(idv[2], src), e3 = __shfl(idv[3], src);
        const int q4 = (int)(slot >> 6);
        const int blk = q4 == 0 ? e0 : (q4 == 1 ? e1 : (q4 == 2 ? e2 : e3));
        row0vec = (lane < nch && (uint32_t)(c0 + lane) < C_ctx) ? encode_row(blk, p0, slot) : -1;   // p0 < T there: the slot is < cnt
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
    // rows given per lane (t = lane & 31: token tk of the chunk, bits vm say which are real)
    auto issue_rows = [&](const char *kbase, const char *vbase, const uint32_t stride, const uint32_t tk, char *dst, char *dstv) {
        if (rb == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 4 * i + r4) * stride;
                dma16(kbase + (tv + (sw0 ^ (64u * (uint32_t)(i & 3)))), dst + i * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 8 * r4 + i) * stride;
                dma16(vbase + (tv + vsw), dstv + i * kVPiecePitch);
            }
        }
    };
    auto issue = [&](int ci) {
        const int stg = ci & (kStages - 1);
        char *dst = my_ring + stg * kStageBytes;
        char *dstv = dst + 8192;
        int tok;
        if (PEND && kctx > 0 && (uint32_t)(c0 + ci) >= C_ctx) {
            // a chunk of partially verified tokens: rows of the draft K / V arrays
            const int pr = (int)((uint32_t)(c0 + ci) - C_ctx) * 32 + n;
            const int ptok = pr < kctx ? pr : -1;
            vmask_st[stg] = (uint32_t)__ballot(ptok >= 0);
            issue_rows(kdb, vdb, stp, (uint32_t)max(ptok, 0), dst, dstv);
            return;
        }
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
                        dma16x4(kb + row0, lane_row_off, sw0, dst);
                        dma16x4(kb + row0 + 4096, lane_row_off, sw0, dst + 4096);
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
                        dma16(kb + row0 + (size_t)(4 * i) * st2 + (lane_row_off + (sw0 ^ (64u * (uint32_t)(i & 3)))), dst + i * 1024);
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
        issue_rows(kb, vb, st2, tk, dst, dstv);
    };

    if (ALIGNED && nch > 0) fill_rows_first();
    // every load above has been consumed here: from now on the only vector-memory
    // operations of this wavefront in flight are its own DMA groups (8 operations each)
    // (as an instruction the compiler knows, not inline assembly: otherwise it assumes that the
    // loads of the prologue may still be in flight at the loop header and waits for vmcnt(0),
    // i.e. for the prefetch just issued, at the first use of Q in every iteration)
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), expcnt and lgkmcnt untouched
    asm volatile("" ::: "memory");
    SPECPV_STAMP(1);   // arguments, lengths, list, query rows, parents are in

    // ---- draft-tree segment of this workgroup's rows (FUSED) --------------------------------
    // Row r of the tile (node koff + m0 + r) is handled by the workgroup with sp = r mod ns_eff, there
    // by wavefront (r / ns_eff) mod 8.  Sixteen lanes per draft node (a lane owns 8 adjacent
    // channels), four nodes of the root path at a time; the result goes to slot nctx of the
    // partial arrays like any other partial.  For a wavefront's first row the first two rounds of
    // K / V rows (8 path nodes) are requested in front of the first context chunks.
    auto draft_row = [&](int row, bool live, bool with_chunks) {
        const int jn = s.koff + m0 + row;
        unsigned long long anc_lo = 0ull, anc_hi = 0ull;
        root_path(jn, s.Mk, kctx, par0, par1, anc_lo, anc_hi);
        const int n0 = pop_node(anc_lo, anc_hi), n1 = pop_node(anc_lo, anc_hi), n2 = pop_node(anc_lo, anc_hi),
                  n3 = pop_node(anc_lo, anc_hi), n4 = pop_node(anc_lo, anc_hi), n5 = pop_node(anc_lo, anc_hi),
                  n6 = pop_node(anc_lo, anc_hi), n7 = pop_node(anc_lo, anc_hi);
        const int na = r4 == 0 ? n0 : (r4 == 1 ? n1 : (r4 == 2 ? n2 : n3));
        const int nb2 = r4 == 0 ? n4 : (r4 == 1 ? n5 : (r4 == 2 ? n6 : n7));
        auto drow = [&](const void *base, int node) -> const uint16_t * {
            return (const uint16_t *)base + (((int64_t)b * s.Mk + max(node, 0)) * s.Hkv + g) * 128 + pos * 8;
        };
        uint4 qd = qd_first;
        if (!with_chunks) qd = *(const uint4 *)((const uint16_t *)s.q + (((int64_t)b * s.M + m0 + row) * s.Hq + h) * 128 + pos * 8);
        // requested in front of the first context chunks; the compiler places the wait (it waits for the
        // chunks as well: in-flight registers that it does not know about are not safe to hold)
        const uint4 ka = *(const uint4 *)drow(s.kd, na), va = *(const uint4 *)drow(s.vd, na);
        const uint4 kb2 = *(const uint4 *)drow(s.kd, nb2), vb2 = *(const uint4 *)drow(s.vd, nb2);
        if (with_chunks) {
            if (nch > 0) issue(0);
            if (nch > 1) issue(1);
        }
        float qv[8];
        Elem<bf16_t>::unpack(qd, qv);
        float md = -INFINITY, ld = 0.f, od[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) od[x] = 0.f;
        auto one = [&](int node, const uint4 &kraw, const uint4 &vraw) {
            float kf[8], vf[8];
            Elem<bf16_t>::unpack(kraw, kf);
            Elem<bf16_t>::unpack(vraw, vf);
            float dot = 0.f;
#pragma unroll
            for (int x = 0; x < 8; ++x) dot = fmaf(qv[x], kf[x], dot);
            const float z = node >= 0 ? row16_sum(dot) * a.scale_log2 : -INFINITY;
            const float m_new = fmaxf(md, z);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(md - m_use);   // 0 while nothing has been seen
            const float pe = __builtin_amdgcn_exp2f(z - m_use);      // 0 for an empty slot
            ld = fmaf(ld, alpha, pe);
#pragma unroll
            for (int x = 0; x < 8; ++x) od[x] = fmaf(od[x], alpha, pe * vf[x]);
            md = m_new;
        };
        one(na, ka, va);
        one(nb2, kb2, vb2);
        while (anc_lo | anc_hi) {   // root paths longer than 8 nodes (these reads queue behind the chunks)
            const int c0n = pop_node(anc_lo, anc_hi), c1n = pop_node(anc_lo, anc_hi), c2n = pop_node(anc_lo, anc_hi),
                      c3n = pop_node(anc_lo, anc_hi);
            const int nc = r4 == 0 ? c0n : (r4 == 1 ? c1n : (r4 == 2 ? c2n : c3n));
            const uint4 kc = *(const uint4 *)drow(s.kd, nc), vc = *(const uint4 *)drow(s.vd, nc);
            one(nc, kc, vc);
        }
        // the four lane groups hold disjoint parts of the path: merge them (lanes ^16, ^32)
        const float m_all = max_xor32(max_xor16(md));          // finite: the node itself is on its path
        const float wgt = __builtin_amdgcn_exp2f(md - m_all);   // 0 for a group without a node
        ld = sum_xor32(sum_xor16(ld * wgt));
#pragma unroll
        for (int x = 0; x < 8; ++x) od[x] = sum_xor32(sum_xor16(od[x] * wgt));
        if (live && r4 == 0) {
            // channels 8 pos .. 8 pos + 7 sit at positions 4 pos .. + 3 and 64 + 4 pos .. + 3 of the stored order
            const int64_t prow = ((int64_t)(b * s.Hq + h) * part.nsplit + nctx) * s.M + m0 + row;
            float *po = part.o + prow * 128;
            *(float4 *)(po + 4 * pos) = make_float4(od[0], od[1], od[2], od[3]);
            *(float4 *)(po + 64 + 4 * pos) = make_float4(od[4], od[5], od[6], od[7]);
            if (pos == 0) *(float2 *)(part.ml + prow * 2) = make_float2(m_all, ld);
        }
    };
    auto draft_rows = [&]() {
        const int rr0 = sp + ns_eff * wave;
        draft_row(min(rr0, rows_tile - 1), rr0 < rows_tile, true);      // requests chunks 0 and 1 on its way
        for (int rr = rr0 + ns_eff * 8; rr < rows_tile; rr += ns_eff * 8) draft_row(rr, true, false);
    };

    f32x16 O[4];
    float m_ref = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[j][i] = 0.f;

    // ---- main loop ---------------------------------------------------------------------
    // The query operands: this wavefront's quarter has landed (the wait for everything requested in the prologue,
    // above); the barrier covers the other wavefronts' quarters.
    auto read_q = [&]() {
        const uint32_t q0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)qstage + (uint32_t)(rb * 8192 + lane * 16);
        const uint32_t qa[8] = {q0, q0 + 1024u, q0 + 2048u, q0 + 3072u, q0 + 4096u, q0 + 5120u, q0 + 6144u, q0 + 7168u};
        uint4 qraw[8];
        lds_read_k<0>(qa, qraw);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = as_bf16x8(qraw[ks]);
    };
    if (FUSED) {
        draft_rows();
    } else {
        if (nch > 0) issue(0);
        if (nch > 1) issue(1);
    }
    SPECPV_STAMP(2);   // first chunks requested, draft rows done
    for (int i = 0; i < nch_max; ++i) {
        const bool active = i < nch;
        const int stg = i & 1;
        if (i < 4) SPECPV_STAMP(12 + i);   // done with chunk i - 1, about to wait for chunk i
        // own half of chunk i has landed (the only younger group is chunk i+1's)
        if (i + 1 < nch) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();          // ... and so has the partner's half
        if (i < 4) SPECPV_STAMP(3 + i);   // chunk i has landed
        if (i == 0) read_q();
        uint4 kf[8];
        uint2 v[16];
        const uint32_t vmask = vmask_st[stg];
        if (active) {
            const uint32_t soff = (uint32_t)stg * kStageBytes;
            const uint32_t k0 = kread[0] + soff, k1 = kread[1] + soff, k2 = kread[2] + soff, k3 = kread[3] + soff;
            const uint32_t ka[8] = {k0, k1, k2, k3, k0 ^ 128u, k1 ^ 128u, k2 ^ 128u, k3 ^ 128u};
            lds_read_k<0>(ka, kf);
            lds_read_v<0>(vread + soff, v);
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
        mx *= a.scale_log2;
        // the reference max only moves when the true max gets more than 2^slack ahead (tested on each lane's half of
        // the chunk's tokens; the row's maximum is formed behind the branch -- in the group kernel the same change
        // measured 3 % slower, so it keeps the exchange in front)
        if (__any(mx > m_ref + kRescaleSlack)) {
            mx = max_xor32(mx);
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
    SPECPV_STAMP(7);   // main loop done

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
        // fp32 partials (single-kernel route): positions 2 lane, 2 lane + 1 of the stored order; fp16 partials:
        // channels 2 lane, 2 lane + 1, normalised by the row's l
        const int chan0 = FUSED ? partial_chan(2 * lane, 128) : 2 * lane;
        const float il = l_row > 0.f ? 1.f / l_row : 0.f;
        float2 acc[RPW];
#pragma unroll
        for (int uu = 0; uu < RPW; ++uu) {
            const int row = wave * RPW + uu;
            acc[uu] = make_float2(0.f, 0.f);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float ww = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wgt[w]), uu));   // uniform: no LDS shuffle
                const float2 x = *(const float2 *)(obuf + ((size_t)w * 64 + row) * kOPitch + chan0);
                acc[uu].x = fmaf(ww, x.x, acc[uu].x);
                acc[uu].y = fmaf(ww, x.y, acc[uu].y);
            }
        }
#pragma unroll
        for (int uu = 0; uu < RPW; ++uu) {
            const int j = m0 + wave * RPW + uu;
            if (j < s.M) {
                if (FUSED) {
                    *(float2 *)(part.o + (prow0 + j) * 128 + 2 * lane) = acc[uu];   // stays in this XCD's L2
                } else {
                    const float ilu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(il), uu));
                    store_partial_half(part.o + (prow0 + j) * 64, lane, acc[uu].x * ilu, acc[uu].y * ilu);   // 128 halves per row
                }
            }
        }
    }
    if (lane < RPW) {
        const int j = m0 + wave * RPW + lane;
        if (j < s.M) *(float2 *)(part.ml + (prow0 + j) * 2) = make_float2(m_row, l_row);
    }
    SPECPV_STAMP(8);   // partial stores issued
    if (!REDO) SPECPV_CLOCKS_END(f.timeline, 3072 + ((size_t)blockIdx.y * gridDim.x + blockIdx.x), C);
    if (!FUSED) {
        // The combine kernel that follows reads the tree's parents and, one trip later, its K / V rows: nobody
        // has touched those in this call yet.  Ask for them here, on the way out (nothing waits for the data):
        // they are then in this XCD's L2, where that kernel's workgroups of the same KV head run.
        if (wave == 0 && s.kd && s.vd && s.parent) {
            const int nw = s.G * nctx, w = hh * nctx + sp;
            const char *base = (lane & 16) ? (const char *)s.vd : (const char *)s.kd;
            for (int node = w; node < s.Mk; node += nw) {
                uint32_t tmp;
                const char *p = base + (((int64_t)b * s.Mk + node) * s.Hkv + g) * 256 + (lane & 15) * 16;
                if (lane < 32) asm volatile("global_load_dword %0, %1, off" : "=v"(tmp) : "v"(p) : "memory");
            }
            if (w == 0 && lane < 2) {
                uint32_t tmp;
                const char *p = (const char *)(s.parent + (int64_t)b * s.Mk) + lane * 256;
                if (lane * 64 < s.Mk) asm volatile("global_load_dword %0, %1, off" : "=v"(tmp) : "v"(p) : "memory");
            }
        }
        return false;
    }

    // ---- arrival; the last workgroup of the tile finishes it (FUSED) ------------------------
    unsigned long long *word = f.arrive + ((int64_t)(b * s.Hq + h) * 2 + rt);
    unsigned long long *sh_word = (unsigned long long *)lds_raw;   // ms / ls are dead
    int nslots, slot_step;
    if (!redo) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // this wavefront's partial stores have reached L2
        __syncthreads();                      // ... and everybody else's
        SPECPV_STAMP(9);   // partial stores acknowledged
        if (threadIdx.x == 0) {
            const unsigned xcc = (unsigned)__builtin_amdgcn_s_getreg(20 | (3 << 11)) & 7u;   // XCC_ID, 4 bits
            const unsigned long long inc = (1ull << 56) | (1ull << (kXccBits * xcc));
            const unsigned long long now = __hip_atomic_fetch_add(word, inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + inc;
            // all arrivals through this XCC's L2?
            const bool here = ((now >> (kXccBits * xcc)) & ((1ull << kXccBits) - 1ull)) == (unsigned long long)nctx;
            sh_word[0] = now >> 56;
            sh_word[1] = (here && !f.force_recompute) ? 1ull : 0ull;
        }
        __syncthreads();
        SPECPV_STAMP(10);  // arrival known
        if ((int)sh_word[0] != nctx) return false;      // not the last one: done
        if (sh_word[1] == 0ull) {
            __syncthreads();                  // sh_word has been read by all
            return true;                      // recompute route: everything of this tile once more, here
        }
        nslots = nctx + 1; slot_step = 1;
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        nslots = 2; slot_step = nctx;        // this pass's partial (slot 0) and its draft segment (slot nctx)
    }
    if (threadIdx.x == 0) __hip_atomic_exchange(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // Merge.  Lane 8 u + x owns the (m, l) pairs of row u of this wavefront's 8 rows for the slots
    // x, x + 8, ...; the weights pass through LDS (a wavefront's own corner: its LDS operations are
    // executed in order, no barrier).  Every lane accumulates positions 2 lane, 2 lane + 1 of the
    // stored order -- two adjacent channels -- over the slots; the rows go in two batches of four,
    // each batch with up to 4 x 16 reads in flight, the first one requested before the weights
    // are worked out.
    {
        constexpr int kMaxSlots = 80;   // 64 splits + the draft segment, rounded up to a multiple of 16
        float *ww = (float *)(lds_raw + 2048) + (size_t)wave * (RPW * kMaxSlots);   // [8 rows][kMaxSlots]
        const int u8 = lane >> 3, x8 = lane & 7;
        const int jrow = m0 + wave * RPW + u8;
        const int64_t pbase = (int64_t)(b * s.Hq + h) * part.nsplit * s.M;
        const int64_t slot_rows = (int64_t)slot_step * s.M;     // rows between consecutive slots
        const int jmax = s.M - 1;
        const int chan = partial_chan(2 * lane, 128);
        auto ml_of = [&](int sl) -> float2 {
            float2 ml = make_float2(-INFINITY, 0.f);
            if (sl < nslots && jrow < s.M) ml = *(const float2 *)(part.ml + (pbase + sl * slot_rows + jrow) * 2);
            return ml;
        };
        // rows u0 .. u0 + 3, slots sl0 .. sl0 + 15 (those below nslots): two adjacent values per lane
        auto fetch = [&](int u0, int sl0, float2 (&x)[4][16]) {
#pragma unroll
            for (int xi = 0; xi < 16; ++xi) {
                if (sl0 + xi < nslots) {   // uniform
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) {
                        const int j = min(m0 + wave * RPW + u0 + uu, jmax);   // rows past M repeat row M-1; never stored
                        x[uu][xi] = *(const float2 *)(part.o + (pbase + (sl0 + xi) * slot_rows + j) * 128 + 2 * lane);
                    }
                } else {
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) x[uu][xi] = make_float2(0.f, 0.f);
                }
            }
        };
        auto accumulate = [&](int u0, int sl0, const float2 (&x)[4][16], float2 (&acc)[4]) {
#pragma unroll
            for (int uu = 0; uu < 4; ++uu) {
                const float *wrow = ww + (u0 + uu) * kMaxSlots + sl0;
#pragma unroll
                for (int x4 = 0; x4 < 4; ++x4) {
                    const float4 w4 = *(const float4 *)(wrow + 4 * x4);
                    const float wv[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                    for (int xi = 0; xi < 4; ++xi) {
                        acc[uu].x = fmaf(wv[xi], x[uu][4 * x4 + xi].x, acc[uu].x);
                        acc[uu].y = fmaf(wv[xi], x[uu][4 * x4 + xi].y, acc[uu].y);
                    }
                }
            }
        };
        const float2 ml0 = ml_of(x8), ml1 = ml_of(x8 + 8);
        float2 xa[4][16];
        fetch(0, 0, xa);
        // weights of the slots and the denominator of each row
        float m_all = fmaxf(ml0.y > 0.f ? ml0.x : -INFINITY, ml1.y > 0.f ? ml1.x : -INFINITY);
        for (int sl = x8 + 16; sl < nslots; sl += 8) {   // more than 16 slots: rare
            const float2 ml = ml_of(sl);
            m_all = fmaxf(m_all, ml.y > 0.f ? ml.x : -INFINITY);
        }
        m_all = oct_max(m_all);
        const float m_use = m_all == -INFINITY ? 0.f : m_all;
        float den = 0.f;
        {
            const float w0 = ml0.y > 0.f ? __builtin_amdgcn_exp2f(ml0.x - m_use) : 0.f;   // 0 for a slot without a valid token
            const float w1 = ml1.y > 0.f ? __builtin_amdgcn_exp2f(ml1.x - m_use) : 0.f;
            den = fmaf(ml0.y, w0, fmaf(ml1.y, w1, 0.f));
            ww[u8 * kMaxSlots + x8] = w0;
            ww[u8 * kMaxSlots + x8 + 8] = w1;
        }
        const int nslots16 = (nslots + 15) & ~15;
        for (int sl = x8 + 16; sl < nslots16; sl += 8) {
            const float2 ml = ml_of(sl);                  // (-inf, 0) past the last slot
            const float w = ml.y > 0.f ? __builtin_amdgcn_exp2f(ml.x - m_use) : 0.f;
            den = fmaf(ml.y, w, den);
            ww[u8 * kMaxSlots + sl] = w;
        }
        den = oct_sum(den);
        const float inv = 1.f / den;   // den > 0: a node attends itself
#pragma unroll 1
        for (int u0 = 0; u0 < RPW; u0 += 4) {
            float2 acc[4];
#pragma unroll
            for (int uu = 0; uu < 4; ++uu) acc[uu] = make_float2(0.f, 0.f);
            if (u0 > 0) fetch(u0, 0, xa);
            accumulate(u0, 0, xa, acc);
#pragma unroll 1
            for (int sl0 = 16; sl0 < nslots; sl0 += 16) {
                fetch(u0, sl0, xa);
                accumulate(u0, sl0, xa, acc);
            }
#pragma unroll
            for (int uu = 0; uu < 4; ++uu) {
                const int j = m0 + wave * RPW + u0 + uu;
                const float iv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(inv), (u0 + uu) * 8));
                const uint32_t packed = (uint32_t)float_to_bf16_bits(acc[uu].x * iv) | ((uint32_t)float_to_bf16_bits(acc[uu].y * iv) << 16);
                if (j < s.M)
                    __builtin_nontemporal_store(packed, (uint32_t *)((uint16_t *)f.out + (((int64_t)b * s.M + j) * s.Hq + h) * 128 + chan));
            }
        }
        if (f.lse && x8 == 0 && jrow < s.M)
            f.lse[((int64_t)b * s.M + jrow) * s.Hq + h] = (m_all + __builtin_amdgcn_logf(den)) * kLn2;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    SPECPV_STAMP(11);  // merged and stored (last workgroup of a tile only)
    return false;
}

template <bool ALIGNED, bool FUSED, bool PEND>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_ctx_mfma_kernel(const int32_t *a_sel_idx, const int32_t *a_sel_count, const int32_t *a_ctx_len,
                          const void *a_q, int a_n_sel, int a_M, int a_Hq, int a_nctx,
                          Shape s, Partials part, MfmaArgs a, FusedArgs f)
{
    // the leading scalar arguments repeat what the first round of reads needs: they arrive in registers
    s.ctx_len = a_ctx_len; s.q = a_q; s.M = a_M; s.Hq = a_Hq;
    a.sel_idx = a_sel_idx; a.sel_count = a_sel_count; a.n_sel = a_n_sel;
    extern __shared__ char lds_raw[];
    const int sp0 = (int)blockIdx.y - (int)a.div_nsplit.div(blockIdx.y) * a_nctx;
    if (attn_ctx_pass<ALIGNED, FUSED, false, PEND>(s, part, a, f, a_nctx, sp0, a_nctx, lds_raw)) {
        if (FUSED) attn_ctx_pass<ALIGNED, true, true, PEND>(s, part, a, f, a_nctx, 0, 1, lds_raw);
    }
}

// ---- group variant: the query heads of a KV head in one workgroup --------------------------
// For long token ranges.  The G x ceil(M / 32) blocks of 32 query rows that share a KV head are
// dealt to workgroups of up to 10 wavefronts, one row block per wavefront (G = 4, M <= 64: one
// workgroup of 8; G = 5: one workgroup of 10; more row blocks: two or more workgroups).  A workgroup
// owns (sequence, KV head, its row blocks, KV split) and walks the split's chunks once for all of
// them: its W wavefronts share ONE ring of eight stages and each brings its share of a chunk's 16 DMA
// operations, so every K / V byte is requested from memory exactly once per workgroup, whatever
// the caches do.
// The ring has two halves of four chunks.  One workgroup barrier per FOUR chunks: at the barrier in
// front of chunks i .. i + 3 all of them have landed (requested one period earlier), every wavefront
// is done with the other half, and chunks i + 4 .. i + 7 are requested into it at once.  (A barrier
// per chunk, with the requests three chunks ahead in a ring of four, cost 430 of 2300 core cycles
// per chunk: it puts the wavefronts of a SIMD back in step every chunk, so that they queue for
// the LDS, the matrix cores and the vector ALU together instead of filling each other's gaps.)
// A wavefront keeps its rows to itself over the whole split, so the epilogue has nothing to
// merge: it only turns the accumulators into row-major partials.
// The chunk loop is unrolled over the eight ring stages: with the stage a compile-time constant,
// stage offsets are immediate fields of the LDS reads and of the requests' LDS addresses, the
// validity words of the stages are scalar registers, and the request of a chunk tests the common
// case (32 valid consecutive rows) first.  What a wavefront executes per chunk besides its
// arithmetic is what this loop pays for: measured in core cycles per chunk and workgroup (128K
// context, 32 splits), 2590 with a run-time stage and a barrier per chunk, 2295 unrolled, 2085
// with the four-chunk period; 1400 for the requests and barriers alone (timing probe), 1024 for
// the matrix instructions.  (The ten-wavefront variant keeps a barrier per chunk, see below.)
constexpr int kGroupStages = 8;   // two halves of kGroupPeriod chunks
constexpr int kGroupPeriod = 4;   // chunks between two workgroup barriers
static_assert(kStageBytes % 256 == 0, "K operand addresses are derived by XOR with multiples of 32 below 256: stages (and the rings) must start 256-byte aligned");

// W wavefronts per workgroup: 2, 4, 6, 8 or 10.  Ten (nine or ten row blocks: G = 5 with up to 64 nodes) means
// three wavefronts on two of the SIMDs, i.e. at most 168 registers each: that variant takes its K and V
// operands in halves.
template <bool ALIGNED, int W>
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(W > 8 ? 3 : 2, W > 8 ? 3 : 2)))
void attn_ctx_mfma_group_kernel(Shape s, Partials part, MfmaArgs a)
{
    SPECPV_CLOCKS_BEGIN;
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
    // chunks of cache tokens, then those of the partially verified tokens (see attn_ctx_mfma_kernel)
    const uint32_t C_ctx = (T + 31u) >> 5;
    const uint32_t C = C_ctx + (((uint32_t)s.kctx + 31u) >> 5);
    const char *kdb = (const char *)s.kd + (((int64_t)b * s.Mk) * s.Hkv + g) * 256;
    const char *vdb = (const char *)s.vd + (((int64_t)b * s.Mk) * s.Hkv + g) * 256;
    const uint32_t stp = (uint32_t)s.Hkv * 256u;
    const int c0 = first_chunk(C, sp), c1 = first_chunk(C, sp + 1);
    const int nch = c1 - c0;                  // the same for all wavefronts: the barriers match up

    const char *kb = (const char *)s.k + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const char *vb = (const char *)s.v + ((int64_t)b * s.sb + (int64_t)g * s.sh) * 2;
    const uint32_t st2 = (uint32_t)s.st * 2u;

    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)ring;
    uint32_t kread[4];   // + stage * kStageBytes; k-step ks + 4: the address XOR 128
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        kread[ks] = ring_addr + (uint32_t)n * 256u + (((uint32_t)(32 * ks + 16 * kg)) ^ (16u * ((uint32_t)n & 15u)));
    const uint32_t vread = ring_addr + 8192u + (uint32_t)(4 * kg + ((lane & 15) >> 2)) * kVPiecePitch +
                           32u * (uint32_t)((lane >> 4) & 1) + 8u * (uint32_t)(lane & 3);   // + stage * kStageBytes

    // ---- chunk -> token rows ------------------------------------------------------------
    // ALIGNED (B % 32 == 0): a chunk lies inside one block, so its 32 rows are consecutive.  The
    // first rows of the next 64 chunks sit in a register (lane t: chunk row_base + t) and are
    // picked with readlane.  Encoding: r >= 0: all 32 rows r .. r+31 are valid tokens (the common
    // case, handled without any further test); -1: no valid token; -2 - r: rows from r on, cut
    // off by the context length; kPendingChunk: a chunk of partially verified tokens.
    constexpr int kPendingChunk = (int)0x80000000;
    int row_base = 0, row0vec = -1;
    auto fill_rows = [&](int cb) {
        row_base = cb;
        int r = -1;
        if (cb + lane < nch && (uint32_t)(c0 + cb + lane) >= C_ctx) r = kPendingChunk;
        if (cb + lane < nch && (uint32_t)(c0 + cb + lane) < C_ctx) {
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
    const char *src_base[NOPS];   // per operation: K or V slab (wave-uniform: scalar registers)
    uint32_t src_off[NOPS];       // ... this lane's bytes from the chunk's first row (one register each)
    int dst_off[NOPS];            // ... and where it lands in the stage
    {
        const int r4 = lane >> 4, pos = lane & 15;
        const uint32_t sw0 = 16u * (uint32_t)(pos ^ r4), vsw = 16u * (uint32_t)pos;
#pragma unroll
        for (int t = 0; t < NOPS; ++t) {
            const int o = min(wave + W * t, 15), i = o & 7;
            if (o < 8) {
                src_base[t] = kb;
                src_off[t] = (uint32_t)(4 * i + r4) * st2 + (sw0 ^ (64u * (uint32_t)(i & 3)));
                dst_off[t] = i * 1024;
            } else {
                src_base[t] = vb;
                src_off[t] = (uint32_t)(8 * r4 + i) * st2 + vsw;
                dst_off[t] = 8192 + i * kVPiecePitch;
            }
        }
    }
    auto issue_rows = [&](const char *kbase, const char *vbase, const uint32_t stride, const uint32_t tk, char *dst) {
        // (the swizzles are recomputed here, from a lane id the compiler cannot see through: kept in registers
        // across the loop for this rare path they cost the ten-wavefront variant its last free registers)
        int lane_o = lane;
        asm volatile("" : "+v"(lane_o));
        const int r4 = lane_o >> 4, pos = lane_o & 15;
        const uint32_t sw0 = 16u * (uint32_t)(pos ^ r4), vsw = 16u * (uint32_t)pos;
#pragma unroll
        for (int t = 0; t < NOPS; ++t) {
            if (16 % W != 0 && t == NOPS - 1 && n_ops != NOPS) continue;
            const int o = wave + W * t, i = o & 7;
            if (o < 8) {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 4 * i + r4) * stride;
                dma16(kbase + (tv + (sw0 ^ (64u * (uint32_t)(i & 3)))), dst + dst_off[t]);
            } else {
                const uint32_t tv = (uint32_t)__shfl((int)tk, 8 * r4 + i) * stride;
                dma16(vbase + (tv + vsw), dst + dst_off[t]);
            }
        }
    };
    // Stage stg of the ring is a compile-time constant in the loop below (unrolled over the stages).
    auto issue = [&](int ci, int stg) __attribute__((always_inline)) -> uint32_t {
        char *dst = ring + stg * kStageBytes;
        int tok;
        if (ALIGNED) {
            if (ci - row_base >= 64) fill_rows(ci);
            const int r0 = __builtin_amdgcn_readlane(row0vec, ci - row_base);
            if (r0 >= 0) {
                const uint32_t row_off = (uint32_t)r0 * st2;   // fits 32 bits (host-checked)
#pragma unroll
                for (int t = 0; t < NOPS; ++t)
                    if (16 % W == 0 || t < NOPS - 1 || n_ops == NOPS) {
                        uint32_t so = src_off[t];
                        // (ten wavefronts: keep the 32-bit offset as it is; the compiler would otherwise carry the 64-bit sum
                        // base + offset of every operation through the loop, in registers that this variant does not have)
                        if (W > 8) asm volatile("" : "+v"(so));
                        __builtin_amdgcn_global_load_lds((glb_void_ptr)((src_base[t] + row_off) + so), (lds_void_ptr)(dst + dst_off[t]), 16, 0, kKvAux);
                    }
                return 0xffffffffu;
            }
            if (r0 == kPendingChunk) {
                const int pr = (int)((uint32_t)(c0 + ci) - C_ctx) * 32 + n;
                const int ptok = pr < s.kctx ? pr : -1;
                issue_rows(kdb, vdb, stp, (uint32_t)max(ptok, 0), dst);
                return (uint32_t)__ballot(ptok >= 0);
            }
            const int rr = -2 - r0;   // r0 == -1 gives -1
            tok = (rr >= 0 && rr + n < L) ? rr + n : -1;
        } else {
            if (s.kctx > 0 && (uint32_t)(c0 + ci) >= C_ctx) {
                const int pr = (int)((uint32_t)(c0 + ci) - C_ctx) * 32 + n;
                const int ptok = pr < s.kctx ? pr : -1;
                issue_rows(kdb, vdb, stp, (uint32_t)max(ptok, 0), dst);
                return (uint32_t)__ballot(ptok >= 0);
            }
            tok = lane_row(ci);
        }
        const uint32_t vm = (uint32_t)__ballot(tok >= 0);
        const uint32_t tk = tok >= 0 ? (uint32_t)tok : 0u;   // row 0 exists (L > 0); masked later
        issue_rows(kb, vb, st2, tk, dst);
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

    // validity bits of the chunks in the ring, one word per stage (the same in every lane)
    uint32_t vm_stage[kGroupStages] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    static_assert(kGroupStages == 8 && kGroupPeriod == 4, "the first requests and the loops below are written for two halves of four stages");
    if (W <= 8) {
        if (0 < nch) vm_stage[0] = issue(0, 0);
        if (1 < nch) vm_stage[1] = issue(1, 1);
        if (2 < nch) vm_stage[2] = issue(2, 2);
        if (3 < nch) vm_stage[3] = issue(3, 3);
    }
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
    // ten wavefronts: operands in halves (16 registers at a time instead of 32)
    auto pv_halves = [&](const uint32_t vaddr, auto off) __attribute__((always_inline)) {
        constexpr int OFF = decltype(off)::value;
        uint2 vh[8];
        lds_read_v_half<OFF>(vaddr, vh);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            O[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(make_uint4(vh[2 * j].x, vh[2 * j].y, vh[2 * j + 1].x, vh[2 * j + 1].y)),
                                                           as_bf16x8(pf0), O[j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        lds_read_v_half<OFF + 512>(vaddr, vh);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            O[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(make_uint4(vh[2 * j].x, vh[2 * j].y, vh[2 * j + 1].x, vh[2 * j + 1].y)),
                                                           as_bf16x8(pf1), O[j], 0, 0, 0);
    };
    // One chunk; its ring stage U = i % 4 is a compile-time constant (the loop below is unrolled over the
    // stages), so that stage offsets are immediate fields of the LDS reads and of the requests' LDS
    // addresses, and the validity words live in scalar registers.
    // Stage U compile-time (the unrolled loop): the stage inside its ring half is an immediate field of the LDS
    // reads (16 bits), the half is reached through the address register.  The ten-wavefront loop passes stage 0
    // and the whole offset at run time (roff).
    auto chunk = [&](const int i, auto stage, const uint32_t roff, const uint32_t vmask) __attribute__((always_inline)) {
        constexpr int U = decltype(stage)::value;
        constexpr int SOFF = (U % kGroupPeriod) * kStageBytes;
        const uint32_t HOFF = (uint32_t)(U / kGroupPeriod) * kGroupPeriod * kStageBytes + roff;
        if (!live) return;
        f32x16 S;
        if (W > 8) {
            // ten wavefronts: operands in halves, the V operands read behind the softmax (pv_halves)
            // (k-step ks reads 32 ks bytes further, modulo the swizzle: an XOR, as the row starts are 128-byte aligned)
            const uint32_t ka0 = kread[0] + HOFF;
            const uint32_t ka[4] = {ka0, ka0 ^ 32u, ka0 ^ 64u, ka0 ^ 96u};
            uint4 kh[4];
            lds_read_k_half<SOFF>(ka, kh);
#pragma unroll
            for (int x = 0; x < 16; ++x) S[x] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kh[ks]), qf[ks], S, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t kb4[4] = {ka0 ^ 128u, ka0 ^ 160u, ka0 ^ 192u, ka0 ^ 224u};
            lds_read_k_half<SOFF>(kb4, kh);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kh[ks]), qf[4 + ks], S, 0, 0, 0);
        } else {
            uint4 kf[8];
            {
                const uint32_t k0 = kread[0] + HOFF, k1 = kread[1] + HOFF, k2 = kread[2] + HOFF, k3 = kread[3] + HOFF;
                const uint32_t ka[8] = {k0, k1, k2, k3, k0 ^ 128u, k1 ^ 128u, k2 ^ 128u, k3 ^ 128u};
                lds_read_k<SOFF>(ka, kf);
            }
            lds_read_v<SOFF>(vread + HOFF, v);
#pragma unroll
            for (int x = 0; x < 16; ++x) S[x] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[ks]), qf[ks], S, 0, 0, 0);
        }

        if (vmask != 0xffffffffu) {
            // (rare: the lane's share of the bits is worked out here, from a value the compiler cannot see through,
            // so that nothing of it is kept in registers across the loop)
            int kg_o = kg;
            asm volatile("" : "+v"(kg_o));
            const uint32_t mine = vmask >> (kg_o * 4);
#pragma unroll
            for (int x = 0; x < 16; ++x)
                if (!((mine >> ((x >> 2) * 8 + (x & 3))) & 1u)) S[x] = -INFINITY;
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
        if (W > 8) pv_halves(vread + HOFF, std::integral_constant<int, SOFF>{});
        else pv();
    };
    // Four chunks between two barriers.  At the barrier in front of chunks i0 .. i0 + 3 (ring half H) every
    // wavefront's requests have landed -- they were made a whole period ago, so the wait is for all of
    // them -- and every wavefront is done with the other half, into which the next four chunks are
    // requested at once; then come four chunks of arithmetic without a request or a wait in between.
    auto period = [&](const int i0, auto half) __attribute__((always_inline)) {
        constexpr int H = decltype(half)::value, S0 = kGroupPeriod * H, N0 = kGroupPeriod * (1 - H);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        if (i0 + 4 < nch) vm_stage[N0] = issue(i0 + 4, N0);
        if (i0 + 5 < nch) vm_stage[N0 + 1] = issue(i0 + 5, N0 + 1);
        if (i0 + 6 < nch) vm_stage[N0 + 2] = issue(i0 + 6, N0 + 2);
        if (i0 + 7 < nch) vm_stage[N0 + 3] = issue(i0 + 7, N0 + 3);
        chunk(i0, std::integral_constant<int, S0>{}, 0u, vm_stage[S0]);
        if (i0 + 1 < nch) chunk(i0 + 1, std::integral_constant<int, S0 + 1>{}, 0u, vm_stage[S0 + 1]);
        if (i0 + 2 < nch) chunk(i0 + 2, std::integral_constant<int, S0 + 2>{}, 0u, vm_stage[S0 + 2]);
        if (i0 + 3 < nch) chunk(i0 + 3, std::integral_constant<int, S0 + 3>{}, 0u, vm_stage[S0 + 3]);
    };
    if (W <= 8) {
        for (int i0 = 0; i0 < nch; i0 += kGroupStages) {
            period(i0, std::integral_constant<int, 0>{});
            if (i0 + kGroupPeriod < nch) period(i0 + kGroupPeriod, std::integral_constant<int, 1>{});
        }
    } else {
        // Ten wavefronts (three on two of the SIMDs, 168 registers): a barrier per chunk, requests three chunks
        // ahead, the stage a run-time value -- measured against the period loop above on the ragged batch of four
        // at G = 5: partial step (16 chunks per workgroup) 32.1 against 37.1 us, full pass 532 against 525 us.
        constexpr int kAhead = 3;
        uint32_t vmv = 0u;   // validity words of the chunks in the ring: lane t holds those of stage t
        for (int c = 0; c < kAhead && c < nch; ++c) {
            const uint32_t vm = issue(c, c);
            vmv = lane == c ? vm : vmv;
        }
        for (int i = 0; i < nch; ++i) {
            // own part of chunk i has landed: kAhead - 1 younger groups of n_ops operations may stay in flight
            // (towards the end of the range there are fewer: wait for all, they are due anyway)
            if (i + kAhead - 1 >= nch) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            else if (n_ops == NOPS) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NOPS * (kAhead - 1)) : "memory");
            else asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NOPS - 1) * (kAhead - 1)) : "memory");
            __builtin_amdgcn_s_barrier();   // ... and so have the others'; chunk i-1 has been read by all
            if (i + kAhead < nch) {
                const int is = (i + kAhead) & (kGroupStages - 1);
                const uint32_t vm = issue(i + kAhead, is);
                vmv = lane == is ? vm : vmv;
            }
            const int rs = i & (kGroupStages - 1);
            chunk(i, std::integral_constant<int, 0>{}, (uint32_t)rs * kStageBytes, (uint32_t)__builtin_amdgcn_readlane((int)vmv, rs));
        }
    }
    __syncthreads();   // every wavefront is done with the ring: the epilogue reuses that LDS

    // ---- one partial per (head, split, node): accumulators -> row-major through LDS ------
    // (ten wavefronts: the staging area holds five at a time, so the second five wait for the first;
    // every wavefront, live or not, passes that one barrier)
    constexpr int kSlots = W > 8 ? W / 2 : W;
    const int slot = wave < kSlots ? wave : wave - kSlots;
    if (W > 8) {
        if (wave >= kSlots) __builtin_amdgcn_s_barrier();
        if (!live) {
            if (wave < kSlots) __builtin_amdgcn_s_barrier();
            return;
        }
    } else if (!live) {
        return;
    }
    l_run = sum_xor32(l_run);
    const int64_t prow0 = ((int64_t)(b * s.Hq + h) * part.nsplit + sp) * s.M;
    {
        // accumulator element 4q + x of tile j is channel 32j + 8q + 4kg + x of this lane's row
        float *dst = obuf + ((size_t)slot * 32 + n) * kOPitch;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(float4 *)(dst + 32 * j + 8 * q + 4 * kg) = make_float4(O[j][4 * q], O[j][4 * q + 1], O[j][4 * q + 2], O[j][4 * q + 3]);
    }
    // a wavefront reads back only what it wrote itself: no barrier.  fp16 partials: channels 2 lane, 2 lane + 1
    // of the row's normalised result (lane uu < 32 holds row uu's l)
    const int jrow0 = m0;
    const float il = l_run > 0.f ? 1.f / l_run : 0.f;
#pragma unroll 8
    for (int uu = 0; uu < 32; ++uu) {
        const float2 x = *(const float2 *)(obuf + ((size_t)slot * 32 + uu) * kOPitch + 2 * lane);
        const float ilu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(il), uu));
        if (jrow0 + uu < s.M) store_partial_half(part.o + (prow0 + jrow0 + uu) * 64, lane, x.x * ilu, x.y * ilu);
    }
    if (kg == 0 && jrow0 + n < s.M) *(float2 *)(part.ml + (prow0 + jrow0 + n) * 2) = make_float2(m_ref, l_run);
    SPECPV_CLOCKS_END(part.timeline, (size_t)blockIdx.y * gridDim.x + blockIdx.x, nch);
    if (W > 8) {
        if (wave < kSlots) __builtin_amdgcn_s_barrier();   // the slot is free for wavefront wave + kSlots
    }
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
    if (g.n_row_blocks == 9 || g.n_row_blocks == 10) {   // one workgroup of ten instead of two of five
        g.parts = 1;
        g.waves = 10;
        return g;
    }
    g.parts = (g.n_row_blocks + 7) / 8;
    const int w = (g.n_row_blocks + g.parts - 1) / g.parts;   // 1 .. 8
    g.waves = w <= 2 ? 2 : (w <= 4 ? 4 : (w <= 6 ? 6 : 8));
    return g;
}
int attn_group_parts(const Shape &s) { return group_layout(s).parts; }

hipError_t launch_attn_ctx_mfma(const Shape &s, const int32_t *sel_idx, const int32_t *sel_count,
                                int n_sel, Partials p, int nctx, int kind, const FusedArgs &f, hipStream_t st)
{
    if (kind != kAttnSplit && kind != kAttnGroup) return hipErrorInvalidValue;
    const bool fused = f.out != nullptr;
    if (fused && (kind != kAttnSplit || nctx > 64 || p.nsplit != nctx + 1)) return hipErrorInvalidValue;
    if (!fused && p.nsplit != nctx) return hipErrorInvalidValue;
    const GroupLayout gl = group_layout(s);
    MfmaArgs a;
    a.sel_idx = sel_idx;
    a.sel_count = sel_count;
    a.n_sel = n_sel;
    a.scale_log2 = kLog2e / sqrtf(128.f);
    a.row_tiles = (s.M + 63) / 64;
    a.rph = gl.rph;
    a.n_row_blocks = gl.n_row_blocks;
    a.n_units = s.batch * s.Hkv * nctx;
    a.n_bg = s.batch * s.Hkv;
    a.div_nsplit = make_fastdiv((uint32_t)nctx);
    a.div_hkv = make_fastdiv((uint32_t)s.Hkv);
    a.div_B = make_fastdiv((uint32_t)s.B);
    // token ranges per split: four (one per token group of a workgroup), or one in the group kernel
    a.div_W = make_fastdiv((uint32_t)nctx * (kind == kAttnGroup ? 1u : 4u));
    const int GR = kind == kAttnGroup ? gl.parts : s.G * a.row_tiles;
    // group kernel: a unit (sequence, KV head, split) per 8 consecutive x; split kernel: (sequence, KV
    // head) bg on XCD bg % 8 with all its splits and query heads (y = (bg / 8) * nctx + split)
    const dim3 grid(8 * GR, kind == kAttnGroup ? (a.n_units + 7) / 8 : ((a.n_bg + 7) / 8) * nctx);
    if (grid.y > 65535u) return hipErrorInvalidConfiguration;
    const bool aligned = s.B % 32 == 0;
    const size_t lds_split = 2048 + (size_t)max(kRingBytes, 4 * 64 * kOPitch * (int)sizeof(float)) + kQStageBytes;
    const size_t lds_group = (size_t)max(kGroupStages * kStageBytes, (gl.waves > 8 ? gl.waves / 2 : gl.waves) * 32 * kOPitch * (int)sizeof(float));
#define SPECPV_SET_LDS(KERN, LDS)                                                                      \
        static PerDeviceOnce once;   /* one per kernel instantiation */                               \
        auto kern = KERN;                                                                              \
        const hipError_t e0 = once.run([&] {                                                           \
            return hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(LDS)); \
        });                                                                                            \
        if (e0 != hipSuccess) return e0
#define SPECPV_LAUNCH_GROUP(WW)                                                                        \
    do {                                                                                               \
        if (aligned) { SPECPV_SET_LDS((attn_ctx_mfma_group_kernel<true, WW>), lds_group);               \
                       hipLaunchKernelGGL(kern, grid, dim3(64 * WW), lds_group, st, s, p, a); }         \
        else { SPECPV_SET_LDS((attn_ctx_mfma_group_kernel<false, WW>), lds_group);                      \
               hipLaunchKernelGGL(kern, grid, dim3(64 * WW), lds_group, st, s, p, a); }                 \
    } while (0)
#define SPECPV_LAUNCH_SPLIT(AL, FU, PE)                                                                \
    do {                                                                                               \
        SPECPV_SET_LDS((attn_ctx_mfma_kernel<AL, FU, PE>), lds_split);                                  \
        hipLaunchKernelGGL(kern, grid, dim3(512), lds_split, st, sel_idx, sel_count, s.ctx_len, s.q,    \
                           n_sel, s.M, s.Hq, nctx, s, p, a, f);                                         \
    } while (0)
    if (kind == kAttnGroup) {
        switch (gl.waves) {
        case 2: SPECPV_LAUNCH_GROUP(2); break;
        case 4: SPECPV_LAUNCH_GROUP(4); break;
        case 6: SPECPV_LAUNCH_GROUP(6); break;
        case 10: SPECPV_LAUNCH_GROUP(10); break;
        default: SPECPV_LAUNCH_GROUP(8); break;
        }
    } else if (fused) {
        if (aligned) SPECPV_LAUNCH_SPLIT(true, true, true); else SPECPV_LAUNCH_SPLIT(false, true, true);
    } else {
        if (s.kctx > 0) { if (aligned) SPECPV_LAUNCH_SPLIT(true, false, true); else SPECPV_LAUNCH_SPLIT(false, false, true); }
        else { if (aligned) SPECPV_LAUNCH_SPLIT(true, false, false); else SPECPV_LAUNCH_SPLIT(false, false, false); }
    }
#undef SPECPV_LAUNCH_SPLIT
#undef SPECPV_LAUNCH_GROUP
#undef SPECPV_SET_LDS
    return hipGetLastError();
}

}  // namespace specpv
