// Internal declarations shared by the HIP translation units of libspecpv.
// Each .hip file owns its kernels and exposes one host launcher; api.hip
// validates arguments and calls the launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "specpv.h"

namespace specpv {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Flat view of one call's tensors, passed by value to the kernels.
struct Shape {
    const void *k, *v;            // context KV, read in place
    int64_t sb, sh, st;           // element strides of k / v: batch, head, token
    const int32_t *ctx_len;       // [batch]
    const void *q;                // [batch, M, Hq, D]
    const void *kd, *vd;          // [batch, Mk, Hkv, D]
    const int32_t *parent;        // [batch, Mk]
    int batch, Hkv, Hq, G, D, B, M, max_blocks;
    // M counts the QUERY nodes (rows of q, out, the partials).  The tree has Mk >= M nodes: its
    // first koff = Mk - M nodes are keys only (partially verified tokens on a partial step);
    // query row r is node koff + r.
    int Mk, koff;
    // Of those, the first kctx (0 or koff) are attended by the context kernels as if they were cache
    // tokens -- they are a chain from which every query node descends, so every row sees all of them --
    // and the draft-tree segment (combine kernel, single-kernel route) stops its root paths there.
    int kctx;
};

// Split-KV partial results of the context part, one per (b, h, split, node):
//   part_ml [batch, Hq, nsplit, M, 2] fp32   (m, l): m = max_t z_t, l = sum_t 2^(z_t - m),
// with z = q.k * log2(e)/sqrt(D).  A split without any valid token stores m = -inf, l = 0.
//   part_o, one of two forms:
//   o_half == 0:  [batch, Hq, nsplit, M, D] fp32   sum_t 2^(z_t - m) v_t   (not normalised).  Inside a row
//     with D = 128 the channels are stored in the order the combine kernel reads them (a lane of 16 owns
//     channels 8 i .. 8 i + 7 and fetches them as two 16-byte pieces, each piece dense over the 16 lanes):
//     channel c sits at partial_pos(c).  D = 64: in order.  (vector-ALU kernel: fp32 inputs and their 1e-5
//     bar; single-kernel route.)
//   o_half == 1:  [batch, Hq, nsplit, M, D] fp16   the split's own softmax result, sum_t 2^(z_t - m) v_t / l
//     (0 if l = 0), channels in order.  A convex combination of V rows, so within fp16's range as long as
//     |v| <= 65504 (larger magnitudes are clamped); its 11 significant bits are 8 times finer than the
//     bf16 output.  Half the bytes of the fp32 form: the partials are the call's second-largest traffic.
struct Partials {
    float *o;
    float *ml;
    int nsplit;
    int o_half;
    unsigned long long *timeline;   // instrumented builds (-DSPECPV_TIMELINE): the combine kernel's time stamps go to rows 2048.. of this buffer
};
__host__ __device__ constexpr int partial_pos(int c, int D)
{
    return D == 128 ? ((c >> 2) & 1) * 64 + (c >> 3) * 4 + (c & 3) : c;
}
// ... and the channel that sits at position p (the inverse)
__host__ __device__ constexpr int partial_chan(int p, int D)
{
    return D == 128 ? ((p & 63) >> 2) * 8 + (p >> 6) * 4 + (p & 3) : p;
}
constexpr bool partial_order_is_a_permutation()
{
    for (int D = 64; D <= 128; D += 64)
        for (int p = 0; p < D; ++p) {
            const int c = partial_chan(p, D);
            if (c < 0 || c >= D || partial_pos(c, D) != p) return false;
            // a lane's 16-byte piece holds four consecutive channels, in order
            if ((p & 3) != 0 && c != partial_chan(p - 1, D) + 1) return false;
        }
    return true;
}
static_assert(partial_order_is_a_permutation(), "partial_pos / partial_chan must be inverse permutations of a row");

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerVec = 4;  // elements per 16-byte vector
    static __device__ __forceinline__ void unpack(const uint4 &u, float *f) {
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
    static __device__ __forceinline__ uint4 pack(const float *f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
    static __device__ __forceinline__ float load(const void *p, int64_t i) { return ((const float *)p)[i]; }
    static __device__ __forceinline__ void store(void *p, int64_t i, float x) { ((float *)p)[i] = x; }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, float x) { __builtin_nontemporal_store(x, (float *)p + i); }
};
struct bf16_t { uint16_t bits; };
__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
// round-to-nearest-even fp32 -> bf16 (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
template <> struct Elem<bf16_t> {
    static constexpr int kPerVec = 8;
    static __device__ __forceinline__ void unpack(const uint4 &u, float *f) {
        f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
        f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
        f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
        f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
    }
    static __device__ __forceinline__ uint4 pack(const float *f) {   // values that are exactly representable
        return make_uint4(float_to_bf16_bits(f[0]) | ((uint32_t)float_to_bf16_bits(f[1]) << 16),
                          float_to_bf16_bits(f[2]) | ((uint32_t)float_to_bf16_bits(f[3]) << 16),
                          float_to_bf16_bits(f[4]) | ((uint32_t)float_to_bf16_bits(f[5]) << 16),
                          float_to_bf16_bits(f[6]) | ((uint32_t)float_to_bf16_bits(f[7]) << 16));
    }
    static __device__ __forceinline__ float load(const void *p, int64_t i) {
        return bf16_bits_to_float(((const uint16_t *)p)[i]);
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, float x) {
        ((uint16_t *)p)[i] = float_to_bf16_bits(x);
    }
    static __device__ __forceinline__ void store_stream(void *p, int64_t i, float x) {
        __builtin_nontemporal_store(float_to_bf16_bits(x), (uint16_t *)p + i);
    }
};

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// ---- launchers (each returns the hipError_t of its launches) ----
hipError_t launch_summarize(const Shape &s, int dtype, int blk_begin, int blk_end,
                            void *kmax, void *kmin, hipStream_t st);
// One selection: kept-block lists of n_row entries (>= ns + k + nr; the rest is padding for later
// commits), ascending, -1 behind the count.
struct TopkArgs {
    int ns, nr, k, n_row;
    int32_t *sel_idx, *sel_count;
};
// kind: SPECPV_SCORE_EQ2 or SPECPV_SCORE_CHANNEL_BOUND.  sel != nullptr: the selection runs in the same
// launch; only where score_select_supported() holds, with arrive pointing to the kArriveBytes of zeroed
// arrival words at the head of a workspace (zero again when the launch has finished).
bool score_select_supported(const Shape &s, int dtype);
hipError_t launch_scores(const Shape &s, int dtype, const void *kmax, const void *kmin,
                         int reduce, int last_node, int kind, float *scores, const TopkArgs *sel,
                         unsigned long long *arrive, hipStream_t st);
// n_row: entries per list row (>= ns + k + nr; the rest is padding for later commits)
hipError_t launch_topk(const Shape &s, const float *scores, int ns, int nr, int k, int n_row,
                       int32_t *sel_idx, int32_t *sel_count, hipStream_t st);
hipError_t launch_attn_ctx_generic(const Shape &s, int dtype, const int32_t *sel_idx,
                                   const int32_t *sel_count, int n_sel, Partials p, hipStream_t st);
bool attn_ctx_mfma_supported(const Shape &s, int dtype);
// Which kernel computes the context part, and with how many KV splits.  kAttnSplit: eight
// wavefronts per (query head, split), for short token ranges; kAttnGroup: the query heads of a KV
// head in one workgroup (two or more for more than eight 32-row blocks), for long ranges;
// kAttnGeneric: any dtype / head dim.
enum AttnKind { kAttnGeneric = 0, kAttnSplit = 1, kAttnGroup = 3 };
struct AttnPlan {
    int nsplit;
    int kind;
};
// The whole call in the eight-wavefront kernel (kAttnSplit only): the draft-tree segment as one more
// partial (slot nctx of nctx + 1), arrival words, the last workgroup of a tile merges and stores.
// out == nullptr: the kernel only writes partials and launch_combine finishes.
struct FusedArgs {
    void *out;                     // [batch, M, Hq, 128] bf16
    float *lse;                    // optional [batch, M, Hq]
    unsigned long long *arrive;    // [batch, Hq, 2] arrival words, zero between calls
    int force_recompute;           // test hook: the last workgroup of a tile takes the recompute route
    unsigned long long *timeline;  // builds with -DSPECPV_TIMELINE: 16 time stamps per workgroup (else unused)
};
constexpr size_t kArriveBytes = 64 << 10;   // head of every workspace: 8192 arrival words
// p.nsplit: slots per (sequence, head) in the partial arrays = nctx, or nctx + 1 when fused
hipError_t launch_attn_ctx_mfma(const Shape &s, const int32_t *sel_idx, const int32_t *sel_count,
                                int n_sel, Partials p, int nctx, int kind, const FusedArgs &f, hipStream_t st);
// workgroups per (sequence, KV head, split) of the kAttnGroup kernel
int attn_group_parts(const Shape &s);
hipError_t launch_combine(const Shape &s, int dtype, Partials p, void *out, float *lse, hipStream_t st);
// to_cache != 0: pending + accepted rows go to the cache tail (lengths, summaries updated);
// otherwise the accepted rows join the pending rows of the buffer.  old_len: [batch] scratch.
// n_layers layers that share shape, strides and counters are committed together.
// lists (n_layers entries, or nullptr): kept-block lists that take in the blocks a commit to the
// cache touches.  dropped ([batch, 2], or nullptr): tokens not stored, list entries not found.
hipError_t launch_commit(const Shape &s, int dtype, int n_layers, void *const *k, void *const *v,
                         void *const *buf_k, void *const *buf_v, int P, int Mt,
                         int32_t *n_pending, const int32_t *accepted, const int32_t *n_accepted,
                         int max_accept, int to_cache, void *const *kmax, void *const *kmin,
                         const specpv_lists *lists, int32_t *dropped, int32_t *old_len,
                         hipStream_t st);

hipError_t launch_gather(const Shape &s, int dtype, const int32_t *sel_idx, const int32_t *sel_count, int n_sel,
                         void *out_k, void *out_v, int32_t *out_len, hipStream_t st);

int device_cu_count();   // of the current device

// One-time set-up per (kernel, device): `fn` runs once for each device it is asked for, also when
// several threads make their first call at the same moment.  Devices beyond 63 run it every time.
struct PerDeviceOnce {
    unsigned long long done = 0;   // bit d: fn has succeeded on device d (accessed atomically)
    template <typename F> hipError_t run(F fn)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool tracked = dev >= 0 && dev < 64;
        if (tracked && ((__atomic_load_n(&done, __ATOMIC_ACQUIRE) >> dev) & 1ull)) return hipSuccess;
        e = fn();   // idempotent: two threads that race here both set the same attribute
        if (e == hipSuccess && tracked) __atomic_fetch_or(&done, 1ull << dev, __ATOMIC_RELEASE);
        return e;
    }
};

}  // namespace specpv
