// Shared host/device helpers of libeoq (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/eoq.h"

struct eoq_ctx {
    hipStream_t stream;
    int device;
    uint32_t *d_status;   // device status word (eoq_flag_bits)
    int32_t *d_scratch;   // EOQ_SCRATCH_SLOTS int32 slots for call-internal statistics
    int64_t *d_partials;  // EOQ_PARTIAL_SLOTS int64 per-workgroup partial sums of the call in flight on this stream
    void *static_scratch; // this device's copy of the file-scope scratch array of eoq_conv_bwd_weight_static
};

// conv_wgrad.hip: device address of that array on `device` (looked up once per device; `device` must be current)
int wgrad_static_scratch_init(int device, void **ptr_out);

constexpr int EOQ_SCRATCH_SLOTS = 64;
// d_scratch slots with a fixed meaning (0, 1: abs-max of eoq_quantize / eoq_update_int8 when the caller gives none)
constexpr int EOQ_SLOT_SPEC_USED = 8;   // exponent the speculative launch in flight coded with
constexpr int EOQ_SLOT_POOL_TMP = 16;   // int64 (two slots): sum of the codes of a speculative pool-backward pass
constexpr int EOQ_SLOT_SPEC_HITS = 24;  // [0] speculative calls whose exponent was right, [1] those that were redone
constexpr int EOQ_PARTIAL_SLOTS = 1 << 20;      // 8 MB: per-wave pairs of the largest benchmark layer
constexpr int CODE_MAX = 127;

#define EOQ_HIP(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return EOQ_ERR_HIP;      \
    } while (0)

#define EOQ_LAUNCH_CHECK()                             \
    do {                                               \
        if (hipGetLastError() != hipSuccess) return EOQ_ERR_HIP; \
    } while (0)

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ---- direct-to-LDS loads ----
// 16 bytes per lane from a buffer straight into LDS (gfx950: buffer_load_dwordx4 ... lds): lane l of the wave writes
// LDS bytes [lds_base + 16 l, lds_base + 16 l + 16) with whatever ITS offset addresses in memory (an in-bounds probe
// confirmed the lane order, and that an out-of-range offset writes zeros).  lds_base is wave-uniform (it travels in
// M0).  Issued through inline assembly on purpose: the compiler, when it knows of such a load, waits for ALL
// outstanding memory operations before the next LDS read, which would drain the prefetch ring at every stage; here the
// waits are written by hand (wait_vmcnt) next to the barriers that publish a stage.
__device__ __forceinline__ void lds_direct_load16(const v4i &rsrc, uint32_t lds_base, int voffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(rsrc)
                 : "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N));
}

// ---- rounding: v * 2^-s to nearest, ties to even (s >= 1); exact left shift for s <= 0 ----
__device__ __forceinline__ int64_t rne_shift64(int64_t v, int s)
{
    if (s <= 0) return v << (-s);
    if (s > 62) s = 62;
    return (v + ((int64_t(1) << (s - 1)) - 1) + ((v >> s) & 1)) >> s;
}

__device__ __forceinline__ int32_t rne_shift7(int32_t v)   // |v| < 2^30
{
    return (v + 63 + ((v >> 7) & 1)) >> 7;
}

// 32-bit forms for |v| < 2^30; LEFT selects the exact left shift (s <= 0) at compile time so that the streaming kernels,
// whose shift is the same for every element, carry no per-element branch
template <bool LEFT>
__device__ __forceinline__ int rne_shift32(int v, int s)
{
    if (LEFT) return v << (-s);
    return (v + ((1 << (s - 1)) - 1) + ((v >> s) & 1)) >> s;
}

template <bool LEFT>
__device__ __forceinline__ int sq_code32(int v, int s)      // clamp(R(v * 2^-s), -127, 127)
{
    const int c = rne_shift32<LEFT>(v, s);
    return c < -CODE_MAX ? -CODE_MAX : (c > CODE_MAX ? CODE_MAX : c);
}

// four codes in [-127, 127] -> one dword of bytes
__device__ __forceinline__ uint32_t pack4_i8(int c0, int c1, int c2, int c3)
{
    // v_perm_b32: selector bytes 0-3 take bytes of the second operand, 4-7 of the first, 0x0c gives zero
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)c1, (uint32_t)c0, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)c3, (uint32_t)c2, 0x0c0c0400u);
    return lo | (hi << 16);
}

// 4 mask bits (bit k for byte k) -> 0xff in every byte whose bit is set
__device__ __forceinline__ uint32_t byte_mask4(uint32_t m4)
{
    return (((m4 & 0xfu) * 0x00204081u) & 0x01010101u) * 0xffu;
}

// sum of the four signed bytes of a dword, added to acc
__device__ __forceinline__ int sum4_i8(uint32_t packed, int acc)
{
    return __builtin_amdgcn_sdot4((int)packed, 0x01010101, acc, false);
}

__device__ __forceinline__ int clamp_i(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// ---- R(log2 M) for an integer M >= 1 (Eq.7's scale exponent): floor(log2 M), plus one iff
// M^2 > 2^(2p+1); equality is impossible for an integer, so the rounding never ties ----
__device__ __forceinline__ int sq_exponent_u32(uint32_t M)
{
    int p = 31 - __clz((int)M);
    uint64_t sq = (uint64_t)M * (uint64_t)M;
    return p + (sq > (uint64_t(1) << (2 * p + 1)) ? 1 : 0);
}

__device__ __forceinline__ int sq_exponent_u64(uint64_t M)   // M < 2^62
{
    int p = 63 - __clzll((long long)M);
    // compare M^2 with 2^(2p+1) without overflowing: M = 2^p * f, f in [1,2): f^2 > 2
    // use 128-bit product via two halves
    unsigned __int128 sq = (unsigned __int128)M * (unsigned __int128)M;
    unsigned __int128 lim = (unsigned __int128)1 << (2 * p + 1);
    return p + (sq > lim ? 1 : 0);
}

// SQ of one value given the tensor's scale exponent r: clamp(R(v * 2^(7-r)), -127, 127)
__device__ __forceinline__ int sq_code(int64_t v, int r)
{
    int64_t c = rne_shift64(v, r - 7);
    return (int)(c < -CODE_MAX ? -CODE_MAX : (c > CODE_MAX ? CODE_MAX : c));
}

// ---- wave / block reductions (wave = 64 lanes) ----
__device__ __forceinline__ int wave_max_i32(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        int t = __shfl_xor(v, o, 64);
        v = t > v ? t : v;
    }
    return v;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        uint32_t t = (uint32_t)__shfl_xor((int)v, o, 64);
        v = t > v ? t : v;
    }
    return v;
}

__device__ __forceinline__ int64_t wave_sum_i64(int64_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        int lo = __shfl_xor((int)(v & 0xffffffff), o, 64);
        int hi = __shfl_xor((int)(v >> 32), o, 64);
        v += (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
    }
    return v;
}

__device__ __forceinline__ void atomic_add_i64(int64_t *p, int64_t v)
{
    atomicAdd((unsigned long long *)p, (unsigned long long)v);
}

// ---- block-level combination (blocks of up to 1024 threads = 16 waves): at most one atomic per block ----
// Atomics on ONE address are served one after the other by the memory side (a few nanoseconds each), so a kernel
// that ends with thousands of them spends longer there than on its data.  Hence: few, large blocks for kernels
// that reduce; and a maximum is only sent when it would raise the value the slot already holds (the slot only
// ever grows, so a stale read can at worst cause an unnecessary atomic).
__device__ __forceinline__ void slot_atomic_max_i32(int32_t *slot, int v)
{
    if (v > *(volatile int32_t *)slot) atomicMax(slot, v);
}

__device__ __forceinline__ void block_atomic_max_i32(int v, int32_t *slot)
{
    __shared__ int sm_max[16];
    v = wave_max_i32(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    if (lane == 0) sm_max[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < nw; ++i) v = sm_max[i] > v ? sm_max[i] : v;
        slot_atomic_max_i32(slot, v);
    }
    __syncthreads();   // the staging array may be reused by the next call
}

__device__ __forceinline__ void block_atomic_add_i64(int64_t v, int64_t *slot)
{
    __shared__ int64_t sm_sum[16];
    v = wave_sum_i64(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    if (lane == 0) sm_sum[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < nw; ++i) v += sm_sum[i];
        if (v) atomic_add_i64(slot, v);
    }
    __syncthreads();
}

// block-wide sum, valid in thread 0 only
__device__ __forceinline__ int64_t block_sum_i64(int64_t v)
{
    __shared__ int64_t sm_bs[16];
    v = wave_sum_i64(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    if (lane == 0) sm_bs[wave] = v;
    __syncthreads();
    if (threadIdx.x == 0)
        for (int i = 1; i < nw; ++i) v += sm_bs[i];
    __syncthreads();
    return v;
}

// ---- block-input merge: both errors are aligned on the finer of their two grids (Ea, Eb: exponents) ----
__device__ __forceinline__ void merge_shifts(int Ea, int Eb, int &sa, int &sb, int &Em, uint32_t *status)
{
    Em = Ea < Eb ? Ea : Eb;
    sa = Ea - Em;
    sb = Eb - Em;
    if (sa > 24 || sb > 24) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, (uint32_t)EOQ_FLAG_EXP_GAP);
        sa = sa > 24 ? 24 : sa;
        sb = sb > 24 ? 24 : sb;
    }
}

// n / d for n < 2^31 through a host-made reciprocal: mul = ceil(2^(31+sh) / d), sh = ceil(log2 d).  (An integer
// division costs about 40 instructions per lane on this chip; kernels whose set-up decomposes pixel indices take
// the reciprocals of their divisors from the host instead.)
struct Recip { uint32_t mul; int sh; };
static inline Recip make_recip(uint32_t d)
{
    Recip r{0x80000000u, 0};
    if (d <= 1) return r;
    int s = 0;
    while ((1ull << s) < d) ++s;
    r.sh = s;
    r.mul = (uint32_t)((((unsigned long long)1 << (31 + s)) + d - 1) / d);
    return r;
}
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t mul, int sh) { return __umulhi(n << 1, mul) >> sh; }
__device__ __forceinline__ uint32_t fast_div(uint32_t n, const Recip &r) { return __umulhi(n << 1, r.mul) >> r.sh; }

static inline int conv_out_dim(int in, int pad, int k, int st) { return (in + 2 * pad - k) / st + 1; }
static inline int conv_out_dim_fwd(int in, int pad, int k, int st) { return (in + 2 * pad - k) / st + 1; }
static inline size_t round_up(size_t v, size_t m) { return (v + m - 1) / m * m; }

// ---- few-channel inputs (C <= 4, the network stem): the image is copied once into a zero-bordered buffer
// with 4 bytes per pixel, so that 4 consecutive pixels of a row are one aligned-to-4, 16-byte k-chunk and the
// filter's columns are walked 4 at a time (S4 groups).  No im2col matrix is materialised.
struct Pad4Geom {
    int Hp, Wp, S4, KP;      // padded extents (pixels), column groups per filter row, padded reduction bytes
    size_t img_bytes, w_bytes;
};
static inline Pad4Geom pad4_geom(const eoq_conv_desc *d)
{
    Pad4Geom g;
    const int Q = conv_out_dim_fwd(d->W, d->pad, d->S, d->stride);
    g.S4 = (d->S + 3) / 4;
    g.Hp = d->H + 2 * d->pad;
    int wp = (Q - 1) * d->stride + 4 * g.S4;
    if (wp < d->W + 2 * d->pad) wp = d->W + 2 * d->pad;
    g.Wp = (wp + 3) / 4 * 4;
    g.KP = d->R * g.S4 * 16;
    g.img_bytes = (size_t)d->N * g.Hp * g.Wp * 4;
    g.w_bytes = (size_t)d->K * g.KP;
    return g;
}

// most partial-sum buffers the weight-gradient kernel may write for a filter of `elems` int32 elements:
// as many as keep the chip busy for small filters, few enough for large ones that their traffic stays small
// Partial-sum buffers lie WGRAD_PART_PAD elements further apart than they need to: filter sizes are powers of two (or
// nine times one), and buffers exactly such a distance apart start on the same memory channels -- the finalize
// kernel, which reads the same element of every buffer at once, then queues up on a few channels.
constexpr size_t WGRAD_PART_PAD = 1088;      // 4352 bytes
static inline int wgrad_max_splits(size_t elems)
{
    size_t cap = ((size_t)48 << 20) / (elems * 4 + 1);
    if (cap < 4) cap = 4;
    if (cap > 1024) cap = 1024;
    return (int)cap;
}
