// HBM-bound passes of the training step: the real-input quantisers (Eq.5-7), the pre-bias
// (Eq.2 line x1), ReLU backward with the scalar-gradient statistics (Eq.3 e1, Eq.4 g_b2 / g_gamma),
// the scale-quantiser passes of the backward chain (Eq.11, Eq.12), the merge of branch and
// shortcut errors, and the 8-bit update (Eq.13).
//
// Every kernel streams 16 elements per lane per iteration (one 16-byte int8 vector, four for
// int32 / fp32 sources) with a grid-stride loop; tails shorter than 16 are done one by one.
// All pointers must be 16-byte aligned.
#include "common.h"

namespace {

constexpr int EW_THREADS = 1024;          // few, large blocks: see the note on same-address atomics in common.h
constexpr unsigned EW_MAX_BLOCKS = 256 * 2;

inline unsigned ew_blocks(size_t n_vec)
{
    size_t b = (n_vec + EW_THREADS - 1) / EW_THREADS;
    if (b < 1) b = 1;
    if (b > EW_MAX_BLOCKS) b = EW_MAX_BLOCKS;
    return (unsigned)b;
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

__device__ __forceinline__ int byte_at(const v4i &v, int i)   // sign-extended byte i (0..15)
{
    return (int)(int8_t)((uint32_t)v[i >> 2] >> (8 * (i & 3)));
}

__device__ __forceinline__ void set_byte(v4i &v, int i, int code)
{
    uint32_t sh = 8 * (i & 3);
    v[i >> 2] = (int)(((uint32_t)v[i >> 2] & ~(0xffu << sh)) | (((uint32_t)code & 0xffu) << sh));
}

// ------------------------------------------------------------------------------------------
// eoq_quantize
// ------------------------------------------------------------------------------------------
__global__ void absmax_f32_kernel(const float *x, size_t n, uint32_t *slot_bits, uint32_t *status)
{
    __shared__ uint32_t red[16];
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t m = 0;
    for (; i < n; i += stride) {
        uint32_t b = __float_as_uint(x[i]) & 0x7fffffffu;
        m = b > m ? b : m;
    }
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (unsigned w = 1; w < (blockDim.x + 63) / 64; ++w) m = red[w] > m ? red[w] : m;
        if (m >= 0x7f800000u) atomicOr(status, (uint32_t)EOQ_FLAG_NONFINITE);
        if (m > *(volatile uint32_t *)slot_bits) atomicMax(slot_bits, m);      // one same-address atomic per block at most
    }
}

// R(log2 |x|max * 2^pre) from the float's bits (Eq.7, scale): value = mant * 2^(e - 23) with an
// integer mantissa, so R(log2) = e - 23 + R(log2 mant), and R(log2 mant) is the integer test.
__device__ __forceinline__ int scale_exponent_f32bits(uint32_t bits)
{
    int e = (int)(bits >> 23);
    uint32_t mant = bits & 0x7fffffu;
    if (e) mant |= 0x800000u; else e = 1;           // denormal: no hidden bit, exponent of the smallest normal
    return e - 127 - 23 + sq_exponent_u32(mant);
}

template <int MODE>
__global__ void quantize_f32_kernel(const float *x, size_t n, int pre_shift, void *q, int32_t *exp_slot,
                                    const uint32_t *slot_bits, uint32_t *status)
{
    int sh = pre_shift + 7;
    bool zero = false;
    if (MODE == EOQ_SQ) {
        uint32_t mb = *slot_bits;
        if (mb == 0 || mb >= 0x7f800000u) {
            zero = true;
            if (blockIdx.x == 0 && threadIdx.x == 0) *exp_slot = 0;
        } else {
            int R = scale_exponent_f32bits(mb) + pre_shift;
            sh = pre_shift + 7 - R;
            if (blockIdx.x == 0 && threadIdx.x == 0) *exp_slot = R - 7;
        }
    }
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    bool bad = false;
    if (MODE != EOQ_Q && (((uintptr_t)x | (uintptr_t)q) & 15) == 0) {
        // int8 output: four elements per lane and iteration (one 16-byte load, one 4-byte store)
        const size_t n4 = n / 4;
        for (size_t j = i; j < n4; j += stride) {
            const float4 xv = ((const float4 *)x)[j];
            const float xs[4] = {xv.x, xv.y, xv.z, xv.w};
            int cd[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float xf = xs[k];
                if (MODE != EOQ_SQ && (__float_as_uint(xf) & 0x7fffffffu) >= 0x7f800000u) { bad = true; xf = 0.f; }
                double v = zero ? 0.0 : rint(ldexp((double)xf, sh));
                v = v < -127.0 ? -127.0 : (v > 127.0 ? 127.0 : v);
                cd[k] = (int)v;
            }
            ((uint32_t *)q)[j] = pack4_i8(cd[0], cd[1], cd[2], cd[3]);
        }
        i += n4 * 4;               // the ragged tail, one element per lane
    }
    for (; i < n; i += stride) {
        float xf = x[i];
        if (MODE != EOQ_SQ && (__float_as_uint(xf) & 0x7fffffffu) >= 0x7f800000u) { bad = true; xf = 0.f; }
        double v = zero ? 0.0 : rint(ldexp((double)xf, sh));
        if (MODE == EOQ_Q) {
            v = v < -2147483648.0 ? -2147483648.0 : (v > 2147483647.0 ? 2147483647.0 : v);
            ((int32_t *)q)[i] = (int32_t)v;
        } else {
            v = v < -127.0 ? -127.0 : (v > 127.0 ? 127.0 : v);
            ((int8_t *)q)[i] = (int8_t)(int)v;
        }
    }
    if (bad) atomicOr(status, (uint32_t)EOQ_FLAG_NONFINITE);
}

// ------------------------------------------------------------------------------------------
// pre-bias
// ------------------------------------------------------------------------------------------
__global__ void pre_bias_kernel(const int8_t *a, size_t n, const int32_t *b_pre, int8_t *u)
{
    const int b = *b_pre;
    const size_t nv = n / 16;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < nv; i += stride) {
        v4i v = ((const v4i *)a)[i], o = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < 16; ++k) set_byte(o, k, clamp_i(byte_at(v, k) + b, -CODE_MAX, CODE_MAX));
        ((v4i *)u)[i] = o;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 15)) {
        size_t t = nv * 16 + threadIdx.x;
        u[t] = (int8_t)clamp_i((int)a[t] + b, -CODE_MAX, CODE_MAX);
    }
}

// ------------------------------------------------------------------------------------------
// ReLU backward + statistics
// ------------------------------------------------------------------------------------------
__global__ void relu_bwd_kernel(const int8_t *e0, const uint16_t *mask16, const int32_t *t, size_t n, int8_t *e1,
                                int64_t *sum_e1, int64_t *sum_e1t, int32_t *absmax)
{
    const size_t nv = n / 16;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    int64_t s1 = 0, st = 0;
    int mx = 0;
    for (; i < nv; i += stride) {
        v4i v = ((const v4i *)e0)[i], o = {0, 0, 0, 0};
        uint32_t m = mask16 ? (uint32_t)mask16[i] : 0xffffu;
        v4i tv[4];
        if (t) {
#pragma unroll
            for (int k = 0; k < 4; ++k) tv[k] = ((const v4i *)t)[i * 4 + k];
        }
        int ls = 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            int e = ((m >> k) & 1u) ? byte_at(v, k) : 0;
            set_byte(o, k, e);
            ls += e;
            int ae = e < 0 ? -e : e;
            mx = ae > mx ? ae : mx;
            if (t) st += (int64_t)e * (int64_t)tv[k >> 2][k & 3];
        }
        s1 += ls;
        if (e1) ((v4i *)e1)[i] = o;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 15)) {
        size_t j = nv * 16 + threadIdx.x;
        bool on = mask16 ? ((((const uint8_t *)mask16)[j >> 3] >> (j & 7)) & 1) : true;
        int e = on ? (int)e0[j] : 0;
        if (e1) e1[j] = (int8_t)e;
        s1 += e;
        int ae = e < 0 ? -e : e;
        mx = ae > mx ? ae : mx;
        if (t) st += (int64_t)e * (int64_t)t[j];
    }
    if (sum_e1) block_atomic_add_i64(s1, sum_e1);
    if (t && sum_e1t) block_atomic_add_i64(st, sum_e1t);
    if (absmax) block_atomic_max_i32(mx, absmax);
}

// ------------------------------------------------------------------------------------------
// sum e (* t): the scalar-parameter sums of Eq.4
// ------------------------------------------------------------------------------------------
__global__ void reduce_sum_kernel(const int8_t *e, const int32_t *t, size_t n, int64_t *sum)
{
    const size_t nv = n / 16;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    int64_t s = 0;
    for (; i < nv; i += stride) {
        const v4i v = ((const v4i *)e)[i];
        if (t) {
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                const v4i tv = ((const v4i *)t)[i * 4 + k4];
#pragma unroll
                for (int k = 0; k < 4; ++k) s += (int64_t)byte_at(v, 4 * k4 + k) * (int64_t)tv[k];
            }
        } else {
            int ls = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) ls = sum4_i8((uint32_t)v[q], ls);
            s += ls;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 15)) {
        const size_t j = nv * 16 + threadIdx.x;
        s += t ? (int64_t)e[j] * (int64_t)t[j] : (int64_t)e[j];
    }
    block_atomic_add_i64(s, sum);
}

// ------------------------------------------------------------------------------------------
// merge: abs-max of a*2^(Ea-Em) + b*2^(Eb-Em)
// ------------------------------------------------------------------------------------------
__global__ void merge_absmax_kernel(const int8_t *a, const int32_t *exp_a, const int8_t *b, const int32_t *exp_b,
                                    size_t n, int32_t *absmax, uint32_t *status)
{
    int sa, sb, Em;
    merge_shifts(*exp_a, *exp_b, sa, sb, Em, status);
    const size_t nv = n / 16;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    int mx = 0;
    for (; i < nv; i += stride) {
        v4i va = ((const v4i *)a)[i], vb = ((const v4i *)b)[i];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            int v = (byte_at(va, k) << sa) + (byte_at(vb, k) << sb);
            v = v < 0 ? -v : v;
            mx = v > mx ? v : mx;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 15)) {
        size_t j = nv * 16 + threadIdx.x;
        int v = ((int)a[j] << sa) + ((int)b[j] << sb);
        v = v < 0 ? -v : v;
        mx = v > mx ? v : mx;
    }
    block_atomic_max_i32(mx, absmax);
}

// ------------------------------------------------------------------------------------------
// scale-quantiser passes (second phase: the abs-max is known)
// ------------------------------------------------------------------------------------------
struct SqArgs {
    const int32_t *acc;
    const int8_t *src_a, *src_b;
    const int32_t *exp_b, *gamma, *absmax, *exp_in;
    int32_t exp_in_off;
    size_t n;
    int8_t *out;
    int32_t *exp_out;
    int64_t *sum_out;
    int32_t *max_code_out;
    uint32_t *status;
    const uint16_t *mask16;      // SQ_MERGE: ReLU mask applied to the output (16 bits per 16 elements)
    int32_t *absmax_out;         // SQ_MERGE with mask: max|out|
    int8_t *out_b;               // SQ_MERGE: second output Q_e(out * gamma)
    int32_t *exp_out_b;
    const int32_t *absmax_m;     // SQ_MERGE with out_b and a mask: max|v| over the elements whose mask bit is set
};

// One 16-element vector of the merge pass in 32-bit arithmetic (|v| < 2^30, |code * gamma| < 2^30): codes of
// a * 2^sa + b * 2^sb under the mask, their sum, optionally Q_e(code * gamma) as a second vector.
template <bool L1, bool L2, bool TWO>
__device__ __forceinline__ void merge_vec32(const v4i a, const v4i b, uint32_t mk, int sa, int sb, int s1, int g, int s2,
                                            v4i &o, v4i &o2, int &sum)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int c[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int av = __builtin_amdgcn_sbfe(a[q], 8 * k, 8), bv = __builtin_amdgcn_sbfe(b[q], 8 * k, 8);
            c[k] = sq_code32<L1>((av << sa) + (bv << sb), s1);
        }
        const uint32_t pk = pack4_i8(c[0], c[1], c[2], c[3]) & byte_mask4(mk >> (4 * q));
        sum = sum4_i8(pk, sum);
        o[q] = (int)pk;
        if (TWO) {
            int d[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) d[k] = sq_code32<L2>(__builtin_amdgcn_sbfe((int)pk, 8 * k, 8) * g, s2);
            o2[q] = (int)pack4_i8(d[0], d[1], d[2], d[3]);
        }
    }
}

template <int MODE>
__global__ void sq_pass_kernel(SqArgs p)
{
    int sa = 0, sb = 0, g = 0;
    int E = *p.exp_in + p.exp_in_off;
    uint64_t M = (uint64_t)(uint32_t)*p.absmax;
    if (MODE == EOQ_RQ_SQ_GAMMA) {
        g = *p.gamma;
        M *= (uint64_t)(g < 0 ? -g : g);
        E -= 7;
    }
    if (MODE == EOQ_RQ_SQ_MERGE) {
        int Em;
        merge_shifts(*p.exp_in + p.exp_in_off, *p.exp_b, sa, sb, Em, p.status);
        E = Em;
    }
    const int r = M ? sq_exponent_u64(M) : 7;
    // second output of the merge pass: the scale quantiser is monotone, so the largest masked code is the code of
    // the largest masked value, and the shift of Q_e(out * gamma) is known before any element has been coded
    int r2 = 7;
    if (MODE == EOQ_RQ_SQ_MERGE && p.out_b) {
        g = *p.gamma;
        const uint64_t Mm = p.absmax_m ? (uint64_t)(uint32_t)*p.absmax_m : M;
        const uint64_t M2 = (Mm ? (uint64_t)sq_code((int64_t)Mm, r) : 0) * (uint64_t)(g < 0 ? -g : g);
        r2 = M2 ? sq_exponent_u64(M2) : 7;
        const int E2 = (M ? E + r - 7 : E) - 7;
        if (blockIdx.x == 0 && threadIdx.x == 0) *p.exp_out_b = M2 ? E2 + r2 - 7 : E2;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *p.exp_out = M ? E + r - 7 : E;
        if (p.max_code_out) *p.max_code_out = M ? sq_code((int64_t)M, r) : 0;
    }
    const size_t nv = p.n / 16;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    int64_t s = 0;
    int mxo = 0;
    if (MODE == EOQ_RQ_SQ_MERGE && !p.absmax_out && (p.n & 15) == 0 && sa <= 22 && sb <= 22 && g > -(1 << 22) && g < (1 << 22)) {
        // the usual case in 32-bit arithmetic, the shifts' directions resolved outside the element loop
        const int s1 = r - 7, s2 = r2 - 7;
        int ls = 0, since = 0;
        for (; i < nv; i += stride) {
            const v4i a = ((const v4i *)p.src_a)[i], b = ((const v4i *)p.src_b)[i];
            const uint32_t mk = p.mask16 ? (uint32_t)p.mask16[i] : 0xffffu;
            v4i o, o2;
            if (!p.out_b) {
                if (s1 <= 0) merge_vec32<true, true, false>(a, b, mk, sa, sb, s1, 0, 0, o, o2, ls);
                else merge_vec32<false, true, false>(a, b, mk, sa, sb, s1, 0, 0, o, o2, ls);
            } else {
                if (s1 <= 0) {
                    if (s2 <= 0) merge_vec32<true, true, true>(a, b, mk, sa, sb, s1, g, s2, o, o2, ls);
                    else merge_vec32<true, false, true>(a, b, mk, sa, sb, s1, g, s2, o, o2, ls);
                } else {
                    if (s2 <= 0) merge_vec32<false, true, true>(a, b, mk, sa, sb, s1, g, s2, o, o2, ls);
                    else merge_vec32<false, false, true>(a, b, mk, sa, sb, s1, g, s2, o, o2, ls);
                }
                ((v4i *)p.out_b)[i] = o2;
            }
            ((v4i *)p.out)[i] = o;
            if (++since == 1 << 16) { s += ls; ls = 0; since = 0; }      // long before 32 bits fill
        }
        s += ls;
        if (p.sum_out) block_atomic_add_i64(s, p.sum_out);
        return;
    }
    for (; i < nv; i += stride) {
        v4i o = {0, 0, 0, 0};
        int ls = 0;
        if (MODE == EOQ_RQ_SQ_ACC) {
            v4i a[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) a[k] = ((const v4i *)p.acc)[i * 4 + k];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                int c = sq_code((int64_t)a[k >> 2][k & 3], r);
                set_byte(o, k, c);
                ls += c;
            }
        } else if (MODE == EOQ_RQ_SQ_GAMMA) {
            v4i a = ((const v4i *)p.src_a)[i];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                int c = sq_code((int64_t)byte_at(a, k) * (int64_t)g, r);
                set_byte(o, k, c);
                ls += c;
            }
        } else {
            v4i a = ((const v4i *)p.src_a)[i], b = ((const v4i *)p.src_b)[i];
            const uint32_t mk = p.mask16 ? (uint32_t)p.mask16[i] : 0xffffu;
            v4i o2 = {0, 0, 0, 0};
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                int c = sq_code((int64_t)((byte_at(a, k) << sa) + (byte_at(b, k) << sb)), r);
                c = ((mk >> k) & 1u) ? c : 0;
                set_byte(o, k, c);
                ls += c;
                const int ac = c < 0 ? -c : c;
                mxo = ac > mxo ? ac : mxo;
                if (p.out_b) set_byte(o2, k, sq_code((int64_t)c * (int64_t)g, r2));
            }
            if (p.out_b) ((v4i *)p.out_b)[i] = o2;
        }
        s += ls;
        ((v4i *)p.out)[i] = o;
    }
    if (blockIdx.x == 0 && threadIdx.x < (p.n & 15)) {
        size_t j = nv * 16 + threadIdx.x;
        int64_t v;
        if (MODE == EOQ_RQ_SQ_ACC) v = p.acc[j];
        else if (MODE == EOQ_RQ_SQ_GAMMA) v = (int64_t)p.src_a[j] * (int64_t)g;
        else v = ((int)p.src_a[j] << sa) + ((int)p.src_b[j] << sb);
        int c = sq_code(v, r);
        p.out[j] = (int8_t)c;
        s += c;
    }
    if (p.sum_out) block_atomic_add_i64(s, p.sum_out);
    if (MODE == EOQ_RQ_SQ_MERGE && p.absmax_out) block_atomic_max_i32(mxo, p.absmax_out);
}

// ------------------------------------------------------------------------------------------
// update
// ------------------------------------------------------------------------------------------
__global__ void absmax_i8_kernel(const int8_t *g, size_t n, int32_t *slot)
{
    const size_t nv = n / 16;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    int mx = 0;
    for (; i < nv; i += stride) {
        v4i v = ((const v4i *)g)[i];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            int a = byte_at(v, k);
            a = a < 0 ? -a : a;
            mx = a > mx ? a : mx;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 15)) {
        int a = g[nv * 16 + threadIdx.x];
        a = a < 0 ? -a : a;
        mx = a > mx ? a : mx;
    }
    block_atomic_max_i32(mx, slot);
}

// delta on the 2^-7 grid for one gradient code (Eq.13): u = SQ(m*g*2^(Eg-j)), d = R(u * 2^(Eu+7))
struct UpdateRule {
    int m, r, sh;   // sh = -(Eu + 7): right shift if positive
    __device__ __forceinline__ int delta(int g) const
    {
        return (int)rne_shift64((int64_t)sq_code((int64_t)m * g, r), sh);
    }
};

// ---- optional stochastic rounding of the update (not the paper's rule; selected by a non-NULL sr_slot) ----
// d = floor((u_code + r) / 2^s) for s = -(Eu + 7) > 0, r = the low s bits (s capped at 62) of a 64-bit hash of
// (seed, tensor id, step, element index); an exact left shift otherwise.  The hash is counter based, so any
// element's draw can be regenerated on its own: z = seed*A + tensor*B + step*C + index*D (mod 2^64), then the
// splitmix64 finaliser.
constexpr uint64_t SR_A = 0x9E3779B97F4A7C15ull, SR_B = 0xC2B2AE3D27D4EB4Full, SR_C = 0xA0761D6478BD642Full,
                   SR_D = 0xD6E8FEB86659FD93ull;

__device__ __forceinline__ uint64_t sr_base(const uint32_t *sr_slot, uint32_t tensor)
{
    return (uint64_t)sr_slot[0] * SR_A + (uint64_t)tensor * SR_B + (uint64_t)sr_slot[1] * SR_C;
}

__device__ __forceinline__ uint64_t sr_word(uint64_t base, uint64_t index)
{
    uint64_t z = base + index * SR_D;
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ int sr_delta(const UpdateRule &u, int g, uint64_t word)
{
    const int64_t c = sq_code((int64_t)u.m * g, u.r);
    if (u.sh <= 0) return (int)(c << (-u.sh));
    const int s = u.sh > 62 ? 62 : u.sh;
    return (int)((c + (int64_t)(word & ((uint64_t(1) << s) - 1))) >> s);
}

__global__ void sr_next_step_kernel(uint32_t *sr_slot) { sr_slot[1] += 1u; }

__device__ __forceinline__ bool make_update_rule(int max_code, int Eg, const int32_t *lr_slot, UpdateRule &u,
                                                 uint32_t *status)
{
    if (max_code == 0) return false;
    u.m = lr_slot[0];
    const int j = lr_slot[1];
    u.r = sq_exponent_u64((uint64_t)u.m * (uint64_t)max_code);
    const int Eu = Eg - j + u.r - 7;
    u.sh = -(Eu + 7);
    if (u.sh < -24) {
        atomicOr(status, (uint32_t)EOQ_FLAG_SHIFT_RANGE);
        u.sh = -24;
    }
    return true;
}

__global__ void update_int8_kernel(int8_t *w, size_t n, const int8_t *g, const int32_t *g_exp, const int32_t *g_max,
                                   const int32_t *lr_slot, uint32_t *status, const uint32_t *sr_slot, uint32_t tensor)
{
    UpdateRule u;
    if (!make_update_rule(*g_max, *g_exp, lr_slot, u, status)) return;
    const uint64_t base = sr_slot ? sr_base(sr_slot, tensor) : 0;
    const size_t nv = n / 16;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < nv; i += stride) {
        v4i wv = ((const v4i *)w)[i], gv = ((const v4i *)g)[i], o = {0, 0, 0, 0};
        if (sr_slot) {
#pragma unroll
            for (int k = 0; k < 16; ++k)
                set_byte(o, k, clamp_i(byte_at(wv, k) - sr_delta(u, byte_at(gv, k), sr_word(base, i * 16 + k)), -CODE_MAX, CODE_MAX));
        } else {
#pragma unroll
            for (int k = 0; k < 16; ++k)
                set_byte(o, k, clamp_i(byte_at(wv, k) - u.delta(byte_at(gv, k)), -CODE_MAX, CODE_MAX));
        }
        ((v4i *)w)[i] = o;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 15)) {
        size_t t = nv * 16 + threadIdx.x;
        const int d = sr_slot ? sr_delta(u, g[t], sr_word(base, t)) : u.delta(g[t]);
        w[t] = (int8_t)clamp_i((int)w[t] - d, -CODE_MAX, CODE_MAX);
    }
}

// ------------------------------------------------------------------------------------------
// Q_g, Q_u and the update of one filter bank in one pass (Eq.12, Eq.13), with the transposed copy
// ------------------------------------------------------------------------------------------
struct GradUpdate {
    const int32_t *acc, *absmax, *exp_in, *lr;
    int32_t exp_in_off;
    int8_t *w, *wt, *g_out;
    int32_t *exp_out, *max_code_out;
    uint32_t *status;
    int K, RS, C;
    size_t n;
    const uint32_t *sr_slot;   // non-NULL: stochastic rounding of the update
    uint32_t tensor;
};

struct GradRule {
    int r;            // Q_g shift exponent
    bool live;        // a non-zero gradient exists
    UpdateRule u;
    bool sr;
    uint64_t sr_base;
};

__device__ __forceinline__ GradRule make_grad_rule(const GradUpdate &p, bool writer)
{
    GradRule gr;
    const uint64_t M = (uint64_t)(uint32_t)*p.absmax;
    const int E = *p.exp_in + p.exp_in_off;
    gr.r = M ? sq_exponent_u64(M) : 7;
    const int Eg = M ? E + gr.r - 7 : E;
    const int gmax = M ? sq_code((int64_t)M, gr.r) : 0;
    if (writer) {
        if (p.exp_out) *p.exp_out = Eg;
        if (p.max_code_out) *p.max_code_out = gmax;
    }
    gr.live = make_update_rule(gmax, Eg, p.lr, gr.u, p.status);
    gr.sr = p.sr_slot != nullptr;
    gr.sr_base = gr.sr ? sr_base(p.sr_slot, p.tensor) : 0;
    return gr;
}

// 16 consecutive elements (the first has linear index i0 in K x R x S x C order): codes of the gradient, new weights
__device__ __forceinline__ void grad_update16(const GradRule &gr, const v4i a[4], v4i wv, v4i &gv, v4i &ov, size_t i0)
{
    gv = v4i{0, 0, 0, 0};
    ov = wv;
    if (!gr.live) return;
    if (gr.sr) {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int g = sq_code((int64_t)a[k >> 2][k & 3], gr.r);
            set_byte(gv, k, g);
            set_byte(ov, k, clamp_i(byte_at(wv, k) - sr_delta(gr.u, g, sr_word(gr.sr_base, i0 + k)), -CODE_MAX, CODE_MAX));
        }
        return;
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int g = sq_code((int64_t)a[k >> 2][k & 3], gr.r);
        set_byte(gv, k, g);
        set_byte(ov, k, clamp_i(byte_at(wv, k) - gr.u.delta(g), -CODE_MAX, CODE_MAX));
    }
}

// any element count, no transposed copy
__global__ void grad_update_flat_kernel(GradUpdate p)
{
    const GradRule gr = make_grad_rule(p, blockIdx.x == 0 && threadIdx.x == 0);
    const size_t nv = p.n / 16;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nv; i += (size_t)gridDim.x * blockDim.x) {
        v4i a[4], gv, ov;
#pragma unroll
        for (int k = 0; k < 4; ++k) a[k] = ((const v4i *)p.acc)[i * 4 + k];
        grad_update16(gr, a, ((const v4i *)p.w)[i], gv, ov, i * 16);
        ((v4i *)p.w)[i] = ov;
        if (p.g_out) ((v4i *)p.g_out)[i] = gv;
    }
    if (blockIdx.x == 0 && threadIdx.x < (p.n & 15)) {
        const size_t t = nv * 16 + threadIdx.x;
        const int g = gr.live ? sq_code((int64_t)p.acc[t], gr.r) : 0;
        const int d = !gr.live ? 0 : (gr.sr ? sr_delta(gr.u, g, sr_word(gr.sr_base, t)) : gr.u.delta(g));
        if (gr.live) p.w[t] = (int8_t)clamp_i((int)p.w[t] - d, -CODE_MAX, CODE_MAX);
        if (p.g_out) p.g_out[t] = (int8_t)g;
    }
}

// K x RS x C filters with K, C multiples of 16: one workgroup per 64 (k) x 64 (c) tile of one tap; the new weights
// also go out in C x RS x K order through a transposing LDS tile
constexpr int GU_LD = 80;
__global__ void __launch_bounds__(256) grad_update_tiled_kernel(GradUpdate p)
{
    __builtin_amdgcn_s_setprio(3);
    __shared__ __align__(16) int8_t tile[64 * GU_LD];
    const GradRule gr = make_grad_rule(p, blockIdx.x == 0 && threadIdx.x == 0);
    const int tiles_c = (p.C + 63) / 64;
    int b = blockIdx.x;
    const int tc = b % tiles_c; b /= tiles_c;
    const int rs = b % p.RS;
    const int tk = b / p.RS;
    const int t = threadIdx.x;
    const int kl = t >> 2, cl = (t & 3) * 16;
    const int k = tk * 64 + kl, c = tc * 64 + cl;
    if (k < p.K && c < p.C) {
        const size_t i = (((size_t)k * p.RS + rs) * p.C + c) / 16;
        v4i a[4], gv, ov;
#pragma unroll
        for (int q = 0; q < 4; ++q) a[q] = ((const v4i *)p.acc)[i * 4 + q];
        grad_update16(gr, a, ((const v4i *)p.w)[i], gv, ov, i * 16);
        ((v4i *)p.w)[i] = ov;
        if (p.g_out) ((v4i *)p.g_out)[i] = gv;
#pragma unroll
        for (int q = 0; q < 16; ++q) tile[(cl + q) * GU_LD + kl] = (int8_t)byte_at(ov, q);
    }
    __syncthreads();
    const int cr = t >> 2, ks = (t & 3) * 16;
    const int c2 = tc * 64 + cr, k2 = tk * 64 + ks;
    if (c2 < p.C && k2 < p.K)
        *(v4i *)(p.wt + ((size_t)c2 * p.RS + rs) * p.K + k2) = *(const v4i *)(tile + cr * GU_LD + ks);
}

__global__ void update_scalars_kernel(int32_t *scalars, const eoq_scalar_grad *descs, int count, const int64_t *sums,
                                      const int32_t *exps, const int32_t *lr_slot, int32_t *g_code_out,
                                      int32_t *g_exp_out, uint32_t *status, const uint32_t *sr_slot,
                                      const uint32_t *tensor_ids)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    const eoq_scalar_grad d = descs[i];
    // exact sum of the terms on the finest grid
    int E0 = exps[d.exp_idx[0]] + d.exp_off[0];
    int64_t S = sums[d.sum_idx[0]];
    if (d.n_terms > 1) {
        int E1 = exps[d.exp_idx[1]] + d.exp_off[1];
        int64_t S1 = sums[d.sum_idx[1]];
        int Em = E0 < E1 ? E0 : E1;
        int s0 = E0 - Em, s1 = E1 - Em;
        if (s0 > 24 || s1 > 24) {
            atomicOr(status, (uint32_t)EOQ_FLAG_EXP_GAP);
            s0 = s0 > 24 ? 24 : s0;
            s1 = s1 > 24 ? 24 : s1;
        }
        S = (S << s0) + (S1 << s1);
        E0 = Em;
    }
    // Q_g of the one-element tensor (Eq.12)
    int gc = 0, Eg = E0;
    if (S) {
        uint64_t M = (uint64_t)(S < 0 ? -S : S);
        int r = sq_exponent_u64(M);
        gc = sq_code(S, r);
        Eg = E0 + r - 7;
    }
    if (g_code_out) g_code_out[i] = gc;
    if (g_exp_out) g_exp_out[i] = Eg;
    // Q_u and the unclamped update (Eq.13, Eq.10)
    UpdateRule u;
    int a = gc < 0 ? -gc : gc;
    if (make_update_rule(a, Eg, lr_slot, u, status))
        scalars[d.param] -= sr_slot ? sr_delta(u, gc, sr_word(sr_base(sr_slot, tensor_ids[i]), 0)) : u.delta(gc);
}

} // namespace

// ============================================================================================
// C ABI
// ============================================================================================
extern "C" int eoq_quantize(eoq_ctx *c, const float *x, size_t n, int mode, int pre_shift, void *q, int32_t *exp_slot)
{
    if (!c || (n && (!x || !q)) || mode < EOQ_Q || mode > EOQ_SQ) return EOQ_ERR_ARG;
    if (mode == EOQ_SQ && !exp_slot) return EOQ_ERR_ARG;
    if (pre_shift < -64 || pre_shift > 64) return EOQ_ERR_ARG;
    uint32_t *slot = (uint32_t *)c->d_scratch;
    const unsigned blocks = ew_blocks(n ? n : 1);
    if (mode == EOQ_SQ) {
        if (int rc = eoq_fill_zero(c, slot, 4)) return rc;
        hipLaunchKernelGGL(absmax_f32_kernel, dim3(blocks), dim3(EW_THREADS), 0, c->stream, x, n, slot, c->d_status);
        hipLaunchKernelGGL(quantize_f32_kernel<EOQ_SQ>, dim3(blocks), dim3(EW_THREADS), 0, c->stream, x, n, pre_shift, q,
                           exp_slot, slot, c->d_status);
    } else if (mode == EOQ_CQ) {
        hipLaunchKernelGGL(quantize_f32_kernel<EOQ_CQ>, dim3(blocks), dim3(EW_THREADS), 0, c->stream, x, n, pre_shift, q,
                           exp_slot, slot, c->d_status);
    } else {
        hipLaunchKernelGGL(quantize_f32_kernel<EOQ_Q>, dim3(blocks), dim3(EW_THREADS), 0, c->stream, x, n, pre_shift, q,
                           exp_slot, slot, c->d_status);
    }
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_pre_bias(eoq_ctx *c, const int8_t *a, size_t n, const int32_t *b_pre, int8_t *u)
{
    if (!c || !b_pre || (n && (!a || !u)) || !aligned16(a) || !aligned16(u)) return EOQ_ERR_ARG;
    if (!n) return EOQ_OK;
    hipLaunchKernelGGL(pre_bias_kernel, dim3(ew_blocks(n / 16)), dim3(EW_THREADS), 0, c->stream, a, n, b_pre, u);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_relu_bwd(eoq_ctx *c, const int8_t *e0, const uint32_t *mask_bits, const int32_t *t_wide, size_t n,
                            int8_t *e1, int64_t *sum_e1, int64_t *sum_e1t, int32_t *absmax_e1)
{
    if (!c || (n && !e0) || !aligned16(e0) || !aligned16(e1) || !aligned16(t_wide) || ((uintptr_t)mask_bits & 3))
        return EOQ_ERR_ARG;
    if (!n) return EOQ_OK;
    hipLaunchKernelGGL(relu_bwd_kernel, dim3(ew_blocks(n / 16)), dim3(EW_THREADS), 0, c->stream, e0,
                       (const uint16_t *)mask_bits, t_wide, n, e1, sum_e1, sum_e1t, absmax_e1);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_reduce_sum_i64(eoq_ctx *c, const int8_t *e, const int32_t *t, size_t n, int64_t *sum)
{
    if (!c || !sum || (n && !e) || !aligned16(e) || !aligned16(t)) return EOQ_ERR_ARG;
    if (!n) return EOQ_OK;
    hipLaunchKernelGGL(reduce_sum_kernel, dim3(ew_blocks(n / 16)), dim3(EW_THREADS), 0, c->stream, e, t, n, sum);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_merge_absmax(eoq_ctx *c, const int8_t *a, const int32_t *exp_a, const int8_t *b,
                                const int32_t *exp_b, size_t n, int32_t *absmax_slot)
{
    if (!c || !exp_a || !exp_b || !absmax_slot || (n && (!a || !b)) || !aligned16(a) || !aligned16(b))
        return EOQ_ERR_ARG;
    if (!n) return EOQ_OK;
    hipLaunchKernelGGL(merge_absmax_kernel, dim3(ew_blocks(n / 16)), dim3(EW_THREADS), 0, c->stream, a, exp_a, b,
                       exp_b, n, absmax_slot, c->d_status);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

int eoq_requant_fwd_standalone(eoq_ctx *c, const eoq_requant_args *a);   // conv_igemm.hip

extern "C" int eoq_requant_epilogue(eoq_ctx *c, const eoq_requant_args *a)
{
    if (!c || !a) return EOQ_ERR_ARG;
    if (a->mode == EOQ_RQ_FWD) return eoq_requant_fwd_standalone(c, a);
    if (a->mode < EOQ_RQ_SQ_ACC || a->mode > EOQ_RQ_SQ_MERGE) return EOQ_ERR_ARG;
    if (!a->absmax || !a->exp_in || !a->exp_out || (a->n && !a->out) || !aligned16(a->out)) return EOQ_ERR_ARG;
    SqArgs p;
    p.acc = a->acc; p.src_a = a->src_a; p.src_b = a->src_b; p.exp_b = a->exp_b; p.gamma = a->gamma;
    p.absmax = a->absmax; p.exp_in = a->exp_in; p.exp_in_off = a->exp_in_off; p.n = a->n; p.out = a->out;
    p.exp_out = a->exp_out; p.sum_out = a->sum_out; p.max_code_out = a->max_code_out; p.status = c->d_status;
    p.mask16 = nullptr; p.absmax_out = nullptr; p.out_b = nullptr; p.exp_out_b = nullptr; p.absmax_m = nullptr;
    if (a->mode == EOQ_RQ_SQ_MERGE) {
        // the mask is addressed in 16-element words: a ragged tail would need its own path
        if ((a->mask_bits || a->absmax_out || a->out_b) && (a->n & 15)) return EOQ_ERR_SHAPE;
        if ((uintptr_t)a->mask_bits & 3) return EOQ_ERR_ARG;
        p.mask16 = (const uint16_t *)a->mask_bits;
        p.absmax_out = a->absmax_out;
        if (a->out_b) {
            if (!a->gamma || !a->exp_out_b || !aligned16(a->out_b) || (a->mask_bits && !a->absmax_masked)) return EOQ_ERR_ARG;
            p.out_b = a->out_b; p.exp_out_b = a->exp_out_b; p.absmax_m = a->mask_bits ? a->absmax_masked : nullptr;
        }
    } else if (a->mask_bits || a->absmax_out || a->out_b) {
        return EOQ_ERR_ARG;
    }
    const dim3 grid(ew_blocks(a->n / 16)), block(EW_THREADS);
    switch (a->mode) {
    case EOQ_RQ_SQ_ACC:
        if ((a->n && !a->acc) || !aligned16(a->acc)) return EOQ_ERR_ARG;
        hipLaunchKernelGGL(sq_pass_kernel<EOQ_RQ_SQ_ACC>, grid, block, 0, c->stream, p);
        break;
    case EOQ_RQ_SQ_GAMMA:
        if ((a->n && !a->src_a) || !a->gamma || !aligned16(a->src_a)) return EOQ_ERR_ARG;
        hipLaunchKernelGGL(sq_pass_kernel<EOQ_RQ_SQ_GAMMA>, grid, block, 0, c->stream, p);
        break;
    default:
        if ((a->n && (!a->src_a || !a->src_b)) || !a->exp_b || !aligned16(a->src_a) || !aligned16(a->src_b))
            return EOQ_ERR_ARG;
        hipLaunchKernelGGL(sq_pass_kernel<EOQ_RQ_SQ_MERGE>, grid, block, 0, c->stream, p);
        break;
    }
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

static int update_int8_impl(eoq_ctx *c, int8_t *w, size_t n, const int8_t *g, const int32_t *g_exp_slot,
                            const int32_t *g_max_code, const int32_t *lr_slot, const uint32_t *sr_slot, uint32_t tensor)
{
    if (!c || !g_exp_slot || !lr_slot || (n && (!w || !g)) || !aligned16(w) || !aligned16(g)) return EOQ_ERR_ARG;
    if (!n) return EOQ_OK;
    const dim3 grid(ew_blocks(n / 16)), block(EW_THREADS);
    if (!g_max_code) {
        int32_t *slot = c->d_scratch + 1;
        if (int rc = eoq_fill_zero(c, slot, 4)) return rc;
        hipLaunchKernelGGL(absmax_i8_kernel, grid, block, 0, c->stream, g, n, slot);
        g_max_code = slot;
    }
    hipLaunchKernelGGL(update_int8_kernel, grid, block, 0, c->stream, w, n, g, g_exp_slot, g_max_code, lr_slot,
                       c->d_status, sr_slot, tensor);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_update_int8(eoq_ctx *c, int8_t *w, size_t n, const int8_t *g, const int32_t *g_exp_slot,
                               const int32_t *g_max_code, const int32_t *lr_slot)
{
    return update_int8_impl(c, w, n, g, g_exp_slot, g_max_code, lr_slot, nullptr, 0);
}

extern "C" int eoq_update_int8_sr(eoq_ctx *c, int8_t *w, size_t n, const int8_t *g, const int32_t *g_exp_slot,
                                  const int32_t *g_max_code, const int32_t *lr_slot, const uint32_t *sr_slot,
                                  uint32_t tensor_id)
{
    if (!sr_slot) return EOQ_ERR_ARG;
    return update_int8_impl(c, w, n, g, g_exp_slot, g_max_code, lr_slot, sr_slot, tensor_id);
}

extern "C" int eoq_sr_next_step(eoq_ctx *c, uint32_t *sr_slot)
{
    if (!c || !sr_slot) return EOQ_ERR_ARG;
    hipLaunchKernelGGL(sr_next_step_kernel, dim3(1), dim3(1), 0, c->stream, sr_slot);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

static int grad_update_impl(eoq_ctx *c, const eoq_conv_desc *d, const int32_t *acc, const int32_t *absmax_slot,
                            const int32_t *exp_in, int32_t exp_in_off, const int32_t *lr_slot, int8_t *w, int8_t *wt,
                            int8_t *g_out, int32_t *exp_out, int32_t *max_code_out, const uint32_t *sr_slot,
                            uint32_t tensor)
{
    if (!c || !d || !acc || !absmax_slot || !exp_in || !lr_slot || !w) return EOQ_ERR_ARG;
    if (d->K <= 0 || d->R <= 0 || d->S <= 0 || d->C <= 0) return EOQ_ERR_SHAPE;
    if (!aligned16(acc) || !aligned16(w) || !aligned16(wt) || !aligned16(g_out)) return EOQ_ERR_ARG;
    GradUpdate p{};
    p.acc = acc; p.absmax = absmax_slot; p.exp_in = exp_in; p.lr = lr_slot; p.exp_in_off = exp_in_off;
    p.w = w; p.wt = wt; p.g_out = g_out; p.exp_out = exp_out; p.max_code_out = max_code_out; p.status = c->d_status;
    p.K = d->K; p.RS = d->R * d->S; p.C = d->C;
    p.n = (size_t)d->K * p.RS * d->C;
    p.sr_slot = sr_slot; p.tensor = tensor;
    if (wt) {
        if (d->K % 16 || d->C % 16) return EOQ_ERR_SHAPE;
        const size_t tiles = (size_t)((d->K + 63) / 64) * p.RS * ((d->C + 63) / 64);
        if (tiles > 0x7fffffffu) return EOQ_ERR_SHAPE;
        hipLaunchKernelGGL(grad_update_tiled_kernel, dim3((unsigned)tiles), dim3(256), 0, c->stream, p);
    } else {
        hipLaunchKernelGGL(grad_update_flat_kernel, dim3(ew_blocks(p.n / 16 + 1)), dim3(EW_THREADS), 0, c->stream, p);
    }
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_grad_update(eoq_ctx *c, const eoq_conv_desc *d, const int32_t *acc, const int32_t *absmax_slot,
                               const int32_t *exp_in, int32_t exp_in_off, const int32_t *lr_slot, int8_t *w, int8_t *wt,
                               int8_t *g_out, int32_t *exp_out, int32_t *max_code_out)
{
    return grad_update_impl(c, d, acc, absmax_slot, exp_in, exp_in_off, lr_slot, w, wt, g_out, exp_out, max_code_out,
                            nullptr, 0);
}

extern "C" int eoq_grad_update_sr(eoq_ctx *c, const eoq_conv_desc *d, const int32_t *acc, const int32_t *absmax_slot,
                                  const int32_t *exp_in, int32_t exp_in_off, const int32_t *lr_slot, int8_t *w,
                                  int8_t *wt, int8_t *g_out, int32_t *exp_out, int32_t *max_code_out,
                                  const uint32_t *sr_slot, uint32_t tensor_id)
{
    if (!sr_slot) return EOQ_ERR_ARG;
    return grad_update_impl(c, d, acc, absmax_slot, exp_in, exp_in_off, lr_slot, w, wt, g_out, exp_out, max_code_out,
                            sr_slot, tensor_id);
}

static int update_scalars_impl(eoq_ctx *c, int32_t *scalars, const eoq_scalar_grad *descs, int32_t count,
                               const int64_t *sums, const int32_t *exps, const int32_t *lr_slot, int32_t *g_code_out,
                               int32_t *g_exp_out, const uint32_t *sr_slot, const uint32_t *tensor_ids)
{
    if (!c || count < 0 || (count && (!scalars || !descs || !sums || !exps)) || !lr_slot) return EOQ_ERR_ARG;
    if (!count) return EOQ_OK;
    hipLaunchKernelGGL(update_scalars_kernel, dim3((count + 63) / 64), dim3(64), 0, c->stream, scalars, descs, count,
                       sums, exps, lr_slot, g_code_out, g_exp_out, c->d_status, sr_slot, tensor_ids);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_update_scalars(eoq_ctx *c, int32_t *scalars, const eoq_scalar_grad *descs, int32_t count,
                                  const int64_t *sums, const int32_t *exps, const int32_t *lr_slot,
                                  int32_t *g_code_out, int32_t *g_exp_out)
{
    return update_scalars_impl(c, scalars, descs, count, sums, exps, lr_slot, g_code_out, g_exp_out, nullptr, nullptr);
}

extern "C" int eoq_update_scalars_sr(eoq_ctx *c, int32_t *scalars, const eoq_scalar_grad *descs, int32_t count,
                                     const int64_t *sums, const int32_t *exps, const int32_t *lr_slot,
                                     int32_t *g_code_out, int32_t *g_exp_out, const uint32_t *sr_slot,
                                     const uint32_t *tensor_ids)
{
    if (!sr_slot || (count && !tensor_ids)) return EOQ_ERR_ARG;
    return update_scalars_impl(c, scalars, descs, count, sums, exps, lr_slot, g_code_out, g_exp_out, sr_slot, tensor_ids);
}
