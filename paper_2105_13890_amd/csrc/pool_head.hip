// Pooling and the float head.  These sit outside Eq.2-13 (the paper quantises every layer except the
// last, Section 5.1) but are on the path of a training step: the stem's max pool, the global average
// pool (kept as an integer sum), and the fp64 classifier with softmax cross-entropy whose input error
// re-enters the integer chain through the scale quantiser.
//
// The head is evaluated in a fixed operation order (sequential fma chains in ascending index, a
// hand-written exp) so that its result does not depend on the machine.  Build without contraction.
#include "common.h"

namespace {

__device__ __forceinline__ int byte_at(const v4i &v, int i)
{
    return (int)(int8_t)((uint32_t)v[i >> 2] >> (8 * (i & 3)));
}
__device__ __forceinline__ void set_byte(v4i &v, int i, int code)
{
    uint32_t sh = 8 * (i & 3);
    v[i >> 2] = (int)(((uint32_t)v[i >> 2] & ~(0xffu << sh)) | (((uint32_t)code & 0xffu) << sh));
}

struct PoolGeom { int N, H, W, C, R, S, stride, pad, P, Q; };

// one lane: 16 channels of one output pixel
__global__ void maxpool_fwd_kernel(PoolGeom g, const int8_t *a, int8_t *y, const int32_t *b_next, int8_t *u_next,
                                   uint8_t *arg)
{
    const int c16 = g.C / 16;
    const size_t total = (size_t)g.N * g.P * g.Q * c16;
    const int b = b_next ? *b_next : 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        int cc = (int)(i % c16);
        size_t pix = i / c16;
        int q = (int)(pix % g.Q);
        size_t t = pix / g.Q;
        int p = (int)(t % g.P), n = (int)(t / g.P);
        int best[16], bi[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) { best[k] = -1000; bi[k] = 0; }
        for (int r = 0; r < g.R; ++r) {
            int h = p * g.stride + r - g.pad;
            if (h < 0 || h >= g.H) continue;
            for (int s = 0; s < g.S; ++s) {
                int x = q * g.stride + s - g.pad;
                if (x < 0 || x >= g.W) continue;
                v4i v = *(const v4i *)(a + (((size_t)n * g.H + h) * g.W + x) * g.C + cc * 16);
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    int e = byte_at(v, k);
                    if (e > best[k]) { best[k] = e; bi[k] = r * g.S + s; }     // strict: the first maximum wins
                }
            }
        }
        v4i o = {0, 0, 0, 0}, ou = {0, 0, 0, 0}, oa = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            set_byte(o, k, best[k]);
            set_byte(ou, k, clamp_i(best[k] + b, -CODE_MAX, CODE_MAX));
            set_byte(oa, k, bi[k]);
        }
        if (y) *(v4i *)(y + pix * g.C + cc * 16) = o;
        if (u_next) *(v4i *)(u_next + pix * g.C + cc * 16) = ou;
        if (arg) *(v4i *)(arg + pix * g.C + cc * 16) = oa;
    }
}

// one lane: 16 channels of one input pixel; it looks at every window that contains the pixel and takes the
// window's error where the forward pass recorded this pixel as the window's winner.
// OUT 0: int32 sums + abs-max;  OUT 1: abs-max only;  OUT 2: Q_e codes (Eq.11) from the abs-max of an OUT 1 launch:
// the sums are cheap to form twice (the gathered tensors are the small, pooled ones), so the wide tensor is never
// written.
// OUT 3 / OUT 4: the same result in one pass when the exponent did not change since the previous training step.  OUT 3
// codes with the exponent of the previous step (spec[0]; copied to *spec_used), takes the true abs-max on the way and
// adds the sum of its codes to *tmp_sum instead of *sum_out; OUT 4 compares: if the exponent was right it only
// commits (exponent, sum) and every workgroup leaves at once, otherwise it is an OUT 2 launch.  Either way it stores
// the exact exponent in spec[0] for the next step and leaves *tmp_sum at zero.
template <int OUT>
__global__ void maxpool_bwd_kernel(PoolGeom g, const uint8_t *arg, const int8_t *e, int32_t *d, int32_t *absmax,
                                   int8_t *q, const int32_t *exp_in, int32_t *exp_out, const uint16_t *mask16,
                                   int64_t *sum_out, int32_t *spec, int32_t *spec_used, int64_t *tmp_sum,
                                   int32_t *counters)
{
    const int c16 = g.C / 16;
    const size_t total = (size_t)g.N * g.H * g.W * c16;
    int mx = 0, r = 7;
    long long sum = 0;
    constexpr bool CODES = OUT >= 2, MAXIMUM = OUT != 2 && OUT != 4;
    const bool first = blockIdx.x == 0 && threadIdx.x == 0;
    if (OUT == 2 || OUT == 4) {
        const uint32_t M = (uint32_t)*absmax;
        r = M ? sq_exponent_u32(M) : 7;
        if (first) *exp_out = M ? *exp_in + r - 7 : *exp_in;
    }
    if (OUT == 4) {
        const bool hit = r == *spec_used;
        if (first) {
            spec[0] = r;
            atomicAdd(counters + (hit ? 0 : 1), 1);
            const long long s = *tmp_sum;
            *tmp_sum = 0;
            if (hit && sum_out && s) atomic_add_i64(sum_out, s);
        }
        if (hit) return;
    }
    if (OUT == 3) {
        const int rs = spec[0];
        if (first) *spec_used = rs;
        r = rs < 0 ? 7 : (rs > 31 ? 31 : rs);
    }
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        int cc = (int)(i % c16);
        size_t pix = i / c16;
        int x = (int)(pix % g.W);
        size_t t = pix / g.W;
        int h = (int)(t % g.H), n = (int)(t / g.H);
        int acc[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[k] = 0;
        // windows p with p*stride - pad <= h <= p*stride - pad + R - 1
        int p_lo = h + g.pad - g.R + 1;
        p_lo = p_lo <= 0 ? 0 : (p_lo + g.stride - 1) / g.stride;
        int p_hi = (h + g.pad) / g.stride;
        if (p_hi > g.P - 1) p_hi = g.P - 1;
        int q_lo = x + g.pad - g.S + 1;
        q_lo = q_lo <= 0 ? 0 : (q_lo + g.stride - 1) / g.stride;
        int q_hi = (x + g.pad) / g.stride;
        if (q_hi > g.Q - 1) q_hi = g.Q - 1;
        for (int p = p_lo; p <= p_hi; ++p)
            for (int qq = q_lo; qq <= q_hi; ++qq) {
                const int my = (h - (p * g.stride - g.pad)) * g.S + (x - (qq * g.stride - g.pad));
                const size_t o = (((size_t)n * g.P + p) * g.Q + qq) * g.C + cc * 16;
                v4i av = *(const v4i *)(arg + o), ev = *(const v4i *)(e + o);
#pragma unroll
                for (int k = 0; k < 16; ++k)
                    if ((byte_at(av, k) & 0xff) == my) acc[k] += byte_at(ev, k);
            }
        if (OUT == 0) {
            int32_t *o = d + pix * g.C + cc * 16;
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                v4i w = {acc[4 * k4], acc[4 * k4 + 1], acc[4 * k4 + 2], acc[4 * k4 + 3]};
                ((v4i *)o)[k4] = w;
            }
        }
        if (CODES) {
            // a sum of at most R*S int8 errors: 32-bit arithmetic, four codes per packed dword
            v4i o;
            const uint32_t mk = mask16 ? (uint32_t)mask16[pix * c16 + cc] : 0xffffu;
            int ls = 0;
            const int sh = r - 7;
            int cd[16];
            if (sh <= 0) {
#pragma unroll
                for (int k = 0; k < 16; ++k) cd[k] = sq_code32<true>(acc[k], sh);
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) cd[k] = sq_code32<false>(acc[k], sh);
            }
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const uint32_t pk = pack4_i8(cd[4 * q4], cd[4 * q4 + 1], cd[4 * q4 + 2], cd[4 * q4 + 3]) &
                                    byte_mask4(mk >> (4 * q4));
                ls = sum4_i8(pk, ls);
                o[q4] = (int)pk;
            }
            sum += ls;
            *(v4i *)(q + pix * g.C + cc * 16) = o;
        }
        if (MAXIMUM) {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                int av = acc[k] < 0 ? -acc[k] : acc[k];
                mx = av > mx ? av : mx;
            }
        }
    }
    if (MAXIMUM) block_atomic_max_i32(mx, absmax);
    if ((OUT == 2 || OUT == 4) && sum_out) block_atomic_add_i64(sum, sum_out);
    if (OUT == 3) block_atomic_add_i64(sum, tmp_sum);
}

// The 3x3 / stride 2 / padding 1 pool of the ImageNet-shaped nets: a lane owns 16 channels of a 2x2 block of input
// pixels (rows 2i, 2i+1, columns 2j, 2j+1).  The block lies in the four windows (i | i+1, j | j+1) and in no other,
// so each window's error and winner index are fetched once for four pixels.  OUT 1: abs-max of the sums; OUT 2: codes.
template <int OUT>
__global__ void __launch_bounds__(256) maxpool_bwd_3s2_kernel(PoolGeom g, const uint8_t *arg, const int8_t *e, int32_t *absmax, int8_t *q,
                                       const int32_t *exp_in, int32_t *exp_out, const uint16_t *mask16,
                                       int64_t *sum_out)
{
    const int c16 = g.C / 16;
    const int H2 = (g.H + 1) / 2, W2 = (g.W + 1) / 2;
    const size_t total = (size_t)g.N * H2 * W2 * c16;
    int mx = 0, r = 7;
    long long sum = 0;
    if (OUT == 2) {
        const uint32_t M = (uint32_t)*absmax;
        r = M ? sq_exponent_u32(M) : 7;
        if (blockIdx.x == 0 && threadIdx.x == 0) *exp_out = M ? *exp_in + r - 7 : *exp_in;
    }
    for (size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < total; i0 += (size_t)gridDim.x * blockDim.x) {
        const int cc = (int)(i0 % c16);
        size_t t = i0 / c16;
        const int j = (int)(t % W2); t /= W2;
        const int i = (int)(t % H2), n = (int)(t / H2);
        int acc[4][16];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[b][k] = 0;
#pragma unroll
        for (int dp = 0; dp < 2; ++dp)
#pragma unroll
            for (int dq = 0; dq < 2; ++dq) {
                const int p = i + dp, qq = j + dq;
                if (p >= g.P || qq >= g.Q) continue;
                const size_t o = (((size_t)n * g.P + p) * g.Q + qq) * g.C + cc * 16;
                const v4i av = *(const v4i *)(arg + o), ev = *(const v4i *)(e + o);
                // pixel (2i+a, 2j+b) is cell (a + 1 - 2dp, b + 1 - 2dq) of window (p, qq)
#pragma unroll
                for (int a = dp; a < 2; ++a)
#pragma unroll
                    for (int b = dq; b < 2; ++b) {
                        const int my = (a + 1 - 2 * dp) * 3 + (b + 1 - 2 * dq);
#pragma unroll
                        for (int k = 0; k < 16; ++k)
                            if ((byte_at(av, k) & 0xff) == my) acc[a * 2 + b][k] += byte_at(ev, k);
                    }
            }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int h = 2 * i + a, x = 2 * j + b;
                if (h >= g.H || x >= g.W) continue;
                if (OUT == 2) {
                    const size_t pix = ((size_t)n * g.H + h) * g.W + x;
                    const uint32_t mk = mask16 ? (uint32_t)mask16[pix * c16 + cc] : 0xffffu;
                    v4i o = {0, 0, 0, 0};
                    int ls = 0;
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const int cd = ((mk >> k) & 1u) ? sq_code((int64_t)acc[a * 2 + b][k], r) : 0;
                        set_byte(o, k, cd);
                        ls += cd;
                    }
                    sum += ls;
                    *(v4i *)(q + pix * g.C + cc * 16) = o;
                } else {
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const int v = acc[a * 2 + b][k] < 0 ? -acc[a * 2 + b][k] : acc[a * 2 + b][k];
                        mx = v > mx ? v : mx;
                    }
                }
            }
    }
    if (OUT == 1) block_atomic_max_i32(mx, absmax);
    if (OUT == 2 && sum_out) block_atomic_add_i64(sum, sum_out);
}

__global__ void gap_sum_kernel(const int8_t *y, int N, int HW, int C, int32_t *sum)
{
    const int c16 = C / 16;
    const int total = N * c16;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        int cc = i % c16, n = i / c16;
        int acc[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[k] = 0;
        for (int p = 0; p < HW; ++p) {
            v4i v = *(const v4i *)(y + ((size_t)n * HW + p) * C + cc * 16);
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[k] += byte_at(v, k);
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) sum[(size_t)n * C + cc * 16 + k] = acc[k];
    }
}

__global__ void broadcast_hw_kernel(const int8_t *codes, int N, int HW, int C, int8_t *e)
{
    const int c16 = C / 16;
    const size_t total = (size_t)N * HW * c16;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        int cc = (int)(i % c16);
        size_t pix = i / c16;
        int n = (int)(pix / HW);
        *(v4i *)(e + pix * C + cc * 16) = *(const v4i *)(codes + (size_t)n * C + cc * 16);
    }
}

// -------------------------------------------------------------------------------------------
// float head
// -------------------------------------------------------------------------------------------
// exp for x <= 0: k = rint(x * log2 e); r = x - k ln2 with ln2 split in two parts; degree-13 Taylor
// polynomial evaluated by Horner with fma; scaled by 2^k.
__device__ double head_exp(double x)
{
    const double LOG2E = 0x1.71547652b82fep+0;
    const double LN2_HI = 0x1.62e42feep-1;
    const double LN2_LO = 0x1.a39ef35793c76p-33;
    if (x < -700.0) x = -700.0;
    const double k = rint(x * LOG2E);
    double r = fma(k, -LN2_HI, x);
    r = fma(k, -LN2_LO, r);
    double p = 1.0 / 6227020800.0;
    p = fma(p, r, 1.0 / 479001600.0);
    p = fma(p, r, 1.0 / 39916800.0);
    p = fma(p, r, 1.0 / 3628800.0);
    p = fma(p, r, 1.0 / 362880.0);
    p = fma(p, r, 1.0 / 40320.0);
    p = fma(p, r, 1.0 / 5040.0);
    p = fma(p, r, 1.0 / 720.0);
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)k);
}

constexpr int HEAD_SOFTMAX_LDS = 4096;      // classes whose exps are staged in LDS (32 KB)

__global__ void head_feat_kernel(const int32_t *gap, int n_elems, double denom, double *feat)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_elems) feat[i] = (double)gap[i] / denom;
}

// The three matrix products of the head, each output one sequential fma chain in ascending reduction index
// (the order is part of the head's definition):
//     out(i,j) = init(j) + sum_k A(i,k) * B(j,k),    A(i,k) = A[i*sAi + k*sAk],  B(j,k) = B[j*sBj + k*sBk]
//   logits : i = sample, j = class,   k = feature          init = bias
//   dfeat  : i = sample, j = feature, k = class            out -> float(a / HW)
//   update : i = class,  j = feature, k = sample           W(i,j) -= lr * a
// A workgroup owns 32 x 32 outputs (2 x 2 per thread: four independent chains hide the fma latency) and walks
// the reduction in chunks of 32 staged in LDS; the next chunk is fetched into registers while the current one
// is multiplied, and every operand is fetched from memory once per 32 outputs instead of once per output.
enum { HEAD_LOGITS = 0, HEAD_DFEAT = 1, HEAD_UPDATE = 2 };
constexpr int HG_T = 32, HG_KC = 32, HG_LD = HG_KC + 2;

struct HeadGemm {
    int I, J, K;
    const double *A, *B;
    long sAi, sAk, sBj, sBk;
    int a_kfast, b_kfast;        // which index is contiguous in memory (decides the loader's thread mapping)
    const double *init;          // HEAD_LOGITS: bias
    double *out;                 // HEAD_LOGITS: logits; HEAD_UPDATE: W (in place)
    float *outf;                 // HEAD_DFEAT
    long so;                     // row stride of the output
    double denom;                // HEAD_DFEAT: HW
    const int32_t *lr_slot;      // HEAD_UPDATE
};

template <int EPI>
__global__ __launch_bounds__(256) void head_gemm_kernel(HeadGemm g)
{
    __shared__ __attribute__((aligned(16))) double sa[HG_T][HG_LD], sb[HG_T][HG_LD];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int i0 = blockIdx.y * HG_T, j0 = blockIdx.x * HG_T;
    // loader: 4 elements of each operand per thread and chunk
    int la_r[4], la_k[4], lb_r[4], lb_k[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int e = tid + 256 * r;
        la_r[r] = g.a_kfast ? e >> 5 : e & 31; la_k[r] = g.a_kfast ? e & 31 : e >> 5;
        lb_r[r] = g.b_kfast ? e >> 5 : e & 31; lb_k[r] = g.b_kfast ? e & 31 : e >> 5;
    }
    double ra[4], rb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ia = i0 + la_r[r], ka = k0 + la_k[r], jb = j0 + lb_r[r], kb = k0 + lb_k[r];
            ra[r] = (ia < g.I && ka < g.K) ? g.A[ia * g.sAi + ka * g.sAk] : 0.0;
            rb[r] = (jb < g.J && kb < g.K) ? g.B[jb * g.sBj + kb * g.sBk] : 0.0;
        }
    };
    double a00 = 0.0, a01 = 0.0, a10 = 0.0, a11 = 0.0;
    if (EPI == HEAD_LOGITS) {
        a00 = a10 = (j0 + tx < g.J) ? g.init[j0 + tx] : 0.0;
        a01 = a11 = (j0 + tx + 16 < g.J) ? g.init[j0 + tx + 16] : 0.0;
    }
    fetch(0);
    for (int k0 = 0; k0 < g.K; k0 += HG_KC) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            sa[la_r[r]][la_k[r]] = ra[r];
            sb[lb_r[r]][lb_k[r]] = rb[r];
        }
        __syncthreads();
        if (k0 + HG_KC < g.K) fetch(k0 + HG_KC);
        const int kmax = g.K - k0 < HG_KC ? g.K - k0 : HG_KC;      // the chains never see a padded term
        if (kmax == HG_KC) {
#pragma unroll
            for (int k = 0; k < HG_KC; ++k) {
                const double x0 = sa[ty][k], x1 = sa[ty + 16][k], y0 = sb[tx][k], y1 = sb[tx + 16][k];
                a00 = fma(x0, y0, a00); a01 = fma(x0, y1, a01);
                a10 = fma(x1, y0, a10); a11 = fma(x1, y1, a11);
            }
        } else {
            for (int k = 0; k < kmax; ++k) {
                const double x0 = sa[ty][k], x1 = sa[ty + 16][k], y0 = sb[tx][k], y1 = sb[tx + 16][k];
                a00 = fma(x0, y0, a00); a01 = fma(x0, y1, a01);
                a10 = fma(x1, y0, a10); a11 = fma(x1, y1, a11);
            }
        }
        __syncthreads();
    }
    double lr = 0.0;
    if (EPI == HEAD_UPDATE) lr = ldexp((double)g.lr_slot[0], -g.lr_slot[1]);
    auto finish = [&](int i, int j, double a) {
        if (i >= g.I || j >= g.J) return;
        const long o = i * g.so + j;
        if (EPI == HEAD_LOGITS) g.out[o] = a;
        else if (EPI == HEAD_DFEAT) g.outf[o] = (float)(a / g.denom);
        else {
            const double step = lr * a;
            g.out[o] = g.out[o] - step;
        }
    };
    finish(i0 + ty, j0 + tx, a00);
    finish(i0 + ty, j0 + tx + 16, a01);
    finish(i0 + ty + 16, j0 + tx, a10);
    finish(i0 + ty + 16, j0 + tx + 16, a11);
}

// per sample (one block): softmax with max subtraction, loss term, dlogits.  The exps are evaluated in
// parallel, the denominator is then summed by one thread in ascending class order (the order is part of
// the head's definition), and the division / one-hot subtraction is parallel again.
__global__ void head_softmax_kernel(int N, int J, const double *logits, const int32_t *labels, double *dl,
                                    double *lossn)
{
    extern __shared__ double s_exp[];          // J doubles when they fit, else the exps stay in global memory
    __shared__ double red[256];
    __shared__ double s_sum;
    const bool staged = J <= HEAD_SOFTMAX_LDS;
    const int n = blockIdx.x;
    const double *lg = logits + (size_t)n * J;
    double *o = dl + (size_t)n * J;
    double *ex = staged ? s_exp : o;
    double m = -1.0e300;
    for (int j = threadIdx.x; j < J; j += blockDim.x) m = lg[j] > m ? lg[j] : m;
    red[threadIdx.x] = m;
    __syncthreads();
    for (int w = blockDim.x / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] = red[threadIdx.x + w] > red[threadIdx.x] ? red[threadIdx.x + w] : red[threadIdx.x];
        __syncthreads();
    }
    m = red[0];
    for (int j = threadIdx.x; j < J; j += blockDim.x) ex[j] = head_exp(lg[j] - m);
    __syncthreads();
    const int lab = labels[n];
    if (threadIdx.x == 0) {
        double sum = 0.0;
        int j = 0;
        for (; j + 8 <= J; j += 8) {           // loads first, then the additions in ascending order
            double v[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = ex[j + t];
#pragma unroll
            for (int t = 0; t < 8; ++t) sum = sum + v[t];
        }
        for (; j < J; ++j) sum = sum + ex[j];
        s_sum = sum;
        lossn[n] = log(sum) - (lg[lab] - m);
    }
    __syncthreads();
    const double sum = s_sum;
    for (int j = threadIdx.x; j < J; j += blockDim.x) {
        const double pj = ex[j] / sum;
        o[j] = (pj - (j == lab ? 1.0 : 0.0)) / (double)N;
    }
}

__global__ void head_loss_kernel(int N, const double *lossn, double *loss)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        double s = 0.0;
        for (int n = 0; n < N; ++n) s = s + lossn[n];
        *loss = s / (double)N;
    }
}

// b[j] -= lr * sum_n dl[n][j] (ascending n)
__global__ void head_bias_update_kernel(int N, int J, const double *dl, double *b, const int32_t *lr_slot)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= J) return;
    const double lr = ldexp((double)lr_slot[0], -lr_slot[1]);
    double s = 0.0;
    for (int n = 0; n < N; ++n) s = s + dl[(size_t)n * J + j];
    const double sb = lr * s;
    b[j] = b[j] - sb;
}

inline unsigned grid_for(size_t total)
{
    size_t b = (total + 255) / 256;
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    return (unsigned)b;
}

} // namespace

extern "C" int eoq_maxpool_fwd(eoq_ctx *c, const int8_t *a, int32_t N, int32_t H, int32_t W, int32_t C, int32_t R,
                               int32_t S, int32_t stride, int32_t pad, int8_t *y, const int32_t *b_next_pre,
                               int8_t *u_next, uint8_t *arg)
{
    if (!c || !a || N <= 0 || H <= 0 || W <= 0 || C <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return EOQ_ERR_ARG;
    if (C % 16 || pad >= R || pad >= S) return EOQ_ERR_SHAPE;
    if (((uintptr_t)a | (uintptr_t)y | (uintptr_t)u_next | (uintptr_t)arg) & 15) return EOQ_ERR_ARG;
    if (R * S > 255) return EOQ_ERR_SHAPE;
    PoolGeom g{N, H, W, C, R, S, stride, pad, conv_out_dim(H, pad, R, stride), conv_out_dim(W, pad, S, stride)};
    if (g.P <= 0 || g.Q <= 0) return EOQ_ERR_SHAPE;
    hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(grid_for((size_t)N * g.P * g.Q * (C / 16))), dim3(256), 0, c->stream,
                       g, a, y, b_next_pre, u_next, arg);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_maxpool_bwd(eoq_ctx *c, const uint8_t *arg, const int8_t *e, int32_t N, int32_t H, int32_t W,
                               int32_t C, int32_t R, int32_t S, int32_t stride, int32_t pad, int32_t *d,
                               int32_t *absmax_slot)
{
    if (!c || !arg || !e || !d || !absmax_slot || N <= 0 || H <= 0 || W <= 0 || C <= 0 || R <= 0 || S <= 0 ||
        stride <= 0 || pad < 0)
        return EOQ_ERR_ARG;
    if (C % 16 || pad >= R || pad >= S) return EOQ_ERR_SHAPE;
    if (((uintptr_t)arg | (uintptr_t)e | (uintptr_t)d) & 15) return EOQ_ERR_ARG;
    PoolGeom g{N, H, W, C, R, S, stride, pad, conv_out_dim(H, pad, R, stride), conv_out_dim(W, pad, S, stride)};
    if (g.P <= 0 || g.Q <= 0) return EOQ_ERR_SHAPE;
    hipLaunchKernelGGL(maxpool_bwd_kernel<0>, dim3(grid_for((size_t)N * H * W * (C / 16))), dim3(256), 0, c->stream, g,
                       arg, e, d, absmax_slot, (int8_t *)nullptr, (const int32_t *)nullptr, (int32_t *)nullptr,
                       (const uint16_t *)nullptr, (int64_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr,
                       (int64_t *)nullptr, (int32_t *)nullptr);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_maxpool_bwd_sq(eoq_ctx *c, const uint8_t *arg, const int8_t *e, int32_t N, int32_t H, int32_t W,
                                  int32_t C, int32_t R, int32_t S, int32_t stride, int32_t pad, int8_t *e_out,
                                  int32_t *absmax_slot, const int32_t *exp_in, int32_t *exp_out,
                                  const uint32_t *mask_bits, int64_t *sum_out, int32_t *spec_state)
{
    if (!c || !arg || !e || !e_out || !absmax_slot || !exp_in || !exp_out || N <= 0 || H <= 0 || W <= 0 || C <= 0 ||
        R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return EOQ_ERR_ARG;
    if (C % 16 || pad >= R || pad >= S) return EOQ_ERR_SHAPE;
    if (((uintptr_t)arg | (uintptr_t)e | (uintptr_t)e_out) & 15 || ((uintptr_t)mask_bits & 3)) return EOQ_ERR_ARG;
    PoolGeom g{N, H, W, C, R, S, stride, pad, conv_out_dim(H, pad, R, stride), conv_out_dim(W, pad, S, stride)};
    if (g.P <= 0 || g.Q <= 0) return EOQ_ERR_SHAPE;
    const uint16_t *mask16 = (const uint16_t *)mask_bits;
    const dim3 grid(grid_for((size_t)N * H * W * (C / 16)));
    if (spec_state) {
        int32_t *used = c->d_scratch + EOQ_SLOT_SPEC_USED;
        int64_t *tmp = (int64_t *)(c->d_scratch + EOQ_SLOT_POOL_TMP);   // zero between calls (context creation; OUT 4 resets it)
        int32_t *cnt = c->d_scratch + EOQ_SLOT_SPEC_HITS;
        hipLaunchKernelGGL(maxpool_bwd_kernel<3>, grid, dim3(256), 0, c->stream, g, arg, e, (int32_t *)nullptr, absmax_slot,
                           e_out, exp_in, exp_out, mask16, sum_out, spec_state, used, tmp, cnt);
        hipLaunchKernelGGL(maxpool_bwd_kernel<4>, grid, dim3(256), 0, c->stream, g, arg, e, (int32_t *)nullptr, absmax_slot,
                           e_out, exp_in, exp_out, mask16, sum_out, spec_state, used, tmp, cnt);
        EOQ_LAUNCH_CHECK();
        return EOQ_OK;
    }
    if (R == 3 && S == 3 && stride == 2 && pad == 1) {
        // the abs-max pass gains from fetching each window once per 2x2 block of pixels; the coding pass does not:
        // its stores want consecutive lanes on consecutive pixels
        const dim3 grid2(grid_for((size_t)N * ((H + 1) / 2) * ((W + 1) / 2) * (C / 16)));
        hipLaunchKernelGGL(maxpool_bwd_3s2_kernel<1>, grid2, dim3(256), 0, c->stream, g, arg, e, absmax_slot,
                           (int8_t *)nullptr, (const int32_t *)nullptr, (int32_t *)nullptr, (const uint16_t *)nullptr,
                           (int64_t *)nullptr);
    } else {
        hipLaunchKernelGGL(maxpool_bwd_kernel<1>, grid, dim3(256), 0, c->stream, g, arg, e, (int32_t *)nullptr,
                           absmax_slot, (int8_t *)nullptr, (const int32_t *)nullptr, (int32_t *)nullptr,
                           (const uint16_t *)nullptr, (int64_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr,
                           (int64_t *)nullptr, (int32_t *)nullptr);
    }
    hipLaunchKernelGGL(maxpool_bwd_kernel<2>, grid, dim3(256), 0, c->stream, g, arg, e, (int32_t *)nullptr, absmax_slot,
                       e_out, exp_in, exp_out, mask16, sum_out, (int32_t *)nullptr, (int32_t *)nullptr,
                       (int64_t *)nullptr, (int32_t *)nullptr);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_gap_sum(eoq_ctx *c, const int8_t *y, int32_t N, int32_t HW, int32_t C, int32_t *sum)
{
    if (!c || !y || !sum || N <= 0 || HW <= 0 || C <= 0 || ((uintptr_t)y & 15)) return EOQ_ERR_ARG;
    if (C % 16) return EOQ_ERR_SHAPE;
    hipLaunchKernelGGL(gap_sum_kernel, dim3(grid_for((size_t)N * (C / 16))), dim3(256), 0, c->stream, y, N, HW, C, sum);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_broadcast_hw(eoq_ctx *c, const int8_t *codes, int32_t N, int32_t HW, int32_t C, int8_t *e)
{
    if (!c || !codes || !e || N <= 0 || HW <= 0 || C <= 0 || (((uintptr_t)codes | (uintptr_t)e) & 15))
        return EOQ_ERR_ARG;
    if (C % 16) return EOQ_ERR_SHAPE;
    hipLaunchKernelGGL(broadcast_hw_kernel, dim3(grid_for((size_t)N * HW * (C / 16))), dim3(256), 0, c->stream, codes,
                       N, HW, C, e);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" size_t eoq_head_workspace_bytes(int32_t N, int32_t F, int32_t J)
{
    if (N <= 0 || F <= 0 || J <= 0) return 0;
    return sizeof(double) * ((size_t)N * F + (size_t)N * J + (size_t)N + 2);
}

extern "C" int eoq_head_fwd_bwd(eoq_ctx *c, int32_t N, int32_t F, int32_t J, int32_t HW, const int32_t *gap_sum,
                                double *Wfc, double *bfc, const int32_t *labels, const int32_t *lr_slot, double *loss,
                                float *d, double *logits, void *ws, size_t ws_bytes)
{
    if (!c || N <= 0 || F <= 0 || J <= 0 || HW <= 0 || !gap_sum || !Wfc || !bfc || !labels || !loss || !d || !logits)
        return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_head_workspace_bytes(N, F, J) || ((uintptr_t)ws & 7)) return EOQ_ERR_WORKSPACE;
    double *feat = (double *)ws;
    double *dl = feat + (size_t)N * F;
    double *lossn = dl + (size_t)N * J;
    hipStream_t s = c->stream;
    hipLaunchKernelGGL(head_feat_kernel, dim3((N * F + 255) / 256), dim3(256), 0, s, gap_sum, N * F,
                       128.0 * (double)HW, feat);
    const dim3 blk(256);
    auto tiles = [](int v) { return (unsigned)((v + HG_T - 1) / HG_T); };
    HeadGemm lg{};
    lg.I = N; lg.J = J; lg.K = F; lg.A = feat; lg.sAi = F; lg.sAk = 1; lg.B = Wfc; lg.sBj = F; lg.sBk = 1;
    lg.a_kfast = 1; lg.b_kfast = 1; lg.init = bfc; lg.out = logits; lg.so = J;
    hipLaunchKernelGGL(head_gemm_kernel<HEAD_LOGITS>, dim3(tiles(J), tiles(N)), blk, 0, s, lg);
    const size_t sm_bytes = J <= HEAD_SOFTMAX_LDS ? sizeof(double) * (size_t)J : 0;
    hipLaunchKernelGGL(head_softmax_kernel, dim3(N), dim3(256), sm_bytes, s, N, J, logits, labels, dl, lossn);
    hipLaunchKernelGGL(head_loss_kernel, dim3(1), dim3(64), 0, s, N, lossn, loss);
    HeadGemm df{};
    df.I = N; df.J = F; df.K = J; df.A = dl; df.sAi = J; df.sAk = 1; df.B = Wfc; df.sBj = 1; df.sBk = F;
    df.a_kfast = 1; df.b_kfast = 0; df.outf = d; df.so = F; df.denom = (double)HW;
    hipLaunchKernelGGL(head_gemm_kernel<HEAD_DFEAT>, dim3(tiles(F), tiles(N)), blk, 0, s, df);
    EOQ_LAUNCH_CHECK();
    // lr_slot == NULL: the classifier's own update is left to a later eoq_head_update on the same workspace
    return lr_slot ? eoq_head_update(c, N, F, J, Wfc, bfc, lr_slot, ws, ws_bytes) : EOQ_OK;
}

extern "C" int eoq_head_update(eoq_ctx *c, int32_t N, int32_t F, int32_t J, double *Wfc, double *bfc,
                               const int32_t *lr_slot, const void *ws, size_t ws_bytes)
{
    if (!c || N <= 0 || F <= 0 || J <= 0 || !Wfc || !bfc || !lr_slot) return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_head_workspace_bytes(N, F, J) || ((uintptr_t)ws & 7)) return EOQ_ERR_WORKSPACE;
    const double *feat = (const double *)ws;
    const double *dl = feat + (size_t)N * F;
    auto tiles = [](int v) { return (unsigned)((v + HG_T - 1) / HG_T); };
    HeadGemm up{};
    up.I = J; up.J = F; up.K = N; up.A = dl; up.sAi = 1; up.sAk = J; up.B = feat; up.sBj = 1; up.sBk = F;
    up.a_kfast = 0; up.b_kfast = 0; up.out = Wfc; up.so = F; up.lr_slot = lr_slot;
    hipLaunchKernelGGL(head_gemm_kernel<HEAD_UPDATE>, dim3(tiles(F), tiles(J)), dim3(256), 0, c->stream, up);
    hipLaunchKernelGGL(head_bias_update_kernel, dim3((J + 255) / 256), dim3(256), 0, c->stream, N, J, dl, bfc, lr_slot);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}
