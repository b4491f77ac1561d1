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
__global__ void maxpool_bwd_kernel(PoolGeom g, const uint8_t *arg, const int8_t *e, int32_t *d, int32_t *absmax)
{
    const int c16 = g.C / 16;
    const size_t total = (size_t)g.N * g.H * g.W * c16;
    int mx = 0;
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
            for (int q = q_lo; q <= q_hi; ++q) {
                const int my = (h - (p * g.stride - g.pad)) * g.S + (x - (q * g.stride - g.pad));
                const size_t o = (((size_t)n * g.P + p) * g.Q + q) * g.C + cc * 16;
                v4i av = *(const v4i *)(arg + o), ev = *(const v4i *)(e + o);
#pragma unroll
                for (int k = 0; k < 16; ++k)
                    if ((byte_at(av, k) & 0xff) == my) acc[k] += byte_at(ev, k);
            }
        int32_t *o = d + pix * g.C + cc * 16;
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
            v4i w = {acc[4 * k4], acc[4 * k4 + 1], acc[4 * k4 + 2], acc[4 * k4 + 3]};
            ((v4i *)o)[k4] = w;
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            int av = acc[k] < 0 ? -acc[k] : acc[k];
            mx = av > mx ? av : mx;
        }
    }
    block_atomic_max_i32(mx, absmax);
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

__global__ void head_feat_kernel(const int32_t *gap, int n_elems, double denom, double *feat)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_elems) feat[i] = (double)gap[i] / denom;
}

// logits[n][j] = b[j] + sum_k feat[n][k] W[j][k], one sequential fma chain per (n,j); tiles of
// 16 x 16 outputs share their operands through LDS.
__global__ void head_logits_kernel(int N, int F, int J, const double *feat, const double *W, const double *b,
                                   double *logits)
{
    __shared__ double sf[16][33], sw[16][33];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n = blockIdx.y * 16 + ty, j = blockIdx.x * 16 + tx;
    double a = (j < J) ? b[j] : 0.0;
    for (int k0 = 0; k0 < F; k0 += 32) {
        for (int t = threadIdx.x; t < 16 * 32; t += 256) {
            int row = t >> 5, col = t & 31;
            int nn = blockIdx.y * 16 + row, jj = blockIdx.x * 16 + row;
            sf[row][col] = (nn < N && k0 + col < F) ? feat[(size_t)nn * F + k0 + col] : 0.0;
            sw[row][col] = (jj < J && k0 + col < F) ? W[(size_t)jj * F + k0 + col] : 0.0;
        }
        __syncthreads();
        const int kmax = F - k0 < 32 ? F - k0 : 32;
        for (int k = 0; k < kmax; ++k) a = fma(sf[ty][k], sw[tx][k], a);
        __syncthreads();
    }
    if (n < N && j < J) logits[(size_t)n * J + j] = a;
}

// per sample (one block): softmax with max subtraction, loss term, dlogits.  The exps are evaluated in
// parallel, the denominator is then summed by one thread in ascending class order (the order is part of
// the head's definition), and the division / one-hot subtraction is parallel again.
__global__ void head_softmax_kernel(int N, int J, const double *logits, const int32_t *labels, double *dl,
                                    double *lossn)
{
    __shared__ double red[256];
    __shared__ double s_sum;
    const int n = blockIdx.x;
    const double *lg = logits + (size_t)n * J;
    double *o = dl + (size_t)n * J;
    double m = -1.0e300;
    for (int j = threadIdx.x; j < J; j += blockDim.x) m = lg[j] > m ? lg[j] : m;
    red[threadIdx.x] = m;
    __syncthreads();
    for (int w = blockDim.x / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] = red[threadIdx.x + w] > red[threadIdx.x] ? red[threadIdx.x + w] : red[threadIdx.x];
        __syncthreads();
    }
    m = red[0];
    for (int j = threadIdx.x; j < J; j += blockDim.x) o[j] = head_exp(lg[j] - m);
    __syncthreads();
    const int lab = labels[n];
    if (threadIdx.x == 0) {
        double sum = 0.0;
        for (int j = 0; j < J; ++j) sum = sum + o[j];
        s_sum = sum;
        lossn[n] = log(sum) - (lg[lab] - m);
    }
    __syncthreads();
    const double sum = s_sum;
    for (int j = threadIdx.x; j < J; j += blockDim.x) {
        const double pj = o[j] / sum;
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

// d[n][k] = (float)((sum_j dl[n][j] W[j][k]) / HW), ascending j
__global__ void head_dfeat_kernel(int N, int F, int J, int HW, const double *dl, const double *W, float *d)
{
    int k = blockIdx.x * blockDim.x + threadIdx.x, n = blockIdx.y;
    if (k >= F) return;
    double a = 0.0;
    for (int j = 0; j < J; ++j) a = fma(dl[(size_t)n * J + j], W[(size_t)j * F + k], a);
    d[(size_t)n * F + k] = (float)(a / (double)HW);
}

// dW[j][k] = sum_n dl[n][j] feat[n][k] (ascending n), W -= lr dW; the k == 0 lane also does the bias
__global__ void head_update_kernel(int N, int F, int J, const double *dl, const double *feat, double *W, double *b,
                                   const int32_t *lr_slot)
{
    int k = blockIdx.x * blockDim.x + threadIdx.x, j = blockIdx.y;
    if (k >= F) return;
    const double lr = ldexp((double)lr_slot[0], -lr_slot[1]);
    double a = 0.0;
    for (int n = 0; n < N; ++n) a = fma(dl[(size_t)n * J + j], feat[(size_t)n * F + k], a);
    const double step = lr * a;
    W[(size_t)j * F + k] = W[(size_t)j * F + k] - step;
    if (k == 0) {
        double s = 0.0;
        for (int n = 0; n < N; ++n) s = s + dl[(size_t)n * J + j];
        const double sb = lr * s;
        b[j] = b[j] - sb;
    }
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
    hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(grid_for((size_t)N * H * W * (C / 16))), dim3(256), 0, c->stream, g, arg,
                       e, d, absmax_slot);
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
    if (!c || N <= 0 || F <= 0 || J <= 0 || HW <= 0 || !gap_sum || !Wfc || !bfc || !labels || !lr_slot || !loss ||
        !d || !logits)
        return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_head_workspace_bytes(N, F, J) || ((uintptr_t)ws & 7)) return EOQ_ERR_WORKSPACE;
    double *feat = (double *)ws;
    double *dl = feat + (size_t)N * F;
    double *lossn = dl + (size_t)N * J;
    hipStream_t s = c->stream;
    hipLaunchKernelGGL(head_feat_kernel, dim3((N * F + 255) / 256), dim3(256), 0, s, gap_sum, N * F,
                       128.0 * (double)HW, feat);
    hipLaunchKernelGGL(head_logits_kernel, dim3((J + 15) / 16, (N + 15) / 16), dim3(256), 0, s, N, F, J, feat, Wfc,
                       bfc, logits);
    hipLaunchKernelGGL(head_softmax_kernel, dim3(N), dim3(256), 0, s, N, J, logits, labels, dl, lossn);
    hipLaunchKernelGGL(head_loss_kernel, dim3(1), dim3(64), 0, s, N, lossn, loss);
    hipLaunchKernelGGL(head_dfeat_kernel, dim3((F + 255) / 256, N), dim3(256), 0, s, N, F, J, HW, dl, Wfc, d);
    hipLaunchKernelGGL(head_update_kernel, dim3((F + 255) / 256, J), dim3(256), 0, s, N, F, J, dl, feat, Wfc, bfc,
                       lr_slot);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}
