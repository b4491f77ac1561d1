// Implicit-GEMM int8 x int8 -> int32 convolution on MFMA for gfx950: the forward convolution of
// Eq.2 with its fused epilogue (Q_a1, multiplier, bias, shortcut, ReLU, Q_a2 -- Eq.9, Eq.10), and the
// backward-data convolution of Eq.3 (same kernel, gathering the error through the transposed
// filters) with the abs-max that the scale quantiser Q_e (Eq.11) needs fused into its epilogue.
//
// GEMM view: rows m = output pixels (N*P*Q), columns = output channels, reduction = (r, s, c).
// The reduction is walked in 16-byte pieces ("k-chunks": 16 consecutive input channels of one filter
// tap), four per LDS stage.  One MFMA v_mfma_i32_32x32x32_i8 consumes two k-chunks: lanes 0-31 supply
// the first, lanes 32-63 the second, identically for both operands, so any (tap, channel) order is
// legal as long as A and B agree.  A workgroup is 4 waves; each wave owns a (BM/WGM) x (BN/WGN) block
// of 32x32 MFMA tiles.  Global -> register -> LDS software pipeline with two LDS buffers, one
// barrier per stage; LDS rows are 64 bytes with the 16-byte chunk index XOR-swizzled by (row/4)%4 so
// that both the 16-byte writes and the MFMA operand reads spread over all banks.
//
// Epilogue: each wave transposes its accumulators through LDS so that one lane owns 16 consecutive
// output channels of one pixel (16-byte int8 stores, 16-bit mask stores, 64-byte int32 stores).
#include "common.h"

namespace {

struct EpiDev {
    const int32_t *gamma, *b_post, *b_next;
    const void *skip;
    int skip_wide, relu;
    int8_t *y, *u_next;
    uint16_t *mask16;
    int32_t *t_wide;
};

struct IgemmParams {
    const int8_t *A;   // input N x H x W x C
    const int8_t *B;   // filters NOUT x (R*S*C)
    int N, H, W, C;
    int P, Q, NOUT;
    int R, S, stride, pad;
    int M, nk16, c16;
    int32_t *acc_out;
    int32_t *absmax;
    EpiDev ep;
};

enum { MODE_FWD = 0, MODE_BWD_DATA = 1 };
enum { EPI_FWD = 0, EPI_ACC = 1 };

__device__ __forceinline__ void set_byte(v4i &v, int i, int code)
{
    uint32_t sh = 8 * (i & 3);
    v[i >> 2] = (int)(((uint32_t)v[i >> 2] & ~(0xffu << sh)) | (((uint32_t)code & 0xffu) << sh));
}
__device__ __forceinline__ int byte_at(const v4i &v, int i)
{
    return (int)(int8_t)((uint32_t)v[i >> 2] >> (8 * (i & 3)));
}

// Forward epilogue for 16 consecutive channels of one pixel (Eq.2 x2..x5 and the next layer's x1).
// off = linear NPQK element offset of the first channel (a multiple of 16).
__device__ __forceinline__ void epilogue16(const int acc[16], size_t off, const EpiDev &ep, int32_t *acc_out,
                                           int gamma, int bpost, int bnext)
{
    if (acc_out) {
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
            v4i w = {acc[4 * k4], acc[4 * k4 + 1], acc[4 * k4 + 2], acc[4 * k4 + 3]};
            ((v4i *)(acc_out + off))[k4] = w;
        }
    }
    int t[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) t[k] = rne_shift7(acc[k]);
    if (ep.t_wide) {
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
            v4i w = {t[4 * k4], t[4 * k4 + 1], t[4 * k4 + 2], t[4 * k4 + 3]};
            ((v4i *)(ep.t_wide + off))[k4] = w;
        }
    }
    if (!ep.relu) return;
    int sk[16];
    if (ep.skip) {
        if (ep.skip_wide) {
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                v4i w = ((const v4i *)((const int32_t *)ep.skip + off))[k4];
                sk[4 * k4] = w[0]; sk[4 * k4 + 1] = w[1]; sk[4 * k4 + 2] = w[2]; sk[4 * k4 + 3] = w[3];
            }
        } else {
            v4i w = *(const v4i *)((const int8_t *)ep.skip + off);
#pragma unroll
            for (int k = 0; k < 16; ++k) sk[k] = byte_at(w, k);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) sk[k] = 0;
    }
    v4i yv = {0, 0, 0, 0}, uv = {0, 0, 0, 0};
    uint32_t mask = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        int64_t z = (int64_t)gamma * (int64_t)t[k] + 128 * ((int64_t)bpost + (int64_t)sk[k]);
        mask |= (z > 0 ? 1u : 0u) << k;
        int64_t yy = rne_shift64(z > 0 ? z : 0, 7);
        int yc = (int)(yy > CODE_MAX ? CODE_MAX : yy);
        set_byte(yv, k, yc);
        set_byte(uv, k, clamp_i(yc + bnext, -CODE_MAX, CODE_MAX));
    }
    if (ep.y) *(v4i *)(ep.y + off) = yv;
    if (ep.u_next) *(v4i *)(ep.u_next + off) = uv;
    if (ep.mask16) ep.mask16[off >> 4] = (uint16_t)mask;
}

template <int BM, int BN, int WGM, int WGN, int MODE, int EPI>
__global__ __launch_bounds__(256) void igemm_kernel(IgemmParams p)
{
    static_assert(WGM * WGN == 4, "4 waves");
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(TM >= 1 && TN >= 1, "tile");
    constexpr int A_ROWS = (BM + 63) / 64, B_ROWS = (BN + 63) / 64;
    constexpr int STAGE_BYTES = (BM + BN) * 64;
    constexpr int EPI_LD = WTN + 4;                       // int32 row stride of the epilogue staging

    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int tiles_n = (p.NOUT + BN - 1) / BN;
    const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- per-thread gather state: which rows / which k-chunk column this thread loads ----
    const int kc = tid & 3, lrow = tid >> 2;
    size_t a_base[A_ROWS];
    int a_h0[A_ROWS], a_w0[A_ROWS];
    bool a_ok[A_ROWS];
#pragma unroll
    for (int i = 0; i < A_ROWS; ++i) {
        int row = lrow + 64 * i;
        int m = m0 + row;
        a_ok[i] = (row < BM) && (m < p.M);
        int mm = a_ok[i] ? m : 0;
        int wo = mm % p.Q;
        int t = mm / p.Q;
        int ho = t % p.P, n = t / p.P;
        a_base[i] = (size_t)n * p.H * p.W * p.C;
        if (MODE == MODE_FWD) { a_h0[i] = ho * p.stride - p.pad; a_w0[i] = wo * p.stride - p.pad; }
        else { a_h0[i] = ho + p.pad; a_w0[i] = wo + p.pad; }
    }
    // tap / channel position of this thread's k-chunk
    int kk = kc, r = 0, s = 0, cc = kc;
    while (cc >= p.c16) { cc -= p.c16; if (++s == p.S) { s = 0; ++r; } }

    v4i ra[A_ROWS], rb[B_ROWS];
    auto load_stage = [&]() {
        const bool tap_ok = kk < p.nk16;
#pragma unroll
        for (int i = 0; i < A_ROWS; ++i) {
            bool v = a_ok[i] && tap_ok;
            int hin, win;
            if (MODE == MODE_FWD) { hin = a_h0[i] + r; win = a_w0[i] + s; }
            else {
                int th = a_h0[i] - r, tw = a_w0[i] - s;
                if (p.stride == 1) { hin = th; win = tw; }
                else {
                    v = v && th >= 0 && tw >= 0 && (th % p.stride == 0) && (tw % p.stride == 0);
                    hin = th / p.stride; win = tw / p.stride;
                }
            }
            v = v && (unsigned)hin < (unsigned)p.H && (unsigned)win < (unsigned)p.W;
            v4i z = {0, 0, 0, 0};
            ra[i] = v ? *(const v4i *)(p.A + a_base[i] + ((size_t)hin * p.W + win) * p.C + cc * 16) : z;
        }
#pragma unroll
        for (int i = 0; i < B_ROWS; ++i) {
            int row = lrow + 64 * i;
            int nr = n0 + row;
            bool v = tap_ok && row < BN && nr < p.NOUT;
            v4i z = {0, 0, 0, 0};
            rb[i] = v ? *(const v4i *)(p.B + ((size_t)nr * p.nk16 + kk) * 16) : z;
        }
        kk += 4;
        cc += 4;
        while (cc >= p.c16) { cc -= p.c16; if (++s == p.S) { s = 0; ++r; } }
    };
    auto store_stage = [&](int buf) {
        int8_t *As = lds + buf * STAGE_BYTES, *Bs = As + BM * 64;
#pragma unroll
        for (int i = 0; i < A_ROWS; ++i) {
            int row = lrow + 64 * i;
            if (row < BM) *(v4i *)(As + row * 64 + ((kc ^ ((row >> 2) & 3)) << 4)) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_ROWS; ++i) {
            int row = lrow + 64 * i;
            if (row < BN) *(v4i *)(Bs + row * 64 + ((kc ^ ((row >> 2) & 3)) << 4)) = rb[i];
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    const int nstages = (p.nk16 + 3) / 4;
    load_stage();
    store_stage(0);
    __syncthreads();
    const int lrow32 = lane & 31, lhalf = lane >> 5;
    for (int st = 0; st < nstages; ++st) {
        const bool more = st + 1 < nstages;
        if (more) load_stage();
        const int8_t *As = lds + (st & 1) * STAGE_BYTES, *Bs = As + BM * 64;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int chunk = 2 * j + lhalf;
            v4i a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int row = wm * WTM + i * 32 + lrow32;
                a[i] = *(const v4i *)(As + row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4));
            }
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                int row = wn * WTN + i * 32 + lrow32;
                b[i] = *(const v4i *)(Bs + row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int jn = 0; jn < TN; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[jn], acc[i][jn], 0, 0, 0);
        }
        if (more) store_stage((st + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: per wave, 32 rows at a time through LDS ----
    int32_t *stg = (int32_t *)lds + wave * 32 * EPI_LD;
    constexpr int GROUPS = WTN / 16;              // 16-channel groups per row of the wave tile
    constexpr int ROWS_PER_PASS = 64 / GROUPS;
    const int grp = lane % GROUPS, prow = lane / GROUPS;
    int gamma = 128, bpost = 0, bnext = 0;
    if (EPI == EPI_FWD) {
        if (p.ep.gamma) gamma = *p.ep.gamma;
        if (p.ep.b_post) bpost = *p.ep.b_post;
        if (p.ep.b_next) bnext = *p.ep.b_next;
    }
    int mx = 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int row = (e >> 2) * 8 + lhalf * 4 + (e & 3);
                stg[row * EPI_LD + jn * 32 + lrow32] = acc[i][jn][e];
            }
        __syncthreads();   // (each wave reads back only what it wrote itself)
#pragma unroll
        for (int ps = 0; ps < 32 / ROWS_PER_PASS; ++ps) {
            const int row = ps * ROWS_PER_PASS + prow;
            const int m = m0 + wm * WTM + i * 32 + row;
            const int ch = n0 + wn * WTN + grp * 16;
            int v[16];
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                v4i w = *(const v4i *)(stg + row * EPI_LD + grp * 16 + 4 * k4);
                v[4 * k4] = w[0]; v[4 * k4 + 1] = w[1]; v[4 * k4 + 2] = w[2]; v[4 * k4 + 3] = w[3];
            }
            if (m < p.M && ch < p.NOUT) {
                const size_t off = (size_t)m * p.NOUT + ch;
                if (EPI == EPI_FWD) {
                    epilogue16(v, off, p.ep, p.acc_out, gamma, bpost, bnext);
                } else {
#pragma unroll
                    for (int k4 = 0; k4 < 4; ++k4) {
                        v4i w = {v[4 * k4], v[4 * k4 + 1], v[4 * k4 + 2], v[4 * k4 + 3]};
                        ((v4i *)(p.acc_out + off))[k4] = w;
                    }
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        int av = v[k] < 0 ? -v[k] : v[k];
                        mx = av > mx ? av : mx;
                    }
                }
            }
        }
        __syncthreads();
    }
    if (EPI == EPI_ACC && p.absmax) block_atomic_max_i32(mx, p.absmax);
}

// ---- small layout kernels -------------------------------------------------------------------
// filters K x R x S x C  ->  C x R x S x K (what the backward-data gather multiplies with)
__global__ void transpose_filters_kernel(const int8_t *w, int K, int RS, int C, int8_t *wt)
{
    size_t total = (size_t)K * RS * C;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        int k = (int)(i % K);
        size_t t = i / K;
        int rs = (int)(t % RS), c = (int)(t / RS);
        wt[i] = w[((size_t)k * RS + rs) * C + c];
    }
}

// explicit im2col for inputs whose channel count is not a multiple of 16: col[m][KP], zero padded
__global__ void im2col_kernel(const int8_t *u, int N, int H, int W, int C, int P, int Q, int R, int S, int stride,
                              int pad, int KP, int8_t *col)
{
    const int chunks = KP / 16;
    const size_t total = (size_t)N * P * Q * chunks;
    const int rsc = R * S * C;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        int ch = (int)(i % chunks);
        size_t m = i / chunks;
        int q = (int)(m % Q);
        size_t t = m / Q;
        int pp = (int)(t % P), n = (int)(t / P);
        v4i o = {0, 0, 0, 0};
#pragma unroll
        for (int b = 0; b < 16; ++b) {
            int j = ch * 16 + b;
            int val = 0;
            if (j < rsc) {
                int c = j % C, rs = j / C;
                int s = rs % S, r = rs / S;
                int h = pp * stride + r - pad, x = q * stride + s - pad;
                if ((unsigned)h < (unsigned)H && (unsigned)x < (unsigned)W)
                    val = u[(((size_t)n * H + h) * W + x) * C + c];
            }
            set_byte(o, b, val);
        }
        *(v4i *)(col + m * KP + ch * 16) = o;
    }
}

__global__ void pad_filters_kernel(const int8_t *w, int K, int rsc, int KP, int8_t *wp)
{
    size_t total = (size_t)K * KP;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        int j = (int)(i % KP);
        size_t k = i / KP;
        wp[i] = j < rsc ? w[k * rsc + j] : (int8_t)0;
    }
}

// standalone forward epilogue on stored accumulators
__global__ void requant_fwd_kernel(const int32_t *acc, size_t n16, EpiDev ep)
{
    const int gamma = ep.gamma ? *ep.gamma : 128, bpost = ep.b_post ? *ep.b_post : 0, bnext = ep.b_next ? *ep.b_next : 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
        int v[16];
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
            v4i w = ((const v4i *)acc)[i * 4 + k4];
            v[4 * k4] = w[0]; v[4 * k4 + 1] = w[1]; v[4 * k4 + 2] = w[2]; v[4 * k4 + 3] = w[3];
        }
        epilogue16(v, i * 16, ep, nullptr, gamma, bpost, bnext);
    }
}

inline unsigned grid_for(size_t total)
{
    size_t b = (total + 255) / 256;
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    return (unsigned)b;
}

template <int BM, int BN, int WGM, int WGN, int MODE, int EPI>
int launch_igemm(eoq_ctx *c, const IgemmParams &p)
{
    constexpr int main_bytes = 2 * (BM + BN) * 64, epi_bytes = 4 * 32 * (BN / WGN + 4) * 4;
    constexpr int lds_bytes = main_bytes > epi_bytes ? main_bytes : epi_bytes;
    static bool attr_done = false;
    auto kern = igemm_kernel<BM, BN, WGM, WGN, MODE, EPI>;
    if (lds_bytes > 48 * 1024 && !attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
            return EOQ_ERR_HIP;
        attr_done = true;
    }
    const long tiles = (long)((p.M + BM - 1) / BM) * ((p.NOUT + BN - 1) / BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(256), lds_bytes, c->stream, p);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

template <int MODE, int EPI>
int dispatch_igemm(eoq_ctx *c, const IgemmParams &p)
{
    // widest column tile the output channels fill, then the tallest row tile that still gives the
    // chip a few waves of workgroups
    const int nout = p.NOUT;
    auto wgs = [&](int bm, int bn) { return (long)((p.M + bm - 1) / bm) * ((nout + bn - 1) / bn); };
    if (nout <= 32) return launch_igemm<128, 32, 4, 1, MODE, EPI>(c, p);
    if (nout <= 64) {
        if (wgs(256, 64) >= 512) return launch_igemm<256, 64, 4, 1, MODE, EPI>(c, p);
        return launch_igemm<128, 64, 2, 2, MODE, EPI>(c, p);
    }
    if (nout % 256 == 0 && wgs(256, 256) >= 512) return launch_igemm<256, 256, 2, 2, MODE, EPI>(c, p);
    if (wgs(256, 128) >= 512) return launch_igemm<256, 128, 2, 2, MODE, EPI>(c, p);
    if (wgs(128, 128) >= 256) return launch_igemm<128, 128, 2, 2, MODE, EPI>(c, p);
    return launch_igemm<128, 64, 2, 2, MODE, EPI>(c, p);
}

bool desc_ok(const eoq_conv_desc *d)
{
    return d && d->N > 0 && d->H > 0 && d->W > 0 && d->C > 0 && d->K > 0 && d->R > 0 && d->S > 0 && d->stride > 0 &&
           d->pad >= 0 && conv_out_dim(d->H, d->pad, d->R, d->stride) > 0 &&
           conv_out_dim(d->W, d->pad, d->S, d->stride) > 0;
}

int fill_epi(const eoq_epilogue *e, EpiDev &o)
{
    o.gamma = e->gamma; o.b_post = e->b_post; o.b_next = e->b_next_pre; o.skip = e->skip;
    o.skip_wide = e->skip_is_wide; o.relu = e->relu; o.y = e->y; o.u_next = e->u_next;
    o.mask16 = (uint16_t *)e->relu_mask_bits; o.t_wide = e->t_wide;
    uintptr_t al = (uintptr_t)e->skip | (uintptr_t)e->y | (uintptr_t)e->u_next | (uintptr_t)e->t_wide;
    if ((al & 15) || ((uintptr_t)e->relu_mask_bits & 3)) return EOQ_ERR_ARG;
    if (!e->relu && !e->t_wide) return EOQ_ERR_ARG;
    return EOQ_OK;
}

} // namespace

// padded reduction length of the explicit im2col path
static inline int im2col_kp(const eoq_conv_desc *d) { return (int)round_up((size_t)d->R * d->S * d->C, 64); }

extern "C" size_t eoq_workspace_bytes(const eoq_conv_desc *d, int op)
{
    if (!desc_ok(d)) return 0;
    const size_t P = conv_out_dim(d->H, d->pad, d->R, d->stride), Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    const size_t M = (size_t)d->N * P * Q;
    const size_t wbytes = (size_t)d->K * d->R * d->S * d->C;
    size_t im2col = 0;
    if (d->C % 16) im2col = round_up(M * im2col_kp(d), 256) + round_up((size_t)d->K * im2col_kp(d), 256);
    switch (op) {
    case EOQ_OP_CONV_FWD: return im2col;
    case EOQ_OP_CONV_BWD_DATA: return round_up(wbytes, 256);
    case EOQ_OP_CONV_BWD_WEIGHT: {
        // split partial sums (int32) sized for the worst split count, see conv_wgrad.hip
        size_t kp = d->C % 16 ? (size_t)im2col_kp(d) : (size_t)d->R * d->S * d->C;
        return im2col + round_up((size_t)d->K * kp * 4 * 64, 256);
    }
    default: return 0;
    }
}

extern "C" int eoq_conv_fwd(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *u, const int8_t *w, int32_t *acc,
                            const eoq_epilogue *ep, void *ws, size_t ws_bytes)
{
    if (!c || !u || !w || (!acc && !ep)) return EOQ_ERR_ARG;
    if (!desc_ok(d)) return EOQ_ERR_SHAPE;
    if (d->K % 16) return EOQ_ERR_SHAPE;
    if (((uintptr_t)u | (uintptr_t)w | (uintptr_t)acc) & 15) return EOQ_ERR_ARG;
    IgemmParams p{};
    p.P = conv_out_dim(d->H, d->pad, d->R, d->stride);
    p.Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    if ((size_t)d->N * p.P * p.Q > 0x7fffffffu || (size_t)d->H * d->W * d->C > 0x7fffffffu) return EOQ_ERR_SHAPE;
    p.M = d->N * p.P * p.Q;
    p.NOUT = d->K;
    p.acc_out = acc;
    p.absmax = nullptr;
    if (ep) {
        if (int rc = fill_epi(ep, p.ep)) return rc;
    }
    if (d->C % 16 == 0) {
        p.A = u; p.B = w;
        p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C;
        p.R = d->R; p.S = d->S; p.stride = d->stride; p.pad = d->pad;
    } else {
        const int KP = im2col_kp(d);
        if (!ws || ws_bytes < eoq_workspace_bytes(d, EOQ_OP_CONV_FWD) || ((uintptr_t)ws & 15)) return EOQ_ERR_WORKSPACE;
        int8_t *col = (int8_t *)ws;
        int8_t *wp = col + round_up((size_t)p.M * KP, 256);
        hipLaunchKernelGGL(im2col_kernel, dim3(grid_for((size_t)p.M * (KP / 16))), dim3(256), 0, c->stream, u, d->N, d->H,
                           d->W, d->C, p.P, p.Q, d->R, d->S, d->stride, d->pad, KP, col);
        hipLaunchKernelGGL(pad_filters_kernel, dim3(grid_for((size_t)d->K * KP)), dim3(256), 0, c->stream, w, d->K,
                           d->R * d->S * d->C, KP, wp);
        EOQ_LAUNCH_CHECK();
        p.A = col; p.B = wp;
        p.N = 1; p.H = 1; p.W = p.M; p.C = KP;     // a 1x1 convolution over M "pixels"
        p.P = 1; p.Q = p.M;
        p.R = 1; p.S = 1; p.stride = 1; p.pad = 0;
    }
    p.c16 = p.C / 16;
    p.nk16 = p.R * p.S * p.c16;
    return ep ? dispatch_igemm<MODE_FWD, EPI_FWD>(c, p) : dispatch_igemm<MODE_FWD, EPI_ACC>(c, p);
}

extern "C" int eoq_conv_bwd_data(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *w, int32_t *d_acc,
                                 int32_t *absmax_slot, void *ws, size_t ws_bytes)
{
    if (!c || !e || !w || !d_acc || !absmax_slot) return EOQ_ERR_ARG;
    if (!desc_ok(d)) return EOQ_ERR_SHAPE;
    if (d->K % 16 || d->C % 16) return EOQ_ERR_SHAPE;
    if (((uintptr_t)e | (uintptr_t)w | (uintptr_t)d_acc) & 15) return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_workspace_bytes(d, EOQ_OP_CONV_BWD_DATA) || ((uintptr_t)ws & 15)) return EOQ_ERR_WORKSPACE;
    const int P = conv_out_dim(d->H, d->pad, d->R, d->stride), Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    if ((size_t)d->N * d->H * d->W > 0x7fffffffu || (size_t)P * Q * d->K > 0x7fffffffu) return EOQ_ERR_SHAPE;
    int8_t *wt = (int8_t *)ws;
    hipLaunchKernelGGL(transpose_filters_kernel, dim3(grid_for((size_t)d->K * d->R * d->S * d->C)), dim3(256), 0,
                       c->stream, w, d->K, d->R * d->S, d->C, wt);
    EOQ_LAUNCH_CHECK();
    IgemmParams p{};
    p.A = e; p.B = wt;
    p.N = d->N; p.H = P; p.W = Q; p.C = d->K;      // the tensor being gathered is the error
    p.P = d->H; p.Q = d->W; p.NOUT = d->C;         // one output row per input pixel
    p.R = d->R; p.S = d->S; p.stride = d->stride; p.pad = d->pad;
    p.M = d->N * d->H * d->W;
    p.c16 = p.C / 16;
    p.nk16 = p.R * p.S * p.c16;
    p.acc_out = d_acc;
    p.absmax = absmax_slot;
    return dispatch_igemm<MODE_BWD_DATA, EPI_ACC>(c, p);
}

int eoq_requant_fwd_standalone(eoq_ctx *c, const eoq_requant_args *a)
{
    if (!a->acc || !a->ep || (a->n % 16) || ((uintptr_t)a->acc & 15)) return EOQ_ERR_ARG;
    EpiDev ep;
    if (int rc = fill_epi(a->ep, ep)) return rc;
    if (!a->n) return EOQ_OK;
    hipLaunchKernelGGL(requant_fwd_kernel, dim3(grid_for(a->n / 16)), dim3(256), 0, c->stream, a->acc, a->n / 16, ep);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}
