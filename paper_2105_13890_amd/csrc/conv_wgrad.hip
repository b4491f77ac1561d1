// Weight-gradient convolution (Eq.4, g_w before Q_g) on int8 MFMA for gfx950:
//     G[k,r,s,c] = sum_{n,p,q} e[n,p,q,k] * u[n, p*stride+r-pad, q*stride+s-pad, c]
//
// GEMM view per filter tap: rows = output channels k, columns = input channels c, reduction = output
// pixels.  Both operands are stored with the reduction index as the SLOW axis (NHWC), which is the
// wrong way round for MFMA operands (each lane must supply 16 consecutive reduction elements).  The
// tiles are therefore kept in LDS in their natural [pixel][channel] layout and read with the gfx950
// transposing LDS load ds_read_b64_tr_b8: within each group of 16 lanes, lanes 2j and 2j+1 address
// the two 8-byte halves of a 16-byte row j (8 rows), and lane i receives byte i of each of the 8 rows --
// i.e. 8 consecutive pixels of channel i.  Because every row is addressed separately, the filter-tap
// shift (r,s) is applied at read time: the input patch (with halo) is staged in LDS once per pixel
// chunk and every tap reads it at a different offset; padding pixels are stored as zeros.
//
// A workgroup (4 waves, WK x WC) owns KT x CT channels for up to TAPS taps and walks a range of pixel
// chunks (PR x PQ output pixels, at most 64, i.e. two MFMA reduction steps); the partial sums of each
// range are written as int32 (a range never exceeds 131072 terms) and combined exactly in int64 by a
// second kernel which also checks the int32 range and takes the abs-max for Q_g.
#include "common.h"

namespace {

constexpr int PIX = 64;          // pixel slots per LDS stage
constexpr int MAX_SPLITS = 64;

struct WgradParams {
    const int8_t *E;   // N x P x Q x K
    const int8_t *U;   // N x H x W x C
    int N, H, W, C, P, Q, K, R, S, stride, pad;
    int RS;
    int PR, PQ;        // chunk shape in output pixels (PR*PQ <= PIX)
    int PH, PW;        // patch shape in staged input pixels
    int pstep;         // input pixels between staged patch pixels (stride for 1x1 filters, else 1)
    int tiles_p, tiles_q, nchunks, chunks_per_split;
    int tap_groups;
    int32_t *part;     // [splits][K][RS][C]
    size_t part_stride;
};

__device__ __forceinline__ v2i lds_read_tr8(const int8_t *p)
{
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)p);
}

template <int WK, int WC, int TK, int TC, int TAPS, int U_LOADS>
__global__ __launch_bounds__(256) void wgrad_kernel(WgradParams p)
{
    static_assert(WK * WC == 4, "4 waves");
    constexpr int KT = WK * TK * 32, CT = WC * TC * 32;
    constexpr int E_LD = KT + 16, U_LD = CT + 16;            // padded LDS row strides (bytes)
    constexpr int E_CH = KT / 16, U_CH = CT / 16;            // 16-byte chunks per row
    constexpr int E_LOADS = (PIX * E_CH + 255) / 256;
    constexpr int E_BYTES = PIX * E_LD;
    constexpr int U_ROWS = U_LOADS * 256 / U_CH;             // patch pixels that fit
    constexpr int U_BYTES = U_ROWS * U_LD;
    constexpr int STAGE_BYTES = E_BYTES + U_BYTES;

    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave / WC, wc = wave % WC;
    const int tiles_k = (p.K + KT - 1) / KT, tiles_c = (p.C + CT - 1) / CT;
    int bid = blockIdx.x;
    const int tile_c = bid % tiles_c; bid /= tiles_c;
    const int tile_k = bid % tiles_k; bid /= tiles_k;
    const int tapg = bid % p.tap_groups;
    const int split = bid / p.tap_groups;
    const int k0 = tile_k * KT, c0 = tile_c * CT, tap0 = tapg * TAPS;

    // ---- loader state (fixed per thread) ----
    int e_dp[E_LOADS], e_dq[E_LOADS], e_col[E_LOADS], e_dst[E_LOADS];
#pragma unroll
    for (int i = 0; i < E_LOADS; ++i) {
        int idx = tid + 256 * i;
        int slot = idx / E_CH;
        e_col[i] = idx % E_CH;
        bool ok = slot < PIX && slot < p.PR * p.PQ && (k0 + e_col[i] * 16) < p.K;
        e_dp[i] = ok ? slot / p.PQ : -1;
        e_dq[i] = ok ? slot % p.PQ : 0;
        e_dst[i] = slot < PIX ? slot * E_LD + e_col[i] * 16 : -1;
    }
    int u_py[U_LOADS], u_px[U_LOADS], u_col[U_LOADS], u_dst[U_LOADS];
    const int npatch = p.PH * p.PW;
#pragma unroll
    for (int i = 0; i < U_LOADS; ++i) {
        int idx = tid + 256 * i;
        int pix = idx / U_CH;
        u_col[i] = idx % U_CH;
        bool ok = pix < npatch && (c0 + u_col[i] * 16) < p.C;
        u_py[i] = ok ? pix / p.PW : -1;
        u_px[i] = ok ? pix % p.PW : 0;
        u_dst[i] = pix < npatch ? pix * U_LD + u_col[i] * 16 : -1;
    }

    // ---- MFMA operand addressing (fixed per lane) ----
    const int g = lane >> 5, grp16 = (lane & 31) >> 4, L = lane & 15;
    int a_off[4], b_pix[4];                       // index jh = 2*j + h : reduction step j, 8-slot half h
#pragma unroll
    for (int jh = 0; jh < 4; ++jh) {
        int slot = (jh >> 1) * 32 + 16 * g + 8 * (jh & 1) + (L >> 1);
        a_off[jh] = slot * E_LD + grp16 * 16 + 8 * (L & 1);
        int dp = 0, dq = 0;
        if (slot < p.PR * p.PQ) { dp = slot / p.PQ; dq = slot % p.PQ; }
        b_pix[jh] = ((dp * p.stride) / p.pstep) * p.PW + (dq * p.stride) / p.pstep;
    }
    const int b_lane = grp16 * 16 + 8 * (L & 1);

    v16i acc[TK][TC][TAPS];
#pragma unroll
    for (int a = 0; a < TK; ++a)
#pragma unroll
        for (int b = 0; b < TC; ++b)
#pragma unroll
            for (int t = 0; t < TAPS; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][t][e] = 0;

    const int ch_begin = split * p.chunks_per_split;
    int ch_end = ch_begin + p.chunks_per_split;
    if (ch_end > p.nchunks) ch_end = p.nchunks;

    v4i re[E_LOADS], ru[U_LOADS];
    auto load_chunk = [&](int ch) {
        int tq = ch % p.tiles_q;
        int t = ch / p.tiles_q;
        int tp = t % p.tiles_p, n = t / p.tiles_p;
        const int p0 = tp * p.PR, q0 = tq * p.PQ;
        const v4i z = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < E_LOADS; ++i) {
            int pp = p0 + e_dp[i], qq = q0 + e_dq[i];
            bool ok = e_dp[i] >= 0 && pp < p.P && qq < p.Q;
            re[i] = ok ? *(const v4i *)(p.E + (((size_t)n * p.P + pp) * p.Q + qq) * p.K + k0 + e_col[i] * 16) : z;
        }
        const int h0 = p0 * p.stride - p.pad, w0 = q0 * p.stride - p.pad;
#pragma unroll
        for (int i = 0; i < U_LOADS; ++i) {
            int hh = h0 + u_py[i] * p.pstep, ww = w0 + u_px[i] * p.pstep;
            bool ok = u_py[i] >= 0 && (unsigned)hh < (unsigned)p.H && (unsigned)ww < (unsigned)p.W;
            ru[i] = ok ? *(const v4i *)(p.U + (((size_t)n * p.H + hh) * p.W + ww) * p.C + c0 + u_col[i] * 16) : z;
        }
    };
    auto store_chunk = [&](int buf) {
        int8_t *Es = lds + buf * STAGE_BYTES, *Us = Es + E_BYTES;
#pragma unroll
        for (int i = 0; i < E_LOADS; ++i)
            if (e_dst[i] >= 0) *(v4i *)(Es + e_dst[i]) = re[i];
#pragma unroll
        for (int i = 0; i < U_LOADS; ++i)
            if (u_dst[i] >= 0) *(v4i *)(Us + u_dst[i]) = ru[i];
    };

    if (ch_begin < ch_end) {
        load_chunk(ch_begin);
        store_chunk(0);
    }
    __syncthreads();
    for (int ch = ch_begin; ch < ch_end; ++ch) {
        const bool more = ch + 1 < ch_end;
        if (more) load_chunk(ch + 1);
        const int8_t *Es = lds + ((ch - ch_begin) & 1) * STAGE_BYTES, *Us = Es + E_BYTES;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            v4i a[TK];
#pragma unroll
            for (int tk = 0; tk < TK; ++tk) {
                const int kb = (wk * TK + tk) * 32;
                v2i lo = lds_read_tr8(Es + a_off[2 * j] + kb);
                v2i hi = lds_read_tr8(Es + a_off[2 * j + 1] + kb);
                a[tk] = v4i{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int tap = tap0 + t;
                if (tap < p.RS) {
                    const int toff = (p.RS == 1) ? 0 : ((tap / p.S) * p.PW + (tap % p.S));
#pragma unroll
                    for (int tc = 0; tc < TC; ++tc) {
                        const int cb = (wc * TC + tc) * 32 + b_lane;
                        v2i lo = lds_read_tr8(Us + (b_pix[2 * j] + toff) * U_LD + cb);
                        v2i hi = lds_read_tr8(Us + (b_pix[2 * j + 1] + toff) * U_LD + cb);
                        v4i b = v4i{lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
                        for (int tk = 0; tk < TK; ++tk)
                            acc[tk][tc][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[tk], b, acc[tk][tc][t], 0, 0, 0);
                    }
                }
            }
        }
        if (more) store_chunk(((ch - ch_begin) + 1) & 1);
        __syncthreads();
    }

    // ---- write this range's partial sums: part[split][k][tap][c] ----
    int32_t *out = p.part + (size_t)split * p.part_stride;
    const int col = lane & 31;
#pragma unroll
    for (int tk = 0; tk < TK; ++tk)
#pragma unroll
        for (int tc = 0; tc < TC; ++tc) {
            const int c = c0 + (wc * TC + tc) * 32 + col;
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int tap = tap0 + t;
                if (tap < p.RS && c < p.C) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int k = k0 + (wk * TK + tk) * 32 + (e >> 2) * 8 + g * 4 + (e & 3);
                        if (k < p.K) out[((size_t)k * p.RS + tap) * p.C + c] = acc[tk][tc][t][e];
                    }
                }
            }
        }
}

// exact combination of the partial sums; int32 range check; abs-max for Q_g.
// ld_in is the row length of the partial buffers (padded reduction for the im2col path), ld_out the
// true R*S*C of the filter.
__global__ void wgrad_finalize_kernel(const int32_t *part, size_t part_stride, int splits, int K, int ld_in, int ld_out,
                                      int32_t *g, int32_t *absmax, uint32_t *status)
{
    const size_t total = (size_t)K * ld_out;
    int mx = 0;
    bool bad = false;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        size_t k = i / ld_out, j = i % ld_out;
        int64_t s = 0;
        for (int sp = 0; sp < splits; ++sp) s += part[(size_t)sp * part_stride + k * ld_in + j];
        if (s > 2147483647LL || s < -2147483648LL) { bad = true; s = s > 0 ? 2147483647LL : -2147483647LL; }
        g[i] = (int32_t)s;
        int64_t a = s < 0 ? -s : s;
        int ai = a > 2147483647LL ? 2147483647 : (int)a;
        mx = ai > mx ? ai : mx;
    }
    block_atomic_max_i32(mx, absmax);
    if (bad) atomicOr(status, (uint32_t)EOQ_FLAG_ACC_OVERFLOW);
}

// explicit im2col (shared shape with the forward path): col[m][KP]
__global__ void wgrad_im2col_kernel(const int8_t *u, int N, int H, int W, int C, int P, int Q, int R, int S,
                                    int stride, int pad, int KP, int8_t *col)
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
            o[b >> 2] = (int)(((uint32_t)o[b >> 2]) | (((uint32_t)val & 0xffu) << (8 * (b & 3))));
        }
        *(v4i *)(col + m * KP + ch * 16) = o;
    }
}

inline unsigned grid_for(size_t total)
{
    size_t b = (total + 255) / 256;
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    return (unsigned)b;
}

// pick the chunk shape PR x PQ (<= 64 output pixels) that wastes the fewest pixel slots
void pick_chunk(int P, int Q, int stride, int R, int S, int max_patch, int &PR, int &PQ, int &PH, int &PW, int &pstep)
{
    pstep = (R == 1 && S == 1) ? stride : 1;
    double best = -1.0;
    PR = 1; PQ = 1;
    for (int pq = 1; pq <= PIX && pq <= Q; ++pq) {
        int pr = PIX / pq;
        if (pr > P) pr = P;
        int ph = ((pr - 1) * stride + R + pstep - 1) / pstep, pw = ((pq - 1) * stride + S + pstep - 1) / pstep;
        if (ph * pw > max_patch) continue;
        double util = (double)Q / (((Q + pq - 1) / pq) * pq) * (double)P / (((P + pr - 1) / pr) * pr) *
                      (double)(pq * pr) / PIX;
        // prefer compact patches on ties
        util -= 1e-6 * (double)(ph * pw) / (double)(pq * pr);
        if (util > best) { best = util; PR = pr; PQ = pq; }
    }
    PH = ((PR - 1) * stride + R + pstep - 1) / pstep;
    PW = ((PQ - 1) * stride + S + pstep - 1) / pstep;
}

template <int WK, int WC, int TK, int TC, int TAPS, int U_LOADS>
int launch_wgrad(eoq_ctx *c, WgradParams p, int RS, int *splits_out)
{
    constexpr int KT = WK * TK * 32, CT = WC * TC * 32;
    constexpr int U_ROWS = U_LOADS * 256 / (CT / 16);
    constexpr int lds_bytes = 2 * (PIX * (KT + 16) + U_ROWS * (CT + 16));
    pick_chunk(p.P, p.Q, p.stride, p.R, p.S, U_ROWS, p.PR, p.PQ, p.PH, p.PW, p.pstep);
    if (p.PH * p.PW > U_ROWS) return EOQ_ERR_SHAPE;
    p.tiles_p = (p.P + p.PR - 1) / p.PR;
    p.tiles_q = (p.Q + p.PQ - 1) / p.PQ;
    p.nchunks = p.N * p.tiles_p * p.tiles_q;
    p.tap_groups = (RS + TAPS - 1) / TAPS;
    const int tiles = ((p.K + KT - 1) / KT) * ((p.C + CT - 1) / CT) * p.tap_groups;
    int splits = 1024 / tiles;
    if (splits < 1) splits = 1;
    if (splits > MAX_SPLITS) splits = MAX_SPLITS;
    if (splits > p.nchunks) splits = p.nchunks;
    p.chunks_per_split = (p.nchunks + splits - 1) / splits;
    if ((long)p.chunks_per_split * PIX > 131072) {           // keep every int32 partial sum exact
        p.chunks_per_split = 131072 / PIX;
    }
    splits = (p.nchunks + p.chunks_per_split - 1) / p.chunks_per_split;
    if (splits > MAX_SPLITS) return EOQ_ERR_SHAPE;
    static bool attr_done = false;
    auto kern = wgrad_kernel<WK, WC, TK, TC, TAPS, U_LOADS>;
    if (lds_bytes > 48 * 1024 && !attr_done) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
            return EOQ_ERR_HIP;
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles * splits)), dim3(256), lds_bytes, c->stream, p);
    EOQ_LAUNCH_CHECK();
    *splits_out = splits;   // number of partial buffers written
    return EOQ_OK;
}

} // namespace

extern "C" int eoq_conv_bwd_weight(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *u,
                                   int32_t *g_acc, int32_t *absmax_slot, void *ws, size_t ws_bytes)
{
    if (!c || !d || !e || !u || !g_acc || !absmax_slot) return EOQ_ERR_ARG;
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->stride <= 0 ||
        d->pad < 0)
        return EOQ_ERR_SHAPE;
    const int P = conv_out_dim(d->H, d->pad, d->R, d->stride), Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    if (P <= 0 || Q <= 0 || d->K % 16) return EOQ_ERR_SHAPE;
    if (((uintptr_t)e | (uintptr_t)u | (uintptr_t)g_acc) & 15) return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_workspace_bytes(d, EOQ_OP_CONV_BWD_WEIGHT) || ((uintptr_t)ws & 15)) return EOQ_ERR_WORKSPACE;

    WgradParams p{};
    p.E = e;
    p.K = d->K;
    int32_t *part;
    const int rsc = d->R * d->S * d->C;
    int ld_in = rsc;
    if (d->C % 16 == 0) {
        p.U = u;
        p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C; p.P = P; p.Q = Q;
        p.R = d->R; p.S = d->S; p.stride = d->stride; p.pad = d->pad;
        part = (int32_t *)ws;
    } else {
        // explicit im2col: a 1x1 weight gradient over M "pixels" with KP padded channels
        const size_t M = (size_t)d->N * P * Q;
        if (M > 0x7fffffffu) return EOQ_ERR_SHAPE;
        const int KP = (int)round_up((size_t)rsc, 64);
        int8_t *col = (int8_t *)ws;
        const size_t col_bytes = round_up(M * KP, 256) + round_up((size_t)d->K * KP, 256);
        part = (int32_t *)((int8_t *)ws + col_bytes);
        hipLaunchKernelGGL(wgrad_im2col_kernel, dim3(grid_for(M * (KP / 16))), dim3(256), 0, c->stream, u, d->N, d->H,
                           d->W, d->C, P, Q, d->R, d->S, d->stride, d->pad, KP, col);
        EOQ_LAUNCH_CHECK();
        p.U = col;
        p.N = 1; p.H = 1; p.W = (int)M; p.C = KP; p.P = 1; p.Q = (int)M;
        p.R = 1; p.S = 1; p.stride = 1; p.pad = 0;
        ld_in = KP;
    }
    p.RS = p.R * p.S;
    p.part = part;
    p.part_stride = (size_t)p.K * p.RS * p.C;
    int splits = 0, rc;
    if (p.RS == 1) {
        if (p.K >= 128) rc = launch_wgrad<2, 2, 2, 2, 1, 4>(c, p, p.RS, &splits);
        else rc = launch_wgrad<2, 2, 1, 2, 1, 4>(c, p, p.RS, &splits);
    } else {
        rc = launch_wgrad<2, 2, 1, 1, 9, 8>(c, p, p.RS, &splits);
    }
    if (rc != EOQ_OK) return rc;
    hipLaunchKernelGGL(wgrad_finalize_kernel, dim3(grid_for((size_t)d->K * rsc)), dim3(256), 0, c->stream, part,
                       p.part_stride, splits, d->K, ld_in, rsc, g_acc, absmax_slot, c->d_status);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}
