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

#include <atomic>
#include <mutex>

namespace {

constexpr int PIX = 64;          // pixel slots per LDS stage

struct WgradParams {
    const int8_t *E;   // N x P x Q x K
    const int8_t *U;   // N x H x W x C
    int N, H, W, C, P, Q, K, R, S, stride, pad;
    int RS;
    int PR, PQ;        // chunk shape in output pixels (PR*PQ <= PIX)
    int PH, PW;        // patch shape in staged input pixels
    int pstep;         // input pixels between staged patch pixels (stride for 1x1 filters, else 1)
    int tiles_p, tiles_q, nchunks, chunks_per_split;
    Recip rPQ, rPW, rTQ, rTP;   // reciprocals of PQ, PW, tiles_q, tiles_p
    int sdiv;                   // stride / pstep (patch pixels per output pixel step)
    int tap_groups;
    int32_t *part;     // [splits][K][RS][C]
    size_t part_stride;
    // few-channel input staged as zero-bordered 4-bytes-per-pixel image: the "channels" of the 1x1 problem are
    // the R*S4 sixteen-byte column groups of the filter window (pad4_S4 > 0 switches this addressing on)
    int pad4_S4, pad4_R, pad4_Wp, pad4_stride;
#ifdef EOQ_TUNE
    unsigned long long *dbg;   // tuning builds: four timestamps per workgroup (entry, set-up done, reduction done, exit)
    int remap;
#endif
};

__device__ __forceinline__ v2i lds_read_tr8(const int8_t *p)
{
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3))) *)p);
}

// The chunks travel through a ring of NS LDS stages filled by direct-to-LDS loads (no staging registers, NS - 1 chunks
// in flight).  Rows are stored unpadded, with the 16-byte chunk index XOR-swizzled by the row so that the eight rows a
// transposing read touches spread over all banks; the swizzle is applied on the memory side (a lane asks for the
// logical chunk that belongs in the slot it fills).
template <int WK, int WC, int TK, int TC, int TAPS, int U_LOADS, bool FULL, int NS>
__device__ __forceinline__ void wgrad_body(const WgradParams &p)
{
    // Wave priority 3 for the kernels of the weight-gradient chain (this one, the reduction of its partial sums, the
    // update, the recompute of x2): in a training step they share the compute units with the error chain's kernels,
    // which spend their time waiting for memory; letting the matrix-bound waves issue first whenever both are ready
    // shortens the step by about 1 % (measured run against run on one machine; the opposite choice, priority for the
    // error chain's convolutions, costs 3 %).  It changes no result and means nothing when a kernel runs alone.
#ifdef EOQ_TUNE
    const unsigned long long ts0 = __builtin_amdgcn_s_memrealtime();
#endif
    __builtin_amdgcn_s_setprio(3);
    static_assert(WK * WC == 4, "4 waves");
    static_assert(NS >= 2, "ring");
    constexpr int KT = WK * TK * 32, CT = WC * TC * 32;      // tile = LDS row lengths (bytes)
    static_assert((KT == 64 || KT == 128) && (CT == 64 || CT == 128), "swizzle periods");
    // chunk-index swizzle of a row of RB bytes: eight consecutive rows cover a 128-byte bank line in eight distinct slots
    auto swz_e = [](int row) { return KT == 128 ? (row & 7) : ((row >> 1) & 3); };
    auto swz_u = [](int row) { return CT == 128 ? (row & 7) : ((row >> 1) & 3); };
    constexpr int E_CH = KT / 16, U_CH = CT / 16;            // 16-byte chunks per row
    constexpr int E_LOADS = (PIX * E_CH + 255) / 256;
    static_assert(PIX * E_CH % 256 == 0, "error tile loads divide evenly");
    constexpr int E_BYTES = PIX * KT;
    constexpr int U_ROWS = U_LOADS * 256 / U_CH;             // patch pixels that fit
    constexpr int U_BYTES = U_ROWS * CT;
    constexpr int STAGE_BYTES = E_BYTES + U_BYTES;
    constexpr int OOB = 0x7fffff00;

    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave / WC, wc = wave % WC;
    const int tiles_k = (p.K + KT - 1) / KT, tiles_c = (p.C + CT - 1) / CT;
    // Consecutive workgroup ids go round-robin over the 8 XCDs (each with its own L2).  Remapped so that an XCD works on
    // a contiguous range of (pixel range, tile) pairs with the pixel range slowest: an XCD then pulls only its own one or
    // two pixel ranges of both operands through its L2, instead of every XCD pulling nearly all of both.
    int bid = blockIdx.x;
#ifdef EOQ_TUNE
    if (p.remap)
#endif
    {
        const int nb = gridDim.x, per = nb >> 3, rem = nb & 7, x = bid & 7;
        bid = x * per + (x < rem ? x : rem) + (bid >> 3);
    }
    const int tile_c = bid % tiles_c; bid /= tiles_c;
    const int tile_k = bid % tiles_k; bid /= tiles_k;
    const int tapg = bid % p.tap_groups;
    const int split = bid / p.tap_groups;
    const int k0 = tile_k * KT, c0 = tile_c * CT, tap0 = tapg * TAPS;

    // Out-of-range offsets make the buffer loads return zeros: padding pixels, pixel slots beyond the
    // chunk and channels beyond the tensor cost neither a branch nor a select.
    // ---- loader state (fixed per thread): offsets relative to the chunk origin ----
    int e_dp[E_LOADS], e_dq[E_LOADS], e_off[E_LOADS];
#pragma unroll
    for (int i = 0; i < E_LOADS; ++i) {
        const int idx = tid + 256 * i;
        const int slot = idx / E_CH, col = (idx % E_CH) ^ swz_e(slot);
        const bool ok = slot < p.PR * p.PQ && (k0 + col * 16) < p.K;
        const int sp = (int)fast_div((uint32_t)slot, p.rPQ);
        e_dp[i] = ok ? sp : 1 << 20;                        // an invalid slot never passes the row test
        e_dq[i] = ok ? slot - sp * p.PQ : 0;
        e_off[i] = ok ? (e_dp[i] * p.Q + e_dq[i]) * p.K + k0 + col * 16 : 0;
    }
    int u_py[U_LOADS], u_px[U_LOADS], u_off[U_LOADS];
    const int npatch = p.PH * p.PW;
#pragma unroll
    for (int i = 0; i < U_LOADS; ++i) {
        const int idx = tid + 256 * i;
        const int pix = idx / U_CH, col = (idx % U_CH) ^ swz_u(pix);
        const bool ok = pix < npatch && (c0 + col * 16) < p.C;
        const int py = (int)fast_div((uint32_t)pix, p.rPW);
        u_py[i] = ok ? py * p.pstep : 1 << 20;
        u_px[i] = ok ? (pix - py * p.PW) * p.pstep : 0;
        if (p.pad4_S4) {
            // slot (py,px) of the chunk, column group cg = (filter row r, 4-column group j)
            const int cg = c0 / 16 + col, r = cg / p.pad4_S4, j = cg % p.pad4_S4;
            u_off[i] = ok ? ((u_py[i] * p.pad4_stride + r) * p.pad4_Wp + u_px[i] * p.pad4_stride) * 4 + j * 16 : 0;
        } else {
            u_off[i] = ok ? (u_py[i] * p.W + u_px[i]) * p.C + c0 + col * 16 : 0;
        }
    }

    // ---- MFMA operand addressing (fixed per lane) ----
    const int g = lane >> 5, grp16 = (lane & 31) >> 4, L = lane & 15;
    // rows this lane reads: error slot and patch pixel, index jh = 2*j + h : reduction step j, 8-slot half h
    int a_row[4], b_row[4];
#pragma unroll
    for (int jh = 0; jh < 4; ++jh) {
        const int slot = (jh >> 1) * 32 + 16 * g + 8 * (jh & 1) + (L >> 1);
        int dp = 0, dq = 0;
        if (slot < p.PR * p.PQ) { dp = (int)fast_div((uint32_t)slot, p.rPQ); dq = slot - dp * p.PQ; }
        a_row[jh] = slot;
        b_row[jh] = dp * p.sdiv * p.PW + dq * p.sdiv;
    }
    // row offset of each tap inside the patch (uniform)
    int tap_off[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
        const int tap = tap0 + t;
        const int rows = (p.RS == 1 || tap >= p.RS) ? 0 : (tap / p.S) * p.PW + (tap % p.S);
        tap_off[t] = rows;
    }
    // byte address of this lane's half of (row, 16-byte chunk), swizzle applied
    auto addr_e = [&](int row, int chunk) { return row * KT + ((chunk ^ swz_e(row)) << 4) + 8 * (L & 1); };
    auto addr_u = [&](int row, int chunk) { return E_BYTES + row * CT + ((chunk ^ swz_u(row)) << 4) + 8 * (L & 1); };

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
    const int nch = ch_end - ch_begin;

    // chunk being loaded: (image, chunk row, chunk column), advanced without divisions (all uniform)
    const int cq = (int)fast_div((uint32_t)ch_begin, p.rTQ);
    int ld_q = ch_begin - cq * p.tiles_q;
    int ld_n = (int)fast_div((uint32_t)cq, p.rTP), ld_p = cq - ld_n * p.tiles_p;

    int ld_i = 0;                                  // chunks requested so far; past the range every load is out of range
#ifdef EOQ_WABL
    auto rd = [&](const int8_t *q) { return (EOQ_WABL & 2) ? v2i{lane + (int)(uintptr_t)q, tid} : lds_read_tr8(q); };
#define lds_read_tr8 rd
#endif
    auto compute_half = [&](int buf, int j) {      // one of the two 32-pixel reduction steps of a chunk
        const int8_t *base = lds + buf;
        v4i a[TK];
#pragma unroll
        for (int tk = 0; tk < TK; ++tk) {
            const int ch = 2 * (wk * TK + tk) + grp16;
            const v2i lo = lds_read_tr8(base + addr_e(a_row[2 * j], ch));
            const v2i hi = lds_read_tr8(base + addr_e(a_row[2 * j + 1], ch));
            a[tk] = v4i{lo[0], lo[1], hi[0], hi[1]};
        }
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            if (FULL || tap0 + t < p.RS) {
#pragma unroll
                for (int tc = 0; tc < TC; ++tc) {
                    const int ch = 2 * (wc * TC + tc) + grp16;
                    const v2i lo = lds_read_tr8(base + addr_u(b_row[2 * j] + tap_off[t], ch));
                    const v2i hi = lds_read_tr8(base + addr_u(b_row[2 * j + 1] + tap_off[t], ch));
                    const v4i b = v4i{lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
                    for (int tk = 0; tk < TK; ++tk) {
#ifdef EOQ_WABL
                        if (EOQ_WABL & 4) { acc[tk][tc][t][0] += a[tk][0] ^ b[0]; acc[tk][tc][t][1] += a[tk][2] ^ b[3]; continue; }
#endif
                        acc[tk][tc][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[tk], b, acc[tk][tc][t], 0, 0, 0);
                    }
                }
            }
        }
    };
#ifdef EOQ_WABL
#undef lds_read_tr8
#endif

#ifdef EOQ_TUNE
    const unsigned long long ts1 = __builtin_amdgcn_s_memrealtime();
#endif
    {
        // Iteration i: wait until this thread's loads of chunk i have landed | barrier | request chunk i+NS-1 into the
        // buffer chunk i-1 was multiplied from | multiply chunk i.  Requests past the range are out of range (zeros, no
        // traffic), so the number of loads in flight at the wait is a compile-time constant.
        constexpr int L = E_LOADS + U_LOADS;
        static_assert((NS - 1) * L < 64, "vmcnt range");
        const uint32_t wave_base = (uint32_t)(uintptr_t)lds + (uint32_t)__builtin_amdgcn_readfirstlane(wave) * 1024u;
        const uint64_t pe = (uint64_t)p.E, pu = (uint64_t)p.U;
        const v4i rs_e = {(int)(uint32_t)pe, (int)((uint32_t)(pe >> 32) & 0xffffu), p.N * p.P * p.Q * p.K, 0x00020000};
        const v4i rs_u = {(int)(uint32_t)pu, (int)((uint32_t)(pu >> 32) & 0xffffu),
                          p.pad4_S4 ? p.N * p.H * p.pad4_Wp * 4 : p.N * p.H * p.W * p.C, 0x00020000};
        auto dma_chunk = [&](int buf) {
#ifdef EOQ_WABL       // timing experiments only (results are then wrong): 1 no loads, 2 no LDS reads, 4 no MFMA
            if (EOQ_WABL & 1) return;
#endif
            const bool live = ld_i < nch;
            ++ld_i;
            const int p0 = ld_p * p.PR, q0 = ld_q * p.PQ;
            const int base_e = ((ld_n * p.P + p0) * p.Q + q0) * p.K;
#pragma unroll
            for (int i = 0; i < E_LOADS; ++i) {
                const bool ok = live && p0 + e_dp[i] < p.P && q0 + e_dq[i] < p.Q;
                lds_direct_load16(rs_e, wave_base + buf + i * 4096, ok ? base_e + e_off[i] : OOB);
            }
            const int h0 = p0 * p.stride - p.pad, w0 = q0 * p.stride - p.pad;
            const int base_u = p.pad4_S4 ? ((ld_n * p.H + p0 * p.pad4_stride) * p.pad4_Wp + q0 * p.pad4_stride) * 4
                                         : ((ld_n * p.H + h0) * p.W + w0) * p.C;
#pragma unroll
            for (int i = 0; i < U_LOADS; ++i) {
                const bool ok = live && (p.pad4_S4 ? (p0 + u_py[i] < p.P && q0 + u_px[i] < p.Q)
                                                   : ((unsigned)(h0 + u_py[i]) < (unsigned)p.H && (unsigned)(w0 + u_px[i]) < (unsigned)p.W));
                lds_direct_load16(rs_u, wave_base + buf + E_BYTES + i * 4096, ok ? base_u + u_off[i] : OOB);
            }
            if (++ld_q == p.tiles_q) { ld_q = 0; if (++ld_p == p.tiles_p) { ld_p = 0; ++ld_n; } }
        };
#pragma unroll
        for (int d = 0; d < NS - 1; ++d) dma_chunk(d * STAGE_BYTES);
        int cur = 0;
        for (int i = 0; i < nch; ++i) {
            wait_vmcnt<(NS - 2) * L>();
            __syncthreads();
            dma_chunk(cur == 0 ? (NS - 1) * STAGE_BYTES : cur - STAGE_BYTES);
            __builtin_amdgcn_sched_barrier(0);
            compute_half(cur, 0);
            compute_half(cur, 1);
            __builtin_amdgcn_sched_barrier(0);
            cur = cur + STAGE_BYTES == NS * STAGE_BYTES ? 0 : cur + STAGE_BYTES;
        }
        wait_vmcnt<0>();          // the out-of-range requests behind the last chunk still write (zeros) to LDS
    }

#ifdef EOQ_TUNE
    const unsigned long long ts2 = __builtin_amdgcn_s_memrealtime();
#endif
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
#ifdef EOQ_TUNE
    if (p.dbg && tid == 0 && blockIdx.x < 8192) {
        unsigned long long *r = p.dbg + 4 * (size_t)blockIdx.x;
        r[0] = ts0; r[1] = ts1; r[2] = ts2; r[3] = __builtin_amdgcn_s_memrealtime();
    }
#endif
}

template <int WK, int WC, int TK, int TC, int TAPS, int U_LOADS, bool FULL, int NS>
__global__ __launch_bounds__(256) void wgrad_kernel(WgradParams p)
{
    wgrad_body<WK, WC, TK, TC, TAPS, U_LOADS, FULL, NS>(p);
}

// Launch bounds by family.  The single-tap (1x1) kernels need 118 registers and 48 KB of LDS (three stages of 16 KB):
// three workgroups per compute unit.  The nine-tap stride-1 kernel, whose 9 x 16 accumulators alone take 144 registers,
// fits 256 (two per compute unit, four stages of 12 KB each); the general nine-tap kernel (strided, 24 KB stages) runs
// one workgroup per SIMD set with the full register file.
template <int WK, int WC, int TK, int TC, int TAPS, int U_LOADS, bool FULL, int NS>
__global__ __launch_bounds__(256, 2) void wgrad_occ2_kernel(WgradParams p)
{
    wgrad_body<WK, WC, TK, TC, TAPS, U_LOADS, FULL, NS>(p);
}

template <int WK, int WC, int TK, int TC, int TAPS, int U_LOADS, bool FULL, int NS>
__global__ __launch_bounds__(256, 3) void wgrad_occ3_kernel(WgradParams p)
{
    wgrad_body<WK, WC, TK, TC, TAPS, U_LOADS, FULL, NS>(p);
}

// exact combination of the partial sums; int32 range check; abs-max for Q_g.
// ld_in is the row length of the partial buffers (padded reduction for the im2col path), ld_out the
// true R*S*C of the filter.  A block covers 64 consecutive filter elements (256-byte rows of the partial
// buffers); its 4 thread rows each sum every fourth partial buffer in int64, combined through LDS.
// pad4_S (> 0): the partial rows hold R x S4 x (4 columns x 4 channel slots); element (r,s,c) of the S x pad4_C filter
// row sits at r*S4*16 + s*4 + c.
__global__ void wgrad_finalize_kernel(const int32_t *part, size_t part_stride, int splits, int K, int ld_in, int ld_out,
                                      int32_t *g, int32_t *absmax, uint32_t *status, int pad4_S, int pad4_C, int pad4_S4)
{
    __shared__ long long red[4][64];
    const size_t total = (size_t)K * ld_out;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    int mx = 0;
    bool bad = false;
    for (size_t i0 = (size_t)blockIdx.x * 64; i0 < total; i0 += (size_t)gridDim.x * 64) {
        const size_t i = i0 + tx;
        long long s = 0;
        if (i < total) {
            const size_t k = i / ld_out;
            size_t j = i % ld_out;
            if (pad4_S) {
                const int c = (int)(j % pad4_C), sx = (int)((j / pad4_C) % pad4_S), r = (int)(j / ((size_t)pad4_C * pad4_S));
                j = (size_t)r * pad4_S4 * 16 + sx * 4 + c;
            }
            const int32_t *src = part + k * ld_in + j;
            for (int sp = ty; sp < splits; sp += 4) s += src[(size_t)sp * part_stride];
        }
        red[ty][tx] = s;
        __syncthreads();
        if (ty == 0 && i < total) {
            s += red[1][tx] + red[2][tx] + red[3][tx];
            if (s > 2147483647LL || s < -2147483648LL) { bad = true; s = s > 0 ? 2147483647LL : -2147483647LL; }
            g[i] = (int32_t)s;
            const long long a = s < 0 ? -s : s;
            const int ai = a > 2147483647LL ? 2147483647 : (int)a;
            mx = ai > mx ? ai : mx;
        }
        __syncthreads();
    }
    block_atomic_max_i32(mx, absmax);
    if (bad) atomicOr(status, (uint32_t)EOQ_FLAG_ACC_OVERFLOW);
}

// contiguous partial buffers (the usual case): a lane owns 4 consecutive elements and sums every SL-th buffer, four
// loads in flight at a time; the SL lanes of a group combine through LDS.  Many loads in flight matter more than
// anything else here: the data is a few megabytes, the kernel's time is memory latency.
template <int SL>
__global__ void __launch_bounds__(256) wgrad_finalize_v4_kernel(const int32_t *part, size_t part_stride, int splits,
                                                                size_t total4, int32_t *g, int32_t *absmax,
                                                                uint32_t *status)
{
    __builtin_amdgcn_s_setprio(3);
    constexpr int QB = 256 / SL;
    __shared__ long long red[SL > 1 ? 256 * 4 : 4];
    const int tx = threadIdx.x % QB, ty = threadIdx.x / QB;
    int mx = 0;
    bool bad = false;
    for (size_t q0 = (size_t)blockIdx.x * QB; q0 < total4; q0 += (size_t)gridDim.x * QB) {
        const size_t q = q0 + tx;
        long long s[4] = {0, 0, 0, 0};
        if (q < total4) {
            const int32_t *src = part + q * 4;
            int sp = ty;
            for (; sp + 3 * SL < splits; sp += 4 * SL) {
                const v4i a = *(const v4i *)(src + (size_t)sp * part_stride);
                const v4i b = *(const v4i *)(src + (size_t)(sp + SL) * part_stride);
                const v4i c = *(const v4i *)(src + (size_t)(sp + 2 * SL) * part_stride);
                const v4i d = *(const v4i *)(src + (size_t)(sp + 3 * SL) * part_stride);
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] += (long long)a[e] + b[e] + c[e] + d[e];
            }
            for (; sp < splits; sp += SL) {
                const v4i a = *(const v4i *)(src + (size_t)sp * part_stride);
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] += a[e];
            }
        }
        if (SL > 1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) red[(ty * QB + tx) * 4 + e] = s[e];
            __syncthreads();
            if (ty == 0)
                for (int y = 1; y < SL; ++y)
#pragma unroll
                    for (int e = 0; e < 4; ++e) s[e] += red[(y * QB + tx) * 4 + e];
        }
        if (ty == 0 && q < total4) {
            v4i o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                long long t = s[e];
                if (t > 2147483647LL || t < -2147483648LL) { bad = true; t = t > 0 ? 2147483647LL : -2147483647LL; }
                o[e] = (int)t;
                const long long a = t < 0 ? -t : t;
                const int ai = a > 2147483647LL ? 2147483647 : (int)a;
                mx = ai > mx ? ai : mx;
            }
            *(v4i *)(g + q * 4) = o;
        }
        if (SL > 1) __syncthreads();
    }
    block_atomic_max_i32(mx, absmax);
    if (bad) atomicOr(status, (uint32_t)EOQ_FLAG_ACC_OVERFLOW);
}

// input N x H x W x C (C <= 4)  ->  zero-bordered N x Hp x Wp x 4
__global__ void wgrad_pad4_input_kernel(const int8_t *u, int N, int H, int W, int C, int pad, int Hp, int Wp, uint32_t *up)
{
    const size_t total = (size_t)N * Hp * Wp;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int x = (int)(i % Wp) - pad;
        const size_t t = i / Wp;
        const int h = (int)(t % Hp) - pad, n = (int)(t / Hp);
        uint32_t v = 0;
        if ((unsigned)h < (unsigned)H && (unsigned)x < (unsigned)W) {
            const int8_t *src = u + (((size_t)n * H + h) * W + x) * C;
            for (int c = 0; c < C; ++c) v |= ((uint32_t)(uint8_t)src[c]) << (8 * c);
        }
        up[i] = v;
    }
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

#ifdef EOQ_TUNE
static unsigned long long *g_wtune_dbg = nullptr;
static int g_wtune_launch = 0;
#endif

template <int WK, int WC, int TK, int TC, int TAPS, int U_LOADS, int NS>
int launch_wgrad(eoq_ctx *c, WgradParams p, int RS, int max_splits, int *splits_out)
{
    constexpr int KT = WK * TK * 32, CT = WC * TC * 32;
    constexpr int U_ROWS = U_LOADS * 256 / (CT / 16);
    constexpr int lds_bytes = NS * (PIX * KT + U_ROWS * CT);
    pick_chunk(p.P, p.Q, p.stride, p.R, p.S, U_ROWS, p.PR, p.PQ, p.PH, p.PW, p.pstep);
    if (p.PH * p.PW > U_ROWS) return EOQ_ERR_SHAPE;
    p.tiles_p = (p.P + p.PR - 1) / p.PR;
    p.tiles_q = (p.Q + p.PQ - 1) / p.PQ;
    p.nchunks = p.N * p.tiles_p * p.tiles_q;
    p.rPQ = make_recip((uint32_t)p.PQ); p.rPW = make_recip((uint32_t)p.PW);
    p.rTQ = make_recip((uint32_t)p.tiles_q); p.rTP = make_recip((uint32_t)p.tiles_p);
    p.sdiv = p.stride / p.pstep;
    p.tap_groups = (RS + TAPS - 1) / TAPS;
    const int tiles = ((p.K + KT - 1) / KT) * ((p.C + CT - 1) / CT) * p.tap_groups;
    // workgroups aimed for when splitting the reduction: with three resident per compute unit and the error chain
    // sharing the chip, 448 measured better than 256 (by 2 % of a ResNet-50 step) and than 768
#ifdef EOQ_TUNE
    static const int target_wgs = getenv("EOQ_WTARGET") ? atoi(getenv("EOQ_WTARGET")) : 448;
    static const int tune_remap = getenv("EOQ_WXCD") ? atoi(getenv("EOQ_WXCD")) : 1;
    p.remap = tune_remap;
#else
    constexpr int target_wgs = 448;
#endif
    int splits = target_wgs / tiles;
    if (splits < 1) splits = 1;
    if (splits > max_splits) splits = max_splits;
    if (splits > p.nchunks) splits = p.nchunks;
    p.chunks_per_split = (p.nchunks + splits - 1) / splits;
    if ((long)p.chunks_per_split * PIX > 131072) {           // keep every int32 partial sum exact
        p.chunks_per_split = 131072 / PIX;
    }
    splits = (p.nchunks + p.chunks_per_split - 1) / p.chunks_per_split;
    if (splits > max_splits) return EOQ_ERR_WORKSPACE;     // the partial sums of the shortest legal ranges do not fit
    static std::atomic<bool> attr_done{false};
    void (*kern_full)(WgradParams) = wgrad_kernel<WK, WC, TK, TC, TAPS, U_LOADS, true, NS>;
    void (*kern_part)(WgradParams) = wgrad_kernel<WK, WC, TK, TC, TAPS, U_LOADS, false, NS>;
    if constexpr (TAPS == 1) {
        kern_full = wgrad_occ3_kernel<WK, WC, TK, TC, TAPS, U_LOADS, true, NS>;
        kern_part = wgrad_occ3_kernel<WK, WC, TK, TC, TAPS, U_LOADS, false, NS>;
    } else if constexpr (U_LOADS == 2) {
        kern_full = wgrad_occ2_kernel<WK, WC, TK, TC, TAPS, U_LOADS, true, NS>;
        kern_part = wgrad_occ2_kernel<WK, WC, TK, TC, TAPS, U_LOADS, false, NS>;
    }
    if (lds_bytes > 48 * 1024 && !attr_done.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute((const void *)kern_full, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess ||
            hipFuncSetAttribute((const void *)kern_part, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
            return EOQ_ERR_HIP;
        attr_done.store(true, std::memory_order_release);
    }
    if ((size_t)p.N * p.P * p.Q * p.K > 0x7fffff00u || (size_t)p.N * p.H * p.W * p.C > 0x7fffff00u) return EOQ_ERR_SHAPE;
#ifdef EOQ_TUNE
    p.dbg = g_wtune_dbg ? g_wtune_dbg + (size_t)(g_wtune_launch++) * 4 * 8192 : nullptr;
#endif
    hipLaunchKernelGGL(RS % TAPS == 0 ? kern_full : kern_part, dim3((unsigned)(tiles * splits)), dim3(256), lds_bytes,
                       c->stream, p);
    EOQ_LAUNCH_CHECK();
    *splits_out = splits;   // number of partial buffers written
    return EOQ_OK;
}

// ---- scratch of the entry point that allocates nothing (eoq_conv_bwd_weight_static) ----------------------
// A file-scope device array: every GPU the library runs on holds its own copy, at its own address, until the
// process ends.  In host code the array's NAME is only a stand-in for the symbol, not a device address: the
// address is looked up once per device (wgrad_static_scratch_init, called by eoq_create with that device
// current) and only that pointer is ever handed to kernels.
constexpr size_t WGRAD_STATIC_BYTES = (size_t)32 << 20;
static __device__ __align__(256) unsigned char wgrad_static_scratch[WGRAD_STATIC_BYTES];
constexpr int WGRAD_MAX_DEVICES = 64;
std::mutex wgrad_static_mutex;
void *wgrad_static_ptr[WGRAD_MAX_DEVICES];

int wgrad_run(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *u, int32_t *g_acc,
              int32_t *absmax_slot, void *ws, size_t ws_bytes, bool caller_ws);

} // namespace

#ifdef EOQ_TUNE
extern "C" void eoq_tune_set_wdbg(unsigned long long *buf) { g_wtune_dbg = buf; g_wtune_launch = 0; }
extern "C" int eoq_tune_wlaunch_index() { return g_wtune_launch; }
#endif

int wgrad_static_scratch_init(int device, void **ptr_out)
{
    if (device < 0 || device >= WGRAD_MAX_DEVICES) return EOQ_ERR_ARG;
    std::lock_guard<std::mutex> lock(wgrad_static_mutex);
    if (!wgrad_static_ptr[device]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(wgrad_static_scratch)) != hipSuccess || !ptr) return EOQ_ERR_HIP;
        wgrad_static_ptr[device] = ptr;
    }
    *ptr_out = wgrad_static_ptr[device];
    return EOQ_OK;
}

extern "C" int eoq_conv_bwd_weight(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *u,
                                   int32_t *g_acc, int32_t *absmax_slot, void *ws, size_t ws_bytes)
{
    if (!c || !d) return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_workspace_bytes(d, EOQ_OP_CONV_BWD_WEIGHT) || ((uintptr_t)ws & 15)) {
        // (argument and shape errors are reported first, as before)
        const int rc = wgrad_run(c, d, e, u, g_acc, absmax_slot, nullptr, 0, true);
        return rc != EOQ_OK ? rc : EOQ_ERR_WORKSPACE;
    }
    return wgrad_run(c, d, e, u, g_acc, absmax_slot, ws, ws_bytes, true);
}

extern "C" int eoq_conv_bwd_weight_static(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *u,
                                          int32_t *g_acc, int32_t *absmax_slot)
{
    if (!c || !d) return EOQ_ERR_ARG;
    if (!c->static_scratch) return EOQ_ERR_HIP;
    return wgrad_run(c, d, e, u, g_acc, absmax_slot, c->static_scratch, WGRAD_STATIC_BYTES, false);
}

namespace {

// ws == nullptr: validate arguments and shape only (no launch).  caller_ws: the workspace was sized by
// eoq_workspace_bytes (its split cap applies); otherwise the split count is whatever fits ws_bytes.
int wgrad_run(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *u, int32_t *g_acc,
              int32_t *absmax_slot, void *ws, size_t ws_bytes, bool caller_ws)
{
    if (!c || !d || !e || !u || !g_acc || !absmax_slot) return EOQ_ERR_ARG;
    if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 || d->stride <= 0 ||
        d->pad < 0)
        return EOQ_ERR_SHAPE;
    const int P = conv_out_dim(d->H, d->pad, d->R, d->stride), Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    if (P <= 0 || Q <= 0 || d->K % 16) return EOQ_ERR_SHAPE;
    if (((uintptr_t)e | (uintptr_t)u | (uintptr_t)g_acc) & 15) return EOQ_ERR_ARG;
    if (!ws) return EOQ_OK;
    // bytes in front of the partial sums: the staged copy of a few-channel or odd-channel input
    // and the elements of one partial-sum buffer (rows padded like the staged input)
    size_t prefix = 0, part_elems = (size_t)d->K * d->R * d->S * d->C;
    if (d->C % 16 && d->C <= 4) {
        const Pad4Geom g = pad4_geom(d);
        prefix = round_up(g.img_bytes, 256) + round_up(g.w_bytes, 256);
        part_elems = (size_t)d->K * g.KP;
    } else if (d->C % 16) {
        const size_t KPx = round_up((size_t)d->R * d->S * d->C, 64);
        prefix = round_up((size_t)d->N * P * Q * KPx, 256) + round_up((size_t)d->K * KPx, 256);
        part_elems = (size_t)d->K * KPx;
    }
    if (prefix >= ws_bytes) return EOQ_ERR_WORKSPACE;
    // as many partial-sum buffers as the scratch holds, at most the cap eoq_workspace_bytes was sized for; the
    // shortest legal ranges (131072 terms) need at least min_splits of them -- all decided before the first launch
    size_t fit = (ws_bytes - prefix) / ((part_elems + WGRAD_PART_PAD) * 4);
    const size_t cap = (size_t)wgrad_max_splits(part_elems);
    if (caller_ws || fit > cap) fit = cap;
    const size_t min_splits = ((size_t)d->N * P * Q + 131071) / 131072;
    if (fit < 1 || fit < min_splits) return EOQ_ERR_WORKSPACE;
    const int max_splits = (int)fit;

    WgradParams p{};
    p.E = e;
    p.K = d->K;
    int32_t *part;
    const int rsc = d->R * d->S * d->C;
    int ld_in = rsc;
    bool pad4 = false;
    if (d->C % 16 == 0) {
        p.U = u;
        p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C; p.P = P; p.Q = Q;
        p.R = d->R; p.S = d->S; p.stride = d->stride; p.pad = d->pad;
        part = (int32_t *)ws;
    } else if (d->C <= 4) {
        // few-channel input (the stem): zero-bordered 4-bytes-per-pixel copy; a 1x1 weight gradient whose
        // "channels" are the R*S4 column groups of the filter window, gathered straight from that copy
        const Pad4Geom g = pad4_geom(d);
        if (g.img_bytes > 0x7fffff00u) return EOQ_ERR_SHAPE;
        int8_t *up = (int8_t *)ws;
        part = (int32_t *)((int8_t *)ws + round_up(g.img_bytes, 256) + round_up(g.w_bytes, 256));
        hipLaunchKernelGGL(wgrad_pad4_input_kernel, dim3(grid_for(g.img_bytes / 4)), dim3(256), 0, c->stream, u, d->N, d->H,
                           d->W, d->C, d->pad, g.Hp, g.Wp, (uint32_t *)up);
        EOQ_LAUNCH_CHECK();
        p.U = up;
        p.N = d->N; p.H = g.Hp; p.W = g.Wp; p.C = g.KP; p.P = P; p.Q = Q;
        p.R = 1; p.S = 1; p.stride = 1; p.pad = 0;
        p.pad4_S4 = g.S4; p.pad4_R = d->R; p.pad4_Wp = g.Wp; p.pad4_stride = d->stride;
        ld_in = g.KP;
        pad4 = true;
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
    p.part_stride = (size_t)p.K * p.RS * p.C + WGRAD_PART_PAD;
    if (p.part_stride != part_elems + WGRAD_PART_PAD) return EOQ_ERR_SHAPE;      // (cannot happen: same geometry)
    int splits = 0, rc;
    if (p.RS == 1) {
        if (p.K >= 128) rc = launch_wgrad<2, 2, 2, 2, 1, 2, 3>(c, p, p.RS, max_splits, &splits);
        else rc = launch_wgrad<2, 2, 1, 2, 1, 2, 3>(c, p, p.RS, max_splits, &splits);
    } else {
        if (p.R == 3 && p.S == 3 && p.stride == 1) rc = launch_wgrad<2, 2, 1, 1, 9, 2, 4>(c, p, p.RS, max_splits, &splits);
        else rc = launch_wgrad<2, 2, 1, 1, 9, 5, 3>(c, p, p.RS, max_splits, &splits);
    }
    if (rc != EOQ_OK) return rc;
    const size_t total = (size_t)d->K * rsc;
    if (ld_in == rsc && total % 4 == 0) {
        const size_t t4 = total / 4;
        auto blocks = [&](int qb) { size_t b = (t4 + qb - 1) / qb; return dim3((unsigned)(b > 4096 ? 4096 : b)); };
        // enough element groups to fill the chip: no split lanes (no LDS, no barriers); otherwise trade them in
        if (splits <= 4 || t4 >= 131072)
            hipLaunchKernelGGL(wgrad_finalize_v4_kernel<1>, blocks(256), dim3(256), 0, c->stream, part, p.part_stride, splits,
                               t4, g_acc, absmax_slot, c->d_status);
        else if (splits <= 32 || t4 >= 32768)
            hipLaunchKernelGGL(wgrad_finalize_v4_kernel<4>, blocks(64), dim3(256), 0, c->stream, part, p.part_stride, splits,
                               t4, g_acc, absmax_slot, c->d_status);
        else
            hipLaunchKernelGGL(wgrad_finalize_v4_kernel<16>, blocks(16), dim3(256), 0, c->stream, part, p.part_stride, splits,
                               t4, g_acc, absmax_slot, c->d_status);
    } else
        hipLaunchKernelGGL(wgrad_finalize_kernel, dim3(grid_for(total * 4)), dim3(256), 0, c->stream, part,
                           p.part_stride, splits, d->K, ld_in, rsc, g_acc, absmax_slot, c->d_status, pad4 ? d->S : 0,
                           d->C, pad4 ? p.pad4_S4 : 0);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

} // namespace
