// Implicit-GEMM int8 x int8 -> int32 convolution on MFMA for gfx950: the forward convolution of
// Eq.2 with its fused epilogue (Q_a1, multiplier, bias, shortcut, ReLU, Q_a2 -- Eq.9, Eq.10), and the
// backward-data convolution of Eq.3 (same kernel, gathering the error through the transposed
// filters) with the abs-max that the scale quantiser Q_e (Eq.11) needs fused into its epilogue.
//
// GEMM view: rows m = output pixels (N*P*Q), columns = output channels, reduction = (r, s, c).
// The reduction is walked in 16-byte pieces ("k-chunks": 16 consecutive input channels of one filter
// tap), four per LDS stage.  One MFMA v_mfma_i32_32x32x32_i8 consumes two k-chunks: lanes 0-31 supply
// the first, lanes 32-63 the second, identically for both operands, so any (tap, channel) order is
// legal as long as A and B agree.  A workgroup is 4 or 8 waves (WGM x WGN); each wave owns a (BM/WGM) x (BN/WGN)
// block of 32x32 MFMA tiles.  With 8 waves every SIMD hosts two of them, and the two run the phases of an
// iteration in opposite order (one multiplies while the other moves data through LDS): four waves in lockstep
// leave the matrix pipes idle while they all read LDS and the LDS idle while they all multiply.  Global -> register -> LDS software pipeline with two LDS buffers, one
// barrier per stage; LDS rows are 64 bytes with the 16-byte chunk index XOR-swizzled by (row/4)%4 so
// that both the 16-byte writes and the MFMA operand reads spread over all banks.
//
// Epilogue: each wave transposes its accumulators through LDS so that one lane owns 16 consecutive
// output channels of one pixel (16-byte int8 stores, 16-bit mask stores, 64-byte int32 stores).
#include "common.h"

#include <atomic>
#ifdef EOQ_TUNE
#include <cstdlib>
#endif

namespace {

struct EpiDev {
    const int32_t *gamma, *b_post, *b_next;
    const void *skip;
    int skip_wide, relu;             // skip_wide: 0 = int8 codes, 1 = int32, 2 = int16
    int t16;                         // t_wide points to int16 instead of int32
    int8_t *y, *u_next;
    uint16_t *mask16;
    int32_t *t_wide;
};

// One parity class of a stride-2 backward-data gather (up to four per launch): its own output grid, taps, filters
struct IgemmCls {
    int P, Q, R, S, pad, pad_w_delta, M, nk16;
    int rm_Hc, rm_Wc, rm_h0, rm_w0;
    int tile_base;                 // first workgroup tile of the class (= its first tile_shift entry)
    int b_off;                     // byte offset of the class's packed filters
    uint32_t mulQ, mulP;           // reciprocals of Q and P (see make_recip)
    int shQ, shP;
};

struct IgemmParams {
    const int8_t *A;   // input N x H x W x C
    const int8_t *B;   // filters NOUT x (R*S*C)
    int N, H, W, C;
    int P, Q, NOUT;
    int R, S, stride, pad;
    int M, nk16, c16;
    uint32_t mulQ, mulP;           // reciprocals of Q and P for the pixel decomposition (filled in by the dispatcher)
    int shQ, shP;
    int xstep;         // bytes per unit of the column origin (C, except for the 4-bytes-per-pixel stem layout)
    int no_pad;        // every tap of every row is in range (physically padded input)
    int gemm;          // 1x1 filter, stride 1, no padding: row m of the GEMM is pixel m of the input
    int32_t *acc_out;
    int32_t *absmax;
    uint32_t *status;  // device status word of the context
    EpiDev ep;
    int pad_w_delta;   // column padding minus row padding (0 except for the parity classes of a stride-2 gather)
    int ncls;          // > 0: the launch covers ncls independent problems that differ in the fields of IgemmCls
    IgemmCls cls[4];
    // EPI_D16: 16-bit block-scaled output of the backward-data convolution (one shift per workgroup tile)
    int16_t *d16;
    int32_t *tile_shift;
    int ts_base;       // first entry of this launch in tile_shift
    // EPI_D16 row remap (parity classes): GEMM row (n, gh, gw) of a rm_Hc x rm_Wc grid is input pixel
    // (n, 2*gh + rm_h0, 2*gw + rm_w0) of the rm_H x rm_W image
    int rm_on, rm_Hc, rm_Wc, rm_H, rm_W, rm_h0, rm_w0;
    // EPI_RELU_BWD: ReLU backward with the Q_a1 output recomputed instead of read back
    const int8_t *rb_e0;
    const uint16_t *rb_mask16;
    int8_t *rb_e1;
    int64_t *rb_sum_e1, *rb_sum_e1t;
    int64_t *rb_part;          // per-workgroup partial sums [tiles][2] (NULL: atomics on the two slots)
    int32_t *rb_absmax;
    // EPI_SPEC: speculative coding of the backward-data sums.  The scale quantiser's shift follows from max|d| of
    // the whole tensor, which is only known when the launch ends -- but it rarely changes from one training step
    // to the next.  The launch codes with the exponent of the previous step (spec[0]) and takes the true maximum on
    // the way; the two launches behind it compare (sp_check) and either commit the staged statistics or redo the
    // work the exact way (EPI_D16 + finishing kernel).  Results are those of the exact path in both cases.
    const int32_t *spec;       // [0] exponent r to try (negative: none yet); EPI_D16 / finish: non-NULL = check first
    int32_t *spec_used;        // scratch copy of spec[0], written by this launch for the two behind it
    int8_t *sp_e4, *sp_e1;     // codes, codes under the mask (either may be NULL)
    const uint16_t *sp_mask16; // mask of sp_e1, or of the merge statistics
    const int8_t *sp_other;    // merge statistics against this tensor ...
    const int32_t *sp_exp_in, *sp_exp_other;
    int32_t sp_exp_off;
    int64_t *sp_part;          // per-wave records {sum e4, sum e1, max merged, max merged under the mask}
#ifdef EOQ_TUNE
    int abl;                   // tuning builds: bit 0 = skip the loads, bit 1 = skip the MFMAs, bit 2 = skip the LDS reads
    unsigned long long *dbg;   // tuning builds: four timestamps per workgroup (entry, set-up done, reduction done, exit)
#endif
};

enum { MODE_FWD = 0, MODE_BWD_DATA = 1 };
enum { EPI_FWD = 0, EPI_ACC = 1, EPI_SPEC = 3, EPI_RELU_BWD = 4, EPI_D16 = 5 };

// did the speculative launch use the right exponent?  (every workgroup of the two launches behind it asks)
__device__ __forceinline__ bool spec_hit(const int32_t *absmax, const int32_t *spec_used)
{
    const uint32_t Mx = (uint32_t)*absmax;
    return (Mx ? sq_exponent_u32(Mx) : 7) == *spec_used;
}

// shifts of the merge (as merge_shifts) without raising a flag: the speculative launch must have no side effect
__device__ __forceinline__ void merge_shifts_quiet(int Ea, int Eb, int &sa, int &sb)
{
    const int Em = Ea < Eb ? Ea : Eb;
    sa = Ea - Em; sb = Eb - Em;
    sa = sa > 24 ? 24 : sa; sb = sb > 24 ? 24 : sb;
}

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
// FAST: z = gamma*t + 128*(b + skip) is known to fit 32 bits (decided once per launch from the accumulator
// bound and the scalar codes), so everything runs in full-rate 32-bit integer instructions; otherwise the
// same arithmetic is carried out in 64 bits.
// int8 shortcut codes are passed in a register (sk8): the caller fetches them for all of a thread's chunks before
// the first is processed, so their latency is paid once and not per chunk.  (Wide shortcut values -- one layer per
// stage -- are read here: holding 16 dwords per chunk ahead of time would cost the kernel its occupancy.)
template <bool FAST>
__device__ __forceinline__ void epilogue16(const int acc[16], size_t off, const EpiDev &ep, int32_t *acc_out,
                                           int gamma, int bpost, int bnext, uint32_t &range_bad, const v4i &sk8)
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
        if (ep.t16) {
            // 16-bit store (the caller knows |t| < 2^15 from the reduction length; a value that does not fit is
            // reported through the status word)
            uint32_t w2[8];
#pragma unroll
            for (int k = 0; k < 16; k += 2) {
                range_bad |= (uint32_t)(t[k] ^ __builtin_amdgcn_sbfe(t[k], 0, 16)) |
                             (uint32_t)(t[k + 1] ^ __builtin_amdgcn_sbfe(t[k + 1], 0, 16));
                w2[k >> 1] = ((uint32_t)t[k] & 0xffffu) | ((uint32_t)t[k + 1] << 16);
            }
            v4i *dst = (v4i *)((int16_t *)ep.t_wide + off);
            dst[0] = v4i{(int)w2[0], (int)w2[1], (int)w2[2], (int)w2[3]};
            dst[1] = v4i{(int)w2[4], (int)w2[5], (int)w2[6], (int)w2[7]};
        } else {
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                v4i w = {t[4 * k4], t[4 * k4 + 1], t[4 * k4 + 2], t[4 * k4 + 3]};
                ((v4i *)(ep.t_wide + off))[k4] = w;
            }
        }
    }
    if (!ep.relu) return;
    int sk[16];
    if (ep.skip) {
        if (ep.skip_wide == 2) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const v4i w = ((const v4i *)((const int16_t *)ep.skip + off))[h];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    sk[8 * h + 2 * j] = __builtin_amdgcn_sbfe(w[j], 0, 16);
                    sk[8 * h + 2 * j + 1] = w[j] >> 16;
                }
            }
        } else if (ep.skip_wide) {
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                const v4i w = ((const v4i *)((const int32_t *)ep.skip + off))[k4];
                sk[4 * k4] = w[0]; sk[4 * k4 + 1] = w[1]; sk[4 * k4 + 2] = w[2]; sk[4 * k4 + 3] = w[3];
            }
            if (FAST) {
                // the 32-bit path was chosen assuming |shortcut| < 2^22: anything a 23-bit signed field cannot
                // hold is reported through the status word instead of silently wrapping
#pragma unroll
                for (int k = 0; k < 16; ++k) range_bad |= (uint32_t)(sk[k] ^ __builtin_amdgcn_sbfe(sk[k], 0, 23));
            }
        } else {
#pragma unroll
            for (int k = 0; k < 16; ++k) sk[k] = byte_at(sk8, k);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) sk[k] = 0;
    }
    uint32_t yw[4] = {0, 0, 0, 0}, uw[4] = {0, 0, 0, 0};
    uint32_t mask = 0;
    const int b128 = bpost << 7;
    // channels are walked from 15 down to 0 so that the mask can be built by shifting one sign bit in per element
    // (alignbit(mask, -z, 31) = mask << 1 | [z > 0]; z != INT_MIN on the 32-bit path).  The three variants are
    // three separate loops: a uniform test inside the loop is not hoisted by the compiler and turns into a branch
    // per element.
    // y codes lie in [0, 127]: they are packed as they are produced, and the next layer's biased input
    // u = clamp(y + b_next, -127, 127) is then formed on whole dwords (see below) instead of element by element
    auto put = [&](int k, int yc) { yw[k >> 2] |= (uint32_t)yc << (8 * (k & 3)); };
    if (FAST && gamma == 128) {
        // multiplier exactly one (every layer without a multiplier, and a block's last layer until its multiplier
        // moves): z = 128 * (t + b + skip) is a multiple of 128, so Q_a2 rounds nothing and
        // y = clamp(t + b + skip, 0, 127), [z > 0] = [t + b + skip > 0] = [y > 0]
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int w = t[k] + sk[k] + bpost;
            put(k, w < 0 ? 0 : (w > CODE_MAX ? CODE_MAX : w));
        }
        // mask bits from the packed codes: byte + 127 carries into bit 7 iff the byte is non-zero (no carry between
        // bytes, a byte is at most 127); one multiply gathers the four bits
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t nz = ((yw[q] + 0x7f7f7f7fu) & 0x80808080u) >> 7;
            mask |= (((nz * 0x00204081u) >> 21) & 0xfu) << (4 * q);
        }
    } else if (FAST) {
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const int k = 15 - kk;
            const int z = __mul24(gamma, t[k]) + ((sk[k] << 7) + b128);      // both factors are below 2^23 here
            mask = __builtin_amdgcn_alignbit(mask, (uint32_t)(-z), 31);
            const int yc = rne_shift7(z);
            put(k, yc < 0 ? 0 : (yc > CODE_MAX ? CODE_MAX : yc));   // = clamp(R(max(z,0)/128)): R is monotone, R(0) = 0
        }
    } else {
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const int k = 15 - kk;
            const int64_t z = (int64_t)gamma * (int64_t)t[k] + 128 * ((int64_t)bpost + (int64_t)sk[k]);
            mask = (mask << 1) | (z > 0 ? 1u : 0u);
            const int64_t yy = rne_shift64(z > 0 ? z : 0, 7);
            put(k, (int)(yy > CODE_MAX ? CODE_MAX : yy));
        }
    }
    if (ep.u_next) {
        // bytes of yw are in [0, 127]
        if (bnext >= 0) {
            // min(y + b, 127): the byte sums stay below 256; a sum with bit 7 set saturates to 127
            const uint32_t b4 = (uint32_t)(bnext > CODE_MAX ? CODE_MAX : bnext) * 0x01010101u;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t sm = yw[q] + b4, ov = sm & 0x80808080u;
                uw[q] = (sm | (ov - (ov >> 7))) & 0x7f7f7f7fu;
            }
        } else if (bnext >= -CODE_MAX) {
            // y + b lies in [-127, 126]: no clamp; add the low seven bits (no carry between bytes), then fix bit 7
            const uint32_t b4 = ((uint32_t)bnext & 0xffu) * 0x01010101u;
#pragma unroll
            for (int q = 0; q < 4; ++q) uw[q] = (yw[q] + (b4 & 0x7f7f7f7fu)) ^ 0x80808080u;
        } else {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int uc = clamp_i((int)((yw[k >> 2] >> (8 * (k & 3))) & 0xffu) + bnext, -CODE_MAX, CODE_MAX);
                uw[k >> 2] |= ((uint32_t)uc & 0xffu) << (8 * (k & 3));
            }
        }
    }
    if (ep.y) *(v4i *)(ep.y + off) = v4i{(int)yw[0], (int)yw[1], (int)yw[2], (int)yw[3]};
    if (ep.u_next) *(v4i *)(ep.u_next + off) = v4i{(int)uw[0], (int)uw[1], (int)uw[2], (int)uw[3]};
    if (ep.mask16) ep.mask16[off >> 4] = (uint16_t)mask;
}

// z fits 32 bits for every element of the launch?  |t| <= tmax (from the reduction length), int8 shortcut
// codes are at most 127, wide shortcut values are Q_a1 outputs of another convolution (|.| < 2^22, i.e. R*S*C of
// that convolution below 33000; the epilogue checks every value it reads and raises EOQ_FLAG_ACC_OVERFLOW).
__device__ __forceinline__ bool epilogue_fits32(const EpiDev &ep, int gamma, int bpost, long long tmax)
{
    const long long ag = gamma < 0 ? -(long long)gamma : gamma, ab = bpost < 0 ? -(long long)bpost : bpost;
    const long long sk = ep.skip ? (ep.skip_wide == 1 ? (1ll << 22) : (ep.skip_wide == 2 ? (1ll << 15) : 127)) : 0;
    return ag < (1 << 23) && tmax < (1 << 23) && ag * tmax + 128 * (ab + sk) < (1ll << 31) - 256;
}

// Main loop: a ring of NS LDS stages (BK bytes of the reduction each) filled by direct-to-LDS loads -- no staging
// registers, no LDS writes by the waves -- one barrier per stage.  Two forms are instantiated:
//   BK = 64, NS = 2 at 128 registers per lane: FOUR workgroups per compute unit.  Measured per workgroup, a layer with a
//     short reduction spends most of its life outside the reduction (0.5-1 us of set-up, 2-6 us of epilogue against
//     2-6 us of loads and MFMAs), so such layers want workgroups in flight, not a deep pipeline; the second stage lets
//     the next loads fly while this stage is multiplied.
//   BK = 128, NS = 2 at 168 registers: whole 128-byte lines per row and load, half as many barriers; wins (by 15-20 %)
//     where at most two workgroups per compute unit exist anyway (the 14x14 layers with 256+ input channels).
// Rings of three and four stages, and 64-byte stages at three workgroups per compute unit, were measured and are no
// faster: the loop is bound by the rate at which a compute unit's memory path delivers 16-byte gathers
// (35-40 B/clk), not by their latency.
template <int BM, int BN, int WGM, int WGN, int BK, int NS, bool UNI, int MODE, int EPI>
__device__ __forceinline__ void igemm_body(const IgemmParams &pin)
{
#ifdef EOQ_TUNE
    const unsigned long long ts0 = __builtin_amdgcn_s_memrealtime();
#endif
    constexpr bool LEAN = BK == 64;                // compiled for 128 registers: epilogue side inputs two chunks ahead
    if (EPI == EPI_D16 && pin.spec && spec_hit(pin.absmax, pin.spec_used)) {           // the speculative launch was right
#ifdef EOQ_TUNE
        if (pin.dbg && threadIdx.x == 0 && blockIdx.x < 8192) {
            unsigned long long *r = pin.dbg + 4 * (size_t)blockIdx.x;
            r[0] = ts0; r[1] = r[2] = ts0; r[3] = __builtin_amdgcn_s_memrealtime();
        }
#endif
        return;
    }
    // (the recompute runs on the weight-gradient chain: see the note on wave priority in conv_wgrad.hip)
    if (EPI == EPI_RELU_BWD) __builtin_amdgcn_s_setprio(3);
    IgemmParams p = pin;           // uniform; patched below when the launch covers several classes
    constexpr int NW = WGM * WGN, NT = NW * 64;
    static_assert(NW == 4, "4 waves");
    static_assert(BK == 64 || BK == 128, "stage depth in bytes");
    static_assert(NS >= 2 && NS <= 4, "ring stages");
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    static_assert(TM >= 1 && TN >= 1, "tile");
    constexpr int CH = BK / 16;                 // k-chunks per LDS row
    constexpr int RPP = NT / CH;                // rows loaded per pass of the workgroup's threads
    constexpr int RP = 16 / CH;                 // rows per 256 bytes of LDS (swizzle period)
    constexpr int A_ROWS = (BM + RPP - 1) / RPP, B_ROWS = (BN + RPP - 1) / RPP;
    // (direct-to-LDS loads fill whole passes of RPP rows: the operand regions are padded to that)
    constexpr int A_REGION = A_ROWS * RPP * BK, B_REGION = B_ROWS * RPP * BK;
    constexpr int STAGE_BYTES = A_REGION + B_REGION;
    constexpr int EPI_LD = WTN + 4;                       // int32 row stride of the epilogue staging

    extern __shared__ __attribute__((aligned(16))) int8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int tiles_n = (p.NOUT + BN - 1) / BN;
    // consecutive workgroup ids go round-robin over the 8 XCDs: remap so that each XCD (own L2) works on
    // a contiguous range of tiles, i.e. neighbouring tiles share their operands in one L2
    int bid = blockIdx.x;
    {
        const int nb = gridDim.x, per = nb / 8;
        if (bid < per * 8) bid = (bid % 8) * per + bid / 8;
    }
    if (EPI == EPI_D16 && p.ncls) {
        int cl = 0;
#pragma unroll
        for (int i = 1; i < 4; ++i)
            if (i < p.ncls && bid >= p.cls[i].tile_base) cl = i;
        const IgemmCls &q = pin.cls[cl];
        p.P = q.P; p.Q = q.Q; p.R = q.R; p.S = q.S; p.pad = q.pad; p.pad_w_delta = q.pad_w_delta; p.M = q.M;
        p.mulQ = q.mulQ; p.shQ = q.shQ; p.mulP = q.mulP; p.shP = q.shP;
        p.nk16 = q.nk16; p.rm_Hc = q.rm_Hc; p.rm_Wc = q.rm_Wc; p.rm_h0 = q.rm_h0; p.rm_w0 = q.rm_w0;
        p.B = pin.B + q.b_off;
        p.ts_base = q.tile_base;
        bid -= q.tile_base;
    }
    const int tile_m = bid / tiles_n, tile_n = bid % tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- per-thread gather state: which rows / which k-chunk column this thread loads ----
    // Everything that depends on the row is folded once into a pointer and a 64-bit tap-validity mask, so the
    // loop only adds a per-stage tap offset (the same for all rows of a thread) and tests one mask bit.
    //   forward:       input pixel = (ho*stride - pad + r, wo*stride - pad + s)
    //   backward data: error pixel = ((ho + pad - r)/stride, (wo + pad - s)/stride) where both divide; for those
    //                  taps (ho+pad-r)/stride = floor((ho+pad)/stride) - floor(r/stride)
    // direct-to-LDS: lane l lands in slot l of its wave's kilobyte, so the swizzle is applied on the memory side --
    // the lane asks for the logical chunk that belongs in its slot
    const int lrow = tid / CH;
    const int kc = (tid % CH) ^ ((lrow / RP) % CH);
    // Buffer descriptors: a lane whose tap falls into the padding (or past the end of the reduction) gets an
    // offset beyond num_records and the hardware returns zeros -- no branch, no select.
    const __amdgpu_buffer_rsrc_t rsrc_a =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.A, 0, p.N * p.H * p.W * p.C, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b =
        __builtin_amdgcn_make_buffer_rsrc((void *)p.B, 0, p.NOUT * p.nk16 * 16, 0x00020000);
    constexpr int OOB = 0x7fffff00;
    int a_off[A_ROWS];
    unsigned long long a_mask[A_ROWS];
#pragma unroll
    for (int i = 0; i < A_ROWS; ++i) {
        const int row = lrow + RPP * i;
        const int m = m0 + row;
        const bool ok = (row < BM) && (m < p.M);
        const int mm = ok ? m : 0;
        if (p.gemm) {                              // uniform: no pixel decomposition, one always-valid tap
            a_mask[i] = ok ? 1ull : 0ull;
            a_off[i] = mm * p.C + kc * 16;
            continue;
        }
        // pixel decomposition by multiply-high with host-made reciprocals (an integer division costs ~40 instructions
        // per lane here, and every workgroup pays this set-up before its first load can leave)
        const int t = (int)fast_div((uint32_t)mm, p.mulQ, p.shQ);
        const int wo = mm - t * p.Q;
        const int n = (int)fast_div((uint32_t)t, p.mulP, p.shP);
        const int ho = t - n * p.P;
        int hb, wb;
        unsigned long long mask = 0;
        if (MODE == MODE_FWD || p.stride == 1) {
            // valid taps form a rectangle [r0, r1) x [s0, s1): one run of column bits, repeated for the valid rows
            int r0, r1, s0, s1;
            if (MODE == MODE_FWD) {
                hb = ho * p.stride - p.pad; wb = wo * p.stride - p.pad;
                r0 = max(0, -hb); r1 = min(p.R, p.H - hb);
                s0 = max(0, -wb); s1 = min(p.S, p.W - wb);
            } else {
                hb = ho + p.pad; wb = wo + p.pad + p.pad_w_delta;          // stride 1: the error pixel of tap r is hb - r
                r0 = max(0, hb - p.H + 1); r1 = min(p.R, hb + 1);
                s0 = max(0, wb - p.W + 1); s1 = min(p.S, wb + 1);
            }
            const unsigned long long colbits = s1 > s0 ? ((~0ull >> (64 - (s1 - s0))) << s0) : 0ull;
            for (int rr = 0; rr < p.R; ++rr)
                if (rr >= r0 && rr < r1) mask |= colbits << (rr * p.S);
        } else {
            const int hp = ho + p.pad, wp = wo + p.pad + p.pad_w_delta;
            hb = hp / p.stride; wb = wp / p.stride;
            const int hm = hp - hb * p.stride, wm_ = wp - wb * p.stride;
            int tap = 0;
            for (int rr = 0, rd = 0, rm = 0; rr < p.R; ++rr) {
                for (int ss = 0, sd = 0, sm = 0; ss < p.S; ++ss, ++tap) {
                    if (rm == hm && sm == wm_ && (unsigned)(hb - rd) < (unsigned)p.H && (unsigned)(wb - sd) < (unsigned)p.W)
                        mask |= 1ull << tap;
                    if (++sm == p.stride) { sm = 0; ++sd; }
                }
                if (++rm == p.stride) { rm = 0; ++rd; }
            }
        }
        if (p.no_pad) mask = ~0ull;
        a_mask[i] = ok ? mask : 0ull;
        a_off[i] = (n * p.H + hb) * p.W * p.C + wb * p.xstep + kc * 16;
    }
    int b_off[B_ROWS];
    bool b_ok[B_ROWS];
#pragma unroll
    for (int i = 0; i < B_ROWS; ++i) {
        const int row = lrow + RPP * i;
        const int nr = n0 + row;
        b_ok[i] = row < BN && nr < p.NOUT;
        b_off[i] = b_ok[i] ? (nr * p.nk16 + kc) * 16 : 0;
    }
    const int wc_step = p.W * p.C;
    // Position of the stage being loaded.  UNI (C a multiple of the stage depth): every chunk of a stage lies in
    // one filter tap, so tap, channel base and offsets are wave-uniform scalars.  Otherwise (C = 16, 32) each
    // thread derives its own tap from its chunk index.
    int ld_r = 0, ld_s = 0, ld_cb = 0, ld_rd = 0, ld_rm = 0, ld_sd = 0, ld_sm = 0, ld_kk = 0;

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    const int lrow32 = lane & 31, lhalf = lane >> 5;
    // LDS read offsets: the swizzle term is the same for every 32-row tile of a wave (32 is a multiple of the
    // swizzle period), so one offset per reduction step and operand is enough; tiles add a constant.
    int rd_a[CH / 2], rd_b[CH / 2];
#pragma unroll
    for (int j = 0; j < CH / 2; ++j) {
        const int chunk = 2 * j + lhalf;
        const int rowa = wm * WTM + lrow32, rowb = wn * WTN + lrow32;
        rd_a[j] = rowa * BK + ((chunk ^ ((rowa / RP) % CH)) << 4);
        rd_b[j] = A_REGION + rowb * BK + ((chunk ^ ((rowb / RP) % CH)) << 4);
    }
    // MFMA operands are double-buffered in registers: the fragments of stage st+1 are read from LDS while
    // the MFMAs of stage st run, so neither the LDS latency nor the global latency sits on the critical path.
    auto read_frags = [&](int buf, v4i (&fa)[CH / 2][TM], v4i (&fb)[CH / 2][TN]) {
        const int8_t *base = lds + buf;
#pragma unroll
        for (int j = 0; j < CH / 2; ++j) {
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[j][i] = *(const v4i *)(base + rd_a[j] + i * 32 * BK);
#pragma unroll
            for (int i = 0; i < TN; ++i) fb[j][i] = *(const v4i *)(base + rd_b[j] + i * 32 * BK);
        }
    };
    auto mfma_half = [&](int j, const v4i (&fa)[CH / 2][TM], const v4i (&fb)[CH / 2][TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
                acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[j][i], fb[j][jn], acc[i][jn], 0, 0, 0);
    };

    const int nstages = (p.nk16 + CH - 1) / CH;
#ifdef EOQ_TUNE
    const unsigned long long ts1 = __builtin_amdgcn_s_memrealtime();
#endif
    {
        // Ring of NS LDS stages filled by direct-to-LDS loads.  Stage st lives in buffer st % NS.  Iteration st:
        //     wait until this thread's loads of stage st have landed | barrier | request stage st+NS-1 | multiply stage st
        // After the barrier every wave's part of stage st is in LDS, and every wave has finished reading stage st-1
        // (its fragments were consumed by MFMAs issued before the barrier), whose buffer is the one stage st+NS-1
        // goes to.  Loads past the end of the reduction are out of range: no traffic, zeros written, never
        // multiplied -- so every iteration issues the same number of loads and the wait count is a constant.
        constexpr int L = A_ROWS + B_ROWS;              // loads per thread and stage
        static_assert((NS - 1) * L < 64, "vmcnt range");
        const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
        const uint32_t wave_base = lds0 + (uint32_t)__builtin_amdgcn_readfirstlane(wave) * (64 / CH) * BK;
        const uint64_t pa = (uint64_t)p.A, pb = (uint64_t)p.B;
        const v4i rs_a = {(int)(uint32_t)pa, (int)((uint32_t)(pa >> 32) & 0xffffu), p.N * p.H * p.W * p.C, 0x00020000};
        const v4i rs_b = {(int)(uint32_t)pb, (int)((uint32_t)(pb >> 32) & 0xffffu), p.NOUT * p.nk16 * 16, 0x00020000};
        auto dma_stage = [&](int buf) {
            bool tap_ok;
            int tap, toff;
            if (UNI) {
                tap_ok = ld_r < p.R;
                tap = tap_ok ? ld_r * p.S + ld_s : 0;
                if (MODE == MODE_FWD) toff = ld_r * wc_step + ld_s * p.C + ld_cb * 16;
                else toff = -(ld_rd * wc_step + ld_sd * p.C) + ld_cb * 16;
            } else {
                const int kk = ld_kk + kc;
                tap_ok = kk < p.nk16;
                const int tp = kk / p.c16, cc = kk - tp * p.c16;
                const int rr = tp / p.S, ss = tp - rr * p.S;
                tap = tap_ok ? tp : 0;
                if (MODE == MODE_FWD) toff = rr * wc_step + ss * p.C + cc * 16;
                else toff = -((rr / p.stride) * wc_step + (ss / p.stride) * p.C) + cc * 16;
                toff -= kc * 16;
            }
#pragma unroll
            for (int i = 0; i < A_ROWS; ++i) {
                const bool v = tap_ok && ((a_mask[i] >> tap) & 1ull);
                lds_direct_load16(rs_a, wave_base + buf + i * RPP * BK, v ? a_off[i] + toff : OOB);
            }
#pragma unroll
            for (int i = 0; i < B_ROWS; ++i)
                lds_direct_load16(rs_b, wave_base + buf + A_REGION + i * RPP * BK,
                                  (tap_ok && b_ok[i]) ? b_off[i] + ld_kk * 16 : OOB);
            ld_kk += CH;
            if (UNI) {
                ld_cb += CH;
                if (ld_cb == p.c16) {
                    ld_cb = 0;
                    ++ld_s;
                    if (++ld_sm == p.stride) { ld_sm = 0; ++ld_sd; }
                    if (ld_s == p.S) {
                        ld_s = 0; ld_sd = 0; ld_sm = 0;
                        ++ld_r;
                        if (++ld_rm == p.stride) { ld_rm = 0; ++ld_rd; }
                    }
                }
            }
        };
#pragma unroll
        for (int d = 0; d < NS - 1; ++d) dma_stage(d * STAGE_BYTES);
        int cur = 0;
        v4i fa[CH / 2][TM], fb[CH / 2][TN];
#ifdef EOQ_TUNE
#pragma unroll
        for (int j = 0; j < CH / 2; ++j) {
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[j][i] = v4i{tid, 1, 2, 3};
#pragma unroll
            for (int i = 0; i < TN; ++i) fb[j][i] = v4i{tid, 5, 6, 7};
        }
#endif
        for (int st = 0; st < nstages; ++st) {
            wait_vmcnt<(NS - 2) * L>();
            __syncthreads();
#ifdef EOQ_TUNE
            if (!(p.abl & 1)) dma_stage(cur == 0 ? (NS - 1) * STAGE_BYTES : cur - STAGE_BYTES);
            __builtin_amdgcn_sched_barrier(0);
            if (!(p.abl & 4)) read_frags(cur, fa, fb);
            if (!(p.abl & 2)) {
#pragma unroll
                for (int j = 0; j < CH / 2; ++j) mfma_half(j, fa, fb);
            } else {
#pragma unroll
                for (int j = 0; j < CH / 2; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i) acc[i][0][0] += fa[j][i][0] + fb[j][0][1];    // keep the reads alive
            }
#else
            dma_stage(cur == 0 ? (NS - 1) * STAGE_BYTES : cur - STAGE_BYTES);
            __builtin_amdgcn_sched_barrier(0);
            read_frags(cur, fa, fb);
#pragma unroll
            for (int j = 0; j < CH / 2; ++j) mfma_half(j, fa, fb);
#endif
            __builtin_amdgcn_sched_barrier(0);
            cur = cur + STAGE_BYTES == NS * STAGE_BYTES ? 0 : cur + STAGE_BYTES;
        }
        wait_vmcnt<0>();          // the tail's out-of-range loads still write (zeros): they land before LDS is reused
        __syncthreads();
    }

#ifdef EOQ_TUNE
    const unsigned long long ts2 = __builtin_amdgcn_s_memrealtime();
#endif
    // ---- epilogue ----
    // Block-scaled 16-bit output (the scale quantiser of Eq.11 needs max|d| of the WHOLE tensor before any element
    // can be coded, so the exact 32-bit sums would have to be stored or recomputed).  Instead each workgroup keeps,
    // relative to the largest magnitude of ITS tile, the top 14 bits of every sum plus a sticky bit (any dropped
    // bit set) -- 16 bits per element.  The final rounding position r-7 (r from the global maximum) lies at least 6
    // bits above the dropped bits of every tile, so round-half-even of the exact sum is recovered exactly from
    // (kept bits, sticky bit): the rounding bit is a kept bit and the sticky bit joins the bits below it.
    int sp_sh = 0, sp_sa = 0, sp_sb = 0, sp_mx = 0, sp_mxm = 0, sp_tmax = 0, sp_tmin = 0;
    long long sp_s1 = 0;
    if (EPI == EPI_SPEC) {
        int r = p.spec[0];
        if (blockIdx.x == 0 && tid == 0) *p.spec_used = r;
        r = r < 0 ? 7 : (r > 31 ? 31 : r);                     // nothing to try yet: any shift will do, the result is redone
        sp_sh = r - 7;
        if (p.sp_other) merge_shifts_quiet(*p.sp_exp_in + p.sp_exp_off + sp_sh, *p.sp_exp_other, sp_sa, sp_sb);
    }
    int d16_s = 0;
    if (EPI == EPI_D16) {
        int mx0 = 0, mn0 = 0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
#pragma unroll
                for (int e = 0; e < 16; e += 2) {
                    // largest and smallest value, two elements per max3 / min3 (one instruction per element; |v| via
                    // negate-and-max would take two)
                    const int a = acc[i][jn][e], b = acc[i][jn][e + 1];
                    mx0 = max(max(mx0, a), b);
                    mn0 = min(min(mn0, a), b);
                }
        mx0 = wave_max_i32(max(mx0, -mn0));
        int *red = (int *)lds;                       // the main loop is done with LDS (barrier above)
        if (lane == 0) red[wave] = mx0;
        __syncthreads();
        int tmax = red[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) tmax = red[w] > tmax ? red[w] : tmax;
        __syncthreads();                             // before the staging below overwrites red[]
        const int ploc = tmax ? 31 - __clz(tmax) : 0;
        d16_s = ploc > 13 ? ploc - 13 : 0;
        if (tid == 0) {
            slot_atomic_max_i32(p.absmax, tmax);
            p.tile_shift[p.ts_base + bid] = d16_s;
        }
    }
    // per wave, 32 rows at a time through LDS
    long long sq_sum = 0, rb_st = 0;
    constexpr int GROUPS = WTN / 16;              // 16-channel groups per row of the wave tile
    constexpr int ROWS_PER_PASS = 64 / GROUPS;
    constexpr int SR = ROWS_PER_PASS <= 16 ? 16 : 32;
    int32_t *stg = (int32_t *)lds + wave * SR * EPI_LD;
    const int grp = lane % GROUPS, prow = lane / GROUPS;
    int gamma = 128, bpost = 0, bnext = 0;
    bool fast = false;
    if (EPI == EPI_FWD) {
        if (p.ep.gamma) gamma = *p.ep.gamma;
        if (p.ep.b_post) bpost = *p.ep.b_post;
        if (p.ep.b_next) bnext = *p.ep.b_next;
        fast = epilogue_fits32(p.ep, gamma, bpost, (127ll * 127 * 16 * p.nk16) / 128 + 1);
    }
    int mx = 0;
    uint32_t range_bad = 0;
    // Side inputs of the epilogue (shortcut values; incoming error and mask words for the ReLU backward step) are
    // requested ahead of the chunk that uses them, so that their latency is not paid chunk by chunk.  The pipelined
    // form asks for ALL chunks of the thread before the first is staged (the registers of the main loop's load ring
    // are free by now); the low-register form keeps PD chunks in flight and refills a slot as soon as it is consumed.
    constexpr int NPASS = 32 / ROWS_PER_PASS;
    constexpr int TP = TM * NPASS;                                   // chunks per thread
    constexpr bool HAS_SIDE = EPI == EPI_FWD || EPI == EPI_RELU_BWD || EPI == EPI_SPEC;
    // (the 2 x 2 forward layout with 128-column tiles serves the layers without ReLU, which have no int8 side input,
    // and is short of registers as it is)
    constexpr bool NO_RING = LEAN && EPI == EPI_FWD && WGN == 2 && BN == 128;
    constexpr int PD = !HAS_SIDE || NO_RING ? 0 : (!LEAN ? TP : (TP < 2 ? TP : 2));
    v4i ring8[PD > 0 ? PD : 1];
    uint32_t ringmk[PD > 0 ? PD : 1];
    auto load_side = [&](int t, v4i &s8, uint32_t &smk) {
        const int i = t / NPASS, ps = t % NPASS;
        const int m = m0 + wm * WTM + i * 32 + ps * ROWS_PER_PASS + prow;
        const int ch = n0 + wn * WTN + grp * 16;
        s8 = v4i{0, 0, 0, 0};
        smk = 0xffffu;
        if (m < p.M && ch < p.NOUT) {
            const size_t off = (size_t)m * p.NOUT + ch;
            if (EPI == EPI_FWD) {
                if (p.ep.skip && p.ep.relu && !p.ep.skip_wide) s8 = *(const v4i *)((const int8_t *)p.ep.skip + off);
            } else if (EPI == EPI_SPEC) {
                if (p.sp_other) s8 = *(const v4i *)(p.sp_other + off);
                if (p.sp_mask16) smk = (uint32_t)p.sp_mask16[off >> 4];
            } else if (EPI == EPI_RELU_BWD) {
                s8 = *(const v4i *)(p.rb_e0 + off);
                if (p.rb_mask16) smk = (uint32_t)p.rb_mask16[off >> 4];
            }
        }
    };
#pragma unroll
    for (int t = 0; t < PD; ++t) load_side(t, ring8[t], ringmk[t]);
    // SR rows of a 32-row accumulator block are staged at a time: 16 where a pass covers at most 16 rows, which
    // halves the staging area -- for 128-column wave tiles that is the difference between two and four workgroups
    // per compute unit
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int hf = 0; hf < 32 / SR; ++hf) {
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int e = hf * (SR / 2); e < (hf + 1) * (SR / 2); ++e) {
                int row = (e >> 2) * 8 + lhalf * 4 + (e & 3) - hf * SR;
                stg[row * EPI_LD + jn * 32 + lrow32] = acc[i][jn][e];
            }
        __syncthreads();   // (each wave reads back only what it wrote itself)
#pragma unroll
        for (int ps = hf * (SR / ROWS_PER_PASS); ps < (hf + 1) * (SR / ROWS_PER_PASS); ++ps) {
            const int row = ps * ROWS_PER_PASS + prow;
            const int m = m0 + wm * WTM + i * 32 + row;
            const int ch = n0 + wn * WTN + grp * 16;
            int v[16];
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                v4i w = *(const v4i *)(stg + (row - hf * SR) * EPI_LD + grp * 16 + 4 * k4);
                v[4 * k4] = w[0]; v[4 * k4 + 1] = w[1]; v[4 * k4 + 2] = w[2]; v[4 * k4 + 3] = w[3];
            }
            v4i side8 = v4i{0, 0, 0, 0};
            uint32_t sidemk = 0xffffu;
            if (HAS_SIDE) {
                const int t = i * NPASS + ps;
                if (PD > 0) {
                    side8 = ring8[t % (PD > 0 ? PD : 1)];
                    sidemk = ringmk[t % (PD > 0 ? PD : 1)];
                    if (t + PD < TP) load_side(t + PD, ring8[t % (PD > 0 ? PD : 1)], ringmk[t % (PD > 0 ? PD : 1)]);
                } else {
                    load_side(t, side8, sidemk);
                }
            }
            if (m < p.M && ch < p.NOUT) {
                size_t off = (size_t)m * p.NOUT + ch;
                if (EPI == EPI_D16 && p.rm_on) {
                    const int hw = p.rm_Hc * p.rm_Wc;
                    const int n = m / hw, r = m - n * hw;
                    const int gh = r / p.rm_Wc, gw = r - gh * p.rm_Wc;
                    off = ((size_t)(n * p.rm_H + 2 * gh + p.rm_h0) * p.rm_W + 2 * gw + p.rm_w0) * p.NOUT + ch;
                }
                if (EPI == EPI_FWD) {
                    if (fast) epilogue16<true>(v, off, p.ep, p.acc_out, gamma, bpost, bnext, range_bad, side8);
                    else epilogue16<false>(v, off, p.ep, p.acc_out, gamma, bpost, bnext, range_bad, side8);
                } else if (EPI == EPI_RELU_BWD) {
                    // Eq.3 e1 = e0 * relu'(x4); Eq.4 sums for g_b2 and g_gamma with x2 = R(acc/128) recomputed
                    const v4i ev = side8;
                    const uint32_t mk = sidemk;
                    v4i o = {0, 0, 0, 0};
                    int ls = 0, lst = 0;
                    // |x2| <= 127^2 * (reduction length) / 128 and |e| <= 127: for reductions of up to 8192
                    // terms sixteen products sum to less than 2^31 and are added in 32 bits
                    const bool narrow = p.nk16 <= 512;
                    if (narrow && !p.rb_e1 && !p.rb_absmax && !p.rb_mask16) {
                        // sums only (the multiplier's gradient): no codes to store, no mask, no maximum
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            ls = sum4_i8((uint32_t)ev[q], ls);
#pragma unroll
                            for (int k = 0; k < 4; ++k)
                                lst += __mul24(__builtin_amdgcn_sbfe(ev[q], 8 * k, 8), rne_shift7(v[4 * q + k]));
                        }
                    } else
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const int e = ((mk >> k) & 1u) ? byte_at(ev, k) : 0;
                        set_byte(o, k, e);
                        ls += e;
                        const int ae = e < 0 ? -e : e;
                        mx = ae > mx ? ae : mx;
                        if (narrow) lst += __mul24(e, rne_shift7(v[k]));
                        else rb_st += (long long)e * (long long)rne_shift7(v[k]);
                    }
                    sq_sum += ls;
                    rb_st += lst;
                    if (p.rb_e1) *(v4i *)(p.rb_e1 + off) = o;
                } else if (EPI == EPI_SPEC) {
                    // Q_e (Eq.11) with the exponent being tried: clamp(R(v * 2^-sh)); |v| < 2^30, 32 bits are exact
                    uint32_t o4[4], o1[4];
                    int ls4 = 0, ls1 = 0;
                    int cd16[16];
                    if (sp_sh <= 0) {                          // (uniform; two loops so that no element carries a branch)
#pragma unroll
                        for (int k = 0; k < 16; ++k) cd16[k] = sq_code32<true>(v[k], sp_sh);
                    } else {
#pragma unroll
                        for (int k = 0; k < 16; ++k) cd16[k] = sq_code32<false>(v[k], sp_sh);
                    }
#pragma unroll
                    for (int k = 0; k < 16; k += 2) {          // running maximum and minimum: max|v| = max(hi, -lo)
                        sp_tmax = max(max(sp_tmax, v[k]), v[k + 1]);
                        sp_tmin = min(min(sp_tmin, v[k]), v[k + 1]);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int *cd = cd16 + 4 * q;
                        const uint32_t pk = pack4_i8(cd[0], cd[1], cd[2], cd[3]);
                        o4[q] = pk;
                        ls4 = sum4_i8(pk, ls4);
                        if (p.sp_e1) {
                            const uint32_t pm = pk & byte_mask4(sidemk >> (4 * q));
                            o1[q] = pm;
                            ls1 = sum4_i8(pm, ls1);
                        }
                        if (p.sp_other) {
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                int mv = (cd[k] << sp_sa) + (__builtin_amdgcn_sbfe(side8[q], 8 * k, 8) << sp_sb);
                                mv = mv < 0 ? -mv : mv;
                                sp_mx = mv > sp_mx ? mv : sp_mx;
                                const int mm = ((sidemk >> (4 * q + k)) & 1u) ? mv : 0;
                                sp_mxm = mm > sp_mxm ? mm : sp_mxm;
                            }
                        }
                    }
                    sq_sum += ls4;
                    sp_s1 += ls1;
                    if (p.sp_e4) *(v4i *)(p.sp_e4 + off) = v4i{(int)o4[0], (int)o4[1], (int)o4[2], (int)o4[3]};
                    if (p.sp_e1) *(v4i *)(p.sp_e1 + off) = v4i{(int)o1[0], (int)o1[1], (int)o1[2], (int)o1[3]};
                } else if (EPI == EPI_D16) {
                    const int smask = (1 << d16_s) - 1;
                    uint32_t w8[8];
#pragma unroll
                    for (int k = 0; k < 16; k += 2) {
                        const int a = v[k], b = v[k + 1];
                        const uint32_t qa = (uint32_t)(((a >> d16_s) << 1) | (((a & smask) + smask) >> d16_s));
                        const uint32_t qb = (uint32_t)(((b >> d16_s) << 1) | (((b & smask) + smask) >> d16_s));
                        w8[k >> 1] = (qa & 0xffffu) | (qb << 16);
                    }
                    v4i *dst = (v4i *)(p.d16 + off);
                    dst[0] = v4i{(int)w8[0], (int)w8[1], (int)w8[2], (int)w8[3]};
                    dst[1] = v4i{(int)w8[4], (int)w8[5], (int)w8[6], (int)w8[7]};
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
    }
#ifdef EOQ_TUNE
    if (pin.dbg && tid == 0 && blockIdx.x < 8192) {
        unsigned long long *r = pin.dbg + 4 * (size_t)blockIdx.x;
        r[0] = ts0; r[1] = ts1; r[2] = ts2; r[3] = __builtin_amdgcn_s_memrealtime();
    }
#endif
    if (EPI == EPI_FWD && range_bad) atomicOr(p.status, (uint32_t)EOQ_FLAG_ACC_OVERFLOW);
    if (EPI == EPI_ACC && p.absmax) block_atomic_max_i32(mx, p.absmax);
    if (EPI == EPI_SPEC) {
        // the true maximum (needed whatever the guess was) and this wave's record for the committing launch
        const int tm = wave_max_i32(max(sp_tmax, -sp_tmin));
        const int64_t a = wave_sum_i64(sq_sum), b = wave_sum_i64(sp_s1);
        const int ma = wave_max_i32(sp_mx), mb = wave_max_i32(sp_mxm);
        if (lane == 0) {
            slot_atomic_max_i32(p.absmax, tm);
            int64_t *rec = p.sp_part + 4 * (size_t)(NW * bid + wave);
            rec[0] = a; rec[1] = b; rec[2] = ma; rec[3] = mb;
        }
    }
    if (EPI == EPI_RELU_BWD) {
        if (p.rb_part) {
            // thousands of workgroups adding to two slots would queue up behind each other: each wave stores its
            // own pair (no barrier, no shared memory), a one-block kernel adds them up afterwards
            const int64_t a = wave_sum_i64(sq_sum), b = wave_sum_i64(rb_st);
            if (lane == 0) { p.rb_part[2 * (NW * bid + wave)] = a; p.rb_part[2 * (NW * bid + wave) + 1] = b; }
        } else {
            if (p.rb_sum_e1) block_atomic_add_i64(sq_sum, p.rb_sum_e1);
            if (p.rb_sum_e1t) block_atomic_add_i64(rb_st, p.rb_sum_e1t);
        }
        if (p.rb_absmax) {
            const int wm_ = wave_max_i32(mx);
            if (lane == 0) slot_atomic_max_i32(p.rb_absmax, wm_);
        }
    }
}

// 64-byte stages: four workgroups per compute unit (128 registers per lane)
template <int BM, int BN, int WGM, int WGN, int BK, int NS, bool UNI, int MODE, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64, 4) void igemm_kernel(IgemmParams pin)
{
    igemm_body<BM, BN, WGM, WGN, BK, NS, UNI, MODE, EPI>(pin);
}

// 128-byte stages (64 KB of LDS per workgroup, two per compute unit): 168 registers per lane
template <int BM, int BN, int WGM, int WGN, int BK, int NS, bool UNI, int MODE, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64, 3) void igemm_wide_kernel(IgemmParams pin)
{
    igemm_body<BM, BN, WGM, WGN, BK, NS, UNI, MODE, EPI>(pin);
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

// Filters of the four parity classes of a stride-2 backward-data gather: class (a, b) takes the taps r = a, a+2, ..
// and s = b, b+2, .. of the K x R x S x C filters, stored as C x Ra x Sa x K (the operand order of the gather) at
// byte offset base[2a+b].
struct ClsPack { int base[4], Ra[2], Sa[2]; };
__global__ void pack_class_filters_kernel(const int8_t *w, int K, int R, int S, int C, ClsPack cp, int8_t *wc)
{
    const size_t total = (size_t)K * R * S * C;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int k = (int)(i % K);             // walk the OUTPUT order of the largest class so that writes coalesce
        size_t t = i / K;
        const int s = (int)(t % S); t /= S;
        const int r = (int)(t % R);
        const int c = (int)(t / R);
        const int a = r & 1, b = s & 1, r2 = r >> 1, s2 = s >> 1;
        wc[cp.base[2 * a + b] + (((size_t)c * cp.Ra[a] + r2) * cp.Sa[b] + s2) * K + k] =
            w[(((size_t)k * R + r) * S + s) * C + c];
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

// input N x H x W x C (C <= 4)  ->  zero-bordered N x Hp x Wp x 4
__global__ void pad4_input_kernel(const int8_t *u, int N, int H, int W, int C, int pad, int Hp, int Wp, uint32_t *up)
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

// filters K x R x S x C (C <= 4)  ->  K x R x S4 x (4 columns x 4 channels), zero padded
__global__ void pad4_filters_kernel(const int8_t *w, int K, int R, int S, int C, int S4, int8_t *wp)
{
    const size_t total = (size_t)K * R * S4 * 16;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(i & 3), sl = (int)((i >> 2) & 3);
        size_t t = i >> 4;
        const int j = (int)(t % S4); t /= S4;
        const int r = (int)(t % R), k = (int)(t / R);
        const int s = 4 * j + sl;
        wp[i] = (s < S && c < C) ? w[(((size_t)k * R + r) * S + s) * C + c] : (int8_t)0;
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
__global__ void requant_fwd_kernel(const int32_t *acc, size_t n16, EpiDev ep, uint32_t *status)
{
    const int gamma = ep.gamma ? *ep.gamma : 128, bpost = ep.b_post ? *ep.b_post : 0, bnext = ep.b_next ? *ep.b_next : 0;
    uint32_t range_bad = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
        int v[16];
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
            v4i w = ((const v4i *)acc)[i * 4 + k4];
            v[4 * k4] = w[0]; v[4 * k4 + 1] = w[1]; v[4 * k4 + 2] = w[2]; v[4 * k4 + 3] = w[3];
        }
        v4i sk8 = {0, 0, 0, 0};
        if (ep.skip && ep.relu && !ep.skip_wide) sk8 = *(const v4i *)((const int8_t *)ep.skip + i * 16);
        epilogue16<false>(v, i * 16, ep, nullptr, gamma, bpost, bnext, range_bad, sk8);
    }
    if (range_bad) atomicOr(status, (uint32_t)EOQ_FLAG_ACC_OVERFLOW);      // a wide value that does not fit its 16-bit store
}

// adds up the per-wave pairs of partial sums (a handful of blocks: two atomics each)
__global__ __launch_bounds__(1024) void pair_reduce_kernel(const int64_t *part, int n, int64_t *sum0, int64_t *sum1)
{
    int64_t a = 0, b = 0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        a += part[2 * i];
        b += part[2 * i + 1];
    }
    a = block_sum_i64(a);
    b = block_sum_i64(b);
    if (threadIdx.x == 0) {
        if (sum0 && a) atomic_add_i64(sum0, a);
        if (sum1 && b) atomic_add_i64(sum1, b);
    }
}

// Second half of the fused backward-data + Q_e call: turns the block-scaled 16-bit sums into the final codes
// e4 = clamp(R(d * 2^(7-r))), r = R(log2 max|d|) (Eq.11), and optionally applies the ReLU backward step of the layer
// below (Eq.3: e1 = e4 * relu'(x4), mask bit per element) with its sums (Eq.4).  One lane: 16 channels of one pixel.
struct D16Finish {
    const int16_t *d16;
    const int32_t *tile_shift;
    int bm_shift, bn_shift, tiles_n;       // tile of element (m, c): (m >> bm_shift) * tiles_n + (c >> bn_shift)
    size_t M;
    int C;
    const int32_t *absmax, *exp_in;
    int32_t exp_in_off;
    int32_t *exp_out;
    int8_t *e4;
    int64_t *sum_e4;
    const uint16_t *mask16;
    int8_t *e1;
    int64_t *sum_e1;
    int32_t *absmax_e1;
    // block-input merge statistics: max|e4 * 2^(E4-Em) + other * 2^(Eo-Em)|, Em = min(E4, Eo)
    const int8_t *mg_other;
    const int32_t *mg_exp_other;
    int32_t *mg_absmax;
    const uint16_t *mg_mask16;       // with mg_absmax_m: the same maximum over the elements whose mask bit is set
    int32_t *mg_absmax_m;
    uint32_t *status;
    // strided 1x1 filter: the sums exist only for the input pixels the filter touched (every sub-th row and column),
    // stored compactly as N x P x Q rows; all other input pixels receive no error
    int sub, H, W, P, Q;
    // stride-2 filters larger than 1x1: four launches, one per parity class (a, b) of (h + pad, w + pad); the sums sit
    // at their final positions, only the tile of an element (for its shift) depends on the class
    int cls_on, cls_pad;
    int cls_hh0[2], cls_ww0[2], cls_Hc[2], cls_Wc[2];
    int cls_base[4], cls_bm_shift[4], cls_bn_shift[4], cls_tiles_n[4];
    // behind a speculative launch (see IgemmParams::spec): if its exponent was right, this kernel only commits what
    // that launch staged -- the per-wave records of sums and maxima -- and stores the exponent for the next step
    int32_t *spec;
    const int32_t *spec_used;
    const int64_t *sp_part;
    int sp_records;
    int32_t *counters;                 // [0] += 1 when the exponent tried was right, [1] += 1 when it was not
};

template <bool RELU>
__global__ __launch_bounds__(1024) void d16_finish_kernel(D16Finish p)
{
    const uint32_t Mx = (uint32_t)*p.absmax;
    const int r = Mx ? sq_exponent_u32(Mx) : 7;
    const int sh = r - 7;
    const int E4 = *p.exp_in + p.exp_in_off + (Mx ? sh : 0);
    if (blockIdx.x == 0 && threadIdx.x == 0) *p.exp_out = E4;
    int mg_sa = 0, mg_sb = 0, mg_mx = 0, mg_mxm = 0;
    if (p.mg_other) {
        int Em;
        merge_shifts(E4, *p.mg_exp_other, mg_sa, mg_sb, Em, p.status);     // (also on the commit path: the flag is real)
    }
    if (p.spec) {
        const bool hit = r == *p.spec_used && (Mx != 0 || r == 7);
        if (hit) {
            // the codes are in place; add up the staged records
            long long a = 0, b = 0;
            int ma = 0, mb = 0;
            for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < p.sp_records; i += gridDim.x * blockDim.x) {
                const int64_t *rec = p.sp_part + 4 * (size_t)i;
                a += rec[0]; b += rec[1];
                ma = (int)rec[2] > ma ? (int)rec[2] : ma;
                mb = (int)rec[3] > mb ? (int)rec[3] : mb;
            }
            if (p.sum_e4) block_atomic_add_i64(a, p.sum_e4);
            if (RELU && p.sum_e1) block_atomic_add_i64(b, p.sum_e1);
            if (!RELU && p.mg_other) block_atomic_max_i32(ma, p.mg_absmax);
            if (!RELU && p.mg_mask16) block_atomic_max_i32(mb, p.mg_absmax_m);
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            p.spec[0] = r;                                                      // what the next step will try
            atomicAdd(p.counters + (hit ? 0 : 1), 1);
        }
        if (hit) return;
    }
    const uint32_t c16 = (uint32_t)p.C >> 4;
    const uint32_t total = (uint32_t)p.M * c16;            // the host checked that this fits 32 bits
    // (pixel, channel group) of this lane's element, advanced by the grid stride without a division per element
    const uint32_t step = gridDim.x * blockDim.x;
    const uint32_t dm = step / c16, dc = step - dm * c16;
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t m = i / c16, cg = i - m * c16;
    int s4 = 0, s1 = 0, mx1 = 0;                           // a lane sees at most 2^27 / lanes elements of |code| <= 127
    long long s4w = 0, s1w = 0;
    int since = 0;
    for (; i < total; i += step) {
        const int c = (int)cg << 4;
        const size_t off = (size_t)m * p.C + c;
        uint32_t mrow = m;                                 // row of the stored sums
        bool have = true;
        if (p.sub) {
            const uint32_t hw = (uint32_t)(p.H * p.W);
            const uint32_t n = m / hw, rem = m - n * hw;
            const uint32_t h = rem / (uint32_t)p.W, x = rem - h * (uint32_t)p.W;
            const uint32_t hp = h / (uint32_t)p.sub, xq = x / (uint32_t)p.sub;
            have = hp * p.sub == h && xq * p.sub == x;
            mrow = (n * p.P + hp) * p.Q + xq;
        }
        int s = 0;
        v4i lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
        if (p.cls_on) {
            const uint32_t hw = (uint32_t)(p.H * p.W);
            const uint32_t n = m / hw, rem = m - n * hw;
            const uint32_t h = rem / (uint32_t)p.W, x = rem - h * (uint32_t)p.W;
            const int a = (int)((h + p.cls_pad) & 1u), b = (int)((x + p.cls_pad) & 1u), cl = a * 2 + b;
            const int gh = (int)((h + p.cls_pad - a) >> 1) - p.cls_hh0[a], gw = (int)((x + p.cls_pad - b) >> 1) - p.cls_ww0[b];
            const uint32_t mc = (n * p.cls_Hc[a] + gh) * p.cls_Wc[b] + gw;
            s = p.tile_shift[p.cls_base[cl] + (mc >> p.cls_bm_shift[cl]) * p.cls_tiles_n[cl] + (c >> p.cls_bn_shift[cl])];
            const size_t src = (size_t)m * p.C + c;
            lo = ((const v4i *)(p.d16 + src))[0];
            hi = ((const v4i *)(p.d16 + src))[1];
        } else if (have) {
            s = p.tile_shift[(mrow >> p.bm_shift) * p.tiles_n + (c >> p.bn_shift)];
            const size_t src = (size_t)mrow * p.C + c;
            lo = ((const v4i *)(p.d16 + src))[0];
            hi = ((const v4i *)(p.d16 + src))[1];
        }
        const int T = sh - s + 1;                          // rounding position inside the stored 16-bit value
        uint32_t o4[4], o1[4] = {0, 0, 0, 0};
        uint32_t mk = 0xffffu;
        if (RELU && p.mask16) mk = (uint32_t)p.mask16[off >> 4];
        v4i ov = {0, 0, 0, 0};
        if (!RELU && p.mg_other) ov = *(const v4i *)(p.mg_other + off);
        if (!RELU && p.mg_mask16) mk = (uint32_t)p.mg_mask16[off >> 4];
        int cd[16];
        if (T >= 1) {
            const int half = (1 << (T - 1)) - 1;
#pragma unroll
            for (int k = 0; k < 16; k += 2) {
                const int w = k < 8 ? lo[k >> 1] : hi[(k - 8) >> 1];
                const int v0 = __builtin_amdgcn_sbfe(w, 0, 16), v1 = w >> 16;
                cd[k] = clamp_i((v0 + half + ((v0 >> T) & 1)) >> T, -CODE_MAX, CODE_MAX);
                cd[k + 1] = clamp_i((v1 + half + ((v1 >> T) & 1)) >> T, -CODE_MAX, CODE_MAX);
            }
        } else {                                           // every sum is below 2^7: the stored value is exactly 2*d
#pragma unroll
            for (int k = 0; k < 16; k += 2) {
                const int w = k < 8 ? lo[k >> 1] : hi[(k - 8) >> 1];
                cd[k] = clamp_i((__builtin_amdgcn_sbfe(w, 0, 16) >> 1) << (-sh), -CODE_MAX, CODE_MAX);
                cd[k + 1] = clamp_i((w >> 17) << (-sh), -CODE_MAX, CODE_MAX);
            }
        }
        // four codes (one output dword) at a time: sums and masks work on packed bytes
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t pk = pack4_i8(cd[4 * q], cd[4 * q + 1], cd[4 * q + 2], cd[4 * q + 3]);
            o4[q] = pk;
            s4 = sum4_i8(pk, s4);
            if (RELU) {
                const uint32_t pm = pk & byte_mask4(mk >> (4 * q));
                o1[q] = pm;
                s1 = sum4_i8(pm, s1);
                if (p.absmax_e1) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int e = __builtin_amdgcn_sbfe((int)pm, 8 * k, 8);
                        const int ae = e < 0 ? -e : e;
                        mx1 = ae > mx1 ? ae : mx1;
                    }
                }
            } else if (p.mg_other) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    int mv = (cd[4 * q + k] << mg_sa) + (__builtin_amdgcn_sbfe(ov[q], 8 * k, 8) << mg_sb);
                    mv = mv < 0 ? -mv : mv;
                    mg_mx = mv > mg_mx ? mv : mg_mx;
                    const int mm = ((mk >> (4 * q + k)) & 1u) ? mv : 0;
                    mg_mxm = mm > mg_mxm ? mm : mg_mxm;
                }
            }
        }
        if (p.e4) *(v4i *)(p.e4 + off) = v4i{(int)o4[0], (int)o4[1], (int)o4[2], (int)o4[3]};
        if (RELU) *(v4i *)(p.e1 + off) = v4i{(int)o1[0], (int)o1[1], (int)o1[2], (int)o1[3]};
        if (++since == 1 << 16) { s4w += s4; s1w += s1; s4 = s1 = 0; since = 0; }      // long before 32 bits fill
        m += dm; cg += dc;
        if (cg >= c16) { cg -= c16; ++m; }
    }
    s4w += s4; s1w += s1;
    if (p.sum_e4) block_atomic_add_i64(s4w, p.sum_e4);
    if (!RELU && p.mg_other) block_atomic_max_i32(mg_mx, p.mg_absmax);
    if (!RELU && p.mg_mask16) block_atomic_max_i32(mg_mxm, p.mg_absmax_m);
    if (RELU) {
        if (p.sum_e1) block_atomic_add_i64(s1w, p.sum_e1);
        if (p.absmax_e1) block_atomic_max_i32(mx1, p.absmax_e1);
    }
}

inline unsigned grid_for(size_t total)
{
    size_t b = (total + 255) / 256;
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    return (unsigned)b;
}

#ifdef EOQ_TUNE
// tuning builds only (never defined for the product library): per-workgroup timestamps and ablation switches
static unsigned long long *g_tune_dbg = nullptr;
static int g_tune_launch = 0;
static int tune_env(const char *name)
{
    const char *e = getenv(name);
    return e ? atoi(e) : 0;
}
#endif

template <int BM, int BN, int WGM, int WGN, int BK, int NS, bool UNI, int MODE, int EPI>
int launch_igemm_u(eoq_ctx *c, const IgemmParams &p)
{
    constexpr int NW = WGM * WGN;
    constexpr int epi_rows = (BN / WGN) >= 64 ? 16 : 32;        // rows staged at a time (SR in the kernel)
    constexpr int CHX = BK / 16, RPPX = NW * 64 / CHX;          // rows per load pass, as in the kernel
    constexpr int stage_rows = ((BM + RPPX - 1) / RPPX + (BN + RPPX - 1) / RPPX) * RPPX;
    constexpr int main_bytes = NS * stage_rows * BK, epi_bytes = NW * epi_rows * (BN / WGN + 4) * 4;
    constexpr int lds_bytes = main_bytes > epi_bytes ? main_bytes : epi_bytes;
    static std::atomic<bool> attr_done{false};     // (setting the attribute twice from two threads is harmless)
    void (*kern)(IgemmParams);
    if constexpr (BK == 128) kern = igemm_wide_kernel<BM, BN, WGM, WGN, BK, NS, UNI, MODE, EPI>;
    else kern = igemm_kernel<BM, BN, WGM, WGN, BK, NS, UNI, MODE, EPI>;
    if (lds_bytes > 48 * 1024 && !attr_done.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
            return EOQ_ERR_HIP;
        attr_done.store(true, std::memory_order_release);
    }
    long tiles = (long)((p.M + BM - 1) / BM) * ((p.NOUT + BN - 1) / BN);
#ifdef EOQ_TUNE
    IgemmParams pt = p;
    pt.abl = tune_env("EOQ_ABL");
    pt.dbg = g_tune_dbg ? g_tune_dbg + (size_t)(g_tune_launch++) * 4 * 8192 : nullptr;
    const IgemmParams &pl = pt;
#else
    const IgemmParams &pl = p;
#endif
    if (p.ncls) {
        IgemmParams q = pl;
        tiles = 0;
        for (int i = 0; i < p.ncls; ++i) {
            q.cls[i].tile_base = (int)tiles;
            tiles += (long)((p.cls[i].M + BM - 1) / BM) * ((p.NOUT + BN - 1) / BN);
        }
        hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(NW * 64), lds_bytes, c->stream, q);
        EOQ_LAUNCH_CHECK();
        return EOQ_OK;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(NW * 64), lds_bytes, c->stream, pl);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

// fewest 128 x 128 workgroups for which that tile is chosen over 128 x 64: three quarters of the compute units (the
// 7 x 7 layers with 512 outputs give 196; their reduction is long and bound by operand delivery, which the larger
// tile halves per multiply-add -- measured 8 % faster on the 3x3, 4 % on the 1x1, than 392 workgroups of 128 x 64)
constexpr long MIN_WGS_128 = 192;
// 128-byte stages: input channels a multiple of 128, a reduction of at least this many 16-byte chunks, and at most
// two 128 x 128 workgroups per compute unit
constexpr int WIDE_MIN_NK16 = 64;
constexpr long WIDE_MAX_WGS = 512;

template <int BM, int BN, int WGM, int WGN, int MODE, int EPI>
int launch_igemm(eoq_ctx *c, const IgemmParams &p, bool wide = false)
{
    if constexpr (BM == 128 && BN == 128 && WGM == 2 && WGN == 2) {
        if (wide) return launch_igemm_u<BM, BN, WGM, WGN, 128, 2, true, MODE, EPI>(c, p);
    }
    if (p.c16 % 4 == 0) return launch_igemm_u<BM, BN, WGM, WGN, 64, 2, true, MODE, EPI>(c, p);
    return launch_igemm_u<BM, BN, WGM, WGN, 64, 2, false, MODE, EPI>(c, p);
}

template <int MODE, int EPI>
int dispatch_igemm(eoq_ctx *c, const IgemmParams &p_in, int *bm_out = nullptr, int *bn_out = nullptr,
                   int *nw_out = nullptr)
{
    auto chosen = [&](int bm, int bn, int nw = 4) {
        if (bm_out) *bm_out = bm;
        if (bn_out) *bn_out = bn;
        if (nw_out) *nw_out = nw;
    };
    IgemmParams p = p_in;
    if (!p.xstep) p.xstep = p.C;
    p.gemm = (p.R == 1 && p.S == 1 && p.stride == 1 && p.pad == 0 && p.pad_w_delta == 0 && !p.no_pad && p.P == p.H &&
              p.Q == p.W) ? 1 : 0;
    if (p.ncls) p.gemm = 0;            // the classes differ in their grids and taps
    {
        const Recip rq = make_recip((uint32_t)p.Q), rp = make_recip((uint32_t)p.P);
        p.mulQ = rq.mul; p.shQ = rq.sh; p.mulP = rp.mul; p.shP = rp.sh;
        for (int i = 0; i < p.ncls; ++i) {
            const Recip cq = make_recip((uint32_t)p.cls[i].Q), cp = make_recip((uint32_t)p.cls[i].P);
            p.cls[i].mulQ = cq.mul; p.cls[i].shQ = cq.sh; p.cls[i].mulP = cp.mul; p.cls[i].shP = cp.sh;
        }
    }
    const int nout = p.NOUT;
    auto wgs = [&](int bm, int bn) { return (long)((p.M + bm - 1) / bm) * ((nout + bn - 1) / bn); };
    // Measured on MI355X: throughput is nearly flat in the tile shape, so small tiles win through occupancy and grid
    // size; the 128x128 tile pays off only for wide outputs with enough workgroups to fill the chip.
    if (nout <= 32) { chosen(128, 32); return launch_igemm<128, 32, 4, 1, MODE, EPI>(c, p); }
    if (nout >= 128 && wgs(128, 128) >= MIN_WGS_128) {
        chosen(128, 128);
        if (p.c16 % 8 == 0 && p.nk16 >= WIDE_MIN_NK16 && wgs(128, 128) <= WIDE_MAX_WGS && !p.ncls)
            return launch_igemm<128, 128, 2, 2, MODE, EPI>(c, p, true);
        // The forward epilogue with int8 outputs stacks the four waves along M, so that a wave owns whole 128-byte
        // output rows and its stores fill cache lines (measured: 3-9 % on the wide 1x1 layers, a loss elsewhere).
        if (EPI == EPI_FWD && p.ep.relu) return launch_igemm<128, 128, EPI == EPI_FWD ? 4 : 2, EPI == EPI_FWD ? 1 : 2, MODE, EPI>(c, p);
        return launch_igemm<128, 128, 2, 2, MODE, EPI>(c, p);
    }
    chosen(128, 64);
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
    o.mask16 = (uint16_t *)e->relu_mask_bits; o.t_wide = e->t_wide; o.t16 = e->t_wide_is_16;
    if (e->skip_is_wide < 0 || e->skip_is_wide > 2 || e->t_wide_is_16 < 0 || e->t_wide_is_16 > 1) return EOQ_ERR_ARG;
    uintptr_t al = (uintptr_t)e->skip | (uintptr_t)e->y | (uintptr_t)e->u_next | (uintptr_t)e->t_wide;
    if ((al & 15) || ((uintptr_t)e->relu_mask_bits & 3)) return EOQ_ERR_ARG;
    if (!e->relu && !e->t_wide) return EOQ_ERR_ARG;
    return EOQ_OK;
}

} // namespace

#ifdef EOQ_TUNE
extern "C" void eoq_tune_set_dbg(unsigned long long *buf) { g_tune_dbg = buf; g_tune_launch = 0; }
extern "C" int eoq_tune_launch_index() { return g_tune_launch; }
#endif

// padded reduction length of the explicit im2col path
static inline int im2col_kp(const eoq_conv_desc *d) { return (int)round_up((size_t)d->R * d->S * d->C, 64); }

extern "C" size_t eoq_workspace_bytes(const eoq_conv_desc *d, int op)
{
    if (!desc_ok(d)) return 0;
    const size_t P = conv_out_dim(d->H, d->pad, d->R, d->stride), Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    const size_t M = (size_t)d->N * P * Q;
    const size_t wbytes = (size_t)d->K * d->R * d->S * d->C;
    size_t im2col = 0, kp = (size_t)d->R * d->S * d->C;
    if (d->C % 16 && d->C <= 4) {
        const Pad4Geom g = pad4_geom(d);
        im2col = round_up(g.img_bytes, 256) + round_up(g.w_bytes, 256);
        kp = (size_t)g.KP;
    } else if (d->C % 16) {
        im2col = round_up(M * im2col_kp(d), 256) + round_up((size_t)d->K * im2col_kp(d), 256);
        kp = (size_t)im2col_kp(d);
    }
    switch (op) {
    case EOQ_OP_CONV_FWD: return im2col;
    case EOQ_OP_CONV_BWD_DATA:
        // transposed filters + 16-bit block-scaled sums + one shift per 64 x 32 tile (the smallest tile)
        return round_up(wbytes, 256) + round_up(2 * (size_t)d->N * d->H * d->W * d->C, 256) +
               round_up(4 * (((size_t)d->N * d->H * d->W + 63) / 64) * (((size_t)d->C + 31) / 32), 256);
    case EOQ_OP_CONV_BWD_WEIGHT:
        // staged input + split partial sums (int32) sized for the worst split count, see conv_wgrad.hip
        return im2col + round_up(((size_t)d->K * kp + WGRAD_PART_PAD) * 4 * wgrad_max_splits((size_t)d->K * kp), 256);
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
    p.status = c->d_status;
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
        if (d->R * d->S > 64) return EOQ_ERR_SHAPE;      // the gather keeps one validity bit per filter tap
        p.A = u; p.B = w;
        p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C;
        p.R = d->R; p.S = d->S; p.stride = d->stride; p.pad = d->pad;
    } else if (d->C <= 4) {
        // few-channel input (the stem): zero-bordered 4-bytes-per-pixel copy, 4 pixels = one k-chunk
        const Pad4Geom g = pad4_geom(d);
        if (d->R * g.S4 > 64) return EOQ_ERR_SHAPE;
        if (!ws || ws_bytes < eoq_workspace_bytes(d, EOQ_OP_CONV_FWD) || ((uintptr_t)ws & 15)) return EOQ_ERR_WORKSPACE;
        if (g.img_bytes > 0x7fffff00u) return EOQ_ERR_SHAPE;
        int8_t *up = (int8_t *)ws;
        int8_t *wp = up + round_up(g.img_bytes, 256);
        hipLaunchKernelGGL(pad4_input_kernel, dim3(grid_for(g.img_bytes / 4)), dim3(256), 0, c->stream, u, d->N, d->H, d->W,
                           d->C, d->pad, g.Hp, g.Wp, (uint32_t *)up);
        hipLaunchKernelGGL(pad4_filters_kernel, dim3(grid_for(g.w_bytes)), dim3(256), 0, c->stream, w, d->K, d->R, d->S,
                           d->C, g.S4, wp);
        EOQ_LAUNCH_CHECK();
        p.A = up; p.B = wp;
        p.N = d->N; p.H = g.Hp; p.W = g.Wp / 4; p.C = 16;       // rows of Wp/4 sixteen-byte units
        p.R = d->R; p.S = g.S4; p.stride = d->stride; p.pad = 0;
        p.xstep = 4; p.no_pad = 1;
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
    if (!p.xstep) p.xstep = p.C;
    p.c16 = p.C / 16;
    p.nk16 = p.R * p.S * p.c16;
    return ep ? dispatch_igemm<MODE_FWD, EPI_FWD>(c, p) : dispatch_igemm<MODE_FWD, EPI_ACC>(c, p);
}

extern "C" int eoq_conv_bwd_data(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *w, int32_t *d_acc,
                                 int32_t *absmax_slot, void *ws, size_t ws_bytes)
{
    if (!c || !e || !w || !d_acc || !absmax_slot) return EOQ_ERR_ARG;
    if (!desc_ok(d)) return EOQ_ERR_SHAPE;
    if (d->K % 16 || d->C % 16 || d->R * d->S > 64) return EOQ_ERR_SHAPE;
    if (((uintptr_t)e | (uintptr_t)w | (uintptr_t)d_acc) & 15) return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_workspace_bytes(d, EOQ_OP_CONV_BWD_DATA) || ((uintptr_t)ws & 15)) return EOQ_ERR_WORKSPACE;
    const int P = conv_out_dim(d->H, d->pad, d->R, d->stride), Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    if ((size_t)d->N * d->H * d->W > 0x7fffffffu || (size_t)P * Q * d->K > 0x7fffffffu) return EOQ_ERR_SHAPE;
    int8_t *wt = (int8_t *)ws;
    hipLaunchKernelGGL(transpose_filters_kernel, dim3(grid_for((size_t)d->K * d->R * d->S * d->C)), dim3(256), 0,
                       c->stream, w, d->K, d->R * d->S, d->C, wt);
    EOQ_LAUNCH_CHECK();
    IgemmParams p{};
    p.status = c->d_status;
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

extern "C" int eoq_relu_bwd_recompute(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *u, const int8_t *w,
                                      const int8_t *e0, const uint32_t *mask_bits, int8_t *e1, int64_t *sum_e1,
                                      int64_t *sum_e1t, int32_t *absmax_e1)
{
    if (!c || !u || !w || !e0 || (!e1 && !sum_e1 && !sum_e1t && !absmax_e1)) return EOQ_ERR_ARG;
    if (!desc_ok(d)) return EOQ_ERR_SHAPE;
    if (d->K % 16 || d->C % 16 || d->R * d->S > 64) return EOQ_ERR_SHAPE;
    if (((uintptr_t)u | (uintptr_t)w | (uintptr_t)e0 | (uintptr_t)e1) & 15 || ((uintptr_t)mask_bits & 3)) return EOQ_ERR_ARG;
    IgemmParams p{};
    p.status = c->d_status;
    p.P = conv_out_dim(d->H, d->pad, d->R, d->stride);
    p.Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    if ((size_t)d->N * p.P * p.Q * d->K > 0x7fffffffu || (size_t)d->N * d->H * d->W * d->C > 0x7fffffffu) return EOQ_ERR_SHAPE;
    p.M = d->N * p.P * p.Q;
    p.NOUT = d->K;
    p.A = u; p.B = w;
    p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C;
    p.R = d->R; p.S = d->S; p.stride = d->stride; p.pad = d->pad;
    p.c16 = p.C / 16;
    p.nk16 = p.R * p.S * p.c16;
    p.rb_e0 = e0; p.rb_mask16 = (const uint16_t *)mask_bits; p.rb_e1 = e1;
    p.rb_sum_e1 = sum_e1; p.rb_sum_e1t = sum_e1t; p.rb_absmax = absmax_e1;
    // every tile shape the dispatcher may choose is at least 64 x 32
    const long max_tiles = (long)((p.M + 63) / 64) * ((p.NOUT + 31) / 32);
    if ((sum_e1 || sum_e1t) && 8 * max_tiles <= EOQ_PARTIAL_SLOTS) p.rb_part = c->d_partials;
    int bm = 0, bn = 0, nw = 4;
    if (int rc = dispatch_igemm<MODE_FWD, EPI_RELU_BWD>(c, p, &bm, &bn, &nw)) return rc;
    if (p.rb_part) {
        const int tiles = ((p.M + bm - 1) / bm) * ((p.NOUT + bn - 1) / bn);
        int rblocks = (nw * tiles + 1023) / 1024;
        if (rblocks > 32) rblocks = 32;
        hipLaunchKernelGGL(pair_reduce_kernel, dim3(rblocks), dim3(1024), 0, c->stream, c->d_partials, nw * tiles, sum_e1,
                           sum_e1t);
        EOQ_LAUNCH_CHECK();
    }
    return EOQ_OK;
}

static int bwd_data_params(const eoq_conv_desc *d, const int8_t *e, const int8_t *wt, IgemmParams &p)
{
    const int P = conv_out_dim(d->H, d->pad, d->R, d->stride), Q = conv_out_dim(d->W, d->pad, d->S, d->stride);
    if ((size_t)d->N * d->H * d->W > 0x7fffffffu || (size_t)d->N * P * Q * d->K > 0x7fffffffu) return EOQ_ERR_SHAPE;
    p.A = e; p.B = wt;
    p.N = d->N; p.H = P; p.W = Q; p.C = d->K;      // the tensor being gathered is the error
    p.P = d->H; p.Q = d->W; p.NOUT = d->C;         // one output row per input pixel
    p.R = d->R; p.S = d->S; p.stride = d->stride; p.pad = d->pad;
    p.M = d->N * d->H * d->W;
    p.c16 = p.C / 16;
    p.nk16 = p.R * p.S * p.c16;
    p.xstep = p.C;
    return EOQ_OK;
}

extern "C" int eoq_transpose_filters(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *w, int8_t *wt)
{
    if (!c || !w || !wt || (((uintptr_t)w | (uintptr_t)wt) & 15)) return EOQ_ERR_ARG;
    if (!desc_ok(d)) return EOQ_ERR_SHAPE;
    hipLaunchKernelGGL(transpose_filters_kernel, dim3(grid_for((size_t)d->K * d->R * d->S * d->C)), dim3(256), 0,
                       c->stream, w, d->K, d->R * d->S, d->C, wt);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

extern "C" int eoq_conv_bwd_data_sq(eoq_ctx *c, const eoq_conv_desc *d, const int8_t *e, const int8_t *w, int8_t *e4,
                                    int32_t *absmax_slot, const int32_t *exp_in, int32_t exp_in_off, int32_t *exp_out,
                                    int64_t *sum_out, const eoq_bwd_fuse *fuse, void *ws, size_t ws_bytes)
{
    const uint32_t *mask_bits = fuse ? fuse->mask_bits : nullptr;
    int8_t *e1 = fuse ? fuse->e1 : nullptr;
    int64_t *sum_e1 = fuse ? fuse->sum_e1 : nullptr;
    int32_t *absmax_e1 = fuse ? fuse->absmax_e1 : nullptr;
    const int8_t *mg_other = fuse ? fuse->merge_other : nullptr;
    if (mg_other && (!e4 || e1 || !fuse->merge_exp_other || !fuse->merge_absmax || ((uintptr_t)mg_other & 15)))
        return EOQ_ERR_ARG;
    const uint32_t *mg_mask = mg_other ? fuse->merge_mask_bits : nullptr;
    if (fuse && !mg_other && (fuse->merge_mask_bits || fuse->merge_absmax_masked)) return EOQ_ERR_ARG;
    if (mg_mask && (!fuse->merge_absmax_masked || ((uintptr_t)mg_mask & 3))) return EOQ_ERR_ARG;
    if (!c || !e || !w || (!e4 && !e1) || !absmax_slot || !exp_in || !exp_out) return EOQ_ERR_ARG;
    if (!desc_ok(d)) return EOQ_ERR_SHAPE;
    if (d->K % 16 || d->C % 16 || d->R * d->S > 64) return EOQ_ERR_SHAPE;
    if ((long long)d->R * d->S * d->K * 127 * 127 >= (1ll << 30)) return EOQ_ERR_SHAPE;   // sums stay below 2^30
    if (((uintptr_t)e | (uintptr_t)w | (uintptr_t)e4 | (uintptr_t)e1) & 15 || ((uintptr_t)mask_bits & 3)) return EOQ_ERR_ARG;
    if (!ws || ws_bytes < eoq_workspace_bytes(d, EOQ_OP_CONV_BWD_DATA) || ((uintptr_t)ws & 15)) return EOQ_ERR_WORKSPACE;
    const size_t M = (size_t)d->N * d->H * d->W;
    const int8_t *wt = fuse ? fuse->w_transposed : nullptr;
    if ((uintptr_t)wt & 15) return EOQ_ERR_ARG;
    int16_t *d16 = (int16_t *)((int8_t *)ws + round_up((size_t)d->K * d->R * d->S * d->C, 256));
    int32_t *tile_shift = (int32_t *)((int8_t *)d16 + round_up(2 * M * d->C, 256));
    const bool cls = d->stride == 2 && d->R >= 2 && d->S >= 2;      // see below
    if (!wt && !cls) {
        hipLaunchKernelGGL(transpose_filters_kernel, dim3(grid_for((size_t)d->K * d->R * d->S * d->C)), dim3(256), 0,
                           c->stream, w, d->K, d->R * d->S, d->C, (int8_t *)ws);
        EOQ_LAUNCH_CHECK();
        wt = (const int8_t *)ws;
    }
    IgemmParams p{};
    p.status = c->d_status;
    // A strided 1x1 filter touches only every stride-th input row and column: the sums are formed for those pixels
    // alone (a stride-1 problem on the P x Q grid of the error) and the streaming kernel writes zeros elsewhere --
    // 1/stride^2 of the multiply-adds of the general gather, which would spend the rest on structural zeros.
    const bool sub = d->R == 1 && d->S == 1 && d->pad == 0 && d->stride > 1;
    eoq_conv_desc dsub = *d;
    if (sub) {
        dsub.H = conv_out_dim(d->H, 0, 1, d->stride);
        dsub.W = conv_out_dim(d->W, 0, 1, d->stride);
        dsub.stride = 1;
    }
    // Stride 2 with a filter larger than 1x1: an input pixel only sees the taps whose parity matches its own, a
    // quarter of them on average.  The four parity classes (a, b) of (h + pad, w + pad) are four stride-1 gathers over
    // the error, each with its own taps (r = a, a+2, ..; s = b, b+2, ..) packed as a small filter -- no multiply-add
    // is spent on a structural zero.
    D16Finish f{};
    int bm = 0, bn = 0;
    if (cls) {
        const int P = conv_out_dim(d->H, d->pad, d->R, 2), Q = conv_out_dim(d->W, d->pad, d->S, 2);
        if ((size_t)d->N * d->H * d->W > 0x7fffffffu || (size_t)d->N * P * Q * d->K > 0x7fffffffu) return EOQ_ERR_SHAPE;
        int8_t *wc = (int8_t *)ws;                     // the four packed filters share the transposed-filter region
        f.cls_on = 1; f.cls_pad = d->pad; f.H = d->H; f.W = d->W;
        ClsPack cp{};
        for (int a = 0; a < 2; ++a) {
            f.cls_hh0[a] = f.cls_ww0[a] = d->pad > a ? (d->pad - a + 1) >> 1 : 0;
            const int first = 2 * f.cls_hh0[a] + a - d->pad;           // first row / column of this parity
            f.cls_Hc[a] = first < d->H ? (d->H - 1 - first) / 2 + 1 : 0;
            f.cls_Wc[a] = first < d->W ? (d->W - 1 - first) / 2 + 1 : 0;
            cp.Ra[a] = (d->R - a + 1) / 2;
            cp.Sa[a] = (d->S - a + 1) / 2;
        }
        p.A = e; p.B = wc;
        p.N = d->N; p.H = P; p.W = Q; p.C = d->K; p.NOUT = d->C;
        p.stride = 1; p.c16 = p.C / 16; p.xstep = p.C;
        p.absmax = absmax_slot; p.d16 = d16; p.tile_shift = tile_shift; p.rm_on = 1; p.rm_H = d->H; p.rm_W = d->W;
        int cls_of[4] = {0, 0, 0, 0}, off = 0;
        for (int a = 0; a < 2; ++a)
            for (int b = 0; b < 2; ++b) {
                cp.base[2 * a + b] = off;
                const int Hc = f.cls_Hc[a], Wc = f.cls_Wc[b];
                if (Hc && Wc) {
                    IgemmCls &q = p.cls[p.ncls];
                    q.P = Hc; q.Q = Wc; q.R = cp.Ra[a]; q.S = cp.Sa[b];
                    q.pad = f.cls_hh0[a]; q.pad_w_delta = f.cls_ww0[b] - f.cls_hh0[a];
                    q.M = d->N * Hc * Wc; q.nk16 = q.R * q.S * p.c16;
                    q.rm_Hc = Hc; q.rm_Wc = Wc;
                    q.rm_h0 = 2 * f.cls_hh0[a] + a - d->pad; q.rm_w0 = 2 * f.cls_ww0[b] + b - d->pad;
                    q.b_off = off;
                    cls_of[p.ncls++] = 2 * a + b;
                    p.M += q.M;                        // the tile heuristic sees the whole launch
                }
                off += d->C * cp.Ra[a] * cp.Sa[b] * d->K;
            }
        hipLaunchKernelGGL(pack_class_filters_kernel, dim3(grid_for((size_t)d->K * d->R * d->S * d->C)), dim3(256), 0,
                           c->stream, w, d->K, d->R, d->S, d->C, cp, wc);
        EOQ_LAUNCH_CHECK();
        // fields the kernel takes from the class table still need sane values for the dispatcher
        p.P = d->H; p.Q = d->W; p.R = cp.Ra[0]; p.S = cp.Sa[0]; p.nk16 = p.R * p.S * p.c16;
        if (int rc = dispatch_igemm<MODE_BWD_DATA, EPI_D16>(c, p, &bm, &bn)) return rc;
        const int tiles_n = (d->C + bn - 1) / bn;
        int base = 0;
        for (int i = 0; i < p.ncls; ++i) {
            const int cl = cls_of[i];
            f.cls_base[cl] = base;
            f.cls_bm_shift[cl] = bm == 64 ? 6 : (bm == 128 ? 7 : 8);
            f.cls_bn_shift[cl] = bn == 32 ? 5 : (bn == 64 ? 6 : 7);
            f.cls_tiles_n[cl] = tiles_n;
            base += ((p.cls[i].M + bm - 1) / bm) * tiles_n;
        }
    } else {
    if (int rc = bwd_data_params(sub ? &dsub : d, e, wt, p)) return rc;
    p.absmax = absmax_slot;
    // speculative launch first (see IgemmParams::spec): general gathers only, and not when max|e1| is wanted (the
    // exact path takes it for free, here it would be one more staged maximum that no caller of this path needs)
    int32_t *spec = (fuse && !sub && !absmax_e1) ? fuse->spec_state : nullptr;
    const long max_tiles = (long)((p.M + 63) / 64) * ((p.NOUT + 31) / 32);
    if (spec && 16 * max_tiles > EOQ_PARTIAL_SLOTS) spec = nullptr;
    if (spec) {
        IgemmParams q = p;
        q.spec = spec; q.spec_used = c->d_scratch + EOQ_SLOT_SPEC_USED;
        q.sp_e4 = e4; q.sp_e1 = e1;
        q.sp_mask16 = e1 ? (const uint16_t *)mask_bits : (const uint16_t *)mg_mask;
        q.sp_other = mg_other;
        q.sp_exp_in = exp_in; q.sp_exp_off = exp_in_off;
        q.sp_exp_other = mg_other ? fuse->merge_exp_other : nullptr;
        q.sp_part = c->d_partials;
        int bm1 = 0, bn1 = 0, nw1 = 4;
        if (int rc = dispatch_igemm<MODE_BWD_DATA, EPI_SPEC>(c, q, &bm1, &bn1, &nw1)) return rc;
        f.spec = spec; f.spec_used = q.spec_used; f.sp_part = c->d_partials; f.counters = c->d_scratch + EOQ_SLOT_SPEC_HITS;
        f.sp_records = nw1 * (int)(((p.M + bm1 - 1) / bm1) * ((p.NOUT + bn1 - 1) / bn1));
        p.spec = spec; p.spec_used = q.spec_used;
    }
    p.d16 = d16;
    p.tile_shift = tile_shift;
    if (int rc = dispatch_igemm<MODE_BWD_DATA, EPI_D16>(c, p, &bm, &bn)) return rc;
    }
    f.d16 = d16; f.tile_shift = tile_shift;
    f.bm_shift = bm == 64 ? 6 : (bm == 128 ? 7 : 8);
    f.bn_shift = bn == 32 ? 5 : (bn == 64 ? 6 : 7);
    f.tiles_n = (d->C + bn - 1) / bn;
    f.M = M; f.C = d->C;
    f.absmax = absmax_slot; f.exp_in = exp_in; f.exp_in_off = exp_in_off; f.exp_out = exp_out;
    f.e4 = e4; f.sum_e4 = sum_out;
    f.mask16 = (const uint16_t *)mask_bits; f.e1 = e1; f.sum_e1 = sum_e1; f.absmax_e1 = absmax_e1;
    f.mg_other = mg_other;
    f.mg_exp_other = mg_other ? fuse->merge_exp_other : nullptr;
    f.mg_absmax = mg_other ? fuse->merge_absmax : nullptr;
    f.mg_mask16 = (const uint16_t *)mg_mask;
    f.mg_absmax_m = mg_mask ? fuse->merge_absmax_masked : nullptr;
    f.status = c->d_status;
    if (sub) { f.sub = d->stride; f.H = d->H; f.W = d->W; f.P = dsub.H; f.Q = dsub.W; }
    if (M * (d->C / 16) > 0x7fffffffu) return EOQ_ERR_SHAPE;
    // few, large blocks: each ends with atomics on the same two or three slots
    size_t fb = (M * (d->C / 16) + 1023) / 1024;
    if (fb > 512) fb = 512;
    if (e1) hipLaunchKernelGGL(d16_finish_kernel<true>, dim3((unsigned)fb), dim3(1024), 0, c->stream, f);
    else hipLaunchKernelGGL(d16_finish_kernel<false>, dim3((unsigned)fb), dim3(1024), 0, c->stream, f);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}

int eoq_requant_fwd_standalone(eoq_ctx *c, const eoq_requant_args *a)
{
    if (!a->acc || !a->ep || (a->n % 16) || ((uintptr_t)a->acc & 15)) return EOQ_ERR_ARG;
    EpiDev ep;
    if (int rc = fill_epi(a->ep, ep)) return rc;
    if (!a->n) return EOQ_OK;
    hipLaunchKernelGGL(requant_fwd_kernel, dim3(grid_for(a->n / 16)), dim3(256), 0, c->stream, a->acc, a->n / 16, ep, c->d_status);
    EOQ_LAUNCH_CHECK();
    return EOQ_OK;
}
