// Stage 2, small-M ("decode") form of Y = X_q W_q + T B_k (Eq. 3 / Eq. 6): a weight-streaming
// kernel bound by HBM bandwidth.  Sec. 2.1 notes that few-token inference is memory-bound; the
// whole job here is to read 0.5625 B per weight once, as contiguous 1 KiB wavefront loads, and to
// hide everything else under that stream.
//
// What shapes the kernel is that on this chip every vector-memory instruction a compute unit
// issues beside the weight stream costs bandwidth, even when it hits in cache: measured on an
// 8192 x 28672 layer, two extra loads per weight record cost 5 %, eight cost 40 %.  So the
// activations reach the MFMA through LDS, filled with as few, fully coalesced 1 KiB loads as
// possible, and each operand read from LDS is used for G column groups.
//
// A workgroup is NWC x NWK wavefronts; wavefront (wc, wk) owns G column groups of 32 and, in step
// it, the K tile NWK it + wk.  The projection kernel leaves the activations as 16-byte cells
// [K / 8][token row] (bf16, exact dequantized X_q) - or, from 16 token rows up, as the MXINT8 codes
// themselves, [K / 16][token row][16 B] with the exponent bytes behind, which the staging wavefront
// scales to the same bf16 cells - so the NWK tiles of a step are one contiguous range that the
// workgroup brings into one of two LDS stages.  A step walks its tile in four
// 64-wide chunks; in chunk c every column group does four 32x32x16 MFMAs against the same four
// operands read from LDS, and the registers that held chunk c of the weight records are refilled
// at once with chunk c of the next tile, so a wavefront always has G whole records in flight and
// loads are issued in the order their data is needed (vector-memory loads retire in order).
// Per record a lane reads 64 B of packed codes (eight whole MXINT4 blocks) and their eight
// exponent bytes, expands 8 codes to bf16 values code * 2^(e-2) with seven VALU instructions
// (unpack_w8) and feeds them to the MFMA (tokens beyond M repeat the last one and are never
// stored); products are exact, accumulation is fp32.  The rank-kp correction is 2*kp further
// "K columns": T_hi and T_lo against B_k's codes, spread over the wavefronts.  T arrives as S
// partial sums (one per K slice of the projection kernel) that the workgroup adds in slice order
// and keeps in LDS as two bf16 terms.  At the end the NWK partial sums of every column group are
// added through LDS in slice order and stored as fp32, or as MXINT8 blocks of 16 along N for the
// next layer.  Up to 64 tokens are two blocks of 32 per wavefront sharing each expanded weight operand.
#include <mutex>
#include <type_traits>

#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

constexpr int kStreamTBytes = 9 * 1024;          // 32 rows x (128 + 8) bf16, rounded up to keep what follows 1 KiB aligned
constexpr int kStreamTBytesBig = 33 * 1024;      // the same for ranks up to 256: 32 rows x (512 + 8) bf16

struct StreamArgs {
    const uint8_t* Wt; const uint8_t* Bt;
    const uint8_t* Xcell;          // activations: bf16 as 16-byte cells [KT*32][R rows] (R = 4), or MXINT8 codes [KT*16][R][16] + exponent bytes [KT*16][R]
    const float* Tpart; int S;
    float* Y; int64_t ldy;
    int8_t* Yc; uint8_t* Ye; int64_t ldyc;           // Yc != null: store Y as MXINT8 (blocks of 16 along N) instead of fp32
    int64_t M, N, KT, N32;
    int kp, kp16;
    int rec_bytes;                 // bytes of a weight record
    int exp_bias;                  // >= 0: exponent nibbles (byte = nibble + exp_bias); -1: exponent bytes
};

// LR = log2 of the token rows per activation cell column (4, 16 or 32 rows).
// ONE: the whole K range of the workgroup is a single step: one activation stage, no loop.
// KSP: workgroups per column block.  KSP = 2 gives narrow layers twice the workgroups: the pair
//      takes alternate steps of the K range and both add their sums into Y, which the projection
//      kernel has zeroed, with hardware fp32 atomics.  0 + a + b does not depend on which of the two
//      arrives first, so the result is the same bits on every run.
// WB: mantissa bits of W_q, 4 or 2 (half the code bytes per record: two 1 KiB loads per record instead of four).
// BIGK: padded ranks above 64 (up to 256): the correction's operands are then not fetched ahead of the main
//      product - there are up to four times as many - but behind it, all of a wavefront's together.
template <int G, int NWC, int NWK, int DT, int LR, bool ONE, int KSP, int WB, bool BIGK>
__global__ __launch_bounds__(64 * NWC * NWK) void stream_kernel(StreamArgs a) {
    static_assert(WB == 4 || WB == 2, "weight mantissas of 4 or 2 bits");
    constexpr int NC = (WB == 4) ? 4 : 2;            // 1 KiB loads per weight record
    static_assert(KSP == 1 || KSP == 2, "one workgroup per column block, or a pair");
    // 64 token rows are two blocks of 32: every expanded weight operand then feeds two MFMAs
    constexpr int MB = (LR == 6) ? 2 : 1;
    static_assert(MB == 1 || KSP == 1, "pairs of workgroups take at most 32 tokens");
    static_assert(DT == 1 || DT == 2, "weights one or two steps ahead");
    static_assert(!ONE || DT == 1, "a single step prefetches nothing");
    constexpr int NW = NWC * NWK;
    constexpr int NG = NWC * G;                      // column groups of the workgroup
    constexpr int R = 1 << LR;
    constexpr int XT = NWK * R * 512;                // bytes of one stage in LDS: NWK tiles x R rows of bf16
    // With 16 token rows and more the activations travel as MXINT8 (16 code bytes per block and row,
    // exponent bytes behind all codes) and become bf16 on the way into LDS: the fill loads are what
    // this kernel pays for beside the weight stream, and this halves their bytes (stream_takes_codes()).
    constexpr bool X8 = LR >= 4 && KSP == 1;         // pairs of workgroups serve layers too small for the halved loads to show
    constexpr int XG = X8 ? XT / 2 : XT;             // bytes of one stage in global memory (codes only)
    constexpr int NL = XG / 1024;                    // 1 KiB loads per stage
    constexpr int XL = (NL + NW - 1) / NW;           // ... per wavefront
    // array length for the staging registers: an aggregate of exactly 32 dwords is turned into one
    // 1024-bit register tuple by the compiler, which costs over a hundred registers here
    constexpr int XLA = (XL == 8) ? 9 : XL;
    static_assert(XG % 1024 == 0, "a stage is a whole number of wavefront loads");
    // T_hi | T_lo of up to 32 tokens x 64 ranks, bf16; a row is padded by 16 bytes so that the token rows
    // of one operand read fall into different banks
    constexpr int kTBytes = (BIGK ? kStreamTBytesBig : kStreamTBytes) * MB;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    uint16_t* tlds = reinterpret_cast<uint16_t*>(lds);                 // [32][2 kp + 8] bf16, kept all along
    const int t_ld = 2 * a.kp + 8;                                     // row stride of tlds in elements
    uint8_t* xlds = lds + kTBytes;                                     // two activation stages
    float* red = reinterpret_cast<float*>(lds + kTBytes);              // reused afterwards: [NWK][NG][4][64 lanes][4]

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wc = wave % NWC, wk = wave / NWC;
    const int t = lane & 31, hh = lane >> 5;

    // column groups of this wavefront (clamped; stores are masked)
    const int64_t cb = blockIdx.x / KSP;             // column block
    const int kh = blockIdx.x % KSP;                 // which of the KSP workgroups of the block
    const int64_t g0 = (cb * NWC + wc) * G;
    const uint8_t* wrec[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        int64_t grp = g0 + g;
        if (grp >= a.N32) grp = a.N32 - 1;
        wrec[g] = a.Wt + grp * a.rec_bytes + lane * 16 + (a.exp_bias >= 0 ? kWCompactCodeOffset : 0);   // this lane's codes
    }
    // Exponent of block 2 c + j of the lane's eight, without a branch in the main loop (a branch there
    // makes the compiler's wait counts worst-case): word c / 2, shifted by (c % 2) * es1 + j * es0,
    // masked, plus the bias.  Bytes: (16, 8, 0xFF, 0); nibbles: (8, 4, 0xF, bias), the second word being
    // the first one shifted down by 16 when it is loaded.
    const bool exp4 = a.exp_bias >= 0;               // wave-uniform
    const int es1 = exp4 ? 8 : 16, es0 = exp4 ? 4 : 8;
    const uint32_t emask = exp4 ? 0xFu : 0xFFu, ebias = exp4 ? (uint32_t)a.exp_bias : 0u;
    // from wrec to this lane's exponent word: nibbles in front of the codes at lane * 4, bytes behind them at lane * 8
    const int e_adj = exp4 ? -(lane * 12) - kWCompactCodeOffset : w_code_bytes(WB) - (lane * 8);
    int trow[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b) {
        trow[b] = t + 32 * b;
        if (trow[b] >= a.M) trow[b] = (int)a.M - 1;  // repeat a valid token; never stored
    }

    const int64_t NI = (a.KT + NWK * KSP - 1) / (NWK * KSP);       // steps, the same for every wavefront
    // step it of this workgroup covers the tiles NWK (it KSP + kh) + 0 .. NWK - 1
    auto tile_raw = [&](int64_t it) { return wk + NWK * (it * KSP + kh); };
    // Tiles past the last one are read again (clamped index) and their arithmetic is skipped.
    auto tile_at = [&](int64_t it) {
        const int64_t tl = tile_raw(it);
        return tl < a.KT ? tl : a.KT - 1;
    };
    // activation stage of step it: XG bytes of the cell (or code) array from (it KSP + kh) XG on, clamped at its end
    const int64_t x_bytes = X8 ? (a.KT * 16 * R * 16) : (a.KT * 32 * R * 16);    // cells, or codes
    const int64_t x_last = x_bytes - 1024;                         // last whole 1 KiB of the array
    const int64_t e_last = a.KT * 16 * R - 64;                     // X8: last 64 exponent bytes
    // load x of this wavefront is 1 KiB number j = wave + NW x of the stage (wave-uniform, so the
    // address arithmetic stays in scalar registers).  As cells its lane writes 16 bytes at
    // swz(1024 j + 16 lane); as codes its lane holds block (64 j + lane) >> LR of token row
    // (64 j + lane) % R, which becomes the two cells 2 block and 2 block + 1 of that row.
    auto swz = [](int off) { return off ^ (((off >> (6 + LR)) & 1) << 7); };
    // LDS placement of a cell: the two lane halves of an operand read are 4 cells apart, which is a
    // multiple of the 256-byte bank period; flipping address bit 7 for the upper half's cells moves
    // them to the other half of the banks.
    int st_dst[XL];
#pragma unroll
    for (int x = 0; x < XL; ++x) {
        const int idx = (wave + NW * x) * 64 + lane;
        st_dst[x] = X8 ? swz(((((idx >> LR) * 2) << LR) + (idx & (R - 1))) << 4) : swz(idx * 16);
    }
    struct XStage {
        u32x4 c[XLA];                                // 16 bytes per load: a cell, or the 16 codes of a block
        uint32_t e[X8 ? XL : 1];                     // X8: the block's exponent byte
    };
    const uint8_t* xlane = a.Xcell + lane * 16;
    const uint8_t* elane = a.Xcell + x_bytes + lane;
    auto fetch_x = [&](XStage& st, int64_t it) {
        const int64_t base = (it * KSP + kh) * XG;
#pragma unroll
        for (int x = 0; x < XL; ++x) {
            const int j = wave + NW * x;
            if (j < NL) {
                int64_t off = base + j * 1024;
                if (off > x_last) off = x_last;
                st.c[x] = *reinterpret_cast<const u32x4*>(xlane + off);
                if constexpr (X8) {
                    int64_t eoff = (base >> 4) + j * 64;
                    if (eoff > e_last) eoff = e_last;
                    st.e[x] = elane[eoff];
                }
            }
        }
    };
    auto store_x = [&](const XStage& st, int buf) {
#pragma unroll
        for (int x = 0; x < XL; ++x) {
            if (wave + NW * x < NL) {
                if constexpr (X8) {
                    Frag f0, f1;
                    int8x16_to_frags(st.c[x], h_scale(st.e[x]), f0, f1);
                    *reinterpret_cast<u32x4*>(xlds + buf * XT + st_dst[x]) = f0.u;
                    *reinterpret_cast<u32x4*>(xlds + buf * XT + st_dst[x] + (16 << LR)) = f1.u;
                } else {
                    *reinterpret_cast<u32x4*>(xlds + buf * XT + st_dst[x]) = st.c[x];
                }
            }
        }
    };
    // operand read: cell 32 wk + 8 c + 4 hh + s of the stage, token row trow
    int rd_base[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b) rd_base[b] = (((32 * wk + 4 * hh) << LR) + trow[b]) << 4;
    const int rd_flip = hh << 7;                     // swz() of an operand address: its cell has bit 2 = hh

    const int64_t tile_stride = a.N32 * a.rec_bytes;             // records are ordered [K tile][column group]
    auto load_wc = [&](int g, int64_t tile, int c) {
        return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrec[g] + tile * tile_stride + c * 1024));
    };
    auto load_we = [&](int g, int64_t tile) {
        // always 8 bytes wide: with nibbles only the first word is used (the buffer is padded behind the last record)
        const u32x2_a4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2_a4*>(wrec[g] + tile * tile_stride + e_adj));
        return u32x2{w[0], exp4 ? w[0] >> 16 : w[1]};
    };

    f32x16 acc[G][MB];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int b = 0; b < MB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[g][b][r] = 0.f;

    // ---- rank-kp correction, part 1: fetch its operands first ---------------------------------------
    // The correction is 2 kp more "K columns" in 64-wide chunks of [T_hi | T_lo].  Lane half hh owns
    // rank blocks jb = 4 ch + 2 hh + {0, 1} of chunk ch: jb < kp16 is T_hi for ranks 16 jb..,
    // otherwise T_lo for ranks 16 (jb - kp16)...  Job j = g * nchunks + ch of this wavefront's column
    // groups goes to K slice j % NWK (every slice holds a partial sum of every group).
    const int nb2 = (kh == 0) ? 2 * a.kp16 : 0;      // the correction is added once: by workgroup 0 of a pair
    const int nchunks = (nb2 + 3) / 4;               // 0, 1 or 2; up to 8 with BIGK
    constexpr int NJ = ((BIGK ? 8 : 2) * G + NWK - 1) / NWK;
    constexpr int NJP = BIGK ? 1 : NJ;               // jobs whose operands are fetched ahead
    u32x4 tail_cw[NJP][2];
    uint32_t tail_eb[NJP][2];
    auto load_tail = [&](int job, int j, u32x4& cw, uint32_t& eb) {
        const int g = nchunks ? job / nchunks : 0, ch = nchunks ? job % nchunks : 0;
        cw = u32x4{0, 0, 0, 0};
        eb = 0;
        const int jb = 4 * ch + 2 * hh + j;
        if (job < G * nchunks && jb < nb2) {
            const int rb = jb >= a.kp16 ? jb - a.kp16 : jb;
            int64_t grp = g0 + g;
            if (grp >= a.N32) grp = a.N32 - 1;
            const uint8_t* rec = a.Bt + (grp * a.kp16 + rb) * kBRecordBytes;
            cw = *reinterpret_cast<const u32x4*>(rec + t * 16);
            eb = rec[512 + t];
        }
    };
#pragma unroll
    for (int q = 0; q < (BIGK ? 0 : NJ); ++q) {
        const int job = wk + NWK * q;                // wave-uniform
        const int g = nchunks ? job / nchunks : 0, ch = nchunks ? job % nchunks : 0;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            tail_cw[q][j] = u32x4{0, 0, 0, 0};
            tail_eb[q][j] = 0;
            const int jb = 4 * ch + 2 * hh + j;
            if (job < G * nchunks && jb < nb2) {
                const int rb = jb >= a.kp16 ? jb - a.kp16 : jb;
                int64_t grp = g0 + g;
                if (grp >= a.N32) grp = a.N32 - 1;
                const uint8_t* rec = a.Bt + (grp * a.kp16 + rb) * kBRecordBytes;
                tail_cw[q][j] = *reinterpret_cast<const u32x4*>(rec + t * 16);
                tail_eb[q][j] = rec[512 + t];
            }
        }
    }
    // T: the workgroup adds the S (<= 8) partial sums of the projection kernel in slice order and
    // leaves T_hi | T_lo as bf16 in LDS.  One item = 4 consecutive ranks of a token.
    constexpr int TI = BIGK ? 1 : (32 * MB * 16 + NW * 64 - 1) / (NW * 64);
    constexpr int SMAX = 8;
    const int t_rows = a.M < 32 * MB ? (int)a.M : 32 * MB;
    const int kp4 = a.kp >> 2;
    const int t_items = (kh == 0) ? t_rows * kp4 : 0;
    // The loads are issued here; the sums are formed (finish_t) once the first weight loads are on
    // their way, so that those do not wait for this round trip.
    f32x4 tpart[TI][SMAX];
#pragma unroll
    for (int i = 0; i < (BIGK ? 0 : TI); ++i) {
        const int item = threadIdx.x + i * NW * 64;
#pragma unroll
        for (int sl = 0; sl < SMAX; ++sl) {
            tpart[i][sl] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (item < t_items && sl < a.S)
                tpart[i][sl] = *reinterpret_cast<const f32x4*>(a.Tpart + (int64_t)sl * a.M * a.kp + 4 * item);
        }
    }
    auto finish_t = [&]() {
        constexpr int TIL = BIGK ? (32 * MB * 64 + NW * 64 - 1) / (NW * 64) : TI;
#pragma unroll
        for (int i = 0; i < TIL; ++i) {
            const int item = threadIdx.x + i * NW * 64;
            if (item >= t_items) continue;
            const int row = item / kp4, r4 = item - row * kp4;
            f32x4 sum;
            if constexpr (BIGK) {
                // loaded here, one item at a time, its slices' loads in flight together (slice order as below)
                f32x4 o[SMAX];
#pragma unroll
                for (int sl = 0; sl < SMAX; ++sl)
                    o[sl] = *reinterpret_cast<const f32x4*>(a.Tpart + (int64_t)(sl < a.S ? sl : a.S - 1) * a.M * a.kp + 4 * item);
                sum = o[0];
#pragma unroll
                for (int sl = 1; sl < SMAX; ++sl)
                    if (sl < a.S) { sum[0] += o[sl][0]; sum[1] += o[sl][1]; sum[2] += o[sl][2]; sum[3] += o[sl][3]; }
            } else {
                sum = tpart[i][0];
#pragma unroll
                for (int sl = 1; sl < SMAX; ++sl) {
                    sum[0] += tpart[i][sl][0]; sum[1] += tpart[i][sl][1];
                    sum[2] += tpart[i][sl][2]; sum[3] += tpart[i][sl][3];
                }
            }
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t hb = f32_bits(sum[e]) & 0xFFFF0000u;
                hi[e] = hb >> 16;
                lo[e] = f32_bits(sum[e] - f32_from_bits(hb)) >> 16;
            }
            uint16_t* dst = tlds + row * t_ld + 4 * r4;
            *reinterpret_cast<u32x2*>(dst) = u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
            *reinterpret_cast<u32x2*>(dst + a.kp) = u32x2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
        }
    };

    // ---- main product ----------------------------------------------------------------------------
    // DT register sets hold the weight records of DT consecutive steps; set it % DT serves step it and
    // is refilled chunk by chunk with the tile of step it + DT.
    {
        u32x4 wcd[DT][G][NC];        // packed codes: one 1 KiB load per chunk (4-bit weights) or per two chunks (2-bit)
        u32x2 wex[DT][G];            // exponent bytes
        {
            XStage st;
            fetch_x(st, 0);
#pragma unroll
            for (int g = 0; g < G; ++g) wex[0][g] = load_we(g, tile_at(0));
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int g = 0; g < G; ++g) wcd[0][g][c] = load_wc(g, tile_at(0), c);
            if constexpr (DT == 2) {
                if (NI > 1) {
#pragma unroll
                    for (int g = 0; g < G; ++g) wex[1][g] = load_we(g, tile_at(1));
#pragma unroll
                    for (int c = 0; c < NC; ++c)
#pragma unroll
                        for (int g = 0; g < G; ++g) wcd[1][g][c] = load_wc(g, tile_at(1), c);
                }
            }
            store_x(st, 0);
            finish_t();
        }
        // PFX: the step fetches the activations of the next one; PFW: it refills its weight set
        auto step = [&](u32x4 (&wc_)[G][NC], u32x2 (&we_)[G], int64_t it, auto pfx, auto pfw) {
            constexpr bool PFX = decltype(pfx)::value, PFW = decltype(pfw)::value;
            __syncthreads();         // stage it % 2 is complete; the other one is free again
            XStage st;
            u32x2 wen[G];
            const int64_t nt = tile_at(it + DT);
            if constexpr (PFX) fetch_x(st, it + 1);
            if constexpr (PFW) {
#pragma unroll
                for (int g = 0; g < G; ++g) wen[g] = load_we(g, nt);
            }
            __builtin_amdgcn_sched_barrier(0);
            const bool live = tile_raw(it) < a.KT;
            const uint8_t* xs = xlds + (ONE ? 0 : (int)(it & 1) * XT);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (live) {
                    Frag xf[MB][4];
#pragma unroll
                    for (int b = 0; b < MB; ++b)
#pragma unroll
                        for (int s = 0; s < 4; ++s) {
                            // for 16 rows and more the operand offsets are multiples of 256 B and leave bit 7 alone
                            const int off = (8 * c + s) << (LR + 4);
                            const int ad = (LR >= 4) ? ((rd_base[b] ^ rd_flip) + off) : ((rd_base[b] + off) ^ rd_flip);
                            xf[b][s].u = *reinterpret_cast<const u32x4*>(xs + ad);
                        }
#pragma unroll
                    for (int g = 0; g < G; ++g) {
#pragma unroll
                        for (int s = 0; s < 4; ++s) {
                            // exponent byte of block 2 c + s / 2 of the lane's eight: a byte, or a nibble plus the layer's bias
                            const uint32_t eb = ((we_[g][c >> 1] >> ((c & 1) * es1 + (s >> 1) * es0)) & emask) + ebias;
                            bf16x8 wv;
                            if constexpr (WB == 4) wv = unpack_w8(wc_[g][c][s], w_scale(eb));
                            else wv = unpack_w8_b2(wc_[g][c >> 1][(c & 1) * 2 + (s >> 1)], s & 1, w2_scale(eb));
#pragma unroll
                            for (int b = 0; b < MB; ++b) acc[g][b] = mfma32(wv, xf[b][s].v, acc[g][b]);
                        }
                    }
                }
                if constexpr (PFW) {
                    // refill what this chunk has just used up: its own 1 KiB, or (2-bit weights) the 1 KiB it shares
                    // with the chunk before it
                    if constexpr (WB == 4) {
#pragma unroll
                        for (int g = 0; g < G; ++g) wc_[g][c] = load_wc(g, nt, c);
                    } else if (c & 1) {
#pragma unroll
                        for (int g = 0; g < G; ++g) wc_[g][c >> 1] = load_wc(g, nt, c >> 1);
                    }
                }
            }
            if constexpr (PFX) store_x(st, (int)((it + 1) & 1));    // waits for the activation loads only
            if constexpr (PFW) {
#pragma unroll
                for (int g = 0; g < G; ++g) we_[g] = wen[g];
            }
        };
        constexpr std::true_type Y_{};
        constexpr std::false_type N_{};
        if constexpr (ONE) {
            step(wcd[0], wex[0], 0, N_, N_);
        } else if constexpr (DT == 1) {
            for (int64_t it = 0; it + 1 < NI; ++it) step(wcd[0], wex[0], it, Y_, Y_);
            step(wcd[0], wex[0], NI - 1, N_, N_);
        } else {
            int64_t it = 0;
            for (; it + 3 < NI; it += 2) {
                step(wcd[0], wex[0], it, Y_, Y_);
                step(wcd[1], wex[1], it + 1, Y_, Y_);
            }
            // one to three steps remain; the tile of step it + j sits in set j % 2
            if (it + 1 == NI) {
                step(wcd[0], wex[0], it, N_, N_);
            } else if (it + 2 == NI) {
                step(wcd[0], wex[0], it, Y_, N_);
                step(wcd[1], wex[1], it + 1, N_, N_);
            } else {
                step(wcd[0], wex[0], it, Y_, Y_);
                step(wcd[1], wex[1], it + 1, Y_, N_);
                step(wcd[0], wex[0], it + 2, N_, N_);
            }
        }
    }

    // ---- rank-kp correction, part 2: the arithmetic ---------------------------------------------------
    // (ranks above 64: the operands of all of this wavefront's jobs are asked for here, in the registers the weight sets
    // have left, instead of one round trip per job)
    constexpr int NJB = BIGK ? NJ : 1;
    u32x4 big_cw[NJB][2];
    uint32_t big_eb[NJB][2];
    if constexpr (BIGK) {
#pragma unroll
        for (int q = 0; q < NJ; ++q)
#pragma unroll
            for (int j = 0; j < 2; ++j) load_tail(wk + NWK * q, j, big_cw[q][j], big_eb[q][j]);
    }
#pragma unroll
    for (int q = 0; q < NJ; ++q) {
        const int job = wk + NWK * q;
        if (job >= G * nchunks) continue;
        const int g = job / nchunks, ch = job % nchunks;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int jb = 4 * ch + 2 * hh + j;
            Frag ta[MB][2];
#pragma unroll
            for (int b = 0; b < MB; ++b) {
                ta[b][0].u = u32x4{0, 0, 0, 0};
                ta[b][1].u = u32x4{0, 0, 0, 0};
                if (jb < nb2) {
                    const uint16_t* src = tlds + trow[b] * t_ld + 16 * jb;
                    ta[b][0].u = *reinterpret_cast<const u32x4*>(src);
                    ta[b][1].u = *reinterpret_cast<const u32x4*>(src + 8);
                }
            }
            Frag bf[2];
            if constexpr (BIGK) {
                int8x16_to_frags(big_cw[q][j], h_scale(big_eb[q][j]), bf[0], bf[1]);
            } else {
                int8x16_to_frags(tail_cw[q][j], h_scale(tail_eb[q][j]), bf[0], bf[1]);
            }
            // g is wave-uniform: pick the accumulator by unrolled comparison so all stay in registers
#pragma unroll
            for (int gg = 0; gg < G; ++gg) {
                if (gg == g) {
#pragma unroll
                    for (int b = 0; b < MB; ++b) {
                        acc[gg][b] = mfma32(bf[0].v, ta[b][0].v, acc[gg][b]);
                        acc[gg][b] = mfma32(bf[1].v, ta[b][1].v, acc[gg][b]);
                    }
                }
            }
        }
    }

    // ---- add the K slices of every column group in slice order -----------------------------------------
    // every wavefront leaves its partial sums in LDS; wavefront v then finishes unit v, v + NW, ... where
    // unit u = (column group, token block, accumulator quarter u % 4)
    constexpr int NGV = NG * MB;                     // (column group, token block) pairs of the workgroup
    __syncthreads();                                 // every wavefront is done with the activation stages
    auto red_at = [&](int k, int q, int r4) {          // lanes side by side: no bank conflicts
        return reinterpret_cast<f32x4*>(red + (((((size_t)k * NGV + q) * 4 + r4) * 64 + lane) * 4));
    };
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int b = 0; b < MB; ++b)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                *red_at(wk, (wc * G + g) * MB + b, r4) =
                    f32x4{acc[g][b][4 * r4], acc[g][b][4 * r4 + 1], acc[g][b][4 * r4 + 2], acc[g][b][4 * r4 + 3]};
    __syncthreads();
    // A pair of workgroups adds into Y with atomics.  They are issued so that one instruction covers two
    // rows of 32 consecutive columns (two cache lines) instead of 64 scattered dwords: the finished
    // sums go through LDS once more to change the lane order.
    float* yt = red + NWK * NGV * 1024;                                // [NG][32 rows][32 columns], behind the partial sums
    // As MXINT8 for the next layer (one workgroup per column block only): a unit is one block of 16
    // columns of a (group, token block) - quarters 2 b and 2 b + 1, eight values in this lane and
    // eight in lane ^ 32 (the same token).
    if (KSP == 1 && a.Yc != nullptr) {
        for (int u = wave; u < NGV * 2; u += NW) {
            const int qv = u >> 1, b = u & 1;
            const int q = qv / MB, row = t + 32 * (qv % MB);
            float v[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 s4 = *red_at(0, qv, 2 * b + h);
#pragma unroll
                for (int k = 1; k < NWK; ++k) {
                    const f32x4 o = *red_at(k, qv, 2 * b + h);
                    s4[0] += o[0]; s4[1] += o[1]; s4[2] += o[2]; s4[3] += o[3];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) v[4 * h + j] = s4[j];
            }
            uint32_t w0, w1;
            const uint32_t eb = requant_half_block(v, w0, w1);
            const int64_t grp = cb * NG + q;
            const int64_t n0 = grp * 32 + 16 * b;
            if (grp < a.N32 && row < a.M && n0 < a.N) {
                int8_t* dst = a.Yc + (int64_t)row * a.ldyc + n0 + 4 * hh;
                *reinterpret_cast<uint32_t*>(dst) = w0;
                *reinterpret_cast<uint32_t*>(dst + 8) = w1;
                if (hh == 0) a.Ye[(int64_t)row * (a.N >> 4) + (n0 >> 4)] = (uint8_t)eb;
            }
        }
        return;
    }
    for (int u = wave; u < NGV * 4; u += NW) {
        const int qv = u >> 2, r4 = u & 3;
        const int q = qv / MB, row = t + 32 * (qv % MB);
        f32x4 v = *red_at(0, qv, r4);
#pragma unroll
        for (int k = 1; k < NWK; ++k) {
            const f32x4 o = *red_at(k, qv, r4);
            v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
        }
        if constexpr (KSP == 2) {
            *reinterpret_cast<f32x4*>(yt + (q * 32 + t) * 32 + 8 * r4 + 4 * hh) = v;
        } else {
            const int64_t grp = cb * NG + q;
            if (grp < a.N32 && row < a.M) {
                const int64_t n = grp * 32 + 8 * r4 + 4 * hh;              // this lane's 4 consecutive columns
                float* dst = a.Y + (int64_t)row * a.ldy + n;
                if (n + 3 < a.N) {
                    *reinterpret_cast<f32x4*>(dst) = v;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (n + j < a.N) dst[j] = v[j];
                }
            }
        }
    }
    if constexpr (KSP == 2) {
        __syncthreads();
        const int pairs = ((int)a.M + 1) >> 1;                         // row pairs per column group
        for (int item = wave; item < NG * pairs; item += NW) {
            const int q = item / pairs, row = 2 * (item - q * pairs) + hh;
            const int64_t grp = cb * NG + q;
            const int64_t n = grp * 32 + t;
            if (grp < a.N32 && row < a.M && n < a.N)
                unsafeAtomicAdd(a.Y + (int64_t)row * a.ldy + n, yt[(q * 32 + row) * 32 + t]);
        }
    }
}

int stream_max_rows() { return 64; }
int stream_cell_rows_log2(int64_t M) { return M <= 4 ? 2 : (M <= 16 ? 4 : (M <= 32 ? 5 : 6)); }

template <int G, int NWC, int NWK, int DT, int LR, bool ONE, int KSP, int WB, bool BIGK>
static hipError_t launch_stream_t(const StreamArgs& a, hipStream_t s) {
    constexpr int STAGING = (ONE ? 1 : 2) * NWK * (1 << LR) * 512;
    constexpr int MB = (LR == 6) ? 2 : 1;
    constexpr int REDUCE = NWK * NWC * G * MB * 4096 + (KSP == 2 ? NWC * G * 4096 : 0);
    constexpr int LDS_BYTES = (BIGK ? kStreamTBytesBig : kStreamTBytes) * MB + (STAGING > REDUCE ? STAGING : REDUCE);
    if constexpr (LDS_BYTES > 160 * 1024 || (MB == 2 && KSP == 2)) {
        return hipErrorInvalidValue;                 // this shape does not fit the 160 KB of LDS
    } else {
        auto kern = stream_kernel<G, NWC, NWK, DT, LR, ONE, KSP, WB, BIGK>;
        // the dynamic LDS limit of this instance, set once per process (calls may come from several threads)
        static std::once_flag once;
        static hipError_t attr_err = hipSuccess;
        std::call_once(once, [&] {
            attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        });
        if (attr_err != hipSuccess) return attr_err;
        dim3 grid((unsigned)((a.N32 + NWC * G - 1) / (NWC * G) * KSP)), block(64 * NWC * NWK);
        hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, s, a);
        return hipGetLastError();
    }
}

template <int G, int NWC, int NWK, int DT, int KSP, int WB, bool BIGK>
static hipError_t launch_stream_rows(const StreamArgs& a, hipStream_t s) {
    if constexpr (DT == 1) {
        if (a.KT <= NWK * KSP) {
            switch (stream_cell_rows_log2(a.M)) {
                case 2: return launch_stream_t<G, NWC, NWK, 1, 2, true, KSP, WB, BIGK>(a, s);
                case 4: return launch_stream_t<G, NWC, NWK, 1, 4, true, KSP, WB, BIGK>(a, s);
                case 5: return launch_stream_t<G, NWC, NWK, 1, 5, true, KSP, WB, BIGK>(a, s);
                default: return launch_stream_t<G, NWC, NWK, 1, 6, true, KSP, WB, BIGK>(a, s);
            }
        }
    }
    switch (stream_cell_rows_log2(a.M)) {
        case 2: return launch_stream_t<G, NWC, NWK, DT, 2, false, KSP, WB, BIGK>(a, s);
        case 4: return launch_stream_t<G, NWC, NWK, DT, 4, false, KSP, WB, BIGK>(a, s);
        case 5: return launch_stream_t<G, NWC, NWK, DT, 5, false, KSP, WB, BIGK>(a, s);
        default: return launch_stream_t<G, NWC, NWK, DT, 6, false, KSP, WB, BIGK>(a, s);
    }
}

// the shapes the automatic choice uses, for the other number formats: 2-bit weights and / or ranks above 64
template <int WB, bool BIGK>
static hipError_t launch_stream_reduced(int v, const StreamArgs& a, hipStream_t s) {
    switch (v) {
        case 11421: return launch_stream_rows<1, 4, 2, 1, 1, WB, BIGK>(a, s);
        case 12241: return launch_stream_rows<2, 2, 4, 1, 1, WB, BIGK>(a, s);
        case 12181: return launch_stream_rows<2, 1, 8, 1, 1, WB, BIGK>(a, s);
        case 12141: return launch_stream_rows<2, 1, 4, 1, 1, WB, BIGK>(a, s);
        case 11181: return launch_stream_rows<1, 1, 8, 1, 1, WB, BIGK>(a, s);
        case 11241: return launch_stream_rows<1, 2, 4, 1, 1, WB, BIGK>(a, s);
        case 21181: return launch_stream_rows<1, 1, 8, 1, 2, WB, BIGK>(a, s);
        case 21141: return launch_stream_rows<1, 1, 4, 1, 2, WB, BIGK>(a, s);
        default: return hipErrorInvalidValue;
    }
}

// variant = 10000 KSP + 1000 G + 100 NWC + 10 (NWK % 16) + DT: KSP workgroups per column block, G
// column groups per wavefront, NWC x NWK wavefronts per workgroup, weights DT steps ahead.
int stream_variant(const Layer& L, int64_t M, int variant) {
    if (variant != 0) return variant;
    if (M > 32) return 11421;                        // 33 to 64 tokens: two blocks of 32 per wavefront, two K slices
    // With ranks above 64 the T rows take 33 KB of LDS: beside them fit four K slices of up to 16 token rows, or two
    // of up to 32 (and nothing for more tokens: the dispatcher sends those to the tiled kernel).
    const bool big = L.kp > 64;
    if (big && M > 16) return 11421;
    if ((L.N32 + 3) / 4 >= 200) return 12241;        // wide layers
    const bool eight = M <= 16 && !big;
    if ((L.N32 + 1) / 2 >= 160) return eight ? 12181 : 12141;
    // narrow layers: one column group per workgroup, and a pair of workgroups per group when that
    // still leaves half of the compute units idle and the K range is worth sharing
    if (L.N32 <= 160 && L.KT >= 8) return eight ? 21181 : 21141;
    return eight ? 11181 : 11241;
}
bool stream_variant_adds_into_y(int variant) { return variant / 10000 == 2; }
int stream_variant_unpaired(const Layer& L, int64_t M) {
    if (L.kp > 64) return M <= 16 ? 11241 : 11421;
    return M <= 16 ? 11181 : 11241;
}
bool stream_takes_codes(int variant, int lr) { return lr >= 4 && !stream_variant_adds_into_y(variant); }

hipError_t launch_stream(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy, const Requant& rq,
                         int variant, hipStream_t s) {
    if (M == 0) return hipSuccess;
    StreamArgs a;
    a.Wt = L.Wt; a.Bt = L.Bt; a.Xcell = reinterpret_cast<const uint8_t*>(ws.Xh);
    a.Tpart = ws.Tpart; a.S = ws.S;
    a.Y = Y; a.ldy = ldy; a.M = M; a.N = L.N; a.KT = L.KT; a.N32 = L.N32; a.kp = L.kp; a.kp16 = L.kp16;
    a.Yc = rq.codes; a.Ye = rq.exps; a.ldyc = rq.ld;
    a.rec_bytes = L.w_rec_bytes; a.exp_bias = L.w_exp_bias;
    const int v = stream_variant(L, M, variant);
    if (rq.codes != nullptr && stream_variant_adds_into_y(v)) return hipErrorInvalidValue;   // a pair's sum is complete only in memory
    const bool bigk = L.kp > 64;
    if (L.w_bits == 2) return bigk ? launch_stream_reduced<2, true>(v, a, s) : launch_stream_reduced<2, false>(v, a, s);
    if (bigk) return launch_stream_reduced<4, true>(v, a, s);
    switch (v) {
        case 11441: return launch_stream_rows<1, 4, 4, 1, 1, 4, false>(a, s);
        case 11421: return launch_stream_rows<1, 4, 2, 1, 1, 4, false>(a, s);
        case 12241: return launch_stream_rows<2, 2, 4, 1, 1, 4, false>(a, s);
        case 12242: return launch_stream_rows<2, 2, 4, 2, 1, 4, false>(a, s);
        case 12181: return launch_stream_rows<2, 1, 8, 1, 1, 4, false>(a, s);
        case 12141: return launch_stream_rows<2, 1, 4, 1, 1, 4, false>(a, s);
        case 11181: return launch_stream_rows<1, 1, 8, 1, 1, 4, false>(a, s);
        case 11101: return launch_stream_rows<1, 1, 16, 1, 1, 4, false>(a, s);
        case 11281: return launch_stream_rows<1, 2, 8, 1, 1, 4, false>(a, s);
        case 11241: return launch_stream_rows<1, 2, 4, 1, 1, 4, false>(a, s);
        case 21181: return launch_stream_rows<1, 1, 8, 1, 2, 4, false>(a, s);
        case 21141: return launch_stream_rows<1, 1, 4, 1, 2, 4, false>(a, s);
        case 22181: return launch_stream_rows<2, 1, 8, 1, 2, 4, false>(a, s);
        case 22421: return launch_stream_rows<2, 4, 2, 1, 2, 4, false>(a, s);
        case 21441: return launch_stream_rows<1, 4, 4, 1, 2, 4, false>(a, s);
        case 21101: return launch_stream_rows<1, 1, 16, 1, 2, 4, false>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lqer
