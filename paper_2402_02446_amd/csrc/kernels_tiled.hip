// Stage 2, large-M ("prefill") form of Y = X_q W_q + T B_k (Eq. 3 / Eq. 6): an MFMA-bound tiled
// GEMM.  Sec. 2.1 observes that run-time dequantization is what costs weight-only schemes in the
// compute-bound regime, so here the weight expansion is kept to seven VALU instructions per 8
// elements (unpack_w8) and runs beside the matrix pipe.
//
// Workgroup tile BM x BN, WR x WC wavefronts, each owning TM x TN tiles of the 32x32x16 bf16
// MFMA (the shape one wavefront per SIMD can keep close to the matrix pipe's peak).  The
// contraction axis is walked in chunks of 64 = four MFMA steps; lane half hh owns blocks 2hh and
// 2hh+1 of a chunk for every operand, so block scales never cross lanes.
//   activations (bf16, exact dequantized X_q, then T_hi | T_lo): global -> registers two or three
//       chunks ahead -> a ring of four LDS stages of XOR-swizzled 16-byte cells -> ds_read_b128
//       operands shared by the wavefronts of a row;
//   weights: each wavefront loads the packed MXINT4 records of its own columns straight into
//       registers (fully coalesced 16-byte loads), three chunks ahead, into four register sets used
//       by name in turn (a copy between sets would force a wait on the newest load), and expands
//       them there;
//   the rank-kp correction is ceil(2 kp / 64) more chunks whose weight operand comes from B_k.
// MFMA operands are swapped (weights first) so a lane ends up with runs of four consecutive
// output columns of one token and stores each as one 16-byte write.
//
// Work split.  The launch is either one workgroup per output tile, or - when the tiles do not fill
// whole rounds of the chip - as many workgroups as the chip holds at once, each taking its share of
// whole tiles and, before them, an equal share of the K tiles of the remaining output tiles (those
// are cut wherever a share ends).  A workgroup whose share starts inside an output tile leaves its
// accumulators in a workspace slot of its own and raises a flag; the workgroup that has the start
// of that output tile adds the later pieces in K order and stores.  A share is one contiguous range,
// so only its first piece can be handed over and only its last piece can wait, and the waiting
// piece needs pieces that are computed first by the workgroups they belong to: no wait depends on
// another wait.  The sum order is fixed by the split, so the result has the same bits every run.
#include <atomic>
#include <mutex>
#include <type_traits>

#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

struct TiledArgs {
    const uint8_t* Wt; const uint8_t* Bt;
    const uint16_t* Xh; int64_t ldxh;
    const float* Tpart; int S; int64_t tp_stride;    // S > 1: T as S fp32 partial sums [S][tp_stride / kp rows][kp]
    float* Y; int64_t ldy;
    int8_t* Yc; uint8_t* Ye; int64_t ldyc;           // Yc != null: store Y as MXINT8 (blocks of 16 along N) instead of fp32
    int64_t M, N, KT, N32;
    int kp, kp16;
    int grid_m, grid_n;
    int group_m;
    // work split (see the head of this file)
    int64_t dp_tiles;          // output tiles taken whole, tile i by workgroup i % gridDim.x
    int64_t sk_units;          // K tile units of the remaining output tiles, shared out in ranges of ...
    int64_t sk_share;          // ... this many per workgroup
    int64_t sk_tile_units;     // units per remaining tile: KT, or KT rounded up to whole shares so that no share
                               // crosses a tile (the units past KT are empty)
    float* Part;               // [gridDim.x][BM * BN] accumulators handed over
    uint32_t* flags;           // [gridDim.x], zero before the launch; 1 = slot written
    int spin_limit;            // polls of a flag before the waiting workgroup gives up (and stores NaN)
    int rec_bytes;             // bytes of a weight record
    int exp_bias;              // >= 0: exponent nibbles (byte = nibble + exp_bias); -1: exponent bytes
};

// MINW = wavefronts per SIMD the register allocation must allow (2 lets two four-wavefront workgroups share a compute unit)
// SPLIT = the workgroup walks a list of pieces (work split); otherwise it computes output tile blockIdx.x
// whole, as straight-line code (the loop over pieces costs the main product a few percent)
// WB = mantissa bits of W_q: 4, or 2 (half the code bytes per record, one 32-bit word per block)
template <int TM, int TN, int WR, int WC, int NS, int MINW, bool SPLIT, int WB>
__global__ __launch_bounds__(64 * WR * WC, MINW) void tiled_kernel(TiledArgs a) {
    static_assert(WB == 4 || WB == 2, "weight mantissas of 4 or 2 bits");
    constexpr int BM = 32 * TM * WR;
    constexpr int NW = WR * WC;
    constexpr int STAGE = BM * 128;                // bytes: BM rows x 64 bf16
    constexpr int NT = 64 * NW;
    constexpr int LPT = BM * 8 / NT;               // 16-byte cells each thread moves per chunk
    // chunks between fetching activations and using them: 3 where the registers allow a second set in flight
    constexpr int XD = (TM * TN * 16 + LPT * 8 <= 144) ? 3 : 2;
    static_assert((BM * 8) % NT == 0, "loader must divide evenly");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform by construction
    const int wr = wave / WC, wc = wave % WC;
    const int t = lane & 31, hh = lane >> 5;

    // ---- workgroup -> position in the work split: consecutive positions land on one XCD ----------
    int lin;
    {
        const int nwg = gridDim.x;
        const int pid = blockIdx.x;
        const int xcd = pid & 7, local = pid >> 3;
        const int per = nwg >> 3, rem = nwg & 7;
        lin = (xcd < rem) ? xcd * (per + 1) + local : rem * (per + 1) + (xcd - rem) * per + local;
    }
    __shared__ int wait_ok;
    const int KT = (int)a.KT;                                  // K tiles and chunks fit 32 bits: scalar compares
    const int main_chunks = KT * 4;
    const int nb2 = 2 * a.kp16;
    const int tail_chunks = (nb2 + 3) / 4;
    static_assert(NS == 4, "stage and register-set indices below assume rings of four");
    constexpr int ROWS_PER_PASS = NT / 8;
    static_assert(ROWS_PER_PASS % 16 == 0, "swizzle must not depend on the pass");
    const int ld_row0 = tid >> 3;
    // (row >> 1) & 7 is the same for every pass because ROWS_PER_PASS is a multiple of 16
    const int ld_dst0 = ld_row0 * 128 + (((tid & 7) ^ ((ld_row0 >> 1) & 7)) << 4);
    // ---- operand reader: in step s this lane reads logical cell 4 hh + s of its TM rows -----------
    // row = (wr TM + tm) 32 + t, so the swizzle term depends on t only
    int rd_off[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
        rd_off[s4] = (wr * TM * 32 + t) * 128 + (((4 * hh + s4) ^ ((t >> 1) & 7)) << 4);
    const int lane16 = lane * 16;
    // exponent of a block without a branch in the main loop: bytes (16, 8, 0xFF, 0) or nibbles (8, 4, 0xF, bias)
    const bool exp4 = a.exp_bias >= 0;                          // wave-uniform
    const int es1 = exp4 ? 8 : 16, es0 = exp4 ? 4 : 8;
    const uint32_t emask = exp4 ? 0xFu : 0xFFu, ebias = exp4 ? (uint32_t)a.exp_bias : 0u;
    // nibbles sit in front of the codes (lane * 4), bytes behind them (lane * 8)
    const int code_off = exp4 ? kWCompactCodeOffset : 0, exp_off = exp4 ? lane16 >> 2 : w_code_bytes(WB) + (lane16 >> 1);

    int64_t dp_next = lin;                                     // next whole tile of this workgroup
    int64_t u = a.sk_share * lin;                              // its range of the shared K tiles
    int64_t u_end = u + a.sk_share;
    if (u_end > a.sk_units) u_end = a.sk_units;
    bool first_piece = true;
  for (;;) {
    // ---- next piece: output tile and K tiles [kt0, kt1) -------------------------------------------
    int64_t tile_lin;
    int kt0, kt1;
    // The shared K tiles come first: the hand-over between workgroups then overlaps with the whole
    // tiles of other workgroups instead of ending the kernel.
    if constexpr (!SPLIT) {
        tile_lin = lin; kt0 = 0; kt1 = KT;
    } else if (u < u_end) {
        const int64_t rt = u / a.sk_tile_units;
        tile_lin = a.dp_tiles + rt;
        kt0 = (int)(u - rt * a.sk_tile_units);
        const int64_t left = u_end - u;
        if (kt0 >= KT) {                                       // only empty units of this tile are left
            u += (left < a.sk_tile_units - kt0) ? left : a.sk_tile_units - kt0;
            continue;
        }
        kt1 = (left < (int64_t)(KT - kt0)) ? kt0 + (int)left : KT;
        u += (kt1 == KT) ? a.sk_tile_units - kt0 : kt1 - kt0;  // past the tile's empty units as well
        if (u > u_end) u = u_end;
    } else if (dp_next < a.dp_tiles) {
        tile_lin = dp_next; kt0 = 0; kt1 = KT;
        dp_next += gridDim.x;
    } else {
        break;
    }
    const bool owner = !SPLIT || (kt0 == 0);                   // this piece stores the tile
    if constexpr (SPLIT) {
        if (!first_piece) __syncthreads();                     // every wavefront is done with the LDS stages
        first_piece = false;
    }
    // output tiles are walked in bands of group_m tile rows
    int tile_m, tile_n;
    {
        const int64_t width = (int64_t)a.group_m * a.grid_n;
        const int grp = (int)(tile_lin / width);
        const int in = (int)(tile_lin - grp * width);
        const int first_m = grp * a.group_m;
        const int gsize = (a.grid_m - first_m < a.group_m) ? a.grid_m - first_m : a.group_m;
        tile_m = first_m + in % gsize;
        tile_n = in / gsize;
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    // ---- activation loader: thread -> 16-byte cells of a stage -----------------------------------
    // Cell j of this thread is row (tid >> 3) + j * (NT / 8), 16-byte column tid & 7.  Rows past M are
    // read as they are (the workspace rows are padded to the tile height) and never stored.
    const uint16_t* ld_base = a.Xh + (m0 + ld_row0) * a.ldxh + 8 * (tid & 7);
    const int64_t ld_stride = (int64_t)ROWS_PER_PASS * a.ldxh;           // elements between passes
    const int64_t g0 = ((int64_t)tile_n * WC + wc) * TN;       // first column group of this wavefront
    auto group_of = [&](int tn) {
        const int64_t g = g0 + tn;
        return g < a.N32 ? g : a.N32 - 1;                      // clamp; the store is masked
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    typedef typename std::conditional<WB == 4, u32x4, u32x2>::type WVec;   // a lane's two blocks of one chunk
    struct WSet {                // packed codes of one chunk for this wavefront's TN column groups
        WVec c[TN];
    };
    struct ESet {                // exponent bytes of one K tile (four chunks) for the same groups
        u32x2 e[TN];
    };
    auto load_wset = [&](WSet& w, int ch) {
        const int64_t tile = ch >> 2;
        const int cc = ch & 3;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const uint8_t* rec = a.Wt + (tile * a.N32 + group_of(tn)) * a.rec_bytes;   // wave-uniform
            if constexpr (WB == 4) w.c[tn] = *reinterpret_cast<const u32x4*>(rec + code_off + cc * 1024 + lane16);
            else w.c[tn] = *reinterpret_cast<const u32x2*>(rec + code_off + (cc >> 1) * 1024 + lane16 + (cc & 1) * 8);
        }
    };
    auto load_eset = [&](ESet& x, int tile_i) {
        const int64_t tile = tile_i;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const uint8_t* rec = a.Wt + (tile * a.N32 + group_of(tn)) * a.rec_bytes;
            // always 8 bytes wide: with nibbles only the first word is used (the buffer is padded behind the last record)
            const u32x2_a4 w = *reinterpret_cast<const u32x2_a4*>(rec + exp_off);
            x.e[tn] = u32x2{w[0], exp4 ? w[0] >> 16 : w[1]};
        }
    };
    auto fetch_x = [&](u32x4 (&st)[LPT], int ch) {
#pragma unroll
        for (int j = 0; j < LPT; ++j) st[j] = *reinterpret_cast<const u32x4*>(ld_base + j * ld_stride + (int64_t)ch * 64);
    };
    // Correction chunk tc when the projection kernel left T as S partial sums (it split K over
    // workgroups): add them in slice order and form the bf16 term this cell holds - T_hi for tail
    // columns below kp, T_lo for the next kp, zero behind.
    auto fetch_t = [&](u32x4 (&st)[LPT], int tc) {
        const int col = (int)tc * 64 + 8 * (tid & 7);
        const bool lo = col >= a.kp;
        const int r0 = lo ? col - a.kp : col;
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            float sum[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] = 0.f;
            if (col < 2 * a.kp) {
                const float* src = a.Tpart + (m0 + ld_row0 + j * ROWS_PER_PASS) * a.kp + r0;
                for (int sl = 0; sl < a.S; ++sl) {
                    const f32x4 p0 = *reinterpret_cast<const f32x4*>(src + sl * a.tp_stride);
                    const f32x4 p1 = *reinterpret_cast<const f32x4*>(src + sl * a.tp_stride + 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) { sum[e] += p0[e]; sum[4 + e] += p1[e]; }
                }
            }
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t hb = f32_bits(sum[e]) & 0xFFFF0000u;
                h[e] = lo ? f32_bits(sum[e] - f32_from_bits(hb)) >> 16 : hb >> 16;
            }
            st[j] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        }
    };
    // any chunk of the activation row: a main one or a correction chunk in either form
    auto fetch_any = [&](u32x4 (&st)[LPT], int ch) {
        if (ch < main_chunks || a.S <= 1) fetch_x(st, ch);
        else fetch_t(st, ch - main_chunks);
    };
    auto store_x = [&](const u32x4 (&st)[LPT], int stage) {
#pragma unroll
        for (int j = 0; j < LPT; ++j)
            *reinterpret_cast<u32x4*>(lds + stage * STAGE + ld_dst0 + j * ROWS_PER_PASS * 128) = st[j];
    };
    // one 64-wide chunk of the main product: c = chunk index within its K tile = stage = register set.
    // The activation operands are read one MFMA step ahead: `xa` holds step 0 on entry and step 0
    // of the next chunk on exit (that stage was completed two barriers ago, so it may be read
    // before the next barrier).
    Frag xa[TM];
    auto read_xa = [&](Frag (&dst)[TM], int stage_idx, int s4) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
            dst[tm].u = *reinterpret_cast<const u32x4*>(lds + stage_idx * STAGE + rd_off[s4] + tm * 4096);
    };
    auto mma_chunk = [&](const WSet& w, const ESet& x, int c) {
        float sc[TN][2];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const uint32_t ew = x.e[tn][c >> 1] >> ((c & 1) * es1);
            sc[tn][0] = (WB == 4) ? w_scale((ew & emask) + ebias) : w2_scale((ew & emask) + ebias);
            sc[tn][1] = (WB == 4) ? w_scale(((ew >> es0) & emask) + ebias) : w2_scale(((ew >> es0) & emask) + ebias);
        }
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            Frag xn[TM];
            if (s4 < 3) read_xa(xn, c, s4 + 1);
            else read_xa(xn, (c + 1) & 3, 0);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                bf16x8 wv;
                if constexpr (WB == 4) wv = unpack_w8(w.c[tn][s4], sc[tn][s4 >> 1]);
                else wv = unpack_w8_b2(w.c[tn][s4 >> 1], s4 & 1, sc[tn][s4 >> 1]);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) acc[tm][tn] = mfma32(wv, xa[tm].v, acc[tm][tn]);
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) xa[tm] = xn[tm];
        }
    };

    // prologue: activations of the piece's first two chunks into stages 0 and 1, the weights of its
    // first three, and (XD == 3) the activations of the third in registers
    // (a K tile is four chunks, so a piece has at least four)
    const int first_ch = kt0 * 4;
    WSet w0, w1, w2, w3;
    ESet ea, eb;
    u32x4 sta[LPT], stb[LPT];                      // activations on their way to LDS (stb: XD == 3 only)
    {
        fetch_x(sta, first_ch);
        load_eset(ea, kt0);
        load_wset(w0, first_ch);
        store_x(sta, 0);
        fetch_x(sta, first_ch + 1);
        load_wset(w1, first_ch + 1);
        store_x(sta, 1);
        if constexpr (XD == 3) fetch_x(sta, first_ch + 2);
        load_wset(w2, first_ch + 2);
    }

    // ---- main product -----------------------------------------------------------------------------
    // chunk ch: barrier; fetch the weights of chunk ch+3 into the register set chunk ch-1 has left,
    // and the activations of chunk ch+XD; arithmetic of chunk ch; write the activations of chunk ch+2
    // into stage (ch+2)%4, which was last read two barriers ago.  With XD == 3 those were fetched
    // during the previous chunk and waited in registers (two sets, used in turn), so both kinds of
    // load have more than two chunks' time to arrive: measured with the loads taken out, a
    // distance of two left a fifth of the kernel's time waiting for them.
    // Exponent bytes of the next tile are fetched during the second chunk of a tile.
    // Every load below is issued unconditionally, with its index clamped at the end of the range:
    // a load inside a branch would make the compiler's wait counts assume the worst case and the
    // LDS write at the end of the chunk would wait for the newest weights as well.
    const int last_main = kt1 * 4 - 1, last_tile = kt1 - 1;
    auto step = [&](const WSet& cur, const ESet& ecur, WSet& fill, ESet& enext, u32x4 (&st_old)[LPT],
                    u32x4 (&st_new)[LPT], int ch, int c) {
        __syncthreads();
        if (ch == first_ch) read_xa(xa, 0, 0);   // later chunks find step 0 already read by the previous one
        fetch_x(st_new, ch + XD < last_main ? ch + XD : last_main);
        // loads retire in order: keep the activation loads ahead of the weight loads, so that the
        // LDS write at the end of this chunk does not have to wait for the weights fetched here
        __builtin_amdgcn_sched_barrier(0);
        load_wset(fill, ch + 3 < last_main ? ch + 3 : last_main);
        if (c == 1) load_eset(enext, (ch >> 2) + 1 < last_tile ? (ch >> 2) + 1 : last_tile);
        mma_chunk(cur, ecur, c);
        store_x(st_old, (c + 2) & 3);  // stage (ch+2)%4: free since two barriers ago, also for a clamped re-write
    };
    // XD == 2: one set, fetched and written in the same chunk
    u32x4 (&st_even_old)[LPT] = sta;
    u32x4 (&st_even_new)[LPT] = (XD == 3) ? stb : sta;
    u32x4 (&st_odd_old)[LPT] = (XD == 3) ? stb : sta;
    u32x4 (&st_odd_new)[LPT] = sta;
    for (int tile = kt0; tile < kt1; tile += 2) {
        step(w0, ea, w3, eb, st_even_old, st_even_new, tile * 4 + 0, 0);
        step(w1, ea, w0, eb, st_odd_old, st_odd_new, tile * 4 + 1, 1);
        step(w2, ea, w1, eb, st_even_old, st_even_new, tile * 4 + 2, 2);
        step(w3, ea, w2, eb, st_odd_old, st_odd_new, tile * 4 + 3, 3);
        if (tile + 1 < kt1) {
            step(w0, eb, w3, ea, st_even_old, st_even_new, tile * 4 + 4, 0);
            step(w1, eb, w0, ea, st_odd_old, st_odd_new, tile * 4 + 5, 1);
            step(w2, eb, w1, ea, st_even_old, st_even_new, tile * 4 + 6, 2);
            step(w3, eb, w2, ea, st_odd_old, st_odd_new, tile * 4 + 7, 3);
        }
    }

    // ---- rank-kp correction: [T_hi | T_lo | 0] against B_k ---------------------------------------
    // The correction chunks are fetched here rather than ahead from the main loop: B_k's
    // records are needed at the same moment and cost the same memory round trip.  Stages 0 and 1 are
    // free: every wavefront is past the barrier of the last main chunk, which reads stage 3.
    // lane half hh owns rank blocks jb = 4 cc + 2 hh + {0, 1} of tail chunk cc
    // Lane indices for everything behind the main loop come through an opaque copy: address terms
    // built from them would otherwise be computed once in front of the loop over pieces and
    // occupy registers all through the main product.
    int t_e = t, hh_e = hh, lane_e = lane;
    if constexpr (SPLIT) asm volatile("" : "+v"(t_e), "+v"(hh_e), "+v"(lane_e));
    const int my_tail = owner ? tail_chunks : 0;              // the piece that stores the tile adds the correction
    // two correction chunks at a time through stages 0 and 1 (ranks up to 64 need one round, 256 four)
    for (int cc0 = 0; cc0 < my_tail; cc0 += 2) {
        {
            u32x4 tst[2][LPT];
            if (cc0 > 0) __syncthreads();                      // every wavefront has read the previous pair of chunks
            fetch_any(tst[0], main_chunks + cc0);
            if (cc0 + 1 < tail_chunks) fetch_any(tst[1], main_chunks + cc0 + 1);
            store_x(tst[0], 0);
            if (cc0 + 1 < tail_chunks) store_x(tst[1], 1);
            __syncthreads();
        }
        for (int cc = cc0; cc < cc0 + 2 && cc < my_tail; ++cc) {
            const uint8_t* stage = lds + (cc & 1) * STAGE;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int jb = 4 * cc + 2 * hh_e + j;
                const bool live = jb < nb2;
                const int rb = live ? (jb < a.kp16 ? jb : jb - a.kp16) : 0;
                Frag bf[TN][2];
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    u32x4 cw = u32x4{0, 0, 0, 0};
                    uint32_t eb = 0;
                    if (live) {
                        const uint8_t* rec = a.Bt + (group_of(tn) * a.kp16 + rb) * kBRecordBytes;
                        cw = *reinterpret_cast<const u32x4*>(rec + t_e * 16);
                        eb = rec[512 + t_e];
                    }
                    int8x16_to_frags(cw, h_scale(eb), bf[tn][0], bf[tn][1]);
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    Frag xa[TM];
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
                        xa[tm].u = *reinterpret_cast<const u32x4*>(stage + rd_off[2 * j + h] + tm * 4096);
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) acc[tm][tn] = mfma32(bf[tn][h].v, xa[tm].v, acc[tm][tn]);
                }
            }
        }
    }

    // ---- a piece that starts inside the tile hands its accumulators over ---------------------------
    // The slot is written and read with device-scope relaxed atomic accesses of 8 bytes: they pass
    // through the XCD's L2 to where every XCD sees them, so neither side needs a cache write-back or
    // invalidate (which would also throw out the weights and activations other workgroups share there).
    constexpr int64_t PART_FLOATS = (int64_t)NW * TM * TN * 1024;          // = BM x BN
    typedef unsigned long long u64;
    union Pair { u64 q; float f[2]; };
    if (SPLIT && !owner) {
        u64* slot = reinterpret_cast<u64*>(a.Part + (int64_t)lin * PART_FLOATS) + (int64_t)wave * TM * TN * 8 * 64 + lane_e;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int h8 = 0; h8 < 8; ++h8) {
                    Pair p;
                    p.f[0] = acc[tm][tn][2 * h8]; p.f[1] = acc[tm][tn][2 * h8 + 1];
                    __hip_atomic_store(slot + ((tm * TN + tn) * 8 + h8) * 64, p.q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
        // The flag may only be raised once every slot store of every wavefront has been acknowledged by the
        // memory system: a workgroup-scope fence does not wait for outstanding vector stores on this chip
        // (and a device-scope release would write the XCD's L2 back), so each wavefront drains its own
        // store counter explicitly, the barrier collects all wavefronts, and only then is the flag stored.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) __hip_atomic_store(a.flags + lin, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        continue;
    }
    // ---- the piece with the start of the tile adds the later pieces, in K order --------------------
    if (SPLIT && kt1 < KT) {
        const int64_t rt = tile_lin - a.dp_tiles;
        const int64_t last_wg = (rt * a.sk_tile_units + a.KT - 1) / a.sk_share;   // workgroup with the tile's last K tile
        for (int64_t w = lin + 1; w <= last_wg; ++w) {
            if (tid == 0) {
                int polls = 0;
                while (__hip_atomic_load(a.flags + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u &&
                       polls < a.spin_limit) {
                    __builtin_amdgcn_s_sleep(8);
                    ++polls;
                }
                wait_ok = (polls < a.spin_limit) ? 1 : 0;
            }
            __syncthreads();
            const bool ok = wait_ok != 0;
            const u64* slot = reinterpret_cast<const u64*>(a.Part + w * PART_FLOATS) + (int64_t)wave * TM * TN * 8 * 64 + lane_e;
            // groups of 32 loads: enough in flight to cover the round trip, few enough to fit beside the accumulators
            constexpr int PER = TM * TN * 8;                   // 8-byte words of this lane in the slot
            constexpr int GRP = PER < 32 ? PER : 32;
            static_assert(PER % GRP == 0, "whole groups");
#pragma unroll
            for (int g0 = 0; g0 < PER; g0 += GRP) {
                Pair p[GRP];
#pragma unroll
                for (int i = 0; i < GRP; ++i)
                    p[i].q = __hip_atomic_load(slot + (g0 + i) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int i = 0; i < GRP; ++i) {
                    const int mt = (g0 + i) / 8, h8 = (g0 + i) % 8;
                    // a piece that never arrived must not pass for a result
                    if (!ok) p[i].f[0] = p[i].f[1] = __builtin_nanf("");
                    acc[mt / TN][mt % TN][2 * h8] += p[i].f[0];
                    acc[mt / TN][mt % TN][2 * h8 + 1] += p[i].f[1];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();                                   // wait_ok may be rewritten
        }
    }

    // ---- store: lane (t, hh) holds columns 8 r4 + 4 hh .. + 3 of token t for every MFMA tile ------
    // As MXINT8 for the next layer: block b of a column group is columns 16 b .. 16 b + 15 = accumulator
    // registers 8 b .. 8 b + 7 of this lane and of lane ^ 32 (the same token).
    if (a.Yc != nullptr) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int64_t row = m0 + (wr * TM + tm) * 32 + t_e;
            if (row >= a.M) continue;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int64_t cg = g0 + tn;
                if (cg >= a.N32) continue;
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    float v[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = acc[tm][tn][8 * b + i];
                    uint32_t w0, w1;
                    const uint32_t eb = requant_half_block(v, w0, w1);
                    const int64_t n0 = cg * 32 + 16 * b;
                    if (n0 < a.N) {
                        int8_t* dst = a.Yc + row * a.ldyc + n0 + 4 * hh_e;
                        *reinterpret_cast<uint32_t*>(dst) = w0;
                        *reinterpret_cast<uint32_t*>(dst + 8) = w1;
                        if (hh_e == 0) a.Ye[row * (a.N >> 4) + (n0 >> 4)] = (uint8_t)eb;
                    }
                }
            }
        }
        if constexpr (!SPLIT) break; else continue;
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t row = m0 + (wr * TM + tm) * 32 + t_e;
        if (row >= a.M) continue;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int64_t cg = g0 + tn;
            if (cg >= a.N32) continue;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int64_t n = cg * 32 + 8 * r4 + 4 * hh_e;
                float* dst = a.Y + row * a.ldy + n;
                const f32x4 v = f32x4{acc[tm][tn][4 * r4], acc[tm][tn][4 * r4 + 1], acc[tm][tn][4 * r4 + 2], acc[tm][tn][4 * r4 + 3]};
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
    if constexpr (!SPLIT) break;
  }   // pieces
}

// Time estimates in microseconds for one tile shape, launched as one workgroup per tile or with the
// work split described at the head of this file.
struct TileShape { int id, bm, bn, share; double pair, single, cut; };
// whole-chip TFLOP/s measured on an 8192 x 28672 layer: `pair` with `share` workgroups on every compute unit
// (M = 4096), `single` with one (M = 128), `cut` for the pieces of tiles cut along K (M = 128 .. 2048)
static const TileShape kShapes[] = {
    {11, 128, 512, 1, 1372.0, 1372.0, 1372.0}, {12, 128, 256, 2, 1300.0, 1000.0, 1150.0}, {4, 128, 128, 2, 1058.0, 800.0, 1058.0},
};
constexpr double kPieceUs = 4.0;       // filling the pipeline and storing the tile, per piece
constexpr double kSplitFixedUs = 38.0; // what a split launch was measured to take beyond this, per workgroup sharing a compute unit: the
                                       // pieces' drain and refill, not the slots' way through memory (the time is the same without them)

struct Split { int64_t grid, dp_tiles, sk_units, sk_share, sk_tile_units; bool aligned; };

static Split whole_tiles(int64_t tiles, int64_t KT) { return Split{tiles, tiles, 0, 1, KT, false}; }

// slots = workgroups the chip holds at once.
// aligned: where the chip holds two or more workgroups per remaining tile, every such tile is cut into the same
// whole number of pieces, one per workgroup, instead of equal shares of all remaining K tiles: a share then never
// crosses a tile, so no workgroup gets a second (possibly tiny) piece.  Measured on 11008 x 4096 at M = 2048
// (128 tiles of 43 K tiles on 256 workgroups): 157 us against 172 us with equal shares.
static Split split_tiles(int64_t tiles, int64_t KT, int64_t slots, bool aligned) {
    Split sp;
    sp.grid = slots;
    sp.dp_tiles = (tiles / slots) * slots;
    const int64_t rem = tiles - sp.dp_tiles;
    if (rem == 0) return whole_tiles(tiles, KT);
    const int64_t p = slots / rem;                           // pieces per remaining tile
    if (aligned && p >= 2 && KT / p >= 2) {
        sp.sk_share = (KT + p - 1) / p;
        sp.sk_tile_units = sp.sk_share * p;
        sp.sk_units = rem * sp.sk_tile_units;
        sp.aligned = true;
        return sp;
    }
    sp.aligned = false;
    sp.sk_tile_units = KT;
    sp.sk_units = rem * KT;
    sp.sk_share = (sp.sk_units + slots - 1) / slots;
    if (sp.sk_share < 2) sp.sk_share = 2;                    // a piece is worth its hand-over
    return sp;
}

// one K tile (256 deep) of one output tile, with `share` workgroups on every compute unit
static double unit_us(const TileShape& sh, int share, int cus) {
    const double rate = (share == sh.share) ? sh.pair : sh.single;       // TFLOP/s = flop/us * 1e-6
    return 2.0 * sh.bm * sh.bn * kTileK * (double)cus * share / (rate * 1e6);
}

static double time_whole(const TileShape& sh, int64_t tiles, int64_t KT, int cus) {
    const int64_t n = (tiles + cus - 1) / cus;               // tiles of the busiest compute unit
    const double full = (double)KT * unit_us(sh, sh.share, cus) + kPieceUs;
    const double alone = (double)KT * unit_us(sh, 1, cus) + kPieceUs;
    return (sh.share == 2) ? (double)(n / 2) * full + (double)(n % 2) * alone : (double)n * full;
}

static double time_split(const TileShape& sh, int64_t tiles, int64_t KT, int cus) {
    const Split sp = split_tiles(tiles, KT, (int64_t)cus * sh.share, true);
    const bool one_piece = sp.aligned;                       // cut along tile boundaries: no workgroup gets two pieces
    if (sp.sk_units == 0) return time_whole(sh, tiles, KT, cus);
    const double rounds = (double)(sp.dp_tiles / sp.grid);
    const double whole_part = rounds * (double)KT * unit_us(sh, sh.share, cus);
    const double cut_part = (double)sp.sk_share * unit_us(sh, sh.share, cus) * sh.pair / sh.cut;
    if (!one_piece) return whole_part + cut_part + (rounds + 2.0) * kPieceUs + kSplitFixedUs * sh.share;
    // cut along tiles: one piece per workgroup; the workgroup with a tile's first piece reads the slots of the
    // others one after the other (about 7 us per 256 KiB slot beyond the first, from launches with 2 and 4 pieces)
    const double pieces = (double)(sp.sk_tile_units / sp.sk_share);
    const double slot_us = 7.0 * (double)sh.bm * sh.bn * 4.0 / 262144.0;
    return whole_part + cut_part + (rounds + 1.0) * kPieceUs + 0.5 * kSplitFixedUs + (pieces - 2.0) * slot_us;
}

// the split has to promise a clear gain: its estimate is the rougher of the two
static bool split_pays(const TileShape& sh, int64_t tiles, int64_t KT, int cus) {
    return time_split(sh, tiles, KT, cus) < 0.95 * time_whole(sh, tiles, KT, cus);
}

// What has to be established once per kernel instance and process: the dynamic LDS limit, and how many of its
// workgroups one compute unit really holds (the work split launches exactly as many workgroups as are resident
// at once, because owners wait for flags that later workgroups raise).
struct KernelSetup {
    std::once_flag once;
    hipError_t err = hipSuccess;
    int resident = 0;            // workgroups per compute unit
};

template <typename Kern>
static hipError_t prepare_kernel(Kern kern, KernelSetup& ks, int lds_bytes, int threads) {
    std::call_once(ks.once, [&] {
        ks.err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (ks.err != hipSuccess) return;
        int n = 0;
        ks.err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, (size_t)lds_bytes);
        ks.resident = n;
    });
    return ks.err;
}

template <typename Kern>
static hipError_t launch_kernel(Kern kern, KernelSetup& ks, int lds_bytes, int64_t grid_x, int threads, const TiledArgs& a, hipStream_t s) {
    const hipError_t e = prepare_kernel(kern, ks, lds_bytes, threads);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid_x), dim3(threads), lds_bytes, s, a);
    return hipGetLastError();
}

// CAN_SPLIT: the shape also exists in the form that walks a list of pieces
template <int WB, int TM, int TN, int WR, int WC, int NS, int MINW = 1, bool CAN_SPLIT = false>
static hipError_t launch_tiled_t(TiledArgs a, int64_t M, int mode, int cus, hipStream_t s) {
    constexpr int BM = 32 * TM * WR, BN = 32 * TN * WC;
    constexpr int LDS_BYTES = NS * BM * 128;
    a.grid_m = (int)((M + BM - 1) / BM);
    a.grid_n = (int)((a.N + BN - 1) / BN);
    a.group_m = 8;
    const int64_t tiles = (int64_t)a.grid_m * a.grid_n;
    TileShape me = {0, BM, BN, MINW, 1.0, 1.0, 1.0};
    for (const TileShape& sh : kShapes)
        if (sh.bm == BM && sh.bn == BN && sh.share == MINW) me = sh;
    static KernelSetup setup_split, setup_whole;
    // The split launches one workgroup per slot and its owners wait for workgroups with higher numbers: all of
    // them must be resident at once.  The number the runtime reports for this instance decides, not the launch
    // bounds; should it ever be lower than the shape assumes, tiles are not cut.
    bool can_split = CAN_SPLIT;
    if constexpr (CAN_SPLIT) {
        const hipError_t e = prepare_kernel(tiled_kernel<TM, TN, WR, WC, NS, MINW, true, WB>, setup_split, LDS_BYTES, 64 * WR * WC);
        if (e != hipSuccess) return e;
        if (setup_split.resident < MINW) can_split = false;
    }
    const int64_t slots = (int64_t)cus * MINW;
    // mode 0: split when the estimate says so; 1: never; 2: whenever there is a remainder to split; 3: the same, always in
    // equal shares of the remaining K tiles (never along tile boundaries)
    bool split = false;
    if (can_split && a.Part != nullptr && (int64_t)BM * BN * 4 * slots <= kTiledPartBytesPerCu * (int64_t)cus && slots <= kTiledFlags) {
        if (mode >= 2) split = true;
        else if (mode == 0) split = split_pays(me, tiles, a.KT, cus);
    }
    if (mode >= 2 && !split) return hipErrorInvalidValue;      // asked for, not available
    const Split sp = split ? split_tiles(tiles, a.KT, slots, mode != 3) : whole_tiles(tiles, a.KT);
    a.dp_tiles = sp.dp_tiles; a.sk_units = sp.sk_units; a.sk_share = sp.sk_share; a.sk_tile_units = sp.sk_tile_units;
    if constexpr (CAN_SPLIT) {
        if (sp.sk_units > 0)
            return launch_kernel(tiled_kernel<TM, TN, WR, WC, NS, MINW, true, WB>, setup_split, LDS_BYTES, sp.grid, 64 * WR * WC, a, s);
    }
    return launch_kernel(tiled_kernel<TM, TN, WR, WC, NS, MINW, false, WB>, setup_whole, LDS_BYTES, tiles, 64 * WR * WC, a, s);
}

__global__ void clear_flags_kernel(uint32_t* flags, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flags[i] = 0u;
}

// For a tiled launch that does not follow the projection kernel (which clears the flags itself).
hipError_t launch_clear_flags(const Workspace& ws, hipStream_t s) {
    if (ws.flags == nullptr) return hipSuccess;
    hipLaunchKernelGGL(clear_flags_kernel, dim3((kTiledFlags + 255) / 256), dim3(256), 0, s, ws.flags, kTiledFlags);
    return hipGetLastError();
}

static std::atomic<int> g_wait_limit{1 << 22};
int tiled_wait_limit() { return g_wait_limit.load(); }
void set_tiled_wait_limit(int polls) { g_wait_limit.store(polls); }

int compute_units() {
    static int cus = 0;                                      // one kind of device per process
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cus = n;
    }
    return cus;
}

hipError_t launch_tiled(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy, const Requant& rq,
                        int variant, hipStream_t s) {
    if (M == 0) return hipSuccess;
    TiledArgs a;
    a.Wt = L.Wt; a.Bt = L.Bt; a.Xh = ws.Xh; a.ldxh = ws.ldxh; a.Y = Y; a.ldy = ldy;
    a.Yc = rq.codes; a.Ye = rq.exps; a.ldyc = rq.ld;
    a.Tpart = ws.Tpart; a.S = ws.S; a.tp_stride = ws.tp_rows * L.kp;
    a.M = M; a.N = L.N; a.KT = L.KT; a.N32 = L.N32; a.kp = L.kp; a.kp16 = L.kp16;
    a.grid_m = a.grid_n = 0; a.group_m = 8;
    a.Part = ws.Part; a.flags = ws.flags;
    a.rec_bytes = L.w_rec_bytes; a.exp_bias = L.w_exp_bias;
    a.spin_limit = tiled_wait_limit();                       // by default about a second of polling
    a.dp_tiles = a.sk_units = 0; a.sk_share = 1; a.sk_tile_units = L.KT;
    const int cus = compute_units();
    // variant = 100 * mode + tile shape; mode 0 = split the work when the estimate says so, 1 = never, 2 = always,
    // 3 = always and in equal shares
    int mode = variant / 100;
    variant %= 100;
    if (mode < 0 || mode > 3) return hipErrorInvalidValue;
    if (variant == 0) {
        // pick the tile shape (and the split) with the lowest estimated time
        double best = 0.0;
        for (const TileShape& entry : kShapes) {
            TileShape sh = entry;
            int64_t KT = L.KT;
            if (L.w_bits == 2) {
                // the 2-bit instances against the table's 4-bit rates, and the correction's extra K columns, which at the
                // ranks such layers come with are no longer small (measured on 4096 x 4096 at 2048 tokens and rank 256:
                // 128 x 512 cut along K 103 us, 128 x 256 114 us, 128 x 128 113 us)
                const double f = sh.id == 11 ? 0.85 : 0.7;
                sh.pair *= f; sh.single *= f; sh.cut *= f;
                KT += (2 * L.kp + kTileK - 1) / kTileK;
            }
            const int64_t tiles = ((M + sh.bm - 1) / sh.bm) * ((L.N + sh.bn - 1) / sh.bn);
            double t = time_whole(sh, tiles, KT, cus);
            if (mode >= 2 && ws.Part != nullptr) t = time_split(sh, tiles, KT, cus);
            else if (mode == 0 && ws.Part != nullptr && split_pays(sh, tiles, KT, cus)) t = time_split(sh, tiles, KT, cus);
            if (variant == 0 || t < best) { best = t; variant = sh.id; }
        }
    }
    if (L.w_bits == 2) {
        // 2-bit weights: the three shapes the automatic choice uses
        switch (variant) {
            case 4: return launch_tiled_t<2, 2, 2, 2, 2, 4, 2, true>(a, M, mode, cus, s);
            case 11: return launch_tiled_t<2, 4, 2, 1, 8, 4, 1, true>(a, M, mode, cus, s);
            case 12: return launch_tiled_t<2, 4, 2, 1, 4, 4, 2, true>(a, M, mode, cus, s);
            default: return hipErrorInvalidValue;
        }
    }
    switch (variant) {
        case 1: return launch_tiled_t<4, 4, 4, 2, 2, 4>(a, M, mode, cus, s);      // 256 x 256
        case 3: return launch_tiled_t<4, 2, 4, 2, 2, 4>(a, M, mode, cus, s);      // 128 x 256
        case 4: return launch_tiled_t<4, 2, 2, 2, 2, 4, 2, true>(a, M, mode, cus, s);   // 128 x 128, two workgroups per compute unit
        case 7: return launch_tiled_t<4, 2, 4, 2, 4, 4>(a, M, mode, cus, s);      // 128 x 512, eight wavefronts
        case 8: return launch_tiled_t<4, 2, 4, 2, 2, 4, 2>(a, M, mode, cus, s);   // 128 x 256, two workgroups per compute unit
        case 11: return launch_tiled_t<4, 4, 2, 1, 8, 4, 1, true>(a, M, mode, cus, s);     // 128 x 512, eight wavefronts, each 128 x 64
        case 12: return launch_tiled_t<4, 4, 2, 1, 4, 4, 2, true>(a, M, mode, cus, s);  // 128 x 256, four wavefronts each 128 x 64, two workgroups per compute unit
        case 13: return launch_tiled_t<4, 4, 2, 1, 4, 4>(a, M, mode, cus, s);     // 128 x 256, four wavefronts each 128 x 64
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lqer
