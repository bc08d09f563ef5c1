// Stage 2, large-M ("prefill") form of Y = X_q W_q + T B_k (Eq. 3 / Eq. 6): an MFMA-bound tiled
// GEMM.  Sec. 2.1 observes that run-time dequantization is what costs weight-only schemes in the
// compute-bound regime, so here the weight expansion is kept to seven VALU instructions per 8
// elements (unpack_w8) and runs beside the matrix pipe.
//
// Workgroup tile BM x BN, WR x WC wavefronts, each owning TM x TN MFMA tiles of 16 x 16.  The
// contraction axis is walked in chunks of 64: per chunk lane q of a wavefront owns block q of the
// four MXINT blocks, for every operand, so block scales never cross lanes.
//   activations (bf16, exact dequantized X_q, then T_hi | T_lo):  global -> LDS (XOR-swizzled
//       16-byte cells, two stages) -> ds_read_b128 operands shared by the wavefronts of a row;
//   weights: each wavefront loads the packed MXINT4 records of its own columns straight into
//       registers (fully coalesced 16-byte loads) and expands them there;
//   the rank-kp correction is ceil(2 kp / 64) more chunks whose weight operand comes from B_k.
// MFMA operands are swapped (weights as the "A" matrix) so a lane ends up with four consecutive
// output columns of one token and stores them as one 16-byte write.
#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

struct TiledArgs {
    const uint8_t* Wt; const uint8_t* Bt;
    const uint16_t* Xh; int64_t ldxh;
    float* Y; int64_t ldy;
    int64_t M, N, KT, N16;
    int kp16;
    int grid_m, grid_n;
    int group_m;
};

template <int TM, int TN, int WR, int WC>
__global__ __launch_bounds__(64 * WR * WC) void tiled_kernel(TiledArgs a) {
    constexpr int BM = 16 * TM * WR;
    constexpr int NT = 64 * WR * WC;
    constexpr int CELLS = BM * 8;                  // 16-byte cells per stage (64 bf16 = 8 cells per row)
    constexpr int LPT = CELLS / NT;                // cells each thread moves per chunk
    static_assert(CELLS % NT == 0, "loader must divide evenly");
    __shared__ __attribute__((aligned(16))) uint8_t lds[2][BM * 128];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave / WC, wc = wave % WC;
    const int t = lane & 15, q = lane >> 4;

    // ---- workgroup -> tile: consecutive ids land on one XCD, tiles are walked in bands ------
    int tile_m, tile_n;
    {
        const int nwg = a.grid_m * a.grid_n;
        const int pid = blockIdx.x;
        const int xcd = pid & 7, local = pid >> 3;
        const int per = nwg >> 3, rem = nwg & 7;
        const int lin = (xcd < rem) ? xcd * (per + 1) + local : rem * (per + 1) + (xcd - rem) * per + local;
        const int width = a.group_m * a.grid_n;
        const int grp = lin / width;
        const int first_m = grp * a.group_m;
        const int gsize = (a.grid_m - first_m < a.group_m) ? a.grid_m - first_m : a.group_m;
        tile_m = first_m + (lin % width) % gsize;
        tile_n = (lin % width) / gsize;
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    const int64_t g0 = ((int64_t)tile_n * WC + wc) * TN;       // first column group of this wavefront

    // ---- activation loader: thread -> cells ------------------------------------------------
    const uint16_t* ld_src[LPT];
    int ld_dst[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int cell = tid + j * NT;
        const int row = cell >> 3, c16 = cell & 7;
        int64_t grow = m0 + row;
        if (grow >= a.M) grow = a.M - 1;                       // duplicate a valid row; never stored
        ld_src[j] = a.Xh + grow * a.ldxh + 8 * c16;
        ld_dst[j] = row * 128 + ((c16 ^ ((row >> 1) & 7)) << 4);
    }
    // ---- operand reader: this lane's cells for its TM row tiles ------------------------------
    int rd_off[TM][2];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int row = (wr * TM + tm) * 16 + t;
#pragma unroll
        for (int h = 0; h < 2; ++h) rd_off[tm][h] = row * 128 + (((2 * q + h) ^ ((row >> 1) & 7)) << 4);
    }
    const uint8_t* wbase[TN];
    int64_t grp[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        grp[tn] = g0 + tn;
        if (grp[tn] >= a.N16) grp[tn] = a.N16 - 1;             // clamp; the store is masked
        wbase[tn] = a.Wt + grp[tn] * a.KT * kWRecordBytes + lane * 16;
    }

    f32x4 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int64_t main_chunks = a.KT * 4;
    const int nb2 = 2 * a.kp16;
    const int tail_chunks = (nb2 + 3) / 4;
    const int64_t chunks = main_chunks + tail_chunks;

    u32x4 st[LPT];             // staging registers of the activation loader
    // prologue: chunk 0 into stage 0; first half tile of weights
#pragma unroll
    for (int j = 0; j < LPT; ++j) st[j] = *reinterpret_cast<const u32x4*>(ld_src[j]);
#pragma unroll
    for (int j = 0; j < LPT; ++j) *reinterpret_cast<u32x4*>(&lds[0][ld_dst[j]]) = st[j];
    u32x4 wcur[TN], wnext[TN];   // packed codes: current / next half tile (two chunks each)
    uint32_t wexp[TN], enext[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        wcur[tn] = *reinterpret_cast<const u32x4*>(wbase[tn]);
        wexp[tn] = *reinterpret_cast<const uint32_t*>(wbase[tn] + 2048 - lane * 12);
        wnext[tn] = wcur[tn];
        enext[tn] = wexp[tn];
    }
    __syncthreads();

    // ---- main product ---------------------------------------------------------------------------
    for (int64_t tile = 0; tile < a.KT; ++tile) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int64_t ch = tile * 4 + p;
            const int stage = p & 1;
            if (ch + 1 < chunks) {
#pragma unroll
                for (int j = 0; j < LPT; ++j)
                    st[j] = *reinterpret_cast<const u32x4*>(ld_src[j] + (ch + 1) * 64);
            }
            if (p == 0) {                                   // second half of this tile
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    wnext[tn] = *reinterpret_cast<const u32x4*>(wbase[tn] + tile * kWRecordBytes + 1024);
            }
            if (p == 2 && tile + 1 < a.KT) {                // first half of the next tile
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const uint8_t* rec = wbase[tn] + (tile + 1) * kWRecordBytes;
                    wnext[tn] = *reinterpret_cast<const u32x4*>(rec);
                    enext[tn] = *reinterpret_cast<const uint32_t*>(rec + 2048 - lane * 12);
                }
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                Frag xa[TM];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    xa[tm].u = *reinterpret_cast<const u32x4*>(&lds[stage][rd_off[tm][h]]);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const float sc = w_scale((wexp[tn] >> (8 * p)) & 0xFFu);
                    const bf16x8 wv = unpack_w8(wcur[tn][2 * (p & 1) + h], sc);
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) acc[tm][tn] = mfma16(wv, xa[tm].v, acc[tm][tn]);
                }
            }
            if (p & 1) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) wcur[tn] = wnext[tn];
                if (p == 3) {
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) wexp[tn] = enext[tn];
                }
            }
            if (ch + 1 < chunks) {
#pragma unroll
                for (int j = 0; j < LPT; ++j)
                    *reinterpret_cast<u32x4*>(&lds[stage ^ 1][ld_dst[j]]) = st[j];
            }
            __syncthreads();
        }
    }

    // ---- rank-kp correction: T_hi | T_lo against B_k -------------------------------------------
    for (int c = 0; c < tail_chunks; ++c) {
        const int64_t ch = main_chunks + c;
        const int stage = c & 1;
        if (ch + 1 < chunks) {
#pragma unroll
            for (int j = 0; j < LPT; ++j)
                st[j] = *reinterpret_cast<const u32x4*>(ld_src[j] + (ch + 1) * 64);
        }
        const int jb = 4 * c + q;                            // block of 16 ranks: T_hi blocks, then T_lo
        const bool live = jb < nb2;
        const int rb = live ? (jb < a.kp16 ? jb : jb - a.kp16) : 0;
        Frag bf[TN][2];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const uint8_t* rec = a.Bt + (grp[tn] * a.kp16 + rb) * kBRecordBytes;
            u32x4 cw = u32x4{0, 0, 0, 0};
            uint32_t eb = 0;
            if (live) {
                cw = *reinterpret_cast<const u32x4*>(rec + t * 16);
                eb = rec[256 + t];
            }
            const float sc = h_scale(eb);
            int8x16_to_frags(cw, sc, bf[tn][0], bf[tn][1]);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            Frag xa[TM];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                xa[tm].u = *reinterpret_cast<const u32x4*>(&lds[stage][rd_off[tm][h]]);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) acc[tm][tn] = mfma16(bf[tn][h].v, xa[tm].v, acc[tm][tn]);
        }
        if (ch + 1 < chunks) {
#pragma unroll
            for (int j = 0; j < LPT; ++j)
                *reinterpret_cast<u32x4*>(&lds[stage ^ 1][ld_dst[j]]) = st[j];
        }
        __syncthreads();
    }

    // ---- store: lane (t, q) holds columns 4q..4q+3 of token t for every MFMA tile ---------------
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t row = m0 + (wr * TM + tm) * 16 + t;
        if (row >= a.M) continue;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int64_t cg = g0 + tn;
            if (cg >= a.N16) continue;
            const int64_t n = cg * 16 + 4 * q;
            float* dst = a.Y + row * a.ldy + n;
            if (n + 3 < a.N) {
                *reinterpret_cast<f32x4*>(dst) = acc[tm][tn];
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < a.N) dst[j] = acc[tm][tn][j];
            }
        }
    }
}

template <int TM, int TN, int WR, int WC>
static hipError_t launch_tiled_t(TiledArgs a, int64_t M, hipStream_t s) {
    constexpr int BM = 16 * TM * WR, BN = 16 * TN * WC;
    a.grid_m = (int)((M + BM - 1) / BM);
    a.grid_n = (int)((a.N + BN - 1) / BN);
    a.group_m = 8;
    dim3 grid((unsigned)(a.grid_m * a.grid_n)), block(64 * WR * WC);
    hipLaunchKernelGGL((tiled_kernel<TM, TN, WR, WC>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_tiled(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy,
                        int variant, hipStream_t s) {
    if (M == 0) return hipSuccess;
    TiledArgs a;
    a.Wt = L.Wt; a.Bt = L.Bt; a.Xh = ws.Xh; a.ldxh = ws.ldxh; a.Y = Y; a.ldy = ldy;
    a.M = M; a.N = L.N; a.KT = L.KT; a.N16 = L.N16; a.kp16 = L.kp16;
    a.grid_m = a.grid_n = 0; a.group_m = 8;
    if (variant == 0) {
        // 256x256 tiles unless they leave compute units idle or the last round mostly empty
        const int64_t t256 = ((M + 255) / 256) * ((L.N + 255) / 256);
        const int64_t rounds = (t256 + 255) / 256;
        const double eff = (double)t256 / (double)(rounds * 256);
        variant = (eff >= 0.85) ? 1 : 2;
    }
    switch (variant) {
        case 1: return launch_tiled_t<8, 8, 2, 2>(a, M, s);      // 256 x 256
        case 2: return launch_tiled_t<8, 4, 2, 2>(a, M, s);      // 256 x 128
        case 3: return launch_tiled_t<4, 8, 2, 2>(a, M, s);      // 128 x 256
        case 4: return launch_tiled_t<4, 4, 2, 2>(a, M, s);      // 128 x 128
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lqer
