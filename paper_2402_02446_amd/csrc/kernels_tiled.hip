// Stage 2, large-M ("prefill") form of Y = X_q W_q + T B_k (Eq. 3 / Eq. 6): an MFMA-bound tiled
// GEMM.  Sec. 2.1 observes that run-time dequantization is what costs weight-only schemes in the
// compute-bound regime, so here the weight expansion is kept to seven VALU instructions per 8
// elements (unpack_w8) and runs beside the matrix pipe.
//
// Workgroup tile BM x BN, WR x WC wavefronts, each owning TM x TN tiles of the 32x32x16 bf16
// MFMA (the shape one wavefront per SIMD can keep close to the matrix pipe's peak).  The
// contraction axis is walked in chunks of 64 = four MFMA steps; lane half hh owns blocks 2hh and
// 2hh+1 of a chunk for every operand, so block scales never cross lanes.
//   activations (bf16, exact dequantized X_q, then T_hi | T_lo): global -> LDS with the direct
//       (no-register) 16-byte loads, into a ring of stages of XOR-swizzled 16-byte cells, then
//       ds_read_b128 operands shared by the wavefronts of a row;
//   weights: each wavefront loads the packed MXINT4 records of its own columns straight into
//       registers (fully coalesced 16-byte loads), one chunk ahead, and expands them there;
//   the rank-kp correction is ceil(2 kp / 64) more chunks whose weight operand comes from B_k.
// MFMA operands are swapped (weights first) so a lane ends up with runs of four consecutive
// output columns of one token and stores each as one 16-byte write.
#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

struct TiledArgs {
    const uint8_t* Wt; const uint8_t* Bt;
    const uint16_t* Xh; int64_t ldxh;
    float* Y; int64_t ldy;
    int64_t M, N, KT, N32;
    int kp16;
    int grid_m, grid_n;
    int group_m;
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

template <int TM, int TN, int WR, int WC, int NS>
__global__ __launch_bounds__(64 * WR * WC) void tiled_kernel(TiledArgs a) {
    constexpr int BM = 32 * TM * WR;
    constexpr int NW = WR * WC;
    constexpr int STAGE = BM * 128;                // bytes: BM rows x 64 bf16
    constexpr int LPT = BM / (8 * NW);             // direct loads per lane per chunk (a load fills 8 rows)
    static_assert(BM % (8 * NW) == 0, "loader must divide evenly");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave / WC, wc = wave % WC;
    const int t = lane & 31, hh = lane >> 5;

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

    // ---- activation loader ---------------------------------------------------------------------
    // Load j of this wavefront fills LDS rows (j*NW + wave)*8 .. +7 of a stage: lane i lands in
    // row i/8, physical cell i%8, so it fetches the logical cell (i%8) ^ ((row>>1)&7) of that row.
    const uint16_t* ld_src[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = (j * NW + wave) * 8 + (lane >> 3);
        const int cell = (lane & 7) ^ ((row >> 1) & 7);
        int64_t grow = m0 + row;
        if (grow >= a.M) grow = a.M - 1;                       // repeat a valid token; never stored
        ld_src[j] = a.Xh + grow * a.ldxh + 8 * cell;
    }
    // ---- operand reader: in step s this lane reads logical cell 4 hh + s of its TM rows -----------
    int rd_off[TM][4];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int row = (wr * TM + tm) * 32 + t;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) rd_off[tm][s4] = row * 128 + (((4 * hh + s4) ^ ((row >> 1) & 7)) << 4);
    }
    const uint8_t* wbase[TN];
    int64_t grp[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        grp[tn] = g0 + tn;
        if (grp[tn] >= a.N32) grp[tn] = a.N32 - 1;             // clamp; the store is masked
        wbase[tn] = a.Wt + grp[tn] * a.KT * kWRecordBytes + lane * 16;
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    const int64_t main_chunks = a.KT * 4;
    const int nb2 = 2 * a.kp16;
    const int tail_chunks = (nb2 + 3) / 4;
    const int64_t chunks = main_chunks + tail_chunks;
    const int uwave = __builtin_amdgcn_readfirstlane(wave);

    // The ring has NS = 4 stages and a K tile has 4 chunks, so chunk ch always uses stage ch % 4.
    auto issue_stage = [&](int64_t ch, int stage) {
#pragma unroll
        for (int j = 0; j < LPT; ++j)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(ld_src[j] + ch * 64),
                                             (lds_ptr_t)(lds + stage * STAGE + (j * NW + uwave) * 1024), 16, 0, 0);
    };
    // Outstanding-load budget when waiting for chunk ch's stage: everything issued after it, i.e.
    // the weight loads and stage loads of the NS-2 iterations in between (weights are issued
    // before the stage loads of the same iteration).
    constexpr int kSteadyVm = (NS - 2) * (LPT + TN);
    static_assert(NS == 4, "stage indices below assume a ring of four");
    static_assert(kSteadyVm < 64, "vmcnt field is 6 bits");
    auto wait_stage = [&](bool steady) {
        if (steady) __builtin_amdgcn_s_waitcnt(0x0F70 | (kSteadyVm & 15) | ((kSteadyVm >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
    };

    // prologue: stages for chunks 0 .. NS-2; first chunk of weights
    u32x4 wcur[TN], wnext[TN];   // packed codes of the current / next chunk
    u32x2 wexp[TN];              // exponent bytes of the current tile
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        wcur[tn] = *reinterpret_cast<const u32x4*>(wbase[tn]);
        wexp[tn] = *reinterpret_cast<const u32x2*>(wbase[tn] + kWExpOffset - lane * 8);
        wnext[tn] = wcur[tn];
    }
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < chunks) issue_stage(p, p);

    // ---- main product -----------------------------------------------------------------------------
    for (int64_t tile = 0; tile < a.KT; ++tile) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t ch = tile * 4 + c;
            // chunk ch's stage has landed (this wavefront's share) ...
            wait_stage(ch >= NS - 2 && ch + NS - 2 < chunks && ch < main_chunks);
            __syncthreads();                                   // ... and everybody else's; stage (ch-1)%4 is free
            if (ch + 1 < main_chunks) {
                const int64_t nt = (ch + 1) >> 2;
                constexpr int kNextC[4] = {1, 2, 3, 0};
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    wnext[tn] = *reinterpret_cast<const u32x4*>(wbase[tn] + nt * kWRecordBytes + kNextC[c] * 1024);
            }
            if (ch + NS - 1 < chunks) issue_stage(ch + NS - 1, (c + NS - 1) & 3);
            const uint8_t* stage = lds + c * STAGE;
            float sc[TN][2];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const uint32_t ew = wexp[tn][c >> 1] >> (16 * (c & 1));
                sc[tn][0] = w_scale(ew & 0xFFu);
                sc[tn][1] = w_scale((ew >> 8) & 0xFFu);
            }
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                Frag xa[TM];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    xa[tm].u = *reinterpret_cast<const u32x4*>(stage + rd_off[tm][s4]);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const bf16x8 wv = unpack_w8(wcur[tn][s4], sc[tn][s4 >> 1]);
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) acc[tm][tn] = mfma32(wv, xa[tm].v, acc[tm][tn]);
                }
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) wcur[tn] = wnext[tn];
            if (c == 3 && tile + 1 < a.KT) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    wexp[tn] = *reinterpret_cast<const u32x2*>(wbase[tn] + (tile + 1) * kWRecordBytes + kWExpOffset - lane * 8);
            }
        }
    }

    // ---- rank-kp correction: [T_hi | T_lo | 0] against B_k ---------------------------------------
    // lane half hh owns rank blocks jb = 4 cc + 2 hh + {0, 1} of tail chunk cc
    for (int cc = 0; cc < tail_chunks; ++cc) {
        const int64_t ch = main_chunks + cc;
        wait_stage(false);
        __syncthreads();
        if (ch + NS - 1 < chunks) issue_stage(ch + NS - 1, (cc + NS - 1) & 3);
        const uint8_t* stage = lds + (cc & 3) * STAGE;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int jb = 4 * cc + 2 * hh + j;
            const bool live = jb < nb2;
            const int rb = live ? (jb < a.kp16 ? jb : jb - a.kp16) : 0;
            Frag bf[TN][2];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                u32x4 cw = u32x4{0, 0, 0, 0};
                uint32_t eb = 0;
                if (live) {
                    const uint8_t* rec = a.Bt + (grp[tn] * a.kp16 + rb) * kBRecordBytes;
                    cw = *reinterpret_cast<const u32x4*>(rec + t * 16);
                    eb = rec[512 + t];
                }
                int8x16_to_frags(cw, h_scale(eb), bf[tn][0], bf[tn][1]);
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                Frag xa[TM];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    xa[tm].u = *reinterpret_cast<const u32x4*>(stage + rd_off[tm][2 * j + h]);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) acc[tm][tn] = mfma32(bf[tn][h].v, xa[tm].v, acc[tm][tn]);
            }
        }
    }

    // ---- store: lane (t, hh) holds columns 8 r4 + 4 hh .. + 3 of token t for every MFMA tile ------
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t row = m0 + (wr * TM + tm) * 32 + t;
        if (row >= a.M) continue;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int64_t cg = g0 + tn;
            if (cg >= a.N32) continue;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int64_t n = cg * 32 + 8 * r4 + 4 * hh;
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
}

template <int TM, int TN, int WR, int WC, int NS>
static hipError_t launch_tiled_t(TiledArgs a, int64_t M, hipStream_t s) {
    constexpr int BM = 32 * TM * WR, BN = 32 * TN * WC;
    constexpr int LDS_BYTES = NS * BM * 128;
    a.grid_m = (int)((M + BM - 1) / BM);
    a.grid_n = (int)((a.N + BN - 1) / BN);
    a.group_m = 8;
    auto kern = tiled_kernel<TM, TN, WR, WC, NS>;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)(a.grid_m * a.grid_n)), block(64 * WR * WC);
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, s, a);
    return hipGetLastError();
}

hipError_t launch_tiled(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy,
                        int variant, hipStream_t s) {
    if (M == 0) return hipSuccess;
    TiledArgs a;
    a.Wt = L.Wt; a.Bt = L.Bt; a.Xh = ws.Xh; a.ldxh = ws.ldxh; a.Y = Y; a.ldy = ldy;
    a.M = M; a.N = L.N; a.KT = L.KT; a.N32 = L.N32; a.kp16 = L.kp16;
    a.grid_m = a.grid_n = 0; a.group_m = 8;
    if (variant == 0) {
        // 256x256 tiles unless they leave compute units idle or the last round mostly empty
        const int64_t t256 = ((M + 255) / 256) * ((L.N + 255) / 256);
        const int64_t rounds = (t256 + 255) / 256;
        const double eff = (double)t256 / (double)(rounds * 256);
        variant = (eff >= 0.85) ? 1 : 2;
    }
    switch (variant) {
        case 1: return launch_tiled_t<4, 4, 2, 2, 4>(a, M, s);      // 256 x 256
        case 2: return launch_tiled_t<4, 2, 2, 2, 4>(a, M, s);      // 256 x 128
        case 3: return launch_tiled_t<2, 4, 2, 2, 4>(a, M, s);      // 128 x 256
        case 4: return launch_tiled_t<2, 2, 2, 2, 4>(a, M, s);      // 128 x 128
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lqer
