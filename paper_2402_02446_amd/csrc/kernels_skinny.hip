// Stage 2, small-M ("decode") form of Y = X_q W_q + T B_k (Eq. 3 / Eq. 6): a weight-streaming
// kernel bound by HBM bandwidth.  Sec. 2.1 notes that few-token inference is memory-bound; the
// whole job here is to read 0.5625 B per weight once, as contiguous 1 KiB wavefront loads, and to
// hide everything else under that stream.
//
// A workgroup owns NG groups of 16 output columns and all of K; its four wavefronts take the
// 256-wide K tiles in turn and their partial sums are added through LDS in a fixed order.  Per
// tile and column group a lane holds four whole MXINT4 blocks (two 16-byte loads) and their four
// exponent bytes (one 4-byte load), expands a block to 16 bf16 values code * 2^(e-2) with seven
// VALU instructions per 8 elements (see unpack_w8) and feeds them to the 16x16x32 bf16 MFMA
// against the dequantized activations; all products are exact and accumulation is fp32.  The
// rank-kp correction is 2*kp further "K columns": T_hi and T_lo against B_k's codes.
#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

struct SkinnyArgs {
    const uint8_t* Wt; const uint8_t* Bt;
    const uint16_t* Xh; int64_t ldxh;
    const float* Tpart; int S;
    float* Y; int64_t ldy;
    int64_t M, N, KT, N16;
    int kp, kp16;
};

struct WRec {           // one lane's share of a W record
    u32x4 c[2];
    uint32_t e;
};

__device__ __forceinline__ WRec load_wrec(const uint8_t* rec, int lane) {
    WRec r;
    r.c[0] = *reinterpret_cast<const u32x4*>(rec + lane * 16);
    r.c[1] = *reinterpret_cast<const u32x4*>(rec + 1024 + lane * 16);
    r.e = *reinterpret_cast<const uint32_t*>(rec + 2048 + lane * 4);
    return r;
}

template <int TM, int NG>
__global__ __launch_bounds__(256) void skinny_kernel(SkinnyArgs a) {
    __shared__ float red[4][TM][NG][64][4];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t = lane & 15, q = lane >> 4;

    int64_t grp[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        grp[g] = (int64_t)blockIdx.x * NG + g;
        if (grp[g] >= a.N16) grp[g] = a.N16 - 1;          // clamp; the store is masked
    }
    const uint16_t* xrow[TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        int64_t row = 16 * tm + t;
        if (row >= a.M) row = a.M - 1;                    // duplicate a valid row; never stored
        xrow[tm] = a.Xh + row * a.ldxh;
    }

    f32x4 acc[TM][NG];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[tm][g] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- main product: stream this wavefront's K tiles ------------------------------------
    int64_t tile = wave;
    WRec cur[NG];
    if (tile < a.KT) {
#pragma unroll
        for (int g = 0; g < NG; ++g) cur[g] = load_wrec(a.Wt + (grp[g] * a.KT + tile) * kWRecordBytes, lane);
    }
    for (; tile < a.KT; tile += 4) {
        WRec nxt[NG];
        const int64_t ntile = (tile + 4 < a.KT) ? tile + 4 : tile;     // re-read on the last round
#pragma unroll
        for (int g = 0; g < NG; ++g) nxt[g] = load_wrec(a.Wt + (grp[g] * a.KT + ntile) * kWRecordBytes, lane);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            Frag xa[TM][2];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const uint16_t* src = xrow[tm] + tile * kTileK + 64 * p + 16 * q;
                xa[tm][0].u = *reinterpret_cast<const u32x4*>(src);
                xa[tm][1].u = *reinterpret_cast<const u32x4*>(src + 8);
            }
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const float sc = w_scale((cur[g].e >> (8 * p)) & 0xFFu);
                const bf16x8 w0 = unpack_w8(cur[g].c[p >> 1][2 * (p & 1)], sc);
                const bf16x8 w1 = unpack_w8(cur[g].c[p >> 1][2 * (p & 1) + 1], sc);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    acc[tm][g] = mfma16(w0, xa[tm][0].v, acc[tm][g]);
                    acc[tm][g] = mfma16(w1, xa[tm][1].v, acc[tm][g]);
                }
            }
        }
#pragma unroll
        for (int g = 0; g < NG; ++g) cur[g] = nxt[g];
    }

    // ---- rank-kp correction: blocks of 16 ranks, T_hi then T_lo, spread over the wavefronts -
    // Block jb in [0, 2*kp16): jb < kp16 is T_hi for ranks 16*jb.., otherwise T_lo.  Lane q takes
    // block q + 4*ch of chunk ch, exactly as in the main loop.
    const int nb2 = 2 * a.kp16;
    const int nchunks = (nb2 + 3) / 4;
    for (int ch = (wave - (int)(a.KT & 3)) & 3; ch < nchunks; ch += 4) {
        // chunk ch is taken by wavefront (KT + ch) mod 4: continues the round-robin of the tiles
        const int jb = 4 * ch + q;
        const bool live = jb < nb2;
        const int rb = live ? (jb < a.kp16 ? jb : jb - a.kp16) : 0;
        const bool is_lo = jb >= a.kp16;
        Frag ta[TM][2];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            if (a.S == 1) {
                const uint16_t* src = xrow[tm] + a.KT * kTileK + 16 * jb;
                if (live) {
                    ta[tm][0].u = *reinterpret_cast<const u32x4*>(src);
                    ta[tm][1].u = *reinterpret_cast<const u32x4*>(src + 8);
                } else {
                    ta[tm][0].u = u32x4{0, 0, 0, 0};
                    ta[tm][1].u = u32x4{0, 0, 0, 0};
                }
            } else {
                int64_t row = 16 * tm + t;
                if (row >= a.M) row = a.M - 1;
                float tv[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) tv[i] = 0.f;
                if (live) {
                    for (int s = 0; s < a.S; ++s) {
                        const float* src = a.Tpart + ((int64_t)s * a.M + row) * a.kp + 16 * rb;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const f32x4 v = *reinterpret_cast<const f32x4*>(src + 4 * i);
                            tv[4 * i] += v[0]; tv[4 * i + 1] += v[1]; tv[4 * i + 2] += v[2]; tv[4 * i + 3] += v[3];
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t hb = f32_bits(tv[i]) & 0xFFFF0000u;
                    const float part = is_lo ? (tv[i] - f32_from_bits(hb)) : f32_from_bits(hb);
                    tv[i] = f32_from_bits(f32_bits(part) & 0xFFFF0000u);
                }
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        ta[tm][h].u[i] = pack_bf16_exact(tv[8 * h + 2 * i], tv[8 * h + 2 * i + 1]);
            }
        }
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const uint8_t* rec = a.Bt + (grp[g] * a.kp16 + rb) * kBRecordBytes;
            u32x4 cw = u32x4{0, 0, 0, 0};
            uint32_t eb = 0;
            if (live) {
                cw = *reinterpret_cast<const u32x4*>(rec + t * 16);
                eb = rec[256 + t];
            }
            const float sc = h_scale(eb);
            Frag bf[2];
            int8x16_to_frags(cw, sc, bf[0], bf[1]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                acc[tm][g] = mfma16(bf[0].v, ta[tm][0].v, acc[tm][g]);
                acc[tm][g] = mfma16(bf[1].v, ta[tm][1].v, acc[tm][g]);
            }
        }
    }

    // ---- add the four wavefronts in a fixed order and store ----------------------------------
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int g = 0; g < NG; ++g)
            *reinterpret_cast<f32x4*>(&red[wave][tm][g][lane][0]) = acc[tm][g];
    __syncthreads();
    for (int item = threadIdx.x; item < TM * NG * 64; item += 256) {
        const int l = item & 63;
        const int g = (item >> 6) % NG;
        const int tm = (item >> 6) / NG;
        f32x4 s = *reinterpret_cast<const f32x4*>(&red[0][tm][g][l][0]);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const f32x4 o = *reinterpret_cast<const f32x4*>(&red[w][tm][g][l][0]);
            s[0] += o[0]; s[1] += o[1]; s[2] += o[2]; s[3] += o[3];
        }
        const int64_t row = 16 * tm + (l & 15);
        const int64_t cg = (int64_t)blockIdx.x * NG + g;
        const int64_t n = cg * 16 + 4 * (l >> 4);
        if (row < a.M && cg < a.N16) {
            float* dst = a.Y + row * a.ldy + n;
            if (n + 3 < a.N) {
                *reinterpret_cast<f32x4*>(dst) = s;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < a.N) dst[j] = s[j];
            }
        }
    }
}

int skinny_max_rows() { return 64; }

template <int TM, int NG>
static hipError_t launch_skinny_t(const SkinnyArgs& a, hipStream_t s) {
    dim3 grid((unsigned)((a.N16 + NG - 1) / NG)), block(256);
    hipLaunchKernelGGL((skinny_kernel<TM, NG>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_skinny(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy,
                         int variant, hipStream_t s) {
    if (M == 0) return hipSuccess;
    SkinnyArgs a;
    a.Wt = L.Wt; a.Bt = L.Bt; a.Xh = ws.Xh; a.ldxh = ws.ldxh; a.Tpart = ws.Tpart; a.S = ws.S;
    a.Y = Y; a.ldy = ldy; a.M = M; a.N = L.N; a.KT = L.KT; a.N16 = L.N16; a.kp = L.kp; a.kp16 = L.kp16;
    const int tm = (int)((M + 15) / 16);
    // variant: 1 -> NG = 1, 2 -> NG = 2, 4 -> NG = 4; automatic keeps at least ~2 workgroups per
    // compute unit so that enough loads are in flight.
    int ng = variant;
    if (ng != 1 && ng != 2 && ng != 4) ng = (L.N16 >= 4 * 512) ? 4 : (L.N16 >= 2 * 512 ? 2 : 1);
    if (tm >= 3 && ng == 4) ng = 2;            // keep the accumulator and LDS footprint bounded
#define LQER_SK(TM_, NG_) return launch_skinny_t<TM_, NG_>(a, s)
    switch (tm) {
        case 1: if (ng == 1) LQER_SK(1, 1); if (ng == 2) LQER_SK(1, 2); LQER_SK(1, 4);
        case 2: if (ng == 1) LQER_SK(2, 1); if (ng == 2) LQER_SK(2, 2); LQER_SK(2, 4);
        case 3: case 4: if (ng == 1) LQER_SK(4, 1); LQER_SK(4, 2);
        default: return hipErrorInvalidValue;
    }
#undef LQER_SK
}

}  // namespace lqer
