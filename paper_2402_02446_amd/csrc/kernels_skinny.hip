// Stage 2, small-M ("decode") form of Y = X_q W_q + T B_k (Eq. 3 / Eq. 6): a weight-streaming
// kernel bound by HBM bandwidth.  Sec. 2.1 notes that few-token inference is memory-bound; the
// whole job here is to read 0.5625 B per weight once, as contiguous 1 KiB wavefront loads, and to
// hide everything else under that stream.
//
// A workgroup owns NG groups of 32 output columns and all of K; its NW wavefronts take the
// 256-wide K tiles in turn and their partial sums are added through LDS in a fixed tree order.
// Per tile and column group a lane reads 64 B of packed codes (eight whole MXINT4 blocks) and
// their eight exponent bytes, expands 8 codes to bf16 values code * 2^(e-2) with seven VALU
// instructions (unpack_w8) and feeds them to the 32x32x16 bf16 MFMA against the dequantized
// activations (tokens beyond M repeat the last one and are never stored); all products are exact
// and accumulation is fp32.  The rank-kp correction is 2*kp further "K columns": T_hi and T_lo
// against B_k's codes.  Weight records are fetched one tile ahead and activations one 64-wide
// chunk ahead, so HBM and L2 latency overlap the arithmetic.
#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

struct SkinnyArgs {
    const uint8_t* Wt; const uint8_t* Bt;
    const uint16_t* Xh; int64_t ldxh;
    const float* Tpart; int S;
    float* Y; int64_t ldy;
    int64_t M, N, KT, N32;
    int kp, kp16;
};

struct WRec {           // one lane's share of a W record
    u32x4 c[4];
    u32x2 e;
};

__device__ __forceinline__ WRec load_wrec(const uint8_t* rec, int lane) {
    WRec r;
#pragma unroll
    for (int c = 0; c < 4; ++c) r.c[c] = *reinterpret_cast<const u32x4*>(rec + c * 1024 + lane * 16);
    r.e = *reinterpret_cast<const u32x2*>(rec + kWExpOffset + lane * 8);
    return r;
}

struct XChunk {         // one lane's activations for a 64-wide chunk: 4 MFMA steps x 8 bf16
    u32x4 s[4];
};

__device__ __forceinline__ XChunk load_xchunk(const uint16_t* p) {
    XChunk x;
#pragma unroll
    for (int s = 0; s < 4; ++s) x.s[s] = *reinterpret_cast<const u32x4*>(p + 8 * s);
    return x;
}

template <int TM, int NG, int NW>
__global__ __launch_bounds__(64 * NW) void skinny_kernel(SkinnyArgs a) {
    __shared__ float red[NW / 2][TM][NG][64][16];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t = lane & 31, hh = lane >> 5;

    int64_t grp[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        grp[g] = (int64_t)blockIdx.x * NG + g;
        if (grp[g] >= a.N32) grp[g] = a.N32 - 1;          // clamp; the store is masked
    }
    const uint16_t* xrow[TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        int64_t row = 32 * tm + t;
        if (row >= a.M) row = a.M - 1;                    // repeat a valid token; never stored
        xrow[tm] = a.Xh + row * a.ldxh + 32 * hh;
    }

    f32x16 acc[TM][NG];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][g][r] = 0.f;

    // ---- main product: stream this wavefront's K tiles ------------------------------------
    int64_t tile = wave;
    if (tile < a.KT) {
        WRec cur[NG];
        XChunk xc[TM];
#pragma unroll
        for (int g = 0; g < NG; ++g) cur[g] = load_wrec(a.Wt + (grp[g] * a.KT + tile) * kWRecordBytes, lane);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) xc[tm] = load_xchunk(xrow[tm] + tile * kTileK);
        for (; tile < a.KT; tile += NW) {
            const bool more = tile + NW < a.KT;
            const int64_t ntile = more ? tile + NW : tile;             // re-read on the last round
            WRec nxt[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g)
                nxt[g] = load_wrec(a.Wt + (grp[g] * a.KT + ntile) * kWRecordBytes, lane);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                XChunk xn[TM];
                const int64_t noff = (c < 3) ? tile * kTileK + 64 * (c + 1) : ntile * kTileK;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) xn[tm] = load_xchunk(xrow[tm] + noff);
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const uint32_t ew = cur[g].e[c >> 1] >> (16 * (c & 1));
                    const float sc0 = w_scale(ew & 0xFFu), sc1 = w_scale((ew >> 8) & 0xFFu);
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const bf16x8 wv = unpack_w8(cur[g].c[c][s], s < 2 ? sc0 : sc1);
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) {
                            Frag xf;
                            xf.u = xc[tm].s[s];
                            acc[tm][g] = mfma32(wv, xf.v, acc[tm][g]);
                        }
                    }
                }
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) xc[tm] = xn[tm];
            }
#pragma unroll
            for (int g = 0; g < NG; ++g) cur[g] = nxt[g];
        }
    }

    // ---- rank-kp correction: 64-wide chunks of [T_hi | T_lo], spread over the wavefronts ----------
    // Lane half hh owns rank blocks jb = 4 ch + 2 hh + {0, 1} of chunk ch, as in the main loop;
    // jb < kp16 is T_hi for ranks 16 jb.., otherwise T_lo for ranks 16 (jb - kp16)...
    const int nb2 = 2 * a.kp16;
    const int nchunks = (nb2 + 3) / 4;
    for (int ch = (wave + NW - (int)(a.KT % NW)) % NW; ch < nchunks; ch += NW) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int jb = 4 * ch + 2 * hh + j;
            const bool live = jb < nb2;
            const bool is_lo = jb >= a.kp16;
            const int rb = live ? (is_lo ? jb - a.kp16 : jb) : 0;
            Frag ta[TM][2];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                if (!live) {
                    ta[tm][0].u = u32x4{0, 0, 0, 0};
                    ta[tm][1].u = u32x4{0, 0, 0, 0};
                } else if (a.S == 1) {
                    const uint16_t* src = xrow[tm] - 32 * hh + a.KT * kTileK + 16 * jb;
                    ta[tm][0].u = *reinterpret_cast<const u32x4*>(src);
                    ta[tm][1].u = *reinterpret_cast<const u32x4*>(src + 8);
                } else {
                    int64_t row = 32 * tm + t;
                    if (row >= a.M) row = a.M - 1;
                    float tv[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) tv[i] = 0.f;
                    for (int s = 0; s < a.S; ++s) {                     // fixed order over the K slices
                        const float* src = a.Tpart + ((int64_t)s * a.M + row) * a.kp + 16 * rb;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const f32x4 v = *reinterpret_cast<const f32x4*>(src + 4 * i);
                            tv[4 * i] += v[0]; tv[4 * i + 1] += v[1]; tv[4 * i + 2] += v[2]; tv[4 * i + 3] += v[3];
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
                u32x4 cw = u32x4{0, 0, 0, 0};
                uint32_t eb = 0;
                if (live) {
                    const uint8_t* rec = a.Bt + (grp[g] * a.kp16 + rb) * kBRecordBytes;
                    cw = *reinterpret_cast<const u32x4*>(rec + t * 16);
                    eb = rec[512 + t];
                }
                Frag bf[2];
                int8x16_to_frags(cw, h_scale(eb), bf[0], bf[1]);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    acc[tm][g] = mfma32(bf[0].v, ta[tm][0].v, acc[tm][g]);
                    acc[tm][g] = mfma32(bf[1].v, ta[tm][1].v, acc[tm][g]);
                }
            }
        }
    }

    // ---- add the wavefronts in a fixed tree order; wavefront 0 stores ------------------------------
#pragma unroll
    for (int off = NW / 2; off >= 1; off >>= 1) {
        if (wave >= off && wave < 2 * off) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int g = 0; g < NG; ++g)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        *reinterpret_cast<f32x4*>(&red[wave - off][tm][g][lane][4 * r4]) =
                            f32x4{acc[tm][g][4 * r4], acc[tm][g][4 * r4 + 1], acc[tm][g][4 * r4 + 2], acc[tm][g][4 * r4 + 3]};
        }
        __syncthreads();
        if (wave < off) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int g = 0; g < NG; ++g)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const f32x4 o = *reinterpret_cast<const f32x4*>(&red[wave][tm][g][lane][4 * r4]);
                        acc[tm][g][4 * r4] += o[0]; acc[tm][g][4 * r4 + 1] += o[1];
                        acc[tm][g][4 * r4 + 2] += o[2]; acc[tm][g][4 * r4 + 3] += o[3];
                    }
        }
        __syncthreads();
    }
    if (wave == 0) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int64_t row = 32 * tm + t;
            if (row >= a.M) continue;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int64_t cg = (int64_t)blockIdx.x * NG + g;
                if (cg >= a.N32) continue;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int64_t n = cg * 32 + 8 * r4 + 4 * hh;       // this lane's 4 consecutive columns
                    float* dst = a.Y + row * a.ldy + n;
                    const f32x4 v = f32x4{acc[tm][g][4 * r4], acc[tm][g][4 * r4 + 1], acc[tm][g][4 * r4 + 2], acc[tm][g][4 * r4 + 3]};
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
}

int skinny_max_rows() { return 64; }

template <int TM, int NG, int NW>
static hipError_t launch_skinny_t(const SkinnyArgs& a, hipStream_t s) {
    dim3 grid((unsigned)((a.N32 + NG - 1) / NG)), block(64 * NW);
    hipLaunchKernelGGL((skinny_kernel<TM, NG, NW>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_skinny(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy,
                         int variant, hipStream_t s) {
    if (M == 0) return hipSuccess;
    SkinnyArgs a;
    a.Wt = L.Wt; a.Bt = L.Bt; a.Xh = ws.Xh; a.ldxh = ws.ldxh; a.Tpart = ws.Tpart; a.S = ws.S;
    a.Y = Y; a.ldy = ldy; a.M = M; a.N = L.N; a.KT = L.KT; a.N32 = L.N32; a.kp = L.kp; a.kp16 = L.kp16;
    const int tm = (M > 32) ? 2 : 1;
    // variant = 10 * NG + log2(NW) - 1 ... kept simple: 1 -> (NG 1, NW 4), 2 -> (1, 8), 3 -> (1, 16), 4 -> (2, 4).
    // Automatic: one column group per workgroup; as many wavefronts as there are K tiles (up to 16)
    // when the layer is too narrow to fill the chip with 4-wavefront workgroups.
    int v = variant;
    if (v < 1 || v > 4) {
        if (L.N32 >= 512) v = 1;
        else if (L.N32 >= 256) v = (L.KT >= 8) ? 2 : 1;
        else v = (L.KT >= 16) ? 3 : (L.KT >= 8 ? 2 : 1);
    }
#define LQER_SK(TM_, NG_, NW_) return launch_skinny_t<TM_, NG_, NW_>(a, s)
    if (tm == 1) {
        switch (v) {
            case 1: LQER_SK(1, 1, 4);
            case 2: LQER_SK(1, 1, 8);
            case 3: LQER_SK(1, 1, 16);
            default: LQER_SK(1, 2, 4);
        }
    } else {
        switch (v) {
            case 1: LQER_SK(2, 1, 4);
            case 2: LQER_SK(2, 1, 8);
            case 3: LQER_SK(2, 1, 16);
            default: LQER_SK(2, 2, 4);
        }
    }
#undef LQER_SK
}

}  // namespace lqer
