// Stage 2, small-M ("decode") form of Y = X_q W_q + T B_k (Eq. 3 / Eq. 6): a weight-streaming
// kernel bound by HBM bandwidth.  Sec. 2.1 notes that few-token inference is memory-bound; the
// whole job here is to read 0.5625 B per weight once, as contiguous 1 KiB wavefront loads, and to
// hide everything else under that stream.
//
// A workgroup is a grid of NWC x NWK wavefronts: wavefront (wc, wk) owns one group of 32 output
// columns and every NWK-th 256-wide K tile, so in each iteration the workgroup works on NWK
// consecutive K tiles.  Their activations (bf16, exact dequantized X_q) are staged once per
// workgroup into LDS and shared by the NWC column groups, which keeps activation traffic at
// 1/NWC-th of what every wavefront fetching its own would cost.  The order of loads matters:
// vector-memory loads retire in order, so a wavefront that waits for a load also waits for every
// load issued before it.  Each iteration therefore issues the (small) activation loads of the
// next iteration first and the weight record of the iteration after next last; when the
// activations are written to LDS at the end of the iteration the weight record stays in flight,
// and three weight records rotate through three named register sets (the loop is unrolled by
// three) so that no register copy ever forces a wait on the newest one.
// Per tile a lane reads 64 B of packed codes (eight whole MXINT4 blocks) and their eight exponent
// bytes, expands 8 codes to bf16 values code * 2^(e-2) with seven VALU instructions (unpack_w8)
// and feeds them to the 32x32x16 bf16 MFMA against the activations (tokens beyond M repeat the
// last one and are never stored); products are exact, accumulation is fp32.  The rank-kp
// correction is 2*kp further "K columns": T_hi and T_lo against B_k's codes.  The NWK partial sums
// of a column group are added through LDS in a fixed tree order.
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

// LR = log2 of the token rows staged (4, 16 or 32).  LDS cell order of a stage is
// [16-byte column of the NWK*256-wide K range][token row], so 16 lanes read 256 contiguous bytes.
template <int NWC, int NWK, int LR>
__global__ __launch_bounds__(64 * NWC * NWK) void skinny_kernel(SkinnyArgs a) {
    constexpr int NW = NWC * NWK;
    constexpr int R = 1 << LR;
    constexpr int XT = NWK * R * 512;                // bytes of one stage: R rows x NWK tiles of bf16
    constexpr int NL = XT / 1024;                    // direct loads (1 KiB each) per stage
    constexpr int XL = (NL + NW - 1) / NW;           // ... per wavefront
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    float* red = reinterpret_cast<float*>(lds);      // reused after the main loop: [NWK/2][NWC][64][16]

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    const int wc = uwave % NWC, wk = uwave / NWC;
    const int t = lane & 31, hh = lane >> 5;

    int64_t grp = (int64_t)blockIdx.x * NWC + wc;
    const bool grp_ok = grp < a.N32;
    if (!grp_ok) grp = a.N32 - 1;                         // clamp; the store is masked
    int64_t trow = t;
    if (trow >= a.M) trow = a.M - 1;                      // repeat a valid token; never stored
    const uint16_t* xrow = a.Xh + trow * a.ldxh + 32 * hh;     // for the correction term (global reads)

    // staging: this wavefront's loads x = 0..XL-1 are cells j = uwave + NW x of 1 KiB of the stage;
    // slot = 64 j + lane -> (16-byte column, row)
    const uint16_t* st_row[XL];
    int st_col[XL];
    int st_dst[XL];
#pragma unroll
    for (int x = 0; x < XL; ++x) {
        const int j = uwave + NW * x;
        const int slot = 64 * (j < NL ? j : 0) + lane;
        int64_t row = slot & (R - 1);
        if (row >= a.M) row = a.M - 1;
        st_row[x] = a.Xh + row * a.ldxh;
        st_col[x] = 8 * (slot >> LR);
        st_dst[x] = (j < NL) ? slot * 16 : -1;
    }
    const int64_t kspan = (int64_t)NWK * kTileK;          // K range of one iteration
    const int64_t NI = (a.KT + NWK - 1) / NWK;            // iterations, the same for every wavefront
    const int64_t kcap = a.KT * kTileK - 8;               // last 16-byte column of a row
    auto fetch_x = [&](int64_t it, u32x4 (&st)[XL]) {
        const int64_t k0 = (it < NI ? it : NI - 1) * kspan;
#pragma unroll
        for (int x = 0; x < XL; ++x) {
            // the last range may run past K_pad: those columns belong to tiles no wavefront
            // computes; clamp them so the loads stay inside the row
            int64_t col = k0 + st_col[x];
            if (col > kcap) col = kcap;
            if (st_dst[x] >= 0) st[x] = *reinterpret_cast<const u32x4*>(st_row[x] + col);
        }
    };
    auto store_x = [&](const u32x4 (&st)[XL], int buf) {
#pragma unroll
        for (int x = 0; x < XL; ++x)
            if (st_dst[x] >= 0) *reinterpret_cast<u32x4*>(lds + buf * XT + st_dst[x]) = st[x];
    };
    // operand read: token row min(t, R-1), 16-byte column 32 wk + 8 c + 4 hh + s of the stage
    const int rd_base = (((32 * wk + 4 * hh) << LR) + (t < R ? t : R - 1)) << 4;

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    // ---- main product ----------------------------------------------------------------------------
    // per iteration: wait, barrier, stage activations of iteration+1, fetch weights of iteration+2,
    // then the arithmetic of this iteration
    {
        auto tile_at = [&](int64_t it) {
            int64_t tl = wk + NWK * it;
            return tl < a.KT ? tl : a.KT - 1;                                // clamped re-read
        };
        const uint8_t* wrec = a.Wt + grp * a.KT * kWRecordBytes;
        // Three weight records rotate through three register sets by name (the loop is unrolled by
        // three); copying one set into another would make the wavefront wait for the newest load.
        WRec wa, wb, wd;
        {
            u32x4 st[XL];
            fetch_x(0, st);
            wa = load_wrec(wrec + tile_at(0) * kWRecordBytes, lane);
            wb = load_wrec(wrec + tile_at(1) * kWRecordBytes, lane);
            store_x(st, 0);
        }
        auto step = [&](const WRec& cur, WRec& fill, int64_t it) {
            const int buf = (int)(it & 1);
            __syncthreads();                 // stage `it` is complete; buffer buf^1 is free again
            u32x4 st[XL];
            fetch_x(it + 1, st);
            __builtin_amdgcn_sched_barrier(0);      // loads retire in order: activations stay ahead of weights
            fill = load_wrec(wrec + tile_at(it + 2) * kWRecordBytes, lane);
            if (wk + NWK * it < a.KT) {
                const uint8_t* xs = lds + buf * XT + rd_base;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        Frag xf;
                        xf.u = *reinterpret_cast<const u32x4*>(xs + ((8 * c + s) << (LR + 4)));
                        const uint32_t ew = cur.e[c >> 1] >> (16 * (c & 1) + 8 * (s >> 1));
                        const bf16x8 wv = unpack_w8(cur.c[c][s], w_scale(ew & 0xFFu));
                        acc = mfma32(wv, xf.v, acc);
                    }
                }
            }
            store_x(st, buf ^ 1);            // waits for the activation loads only; `fill` stays in flight
        };
        for (int64_t it = 0; it < NI; it += 3) {
            step(wa, wd, it);
            if (it + 1 < NI) step(wb, wa, it + 1);
            if (it + 2 < NI) step(wd, wb, it + 2);
        }
    }

    // ---- rank-kp correction: 64-wide chunks of [T_hi | T_lo], spread over the K slices ----------
    // Lane half hh owns rank blocks jb = 4 ch + 2 hh + {0, 1} of chunk ch, as in the main loop;
    // jb < kp16 is T_hi for ranks 16 jb.., otherwise T_lo for ranks 16 (jb - kp16)...
    const int nb2 = 2 * a.kp16;
    const int nchunks = (nb2 + 3) / 4;
    for (int ch = wk; ch < nchunks; ch += NWK) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int jb = 4 * ch + 2 * hh + j;
            const bool live = jb < nb2;
            const bool is_lo = jb >= a.kp16;
            const int rb = live ? (is_lo ? jb - a.kp16 : jb) : 0;
            Frag ta[2];
            if (!live) {
                ta[0].u = u32x4{0, 0, 0, 0};
                ta[1].u = u32x4{0, 0, 0, 0};
            } else if (a.S == 1) {
                const uint16_t* src = xrow - 32 * hh + a.KT * kTileK + 16 * jb;
                ta[0].u = *reinterpret_cast<const u32x4*>(src);
                ta[1].u = *reinterpret_cast<const u32x4*>(src + 8);
            } else {
                float tv[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) tv[i] = 0.f;
                for (int sl = 0; sl < a.S; ++sl) {                      // fixed order over the K slices
                    const float* src = a.Tpart + ((int64_t)sl * a.M + trow) * a.kp + 16 * rb;
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
                        ta[h].u[i] = pack_bf16_exact(tv[8 * h + 2 * i], tv[8 * h + 2 * i + 1]);
            }
            u32x4 cw = u32x4{0, 0, 0, 0};
            uint32_t eb = 0;
            if (live) {
                const uint8_t* rec = a.Bt + (grp * a.kp16 + rb) * kBRecordBytes;
                cw = *reinterpret_cast<const u32x4*>(rec + t * 16);
                eb = rec[512 + t];
            }
            Frag bf[2];
            int8x16_to_frags(cw, h_scale(eb), bf[0], bf[1]);
            acc = mfma32(bf[0].v, ta[0].v, acc);
            acc = mfma32(bf[1].v, ta[1].v, acc);
        }
    }

    // ---- add the K slices of each column group in a fixed tree order; slice 0 stores ---------------
    __syncthreads();                             // every wavefront is done with the staging buffers
    auto red_at = [&](int k, int r4) {
        return reinterpret_cast<f32x4*>(red + (((size_t)k * NWC + wc) * 64 + lane) * 16 + 4 * r4);
    };
#pragma unroll
    for (int off = NWK / 2; off >= 1; off >>= 1) {
        if (wk >= off && wk < 2 * off) {
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                *red_at(wk - off, r4) = f32x4{acc[4 * r4], acc[4 * r4 + 1], acc[4 * r4 + 2], acc[4 * r4 + 3]};
        }
        __syncthreads();
        if (wk < off) {
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const f32x4 o = *red_at(wk, r4);
                acc[4 * r4] += o[0]; acc[4 * r4 + 1] += o[1]; acc[4 * r4 + 2] += o[2]; acc[4 * r4 + 3] += o[3];
            }
        }
        __syncthreads();
    }
    if (wk == 0 && grp_ok && t < a.M) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int64_t n = grp * 32 + 8 * r4 + 4 * hh;              // this lane's 4 consecutive columns
            float* dst = a.Y + (int64_t)t * a.ldy + n;
            const f32x4 v = f32x4{acc[4 * r4], acc[4 * r4 + 1], acc[4 * r4 + 2], acc[4 * r4 + 3]};
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

int skinny_max_rows() { return 32; }

template <int NWC, int NWK, int LR>
static hipError_t launch_skinny_t(const SkinnyArgs& a, hipStream_t s) {
    constexpr int XT = NWK * (1 << LR) * 512;
    constexpr int STAGING = 2 * XT;
    constexpr int REDUCE = (NWK / 2) * NWC * 4096;
    constexpr int LDS_BYTES = STAGING > REDUCE ? STAGING : REDUCE;
    static_assert(LDS_BYTES <= 160 * 1024, "does not fit the 160 KB of LDS");
    auto kern = skinny_kernel<NWC, NWK, LR>;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((unsigned)((a.N32 + NWC - 1) / NWC)), block(64 * NWC * NWK);
    hipLaunchKernelGGL(kern, grid, block, LDS_BYTES, s, a);
    return hipGetLastError();
}

template <int NWC, int NWK>
static hipError_t launch_skinny_rows(const SkinnyArgs& a, hipStream_t s) {
    if (a.M <= 4) return launch_skinny_t<NWC, NWK, 2>(a, s);
    if constexpr (NWK <= 8) {
        if (a.M <= 16) return launch_skinny_t<NWC, NWK, 4>(a, s);
    }
    if constexpr (NWK <= 4) {
        return launch_skinny_t<NWC, NWK, 5>(a, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_skinny(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy,
                         int variant, hipStream_t s) {
    if (M == 0) return hipSuccess;
    SkinnyArgs a;
    a.Wt = L.Wt; a.Bt = L.Bt; a.Xh = ws.Xh; a.ldxh = ws.ldxh; a.Tpart = ws.Tpart; a.S = ws.S;
    a.Y = Y; a.ldy = ldy; a.M = M; a.N = L.N; a.KT = L.KT; a.N32 = L.N32; a.kp = L.kp; a.kp16 = L.kp16;
    // variant = 100 * NWC + NWK (column-group wavefronts x K slices per workgroup); 0 = automatic:
    // wide layers share staged activations between many column groups, narrow layers split K
    // further so that the chip still has enough loads in flight.  The staging buffers bound the
    // K slices: 16 token rows allow 8, 32 rows allow 4.
    int v = variant;
    if (v == 0) {
        if (L.N32 >= 512) v = 404;
        else if (L.N32 >= 256) v = 204;
        else v = (M <= 4) ? 116 : (M <= 16 ? 108 : 204);
    }
    const int max_k = (M <= 4) ? 16 : (M <= 16 ? 8 : 4);
    if (v % 100 > max_k) return hipErrorInvalidValue;
    switch (v) {
        case 802: return launch_skinny_rows<8, 2>(a, s);
        case 404: return launch_skinny_rows<4, 4>(a, s);
        case 402: return launch_skinny_rows<4, 2>(a, s);
        case 208: return launch_skinny_rows<2, 8>(a, s);
        case 204: return launch_skinny_rows<2, 4>(a, s);
        case 116: return launch_skinny_rows<1, 16>(a, s);
        case 108: return launch_skinny_rows<1, 8>(a, s);
        case 104: return launch_skinny_rows<1, 4>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lqer
