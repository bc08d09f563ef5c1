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
// of a column group are added through LDS in slice order.
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
// NIP = 0: the general, pipelined loop over any number of iterations.  NIP = 2 or 4: short layers
// whose K range is covered in at most NIP iterations fetch every weight record and every
// activation stage up front (all HBM requests in flight at once), synchronise once and then do
// all the arithmetic; with so few iterations a two-deep pipeline would pay the memory latency
// several times over.
template <int NWC, int NWK, int LR, int NIP>
__global__ __launch_bounds__(64 * NWC * NWK) void skinny_kernel(SkinnyArgs a) {
    constexpr int NW = NWC * NWK;
    constexpr int R = 1 << LR;
    constexpr int XT = NWK * R * 512;                // bytes of one stage: R rows x NWK tiles of bf16
    constexpr int NL = XT / 1024;                    // direct loads (1 KiB each) per stage
    constexpr int XL = (NL + NW - 1) / NW;           // ... per wavefront
    constexpr int kTBytes = 32 * 128 * 2;            // T_hi | T_lo of up to 32 tokens x 64 ranks, bf16
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    uint16_t* tlds = reinterpret_cast<uint16_t*>(lds);                 // [32][2 kp] bf16, kept all along
    uint8_t* xlds = lds + kTBytes;                                     // the activation stages (2, or NIP)
    float* red = reinterpret_cast<float*>(lds + kTBytes);              // reused after the main loop: [NWK-1][NWC][64][16]

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
            if (st_dst[x] >= 0) *reinterpret_cast<u32x4*>(xlds + buf * XT + st_dst[x]) = st[x];
    };
    // operand read: token row min(t, R-1), 16-byte column 32 wk + 8 c + 4 hh + s of the stage
    const int rd_base = (((32 * wk + 4 * hh) << LR) + (t < R ? t : R - 1)) << 4;

    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    // ---- rank-kp correction, part 1: fetch its operands first ---------------------------------------
    // The correction is 2 kp more "K columns" in 64-wide chunks of [T_hi | T_lo]; chunk ch belongs to
    // K slice ch.  Lane half hh owns rank blocks jb = 4 ch + 2 hh + {0, 1}: jb < kp16 is T_hi for
    // ranks 16 jb.., otherwise T_lo for ranks 16 (jb - kp16)...  Its loads are issued before
    // anything else so that their latency hides behind the first weight records.
    const int nb2 = 2 * a.kp16;
    const int nchunks = (nb2 + 3) / 4;
    const bool has_tail = wk < nchunks;              // NWK >= 2 >= nchunks: at most one chunk each
    u32x4 tail_cw[2] = {u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}};
    uint32_t tail_eb[2] = {0, 0};
    bool tail_live[2] = {false, false};
    int tail_jb[2] = {0, 0};
    if (has_tail) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int jb = 4 * wk + 2 * hh + j;
            tail_jb[j] = jb;
            tail_live[j] = jb < nb2;
            if (tail_live[j]) {
                const int rb = jb >= a.kp16 ? jb - a.kp16 : jb;
                const uint8_t* rec = a.Bt + (grp * a.kp16 + rb) * kBRecordBytes;
                tail_cw[j] = *reinterpret_cast<const u32x4*>(rec + t * 16);
                tail_eb[j] = rec[512 + t];
            }
        }
    }
    // T itself: when the projection kernel left S (<= 8) partial sums, the whole workgroup adds them
    // in slice order and leaves T_hi | T_lo as bf16 in LDS.  One item = 4 consecutive ranks of a
    // token; a thread owns at most TI items.  The loads are issued here, the sums are formed after
    // the first weight loads have been issued (so those stay in flight meanwhile).
    constexpr int TI = (32 * 16 + NW * 64 - 1) / (NW * 64);
    constexpr int SMAX = 8;
    f32x4 tpart[TI][SMAX];
    const int t_rows = a.M < 32 ? (int)a.M : 32;
    const int kp4 = a.kp >> 2;
    const int t_items = (a.S > 1) ? t_rows * kp4 : 0;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
        const int item = threadIdx.x + i * NW * 64;
        const int it2 = item < t_items ? item : 0;
        const int row = kp4 ? it2 / kp4 : 0, r4 = it2 - row * kp4;
#pragma unroll
        for (int sl = 0; sl < SMAX; ++sl) {
            tpart[i][sl] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (item < t_items && sl < a.S)
                tpart[i][sl] = *reinterpret_cast<const f32x4*>(a.Tpart + ((int64_t)sl * a.M + row) * a.kp + 4 * r4);
        }
    }
    auto finish_t = [&]() {
#pragma unroll
        for (int i = 0; i < TI; ++i) {
            const int item = threadIdx.x + i * NW * 64;
            if (item >= t_items) continue;
            const int row = item / kp4, r4 = item - row * kp4;
            f32x4 sum = tpart[i][0];
#pragma unroll
            for (int sl = 1; sl < SMAX; ++sl) {
                sum[0] += tpart[i][sl][0]; sum[1] += tpart[i][sl][1];
                sum[2] += tpart[i][sl][2]; sum[3] += tpart[i][sl][3];
            }
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t hb = f32_bits(sum[e]) & 0xFFFF0000u;
                hi[e] = hb >> 16;
                lo[e] = f32_bits(sum[e] - f32_from_bits(hb)) >> 16;
            }
            uint16_t* dst = tlds + row * 2 * a.kp + 4 * r4;
            *reinterpret_cast<u32x2*>(dst) = u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
            *reinterpret_cast<u32x2*>(dst + a.kp) = u32x2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
        }
    };

    // ---- main product ----------------------------------------------------------------------------
    // per iteration: barrier, fetch activations of iteration+1, fetch weights of iteration+2,
    // the arithmetic of this iteration, then write the fetched activations to LDS
    {
        auto tile_at = [&](int64_t it) {
            int64_t tl = wk + NWK * it;
            return tl < a.KT ? tl : a.KT - 1;                                // clamped re-read
        };
        const uint8_t* wrec = a.Wt + grp * a.KT * kWRecordBytes;
        auto mma_tile = [&](const WRec& cur, int64_t it, int stage) {
            if (wk + NWK * it < a.KT) {
                const uint8_t* xs = xlds + stage * XT + rd_base;
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
        };
        if constexpr (NIP > 0) {
            WRec w[NIP];
            u32x4 st[NIP][XL];
#pragma unroll
            for (int i = 0; i < NIP; ++i) fetch_x(i, st[i]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NIP; ++i) w[i] = load_wrec(wrec + tile_at(i) * kWRecordBytes, lane);
            finish_t();
#pragma unroll
            for (int i = 0; i < NIP; ++i) store_x(st[i], i);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NIP; ++i) mma_tile(w[i], i, i);
        } else {
        // Three weight records rotate through three register sets by name (the loop is unrolled by
        // three); copying one set into another would make the wavefront wait for the newest load.
        WRec wa, wb, wd;
        {
            u32x4 st[XL];
            fetch_x(0, st);
            wa = load_wrec(wrec + tile_at(0) * kWRecordBytes, lane);
            wb = load_wrec(wrec + tile_at(1) * kWRecordBytes, lane);
            finish_t();
            store_x(st, 0);
        }
        // All loads of a full step are unconditional (indices clamped): a load inside a branch would
        // make the compiler's wait counts assume the worst case.  The last iteration is peeled off
        // instead and fetches nothing.
        auto step = [&](const WRec& cur, WRec& fill, int64_t it) {
            __syncthreads();                 // stage `it` is complete; the other buffer is free again
            u32x4 st[XL];
            fetch_x(it + 1, st);
            __builtin_amdgcn_sched_barrier(0);      // loads retire in order: activations stay ahead of weights
            fill = load_wrec(wrec + tile_at(it + 2) * kWRecordBytes, lane);
            mma_tile(cur, it, (int)(it & 1));
            store_x(st, (int)((it + 1) & 1));    // waits for the activation loads only; `fill` stays in flight
        };
        auto last_step = [&](const WRec& cur, int64_t it) {
            __syncthreads();
            mma_tile(cur, it, (int)(it & 1));
        };
        int64_t it = 0;
        for (; it + 3 < NI; it += 3) {
            step(wa, wd, it);
            step(wb, wa, it + 1);
            step(wd, wb, it + 2);
        }
        // one to three iterations remain; the record of iteration it+k sits in set (wa, wb, wd)[k]
        if (it + 1 == NI) {
            last_step(wa, it);
        } else if (it + 2 == NI) {
            step(wa, wd, it);
            last_step(wb, it + 1);
        } else {
            step(wa, wd, it);
            step(wb, wa, it + 1);
            last_step(wd, it + 2);
        }
        }
    }

    // ---- rank-kp correction, part 2: the arithmetic ---------------------------------------------------
    if (has_tail) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            Frag ta[2];
            ta[0].u = u32x4{0, 0, 0, 0};
            ta[1].u = u32x4{0, 0, 0, 0};
            if (tail_live[j]) {
                if (a.S == 1) {                  // T was final: it sits behind the activations of the row
                    const uint16_t* src = xrow - 32 * hh + a.KT * kTileK + 16 * tail_jb[j];
                    ta[0].u = *reinterpret_cast<const u32x4*>(src);
                    ta[1].u = *reinterpret_cast<const u32x4*>(src + 8);
                } else {
                    const uint16_t* src = tlds + (int)trow * 2 * a.kp + 16 * tail_jb[j];
                    ta[0].u = *reinterpret_cast<const u32x4*>(src);
                    ta[1].u = *reinterpret_cast<const u32x4*>(src + 8);
                }
            }
            Frag bf[2];
            int8x16_to_frags(tail_cw[j], h_scale(tail_eb[j]), bf[0], bf[1]);
            acc = mfma32(bf[0].v, ta[0].v, acc);
            acc = mfma32(bf[1].v, ta[1].v, acc);
        }
    }

    // ---- add the K slices of each column group in slice order; slice 0 stores -----------------------
    __syncthreads();                             // every wavefront is done with the staging buffers
    auto red_at = [&](int k, int r4) {
        return reinterpret_cast<f32x4*>(red + (((size_t)k * NWC + wc) * 64 + lane) * 16 + 4 * r4);
    };
    if (wk > 0) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
            *red_at(wk - 1, r4) = f32x4{acc[4 * r4], acc[4 * r4 + 1], acc[4 * r4 + 2], acc[4 * r4 + 3]};
    }
    __syncthreads();
    if (wk == 0) {
#pragma unroll
        for (int k = 0; k < NWK - 1; ++k)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const f32x4 o = *red_at(k, r4);
                acc[4 * r4] += o[0]; acc[4 * r4 + 1] += o[1]; acc[4 * r4 + 2] += o[2]; acc[4 * r4 + 3] += o[3];
            }
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

template <int NWC, int NWK, int LR, int NIP>
static hipError_t launch_skinny_t(const SkinnyArgs& a, hipStream_t s) {
    constexpr int XT = NWK * (1 << LR) * 512;
    constexpr int STAGING = (NIP > 0 ? NIP : 2) * XT;
    constexpr int REDUCE = (NWK - 1) * NWC * 4096;
    constexpr int LDS_BYTES = 32 * 128 * 2 + (STAGING > REDUCE ? STAGING : REDUCE);
    static_assert(LDS_BYTES <= 160 * 1024, "does not fit the 160 KB of LDS");
    auto kern = skinny_kernel<NWC, NWK, LR, NIP>;
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

// picks the preloading form when the K range fits in 2 or 4 iterations and their stages fit LDS
template <int NWC, int NWK, int LR>
static hipError_t launch_skinny_k(const SkinnyArgs& a, hipStream_t s) {
    constexpr int XT = NWK * (1 << LR) * 512;
    const int64_t NI = (a.KT + NWK - 1) / NWK;
    if constexpr (2 * XT <= 128 * 1024) {
        if (NI <= 2) return launch_skinny_t<NWC, NWK, LR, 2>(a, s);
    }
    if constexpr (4 * XT <= 128 * 1024) {
        if (NI <= 4) return launch_skinny_t<NWC, NWK, LR, 4>(a, s);
    }
    return launch_skinny_t<NWC, NWK, LR, 0>(a, s);
}

template <int NWC, int NWK>
static hipError_t launch_skinny_rows(const SkinnyArgs& a, hipStream_t s) {
    if (a.M <= 4) return launch_skinny_k<NWC, NWK, 2>(a, s);
    if constexpr (NWK <= 8) {
        if (a.M <= 16) return launch_skinny_k<NWC, NWK, 4>(a, s);
    }
    if constexpr (NWK <= 4) {
        return launch_skinny_k<NWC, NWK, 5>(a, s);
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
        if (L.N32 >= 512) v = (M <= 16) ? 404 : 402;
        else if (L.N32 >= 256) v = 204;
        else v = (M <= 16) ? 108 : 104;
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
