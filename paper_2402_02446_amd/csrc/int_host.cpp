// Host side of the scaled-integer variant of the layer (Table 2, "L2QER-INT": INT4 weights in groups of 128 with
// FP16 scales, INT8 rank-k factors with the same grouping, INT8 activations with one scale per token; Sec. 2.1 for the
// form of such formats): import / export of canonical arrays, the offline step, workspace plan and the two launches
// of the forward pass.  The kernels are in kernels_int.hip.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "lqer_internal.h"
#include "host_parallel.h"

namespace lqer {

// declared in kernels_int.hip
struct IntGemmArgs {
    const int8_t* Xc; int64_t ldxc;
    const float* Xs;
    const uint8_t* Wt;
    const float* Wsc;
    int64_t M, N, N32, G;
    float* Out; int64_t ldo;
    int64_t g_per_z;
    int64_t out_z_stride;
    const float* T; int64_t ldt;
    int S; int64_t t_stride;
    const uint8_t* Bt; const float* Bsc;
    int kp16;
    int tail_plane;
};
hipError_t launch_int_gemm(bool projection, const IntGemmArgs& a, hipStream_t s);
hipError_t launch_int_reduce_planes(const float* P, int planes, int64_t plane_stride, int64_t M, int64_t N, int64_t ldp,
                                    float* Y, int64_t ldy, hipStream_t s);

static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

static float fp16_to_float(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

// x >= 0 -> the nearest fp16 (ties to even) in one rounding step, as bits; false when it is not finite in fp16
static bool double_to_fp16(double x, uint16_t* bits) {
    if (x == 0.0) { *bits = 0; return true; }
    int ex;
    (void)std::frexp(x, &ex);                        // x = m 2^ex, m in [0.5, 1)
    int e = ex - 1;
    if (e < -14) e = -14;                            // subnormal range: fixed spacing 2^-24
    const double q = std::nearbyint(std::ldexp(x, 10 - e));          // in units of the spacing at e; ties to even
    const double v = std::ldexp(q, e - 10);
    if (v >= 65520.0) return false;
    *bits = __builtin_bit_cast(uint16_t, (_Float16)(float)v);        // v is an fp16 number: exact
    return true;
}

// One group of `len` values with stride -> codes and the FP16 scale (amax / qmax, 1 for an all-zero group).
static int quantize_group(const double* v, int64_t stride, int len, int qmax, int8_t* codes, int64_t cstride, uint16_t* scale) {
    double amax = 0.0;
    for (int i = 0; i < len; ++i) amax = std::max(amax, std::fabs(v[i * stride]));
    uint16_t sb = 0x3C00;                            // 1.0
    if (amax > 0.0 && (!double_to_fp16(amax / qmax, &sb) || sb == 0)) return LQER_ERR_VALUE;   // scale outside the fp16 range
    const double s = (double)fp16_to_float(sb);
    for (int i = 0; i < len; ++i) {
        double r = std::nearbyint(v[i * stride] / s);
        r = std::min((double)qmax, std::max((double)-qmax, r));
        codes[i * cstride] = (int8_t)r;
    }
    *scale = sb;
    return LQER_OK;
}

static int upload_floats(const std::vector<float>& host, float** dev) {
    *dev = nullptr;
    if (host.empty()) return LQER_OK;
    if (hipMalloc((void**)dev, host.size() * 4) != hipSuccess) return LQER_ERR_HIP;
    if (hipMemcpy(*dev, host.data(), host.size() * 4, hipMemcpyHostToDevice) != hipSuccess) return LQER_ERR_HIP;
    return LQER_OK;
}

// position of element e (0..127) of a K group in the order the kernel reads activations and 8-bit weights:
// every run of 32 as its 16 even elements followed by its 16 odd ones
static inline int perm_pos(int e) { return (e & ~31) + ((e & 1) << 4) + ((e & 31) >> 1); }

// K planes of the projection: it has few output columns, so with few token tiles its K groups are spread over
// workgroups (each keeps at least two groups: a workgroup's groups are a chain of dependent memory round trips, which
// is what a few-token call waits for); a small kernel then adds the planes' partial T in plane order.
static int projection_planes(const Layer& L, int64_t M) {
    const int64_t tiles = (M + 127) / 128, G = L.K / 128;
    int64_t s = 1;
    while (tiles * s < 256 && s < 16 && G / (2 * s) >= 2) s *= 2;
    return (int)s;
}

// K planes of the main product: with few output tiles (few tokens) its K groups are spread over workgroups as well,
// each plane leaving partial sums of Y in the workspace for a small kernel to add up; the rank-k correction then gets a
// plane of its own.  Two workgroups fit a compute unit: the fewest groups per plane (at least two) that keep the launch
// within 512 workgroups.
static int main_planes(const Layer& L, int64_t M) {
    const int64_t tiles = ((M + 127) / 128) * ((L.N + 127) / 128), G = L.K / 128, cap = 512;
    const int64_t extra = L.kp > 0 ? 1 : 0;
    if (tiles * (2 + extra) > cap) return 1;
    int64_t g = 2;                                     // K groups per plane
    while (g < G && tiles * ((G + g - 1) / g + extra) > cap) ++g;
    return (int)((G + g - 1) / g);
}

size_t int_workspace_bytes(const Layer& L, int64_t M) {
    if (M <= 0) return 0;
    const int64_t mp = round_up(M, 128);
    const int sm = main_planes(L, M);
    return (size_t)(round_up(mp * L.K, 256) + round_up(mp * 4, 256) +
                    round_up((int64_t)projection_planes(L, M) * mp * (int64_t)L.kp32 * 32 * 4, 256) +
                    (sm > 1 ? (int64_t)(sm + 1) * M * round_up(L.N, 4) * 4 : 0));       // (the planes of Y hold the M real rows only)
}

int forward_int(const Layer& L, const float* X, int64_t ldx, int64_t M, float* Y, int64_t ldy, void* ws, size_t ws_bytes,
                hipStream_t s) {
    if (int_workspace_bytes(L, M) > ws_bytes) return LQER_ERR_WORKSPACE;
    const int64_t mp = round_up(M, 128);
    int8_t* Xc = (int8_t*)ws;
    float* Xs = (float*)((uint8_t*)ws + round_up(mp * L.K, 256));
    float* T = (float*)((uint8_t*)Xs + round_up(mp * 4, 256));
    const int64_t ldt = (int64_t)L.kp32 * 32;
    if (launch_quant_token(X, M, L.K, ldx, Xc, L.K, Xs, nullptr, true, s) != hipSuccess) return LQER_ERR_HIP;
    IntGemmArgs a;
    a.Xc = Xc; a.ldxc = L.K; a.Xs = Xs; a.G = L.K / 128; a.M = M;
    const int S = projection_planes(L, M);
    a.T = nullptr; a.ldt = ldt; a.Bt = nullptr; a.Bsc = nullptr; a.kp16 = 0;
    a.S = S; a.t_stride = mp * ldt; a.tail_plane = 0;
    if (L.kp > 0) {
        a.Wt = L.At; a.Wsc = L.Asc; a.N = ldt; a.N32 = L.kp32; a.Out = T; a.ldo = ldt;
        a.g_per_z = (a.G + S - 1) / S; a.out_z_stride = mp * ldt;
        if (launch_int_gemm(true, a, s) != hipSuccess) return LQER_ERR_HIP;
        const int planes = (int)((a.G + a.g_per_z - 1) / a.g_per_z);
        // the planes' partial T are added up (in plane order, into the first) before the main kernel reads them: inside
        // it that sum would be a chain of dependent loads in front of every rank block
        if (planes > 1 && launch_int_reduce_planes(T, planes, mp * ldt, mp, ldt, ldt, T, ldt, s) != hipSuccess) return LQER_ERR_HIP;
        a.S = 1;
    }
    a.Wt = L.Wt; a.Wsc = L.Wsc; a.N = L.N; a.N32 = L.N32; a.Out = Y; a.ldo = ldy;
    a.g_per_z = a.G; a.out_z_stride = 0;
    a.T = T; a.Bt = L.Bt; a.Bsc = L.Bsc; a.kp16 = L.kp16;
    const int sm = main_planes(L, M);
    if (sm > 1) {
        float* P = (float*)((uint8_t*)T + round_up((int64_t)S * mp * ldt * 4, 256));
        const int64_t ldp = round_up(L.N, 4);
        a.Out = P; a.ldo = ldp; a.g_per_z = (a.G + sm - 1) / sm; a.out_z_stride = M * ldp;
        a.tail_plane = L.kp > 0 ? 1 : 0;
        if (launch_int_gemm(false, a, s) != hipSuccess) return LQER_ERR_HIP;
        const int planes = (int)((a.G + a.g_per_z - 1) / a.g_per_z) + a.tail_plane;
        if (launch_int_reduce_planes(P, planes, M * ldp, M, L.N, ldp, Y, ldy, s) != hipSuccess) return LQER_ERR_HIP;
        return LQER_OK;
    }
    if (launch_int_gemm(false, a, s) != hipSuccess) return LQER_ERR_HIP;
    return LQER_OK;
}

// INT8 g128 factors from A (K x k) and B (k x N), then the import
static int pack_int_factors_and_import(int64_t K, int64_t N, int k, const std::vector<uint8_t>& Wc, const std::vector<uint16_t>& Ws,
                                       const std::vector<double>& A, const std::vector<double>& B, lqer_layer** out) {
    const int kp = (k + 15) / 16 * 16;
    const int64_t G = K / 128;
    std::vector<int8_t> Ac((size_t)kp * K, 0), Bc((size_t)N * kp, 0);
    std::vector<uint16_t> As((size_t)kp * G, 0x3C00), Bs((size_t)N, 0x3C00);
    for (int r = 0; r < k; ++r)
        for (int64_t g = 0; g < G; ++g) {
            const int st = quantize_group(&A[(size_t)g * 128 * k + r], k, 128, 127, &Ac[(size_t)r * K + g * 128], 1, &As[(size_t)r * G + g]);
            if (st != LQER_OK) return st;
        }
    std::vector<double> col(kp > 0 ? kp : 1);
    for (int64_t n = 0; n < N && kp > 0; ++n) {
        for (int r = 0; r < kp; ++r) col[r] = r < k ? B[(size_t)r * N + n] : 0.0;
        const int st = quantize_group(col.data(), 1, kp, 127, &Bc[(size_t)n * kp], 1, &Bs[n]);
        if (st != LQER_OK) return st;
    }
    return lqer_int_layer_import(K, N, k, Wc.data(), Ws.data(), kp ? Ac.data() : nullptr, kp ? As.data() : nullptr,
                                 kp ? Bc.data() : nullptr, kp ? Bs.data() : nullptr, out);
}

int build_factors_int(const float* W_host, int64_t K, int64_t N, const std::vector<double>& s, int k, lqer_layer** out) {
    if ((K & 127) != 0) return LQER_ERR_SHAPE;
    const int kp = (k + 15) / 16 * 16;
    if (kp > 128) return LQER_ERR_UNSUPPORTED;
    const int64_t G = K / 128;
    for (int64_t i = 0; i < K * N; ++i)
        if (!std::isfinite(W_host[i])) return LQER_ERR_VALUE;
    std::vector<uint8_t> Wc((size_t)N * (K / 2));
    std::vector<uint16_t> Ws((size_t)N * G);
    std::vector<double> Gm;
    if (k > 0) Gm.resize((size_t)K * N);
    std::vector<int> status((size_t)N, LQER_OK);
    parallel_for(N, [&](int64_t n) {
        double col[128];
        int8_t codes[128];
        for (int64_t g = 0; g < G; ++g) {
            for (int i = 0; i < 128; ++i) col[i] = (double)W_host[(g * 128 + i) * N + n];
            uint16_t sb;
            const int st = quantize_group(col, 1, 128, 7, codes, 1, &sb);
            if (st != LQER_OK) { status[n] = st; return; }
            Ws[n * G + g] = sb;
            for (int i = 0; i < 64; ++i)
                Wc[n * (K / 2) + g * 64 + i] = (uint8_t)((codes[2 * i] & 0xF) | ((codes[2 * i + 1] & 0xF) << 4));
            if (k > 0) {
                const double sc = (double)fp16_to_float(sb);
                for (int i = 0; i < 128; ++i) {
                    const int64_t row = g * 128 + i;
                    Gm[(size_t)row * N + n] = s[row] * (col[i] - codes[i] * sc);
                }
            }
        }
    }, 8);
    for (int64_t n = 0; n < N; ++n)
        if (status[n] != LQER_OK) return status[n];
    std::vector<double> A, B;
    if (k > 0) {
        const int st = truncated_split(Gm, K, N, s, k, A, B);
        if (st != LQER_OK) return st;
        Gm.clear();
        Gm.shrink_to_fit();
    }
    return pack_int_factors_and_import(K, N, k, Wc, Ws, A, B, out);
}

}  // namespace lqer

using namespace lqer;

extern "C" {

int lqer_quantize_int8_token(const float* x_dev, int64_t rows, int64_t cols, int64_t ld, int8_t* codes_dev,
                             uint16_t* scales_dev, void* hip_stream) {
    if (rows < 0 || cols < 0 || (cols & 3) != 0 || ld < cols) return LQER_ERR_SHAPE;
    if (rows == 0 || cols == 0) return LQER_OK;
    if (!x_dev || !codes_dev || !scales_dev) return LQER_ERR_NULL;
    if ((ld & 3) != 0 || ((uintptr_t)x_dev & 15) != 0 || ((uintptr_t)codes_dev & 3) != 0) return LQER_ERR_SHAPE;
    if (launch_quant_token(x_dev, rows, cols, ld, codes_dev, cols, nullptr, scales_dev, false, (hipStream_t)hip_stream) != hipSuccess)
        return LQER_ERR_HIP;
    return LQER_OK;
}

int lqer_int_layer_import(int64_t K, int64_t N, int k, const uint8_t* Wc, const uint16_t* Ws, const int8_t* Ac,
                          const uint16_t* As, const int8_t* Bc, const uint16_t* Bs, lqer_layer** out) {
    if (!out) return LQER_ERR_NULL;
    *out = nullptr;
    if (K <= 0 || N <= 0 || (K & 127) != 0 || k < 0 || k > K || k > N) return LQER_ERR_SHAPE;
    if (!Wc || !Ws) return LQER_ERR_NULL;
    if (k > 0 && (!Ac || !As || !Bc || !Bs)) return LQER_ERR_NULL;
    const int kp = (k + 15) / 16 * 16;
    if (kp > 128) return LQER_ERR_UNSUPPORTED;
    lqer_layer* h = new (std::nothrow) lqer_layer;
    if (!h) return LQER_ERR_NO_MEMORY;
    Layer& L = h->L;
    L.K = K; L.N = N; L.k = k; L.kp = kp;
    L.KT = (K + kTileK - 1) / kTileK;
    L.N32 = (N + 31) / 32;
    L.kp16 = kp / 16;
    L.kp32 = (kp + 31) / 32;
    L.act_bits = 8; L.w_bits = 4; L.w_rec_bytes = 2048; L.w_exp_bias = -1;
    L.format = 1;
    L.Wt = L.At = L.Bt = nullptr;
    L.Wsc = L.Asc = L.Bsc = nullptr;
    const int64_t G = K / 128;
    int st = LQER_OK;
    if (hipGetDevice(&L.device) != hipSuccess) { delete h; return LQER_ERR_HIP; }
    auto finite_scale = [](uint16_t b) { return (b & 0x7C00) != 0x7C00 && (b & 0x8000) == 0 && b != 0; };   // positive, finite, non-zero
    try {
        // canonical copies for export
        h->iWc.assign(Wc, Wc + (size_t)N * (K / 2));
        h->iWs.assign(Ws, Ws + (size_t)N * G);
        if (kp > 0) {
            h->iAc.assign(Ac, Ac + (size_t)kp * K);
            h->iAs.assign(As, As + (size_t)kp * G);
            h->iBc.assign(Bc, Bc + (size_t)N * kp);
            h->iBs.assign(Bs, Bs + (size_t)N);
        }
        for (uint16_t b : h->iWs) if (!finite_scale(b)) st = LQER_ERR_VALUE;
        for (uint16_t b : h->iAs) if (!finite_scale(b)) st = LQER_ERR_VALUE;
        for (uint16_t b : h->iBs) if (!finite_scale(b)) st = LQER_ERR_VALUE;
        // W_q: [N32][G] records of [2 spans][64 lanes][16 B] canonical nibbles; scales / 16 as fp32 [N32][G][32]
        if (st == LQER_OK) {
            std::vector<uint8_t> rec((size_t)(L.N32 * G) * 2048, 0);
            std::vector<float> sc((size_t)(L.N32 * G) * 32, 0.f);
            std::vector<int> bad((size_t)L.N32, 0);
            parallel_for(L.N32, [&](int64_t g32) {
                for (int64_t g = 0; g < G; ++g) {
                    uint8_t* r = rec.data() + (size_t)(g32 * G + g) * 2048;
                    for (int lane = 0; lane < 64; ++lane) {
                        const int i = lane & 31, hh = lane >> 5;
                        const int64_t n = g32 * 32 + i;
                        if (n >= N) continue;
                        for (int sp = 0; sp < 2; ++sp) {
                            const uint8_t* src = Wc + n * (K / 2) + (g * 128 + sp * 64 + hh * 32) / 2;
                            for (int j = 0; j < 16; ++j)
                                if ((src[j] & 0xF) == 8 || (src[j] >> 4) == 8) bad[g32] = 1;     // -8 is no code of the symmetric format
                            memcpy(r + sp * 1024 + lane * 16, src, 16);
                        }
                    }
                    for (int i = 0; i < 32; ++i) {
                        const int64_t n = g32 * 32 + i;
                        if (n < N) sc[(size_t)(g32 * G + g) * 32 + i] = fp16_to_float(Ws[n * G + g]) * 0.0625f;
                    }
                }
            });
            for (int b : bad) if (b) st = LQER_ERR_VALUE;
            if (st == LQER_OK) st = upload(rec, &L.Wt);
            if (st == LQER_OK) st = upload_floats(sc, &L.Wsc);
        }
        if (st == LQER_OK && kp > 0) {
            // A_k as 8-bit "weights": [kp32][G] records of [4 steps][64 lanes][16 B], K permuted like the activations
            std::vector<uint8_t> rec((size_t)(L.kp32 * G) * 4096, 0);
            std::vector<float> sc((size_t)(L.kp32 * G) * 32, 0.f);
            for (int g32 = 0; g32 < L.kp32; ++g32)
                for (int64_t g = 0; g < G; ++g) {
                    uint8_t* r = rec.data() + (size_t)(g32 * G + g) * 4096;
                    for (int i = 0; i < 32; ++i) {
                        const int row = g32 * 32 + i;
                        if (row >= kp) continue;
                        sc[(size_t)(g32 * G + g) * 32 + i] = fp16_to_float(As[(size_t)row * G + g]);
                        for (int e = 0; e < 128; ++e) {
                            // the kernel's MFMA (sp, p) of a group meets bytes 64 sp + 32 hh + 16 p + j of the token's 128
                            const int pos = perm_pos(e);
                            const int sp = pos >> 6, hh2 = (pos >> 5) & 1, p = (pos >> 4) & 1, j = pos & 15;
                            r[(2 * sp + p) * 1024 + (hh2 * 32 + i) * 16 + j] = (uint8_t)Ac[(size_t)row * K + g * 128 + e];
                        }
                    }
                }
            st = upload(rec, &L.At);
            if (st == LQER_OK) st = upload_floats(sc, &L.Asc);
        }
        if (st == LQER_OK && kp > 0) {
            std::vector<uint8_t> buf;
            st = tile_b(L, Bc, nullptr, buf);
            if (st == LQER_OK) st = upload(buf, &L.Bt);
            std::vector<float> sc((size_t)L.N32 * 32, 0.f);
            for (int64_t n = 0; n < N; ++n) sc[n] = fp16_to_float(Bs[n]);
            if (st == LQER_OK) st = upload_floats(sc, &L.Bsc);
        }
    } catch (...) {
        st = LQER_ERR_NO_MEMORY;
    }
    if (st != LQER_OK) {
        free_device(L);
        delete h;
        return st;
    }
    *out = h;
    return LQER_OK;
}

int lqer_int_layer_export(const lqer_layer* layer, uint8_t* Wc, uint16_t* Ws, int8_t* Ac, uint16_t* As, int8_t* Bc,
                          uint16_t* Bs) {
    if (!layer) return LQER_ERR_NULL;
    if (layer->L.format != 1) return LQER_ERR_UNSUPPORTED;
    if (Wc) memcpy(Wc, layer->iWc.data(), layer->iWc.size());
    if (Ws) memcpy(Ws, layer->iWs.data(), layer->iWs.size() * 2);
    if (Ac) memcpy(Ac, layer->iAc.data(), layer->iAc.size());
    if (As) memcpy(As, layer->iAs.data(), layer->iAs.size() * 2);
    if (Bc) memcpy(Bc, layer->iBc.data(), layer->iBc.size());
    if (Bs) memcpy(Bs, layer->iBs.data(), layer->iBs.size() * 2);
    return LQER_OK;
}

}  // extern "C"
