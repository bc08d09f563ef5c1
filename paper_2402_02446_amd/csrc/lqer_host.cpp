// Host side of liblqer: the C ABI, layer import/export (canonical bytes <-> tiled device layout),
// workspace planning and the dispatch between the streaming and the tiled main kernel.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "lqer_internal.h"
#include "host_parallel.h"

namespace lqer {

static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

// ---- W code words -------------------------------------------------------------------------------
// 8 signed codes (-7..7) -> one 32-bit word, layout documented in lqer_internal.h.
static uint32_t encode_word(const int8_t* c) {
    uint32_t w = 0;
    for (int i = 0; i < 4; ++i) {
        const int lo = c[i], hi = c[4 + i];
        const uint32_t mag_lo = (uint32_t)(lo < 0 ? -lo : lo), s_lo = lo < 0;
        const uint32_t mag_hi = (uint32_t)(hi < 0 ? -hi : hi), s_hi = hi < 0;
        w |= (mag_lo | (s_lo << 7) | (mag_hi << 4)) << (8 * i);
        w |= (s_hi << 3) << (8 * ((i + 1) & 3));
    }
    return w;
}

static void decode_word(uint32_t w, int8_t* c) {
    for (int i = 0; i < 4; ++i) {
        const uint32_t b = (w >> (8 * i)) & 0xFF;
        const uint32_t bn = (w >> (8 * ((i + 1) & 3))) & 0xFF;
        const int mag_lo = b & 7, s_lo = (b >> 7) & 1;
        const int mag_hi = (b >> 4) & 7, s_hi = (bn >> 3) & 1;
        c[i] = (int8_t)(s_lo ? -mag_lo : mag_lo);
        c[4 + i] = (int8_t)(s_hi ? -mag_hi : mag_hi);
    }
}

static inline int nibble_to_code(uint32_t v) { return v < 8 ? (int)v : (int)v - 16; }

// 16 codes (-1, 0, 1) of one block -> one 32-bit word, layout documented in lqer_internal.h
static uint32_t encode_word2(const int8_t* c) {
    uint32_t w = 0;
    for (int x = 0; x < 4; ++x)
        for (int i = 0; i < 4; ++i) {
            const int v = c[4 * x + i];
            if (v != 0) w |= 1u << (8 * i + 2 * x);
            if (v < 0) w |= 1u << ((8 * i + 2 * x + 7) & 31);
        }
    return w;
}

static void decode_word2(uint32_t w, int8_t* c) {
    for (int x = 0; x < 4; ++x)
        for (int i = 0; i < 4; ++i) {
            const int mag = (w >> (8 * i + 2 * x)) & 1, sg = (w >> ((8 * i + 2 * x + 7) & 31)) & 1;
            c[4 * x + i] = (int8_t)(sg ? -mag : mag);
        }
}

// the 16 codes of block kb of column n from the canonical bytes (4 bits: nibbles, 2 bits: bit pairs); false on an
// excluded value (nibble -8, bit pair -2)
static bool canonical_block(const uint8_t* Wc, int bits, int64_t K, int64_t n, int64_t kb, int8_t* codes) {
    bool ok = true;
    if (bits == 4) {
        const uint8_t* src = Wc + n * (K / 2) + kb * 8;
        for (int e = 0; e < 8; ++e) {
            const uint32_t lo = src[e] & 0xF, hi = src[e] >> 4;
            if (lo == 8 || hi == 8) ok = false;
            codes[2 * e] = (int8_t)nibble_to_code(lo);
            codes[2 * e + 1] = (int8_t)nibble_to_code(hi);
        }
    } else {
        const uint8_t* src = Wc + n * (K / 4) + kb * 4;
        for (int e = 0; e < 16; ++e) {
            const uint32_t v = (src[e >> 2] >> (2 * (e & 3))) & 3;
            if (v == 2) ok = false;
            codes[e] = (int8_t)(v == 3 ? -1 : (int)v);
        }
    }
    return ok;
}

static void store_canonical_block(uint8_t* Wc, int bits, int64_t K, int64_t n, int64_t kb, const int8_t* codes) {
    if (bits == 4) {
        uint8_t* dst = Wc + n * (K / 2) + kb * 8;
        for (int e = 0; e < 8; ++e) dst[e] = (uint8_t)((codes[2 * e] & 0xF) | ((codes[2 * e + 1] & 0xF) << 4));
    } else {
        uint8_t* dst = Wc + n * (K / 4) + kb * 4;
        for (int e = 0; e < 4; ++e)
            dst[e] = (uint8_t)((codes[4 * e] & 3) | ((codes[4 * e + 1] & 3) << 2) | ((codes[4 * e + 2] & 3) << 4) |
                               ((codes[4 * e + 3] & 3) << 6));
    }
}

// canonical Wc/We -> tiled records.  Returns LQER_ERR_VALUE on a -8 nibble or an exponent byte > 247.
// Chooses the record form: exponent nibbles when the layer's exponent bytes span at most 16 values.
static int tile_weights(Layer& L, const uint8_t* Wc, const uint8_t* We, std::vector<uint8_t>& out) {
    const int64_t nblk = L.K / 16;
    int lo = 255, hi = 0;
    for (int64_t n = 0; n < L.N; ++n)
        for (int64_t kb = 0; kb < nblk; ++kb) {
            const int e = We[n * nblk + kb];
            if (e > kMaxWExpByte) return LQER_ERR_VALUE;
            lo = e < lo ? e : lo;
            hi = e > hi ? e : hi;
        }
    const bool compact = hi - lo <= 15;
    const int bits = L.w_bits;
    L.w_exp_bias = compact ? lo : -1;
    L.w_rec_bytes = w_record_bytes(bits, compact);
    const int kRec = L.w_rec_bytes, bias = L.w_exp_bias;
    const int code_off = compact ? kWCompactCodeOffset : 0, exp_off = w_code_bytes(bits);
    out.assign((size_t)(L.N32 * L.KT) * kRec + kWTailPad, 0);
    std::atomic<int> bad{0};
    parallel_for(L.N32, [&](int64_t g) {
        for (int64_t tile = 0; tile < L.KT; ++tile) {
            uint8_t* rec = out.data() + (size_t)(tile * L.N32 + g) * kRec;
            for (int lane = 0; lane < 64; ++lane) {
                const int i = lane & 31, hh = lane >> 5;
                const int64_t n = g * 32 + i;
                for (int c = 0; c < 4; ++c)
                    for (int j = 0; j < 2; ++j) {
                        const int64_t kb = tile * 16 + 4 * c + 2 * hh + j;
                        int8_t codes[16] = {0};
                        uint8_t eb = (uint8_t)(bias >= 0 ? bias : 0);       // padding blocks: zero codes, any exponent
                        if (n < L.N && kb < nblk) {
                            if (!canonical_block(Wc, bits, L.K, n, kb, codes)) bad.store(1, std::memory_order_relaxed);
                            eb = We[n * nblk + kb];
                        }
                        if (bits == 4) {
                            const uint32_t w0 = encode_word(codes), w1 = encode_word(codes + 8);
                            uint8_t* dst = rec + code_off + c * 1024 + lane * 16 + j * 8;
                            memcpy(dst, &w0, 4);
                            memcpy(dst + 4, &w1, 4);
                        } else {
                            const uint32_t w = encode_word2(codes);
                            memcpy(rec + code_off + (c >> 1) * 1024 + lane * 16 + ((c & 1) * 2 + j) * 4, &w, 4);
                        }
                        if (bias >= 0) {
                            uint8_t& b2 = rec[lane * 4 + c];                            // nibble 2c + j of the lane's word
                            b2 = (uint8_t)(b2 | ((eb - bias) << (4 * j)));
                        } else {
                            rec[exp_off + lane * 8 + 2 * c + j] = eb;
                        }
                    }
            }
        }
    });
    return bad.load() ? LQER_ERR_VALUE : LQER_OK;
}

static void untile_weights(const Layer& L, const std::vector<uint8_t>& in, uint8_t* Wc, uint8_t* We) {
    const int64_t nblk = L.K / 16;
    const int bits = L.w_bits;
    const int code_off = L.w_exp_bias >= 0 ? kWCompactCodeOffset : 0, exp_off = w_code_bytes(bits);
    parallel_for(L.N32, [&](int64_t g) {
        for (int64_t tile = 0; tile < L.KT; ++tile) {
            const uint8_t* rec = in.data() + (size_t)(tile * L.N32 + g) * L.w_rec_bytes;
            for (int lane = 0; lane < 64; ++lane) {
                const int i = lane & 31, hh = lane >> 5;
                const int64_t n = g * 32 + i;
                if (n >= L.N) continue;
                for (int c = 0; c < 4; ++c)
                    for (int j = 0; j < 2; ++j) {
                        const int64_t kb = tile * 16 + 4 * c + 2 * hh + j;
                        if (kb >= nblk) continue;
                        int8_t codes[16];
                        if (bits == 4) {
                            uint32_t w0, w1;
                            const uint8_t* src = rec + code_off + c * 1024 + lane * 16 + j * 8;
                            memcpy(&w0, src, 4);
                            memcpy(&w1, src + 4, 4);
                            decode_word(w0, codes);
                            decode_word(w1, codes + 8);
                        } else {
                            uint32_t w;
                            memcpy(&w, rec + code_off + (c >> 1) * 1024 + lane * 16 + ((c & 1) * 2 + j) * 4, 4);
                            decode_word2(w, codes);
                        }
                        if (Wc) store_canonical_block(Wc, bits, L.K, n, kb, codes);
                        if (We) We[n * nblk + kb] = L.w_exp_bias >= 0
                                ? (uint8_t)(((rec[lane * 4 + c] >> (4 * j)) & 0xF) + L.w_exp_bias)
                                : rec[exp_off + lane * 8 + 2 * c + j];
                    }
            }
        }
    });
}

// bf16 bit pattern of code * 2^(eb - 127 - 6): exact (7 significand bits), computed through fp32
static uint16_t a_value_bf16(int code, int eb) {
    const float v = std::ldexp((float)code, eb - 127 - 6);
    uint32_t bits;
    memcpy(&bits, &v, 4);
    return (uint16_t)(bits >> 16);
}

// canonical Ac/Ae -> records of exact bf16 values in the MFMA operand order of the projection kernel
static int tile_a(const Layer& L, const int8_t* Ac, const uint8_t* Ae, std::vector<uint8_t>& out) {
    const int64_t nblk = L.K / 16;
    out.assign((size_t)(L.kp16 * L.KT) * kARecordBytes, 0);
    for (int64_t i = 0; i < (int64_t)L.kp * nblk; ++i)
        if (Ae[i] == 255) return LQER_ERR_VALUE;
    for (int g = 0; g < L.kp16; ++g)
        for (int64_t tile = 0; tile < L.KT; ++tile) {
            uint8_t* rec = out.data() + (size_t)(g * L.KT + tile) * kARecordBytes;
            for (int lane = 0; lane < 64; ++lane) {
                const int c = lane & 15, q = lane >> 4;
                const int64_t r = g * 16 + c;
                for (int p = 0; p < 4; ++p) {
                    const int64_t kb = tile * 16 + q + 4 * p;
                    if (kb >= nblk) continue;
                    const int eb = Ae[r * nblk + kb];
                    for (int h = 0; h < 2; ++h) {
                        uint16_t v[8];
                        for (int i = 0; i < 8; ++i) v[i] = a_value_bf16(Ac[r * L.K + kb * 16 + 8 * h + i], eb);
                        memcpy(rec + (2 * p + h) * 1024 + lane * 16, v, 16);
                    }
                }
            }
        }
    return LQER_OK;
}

// inverse, given the exponent bytes (kept on the host: a block's exponent is not recoverable from
// its values when the largest code is below 64)
static void untile_a(const Layer& L, const std::vector<uint8_t>& in, const std::vector<uint8_t>& Ae_host,
                     int8_t* Ac, uint8_t* Ae) {
    const int64_t nblk = L.K / 16;
    if (Ae) memcpy(Ae, Ae_host.data(), Ae_host.size());
    if (!Ac) return;
    for (int g = 0; g < L.kp16; ++g)
        for (int64_t tile = 0; tile < L.KT; ++tile) {
            const uint8_t* rec = in.data() + (size_t)(g * L.KT + tile) * kARecordBytes;
            for (int lane = 0; lane < 64; ++lane) {
                const int c = lane & 15, q = lane >> 4;
                const int64_t r = g * 16 + c;
                for (int p = 0; p < 4; ++p) {
                    const int64_t kb = tile * 16 + q + 4 * p;
                    if (kb >= nblk) continue;
                    const int eb = Ae_host[r * nblk + kb];
                    for (int h = 0; h < 2; ++h) {
                        uint16_t v[8];
                        memcpy(v, rec + (2 * p + h) * 1024 + lane * 16, 16);
                        for (int i = 0; i < 8; ++i) {
                            const uint32_t bits = (uint32_t)v[i] << 16;
                            float f;
                            memcpy(&f, &bits, 4);
                            Ac[r * L.K + kb * 16 + 8 * h + i] = (int8_t)std::lrint(std::ldexp(f, 6 - (eb - 127)));
                        }
                    }
                }
            }
        }
}

int tile_b(const Layer& L, const int8_t* Bc, const uint8_t* Be, std::vector<uint8_t>& out) {
    out.assign((size_t)(L.N32 * L.kp16) * kBRecordBytes, 0);
    for (int64_t i = 0; Be && i < L.N * L.kp16; ++i)
        if (Be[i] == 255) return LQER_ERR_VALUE;
    for (int64_t g = 0; g < L.N32; ++g)
        for (int rb = 0; rb < L.kp16; ++rb) {
            uint8_t* rec = out.data() + (size_t)(g * L.kp16 + rb) * kBRecordBytes;
            for (int c = 0; c < 32; ++c) {
                const int64_t n = g * 32 + c;
                if (n >= L.N) continue;
                memcpy(rec + c * 16, Bc + n * L.kp + rb * 16, 16);
                rec[512 + c] = Be ? Be[n * L.kp16 + rb] : 0;
            }
        }
    return LQER_OK;
}

static void untile_b(const Layer& L, const std::vector<uint8_t>& in, int8_t* Bc, uint8_t* Be) {
    for (int64_t g = 0; g < L.N32; ++g)
        for (int rb = 0; rb < L.kp16; ++rb) {
            const uint8_t* rec = in.data() + (size_t)(g * L.kp16 + rb) * kBRecordBytes;
            for (int c = 0; c < 32; ++c) {
                const int64_t n = g * 32 + c;
                if (n >= L.N) continue;
                if (Bc) memcpy(Bc + n * L.kp + rb * 16, rec + c * 16, 16);
                if (Be) Be[n * L.kp16 + rb] = rec[512 + c];
            }
        }
}

void free_device(Layer& L) {
    if (L.Wt) (void)hipFree(L.Wt);
    if (L.At) (void)hipFree(L.At);
    if (L.Bt) (void)hipFree(L.Bt);
    if (L.Wsc) (void)hipFree(L.Wsc);
    if (L.Asc) (void)hipFree(L.Asc);
    if (L.Bsc) (void)hipFree(L.Bsc);
    L.Wt = L.At = L.Bt = nullptr;
    L.Wsc = L.Asc = L.Bsc = nullptr;
}

int upload(const std::vector<uint8_t>& host, uint8_t** dev) {
    *dev = nullptr;
    if (host.empty()) return LQER_OK;
    if (hipMalloc((void**)dev, host.size()) != hipSuccess) return LQER_ERR_HIP;
    if (hipMemcpy(*dev, host.data(), host.size(), hipMemcpyHostToDevice) != hipSuccess) return LQER_ERR_HIP;
    return LQER_OK;
}

static int download(const uint8_t* dev, size_t bytes, std::vector<uint8_t>& host) {
    host.resize(bytes);
    if (bytes == 0) return LQER_OK;
    if (hipMemcpy(host.data(), dev, bytes, hipMemcpyDeviceToHost) != hipSuccess) return LQER_ERR_HIP;
    return LQER_OK;
}

// path 1 = streaming kernel (activations as 16-byte cells, T as partial sums), 2 = tiled
// with_slots = false leaves out the slots of the tiled kernel's work split (it then never cuts tiles)
static Workspace plan_workspace(const Layer& L, int64_t M, int path, void* base, bool with_slots = true) {
    Workspace ws;
    ws.ldxh = L.KT * kTileK + round_up(2 * (int64_t)L.kp, 64);
    ws.S = prep_slices(L, M, path);
    ws.cells = (path == 1);
    ws.lr = stream_cell_rows_log2(M);
    ws.x8 = false;
    // the tiled kernel reads whole tiles of Xh, 96 to 256 rows high (rows past M hold whatever was there)
    const int64_t xh_rows = (path == 2) ? round_up(M + 95, 256) : (ws.cells ? (int64_t)1 << ws.lr : M);
    const size_t xh_bytes = (size_t)round_up(xh_rows * ws.ldxh * 2, 256);
    // T travels as partial sums on the streaming path and whenever the projection kernel splits K
    const bool partial = L.kp > 0 && (path == 1 || ws.S > 1);
    ws.tp_rows = (path == 2) ? xh_rows : M;
    const size_t tp_bytes = partial ? (size_t)round_up((int64_t)ws.S * ws.tp_rows * L.kp * 4, 256) : 0;
    ws.Xh = (uint16_t*)base;
    ws.Tpart = partial ? (float*)((uint8_t*)base + xh_bytes) : nullptr;
    ws.bytes = xh_bytes + tp_bytes;
    // tiled path: slots for accumulators handed between workgroups, and their flags
    ws.Part = nullptr;
    ws.flags = nullptr;
    if (path == 2) {
        ws.flags = (uint32_t*)((uint8_t*)base + ws.bytes);
        ws.bytes += (size_t)kTiledFlags * 4;
        if (with_slots) {
            ws.Part = (float*)((uint8_t*)base + ws.bytes);
            ws.bytes += (size_t)(kTiledPartBytesPerCu * compute_units());
        }
    }
    return ws;
}

static int pick_path(const Layer& L, int64_t M) {
    if (L.format == 1) return 3;                     // the scaled-integer variant has one kernel for every token count
    // The streaming kernel takes up to 32 tokens for any layer, and up to 64 (two blocks of 32 per
    // wavefront) for layers wide enough to fill the chip with four column groups per workgroup.
    if (M <= 32) return 1;
    // (with ranks above 64 the T rows of 64 tokens do not fit the streaming kernel's LDS)
    if (M <= stream_max_rows() && L.N32 >= 512 && L.kp <= 64) return 1;
    return 2;
}

static int forward_impl(const lqer_layer* layer, const float* X, int64_t ldx, const int8_t* Xc,
                        const uint8_t* Xe, int64_t M, float* Y, int64_t ldy, void* wsp, size_t ws_bytes,
                        void* stream, const lqer_launch_opts* opts, const Requant& rq = Requant{nullptr, nullptr, 0},
                        bool with_slots = true) {
    if (!layer) return LQER_ERR_NULL;
    const Layer& L = layer->L;
    if (M < 0) return LQER_ERR_SHAPE;
    if (L.format == 1) {
        // the scaled-integer variant: fp32 in, fp32 out, one launch shape
        if (Xc || rq.codes || (opts && (opts->path != 0 || opts->variant != 0 || opts->stages != 0))) return LQER_ERR_UNSUPPORTED;
        if (M == 0) return LQER_OK;
        if (!X || !Y) return LQER_ERR_NULL;
        if (ldx < L.K || (ldx & 3) != 0 || ((uintptr_t)X & 15) != 0) return LQER_ERR_SHAPE;
        if (ldy < L.N || (ldy & 3) != 0 || ((uintptr_t)Y & 15) != 0) return LQER_ERR_SHAPE;
        if (!wsp || ((uintptr_t)wsp & 255) != 0) return LQER_ERR_WORKSPACE;
        return forward_int(L, X, ldx, M, Y, ldy, wsp, ws_bytes, (hipStream_t)stream);
    }
    if (M == 0) return LQER_OK;
    const bool requant = rq.codes != nullptr;
    if (requant) {
        // Y leaves as MXINT8 with blocks of 16 along N: the next layer's contraction axis
        if (!rq.exps) return LQER_ERR_NULL;
        if ((L.N & 15) != 0 || rq.ld < L.N || (rq.ld & 3) != 0 || ((uintptr_t)rq.codes & 3) != 0) return LQER_ERR_SHAPE;
        ldy = L.N;                                   // no fp32 Y: keep the checks below quiet
    } else if (!Y) {
        return LQER_ERR_NULL;
    }
    if (Xc) {
        if (!Xe) return LQER_ERR_NULL;
        if (((uintptr_t)Xc & 15) != 0) return LQER_ERR_SHAPE;
    } else {
        if (!X) return LQER_ERR_NULL;
        if (ldx < L.K || (ldx & 3) != 0 || ((uintptr_t)X & 15) != 0) return LQER_ERR_SHAPE;
    }
    if (!requant && (ldy < L.N || (ldy & 3) != 0 || ((uintptr_t)Y & 15) != 0)) return LQER_ERR_SHAPE;
    int path = opts ? opts->path : 0;
    int variant = opts ? opts->variant : 0;
    int stages = opts ? opts->stages : 0;
    if (path < 0 || path > 2 || (stages & ~3) != 0) return LQER_ERR_SHAPE;
    if (path == 0) path = pick_path(L, M);
    if (path == 1 && M > stream_max_rows()) return LQER_ERR_SHAPE;
    // a pair of workgroups completes its sum only in memory: with MXINT8 output take the unpaired shape
    if (requant && path == 1 && variant == 0 && stream_variant_adds_into_y(stream_variant(L, M, 0)))
        variant = stream_variant_unpaired(L, M);
    if (stages == 0) stages = 3;
    if (!wsp || ((uintptr_t)wsp & 255) != 0) return LQER_ERR_WORKSPACE;
    Workspace ws = plan_workspace(L, M, path, wsp, with_slots);
    if (ws.bytes > ws_bytes) return LQER_ERR_WORKSPACE;
    if (path == 1) ws.x8 = stream_takes_codes(stream_variant(L, M, variant), ws.lr);
    hipStream_t s = (hipStream_t)stream;
    if (stages & 1) {
        const bool zero_y = (path == 1) && stream_variant_adds_into_y(stream_variant(L, M, variant));
        if (launch_prep(L, X, ldx, Xc, Xe, M, ws, zero_y ? Y : nullptr, ldy, s) != hipSuccess) return LQER_ERR_HIP;
    }
    if (stages & 2) {
        if (!(stages & 1) && path == 2 && launch_clear_flags(ws, s) != hipSuccess) return LQER_ERR_HIP;
        const hipError_t e = (path == 1) ? launch_stream(L, M, ws, Y, ldy, rq, variant, s)
                                         : launch_tiled(L, M, ws, Y, ldy, rq, variant, s);
        if (e == hipErrorInvalidValue) return LQER_ERR_SHAPE;
        if (e != hipSuccess) return LQER_ERR_HIP;
    }
    return LQER_OK;
}

// One workspace plan that serves every layer of a group applied to the same activations on the tiled path:
// the plan of a layer with the group's K and its widest padded rank.
static Layer shared_plan_layer(const lqer_layer* const* layers, int n) {
    Layer Lp = layers[0]->L;
    for (int i = 1; i < n; ++i)
        if (layers[i]->L.kp > Lp.kp) { Lp.kp = layers[i]->L.kp; Lp.kp16 = layers[i]->L.kp16; }
    return Lp;
}

static bool shared_group_ok(const lqer_layer* const* layers, int n) {
    if (!layers || n < 1) return false;
    for (int i = 0; i < n; ++i) {
        if (!layers[i] || layers[i]->L.format != 0) return false;
        if (layers[i]->L.K != layers[0]->L.K || layers[i]->L.act_bits != layers[0]->L.act_bits) return false;
    }
    return true;
}

static bool shared_group_tiled(const lqer_layer* const* layers, int n, int64_t M) {
    for (int i = 0; i < n; ++i)
        if (pick_path(layers[i]->L, M) != 2) return false;
    return true;
}

int forward_in_scratch(const lqer_layer* layer, const float* X, int64_t M, int64_t ldx, float* Y, int64_t ldy,
                       void* scratch, size_t scratch_bytes, void* stream) {
    return forward_impl(layer, X, ldx, nullptr, nullptr, M, Y, ldy, scratch, scratch_bytes, stream, nullptr,
                        Requant{nullptr, nullptr, 0}, false);
}

}  // namespace lqer

using namespace lqer;

extern "C" {

const char* lqer_status_string(int status) {
    switch (status) {
        case LQER_OK: return "ok";
        case LQER_ERR_NULL: return "null pointer";
        case LQER_ERR_SHAPE: return "bad shape, stride or alignment";
        case LQER_ERR_UNSUPPORTED: return "unsupported format";
        case LQER_ERR_SINGULAR_SCALE: return "singular activation scale";
        case LQER_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LQER_ERR_HIP: return "HIP runtime error";
        case LQER_ERR_NO_CONVERGENCE: return "truncated SVD did not converge";
        case LQER_ERR_VALUE: return "packed bytes hold an excluded value";
        case LQER_ERR_NO_MEMORY: return "host allocation failed";
        default: return "unknown status";
    }
}

int lqer_quantize_mx(const float* x_dev, int64_t rows, int64_t cols, int64_t ld, int elem_bits,
                     int exp_bits, void* codes_dev, uint8_t* exps_dev, void* hip_stream) {
    if (elem_bits != 4 && elem_bits != 6 && elem_bits != 8) return LQER_ERR_UNSUPPORTED;
    if (exp_bits != 8) return LQER_ERR_UNSUPPORTED;
    if (rows < 0 || cols < 0 || (cols & 15) != 0 || ld < cols) return LQER_ERR_SHAPE;
    if (rows == 0 || cols == 0) return LQER_OK;
    if (!x_dev || !codes_dev || !exps_dev) return LQER_ERR_NULL;
    if ((ld & 3) != 0 || ((uintptr_t)x_dev & 15) != 0 || ((uintptr_t)codes_dev & 3) != 0) return LQER_ERR_SHAPE;
    if (launch_quantize_mx(x_dev, rows, cols, ld, elem_bits, codes_dev, exps_dev, (hipStream_t)hip_stream) !=
        hipSuccess)
        return LQER_ERR_HIP;
    return LQER_OK;
}

int lqer_layer_import(int64_t K, int64_t N, int k, const uint8_t* Wc, const uint8_t* We, const int8_t* Ac,
                      const uint8_t* Ae, const int8_t* Bc, const uint8_t* Be, lqer_layer** out) {
    return lqer_layer_import_w(4, K, N, k, Wc, We, Ac, Ae, Bc, Be, out);
}

int lqer_layer_weight_bits(const lqer_layer* layer) { return layer ? layer->L.w_bits : 0; }

int lqer_layer_import_w(int w_bits, int64_t K, int64_t N, int k, const uint8_t* Wc, const uint8_t* We, const int8_t* Ac,
                        const uint8_t* Ae, const int8_t* Bc, const uint8_t* Be, lqer_layer** out) {
    if (!out) return LQER_ERR_NULL;
    *out = nullptr;
    if (w_bits != 4 && w_bits != 2) return LQER_ERR_UNSUPPORTED;
    if (K <= 0 || N <= 0 || (K & 15) != 0 || k < 0 || k > K || k > N) return LQER_ERR_SHAPE;
    if (!Wc || !We) return LQER_ERR_NULL;
    if (k > 0 && (!Ac || !Ae || !Bc || !Be)) return LQER_ERR_NULL;
    const int kp = (k + 15) / 16 * 16;
    if (kp > kMaxRank) return LQER_ERR_UNSUPPORTED;
    lqer_layer* h = new (std::nothrow) lqer_layer;
    if (!h) return LQER_ERR_NO_MEMORY;
    Layer& L = h->L;
    L.K = K; L.N = N; L.k = k; L.kp = kp;
    L.KT = (K + kTileK - 1) / kTileK;
    L.N32 = (N + 31) / 32;
    L.kp16 = kp / 16;
    L.act_bits = 8;
    L.format = 0; L.kp32 = 0;
    L.Wsc = L.Asc = L.Bsc = nullptr;
    L.w_bits = w_bits;
    L.w_rec_bytes = w_record_bytes(w_bits, false);
    L.w_exp_bias = -1;
    L.Wt = L.At = L.Bt = nullptr;
    if (hipGetDevice(&L.device) != hipSuccess) { delete h; return LQER_ERR_HIP; }
    int st;
    try {
        {
            std::vector<uint8_t> buf;
            st = tile_weights(L, Wc, We, buf);
            if (st == LQER_OK) st = upload(buf, &L.Wt);
        }
        if (st == LQER_OK && kp > 0) {
            std::vector<uint8_t> buf;
            st = tile_a(L, Ac, Ae, buf);
            if (st == LQER_OK) st = upload(buf, &L.At);
            if (st == LQER_OK) h->Ae_host.assign(Ae, Ae + (size_t)kp * (K / 16));
        }
        if (st == LQER_OK && kp > 0) {
            std::vector<uint8_t> buf;
            st = tile_b(L, Bc, Be, buf);
            if (st == LQER_OK) st = upload(buf, &L.Bt);
        }
    } catch (...) {                                  // a host allocation failed: nothing may leave through the C ABI
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

int lqer_layer_export(const lqer_layer* layer, uint8_t* Wc, uint8_t* We, int8_t* Ac, uint8_t* Ae, int8_t* Bc,
                      uint8_t* Be) {
    if (!layer) return LQER_ERR_NULL;
    const Layer& L = layer->L;
    if (L.format != 0) return LQER_ERR_UNSUPPORTED;  // lqer_int_layer_export is the call for that format
    try {
    std::vector<uint8_t> buf;
    int st;
    if (Wc || We) {
        st = download(L.Wt, (size_t)(L.N32 * L.KT) * L.w_rec_bytes, buf);
        if (st != LQER_OK) return st;
        untile_weights(L, buf, Wc, We);
    }
    if (L.kp > 0 && (Ac || Ae)) {
        st = download(L.At, (size_t)(L.kp16 * L.KT) * kARecordBytes, buf);
        if (st != LQER_OK) return st;
        untile_a(L, buf, layer->Ae_host, Ac, Ae);
    }
    if (L.kp > 0 && (Bc || Be)) {
        st = download(L.Bt, (size_t)(L.N32 * L.kp16) * kBRecordBytes, buf);
        if (st != LQER_OK) return st;
        untile_b(L, buf, Bc, Be);
    }
    return LQER_OK;
    } catch (...) {                                  // a host allocation failed
        return LQER_ERR_NO_MEMORY;
    }
}

int lqer_layer_dims(const lqer_layer* layer, int64_t* K, int64_t* N, int* k, int* kp) {
    if (!layer) return LQER_ERR_NULL;
    if (K) *K = layer->L.K;
    if (N) *N = layer->L.N;
    if (k) *k = layer->L.k;
    if (kp) *kp = layer->L.kp;
    return LQER_OK;
}

int lqer_layer_set_activation_bits(lqer_layer* layer, int bits) {
    if (!layer) return LQER_ERR_NULL;
    if ((bits != 8 && bits != 6) || layer->L.format != 0) return LQER_ERR_UNSUPPORTED;
    layer->L.act_bits = bits;
    return LQER_OK;
}

int lqer_layer_free(lqer_layer* layer) {
    if (!layer) return LQER_OK;
    free_device(layer->L);
    delete layer;
    return LQER_OK;
}

size_t lqer_linear_workspace_bytes_ex(const lqer_layer* layer, int64_t M, int path) {
    if (!layer || M <= 0 || path < 0 || path > 2) return 0;
    const Layer& L = layer->L;
    if (L.format == 1) return path == 0 ? int_workspace_bytes(L, M) : 0;
    if (path == 0) path = pick_path(L, M);
    if (path == 1 && M > stream_max_rows()) return 0;
    return plan_workspace(L, M, path, nullptr).bytes;
}

size_t lqer_linear_workspace_bytes(const lqer_layer* layer, int64_t M) {
    return lqer_linear_workspace_bytes_ex(layer, M, 0);
}

int lqer_linear_forward_requant(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx,
                                int8_t* Yc_dev, int64_t ldyc, uint8_t* Ye_dev, void* workspace_dev,
                                size_t workspace_bytes, void* hip_stream, const lqer_launch_opts* opts) {
    if (!Yc_dev) return LQER_ERR_NULL;
    return forward_impl(layer, X_dev, ldx, nullptr, nullptr, M, nullptr, 0, workspace_dev, workspace_bytes,
                        hip_stream, opts, Requant{Yc_dev, Ye_dev, ldyc});
}

size_t lqer_linear_shared_workspace_bytes(const lqer_layer* const* layers, int n_layers, int64_t M) {
    if (!shared_group_ok(layers, n_layers) || M <= 0) return 0;
    size_t need = 0;
    for (int i = 0; i < n_layers; ++i) {
        const size_t b = plan_workspace(layers[i]->L, M, pick_path(layers[i]->L, M), nullptr).bytes;
        if (b > need) need = b;
    }
    if (shared_group_tiled(layers, n_layers, M)) {
        const size_t b = plan_workspace(shared_plan_layer(layers, n_layers), M, 2, nullptr).bytes;
        if (b > need) need = b;
    }
    return need;
}

int lqer_linear_forward_shared(const lqer_layer* const* layers, int n_layers, const float* X_dev, int64_t M,
                               int64_t ldx, float* const* Y_dev, const int64_t* ldy, void* workspace_dev,
                               size_t workspace_bytes, void* hip_stream) {
    if (!layers || !Y_dev || !ldy || n_layers < 1) return LQER_ERR_NULL;
    for (int i = 0; i < n_layers; ++i)
        if (!layers[i] || !Y_dev[i]) return LQER_ERR_NULL;
    if (!shared_group_ok(layers, n_layers)) return LQER_ERR_SHAPE;
    if (M < 0) return LQER_ERR_SHAPE;
    if (M == 0) return LQER_OK;
    if (!X_dev) return LQER_ERR_NULL;
    const int64_t K = layers[0]->L.K;
    if (ldx < K || (ldx & 3) != 0 || ((uintptr_t)X_dev & 15) != 0) return LQER_ERR_SHAPE;
    for (int i = 0; i < n_layers; ++i)
        if (ldy[i] < layers[i]->L.N || (ldy[i] & 3) != 0 || ((uintptr_t)Y_dev[i] & 15) != 0) return LQER_ERR_SHAPE;
    if (!workspace_dev || ((uintptr_t)workspace_dev & 255) != 0) return LQER_ERR_WORKSPACE;
    if (workspace_bytes < lqer_linear_shared_workspace_bytes(layers, n_layers, M)) return LQER_ERR_WORKSPACE;
    if (!shared_group_tiled(layers, n_layers, M)) {
        // few tokens: the streaming path keeps its per-layer activation layouts; one full call per layer
        for (int i = 0; i < n_layers; ++i) {
            const int st = forward_impl(layers[i], X_dev, ldx, nullptr, nullptr, M, Y_dev[i], ldy[i], workspace_dev,
                                        workspace_bytes, hip_stream, nullptr);
            if (st != LQER_OK) return st;
        }
        return LQER_OK;
    }
    const Workspace ws = plan_workspace(shared_plan_layer(layers, n_layers), M, 2, workspace_dev);
    hipStream_t s = (hipStream_t)hip_stream;
    for (int i = 0; i < n_layers; ++i) {
        const Layer& L = layers[i]->L;
        hipError_t e;
        if (i == 0) e = launch_prep(L, X_dev, ldx, nullptr, nullptr, M, ws, nullptr, 0, s);
        else if (L.kp > 0) e = launch_prep(L, nullptr, 0, nullptr, nullptr, M, ws, nullptr, 0, s, true);
        else e = launch_clear_flags(ws, s);          // nothing to project; the main kernel still wants its flags cleared
        if (e != hipSuccess) return LQER_ERR_HIP;
        e = launch_tiled(L, M, ws, Y_dev[i], ldy[i], Requant{nullptr, nullptr, 0}, 0, s);
        if (e == hipErrorInvalidValue) return LQER_ERR_SHAPE;
        if (e != hipSuccess) return LQER_ERR_HIP;
    }
    return LQER_OK;
}

// Host-only check of the layout transforms (no device call): pseudo-random canonical bytes are tiled into the device
// records and untiled again for 4- and 2-bit weights, both exponent forms, ragged K, N and ranks; meant to be run in a
// build with host sanitizers.  Returns LQER_OK, or LQER_ERR_VALUE at the first difference.
int lqer_selftest_layouts(void) {
    try {
        uint64_t state = 0x243F6A8885A308D3ull;
        auto rnd = [&state]() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(state >> 33); };
        const int64_t shapes[][3] = {{16, 1, 0}, {48, 40, 8}, {272, 100, 33}, {1040, 65, 256}, {2304, 31, 64}};
        for (int bits = 2; bits <= 4; bits += 2)
            for (int wide = 0; wide < 2; ++wide)
                for (const auto& sh : shapes) {
                    Layer L{};
                    L.K = sh[0]; L.N = sh[1]; L.k = (int)std::min<int64_t>(sh[2], std::min(sh[0], sh[1]));
                    L.kp = (L.k + 15) / 16 * 16; L.kp16 = L.kp / 16;
                    L.KT = (L.K + kTileK - 1) / kTileK; L.N32 = (L.N + 31) / 32;
                    L.w_bits = bits;
                    const int64_t nblk = L.K / 16, wrow = L.K * bits / 8;
                    std::vector<uint8_t> Wc((size_t)L.N * wrow), We((size_t)L.N * nblk), Ae((size_t)L.kp * nblk), Be((size_t)L.N * L.kp16);
                    std::vector<int8_t> Ac((size_t)L.kp * L.K), Bc((size_t)L.N * L.kp);
                    for (auto& b : Wc) {
                        if (bits == 4) { const uint32_t lo = rnd() % 15, hi = rnd() % 15; b = (uint8_t)((lo >= 8 ? lo + 1 : lo) | ((hi >= 8 ? hi + 1 : hi) << 4)); }
                        else { b = 0; for (int j = 0; j < 4; ++j) { const uint32_t v = rnd() % 3; b = (uint8_t)(b | ((v == 2 ? 3u : v) << (2 * j))); } }
                    }
                    for (auto& e : We) e = (uint8_t)(wide ? rnd() % 246 : 110 + rnd() % 16);
                    for (auto& e : Ae) e = (uint8_t)(30 + rnd() % 220);    // (code * 2^(e-6) must be a normal bf16 number)
                    for (auto& e : Be) e = (uint8_t)(rnd() % 255);
                    for (auto& c : Ac) c = (int8_t)((int)(rnd() % 255) - 127);
                    for (auto& c : Bc) c = (int8_t)((int)(rnd() % 255) - 127);
                    std::vector<uint8_t> rec, Wc2(Wc.size()), We2(We.size());
                    if (tile_weights(L, Wc.data(), We.data(), rec) != LQER_OK) return LQER_ERR_VALUE;
                    if (L.N * nblk >= 256 && (L.w_exp_bias >= 0) != (wide == 0)) return LQER_ERR_VALUE;   // both exponent forms are exercised
                    rec.resize(rec.size() - kWTailPad);
                    untile_weights(L, rec, Wc2.data(), We2.data());
                    if (Wc2 != Wc || We2 != We) return LQER_ERR_VALUE;
                    if (L.kp > 0) {
                        std::vector<uint8_t> ra, rb, Ae2(Ae.size()), Be2(Be.size());
                        std::vector<int8_t> Ac2(Ac.size()), Bc2(Bc.size());
                        if (tile_a(L, Ac.data(), Ae.data(), ra) != LQER_OK || tile_b(L, Bc.data(), Be.data(), rb) != LQER_OK) return LQER_ERR_VALUE;
                        untile_a(L, ra, Ae, Ac2.data(), Ae2.data());
                        untile_b(L, rb, Bc2.data(), Be2.data());
                        if (Ac2 != Ac || Ae2 != Ae || Bc2 != Bc || Be2 != Be) return LQER_ERR_VALUE;
                    }
                }
        return LQER_OK;
    } catch (...) {
        return LQER_ERR_NO_MEMORY;
    }
}

int lqer_set_wait_limit(int polls) {
    if (polls < 0) return LQER_ERR_SHAPE;
    set_tiled_wait_limit(polls);
    return LQER_OK;
}

int lqer_linear_path(const lqer_layer* layer, int64_t M) {
    if (!layer) return 0;
    return pick_path(layer->L, M);
}

int lqer_linear_forward(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx, float* Y_dev,
                        int64_t ldy, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    return forward_impl(layer, X_dev, ldx, nullptr, nullptr, M, Y_dev, ldy, workspace_dev, workspace_bytes,
                        hip_stream, nullptr);
}

int lqer_linear_forward_q(const lqer_layer* layer, const int8_t* Xc_dev, const uint8_t* Xe_dev, int64_t M,
                          float* Y_dev, int64_t ldy, void* workspace_dev, size_t workspace_bytes,
                          void* hip_stream) {
    if (!Xc_dev) return LQER_ERR_NULL;
    return forward_impl(layer, nullptr, 0, Xc_dev, Xe_dev, M, Y_dev, ldy, workspace_dev, workspace_bytes,
                        hip_stream, nullptr);
}

int lqer_linear_forward_ex(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx, float* Y_dev,
                           int64_t ldy, void* workspace_dev, size_t workspace_bytes, void* hip_stream,
                           const lqer_launch_opts* opts) {
    return forward_impl(layer, X_dev, ldx, nullptr, nullptr, M, Y_dev, ldy, workspace_dev, workspace_bytes,
                        hip_stream, opts);
}

}  // extern "C"
