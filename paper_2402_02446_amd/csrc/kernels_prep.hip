// Stage 1 of the forward pass: quantize activations to MXINT8 (Sec. 4.1, block [1,16]; MXINT6 for the
// W4A6 setup of Table 2) and compute the low-rank projection T = X_q A_k (Eq. 3 / Eq. 6, first small
// matmul).
//
// One workgroup owns 16 token rows and a K slice; its eight wavefronts take the slice's 256-wide
// K tiles in turn.  Lane (t = lane % 16, q = lane / 16) owns the blocks q + 4p (p = 0..3) of a
// tile for token t: it finds the block maximum, quantizes, and keeps the dequantized values
// code * 2^(e-6) - exact in bf16 - both for the store to the bf16 activation matrix the main
// kernels read and as its MFMA operand.  A_k arrives already dequantized to bf16 (exactly, at
// import), so every product entering the fp32 MFMA accumulator is exact.
//
// S == 1: T is final; it is split into two bf16 terms T_hi + T_lo and stored behind the
//         activations of the same row, where the main kernel treats it as 2*kp more K columns.
// S  > 1: each K slice stores an fp32 partial T; the main kernel adds the slices in a fixed order.
// For the streaming kernel the activations are stored as 16-byte cells [K / 8][token row] instead
// (or as the codes themselves, see the store below); extra workgroups clear Y or the tiled
// kernel's flags where the main kernel needs that.
#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

struct PrepArgs {
    const float* X; int64_t ldx;
    const int8_t* Xc; const uint8_t* Xe;
    int64_t M, K;
    int64_t KT;            // K tiles
    int tiles_per_slice;
    int kp, kp16;
    int groups_per_wg;     // rank groups one plane of grid.z computes: at most 4 (the last plane may have fewer)
    int g_first;           // first rank group of plane 0
    const uint8_t* At;
    uint16_t* Xh; int64_t ldxh;
    int64_t tail_cols;     // columns behind K_pad in Xh (T_hi | T_lo | zero padding)
    float* Tpart;
    int64_t tp_rows;       // rows per slice of Tpart
    int lr;                // CELLS: log2 of the token rows per 16-byte cell column
    int act_frac;          // fraction bits of the activation codes: 6 (MXINT8) or 4 (MXINT6)
    bool x8;               // CELLS: store MXINT8 codes [block][row][16] and exponent bytes [block][row] instead of bf16 cells
    float* Yz; int64_t ldy, N;   // Yz != null: extra workgroups clear Y[M][N] for a main kernel that adds into it
    int nslices;                 // K slices = the part of grid.y that does the projection
    uint32_t* flags; int nflags; // flags != null: words the first workgroup clears for the main kernel
};

__device__ __forceinline__ void split_bf16(float t, uint16_t& hi, uint16_t& lo) {
    const uint32_t hb = f32_bits(t) & 0xFFFF0000u;
    hi = (uint16_t)(hb >> 16);
    const float rem = t - f32_from_bits(hb);              // exact
    lo = (uint16_t)(f32_bits(rem) >> 16);
}

constexpr int kPrepWaves = 8;

// CELLS: the activations are stored for the streaming kernel, as 16-byte cells (8 consecutive K
// elements) ordered [K / 8][token row]; otherwise row-major for the tiled kernel.
// SRC: where the activations come from: 0 = fp32 X (quantized here), 1 = MXINT codes and exponent bytes,
// 2 = the bf16 matrix an earlier launch on the same X left in the workspace (nothing is stored again: only T
// is computed, for another layer applied to the same activations).
template <int CTRL>
__device__ __forceinline__ float dpp_quad(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <int SRC, bool FINAL, int MAXG, bool CELLS, bool RW = false>
__global__ __launch_bounds__(64 * kPrepWaves, RW ? 4 : 1) void prep_kernel(PrepArgs a) {
    static_assert(!RW || (SRC == 0 && !CELLS), "the row-wise form reads fp32 rows and writes row-major bf16");
    // ROWWISE (fp32 X in, row-major bf16 out: the prefill case, bound by HBM): a wavefront reads and writes whole rows
    // of its 16 x 256 tile - 1 KiB per load, 512 B per store, every cache line touched by one instruction - with the
    // four lanes of a quad sharing a block, and turns the tile into the MFMA operand order (lane = token, 16-byte
    // runs of one block) through 8 KB of LDS of its own; the sums of T go through the same memory afterwards.
    // Chosen by the launcher for launches of many workgroups; with few (prefill calls of a few thousand tokens, where K
    // is split over workgroups) the longer chain load - quantize - LDS - MFMA per tile and the two workgroups per
    // compute unit cost more than the coalescing gains (measured: 8192 wide, 4096 tokens 46 -> 52 us; 65536 tokens of
    // 4096 channels 373 -> 308 us), and the lane-per-block form below is used.
    constexpr bool ROWWISE = RW;
    constexpr int RED_BYTES = kPrepWaves * MAXG * 64 * 16;
    constexpr int SMEM_BYTES = ROWWISE ? (kPrepWaves * 8192 > RED_BYTES ? kPrepWaves * 8192 : RED_BYTES) : RED_BYTES;
    __shared__ __attribute__((aligned(16))) uint8_t smem[SMEM_BYTES];
    float (*red)[MAXG][64][4] = reinterpret_cast<float (*)[MAXG][64][4]>(smem);

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;              // 1 .. kPrepWaves
    const int t = lane & 15, q = lane >> 4;
    const int64_t row = (int64_t)blockIdx.x * 16 + t;
    const bool row_ok = row < a.M;
    const int slice = blockIdx.y;
    const int g0 = a.g_first + blockIdx.z * a.groups_per_wg;
    const int ng = (a.kp16 - g0 < a.groups_per_wg) ? a.kp16 - g0 : a.groups_per_wg;   // rank groups of this plane
    const bool store_x = (blockIdx.z == 0) && SRC != 2;
    const int64_t nblk = a.K / 16;

    f32x4 acc[MAXG];
#pragma unroll
    for (int g = 0; g < MAXG; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (a.flags != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
        for (int i = threadIdx.x; i < a.nflags; i += blockDim.x) a.flags[i] = 0u;

    // Workgroups behind the a.nslices K slices (grid.y) only clear Y for a main kernel that adds into it,
    // so the clearing runs beside the projection instead of in front of it.
    if ((int)blockIdx.y >= a.nslices) {
        if (blockIdx.z != 0) return;                 // one plane of grid.z clears
        const int64_t n4 = (a.N + 3) / 4;
        const int64_t nthreads = (int64_t)gridDim.x * (gridDim.y - a.nslices) * blockDim.x;
        const int64_t me = ((int64_t)(blockIdx.y - a.nslices) * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
        for (int64_t i = me; i < a.M * n4; i += nthreads) {
            const int64_t r = i / n4, c = 4 * (i - r * n4);
            float* dst = a.Yz + r * a.ldy + c;
            if (c + 3 < a.N) {
                *reinterpret_cast<f32x4*>(dst) = f32x4{0.f, 0.f, 0.f, 0.f};
            } else {
                for (int64_t j = c; j < a.N; ++j) a.Yz[r * a.ldy + j] = 0.f;
            }
        }
        return;
    }

    const int64_t tile_begin = (int64_t)slice * a.tiles_per_slice;
    int64_t tile_end = tile_begin + a.tiles_per_slice;
    if (tile_end > a.KT) tile_end = a.KT;

    for (int64_t tile = tile_begin + wave; tile < tile_end; tile += nwaves) {
        Frag xf[4][2];                                       // [p][half]
        // Few-token calls are bound by latency, not bandwidth: request A_k's records before the
        // activations are even loaded, so that one memory round trip covers both.
        Frag apre[CELLS ? MAXG : 1][4][2];
        if constexpr (CELLS) {
#pragma unroll
            for (int g = 0; g < MAXG; ++g) {
                if (g < ng) {
                    const uint8_t* rec = a.At + ((int64_t)(g0 + g) * a.KT + tile) * kARecordBytes;
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        apre[g][p][0].u = *reinterpret_cast<const u32x4*>(rec + (2 * p) * 1024 + lane * 16);
                        apre[g][p][1].u = *reinterpret_cast<const u32x4*>(rec + (2 * p + 1) * 1024 + lane * 16);
                    }
                }
            }
        }
        if constexpr (ROWWISE) {
            uint8_t* tl = smem + wave * 8192;                 // [16 rows][32 cells of 16 B], cell index XOR row
            const int64_t col = tile * kTileK + 4 * lane;     // this lane's four columns (K is a multiple of 16: all in or all out)
            const bool col_ok = col < a.K;
            // four batches of four rows: the next batch's loads are on their way while one is quantized.  Rows past M
            // repeat the last one (their stores are skipped); columns past K are zeroed after the load.
            const int64_t row0 = (int64_t)blockIdx.x * 16;
            const int64_t last = a.M - 1 - row0;              // >= 0: the grid covers M
            const int64_t ccol = col_ok ? col : 0;
            const float* xsrc = a.X + row0 * a.ldx + ccol;
            uint16_t* xdst = a.Xh + row0 * a.ldxh + col;
            const float keep = col_ok ? 1.0f : 0.0f;
            auto load_rows = [&](f32x4 (&v)[4], int i0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t r = (i0 + i) <= last ? (i0 + i) : last;
                    v[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xsrc + r * a.ldx));
                }
            };
            const float lim = (float)((2 << a.act_frac) - 1);
            auto quantize_rows = [&](const f32x4 (&v)[4], int i0) {
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    const int i = i0 + ii;
                    const f32x4 x = v[ii] * keep;
                    float m = __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(x[0]), __builtin_fabsf(x[1])),
                                              __builtin_fmaxf(__builtin_fabsf(x[2]), __builtin_fabsf(x[3])));
                    m = __builtin_fmaxf(m, dpp_quad<0xB1>(m));    // quad_perm [1,0,3,2]
                    m = __builtin_fmaxf(m, dpp_quad<0x4E>(m));    // quad_perm [2,3,0,1]
                    const uint32_t eb = (f32_bits(m) >> 23) & 0xFFu;
                    const int sh = a.act_frac - ((int)eb - 127);
                    const float scale = x_scale(eb, a.act_frac);
                    float c[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float r = __builtin_rintf(__builtin_amdgcn_ldexpf(x[j], sh));
                        c[j] = __builtin_fminf(__builtin_fmaxf(r, -lim), lim) * scale;
                    }
                    const u32x2 w = u32x2{pack_bf16_exact(c[0], c[1]), pack_bf16_exact(c[2], c[3])};
                    // columns between K and the end of the last tile are written as zeros: the main kernel reads whole tiles
                    if (store_x && i <= last) *reinterpret_cast<u32x2*>(xdst + i * a.ldxh) = w;
                    *reinterpret_cast<u32x2*>(tl + i * 512 + (((lane >> 1) ^ i) << 4) + (lane & 1) * 8) = w;
                }
            };
            f32x4 va[4], vb[4];
            load_rows(va, 0);
            load_rows(vb, 4);
            __builtin_amdgcn_wave_barrier();                  // the previous tile's operand reads are issued before these writes
            quantize_rows(va, 0);
            load_rows(va, 8);
            quantize_rows(vb, 4);
            load_rows(vb, 12);
            quantize_rows(va, 8);
            quantize_rows(vb, 12);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    xf[p][h].u = *reinterpret_cast<const u32x4*>(tl + t * 512 + (((2 * (q + 4 * p) + h) ^ t) << 4));
        }
#pragma unroll
        for (int p = 0; p < (ROWWISE ? 0 : 4); ++p) {
            const int64_t kb = tile * 16 + q + 4 * p;        // block index along K
            const bool ok = row_ok && kb < nblk;
            float scale = 0.f;
            float r[16];
            u32x4 cw = u32x4{0, 0, 0, 0};                     // the block's 16 codes as bytes (FROM_CODES, or CELLS of 16+ rows)
            uint32_t eb = 0;
            if constexpr (SRC == 2) {
                static_assert(SRC != 2 || !CELLS, "the stored matrix is read back in its row-major form only");
                const uint16_t* src = a.Xh + row * a.ldxh + kb * 16;
                xf[p][0].u = ok ? *reinterpret_cast<const u32x4*>(src) : u32x4{0, 0, 0, 0};
                xf[p][1].u = ok ? *reinterpret_cast<const u32x4*>(src + 8) : u32x4{0, 0, 0, 0};
            } else if constexpr (SRC == 1) {
                if (ok) {
                    cw = *reinterpret_cast<const u32x4*>(a.Xc + row * a.K + kb * 16);
                    eb = a.Xe[row * nblk + kb];
                }
                scale = x_scale(eb, a.act_frac);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = cw[i];
                    r[4 * i + 0] = (float)(int)(int8_t)(w & 0xFF);
                    r[4 * i + 1] = (float)(int)(int8_t)((w >> 8) & 0xFF);
                    r[4 * i + 2] = (float)(int)(int8_t)((w >> 16) & 0xFF);
                    r[4 * i + 3] = (float)(int)(int8_t)(w >> 24);
                }
            } else {
                float4 v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    v[i] = ok ? *reinterpret_cast<const float4*>(a.X + row * a.ldx + kb * 16 + 4 * i)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
                float m = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(v[i].x), __builtin_fabsf(v[i].y)),
                                                           __builtin_fmaxf(__builtin_fabsf(v[i].z), __builtin_fabsf(v[i].w))));
                }
                eb = (f32_bits(m) >> 23) & 0xFFu;
                const int sh = a.act_frac - ((int)eb - 127);
                const float lim = (float)((2 << a.act_frac) - 1);             // 127 or 31
                scale = x_scale(eb, a.act_frac);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float in[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float c = __builtin_rintf(__builtin_amdgcn_ldexpf(in[j], sh));
                        r[4 * i + j] = __builtin_fminf(__builtin_fmaxf(c, -lim), lim);
                    }
                    if constexpr (CELLS)
                        cw[i] = ((uint32_t)(int)r[4 * i] & 0xFFu) | (((uint32_t)(int)r[4 * i + 1] & 0xFFu) << 8) |
                                (((uint32_t)(int)r[4 * i + 2] & 0xFFu) << 16) | ((uint32_t)(int)r[4 * i + 3] << 24);
                }
            }
            if constexpr (SRC != 2) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        xf[p][h].u[i] = pack_bf16_exact(r[8 * h + 2 * i] * scale, r[8 * h + 2 * i + 1] * scale);
            }
            if (store_x && row_ok) {
                if (CELLS) {
                    const int64_t blk = tile * 16 + q + 4 * p;
                    if (a.x8) {
                        // 16 token rows and more: MXINT8 as it is, 16 code bytes per (block, row), and the
                        // exponent bytes [block][row] behind all codes; the main kernel converts
                        uint8_t* base = reinterpret_cast<uint8_t*>(a.Xh);
                        const int64_t entry = (blk << a.lr) + row;
                        *reinterpret_cast<u32x4*>(base + entry * 16) = cw;
                        // the main kernel scales codes by 2^(byte - 127 - 6): narrower codes carry the difference in the byte
                        const uint32_t ebs = eb + (6 - a.act_frac);
                        base[((a.KT * 16) << (a.lr + 4)) + entry] = (uint8_t)(ebs < 254u ? ebs : 254u);
                    } else {
                        uint16_t* dst = a.Xh + ((((blk * 2) << a.lr) + row) << 3);
                        *reinterpret_cast<u32x4*>(dst) = xf[p][0].u;
                        *reinterpret_cast<u32x4*>(dst + (8 << a.lr)) = xf[p][1].u;
                    }
                } else {
                    uint16_t* dst = a.Xh + row * a.ldxh + (tile * 16 + q + 4 * p) * 16;
                    *reinterpret_cast<u32x4*>(dst) = xf[p][0].u;
                    *reinterpret_cast<u32x4*>(dst + 8) = xf[p][1].u;
                }
            }
        }
#pragma unroll
        for (int g = 0; g < MAXG; ++g) {
            if (g < ng) {
                const uint8_t* rec = a.At + ((int64_t)(g0 + g) * a.KT + tile) * kARecordBytes;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    Frag af[2];
                    if constexpr (CELLS) {
                        af[0] = apre[g][p][0];
                        af[1] = apre[g][p][1];
                    } else {
                        af[0].u = *reinterpret_cast<const u32x4*>(rec + (2 * p) * 1024 + lane * 16);
                        af[1].u = *reinterpret_cast<const u32x4*>(rec + (2 * p + 1) * 1024 + lane * 16);
                    }
                    acc[g] = mfma16(af[0].v, xf[p][0].v, acc[g]);
                    acc[g] = mfma16(af[1].v, xf[p][1].v, acc[g]);
                }
                // one rank group's eight loads in flight at a time: all of them at once cost the registers of a second workgroup
                if constexpr (ROWWISE) __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    if (a.kp == 0) {
        // no low-rank branch: only the zero padding behind K_pad (none) remains
        return;
    }

    // add the wavefronts' partial T in a fixed order
    if constexpr (ROWWISE) __syncthreads();          // the sums reuse the tiles' memory: every wavefront is done with its tile
#pragma unroll
    for (int g = 0; g < MAXG; ++g)
        *reinterpret_cast<f32x4*>(&red[wave][g][lane][0]) = acc[g];
    __syncthreads();
    for (int item = threadIdx.x; item < ng * 64; item += blockDim.x) {
        const int g = item >> 6, l = item & 63;
        f32x4 s = *reinterpret_cast<const f32x4*>(&red[0][g][l][0]);
        for (int w = 1; w < nwaves; ++w) {
            const f32x4 o = *reinterpret_cast<const f32x4*>(&red[w][g][l][0]);
            s[0] += o[0]; s[1] += o[1]; s[2] += o[2]; s[3] += o[3];
        }
        const int64_t orow = (int64_t)blockIdx.x * 16 + (l & 15);
        const int r0 = (g0 + g) * 16 + 4 * (l >> 4);          // first of this lane's 4 ranks
        if (orow < a.M) {
            if (FINAL) {
                uint16_t hi[4], lo[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) split_bf16(s[j], hi[j], lo[j]);
                uint16_t* base = a.Xh + orow * a.ldxh + a.KT * kTileK;
                *reinterpret_cast<u32x2*>(base + r0) =
                    u32x2{(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
                *reinterpret_cast<u32x2*>(base + a.kp + r0) =
                    u32x2{(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
            } else {
                *reinterpret_cast<f32x4*>(a.Tpart + ((int64_t)slice * a.tp_rows + orow) * a.kp + r0) = s;
            }
        }
    }
    // zero the padding behind T_hi | T_lo so the main kernel can read whole 64-column chunks
    if (FINAL && blockIdx.z == 0) {
        const int pad = (int)(a.tail_cols - 2 * a.kp);
        for (int item = threadIdx.x; item < 16 * pad; item += blockDim.x) {
            const int64_t orow = (int64_t)blockIdx.x * 16 + item / pad;
            if (orow < a.M) a.Xh[orow * a.ldxh + a.KT * kTileK + 2 * a.kp + item % pad] = 0;
        }
    }
}

template <int SRC, bool FINAL, int MAXG, bool CELLS>
static void launch_prep_t(dim3 grid, dim3 block, hipStream_t s, const PrepArgs& a, bool rowwise) {
    if constexpr (SRC == 0 && !CELLS) {
        if (rowwise) {
            hipLaunchKernelGGL((prep_kernel<SRC, FINAL, MAXG, CELLS, true>), grid, block, 0, s, a);
            return;
        }
    }
    hipLaunchKernelGGL((prep_kernel<SRC, FINAL, MAXG, CELLS, false>), grid, block, 0, s, a);
}

int prep_slices(const Layer& L, int64_t M, int path) {
    if (path != 1) {
        // tiled path: one workgroup per 16 token rows; when that leaves compute units idle, split K
        // as well (each slice keeps at least two tiles) and let the tiled kernel add the partial T
        const int64_t rg = (M + 15) / 16;
        int64_t s = 1;
        while (rg * s < 512 && s < 8 && L.KT / (2 * s) >= 2) s *= 2;
        return (int)s;
    }
    // streaming path: at most two row groups, so K is spread over workgroups (the main kernel adds
    // up to 8 partial sums); one wavefront per K tile of a slice, at most kPrepWaves.
    int64_t s = L.KT;
    if (s > 8) s = 8;
    if (s < 1) s = 1;
    return (int)s;
}

hipError_t launch_prep(const Layer& L, const float* X, int64_t ldx, const int8_t* Xc, const uint8_t* Xe,
                       int64_t M, const Workspace& ws, float* y_zero, int64_t ldy, hipStream_t s, bool reuse_xh) {
    if (M == 0) return hipSuccess;
    if (reuse_xh && (ws.cells || X != nullptr || Xc != nullptr)) return hipErrorInvalidValue;
    PrepArgs a;
    a.X = X; a.ldx = ldx; a.Xc = Xc; a.Xe = Xe;
    a.M = M; a.K = L.K; a.KT = L.KT;
    a.tiles_per_slice = (int)((L.KT + ws.S - 1) / ws.S);
    a.kp = L.kp; a.kp16 = L.kp16;
    a.groups_per_wg = L.kp16;
    // Few-token calls are bound by the latency of reading A_k (1 MB for K = 8192, kp = 64) with a handful of
    // workgroups: there every rank group gets workgroups of its own (grid.z), each quantizing the few
    // rows again; 1 us less on the 70B-shaped layer.
    int gz = 1;
    if (ws.cells && L.kp16 > 1) { gz = L.kp16; a.groups_per_wg = 1; }
    // More than four rank groups (ranks above 64), row-major layout: this launch does the first four; the others
    // follow in a second launch that reads the bf16 activations this one stores (half the bytes, nothing to
    // quantize), in planes of four groups.  (An input that is already the stored matrix takes planes at once.)
    const bool two_launches = !ws.cells && L.kp16 > 4 && !reuse_xh;
    if (!ws.cells && L.kp16 > 4) { gz = reuse_xh ? (L.kp16 + 3) / 4 : 1; a.groups_per_wg = 4; }
    a.g_first = 0;
    a.At = L.At; a.Xh = ws.Xh; a.ldxh = ws.ldxh;
    a.tail_cols = ws.ldxh - L.KT * kTileK;
    a.Tpart = ws.Tpart;
    a.tp_rows = ws.tp_rows;
    a.lr = ws.lr;
    a.x8 = ws.x8;
    a.act_frac = L.act_bits - 2;
    a.Yz = y_zero; a.ldy = ldy; a.N = L.N;
    a.nslices = ws.S;
    a.flags = ws.flags; a.nflags = ws.flags ? kTiledFlags : 0;
    const bool cells = ws.cells;
    int nwaves = a.tiles_per_slice;
    if (nwaves > kPrepWaves) nwaves = kPrepWaves;
    if (nwaves < 1) nwaves = 1;
    dim3 block(64 * nwaves);
    // clearing workgroups: about four 16-byte stores per thread
    const int64_t rg = (M + 15) / 16;
    const int64_t zero_wgs = y_zero ? (M * ((L.N + 3) / 4) + 4 * block.x * rg - 1) / (4 * block.x * rg) : 0;
    dim3 grid((unsigned)rg, (unsigned)(ws.S + zero_wgs), (unsigned)gz);
    const int src = reuse_xh ? 2 : (Xc != nullptr ? 1 : 0);
    const bool fin = (ws.Tpart == nullptr);          // T final (hi/lo behind the row) or partial sums
    if (cells && fin && L.kp > 0) return hipErrorInvalidValue;
    if (a.groups_per_wg > 4) return hipErrorInvalidValue;
    // the row-wise form for fp32 input in row-major layout when the launch has workgroups to spare
    const bool rowwise = !cells && src == 0 && (int64_t)grid.x * ws.S * gz >= 2048;
#define LQER_PREP(FC, FN, MG, CL) launch_prep_t<FC, FN, MG, CL>(grid, block, s, a, rowwise)
#define LQER_PREP_G(FC, FN, CL) do { if (a.groups_per_wg <= 1) LQER_PREP(FC, FN, 1, CL); else LQER_PREP(FC, FN, 4, CL); } while (0)
#define LQER_PREP_C(FN, CL) do { if (src == 1) LQER_PREP_G(1, FN, CL); else LQER_PREP_G(0, FN, CL); } while (0)
    if (cells) LQER_PREP_C(false, true);
    else if (src == 2) { if (fin) LQER_PREP_G(2, true, false); else LQER_PREP_G(2, false, false); }
    else if (fin) LQER_PREP_C(true, false);
    else LQER_PREP_C(false, false);
    if (two_launches) {
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        a.g_first = 4;
        grid.z = (unsigned)((L.kp16 - 4 + 3) / 4);
        grid.y = (unsigned)ws.S;
        if (fin) LQER_PREP_G(2, true, false); else LQER_PREP_G(2, false, false);
    }
#undef LQER_PREP_C
#undef LQER_PREP_G
#undef LQER_PREP
    return hipGetLastError();
}

}  // namespace lqer
