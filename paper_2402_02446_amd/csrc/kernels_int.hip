// The scaled-integer variant of the layer (Table 2, "L2QER-INT": INT4 weights in groups of 128 with FP16 scales,
// INT8 activations with one scale per token, INT8 rank-k factors; Sec. 2.1 for the form of such formats):
//   Y[t][n] = s_t sum_g sW[n][g] I_W[t][n][g]  +  sum_r T[t][r] Bc[r][n] sB[n],   T[t][r] = s_t sum_g sA[r][g] I_A[t][r][g]
// with I the exact integer inner product of one group of 128 codes.  An FP16 scale times a code is no bf16 number, so
// the scales cannot be folded into the operands the way MXINT's powers of two are; instead the integer products run on
// the int8 matrix cores (32x32x32, exact in i32) and every group's sum is converted and scaled once, in fp32.
//
//   quant_token_kernel   per-token INT8 quantizer (one workgroup per token row: row maximum, then codes)
//   int_gemm_kernel      128 tokens x 128 columns per workgroup, four wavefronts of 64 x 64; one K group per step:
//                        activation codes and the group's 128 scales through double-buffered LDS (the tile XOR-swizzled),
//                        packed weights straight into registers, all asked for one group ahead at the top of the step.  <4, true>: the main product with the rank-k correction
//                        (T_hi | T_lo against B_k's codes on the bf16 matrix cores, one scale per column) in the
//                        epilogue; <8, false>: the projection T = X_q A_k, A_k as 8-bit "weights".
//
// Weight codes keep their canonical nibbles: of a 32-bit word (8 elements) `(w << 4) & 0xF0F0F0F0` are the even
// elements times 16 as int8 and `w & 0xF0F0F0F0` the odd ones - two instructions per 8 weights; the factor 16 is
// folded into the scale table.  A lane's 16 bytes (32 consecutive K) thus feed two MFMAs, one with the even and one
// with the odd elements, and the activation codes are stored in the same order: every run of 32 as its 16 even
// elements followed by its 16 odd ones (the contraction does not care about the order, only that both sides agree).
#include <mutex>

#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

// ---- per-token INT8 quantizer ----------------------------------------------------------------------------------
// PERM: codes in the order the product kernel reads them (see above); otherwise canonical.
template <bool PERM>
__global__ __launch_bounds__(256) void quant_token_kernel(const float* __restrict__ X, int64_t ldx, int64_t K,
                                                          int8_t* __restrict__ codes, int64_t ldc, float* scale_f32,
                                                          uint16_t* scale_f16) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const float* x = X + row * ldx;
    const int64_t n4 = K >> 2;
    float m = 0.f;
    for (int64_t i = threadIdx.x; i < n4; i += 256) {
        const float4 v = *reinterpret_cast<const float4*>(x + 4 * i);
        m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(v.x), __builtin_fabsf(v.y)),
                                               __builtin_fmaxf(__builtin_fabsf(v.z), __builtin_fabsf(v.w))));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = __builtin_fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = __builtin_fmaxf(__builtin_fmaxf(red[0], red[1]), __builtin_fmaxf(red[2], red[3]));
    // s = fp16(amax / 127), the division in fp32 and correctly rounded; 1 for an all-zero row
    const _Float16 sh = (m == 0.f) ? (_Float16)1.0f : (_Float16)__fdiv_rn(m, 127.0f);
    const float s = (float)sh;
    if (threadIdx.x == 0) {
        if (scale_f32) scale_f32[row] = s;
        if (scale_f16) scale_f16[row] = __builtin_bit_cast(uint16_t, sh);
    }
    int8_t* c = codes + row * ldc;
    for (int64_t i = threadIdx.x; i < n4; i += 256) {
        const float4 v = *reinterpret_cast<const float4*>(x + 4 * i);
        const float in[4] = {v.x, v.y, v.z, v.w};
        uint32_t q[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float r = __builtin_rintf(__fdiv_rn(in[j], s));
            r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
            q[j] = (uint32_t)(int)r & 0xFFu;
        }
        if (PERM) {
            const int64_t e0 = 4 * i, span = e0 & ~(int64_t)31, h = (e0 & 31) >> 1;   // elements e0, e0+2 even; e0+1, e0+3 odd
            *reinterpret_cast<uint16_t*>(c + span + h) = (uint16_t)(q[0] | (q[2] << 8));
            *reinterpret_cast<uint16_t*>(c + span + 16 + h) = (uint16_t)(q[1] | (q[3] << 8));
        } else {
            *reinterpret_cast<uint32_t*>(c + 4 * i) = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
        }
    }
}

hipError_t launch_quant_token(const float* X, int64_t rows, int64_t K, int64_t ldx, int8_t* codes, int64_t ldc,
                              float* scale_f32, uint16_t* scale_f16, bool perm, hipStream_t s) {
    if (rows == 0) return hipSuccess;
    if (perm) hipLaunchKernelGGL(quant_token_kernel<true>, dim3((unsigned)rows), dim3(256), 0, s, X, ldx, K, codes, ldc, scale_f32, scale_f16);
    else hipLaunchKernelGGL(quant_token_kernel<false>, dim3((unsigned)rows), dim3(256), 0, s, X, ldx, K, codes, ldc, scale_f32, scale_f16);
    return hipGetLastError();
}

// ---- the product kernel ------------------------------------------------------------------------------------------
struct IntGemmArgs {
    const int8_t* Xc; int64_t ldxc;      // activation codes [rows padded to 128][K], permuted order
    const float* Xs;                     // token scales [rows padded]
    const uint8_t* Wt;                   // weight records [N32][G][rec]: 4 bits: [2 spans][64 lanes][16 B]; 8 bits: [4 steps][64 lanes][16 B]
    const float* Wsc;                    // scales [N32][G][32] (4 bits: already divided by 16)
    int64_t M, N, N32, G;
    float* Out; int64_t ldo;             // Y [M][ldo], or T [S][rows padded][ldo] for the projection
    int64_t g_per_z;                     // K groups per plane of grid.z (the projection splits K over S planes; G otherwise)
    int64_t out_z_stride;                // floats between the planes' outputs
    // rank-k correction (TAIL)
    const float* T; int64_t ldt;         // [S][rows padded][ldt] fp32 partial sums of T, added in plane order
    int S; int64_t t_stride;
    const uint8_t* Bt; const float* Bsc; // B_k records [N32][kp16][kBRecordBytes], scales [N32 * 32]
    int kp16;
    int tail_plane;                      // 1: grid.z has one more plane than K planes, which computes only the correction
};

template <int WB, bool TAIL>
__global__ __launch_bounds__(256, 2) void int_gemm_kernel(IntGemmArgs a) {
    constexpr int TM = 2, TN = 2;
    constexpr int NL = (WB == 4) ? 2 : 4;            // 16-byte loads per lane, column group and K group
    constexpr int REC = NL * 1024;
    __shared__ __attribute__((aligned(1024))) uint8_t xs[2][128 * 128];
    __shared__ __attribute__((aligned(16))) float ss[2][128];      // the K group's scales of the tile's 128 columns

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const int t = lane & 31, hh = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.y * 128;
    const int64_t g0 = ((int64_t)blockIdx.x * 2 + wc) * TN;        // first column group of this wavefront
    auto clamp_group = [&](int64_t g) { return g < a.N32 ? g : a.N32 - 1; };   // (the store is masked)
    auto group_of = [&](int tn) { return clamp_group(g0 + tn); };
    // activation loader: thread -> four 16-byte cells of a 128 x 128 byte tile
    const int ld_row = tid >> 3, ld_cell = tid & 7;
    const int8_t* ld_src = a.Xc + (m0 + ld_row) * a.ldxc + ld_cell * 16;
    const int ld_dst = ld_row * 128 + ((ld_cell ^ ((ld_row >> 1) & 7)) << 4);   // rows 32 apart share the swizzle term
    // scale loader: the first 32 threads bring the 4 x 32 scales of the tile's column groups (four floats each)
    const float* sc_src = a.Wsc + clamp_group((int64_t)blockIdx.x * 4 + ((tid >> 3) & 3)) * a.G * 32 + (tid & 7) * 4;
    const int sc_dst = ((tid >> 3) & 3) * 32 + (tid & 7) * 4;
    struct XStage { u32x4 x[4]; f32x4 s; };
    auto fetch_x = [&](XStage& st, int64_t g) {
#pragma unroll
        for (int j = 0; j < 4; ++j) st.x[j] = *reinterpret_cast<const u32x4*>(ld_src + (int64_t)j * 32 * a.ldxc + g * 128);
        st.s = *reinterpret_cast<const f32x4*>(sc_src + g * 32);     // (every thread: the wavefronts beyond the first ask for the same lines again)
    };
    auto store_x = [&](const XStage& st, int buf) {
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4*>(&xs[buf][ld_dst + j * 32 * 128]) = st.x[j];
        if (tid < 32) *reinterpret_cast<f32x4*>(&ss[buf][sc_dst]) = st.s;
    };
    struct WSet { u32x4 c[TN][NL]; };
    auto load_w = [&](WSet& w, int64_t g) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const uint8_t* rec = a.Wt + (group_of(tn) * a.G + g) * REC + lane * 16;
#pragma unroll
            for (int l = 0; l < NL; ++l) w.c[tn][l] = *reinterpret_cast<const u32x4*>(rec + l * 1024);
        }
    };
    // operand read: MFMA (sp, p) of a group uses bytes 64 sp + 32 hh + 16 p .. + 15 of the token's 128: cell 4 sp + 2 hh + p
    const int rd_row = wr * 64 + t;
    auto read_x = [&](int buf, int tm, int sp, int p) {
        const int row = rd_row + tm * 32;
        const int cell = (4 * sp + 2 * hh + p) ^ ((row >> 1) & 7);   // rows are 128 B = half of the banks: 16 rows of a read hit 16 different bank groups
        return *reinterpret_cast<const i32x4*>(&xs[buf][row * 128 + (cell << 4)]);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

    float st[TM];                                    // token scales (for the epilogue; asked for here, ahead of the loop)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) st[tm] = a.Xs[m0 + wr * 64 + tm * 32 + t];

    // this workgroup's K groups [gb, ge)
    const bool tail_only = TAIL && a.tail_plane && blockIdx.z + 1 == gridDim.z;    // (its range is empty: acc stays zero)
    const int64_t gb = tail_only ? 0 : (int64_t)blockIdx.z * a.g_per_z;
    const int64_t ge = tail_only ? 0 : (gb + a.g_per_z < a.G ? gb + a.g_per_z : a.G);
    WSet w0, w1;
    XStage stx;
    fetch_x(stx, gb);
    load_w(w0, gb);
    store_x(stx, 0);

    // One K group.  The next group's activations, scales and weights are asked for first and stay in flight through the
    // step (they land in LDS / become `cur` at its end); the column groups are worked one after the other, so that the
    // conversion and scaling of one's sums can run beside the MFMAs of the other.
    auto step = [&](const WSet& cur, WSet& nxt, int64_t g) {
        __syncthreads();                             // tile g is complete; the other buffer is free again
        const int buf = (int)((g - gb) & 1);
        const int64_t gn = g + 1 < ge ? g + 1 : g;   // clamped: loads stay unconditional
        fetch_x(stx, gn);
        load_w(nxt, gn);
        __builtin_amdgcn_sched_barrier(0);           // (not to be sunk towards their uses: that would put the round trip on the step's path)
        i32x4 xb[2][2][TM];
#pragma unroll
        for (int sp = 0; sp < 2; ++sp)
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) xb[sp][p][tm] = read_x(buf, tm, sp, p);
        auto products = [&](i32x16 (&ia)[TM], int tn) {
#pragma unroll
            for (int sp = 0; sp < 2; ++sp)
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    i32x4 wv;
                    if constexpr (WB == 4) {
                        const u32x4 c = cur.c[tn][sp];
#pragma unroll
                        for (int e = 0; e < 4; ++e) wv[e] = (int)((p == 0 ? c[e] << 4 : c[e]) & 0xF0F0F0F0u);
                    } else {
                        wv = __builtin_bit_cast(i32x4, cur.c[tn][2 * sp + p]);
                    }
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        if (sp == 0 && p == 0) {
                            i32x16 z;
#pragma unroll
                            for (int r = 0; r < 16; ++r) z[r] = 0;
                            ia[tm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv, xb[sp][p][tm], z, 0, 0, 0);
                        } else {
                            ia[tm] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv, xb[sp][p][tm], ia[tm], 0, 0, 0);
                        }
                    }
                }
        };
        // the group's exact integer sums, scaled once: register r of a lane is column 8 (r / 4) + 4 hh + r % 4
        auto fold = [&](const i32x16 (&ia)[TM], int tn) {
            f32x4 sc[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) sc[q] = *reinterpret_cast<const f32x4*>(&ss[buf][(wc * 2 + tn) * 32 + 8 * q + 4 * hh]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[tm][tn][r] += (float)ia[tm][r] * sc[r >> 2][r & 3];
        };
        // (the empty asm statements keep the arithmetic where it is written: nothing else orders pure instructions
        // against the scheduling barriers, and left alone they all sink to the end of the step)
        i32x16 ia0[TM], ia1[TM];
        products(ia0, 0);
        asm volatile("" : "+v"(ia0[0]), "+v"(ia0[1]));
        __builtin_amdgcn_sched_barrier(0);
        // the second column group's MFMAs run while the first one's sums are converted and scaled
        products(ia1, 1);
        fold(ia0, 0);
        asm volatile("" : "+v"(ia1[0]), "+v"(ia1[1]), "+v"(acc[0][0]), "+v"(acc[1][0]));
        __builtin_amdgcn_sched_barrier(0);
        fold(ia1, 1);
        asm volatile("" : "+v"(acc[0][1]), "+v"(acc[1][1]));
        __builtin_amdgcn_sched_barrier(0);
        store_x(stx, buf ^ 1);                       // last read two barriers ago (a clamped re-write of the last tile is harmless)
    };
    for (int64_t g = gb; g < ge; g += 2) {
        step(w0, w1, g);
        if (g + 1 < ge) step(w1, w0, g + 1);
    }

    // ---- epilogue: token scale, rank-k correction, store ----------------------------------------------------------
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] *= st[tm];
    if constexpr (TAIL) {
        if (a.kp16 > 0 && (a.tail_plane ? tail_only : blockIdx.z == 0)) {
            f32x16 ta[TM][TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) ta[tm][tn][r] = 0.f;
            // one 32x32x16 step per rank block and bf16 term: lane half hh takes ranks 8 hh .. + 7 of the block on both sides
            for (int rb = 0; rb < a.kp16; ++rb) {
                Frag bf[TN];
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const uint8_t* rec = a.Bt + (group_of(tn) * a.kp16 + rb) * kBRecordBytes;
                    const u32x4 cw = *reinterpret_cast<const u32x4*>(rec + t * 16);
                    Frag f0, f1;
                    int8x16_to_frags(cw, 1.0f, f0, f1);
                    bf[tn] = hh ? f1 : f0;
                }
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const float* src = a.T + (m0 + wr * 64 + tm * 32 + t) * a.ldt + rb * 16 + 8 * hh;
                    f32x4 p0 = *reinterpret_cast<const f32x4*>(src), p1 = *reinterpret_cast<const f32x4*>(src + 4);
                    for (int z0 = 1; z0 < a.S; z0 += 8) {                // the projection's K planes, in plane order;
                        f32x4 q[8][2];                                   // eight planes' loads in flight at a time
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const int z = z0 + j < a.S ? z0 + j : a.S - 1;
                            q[j][0] = *reinterpret_cast<const f32x4*>(src + z * a.t_stride);
                            q[j][1] = *reinterpret_cast<const f32x4*>(src + z * a.t_stride + 4);
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            if (z0 + j < a.S) {
                                p0 += q[j][0];
                                p1 += q[j][1];
                            }
                    }
                    const float v[8] = {p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
                    Frag hi, lo;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        uint32_t h2[2], l2[2];
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const uint32_t hb = f32_bits(v[2 * e + j]) & 0xFFFF0000u;
                            h2[j] = hb >> 16;
                            l2[j] = f32_bits(v[2 * e + j] - f32_from_bits(hb)) >> 16;
                        }
                        hi.u[e] = h2[0] | (h2[1] << 16);
                        lo.u[e] = l2[0] | (l2[1] << 16);
                    }
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        ta[tm][tn] = mfma32(bf[tn].v, hi.v, ta[tm][tn]);
                        ta[tm][tn] = mfma32(bf[tn].v, lo.v, ta[tm][tn]);
                    }
                }
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const float* s = a.Bsc + group_of(tn) * 32 + 4 * hh;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 sb = *reinterpret_cast<const f32x4*>(s + 8 * q);
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[tm][tn][4 * q + j] += ta[tm][tn][4 * q + j] * sb[j];
                }
            }
        }
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int64_t row = m0 + wr * 64 + tm * 32 + t;
        if (TAIL && row >= a.M) continue;            // (the projection writes its padded rows too: the tail reads them)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int64_t cg = g0 + tn;
            if (cg >= a.N32) continue;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int64_t n = cg * 32 + 8 * r4 + 4 * hh;
                float* dst = a.Out + (int64_t)blockIdx.z * a.out_z_stride + row * a.ldo + n;
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

// Few-token calls split the K groups of the projection and of the main product over planes of workgroups, each leaving
// its share of T or Y in the workspace; this adds the planes in plane order (the same bits on every run).
// Y may be the first plane itself (a thread reads all of its elements before it writes them).
__global__ __launch_bounds__(256) void int_reduce_planes_kernel(const float* P, int planes, int64_t plane_stride,
                                                                int64_t M, int64_t N, int64_t ldp, float* Y, int64_t ldy) {
    const int64_t n4 = (N + 3) / 4;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M * n4) return;
    const int64_t r = i / n4, c = 4 * (i - r * n4);
    const float* src = P + r * ldp + c;
    f32x4 v = *reinterpret_cast<const f32x4*>(src);
    for (int z0 = 1; z0 < planes; z0 += 8) {         // eight loads in flight, added in plane order
        f32x4 q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = *reinterpret_cast<const f32x4*>(src + (z0 + j < planes ? z0 + j : planes - 1) * plane_stride);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (z0 + j < planes) v += q[j];
    }
    float* dst = Y + r * ldy + c;
    if (c + 3 < N) {
        *reinterpret_cast<f32x4*>(dst) = v;
    } else {
        for (int j = 0; c + j < N; ++j) dst[j] = v[j];
    }
}

hipError_t launch_int_reduce_planes(const float* P, int planes, int64_t plane_stride, int64_t M, int64_t N, int64_t ldp,
                                    float* Y, int64_t ldy, hipStream_t s) {
    const int64_t items = M * ((N + 3) / 4);
    hipLaunchKernelGGL(int_reduce_planes_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, P, planes, plane_stride, M, N, ldp, Y, ldy);
    return hipGetLastError();
}

// Projection T = X_q A_k (Out = T, N = padded rank) or main product with the correction.
hipError_t launch_int_gemm(bool projection, const IntGemmArgs& a, hipStream_t s) {
    if (a.M == 0) return hipSuccess;
    const unsigned planes = (unsigned)((a.G + a.g_per_z - 1) / a.g_per_z) + (projection ? 0u : (unsigned)a.tail_plane);
    const dim3 grid((unsigned)((a.N + 127) / 128), (unsigned)((a.M + 127) / 128), planes), block(256);
    if (projection) hipLaunchKernelGGL((int_gemm_kernel<8, false>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((int_gemm_kernel<4, true>), grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace lqer
