// MX block quantizer (Sec. 2.2; block [1,16] of Sec. 4.1): fp32 rows -> MXINT codes + exponent bytes.
//
// HBM-bound: 4 B read and 1 + 1/16 B written per element (8- and 6-bit codes, one byte each).  Each lane loads one
// float4, so a wavefront load is one contiguous 1 KiB; the four lanes of a quad hold one
// 16-element block and agree on its maximum with two DPP quad permutes.  The shared exponent is
// the biased exponent field of that fp32 maximum.  The activations are read once and with streaming loads
// (each cache line belongs to exactly one load instruction), which keeps them from displacing the stored codes.
#include "lqer_internal.h"
#include "mx_device.h"

namespace lqer {

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(float,
        __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <int BITS>
__device__ __forceinline__ int mx_code(float v, int e_unbiased) {
    constexpr float lim = (float)((1 << (BITS - 1)) - 1);
    float r = __builtin_rintf(__builtin_amdgcn_ldexpf(v, (BITS - 2) - e_unbiased));
    r = __builtin_fminf(__builtin_fmaxf(r, -lim), lim);
    return (int)r;
}

template <int BITS, int UNROLL>
__global__ __launch_bounds__(256) void quantize_mx_kernel(const float* __restrict__ x, int64_t rows,
                                                          int64_t cols4, int64_t ld,
                                                          uint8_t* __restrict__ codes,
                                                          uint8_t* __restrict__ exps) {
    const int64_t total = rows * cols4;                       // float4 items; a multiple of 4
    const int64_t nthreads = (int64_t)gridDim.x * blockDim.x;
    // (row, column) of this thread's items without a division per item: one division here, then every
    // step of nthreads items moves by the same (rows, columns) with a carry
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t step_r = nthreads / cols4, step_c = nthreads - step_r * cols4;      // wave-uniform
    int64_t r_next = first / cols4, c_next = first - r_next * cols4;
    for (int64_t base = first; base < total; base += nthreads * UNROLL) {
        float4 v[UNROLL];
        int64_t row[UNROLL], c4[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = base + (int64_t)u * nthreads;
            row[u] = r_next;
            c4[u] = c_next;
            c_next += step_c;
            r_next += step_r;
            if (c_next >= cols4) { c_next -= cols4; ++r_next; }
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < total) {
                const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x + row[u] * ld + 4 * c4[u]));
                v[u] = make_float4(t[0], t[1], t[2], t[3]);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t i = base + (int64_t)u * nthreads;
            float m = __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(v[u].x), __builtin_fabsf(v[u].y)),
                                      __builtin_fmaxf(__builtin_fabsf(v[u].z), __builtin_fabsf(v[u].w)));
            m = __builtin_fmaxf(m, dpp_f32<0xB1>(m));          // quad_perm [1,0,3,2]
            m = __builtin_fmaxf(m, dpp_f32<0x4E>(m));          // quad_perm [2,3,0,1]
            const uint32_t eb = (f32_bits(m) >> 23) & 0xFFu;
            const int e = (int)eb - 127;
            const int c0 = mx_code<BITS>(v[u].x, e), c1 = mx_code<BITS>(v[u].y, e);
            const int c2 = mx_code<BITS>(v[u].z, e), c3 = mx_code<BITS>(v[u].w, e);
            if (i < total) {
                const int64_t elem = row[u] * cols4 * 4 + 4 * c4[u];
                if (BITS >= 6) {
                    const uint32_t w = (uint32_t)(c0 & 0xFF) | ((uint32_t)(c1 & 0xFF) << 8) |
                                       ((uint32_t)(c2 & 0xFF) << 16) | ((uint32_t)(c3 & 0xFF) << 24);
                    *reinterpret_cast<uint32_t*>(codes + elem) = w;
                } else {
                    const uint16_t w = (uint16_t)((c0 & 0xF) | ((c1 & 0xF) << 4) |
                                                  ((c2 & 0xF) << 8) | ((c3 & 0xF) << 12));
                    *reinterpret_cast<uint16_t*>(codes + elem / 2) = w;
                }
                if ((c4[u] & 3) == 0) exps[row[u] * (cols4 / 4) + (c4[u] >> 2)] = (uint8_t)eb;
            }
        }
    }
}

hipError_t launch_quantize_mx(const float* x, int64_t rows, int64_t cols, int64_t ld, int bits,
                              void* codes, uint8_t* exps, hipStream_t s) {
    const int64_t cols4 = cols / 4;
    const int64_t total = rows * cols4;
    if (total == 0) return hipSuccess;
    constexpr int UNROLL = 4;
    int64_t blocks = (total + 256 * UNROLL - 1) / (256 * UNROLL);
    const int64_t cap = 256 * 16;                  // 16 workgroups per compute unit is plenty
    if (blocks > cap) blocks = cap;
    dim3 grid((unsigned)blocks), block(256);
    if (bits == 8)
        hipLaunchKernelGGL((quantize_mx_kernel<8, UNROLL>), grid, block, 0, s, x, rows, cols4, ld,
                           (uint8_t*)codes, exps);
    else if (bits == 6)
        hipLaunchKernelGGL((quantize_mx_kernel<6, UNROLL>), grid, block, 0, s, x, rows, cols4, ld,
                           (uint8_t*)codes, exps);
    else
        hipLaunchKernelGGL((quantize_mx_kernel<4, UNROLL>), grid, block, 0, s, x, rows, cols4, ld,
                           (uint8_t*)codes, exps);
    return hipGetLastError();
}

}  // namespace lqer
