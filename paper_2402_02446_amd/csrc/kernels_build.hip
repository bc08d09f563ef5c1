// Offline construction of an LQER / L2QER layer with the heavy steps on the device (Sec. 3.1
// Eq. 1-2; Sec. 3.2 Eq. 4-5; App. A Eq. 7-8):
//   calibration magnitudes (App. A), W_q = q(W) in MXINT4 with G = S (W - W_q) formed in the same
//   pass, and the two tall-skinny products per subspace iteration (G Z and G^T Q) run as HIP
//   kernels in fp32; the l x l steps (Cholesky factor for the orthonormalization, eigenvectors of
//   the projected Gram matrix) and the final MXINT8 packing of A_k and B_k stay on the host in
//   fp64.  The iteration is the one of the host path: a range finder with power iterations that
//   stops when the energy of the leading k directions stops growing.
// The products are bound by reading G (K N fp32) once per pass; they are plain FMA kernels.
#include <cmath>
#include <vector>

#include "lqer_internal.h"
#include "mx_device.h"
#include "build_common.h"

namespace lqer {

// abar[c] = max over samples of the mean |x| of channel c; rows are added in order, in fp64, so the
// result has the bits of the host path.
__global__ __launch_bounds__(256) void calib_magnitude_kernel(const float* __restrict__ x, int64_t n_samples,
                                                              int64_t rows, int64_t K, double* __restrict__ abar) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= K) return;
    double m = 0.0;
    for (int64_t i = 0; i < n_samples; ++i) {
        double a = 0.0;
        for (int64_t r = 0; r < rows; ++r) a += fabs((double)x[(i * rows + r) * K + c]);
        a /= (double)rows;
        m = a > m ? a : m;
    }
    abar[c] = m;
}

// Largest |w| of the tensor as fp32 bits (non-negative floats order like their bit patterns): with 4-bit
// shared exponents its exponent field fixes the lowest exponent the tensor can store.  *out is zero before.
__global__ __launch_bounds__(256) void absmax_bits_kernel(const float* __restrict__ W, int64_t count, uint32_t* __restrict__ out) {
    uint32_t m = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        m = max(m, f32_bits(__builtin_fabsf(W[i])));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    if ((threadIdx.x & 63) == 0) atomicMax(out, m);
}

// One thread per MXINT4 block (16 consecutive k of one column n): codes and exponent byte in the
// canonical layout, and G = s[k] (w - dq(q(w))) in fp32 (the difference itself is exact).
// flag: set when a weight is not finite.
// amax_bits != null: 4-bit shared exponents - blocks more than 15 binades below the tensor's largest are
// quantized with the lowest exponent byte that can be stored.
__global__ __launch_bounds__(256) void quantize_w_kernel(const float* __restrict__ W, int64_t K, int64_t N,
                                                         const float* __restrict__ s, uint8_t* __restrict__ Wc,
                                                         uint8_t* __restrict__ We, float* __restrict__ G,
                                                         int* __restrict__ flag, const uint32_t* __restrict__ amax_bits) {
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t kb = blockIdx.y;
    if (n >= N) return;
    float v[16];
    float m = 0.f;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        v[i] = W[(kb * 16 + i) * N + n];
        bad |= !(__builtin_fabsf(v[i]) <= 3.4028234e38f);
        m = __builtin_fmaxf(m, __builtin_fabsf(v[i]));
    }
    if (bad) {
        *flag = 1;
        return;
    }
    uint32_t eb = (f32_bits(m) >> 23) & 0xFFu;
    if (amax_bits != nullptr) {
        const uint32_t top = (*amax_bits >> 23) & 0xFFu;
        const uint32_t floor_byte = top > 15u ? top - 15u : 0u;
        if (eb < floor_byte) eb = floor_byte;
    }
    const int e = (int)eb - 127;
    int c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float r = __builtin_rintf(__builtin_amdgcn_ldexpf(v[i], 2 - e));
        r = __builtin_fminf(__builtin_fmaxf(r, -7.0f), 7.0f);
        c[i] = (int)r;
    }
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        lo |= (uint32_t)(c[i] & 0xF) << (4 * i);
        hi |= (uint32_t)(c[8 + i] & 0xF) << (4 * i);
    }
    *reinterpret_cast<u32x2*>(Wc + n * (K / 2) + kb * 8) = u32x2{lo, hi};
    We[n * (K / 16) + kb] = (uint8_t)eb;
    if (G != nullptr) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t row = kb * 16 + i;
            G[row * N + n] = s[row] * (v[i] - __builtin_amdgcn_ldexpf((float)c[i], e - 2));
        }
    }
}

// Tall-skinny product with a small right-hand side of l <= 80 columns.
//   TRANS = false: out[r][c] = sum_j A[r][j] B[j][c]      (A is R x C, B is C x l, out R x l)
//   TRANS = true : out[q][c] = sum_r A[r][q] B[r][c]      (A is R x C, B is R x l, out C x l)
// A workgroup owns 64 output rows and one slice of the contraction range; it writes a partial
// result part[slice][out rows][l], which ts_reduce_kernel adds in slice order (same bits every run).
constexpr int kTsRows = 64, kTsDepth = 32, kTsMaxL = 80;

template <bool TRANS>
__global__ __launch_bounds__(256) void ts_gemm_kernel(const float* __restrict__ A, int64_t R, int64_t C,
                                                      const float* __restrict__ B, int l, float* __restrict__ part,
                                                      int64_t depth_per_slice) {
    __shared__ float As[kTsDepth][kTsRows + 4];       // [contraction index][output row]
    __shared__ float Bs[kTsDepth][kTsMaxL];
    const int tid = threadIdx.x;
    const int64_t out_rows = TRANS ? C : R, depth = TRANS ? R : C;
    const int64_t o0 = (int64_t)blockIdx.x * kTsRows;
    const int64_t j_begin = (int64_t)blockIdx.y * depth_per_slice;
    int64_t j_end = j_begin + depth_per_slice;
    if (j_end > depth) j_end = depth;
    const int og = tid & 15, cg = tid >> 4;           // this thread: output rows 4 og .. + 3, columns cg + 16 q
    float acc[4][5];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 5; ++q) acc[i][q] = 0.f;

    for (int64_t j0 = j_begin; j0 < j_end; j0 += kTsDepth) {
        __syncthreads();
        // A tile: 64 output rows x 32 contraction indices, zero outside the matrix or the slice
        if (TRANS) {
            const int o = tid & 63;
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int j = (tid >> 6) + 4 * p;
                const int64_t r = j0 + j, q = o0 + o;
                As[j][o] = (r < j_end && q < C) ? A[r * C + q] : 0.f;
            }
        } else {
            const int j = tid & 31;
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int o = (tid >> 5) + 8 * p;
                const int64_t r = o0 + o, q = j0 + j;
                As[j][o] = (r < R && q < j_end) ? A[r * C + q] : 0.f;
            }
        }
        for (int i = tid; i < kTsDepth * l; i += 256) {
            const int j = i / l, c = i - j * l;
            Bs[j][c] = (j0 + j < j_end) ? B[(j0 + j) * l + c] : 0.f;
        }
        __syncthreads();
#pragma unroll 4
        for (int j = 0; j < kTsDepth; ++j) {
            float a[4], b[5];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[j][4 * og + i];
#pragma unroll
            for (int q = 0; q < 5; ++q) b[q] = (cg + 16 * q < l) ? Bs[j][cg + 16 * q] : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int q = 0; q < 5; ++q) acc[i][q] += a[i] * b[q];
        }
    }
    float* dst = part + (int64_t)blockIdx.y * out_rows * l;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t o = o0 + 4 * og + i;
        if (o >= out_rows) continue;
#pragma unroll
        for (int q = 0; q < 5; ++q)
            if (cg + 16 * q < l) dst[o * l + cg + 16 * q] = acc[i][q];
    }
}

__global__ __launch_bounds__(256) void ts_reduce_kernel(const float* __restrict__ part, int slices, int64_t n,
                                                        float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int k = 0; k < slices; ++k) s += part[(int64_t)k * n + i];
    out[i] = s;
}

// out[r][c] = sum_j X[r][j] Mx[j][c] for a small matrix Mx (l x m, both <= 80) held in LDS.
__global__ __launch_bounds__(256) void right_mul_kernel(const float* __restrict__ X, int64_t rows, int l,
                                                        const float* __restrict__ Mx, int m, float* __restrict__ out) {
    __shared__ float Ms[kTsMaxL * kTsMaxL];
    for (int i = threadIdx.x; i < l * m; i += 256) Ms[i] = Mx[i];
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
    const int cq = threadIdx.x >> 6;                  // columns cq + 4 q
    if (r >= rows) return;
    float acc[kTsMaxL / 4];
#pragma unroll
    for (int q = 0; q < kTsMaxL / 4; ++q) acc[q] = 0.f;
    for (int j = 0; j < l; ++j) {
        const float x = X[r * l + j];
#pragma unroll
        for (int q = 0; q < kTsMaxL / 4; ++q)
            if (cq + 4 * q < m) acc[q] += x * Ms[j * m + cq + 4 * q];
    }
#pragma unroll
    for (int q = 0; q < kTsMaxL / 4; ++q)
        if (cq + 4 * q < m) out[r * m + cq + 4 * q] = acc[q];
}

namespace {

struct DevBuf {                                       // frees on scope exit
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 1); }
    template <class T> T* as() const { return reinterpret_cast<T*>(p); }
};

struct TsPlan { int slices; int64_t depth_per_slice; };

// enough workgroups to fill the chip, slices a whole number of tiles deep
TsPlan ts_plan(int64_t out_rows, int64_t depth) {
    const int64_t blocks = (out_rows + kTsRows - 1) / kTsRows;
    int64_t slices = (1024 + blocks - 1) / blocks;
    const int64_t max_slices = (depth + 4 * kTsDepth - 1) / (4 * kTsDepth);
    if (slices > max_slices) slices = max_slices;
    if (slices < 1) slices = 1;
    int64_t dps = (depth + slices - 1) / slices;
    dps = (dps + kTsDepth - 1) / kTsDepth * kTsDepth;
    slices = (depth + dps - 1) / dps;
    return TsPlan{(int)slices, dps};
}

// out (out_rows x l) = A B or A^T B through partial sums in `part`
template <bool TRANS>
hipError_t ts_gemm(const float* A, int64_t R, int64_t C, const float* B, int l, float* part, float* out, hipStream_t s) {
    const int64_t out_rows = TRANS ? C : R, depth = TRANS ? R : C;
    const TsPlan p = ts_plan(out_rows, depth);
    dim3 grid((unsigned)((out_rows + kTsRows - 1) / kTsRows), (unsigned)p.slices);
    hipLaunchKernelGGL((ts_gemm_kernel<TRANS>), grid, dim3(256), 0, s, A, R, C, B, l, part, p.depth_per_slice);
    const int64_t n = out_rows * l;
    hipLaunchKernelGGL(ts_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, part, p.slices, n, out);
    return hipGetLastError();
}

size_t ts_part_floats(int64_t out_rows, int64_t depth, int l) {
    return (size_t)ts_plan(out_rows, depth).slices * out_rows * l;
}

// Upper Cholesky factor of the symmetric positive definite C (l x l): C = Rt^T Rt; returns Rt^-1
// (upper triangular) or false when C is not numerically positive definite.
bool inverse_cholesky_factor(const std::vector<double>& C, int l, std::vector<double>& Rinv) {
    std::vector<double> Rt((size_t)l * l, 0.0);
    for (int j = 0; j < l; ++j) {
        double d = C[j * l + j];
        for (int p = 0; p < j; ++p) d -= Rt[p * l + j] * Rt[p * l + j];
        if (!(d > 1e-12 * std::fabs(C[j * l + j])) || !std::isfinite(d)) return false;
        const double rjj = std::sqrt(d);
        Rt[j * l + j] = rjj;
        for (int i = j + 1; i < l; ++i) {
            double v = C[j * l + i];
            for (int p = 0; p < j; ++p) v -= Rt[p * l + j] * Rt[p * l + i];
            Rt[j * l + i] = v / rjj;
        }
    }
    Rinv.assign((size_t)l * l, 0.0);
    for (int c = 0; c < l; ++c) {                     // back substitution, column by column
        Rinv[c * l + c] = 1.0 / Rt[c * l + c];
        for (int r = c - 1; r >= 0; --r) {
            double v = 0.0;
            for (int p = r + 1; p <= c; ++p) v += Rt[r * l + p] * Rinv[p * l + c];
            Rinv[r * l + c] = -v / Rt[r * l + r];
        }
    }
    return true;
}

struct Work {                                         // device scratch of one truncated split
    float *G, *Y, *Z, *T, *part, *Cs, *Ms;
    int64_t K, N;
    int l;
    hipStream_t s;
};

// Orthonormalizes the l columns of X (rows x l) in place: X <- X Rt^-1 with Rt from the Gram
// matrix X^T X, twice (the second pass removes what the fp32 Gram matrix of the first left).
int chol_qr2(const Work& w, float* X, int64_t rows) {
    const int l = w.l;
    std::vector<float> cf((size_t)l * l);
    std::vector<double> C((size_t)l * l), Rinv;
    for (int pass = 0; pass < 2; ++pass) {
        if (ts_gemm<true>(X, rows, l, X, l, w.part, w.Cs, w.s) != hipSuccess) return LQER_ERR_HIP;
        if (hipMemcpyAsync(cf.data(), w.Cs, cf.size() * 4, hipMemcpyDeviceToHost, w.s) != hipSuccess ||
            hipStreamSynchronize(w.s) != hipSuccess)
            return LQER_ERR_HIP;
        for (size_t i = 0; i < cf.size(); ++i) C[i] = cf[i];
        if (!inverse_cholesky_factor(C, l, Rinv)) return LQER_ERR_NO_CONVERGENCE;
        for (size_t i = 0; i < cf.size(); ++i) cf[i] = (float)Rinv[i];
        if (hipMemcpyAsync(w.Ms, cf.data(), cf.size() * 4, hipMemcpyHostToDevice, w.s) != hipSuccess) return LQER_ERR_HIP;
        hipLaunchKernelGGL(right_mul_kernel, dim3((unsigned)((rows + 63) / 64)), dim3(256), 0, w.s, X, rows, l, w.Ms, l, w.T);
        if (hipMemcpyAsync(X, w.T, (size_t)rows * l * 4, hipMemcpyDeviceToDevice, w.s) != hipSuccess) return LQER_ERR_HIP;
        if (hipStreamSynchronize(w.s) != hipSuccess) return LQER_ERR_HIP;      // cf is reused by the next pass
    }
    return LQER_OK;
}

// Leading-k split of G = S E (K x N) on the device: A = S^-1 U_k (K x k), B = Sigma_k V_k^T (k x N).
int truncated_split_device(const Work& w, const std::vector<double>& s, int k, std::vector<double>& A,
                           std::vector<double>& B) {
    const int64_t K = w.K, N = w.N;
    const int l = w.l;
    const int64_t mn = K < N ? K : N;
    {
        Rng rng{0x1234ABCDull};
        std::vector<float> z0((size_t)N * l);
        for (auto& z : z0) z = (float)rng.normal();
        if (hipMemcpyAsync(w.Z, z0.data(), z0.size() * 4, hipMemcpyHostToDevice, w.s) != hipSuccess ||
            hipStreamSynchronize(w.s) != hipSuccess)
            return LQER_ERR_HIP;
    }
    if (ts_gemm<false>(w.G, K, N, w.Z, l, w.part, w.Y, w.s) != hipSuccess) return LQER_ERR_HIP;
    const int max_iter = (l == mn) ? 1 : 40;
    double prev = -1.0;
    bool converged = false;
    std::vector<float> cf((size_t)l * l), us((size_t)l * k);
    std::vector<double> C((size_t)l * l), d, V;
    for (int it = 0; it < max_iter; ++it) {
        int st = chol_qr2(w, w.Y, K);                                         // Q
        if (st != LQER_OK) return st;
        if (ts_gemm<true>(w.G, K, N, w.Y, l, w.part, w.Z, w.s) != hipSuccess) return LQER_ERR_HIP;   // Z = G^T Q
        if (ts_gemm<true>(w.Z, N, l, w.Z, l, w.part, w.Cs, w.s) != hipSuccess) return LQER_ERR_HIP;  // Z^T Z
        if (hipMemcpyAsync(cf.data(), w.Cs, cf.size() * 4, hipMemcpyDeviceToHost, w.s) != hipSuccess ||
            hipStreamSynchronize(w.s) != hipSuccess)
            return LQER_ERR_HIP;
        for (int a = 0; a < l; ++a)
            for (int b = 0; b < l; ++b) C[a * l + b] = 0.5 * ((double)cf[a * l + b] + (double)cf[b * l + a]);
        if (!jacobi_eig(C, l, d, V)) return LQER_ERR_NO_CONVERGENCE;
        std::vector<int> order(l);
        for (int i = 0; i < l; ++i) order[i] = i;
        std::sort(order.begin(), order.end(), [&](int a, int b) { return d[a] > d[b]; });
        double energy = 0.0;
        for (int i = 0; i < k; ++i) energy += d[order[i]];
        for (int i = 0; i < k; ++i)
            for (int r = 0; r < l; ++r) us[(size_t)r * k + i] = (float)V[r * l + order[i]];
        // fp32 products: the energy is known to about 1e-6 of itself
        if (l == mn || (prev >= 0.0 && energy - prev <= 1e-5 * energy)) {
            converged = true;
            break;
        }
        prev = energy;
        st = chol_qr2(w, w.Z, N);
        if (st != LQER_OK) return st;
        if (ts_gemm<false>(w.G, K, N, w.Z, l, w.part, w.Y, w.s) != hipSuccess) return LQER_ERR_HIP;
    }
    if (!converged) return LQER_ERR_NO_CONVERGENCE;
    // Y holds Q (K x l), Z = G^T Q (N x l): A = S^-1 Q Us, B = (Z Us)^T
    std::vector<float> ya((size_t)K * k), zb((size_t)N * k);
    if (hipMemcpyAsync(w.Ms, us.data(), us.size() * 4, hipMemcpyHostToDevice, w.s) != hipSuccess) return LQER_ERR_HIP;
    hipLaunchKernelGGL(right_mul_kernel, dim3((unsigned)((K + 63) / 64)), dim3(256), 0, w.s, w.Y, K, l, w.Ms, k, w.T);
    if (hipMemcpyAsync(ya.data(), w.T, ya.size() * 4, hipMemcpyDeviceToHost, w.s) != hipSuccess) return LQER_ERR_HIP;
    hipLaunchKernelGGL(right_mul_kernel, dim3((unsigned)((N + 63) / 64)), dim3(256), 0, w.s, w.Z, N, l, w.Ms, k, w.T);
    if (hipMemcpyAsync(zb.data(), w.T, zb.size() * 4, hipMemcpyDeviceToHost, w.s) != hipSuccess ||
        hipStreamSynchronize(w.s) != hipSuccess)
        return LQER_ERR_HIP;
    A.assign((size_t)K * k, 0.0);
    for (int64_t i = 0; i < K; ++i)
        for (int c = 0; c < k; ++c) A[i * k + c] = (double)ya[i * k + c] / s[i];
    B.assign((size_t)k * N, 0.0);
    for (int64_t j = 0; j < N; ++j)
        for (int c = 0; c < k; ++c) B[(size_t)c * N + j] = (double)zb[j * k + c];
    return LQER_OK;
}

}  // namespace
}  // namespace lqer

using namespace lqer;

extern "C" int lqer_build_factors_device(const float* W_dev, int64_t K, int64_t N, const float* calib_dev,
                                         int64_t n_samples, int64_t rows_per_sample, int k, int mode,
                                         const lqer_config* cfg, void* hip_stream, lqer_layer** out) try {
    if (!out) return LQER_ERR_NULL;
    *out = nullptr;
    if (cfg && (cfg->w_bits != 4 || cfg->h_bits != 8 || (cfg->exp_bits != 8 && cfg->exp_bits != 4) || cfg->block != 16))
        return LQER_ERR_UNSUPPORTED;
    const int exp_bits = cfg ? cfg->exp_bits : 8;
    if (K <= 0 || N <= 0 || (K & 15) != 0 || k < 0 || k > K || k > N) return LQER_ERR_SHAPE;
    if (mode != 0 && mode != 1) return LQER_ERR_UNSUPPORTED;
    if (!W_dev) return LQER_ERR_NULL;
    if (mode == 1 && (!calib_dev || n_samples <= 0 || rows_per_sample <= 0))
        return calib_dev ? LQER_ERR_SHAPE : LQER_ERR_NULL;
    const int kp = (k + 15) / 16 * 16;
    if (kp > 64) return LQER_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t nblk = K / 16;

    // S (App. A)
    std::vector<double> sc((size_t)K, 1.0);
    if (mode == 1) {
        DevBuf ab;
        if (ab.alloc((size_t)K * 8) != hipSuccess) return LQER_ERR_HIP;
        hipLaunchKernelGGL(calib_magnitude_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, s, calib_dev,
                           n_samples, rows_per_sample, K, ab.as<double>());
        std::vector<double> abar((size_t)K);
        if (hipGetLastError() != hipSuccess ||
            hipMemcpyAsync(abar.data(), ab.p, (size_t)K * 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return LQER_ERR_HIP;
        const int st = scale_from_magnitudes(abar, sc);
        if (st != LQER_OK) return st;
    }

    // W_q and G = S (W - W_q)
    const int l = (int)std::min<int64_t>(k + 16, std::min(K, N));
    DevBuf dWc, dWe, dS, dG, dFlag;
    if (dWc.alloc((size_t)N * (K / 2)) != hipSuccess || dWe.alloc((size_t)N * nblk) != hipSuccess ||
        dS.alloc((size_t)K * 4) != hipSuccess || dFlag.alloc(8) != hipSuccess ||
        (k > 0 && dG.alloc((size_t)K * N * 4) != hipSuccess))
        return LQER_ERR_HIP;
    {
        std::vector<float> sf((size_t)K);
        for (int64_t i = 0; i < K; ++i) sf[i] = (float)sc[i];
        if (hipMemcpyAsync(dS.p, sf.data(), (size_t)K * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemsetAsync(dFlag.p, 0, 8, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
            return LQER_ERR_HIP;
    }
    uint32_t* amax_bits = nullptr;                   // the second word of dFlag
    if (exp_bits == 4) {
        amax_bits = reinterpret_cast<uint32_t*>(dFlag.p) + 1;
        hipLaunchKernelGGL(absmax_bits_kernel, dim3(1024), dim3(256), 0, s, W_dev, K * N, amax_bits);
    }
    hipLaunchKernelGGL(quantize_w_kernel, dim3((unsigned)((N + 255) / 256), (unsigned)nblk), dim3(256), 0, s, W_dev, K, N,
                       dS.as<float>(), dWc.as<uint8_t>(), dWe.as<uint8_t>(), k > 0 ? dG.as<float>() : nullptr,
                       dFlag.as<int>(), amax_bits);
    std::vector<uint8_t> Wc((size_t)N * (K / 2)), We((size_t)N * nblk);
    int flag = 0;
    if (hipGetLastError() != hipSuccess ||
        hipMemcpyAsync(&flag, dFlag.p, 4, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(Wc.data(), dWc.p, Wc.size(), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(We.data(), dWe.p, We.size(), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return LQER_ERR_HIP;
    if (flag) return LQER_ERR_VALUE;

    std::vector<double> A, B;
    if (k > 0) {
        const int64_t big = std::max(K, N);
        const size_t part_floats = std::max(std::max(ts_part_floats(K, N, l), ts_part_floats(N, K, l)),
                                            std::max(ts_part_floats(l, K, l), ts_part_floats(l, N, l)));
        DevBuf dY, dZ, dT, dPart, dCs, dMs;
        if (dY.alloc((size_t)K * l * 4) != hipSuccess || dZ.alloc((size_t)N * l * 4) != hipSuccess ||
            dT.alloc((size_t)big * l * 4) != hipSuccess || dPart.alloc(part_floats * 4) != hipSuccess ||
            dCs.alloc((size_t)l * l * 4) != hipSuccess || dMs.alloc((size_t)kTsMaxL * kTsMaxL * 4) != hipSuccess)
            return LQER_ERR_HIP;
        Work w{dG.as<float>(), dY.as<float>(), dZ.as<float>(), dT.as<float>(), dPart.as<float>(), dCs.as<float>(),
               dMs.as<float>(), K, N, l, s};
        const int st = truncated_split_device(w, sc, k, A, B);
        if (st != LQER_OK) return st;
    }
    return pack_factors_and_import(K, N, k, Wc, We, A, B, exp_bits, out);
} catch (...) {                                      // a host allocation failed: nothing may leave through the C ABI
    return LQER_ERR_NO_MEMORY;
}
