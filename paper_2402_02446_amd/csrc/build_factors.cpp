// Offline construction of an LQER / L2QER layer on the host (Sec. 3.1 Eq. 1-2; Sec. 3.2 Eq. 4-5;
// App. A Eq. 7-8), in fp64:
//   W_q = q(W) in MXINT4 (blocks of 16 down each column, Sec. 4.1), E_q = W - W_q,
//   S from the calibration samples, the k leading singular triplets of S E_q,
//   A_k = S^-1 U_k, B_k = Sigma_k V_k^T, both quantized to MXINT8.
// The truncated SVD is a randomized block subspace iteration (range finder with power
// iterations, then an exact eigen-decomposition of the small projected Gram matrix by cyclic
// Jacobi), iterated until the energy captured by the leading k directions stops growing.
#include <cmath>
#include <cstring>
#include <vector>

#include "lqer_internal.h"
#include "host_parallel.h"
#include "build_common.h"

namespace lqer {

// ---- small dense helpers ------------------------------------------------------------------------
// Orthonormalize the l columns of Y (rows x l, row-major) with two passes of modified Gram-Schmidt.
static void orthonormalize(std::vector<double>& Y, int64_t rows, int l) {
    std::vector<double> col(rows);
    for (int j = 0; j < l; ++j) {
        for (int pass = 0; pass < 2; ++pass) {
            for (int i = 0; i < j; ++i) {
                double dot = 0.0;
                for (int64_t r = 0; r < rows; ++r) dot += Y[r * l + i] * Y[r * l + j];
                for (int64_t r = 0; r < rows; ++r) Y[r * l + j] -= dot * Y[r * l + i];
            }
        }
        double nrm = 0.0;
        for (int64_t r = 0; r < rows; ++r) nrm += Y[r * l + j] * Y[r * l + j];
        nrm = std::sqrt(nrm);
        const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
        for (int64_t r = 0; r < rows; ++r) Y[r * l + j] *= inv;
    }
}

// C (K x l) = G (K x N) * Z (N x l)
static void gemm_nn(const std::vector<double>& G, int64_t K, int64_t N, const std::vector<double>& Z, int l,
                    std::vector<double>& C) {
    C.assign((size_t)K * l, 0.0);
    parallel_for(K, [&](int64_t i) {
        double* c = &C[(size_t)i * l];
        const double* g = &G[(size_t)i * N];
        for (int64_t j = 0; j < N; ++j) {
            const double gij = g[j];
            const double* z = &Z[(size_t)j * l];
            for (int t = 0; t < l; ++t) c[t] += gij * z[t];
        }
    }, 16);
}

// Z (N x l) = G^T (N x K) * Y (K x l)
static void gemm_tn(const std::vector<double>& G, int64_t K, int64_t N, const std::vector<double>& Y, int l,
                    std::vector<double>& Z) {
    Z.assign((size_t)N * l, 0.0);
    const int64_t jb = 64;
    const int64_t nblocks = (N + jb - 1) / jb;
    parallel_for(nblocks, [&](int64_t b) {
        const int64_t j0 = b * jb, j1 = std::min(N, j0 + jb);
        for (int64_t i = 0; i < K; ++i) {
            const double* y = &Y[(size_t)i * l];
            const double* g = &G[(size_t)i * N];
            for (int64_t j = j0; j < j1; ++j) {
                const double gij = g[j];
                double* z = &Z[(size_t)j * l];
                for (int t = 0; t < l; ++t) z[t] += gij * y[t];
            }
        }
    });
}

// Leading-k split of G = S E (K x N): A = S^-1 U_k (K x k), B = Sigma_k V_k^T (k x N).
int truncated_split(const std::vector<double>& G, int64_t K, int64_t N, const std::vector<double>& s,
                           int k, std::vector<double>& A, std::vector<double>& B) {
    const int64_t mn = std::min(K, N);
    int l = k + 16;
    if (l > mn) l = (int)mn;
    Rng rng{0x1234ABCDull};
    std::vector<double> Z((size_t)N * l), Y, Bs, C((size_t)l * l), d, V;
    for (auto& z : Z) z = rng.normal();
    gemm_nn(G, K, N, Z, l, Y);
    double prev = -1.0;
    const int max_iter = (l == mn) ? 1 : 60;
    bool converged = false;
    std::vector<double> Us;
    for (int it = 0; it < max_iter; ++it) {
        orthonormalize(Y, K, l);                      // Q
        gemm_tn(G, K, N, Y, l, Z);                    // Z = G^T Q   (N x l);  B_small = Z^T
        // Gram matrix of the projected rows: C = Z^T Z = B_small B_small^T
        for (int a = 0; a < l; ++a)
            for (int b = a; b < l; ++b) {
                double acc = 0.0;
                for (int64_t j = 0; j < N; ++j) acc += Z[j * l + a] * Z[j * l + b];
                C[a * l + b] = C[b * l + a] = acc;
            }
        std::vector<double> Cw = C;
        if (!jacobi_eig(Cw, l, d, V)) return LQER_ERR_NO_CONVERGENCE;
        std::vector<int> order(l);
        for (int i = 0; i < l; ++i) order[i] = i;
        std::sort(order.begin(), order.end(), [&](int a, int b) { return d[a] > d[b]; });
        double energy = 0.0;
        for (int i = 0; i < k; ++i) energy += d[order[i]];
        Us.assign((size_t)l * k, 0.0);
        for (int i = 0; i < k; ++i)
            for (int r = 0; r < l; ++r) Us[r * k + i] = V[r * l + order[i]];
        if (l == mn || (prev >= 0.0 && energy - prev <= 1e-7 * energy)) {
            converged = true;
            break;
        }
        prev = energy;
        // power step: Y = G (G^T Q) with the fresh Z, re-orthonormalized for stability
        orthonormalize(Z, N, l);
        gemm_nn(G, K, N, Z, l, Y);
    }
    if (!converged) return LQER_ERR_NO_CONVERGENCE;
    // here Y holds Q (orthonormal, K x l) and Z = G^T Q from the last pass
    A.assign((size_t)K * k, 0.0);
    for (int64_t i = 0; i < K; ++i)
        for (int c = 0; c < k; ++c) {
            double acc = 0.0;
            for (int r = 0; r < l; ++r) acc += Y[i * l + r] * Us[r * k + c];
            A[i * k + c] = acc / s[i];
        }
    B.assign((size_t)k * N, 0.0);
    for (int64_t j = 0; j < N; ++j)
        for (int c = 0; c < k; ++c) {
            double acc = 0.0;
            for (int r = 0; r < l; ++r) acc += Us[r * k + c] * Z[j * l + r];
            B[(size_t)c * N + j] = acc;
        }
    return LQER_OK;
}

// A (K x k) and B (k x N) -> MXINT8 bytes in the canonical layouts, then the layer handle.
int pack_factors_and_import(int64_t K, int64_t N, int k, const std::vector<uint8_t>& Wc, const std::vector<uint8_t>& We,
                            const std::vector<double>& A, const std::vector<double>& B, int exp_bits, lqer_layer** out,
                            int w_bits) {
    const int kp = (k + 15) / 16 * 16;
    const int64_t nblk = K / 16;
    std::vector<int8_t> Ac, Bc;
    std::vector<uint8_t> Ae, Be;
    if (k > 0) {
        // A_k: K x k -> MXINT8 blocks down K, stored [kp][K]
        // (the zero rows and columns of the padding are blocks of the tensor like any other: exponent -127)
        Ac.assign((size_t)kp * K, 0);
        Ae.assign((size_t)kp * nblk, 0);
        int top = -127;
        for (int r = 0; r < k; ++r)
            for (int64_t kb = 0; kb < nblk; ++kb) top = std::max(top, mx_block_exponent(&A[(size_t)kb * 16 * k + r], k));
        const int a_floor = mx_exponent_floor(top, exp_bits);
        for (int r = 0; r < kp; ++r)
            for (int64_t kb = 0; kb < nblk; ++kb) {
                if (r < k) mx_block(&A[(size_t)kb * 16 * k + r], k, 8, &Ac[(size_t)r * K + kb * 16], &Ae[(size_t)r * nblk + kb], a_floor);
                else Ae[(size_t)r * nblk + kb] = (uint8_t)(a_floor + 127);
            }
        // B_k: k x N (zero padded to kp) -> MXINT8 blocks down k, stored [N][kp]
        Bc.assign((size_t)N * kp, 0);
        Be.assign((size_t)N * (kp / 16), 0);
        std::vector<double> colb(16);
        auto b_block = [&](int64_t n, int rb) {
            for (int i = 0; i < 16; ++i) {
                const int r = rb * 16 + i;
                colb[i] = (r < k) ? B[(size_t)r * N + n] : 0.0;
            }
        };
        top = -127;
        for (int64_t n = 0; n < N; ++n)
            for (int rb = 0; rb < kp / 16; ++rb) {
                b_block(n, rb);
                top = std::max(top, mx_block_exponent(colb.data(), 1));
            }
        const int b_floor = mx_exponent_floor(top, exp_bits);
        for (int64_t n = 0; n < N; ++n)
            for (int rb = 0; rb < kp / 16; ++rb) {
                b_block(n, rb);
                mx_block(colb.data(), 1, 8, &Bc[(size_t)n * kp + rb * 16], &Be[(size_t)n * (kp / 16) + rb], b_floor);
            }
    }
    return lqer_layer_import_w(w_bits, K, N, k, Wc.data(), We.data(), k > 0 ? Ac.data() : nullptr,
                               k > 0 ? Ae.data() : nullptr, k > 0 ? Bc.data() : nullptr,
                               k > 0 ? Be.data() : nullptr, out);
}

// S of App. A from the per-channel magnitudes abar (maximum over samples of the mean |x|): geometric-mean normalisation.
int scale_from_magnitudes(const std::vector<double>& abar, std::vector<double>& s) {
    const int64_t K = (int64_t)abar.size();
    double lo = abar[0], hi = abar[0];
    for (int64_t c = 0; c < K; ++c) {
        if (!(abar[c] > 0.0) || !std::isfinite(abar[c])) return LQER_ERR_SINGULAR_SCALE;
        lo = std::min(lo, abar[c]);
        hi = std::max(hi, abar[c]);
    }
    const double norm = std::sqrt(lo * hi);
    if (!(norm > 0.0) || !std::isfinite(norm)) return LQER_ERR_SINGULAR_SCALE;
    s.resize((size_t)K);
    for (int64_t c = 0; c < K; ++c) s[c] = abar[c] / norm;
    return LQER_OK;
}

}  // namespace lqer

using namespace lqer;

extern "C" int lqer_build_factors(const float* W_host, int64_t K, int64_t N, const float* calib_host,
                                  int64_t n_samples, int64_t rows_per_sample, int k, int mode,
                                  const lqer_config* cfg, lqer_layer** out) try {
    if (!out) return LQER_ERR_NULL;
    *out = nullptr;
    // {4, 8, 16, 128}: the scaled-integer variant (Table 2 "L2QER-INT": INT4 weights in groups of 128 with FP16 scales)
    const bool int_format = cfg && cfg->w_bits == 4 && cfg->h_bits == 8 && cfg->exp_bits == 16 && cfg->block == 128;
    if (cfg && !int_format &&
        ((cfg->w_bits != 4 && cfg->w_bits != 2) || cfg->h_bits != 8 || (cfg->exp_bits != 8 && cfg->exp_bits != 4) || cfg->block != 16))
        return LQER_ERR_UNSUPPORTED;
    const int exp_bits = cfg ? cfg->exp_bits : 8;
    const int w_bits = cfg ? cfg->w_bits : 4;
    if (K <= 0 || N <= 0 || (K & 15) != 0 || k < 0 || k > K || k > N) return LQER_ERR_SHAPE;
    if (mode != 0 && mode != 1) return LQER_ERR_UNSUPPORTED;
    if (!W_host) return LQER_ERR_NULL;
    if (mode == 1 && (!calib_host || n_samples <= 0 || rows_per_sample <= 0))
        return calib_host ? LQER_ERR_SHAPE : LQER_ERR_NULL;
    const int kp = (k + 15) / 16 * 16;
    if (kp > kMaxRank) return LQER_ERR_UNSUPPORTED;
    const int64_t nblk = K / 16;

    // S (App. A): per-sample mean magnitude, maximum over samples, geometric-mean normalisation
    std::vector<double> s((size_t)K, 1.0);
    if (mode == 1) {
        std::vector<double> abar((size_t)K, 0.0);
        for (int64_t i = 0; i < n_samples; ++i) {
            std::vector<double> a((size_t)K, 0.0);
            for (int64_t r = 0; r < rows_per_sample; ++r) {
                const float* row = calib_host + ((size_t)i * rows_per_sample + r) * K;
                for (int64_t c = 0; c < K; ++c) a[c] += std::fabs((double)row[c]);
            }
            for (int64_t c = 0; c < K; ++c) abar[c] = std::max(abar[c], a[c] / (double)rows_per_sample);
        }
        const int st = scale_from_magnitudes(abar, s);
        if (st != LQER_OK) return st;
    }

    if (int_format) return build_factors_int(W_host, K, N, s, k, out);

    // W_q and G = S (W - W_q)
    const int64_t wc_row = w_bits == 4 ? K / 2 : K / 4;      // bytes of one column's codes
    std::vector<uint8_t> Wc((size_t)N * wc_row), We((size_t)N * nblk);
    std::vector<double> G;
    if (k > 0) G.resize((size_t)K * N);
    for (int64_t i = 0; i < K * N; ++i)
        if (!std::isfinite(W_host[i])) return LQER_ERR_VALUE;
    // 4-bit shared exponents: the exponent of the tensor's largest block fixes the lowest one that can be stored
    int w_floor = -127;
    if (exp_bits == 4) {
        float amax = 0.f;
        for (int64_t i = 0; i < K * N; ++i) amax = std::max(amax, std::fabs(W_host[i]));
        const double one[16] = {(double)amax};
        w_floor = mx_exponent_floor(mx_block_exponent(one, 1), exp_bits);
    }
    parallel_for(N, [&](int64_t n) {
        double col[16];
        int8_t codes[16];
        for (int64_t kb = 0; kb < nblk; ++kb) {
            for (int i = 0; i < 16; ++i) col[i] = (double)W_host[(kb * 16 + i) * N + n];
            uint8_t eb;
            mx_block(col, 1, w_bits, codes, &eb, w_floor);
            We[n * nblk + kb] = eb;
            if (w_bits == 4) {
                for (int i = 0; i < 8; ++i)
                    Wc[n * wc_row + kb * 8 + i] = (uint8_t)((codes[2 * i] & 0xF) | ((codes[2 * i + 1] & 0xF) << 4));
            } else {
                for (int i = 0; i < 4; ++i)
                    Wc[n * wc_row + kb * 4 + i] = (uint8_t)((codes[4 * i] & 3) | ((codes[4 * i + 1] & 3) << 2) |
                                                            ((codes[4 * i + 2] & 3) << 4) | ((codes[4 * i + 3] & 3) << 6));
            }
            if (k > 0) {
                const double scale = std::ldexp(1.0, (int)eb - 127 - (w_bits - 2));
                for (int i = 0; i < 16; ++i) {
                    const int64_t row = kb * 16 + i;
                    G[(size_t)row * N + n] = s[row] * (col[i] - codes[i] * scale);
                }
            }
        }
    }, 8);

    std::vector<double> A, B;
    if (k > 0) {
        const int st = truncated_split(G, K, N, s, k, A, B);
        if (st != LQER_OK) return st;
        G.clear();
        G.shrink_to_fit();
    }
    return pack_factors_and_import(K, N, k, Wc, We, A, B, exp_bits, out, w_bits);
} catch (...) {                                      // a host allocation failed: nothing may leave through the C ABI
    return LQER_ERR_NO_MEMORY;
}
