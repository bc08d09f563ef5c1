// Host-side pieces shared by the two offline constructions (host fp64, and device GEMMs with the
// small dense steps on the host): MXINT block quantization, symmetric eigen-decomposition, the
// reproducible normal stream of the range finder.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

namespace lqer {

// ---- MXINT quantization of one block of 16 doubles (Sec. 2.2 / 4.1 reading, see lqer.h) ---------
// The block's own shared exponent: floor(log2 max|v|) clamped to [-127, 127], -127 for an all-zero block.
inline int mx_block_exponent(const double* v, int stride) {
    double amax = 0.0;
    for (int i = 0; i < 16; ++i) amax = std::max(amax, std::fabs(v[i * stride]));
    int e = -127;
    if (amax > 0.0) {
        int ex;
        (void)std::frexp(amax, &ex);          // amax = m * 2^ex, m in [0.5, 1)
        e = ex - 1;
        if (e < -127) e = -127;
        if (e > 127) e = 127;
    }
    return e;
}

// Lowest exponent a tensor with `exp_bits`-bit shared exponents can store when its largest block has
// exponent `top`: 4-bit exponents reach 15 binades below the largest block (one bias per tensor).
inline int mx_exponent_floor(int top, int exp_bits) {
    return exp_bits == 4 ? std::max(top - 15, -127) : -127;
}

// e_floor: blocks below it are quantized with e_floor (4-bit shared exponents; -127 = no floor).
inline void mx_block(const double* v, int stride, int bits, int8_t* codes, uint8_t* ebyte, int e_floor = -127) {
    int e = mx_block_exponent(v, stride);
    if (e < e_floor) e = e_floor;
    const int lim = (1 << (bits - 1)) - 1;
    for (int i = 0; i < 16; ++i) {
        double r = std::nearbyint(std::ldexp(v[i * stride], (bits - 2) - e));   // ties to even
        if (r > lim) r = lim;
        if (r < -lim) r = -lim;
        codes[i] = (int8_t)r;
    }
    *ebyte = (uint8_t)(e + 127);
}

// Symmetric eigen-decomposition by cyclic Jacobi: A (l x l, destroyed) -> eigenvalues d, vectors V (columns).
inline bool jacobi_eig(std::vector<double>& A, int l, std::vector<double>& d, std::vector<double>& V) {
    V.assign((size_t)l * l, 0.0);
    for (int i = 0; i < l; ++i) V[i * l + i] = 1.0;
    for (int sweep = 0; sweep < 100; ++sweep) {
        double off = 0.0, diag = 0.0;
        for (int i = 0; i < l; ++i)
            for (int j = 0; j < l; ++j) (i == j ? diag : off) += A[i * l + j] * A[i * l + j];
        if (off <= 1e-30 * diag || off == 0.0) {
            d.resize(l);
            for (int i = 0; i < l; ++i) d[i] = A[i * l + i];
            return true;
        }
        for (int p = 0; p < l - 1; ++p)
            for (int q = p + 1; q < l; ++q) {
                const double apq = A[p * l + q];
                if (apq == 0.0) continue;
                const double theta = (A[q * l + q] - A[p * l + p]) / (2.0 * apq);
                const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
                const double c = 1.0 / std::sqrt(t * t + 1.0), s = t * c;
                for (int i = 0; i < l; ++i) {
                    const double aip = A[i * l + p], aiq = A[i * l + q];
                    A[i * l + p] = c * aip - s * aiq;
                    A[i * l + q] = s * aip + c * aiq;
                }
                for (int i = 0; i < l; ++i) {
                    const double api = A[p * l + i], aqi = A[q * l + i];
                    A[p * l + i] = c * api - s * aqi;
                    A[q * l + i] = s * api + c * aqi;
                }
                for (int i = 0; i < l; ++i) {
                    const double vip = V[i * l + p], viq = V[i * l + q];
                    V[i * l + p] = c * vip - s * viq;
                    V[i * l + q] = s * vip + c * viq;
                }
            }
    }
    return false;
}

// splitmix64 -> standard normal (Box-Muller); a fixed stream so the build is reproducible.
struct Rng {
    uint64_t s;
    uint64_t next() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return ((next() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
    double normal() {
        const double u = uniform(), v = uniform();
        return std::sqrt(-2.0 * std::log(u)) * std::cos(6.283185307179586 * v);
    }
};

}  // namespace lqer
