// Internal declarations shared by the host side and the kernel launchers of liblqer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>
#include "lqer.h"

namespace lqer { struct Layer; }

namespace lqer {

// ---- internal device layout of one layer ------------------------------------------------
//
// The main kernels use the 32x32x16 bf16 MFMA with the weights as its first operand: lane
// (i = lane % 32, hh = lane / 32) supplies 8 consecutive K elements of output column i, and the
// 16-wide K step splits between the two lane halves.  The K axis is permuted inside every
// 64-wide chunk so that a lane owns whole MXINT blocks: in MFMA step s (0..3) of a chunk, lane
// half hh covers k = 32 hh + 8 s .. + 7, i.e. hh owns blocks 2hh and 2hh+1 of the chunk and no
// block scale ever crosses lanes.  Activations follow the same permutation simply by reading
// 16 bytes at that offset.
//
// W_q record = [32 columns] x [256 K], 4608 B, read by one wavefront with coalesced 16-byte loads:
//   codes[4 chunks][64 lanes][16 B]  lane's 16 B = blocks (4c + 2hh), (4c + 2hh + 1) of the tile,
//                                    two 32-bit words (8 elements each) per block
//   exps[64 lanes][8 B]              byte 2c + j = exponent byte of block 4c + 2hh + j
//   records are ordered [K tile][column group]: what the streaming kernel reads at one time is then one
//   contiguous range (a few percent more HBM bandwidth than group-major order).
//   Compact form (chosen at import when the layer's exponent bytes span at most 16 values, which real
//   weight matrices do): exps[64 lanes][4 B] in front of the codes, nibble 2c + j = exponent byte of block
//   4c + 2hh + j minus the layer's smallest exponent byte; 4352 B per record, 0.53125 B per weight - the footprint of
//   the 4-bit shared exponents Sec. 4.1 gives the weights.  The canonical bytes are unchanged.
//
// A 32-bit code word holds 8 consecutive K elements e0..e7 as sign-magnitude nibbles placed so
// that two mask operations yield fp8 (E4M3) subnormal bytes  s0000mmm = +-m * 2^-9:
//   byte i:  bit 7 = sign(e_i), bits 6..4 = |e_{4+i}|, bit 3 = sign(e_{4+(i+3)%4}), bits 2..0 = |e_i|
//   r0 = w & 0x87878787            -> bytes e0 e1 e2 e3
//   r1 = rotr(w, 4) & 0x87878787   -> bytes e4 e5 e6 e7
// The MX scale-and-convert instruction then turns two such bytes into two bf16 values
// code * 2^(e-2) exactly.
//
// A_k (used by the projection kernel with the 16x16x32 MFMA, lane = c + 16 q owning blocks
//      q + 4p): records of [16 ranks] x [256 K] holding the dequantized values code * 2^(e-6) as
//      bf16 (exact): values[8][64 lanes][16 B], entry 2p + h = half h (8 elements) of block q + 4p;
//      ordered [rank group][K tile].  The exponent bytes stay on the host for export.  A_k is
//      K*kp elements, well under 1 % of the layer, so the extra byte per element is negligible and
//      the projection kernel needs no conversion at all.
// B_k: records of [32 columns] x [16 ranks] (one MXINT block per column): codes[32 columns][16 B]
//      + exps[32 columns][1 B]; ordered [column group][rank block].

// 2-bit weights (the W2A8 setup of Sec. 4.1 / Sec. 4.4): the same record with half the code bytes,
//   codes[2 halves][64 lanes][16 B]   lane's 16 B of half h = its blocks of chunks 2h and 2h+1, one 32-bit word per
//                                     block: words (chunk 2h: block 2hh, 2hh+1; chunk 2h+1: block 2hh, 2hh+1)
//   and the exponents as above (512 B of bytes behind the codes, or 256 B of nibbles in front): 2560 / 2304 B.
// A word holds the block's 16 codes e0..e15 (-1, 0, 1) as sign and magnitude bits placed so that a rotation and
// one mask yield four fp8 (E4M3) subnormal bytes s0000001 = +-2^-9:
//   magnitude of e[4x + i] at bit 8 i + 2 x, its sign at bit (8 i + 2 x + 7) mod 32        (x, i = 0..3)
//   rotr(w, 2 x) & 0x81818181  -> bytes e[4x], e[4x+1], e[4x+2], e[4x+3]
// MFMA step s of a chunk uses elements 8 (s % 2) .. + 7 of block s / 2: extractions x = 2 (s % 2) and x + 1.

constexpr int kTileK = 256;          // K covered by one W / A record
constexpr int kWRecordBytes = 4608;  // with one exponent byte per block
constexpr int kWRecordBytesCompact = 4352;   // with exponent nibbles (below)
constexpr int kWExpOffset = 4096;     // exponent bytes sit behind the codes; exponent nibbles (256 B) in front of them:
constexpr int kWCompactCodeOffset = 256;   // their 8-byte reads then run over into a line the wavefront needs anyway
// bytes of a record's codes, its size with exponent bytes / nibbles, for b-bit weights (b = 4 or 2)
constexpr int w_code_bytes(int bits) { return bits == 4 ? 4096 : 2048; }
constexpr int w_record_bytes(int bits, bool compact) { return w_code_bytes(bits) + (compact ? 256 : 512); }
constexpr int kMaxRank = 256;        // padded rank kp the kernels take (Sec. 4.1 runs W2A8 with k = 256)
constexpr int kWTailPad = 16;        // bytes behind the last record: exponent words are read 8 bytes wide in both forms
constexpr int kARecordBytes = 8192;
constexpr int kBRecordBytes = 544;
constexpr int kMaxWExpByte = 245;    // (byte + 7), for 2-bit weights (byte + 9), must stay a finite fp32 exponent field

struct Layer {
    int64_t K, N;
    int k, kp;
    int64_t KT;        // K tiles of 256
    int64_t N32;       // column groups of 32
    int kp16;          // rank groups (= MXINT blocks along k) of 16
    int device;
    int w_bits;        // mantissa width of W_q: 4 or 2
    int w_rec_bytes;   // w_record_bytes(w_bits, compact)
    int w_exp_bias;    // compact records: exponent byte = nibble + this; -1: one byte per block
    int act_bits;      // width of the activation codes: 8 or 6
    uint8_t* Wt;       // device, N32*KT records
    uint8_t* At;       // device, kp16*KT records
    uint8_t* Bt;       // device, N32*kp16 records
    // The scaled-integer variant (Table 2 "L2QER-INT"; kernels_int.hip): format 1.  Wt then holds [N32][K/128] records of
    // canonical nibbles ([2 spans of 64 K][64 lanes][16 B]), At [kp32][K/128] records of int8 codes ([4][64 lanes][16 B],
    // K permuted like the activations), Bt the B_k records above (exponent bytes unused), and the scale tables are fp32:
    int format;        // 0 = MXINT, 1 = INT (INT4 g128 weights, INT8 g128 factors, INT8 per-token activations)
    int kp32;          // INT: rank groups of 32 (the projection's output columns)
    float* Wsc;        // INT: [N32][K/128][32], W_q's FP16 scales divided by 16 (the kernel multiplies codes by 16)
    float* Asc;        // INT: [kp32][K/128][32]
    float* Bsc;        // INT: [N32 * 32]
};

// Workspace layout for one forward call.
struct Workspace {
    int64_t ldxh;        // row stride of Xh in bf16 elements = KT*256 + roundup(2*kp, 64)
    int S;               // K slices of the T partial sums (1 = T final, written into Xh)
    uint16_t* Xh;        // [M][ldxh] bf16 : dequantized X_q | T_hi | T_lo; or cells (below)
    float* Tpart;        // [S][tp_rows][kp] fp32 partial sums of T, or null when T is final in Xh
    int64_t tp_rows;     // rows per slice of Tpart (M, or M padded to the tile height for the tiled kernel)
    bool cells;          // streaming kernel: Xh holds 16-byte cells [KT*32][1 << lr token rows]
    int lr;
    bool x8;             // streaming kernel: the cells hold MXINT8 codes and exponent bytes (set per launch)
    float* Part;         // tiled kernel: accumulators handed from one workgroup to another, or null
    uint32_t* flags;     // tiled kernel: kTiledFlags words, cleared by the projection kernel
    size_t bytes;
};

// The tiled kernel may cut output tiles along K between workgroups; each workgroup resident on the
// chip then has one slot of tile size in the workspace: 256 KiB per compute unit covers every tile
// shape (128 x 512 with one workgroup per compute unit, 128 x 256 with two).
constexpr int64_t kTiledPartBytesPerCu = 256 * 1024;
constexpr int kTiledFlags = 1024;

}  // namespace lqer

struct lqer_layer {
    lqer::Layer L;
    std::vector<uint8_t> Ae_host;     // A_k's exponent bytes [kp][K/16], needed again only by export
    // INT layers keep their canonical arrays for export
    std::vector<uint8_t> iWc;
    std::vector<int8_t> iAc, iBc;
    std::vector<uint16_t> iWs, iAs, iBs;
};

namespace lqer {

// ---- kernel launchers (each returns the hipError_t of its launch) ------------------------
hipError_t launch_quantize_mx(const float* x, int64_t rows, int64_t cols, int64_t ld, int bits,
                              void* codes, uint8_t* exps, hipStream_t s);

// Quantize X (or take codes) -> Xh bf16, and T = X_q A_k.  S == 1 writes T_hi/T_lo into Xh,
// S > 1 writes fp32 partial sums per K slice.
// y_zero != null: also clears Y[M][N] (row stride ldy) for a main kernel that adds into it.
// Clears ws.flags when the workspace has them.
// reuse_xh (tiled path, X and Xc null): Xh already holds these activations from an earlier launch with the same
// workspace plan; only T is computed, for another layer applied to them.
hipError_t launch_prep(const Layer& L, const float* X, int64_t ldx, const int8_t* Xc, const uint8_t* Xe,
                       int64_t M, const Workspace& ws, float* y_zero, int64_t ldy, hipStream_t s, bool reuse_xh = false);

// Output of the main kernels as MXINT8 (blocks of 16 along N) instead of fp32 Y; codes == null: fp32.
struct Requant {
    int8_t* codes;       // [M][ld] int8
    uint8_t* exps;       // [M][N/16]
    int64_t ld;
};

// Streaming (small M) main kernel.  variant 0 = automatic.
hipError_t launch_stream(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy, const Requant& rq,
                         int variant, hipStream_t s);
int stream_variant_unpaired(const Layer& L, int64_t M);                          // the shape used when pairs of workgroups are ruled out
int stream_max_rows();
int stream_variant(const Layer& L, int64_t M, int variant);      // resolves 0 = automatic
bool stream_variant_adds_into_y(int variant);                    // Y must be zero before the launch
bool stream_takes_codes(int variant, int lr);                    // activations as MXINT8 codes + exponent bytes instead of bf16 cells
int stream_cell_rows_log2(int64_t M);
// Tiled MFMA (large M) main kernel.
hipError_t launch_tiled(const Layer& L, int64_t M, const Workspace& ws, float* Y, int64_t ldy, const Requant& rq,
                        int variant, hipStream_t s);

hipError_t launch_clear_flags(const Workspace& ws, hipStream_t s);
// polls of a hand-over flag before a waiting workgroup of the tiled kernel gives up and stores NaN
int tiled_wait_limit();
void set_tiled_wait_limit(int polls);

// ---- offline construction, shared host steps (build_factors.cpp) ---------------------------
// exp_bits: width of A_k's and B_k's shared exponents (8, or 4 with one bias per tensor)
int pack_factors_and_import(int64_t K, int64_t N, int k, const std::vector<uint8_t>& Wc, const std::vector<uint8_t>& We,
                            const std::vector<double>& A, const std::vector<double>& B, int exp_bits, lqer_layer** out,
                            int w_bits = 4);
int scale_from_magnitudes(const std::vector<double>& abar, std::vector<double>& s);

// ---- the scaled-integer variant (int_host.cpp, kernels_int.hip) ------------------------------------------------------
hipError_t launch_quant_token(const float* X, int64_t rows, int64_t K, int64_t ldx, int8_t* codes, int64_t ldc,
                              float* scale_f32, uint16_t* scale_f16, bool perm, hipStream_t s);
size_t int_workspace_bytes(const Layer& L, int64_t M);
int forward_int(const Layer& L, const float* X, int64_t ldx, int64_t M, float* Y, int64_t ldy, void* ws, size_t ws_bytes,
                hipStream_t s);
void free_device(Layer& L);
int upload(const std::vector<uint8_t>& host, uint8_t** dev);
// canonical B_k codes -> the records both formats use (exponent bytes from Be, or zero when Be is null)
int tile_b(const Layer& L, const int8_t* Bc, const uint8_t* Be, std::vector<uint8_t>& out);
// rank-k split of G = S E_q (K x N, fp64): A = S^-1 U_k (K x k), B = Sigma_k V_k^T (k x N)
int truncated_split(const std::vector<double>& G, int64_t K, int64_t N, const std::vector<double>& s, int k,
                    std::vector<double>& A, std::vector<double>& B);
int build_factors_int(const float* W_host, int64_t K, int64_t N, const std::vector<double>& s, int k, lqer_layer** out);

int prep_slices(const Layer& L, int64_t M, int path);
// lqer_linear_forward with the given scratch as its workspace, planned without the slots of the tiled kernel's
// work split (output tiles are then never cut); LQER_ERR_WORKSPACE when the plan does not fit scratch_bytes
int forward_in_scratch(const lqer_layer* layer, const float* X, int64_t M, int64_t ldx, float* Y, int64_t ldy,
                       void* scratch, size_t scratch_bytes, void* stream);
int compute_units();               // of the current device

}  // namespace lqer
