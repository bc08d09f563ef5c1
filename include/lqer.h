/*
 * lqer.h - C ABI of the MI355X (gfx950) LQER W4A8 linear layer.
 *
 * The layer computes (arXiv 2402.02446, Eq. 3 and Eq. 6)
 *
 *        Y = X_q W_q + (X_q A_k) B_k
 *
 * with X_q = MXINT8 activations quantized on the fly, W_q = MXINT4 weights and
 * A_k, B_k = MXINT8 rank-k factors of the (activation-scaled) quantization
 * error S (W - W_q) (Eq. 1-2, Eq. 4-5, App. A).  Every MXINT tensor uses blocks
 * of 16 along the contraction axis and one biased-127 exponent byte per block
 * (Sec. 2.2, Sec. 4.1).
 *
 * Conventions
 *   M = tokens (the paper's t), K = in-features (m), N = out-features (n),
 *   k = rank, kp = k rounded up to a multiple of 16.  W is K x N (Y = X W).
 *   "_dev" pointers are device memory, "_host" pointers are host memory.
 *   Every call returns an lqer_status; none throws or aborts.  Argument errors
 *   are reported before anything is launched.  Launches are asynchronous on
 *   the given HIP stream (a hipStream_t passed as void*; NULL = default stream).
 *
 * MXINT element format (b-bit mantissa, block of 16, exponent byte eb):
 *   e = eb - 127 = floor(log2 max|v|) clamped to [-127,127] (-127 for an all-zero block),
 *   value = code * 2^(e - (b-2)),  code = round-half-even(v / 2^(e-(b-2))) saturated
 *   to +-(2^(b-1) - 1).  Inputs must be finite.
 *
 * Canonical packed layouts (contraction axis contiguous everywhere):
 *   Wc[N][K/2]   two 4-bit two's-complement codes per byte, element 2i in the low nibble
 *   We[N][K/16]  exponent bytes
 *   Ac[kp][K] int8, Ae[kp][K/16];   Bc[N][kp] int8, Be[N][kp/16]
 *   Xc[M][K]  int8, Xe[M][K/16]
 */
#ifndef LQER_H
#define LQER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LQER_OK = 0,
    LQER_ERR_NULL = 1,            /* a required pointer is NULL */
    LQER_ERR_SHAPE = 2,           /* K % 16 != 0, k > min(K,N), ld < cols, negative size ... */
    LQER_ERR_UNSUPPORTED = 3,     /* a mantissa or exponent width, block size or rank (kp > 256) this build does not take */
    LQER_ERR_SINGULAR_SCALE = 4,  /* a calibrated channel magnitude is <= 0 or not finite (Sec. 3.2 needs S^-1) */
    LQER_ERR_WORKSPACE = 5,       /* workspace NULL, misaligned or too small */
    LQER_ERR_HIP = 6,             /* a HIP runtime call or launch failed */
    LQER_ERR_NO_CONVERGENCE = 7,  /* the truncated SVD did not reach its tolerance */
    LQER_ERR_VALUE = 8,           /* packed bytes hold a value the format excludes (nibble -8, exponent byte out of range) */
    LQER_ERR_NO_MEMORY = 9        /* a host allocation failed (import, export and the offline step build host copies) */
} lqer_status;

/*
 * Number-format description for lqer_build_factors: {4 or 2, 8, 8 or 4, 16}, or {4, 8, 16, 128} for the
 * scaled-integer variant (see lqer_int_layer_import).
 * exp_bits is the width of the shared exponents of W_q, A_k and B_k (Sec. 4.1 gives them 4 bits;
 * activations always keep 8).  The paper states no bias for the 4-bit field; here each of the
 * three tensors has one bias of its own, chosen so that its largest block keeps its exponent:
 * with top = the largest block exponent of the tensor, a block is quantized with
 * max(own exponent, top - 15), i.e. blocks more than 15 binades below the largest lose their low
 * bits.  The layer still carries one exponent byte per block (lqer_layer_export); within one tensor
 * the bytes then span at most 16 consecutive values, so byte - (largest byte - 15) fits a nibble.
 */
typedef struct {
    int w_bits;     /* mantissa bits of W_q               (4 or 2) */
    int h_bits;     /* mantissa bits of X, A_k, B_k       (8) */
    int exp_bits;   /* shared exponent bits of W_q, A_k, B_k   (8 or 4) */
    int block;      /* block size                         (16) */
} lqer_config;

/* Opaque layer: owns the device copies of W_q, A_k, B_k (in an internal tiled layout). */
typedef struct lqer_layer lqer_layer;

/* Short English name of a status code; never NULL. */
const char* lqer_status_string(int status);

/*
 * MX block quantizer (Sec. 2.2; block shape [1,16] of Sec. 4.1): blocks of 16 along
 * the contiguous axis of a row-major fp32 matrix.
 *   x_dev      [rows][ld] fp32, device; only the first `cols` of each row are read
 *   cols       multiple of 16;  ld >= cols
 *   elem_bits  8 or 6 (codes_dev = int8 [rows][cols]) or 4 (codes_dev = uint8 [rows][cols/2], canonical nibbles)
 *   exp_bits   8
 *   exps_dev   uint8 [rows][cols/16]
 * rows == 0 is a no-op.  Caller owns all buffers.
 */
int lqer_quantize_mx(const float* x_dev, int64_t rows, int64_t cols, int64_t ld,
                     int elem_bits, int exp_bits,
                     void* codes_dev, uint8_t* exps_dev, void* hip_stream);

/*
 * Offline construction (Sec. 3.1 Eq. 1-2; Sec. 3.2 Eq. 4-5; App. A Eq. 7-8).
 *   W_host      [K][N] fp32 row-major, host
 *   calib_host  [n_samples][rows_per_sample][K] fp32, host (ignored when mode == 0; may be NULL then)
 *   k           rank, 0 <= k <= min(K, N), at most 256 (LQER_ERR_UNSUPPORTED above)
 *   mode        0 = LQER (S = I), 1 = L2QER (S from calib_host)
 *   cfg         NULL = {4, 8, 8, 16}; {4, 8, 4, 16} selects 4-bit shared exponents (see lqer_config);
 *               w_bits = 2 selects 2-bit weight mantissas (the W2A8 setup, Sec. 4.1 / Sec. 4.4)
 *   out         receives an owning handle; release with lqer_layer_free
 * Computes W_q = q(W), E_q = W - W_q, S, the k leading singular triplets of S E_q,
 * A_k = S^-1 U_k, B_k = Sigma_k V_k^T, quantizes A_k and B_k to MXINT8 and uploads
 * everything to the current device.  Synchronous.
 */
int lqer_build_factors(const float* W_host, int64_t K, int64_t N,
                       const float* calib_host, int64_t n_samples, int64_t rows_per_sample,
                       int k, int mode, const lqer_config* cfg, lqer_layer** out);

/*
 * The same construction (Sec. 3.1 Eq. 1-2; Sec. 3.2 Eq. 4-5; App. A Eq. 7-8) with W and the
 * calibration samples already on the device:
 *   W_dev       [K][N] fp32 row-major, device
 *   calib_dev   [n_samples][rows_per_sample][K] fp32, device (ignored when mode == 0; may be NULL then)
 *   hip_stream  the stream the kernels run on
 * The calibration magnitudes, W_q, S (W - W_q) and the two products of every subspace iteration
 * are computed by device kernels in fp32 (the magnitudes in fp64, with the bits of the host
 * path); the l x l steps and the MXINT8 packing of A_k and B_k run on the host.  W_q has the
 * bits lqer_build_factors gives; A_k and B_k agree with it up to the rotation freedom of the
 * truncated SVD and fp32 rounding.  Allocates and frees its own device scratch (K N fp32 plus
 * small buffers).  Synchronous; same status codes.
 */
int lqer_build_factors_device(const float* W_dev, int64_t K, int64_t N,
                              const float* calib_dev, int64_t n_samples, int64_t rows_per_sample,
                              int k, int mode, const lqer_config* cfg, void* hip_stream, lqer_layer** out);

/*
 * Layer from / to canonical packed bytes (host pointers, layouts above).
 * Import copies; the caller keeps its buffers.  Ac/Ae/Bc/Be may be NULL when k == 0.
 * Wc nibbles must not be -8; We bytes must be <= 245; Ae, Be bytes must be <= 254
 * (LQER_ERR_VALUE otherwise).  Export writes exactly the bytes that were imported
 * (or that lqer_build_factors produced); any output pointer may be NULL to skip it.
 * The padded rank kp may not exceed 256 (LQER_ERR_UNSUPPORTED): the kernels take up to the
 * k = 256 that Sec. 4.1 pairs with 2-bit weights.
 * lqer_layer_import_w: the same with the mantissa width of W_q given, 4 or 2 (the W2A8 setup of
 * Sec. 4.1 / Sec. 4.4: 1 sign and 1 integer bit, value = code * 2^e, code in {-1, 0, 1}).  For
 * 2 bits Wc is [N][K/4]: four two's-complement bit pairs per byte, element 4i in bits 0-1; the
 * pair -2 is excluded (LQER_ERR_VALUE).  lqer_layer_export writes the width the layer has
 * (lqer_layer_weight_bits; 0 for a NULL handle).
 */
int lqer_layer_import(int64_t K, int64_t N, int k,
                      const uint8_t* Wc, const uint8_t* We,
                      const int8_t* Ac, const uint8_t* Ae,
                      const int8_t* Bc, const uint8_t* Be, lqer_layer** out);
int lqer_layer_import_w(int w_bits, int64_t K, int64_t N, int k,
                        const uint8_t* Wc, const uint8_t* We,
                        const int8_t* Ac, const uint8_t* Ae,
                        const int8_t* Bc, const uint8_t* Be, lqer_layer** out);
int lqer_layer_weight_bits(const lqer_layer* layer);
int lqer_layer_export(const lqer_layer* layer, uint8_t* Wc, uint8_t* We,
                      int8_t* Ac, uint8_t* Ae, int8_t* Bc, uint8_t* Be);
int lqer_layer_dims(const lqer_layer* layer, int64_t* K, int64_t* N, int* k, int* kp);
/*
 * Width of the activation codes the forward pass quantizes X to: 8 (W4A8, the default) or 6
 * (the W4A6 setup of Table 2; Sec. 4.1 keeps the 8-bit shared exponent for activations).
 * lqer_linear_forward_q then expects codes of that width (int8 storage either way).
 * With 6 bits, block maxima of 2^125 and above are outside the supported range.
 */
int lqer_layer_set_activation_bits(lqer_layer* layer, int bits);
int lqer_layer_free(lqer_layer* layer);

/*
 * Forward pass (Eq. 3 / Eq. 6).
 *   X_dev  [M][ldx] fp32 device (ldx >= K);  Y_dev [M][ldy] fp32 device (ldy >= N)
 *          X_dev and Y_dev must be 16-byte aligned and ldx, ldy multiples of 4 (rows are read and written
 *          16 bytes at a time); LQER_ERR_SHAPE otherwise.  Xc_dev of lqer_linear_forward_q: 16-byte aligned.
 *   workspace_dev  device scratch of at least lqer_linear_workspace_bytes(layer, M)
 *                  bytes, 256-byte aligned, caller-owned; its contents are scratch.
 *                  (lqer_linear_workspace_bytes_ex: the same for a forced path of lqer_linear_forward_ex,
 *                  0 = the automatic one; a few hundred KiB for small M, 64 MiB more for the tiled kernel)
 * Steps, all in this library's kernels: quantize X to MXINT8 (Sec. 4.1), T = X_q A_k,
 * Y = X_q W_q + T B_k accumulated in fp32 in one pass over Y.  M == 0 is a no-op.
 * Calls on different streams need distinct workspaces.  The library allocates nothing here,
 * uses only the given stream and no host synchronisation, so the call can be captured in a HIP
 * graph.  Results are the same bits on every run.
 * For large M the workspace also holds one slot of 256 KiB per compute unit: when the output
 * tiles do not fill whole rounds of the chip, workgroups cut the remaining tiles along K, hand
 * their partial sums over through these slots and the receiving workgroup polls a flag.  The
 * poll is bounded (about a second): the kernel always ends, and a tile whose partner never
 * arrived is stored as NaN, never as a wrong number.
 * lqer_linear_forward_q takes activations that are already quantized
 * (Xc int8 [M][K], Xe uint8 [M][K/16], canonical, device).
 */
size_t lqer_linear_workspace_bytes(const lqer_layer* layer, int64_t M);
size_t lqer_linear_workspace_bytes_ex(const lqer_layer* layer, int64_t M, int path);
int lqer_linear_forward(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx,
                        float* Y_dev, int64_t ldy,
                        void* workspace_dev, size_t workspace_bytes, void* hip_stream);
int lqer_linear_forward_q(const lqer_layer* layer, const int8_t* Xc_dev, const uint8_t* Xe_dev,
                          int64_t M, float* Y_dev, int64_t ldy,
                          void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * Launch control for measurement and tuning (Sec. 2.1 distinguishes the memory-bound
 * and the compute-bound regime; the dispatcher picks by M, this overrides it).
 *   path    0 = automatic, 1 = streaming kernel (small M), 2 = tiled MFMA kernel (large M)
 *   variant 0 = automatic, otherwise a tile-shape index of the chosen path (for tuning; an index the
 *           path does not have returns LQER_ERR_SHAPE).  Tiled path: 100 * mode + shape, mode 0 = cut
 *           output tiles along K between workgroups when the estimate says it pays, 1 = never,
 *           2 = whenever tiles are left over, 3 = the same in equal shares of the left-over K tiles
 *           instead of along tile boundaries
 *   stages  bit 0 = quantize + T, bit 1 = main product; 0 = both
 * Same contract as lqer_linear_forward otherwise.  Running stage bit 1 alone reuses
 * what an earlier call with bit 0 left in the same workspace - with the same M, path and
 * variant - and, on narrow layers where the streaming kernel runs pairs of workgroups that
 * add into Y, needs the Y that call cleared: run alone a second time it adds onto the result.
 */
typedef struct {
    int path;
    int variant;
    int stages;
} lqer_launch_opts;
int lqer_linear_forward_ex(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx,
                           float* Y_dev, int64_t ldy,
                           void* workspace_dev, size_t workspace_bytes, void* hip_stream,
                           const lqer_launch_opts* opts);

/*
 * Forward pass whose result leaves as MXINT8, ready to be the next layer's X_q: the
 * weight-activation flow of Table 1 quantizes a layer's output again; here the quantizer
 * (Sec. 2.2, block [1,16] of Sec. 4.1) is applied to the fp32 accumulators in the epilogue of
 * the main kernel instead of in a pass over a stored Y.
 *   Yc_dev  int8 [M][ldyc] device (ldyc >= N, multiple of 4; Yc_dev 4-byte aligned)
 *   Ye_dev  uint8 [M][N/16] device; N must be a multiple of 16
 *   opts    as for lqer_linear_forward_ex, or NULL.  Shapes of the streaming kernel that run
 *           pairs of workgroups cannot quantize in the kernel: automatic choice avoids them,
 *           forcing one returns LQER_ERR_SHAPE.
 * The codes and exponent bytes are those lqer_quantize_mx gives for the fp32 Y that
 * lqer_linear_forward_ex produces with the same path and variant.  Same contract otherwise.
 */
int lqer_linear_forward_requant(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx,
                                int8_t* Yc_dev, int64_t ldyc, uint8_t* Ye_dev,
                                void* workspace_dev, size_t workspace_bytes, void* hip_stream,
                                const lqer_launch_opts* opts);

/*
 * Several layers applied to the same activations (q/k/v, or gate/up, of a decoder block): in the
 * weight-activation flow of Table 1 the activations are quantized once (Sec. 4.1) and every
 * layer that consumes them sees the same X_q.  Here X is quantized by the first layer's
 * projection step; for the others only T = X_q A_k (Eq. 3) is computed, from the X_q already in the
 * workspace.  Each Y_dev[i] holds the same bits as lqer_linear_forward(layers[i], ...) gives.
 *   layers   n_layers handles with the same K and the same activation width (LQER_ERR_SHAPE otherwise)
 *   Y_dev    n_layers device pointers, Y_dev[i] fp32 [M][ldy[i]], ldy[i] >= N of layer i
 *   workspace_dev  at least lqer_linear_shared_workspace_bytes(layers, n_layers, M) bytes
 * For token counts that take the streaming kernel the call is n_layers full forward passes.
 * Same contract as lqer_linear_forward otherwise.
 */
size_t lqer_linear_shared_workspace_bytes(const lqer_layer* const* layers, int n_layers, int64_t M);
int lqer_linear_forward_shared(const lqer_layer* const* layers, int n_layers, const float* X_dev,
                               int64_t M, int64_t ldx, float* const* Y_dev, const int64_t* ldy,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * For callers that test the failure path of the bounded wait described at lqer_linear_forward:
 * the number of polls after which a workgroup waiting for another one's partial sums gives up
 * (process-wide; the default, 1 << 22, is about a second).  With 0 every such wait gives up at
 * once: the kernel still ends normally and every output tile that was cut between workgroups
 * is stored as NaN.  Negative values return LQER_ERR_SHAPE.
 */
int lqer_set_wait_limit(int polls);

/*
 * The scaled-integer variant of the layer (Table 2, rows "L2QER-INT": INT4 weights in groups of 128, "g128", and 8-bit
 * activations; Sec. 2.1 for the form of such formats: a scale factor per weight group, per-token scalars for the
 * activations, an inner product = a fixed-point inner product times an FP16 product of scalars).  The paper prints no
 * formula; the reading here is the plain symmetric one:
 *   weights, A_k, B_k: groups of 128 along the contraction axis (B_k: its kp <= 128 ranks are one group per column),
 *       s = fp16(amax / qmax) rounded to nearest even (1 for an all-zero group), code = clamp(rne(v / s), -qmax, qmax),
 *       qmax = 7 for W_q (4 bits), 127 for A_k, B_k (8 bits);
 *   activations: s_t = fp16(amax_t / 127) and code = clamp(rne(x / s_t), -127, 127), both divisions in fp32.
 * Canonical arrays (host, contraction axis contiguous; scales are FP16 bit patterns):
 *   Wc[N][K/2] nibbles as above, Ws[N][K/128];  Ac[kp][K] int8, As[kp][K/128];  Bc[N][kp] int8, Bs[N].
 * K must be a multiple of 128 and kp at most 128 (LQER_ERR_SHAPE / LQER_ERR_UNSUPPORTED); nibble -8, and scales that
 * are zero, negative or not finite, are excluded (LQER_ERR_VALUE).
 * lqer_build_factors with cfg = {4, 8, 16, 128} builds such a layer (same steps, Sec. 3.1-3.2 and App. A).
 * An INT layer runs through lqer_linear_forward, lqer_linear_forward_static and lqer_linear_workspace_bytes
 * (lqer_linear_path reports 3: one kernel, int8 matrix cores, for every token count); the entry points that take
 * MXINT codes, launch options, MXINT8 output or layer groups return LQER_ERR_UNSUPPORTED for it, and
 * lqer_layer_export does too (lqer_int_layer_export is its counterpart).
 * lqer_quantize_int8_token is the stand-alone per-token quantizer: x_dev [rows][ld] fp32 (16-byte aligned, ld and
 * cols multiples of 4), codes_dev int8 [rows][cols], scales_dev FP16 bit patterns [rows].
 */
int lqer_int_layer_import(int64_t K, int64_t N, int k,
                          const uint8_t* Wc, const uint16_t* Ws,
                          const int8_t* Ac, const uint16_t* As,
                          const int8_t* Bc, const uint16_t* Bs, lqer_layer** out);
int lqer_int_layer_export(const lqer_layer* layer, uint8_t* Wc, uint16_t* Ws,
                          int8_t* Ac, uint16_t* As, int8_t* Bc, uint16_t* Bs);
int lqer_quantize_int8_token(const float* x_dev, int64_t rows, int64_t cols, int64_t ld,
                             int8_t* codes_dev, uint16_t* scales_dev, void* hip_stream);

/*
 * lqer_linear_forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * same kernels and the same bits in Y as lqer_linear_forward with an automatic launch whose tiles
 * are not cut between workgroups; the scratch that call takes as `workspace_dev` is a device array
 * inside the library, 32 MiB on every GPU the library is used on, held until the process ends.
 *   - Sizes whose scratch need exceeds 32 MiB return LQER_ERR_WORKSPACE before anything is launched
 *     (the need is about 2 (M + 255) (K + 128) bytes for more than 64 tokens - e.g. M = 1024 at
 *     K = 8192 fits, M = 4096 does not - and well under 2 MiB up to 64 tokens).
 *   - The call allocates and frees nothing and synchronises nothing.  Its first use on a device looks
 *     up the address of that device's array (with that device current): make one call outside any
 *     graph capture first.
 *   - Every call on a GPU uses that GPU's one array, which keeps the last call's contents (each call
 *     overwrites or clears what it reads): calls that overlap in time on one GPU - two streams, two
 *     threads - race.  Calls on one stream, or ordered by events, are safe.
 */
int lqer_linear_forward_static(const lqer_layer* layer, const float* X_dev, int64_t M, int64_t ldx,
                               float* Y_dev, int64_t ldy, void* hip_stream);

/*
 * Diagnostic, host only (no device call, runs without a GPU): tiles pseudo-random canonical bytes into the device
 * record layouts of Sec. 4.1's formats (4- and 2-bit weights, both exponent forms, ragged sizes, ranks to 256) and back,
 * and compares.  LQER_OK, or LQER_ERR_VALUE at the first difference.  Meant for builds with host sanitizers.
 */
int lqer_selftest_layouts(void);

/* Which path the dispatcher picks for this layer at M tokens: 1 = streaming, 2 = tiled MFMA, 3 = the INT variant's kernel. */
int lqer_linear_path(const lqer_layer* layer, int64_t M);

#ifdef __cplusplus
}
#endif
#endif /* LQER_H */
