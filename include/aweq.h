/*
 * libaweq -- AWEQ (arXiv 2311.01305) per-linear-layer calibration + quantization path
 * for AMD MI355X (gfx950).  C ABI.
 *
 * Notation (the paper's): X[T x K] calibration activations (T tokens, K input channels),
 * W[N x K] the linear weight in PyTorch layout (the paper writes Y = X W with W as K x N,
 * Sec. 3.1 Eq. 3; its "channel i" is the column index k of both X and W here),
 * s[K] the equalization factors, Step / Z the quantizer's scale and zero point (Eq. 1-2).
 *
 * Conventions for every entry point
 *   - every pointer is a DEVICE pointer owned by the caller, unless marked "host";
 *     matrices are row-major with the K index contiguous and a leading dimension in
 *     elements; rows must start 16-byte aligned;
 *   - the library allocates nothing, frees nothing and never synchronises: each call
 *     enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and returns; scratch memory comes from the caller (`ws`, `ws_bytes`; ask
 *     aweq_workspace_size; 16-byte aligned; its contents need no initialisation), and may be
 *     reused by the next call on the same stream; entry points without a `ws` argument need none;
 *   - the return value is 0 or a negative AWEQ_ERR_* code found on the HOST before
 *     anything is launched (bad pointer, shape, dtype, alignment, workspace);
 *   - numeric conditions met on the device are OR-ed into the optional device word
 *     `status` (AWEQ_ST_* bits); inputs are expected to be finite;
 *   - calls on different streams must not share output or workspace buffers.
 */
#ifndef AWEQ_H
#define AWEQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { AWEQ_F32 = 0, AWEQ_F16 = 1, AWEQ_I8 = 2 } aweq_dtype;

enum {
    AWEQ_OK = 0,
    AWEQ_ERR_NULL = -1,      /* a required pointer is NULL */
    AWEQ_ERR_SHAPE = -2,     /* a dimension is <= 0, a leading dimension is too small, K % 8 != 0 */
    AWEQ_ERR_DTYPE = -3,     /* dtype not supported by this entry point */
    AWEQ_ERR_BITS = -4,      /* bits not in {8, 4, 3} */
    AWEQ_ERR_GROUP = -5,     /* group does not divide K or is not a supported size */
    AWEQ_ERR_ALIGN = -6,     /* a pointer or row pitch is not 16-byte aligned */
    AWEQ_ERR_WORKSPACE = -7, /* ws is NULL or smaller than aweq_workspace_size says */
    AWEQ_ERR_LAUNCH = -8     /* the HIP runtime refused a launch */
};

/* bits of the device status word */
enum {
    AWEQ_ST_DEGENERATE = 1u, /* Eq. 2 gave a non-positive or non-finite Step; Step := 1 was used */
    AWEQ_ST_NONFINITE = 2u,  /* NaN / Inf seen in the input (results unspecified) */
    AWEQ_ST_BIGQUOT = 4u,    /* |x / Step| >= 2^24: quotient saturated */
    AWEQ_ST_SCALEGUARD = 8u, /* Eq. 10: a channel range was < 1e-5 (s := 1) or s was clamped to [1e-4, 1e4] */
    AWEQ_ST_ZEROPOINT = 16u  /* stage 4 de-quantisation met a zero point outside [0, 255] (a slice whose range does not
                                contain 0): its 32-bit integer part is exact only while it fits in 32 bits */
};

typedef enum {
    AWEQ_OP_CALIB_STATS = 0,
    AWEQ_OP_EQUALIZE = 1,
    AWEQ_OP_QUANT_WEIGHT = 2,
    AWEQ_OP_W8A8_GEMM = 3,
    AWEQ_OP_BIAS_CORRECT = 4,
    AWEQ_OP_WONLY_GEMM = 5,
    AWEQ_OP_QUANT_ACT = 6
} aweq_op;

enum { AWEQ_BIAS_W8A8 = 0, AWEQ_BIAS_WEIGHT_ONLY = 1 };

/* values of aweq_equalize's enable_awe */
enum {
    AWEQ_SCALE_NONE = 0,   /* s = 1: equalization off (the ablation of Sec. 4.4) */
    AWEQ_SCALE_RANGE = 1,  /* Eq. 10 on the channel ranges: the method */
    AWEQ_SCALE_ABSMAX = 2  /* Eq. 10's form on the channels' maximum absolute values instead of their ranges: the
                              difficulty definition the method replaces (Sec. 1, Sec. 3.2), kept as a switch for
                              comparisons on the same layers */
};

/* Bytes of workspace the op needs for a [rows x K] input (rows = T or N as the op reads
 * it) and N output channels; 0 when it needs none.  Host function, no GPU needed. */
size_t aweq_workspace_size(aweq_op op, int64_t rows, int64_t K, int64_t N);

/* Name of an AWEQ_ERR_* code.  Host function. */
const char* aweq_status_string(int code);

/* ---- K-panel layout of the int8 GEMM operands (a storage format of this library, chosen so
 * that the matrix-core kernel of stage 4 reads whole cache lines: not part of the method).
 * An int8 matrix M[rows x K] is cut along K into ceil(K / 64) panels of 64 columns; panel p
 * stores bytes M[r][64 p .. 64 p + 63] of every row r back to back:
 *     byte offset of M[r][k] = ((k / 64) * rows + r) * 64 + k % 64,
 * columns past K in the last panel are zero.  xq (stage 4a / 4) and the 8-bit codes of stage 3
 * with group <= 0 use it.  aweq_panel_bytes: size of such a buffer (host function).
 * aweq_pack_panels_i8 / aweq_unpack_panels_i8 convert from / to a row-major [rows x K] int8
 * matrix of pitch ld bytes (K % 8 == 0, ld % 8 == 0, both pointers 8-byte aligned). */
size_t aweq_panel_bytes(int64_t rows, int64_t K);
int aweq_pack_panels_i8(const int8_t* src, int64_t rows, int64_t K, int64_t ld, int8_t* panels, void* stream);
int aweq_unpack_panels_i8(const int8_t* panels, int64_t rows, int64_t K, int8_t* dst, int64_t ld, void* stream);

/* ---- Stage 1: range statistics (Sec. 3.2: channel range = channel max - channel min,
 * tensor range = max - min over all channels, Eq. 4 p_i = r_i / R; Sec. 3.3: E[x] is
 * collected in the same pass).
 * M[rows x K] (F32 or F16, pitch ld) -> cmin[K], cmax[K] (exact), csum[K] (fp64 column
 * sums, nullable), count (uint64 scalar, nullable).  accumulate = 0 starts from
 * (+inf, -inf, 0, 0); accumulate = 1 merges into what the buffers hold (further
 * calibration batches; or a second weight sharing the same input: min of mins, max of
 * maxes).  finalize = 1 also writes r[K] = cmax - cmin, R[1] = max_k cmax - min_k cmin and
 * (nullable) p[K] = r / R.  Needs workspace. */
int aweq_calib_stats(const void* M, aweq_dtype dt, int64_t rows, int64_t K, int64_t ld,
                     float* cmin, float* cmax, double* csum, uint64_t* count,
                     int accumulate, int finalize, float* r, float* R, float* p,
                     void* ws, size_t ws_bytes, uint32_t* status, void* stream);

/* ---- Stage 1 for callers that cannot allocate or pass scratch memory (code under HIP graph capture
 * with a fixed argument list, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and results as aweq_calib_stats, with the per-slice partial rows kept in a device array of
 * AWEQ_STATIC_SCRATCH_BYTES that is part of the library (every GPU the library runs on holds one
 * copy until the process ends) instead of a caller's workspace.  The call allocates nothing.
 * AWEQ_ERR_WORKSPACE when aweq_workspace_size(AWEQ_OP_CALIB_STATS, rows, K, 0) exceeds
 * AWEQ_STATIC_SCRATCH_BYTES (all configurations up to 262144 x 22016 binary16 fit).  The device
 * that owns `stream` must be the current device.  All calls on one GPU share that GPU's array:
 * calls that overlap on one GPU (different streams) race; calls on one stream do not. */
#define AWEQ_STATIC_SCRATCH_BYTES (16u << 20)
int aweq_calib_stats_static(const void* M, aweq_dtype dt, int64_t rows, int64_t K, int64_t ld,
                            float* cmin, float* cmax, double* csum, uint64_t* count,
                            int accumulate, int finalize, float* r, float* R, float* p,
                            uint32_t* status, void* stream);

/* ---- Stage 2: activation-weight equalization (Sec. 3.1 Eq. 3, Sec. 3.2 Eq. 10).
 * From the column statistics of X (xmin, xmax, xsum, host scalar count = T) and of W
 * (wmin, wmax): s[k] = sqrt(r_x r_w) / r_w evaluated in fp64 on the raw channel ranges,
 * inv_s[k] = 1 / s[k]  (enable_awe = AWEQ_SCALE_RANGE; AWEQ_SCALE_NONE: s = 1, the ablation switch of
 * Sec. 4.4; AWEQ_SCALE_ABSMAX: the same formula with m = max(|min|, |max|) of the channel in place of r).
 * Guards: a channel with r_x < 1e-5 or r_w < 1e-5 gets s = 1; s is clamped to [1e-4, 1e4].
 * Fold, weight side: W_hat[n,k] = W[n,k] * s[k], one fp32 multiply rounded to dt
 * (W has pitch ldw, W_hat pitch ldwh; W_hat may alias W when the pitches agree; W = NULL skips the
 * fold).  Activation side: the equalised
 * activation X_hat[t,k] = X[t,k] * inv_s[k] is never stored; its tensor range
 * xhat_range[2] = {min, max}, its mean mu_xhat[K] = (xsum / count) * inv_s and the static
 * int8 activation quantizer derived from that range by Eq. 2 (act_step[1], act_zero[1])
 * are written instead.  prev_scale[K] (nullable) is multiplied by inv_s so the caller can
 * fuse diag(s)^-1 into the preceding block.  mu_xhat / xsum nullable together. */
int aweq_equalize(const float* xmin, const float* xmax, const double* xsum, uint64_t count,
                  const float* wmin, const float* wmax, int64_t K, int enable_awe,
                  float* s, float* inv_s,
                  const void* W, void* W_hat, aweq_dtype dt, int64_t N, int64_t ldw, int64_t ldwh,
                  float* prev_scale, float* xhat_range, float* mu_xhat,
                  float* act_step, int32_t* act_zero,
                  uint32_t* status, void* stream);

/* ---- Stage 3: weight quantizer, Eq. 1-2: Step = (max - min) / (2^b - 1),
 * Z = -round(min / Step), u = clamp(round(w / Step) + Z, 0, 2^b - 1); round-to-nearest
 * with ties to even, true fp32 division.  A slice with max == min uses Step = 1.
 * group = 0: one (Step, Z) per row n -> step[N], zero[N];
 * group = g > 0 (a power of two in [8, 512] dividing K): one per g consecutive k inside a
 *   row -> step/zero[N x K/g];
 * group = -1: one for the whole tensor -> step[1], zero[1] (needs workspace).
 * codes: bits 8 -> int8 u - 128; for group <= 0 in the K-panel layout (aweq_panel_bytes(N, K)
 * bytes: the weight operand of stage 4), for group > 0 row-major, N*K bytes; bits 4 -> two
 * codes per byte, even k in the low nibble, N*K/2 bytes; bits 3 -> per row a little-endian bit stream with code k in bits
 * [3k, 3k+3), N*3K/8 bytes (K % 32 == 0).  rowsum_w[N] = sum_k (u - 128), bits 8 only,
 * nullable. */
int aweq_quant_weight(const void* W_hat, aweq_dtype dt, int64_t N, int64_t K, int64_t ldw,
                      int bits, int group, void* codes, float* step, int32_t* zero,
                      int32_t* rowsum_w, void* ws, size_t ws_bytes,
                      uint32_t* status, void* stream);

/* ---- Stages 2b + 3 in one pass over W (per-row quantizer, group = 0): W_hat[n,k] = W[n,k] * s[k]
 * rounded to dt (Eq. 3; W_hat has pitch ldwh and may alias W when ldwh = ldw) is written and quantised from registers,
 * with the outputs of aweq_quant_weight(group = 0).  Same results as aweq_equalize's fold followed by
 * aweq_quant_weight; call aweq_equalize with W = NULL for the scales first. */
int aweq_fold_quant_weight(const void* W, aweq_dtype dt, int64_t N, int64_t K, int64_t ldw,
                           const float* s, void* W_hat, int64_t ldwh, int bits, void* codes, float* step,
                           int32_t* zero, int32_t* rowsum_w, uint32_t* status, void* stream);

/* ---- Stage 4a (helper, also run by aweq_w8a8_gemm): static per-tensor int8 activation
 * quantizer (Eq. 1 with b = 8) applied to X_hat = X * inv_s on the fly:
 * xq[t,k] = clamp(round((X[t,k] * inv_s[k]) / Step_x) + Z_x, 0, 255) - 128,
 * rowsum_x[T] = sum_k xq (int32, nullable), colsum_xq[K] = sum_t xq (int64, nullable).
 * xq is written in the K-panel layout (aweq_panel_bytes(T, K) bytes); xq = NULL computes the sums
 * only (one read of X, nothing written per element: what a calibration without the forward needs).
 * act_step / act_zero are the device scalars aweq_equalize wrote.  The sums are formed without
 * atomics, in a fixed order: per-slice partial sums in the workspace
 * (aweq_workspace_size(AWEQ_OP_QUANT_ACT, T, K, 0) bytes; needed when colsum_xq is asked for, or
 * rowsum_x with K > 512) and a merge kernel.  AWEQ_ST_BIGQUOT: some |X_hat / Step| reached 2^24
 * (Step and Z not from this data); the quotient is then rounded, saturated at +-2^30, and clamped
 * as Eq. 1 says. */
int aweq_quant_act(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx,
                   const float* inv_s, const float* act_step, const int32_t* act_zero,
                   int8_t* xq, int32_t* rowsum_x, int64_t* colsum_xq,
                   void* ws, size_t ws_bytes, uint32_t* status, void* stream);

/* ---- Stage 4: W8A8 forward (Sec. 1-2: INT8 weights and activations).
 * x_dt F16 / F32: X is quantised into xq[T x K] first (stage 4a; xq, inv_s, act_step,
 * act_zero required).  x_dt I8: X already holds xq in the K-panel layout (ldx = K), stage 4a
 * is skipped.  wq[N x K]: the 8-bit codes of stage 3 (group <= 0), K-panel layout.
 * acc[t,n] = sum_k xq[t,k] wq[n,k], int8 x int8 -> int32 on the matrix cores (K <= 32768).
 * Outputs, each nullable: out_i32[T x N] (pitch ldo) the raw accumulator;
 * out_deq[T x N] (F16 or F32, pitch ldo) the de-quantised output
 *   Step_x Step_w[n] (acc - Z'x rowsum_w[n] - Z'w[n] rowsum_x[t] + K Z'x Z'w[n]) + bias[n],
 *   Z' = Z - 128 (needs rowsum_x, rowsum_w, step_w, zero_w; bias nullable);
 *   The integer in parentheses is formed in 32-bit arithmetic: exact whenever it fits, which zero
 *   points in [0, 255] (ranges that contain 0) guarantee for K <= 32768; other zero points are
 *   handled the same way and raise AWEQ_ST_ZEROPOINT;
 * colsum_acc[N] = sum_t acc[t,n] (int64; what stage 5 needs; always the sum of the accumulator
 *   itself, whatever the zero points).
 * w_group = 0: step_w[N] / zero_w[N] hold one entry per output channel (stage 3 with group = 0);
 * w_group = -1: step_w[1] / zero_w[1], one for the tensor (stage 3 with group = -1, the paper's
 * per-tensor setting, Sec. 3); rowsum_w[N] is per output channel in both cases.
 * ws: the workspace of stage 4a when X is F16 / F32 (aweq_workspace_size(AWEQ_OP_W8A8_GEMM, T, K, N));
 * not needed (NULL) for x_dt = I8. */
int aweq_w8a8_gemm(const void* X, aweq_dtype x_dt, int64_t T, int64_t K, int64_t ldx,
                   const float* inv_s, const float* act_step, const int32_t* act_zero,
                   int8_t* xq, int32_t* rowsum_x, int64_t* colsum_xq,
                   const int8_t* wq, int64_t N, const float* step_w, const int32_t* zero_w, int w_group,
                   const int32_t* rowsum_w, const float* bias,
                   int32_t* out_i32, void* out_deq, aweq_dtype out_dt, int64_t ldo,
                   int64_t* colsum_acc, void* ws, size_t ws_bytes,
                   uint32_t* status, void* stream);

/* ---- Stage 4 with fused epilogues for the layer that consumes this one's output (statistics of
 * Sec. 3.2 / Sec. 3.3's E[x] and the quantizer of Eq. 1 applied where the output is produced
 * instead of in passes of their own over it).  The GEMM and the de-quantisation are those of
 * aweq_w8a8_gemm with x_dt = I8 and w_group = 0 (per-channel weight scales); y[t,n] = act(de-quantised output + bias) rounded to binary16,
 * act = 0 (none) or 1 (ReLU, OPT's fc1 -> fc2).  Outputs:
 *  out_f16[T x N] (pitch ldo, nullable): y itself;
 *  colsum_acc[N] (required): as in aweq_w8a8_gemm, for this layer's stage 5;
 *  statistics (ycmin non-NULL): ycmin[N], ycmax[N], ycsum[N] (nullable), ycount[1] (nullable) =
 *    what aweq_calib_stats(y, F16, rows = T, K = N, accumulate) returns on the stored output:
 *    extremes exact, sums exact (integer accumulation in units of 2^-24), independent of the
 *    launch; needs ws of aweq_workspace_size(AWEQ_OP_W8A8_GEMM, T, K, N) bytes;
 *  next-layer codes (yq non-NULL): yq[T x N] in the K-panel layout (aweq_panel_bytes(T, N) bytes),
 *    rowsum_y[T] (nullable), colsum_yq[N] (nullable) = what aweq_quant_act(y, F16, T, N, ...,
 *    next_inv_s[N], next_step[1], next_zero[1]) returns (true division).
 * At least one of the two.  Shapes the tiled kernel takes only: N % 4 == 0, 16-byte aligned
 * vectors and outputs (AWEQ_ERR_SHAPE / AWEQ_ERR_ALIGN otherwise). */
int aweq_w8a8_gemm_fused(const int8_t* xq, int64_t T, int64_t K, const int8_t* wq, int64_t N,
                         const float* act_step, const int32_t* act_zero,
                         const float* step_w, const int32_t* zero_w,
                         const int32_t* rowsum_x, const int32_t* rowsum_w, const float* bias, int act,
                         void* out_f16, int64_t ldo, int64_t* colsum_acc,
                         float* ycmin, float* ycmax, double* ycsum, uint64_t* ycount, int accumulate,
                         const float* next_inv_s, const float* next_step, const int32_t* next_zero,
                         int8_t* yq, int32_t* rowsum_y, int64_t* colsum_yq,
                         void* ws, size_t ws_bytes, uint32_t* status, void* stream);

/* ---- Stage 5: quantization bias correction (Sec. 3.3, Eq. 11-15).
 * delta[n] = mean over the calibration tokens of the FP output of the equalised layer
 * minus the mean output of the quantised layer; bias_out = bias_in + delta (the paper
 * subtracts E[y~ - y]).  enable_bc = 0 still writes delta but copies the bias unchanged.
 * mode AWEQ_BIAS_W8A8: mean FP output = W_hat mu_xhat (fp64 accumulation); mean int8-path
 *   output from colsum_acc, colsum_xq, rowsum_w, act_step/act_zero and step_w/zero_w (group = 0:
 *   [N], one per output channel; group = -1: [1], per tensor) as exact integers, count = T.  colsum_acc = NULL: the sums over tokens of the accumulator are
 *   formed from the weight codes instead (codes = the 8-bit per-row / per-tensor codes in the
 *   K-panel layout, bits = 8, group <= 0): sum_t acc[t,n] = sum_k wq[n,k] colsum_xq[k], the same
 *   integers, so the correction can be calibrated without running the forward.
 * mode AWEQ_BIAS_WEIGHT_ONLY (Eq. 12-15): delta[n] = -sum_k (W~[n,k] - W_hat[n,k]) mu_xhat[k]
 *   with W~ de-quantised from codes / bits / group / step_w / zero_w as laid out by
 *   aweq_quant_weight.
 * bias_in nullable (= zeros); delta, bias_out fp32[N]. */
int aweq_bias_correct(int mode, const void* W_hat, aweq_dtype dt, int64_t N, int64_t K, int64_t ldw,
                      const float* mu_xhat, uint64_t count,
                      const int64_t* colsum_acc, const int64_t* colsum_xq, const int32_t* rowsum_w,
                      const float* act_step, const int32_t* act_zero,
                      const void* codes, int bits, int group,
                      const float* step_w, const int32_t* zero_w,
                      const float* bias_in, float* delta, float* bias_out, int enable_bc,
                      uint32_t* status, void* stream);

/* ---- Weight-only forward (Sec. 4.2, Table 1: INT4 / INT3 weights, FP16 activations):
 * y[t,n] = sum_k x_hat[t,k] w~[n,k] + bias[n], w~ = Step (u - Z) the de-quantised weight of Eq. 1.
 * X_hat[T x K]: binary16 equalised activations, row-major, pitch ldx (the caller has folded
 * diag(s)^-1 into what produces them, Eq. 3); codes / step_w / zero_w: what aweq_quant_weight wrote
 * for bits in {4, 3} and the same group (group > 0: a multiple of 32 dividing K; 0: per row; -1: per
 * tensor); bias[N] fp32 nullable; out[T x N] F16 or F32, pitch ldo.  K % 64 == 0, N % 4 == 0,
 * ldo % 4 == 0, 16-byte aligned pointers.  Arithmetic: the weight operand is binary16,
 * w~_h = RN16((u - Z) * RN16(Step)), written once per call into the workspace (N * K * 2 bytes:
 * aweq_workspace_size(AWEQ_OP_WONLY_GEMM, T, K, N)); products are exact in fp32 and accumulated in
 * fp32 on the matrix cores (summation order unspecified). */
int aweq_wonly_gemm(const void* X_hat, int64_t T, int64_t K, int64_t ldx,
                    const void* codes, int bits, int group,
                    const float* step_w, const int32_t* zero_w, int64_t N,
                    const float* bias, void* out, aweq_dtype out_dt, int64_t ldo,
                    void* ws, size_t ws_bytes, uint32_t* status, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AWEQ_H */
