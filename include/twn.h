/* twn.h — C ABI of the MI355X (gfx950) Ternary Weight Networks hot path.
 *
 * The library implements, as HIP kernels, the two halves of the method of
 * "Ternary Weight Networks" (arXiv 1605.04711):
 *   1. threshold ternarization of float32 weights (Sec. 2.3: Eq. 3, Eq. 5 and
 *      the rule of thumb Delta = f * mean|W|; Alg. 1 steps 3-7), emitted as
 *      2-bit codes (Sec. 2.1 "Model compression") plus Delta, alpha, |I_Delta|;
 *   2. the forward block Z = X * (alpha W~) (Eq. 2; Alg. 1 step 8) for
 *      convolutions and inner products, and its straight-through backward
 *      (Alg. 1 steps 9-10: gradients computed with T = alpha W~ and handed to
 *      the float32 master weights).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *     Descriptors (`twn_*_desc`, `twn_epilogue`) are HOST structs, read before
 *     the call returns.
 *   - The caller owns every buffer.  The library never allocates, frees or
 *     keeps device memory; scratch space is passed in as `workspace`
 *     (size from the matching `*_workspace_bytes` host function; contents on
 *     entry are irrelevant and on exit unspecified; may be NULL when 0 bytes).
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls
 *     only enqueue work; none synchronises.  Scalar results (Delta, alpha, nnz)
 *     are written to device memory and are consumed from there by later calls.
 *   - Return value: TWN_OK or a negative twn_status.  Arguments are validated
 *     on the host before anything is launched, so every error except
 *     TWN_ERR_HIP is raised without touching the GPU and leaves all buffers
 *     untouched.  Nothing throws or aborts.
 *   - Finite inputs are a precondition (NaN/Inf give unspecified results).
 *
 * Packed ternary weight format ("twn2")
 *   A filter bank [rows][C][R][S] is stored as a matrix [rows][K], K = R*S*C,
 *   with k = (r*S + s)*C + c (input channel fastest, matching NHWC activations).
 *   Each row is padded with zero codes to a multiple of 128 weights and takes
 *   twn_packed_words_per_row(K) = 8*ceil(K/128) little-endian uint32 words.
 *   Word j of a row holds the codes k = 16j..16j+15: the code of k = 16j+2i is
 *   in bits [2i, 2i+1], the code of k = 16j+2i+1 in bits [16+2i, 17+2i]
 *   (i = 0..7).  A 2-bit field is (bit0: weight non-zero, bit1: weight
 *   negative): 00 = 0, 01 = +1, 11 = -1; 10 is never produced.  The transposed
 *   copy used by the backward-data pass has one row per input channel c and
 *   K_T = R*S*rows with k_T = (r*S + s)*rows + o.  Packed buffers must be
 *   16-byte aligned.
 */
#ifndef TWN_H
#define TWN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TWN_OK = 0,
    TWN_ERR_NULL = -1,        /* a required pointer is NULL */
    TWN_ERR_SHAPE = -2,       /* non-positive / inconsistent / too large sizes */
    TWN_ERR_ALIGN = -3,       /* a pointer or leading dimension is misaligned */
    TWN_ERR_UNSUPPORTED = -4, /* dtype / variant / option not implemented */
    TWN_ERR_WORKSPACE = -5,   /* workspace NULL or too small */
    TWN_ERR_HIP = -6          /* the HIP runtime refused a launch */
} twn_status;

typedef enum { TWN_F32 = 0, TWN_BF16 = 1 } twn_dtype;

/* How the contraction consumes the ternary weights (Eq. 2 allows alpha to sit
 * on the weights, on the inputs or on the outputs). */
typedef enum {
    TWN_VAR_BF16_POSTSCALE = 0,     /* 2-bit codes -> exact bf16 in registers, bf16 MFMA, alpha in the fp32 epilogue */
    TWN_VAR_BF16_ALPHA_LDS = 1,     /* comparison: 2-bit codes -> the paper's operand alpha*W~ itself, bf16 {-alpha,0,+alpha}
                                       with alpha rounded to bf16, built when the codes are expanded; bf16 MFMA; no scaling
                                       of the sum afterwards.  Forward and backward-data. */
    TWN_VAR_I8_STORED_POSTSCALE = 2,/* comparison: weights stored as int8 {-1,0,1} [rows][K] (8 bits per weight, from
                                       twn_unpack_i8), bf16 MFMA, alpha afterwards.  Forward only; K % 8 == 0 and the
                                       weights 8-byte aligned, else TWN_ERR_UNSUPPORTED. */
    TWN_VAR_FP32 = 3,               /* float32 activations and outputs, vector-ALU FMAs with float64 running sums */
    TWN_VAR_BF16_SIGN1_POSTSCALE = 4,/* the binary-weight comparison of Sec. 3: 1-bit sign codes from twn_binarize
                                       (twn1 format) -> exact bf16 +-1, bf16 MFMA, alpha afterwards.  Forward only. */
    TWN_VAR_ADDSUB_SPARSE = 5       /* comparison: Eq. 2's multiplication-free form (Sec. 2.1 "Computational requirement").
                                       bf16 activations, the ordinary 2-bit codes; float32 additions and subtractions on
                                       the vector ALUs, one per non-zero code and pixel, none for a zero code; alpha and
                                       the block tail once per output.  Forward only; channel count, K and the pixel
                                       stride of X multiples of 8 and X, weights 16-byte aligned, else
                                       TWN_ERR_UNSUPPORTED. */
} twn_variant;

/* Filter bank [rows][C][R][S], float32, contiguous (fully-connected: R=S=1). */
typedef struct {
    int32_t rows, C, R, S;
} twn_weight_desc;

/* Y[M][N] = alpha * X[M][K] . W~[N][K]^T  (+ bias[N]) */
typedef struct {
    int64_t M;
    int32_t N, K;
    int32_t x_dtype, y_dtype;   /* twn_dtype */
    int32_t variant;            /* twn_variant */
    int64_t ldx, ldy;           /* row strides in elements; 0 = dense (K, N) */
    int32_t alpha_groups;       /* 1 = one alpha for the layer; N = one per output row group (must divide N) */
} twn_gemm_desc;

/* NHWC activations [N][H][W][C], filters [O][C][R][S], output [N][P][Q][O]
 * with P = (H + 2*pad_h - dil_h*(R-1) - 1)/stride_h + 1 (same for Q). */
typedef struct {
    int32_t N, H, W, C;
    int32_t O, R, S;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    int32_t x_dtype, y_dtype;   /* twn_dtype; for the backward, x_dtype covers X and dY, y_dtype covers dX */
    int32_t variant;            /* twn_variant */
    int32_t alpha_groups;       /* 1 or a divisor of O */
} twn_conv_desc;

/* Optional fused tail of the forward block (X_next = g(Z) of Eq. 2, with the
 * batch-norm affine of the ternary block of Sec. 2.4 folded to scale/shift):
 *   y = relu?( (alpha*acc) * scale[o] + shift[o] + residual )
 * scale / shift: float32 [O] or NULL; residual: same shape and dtype as Y or
 * NULL; relu: 0/1.  `shift` alone is a bias. */
typedef struct {
    const float* scale;
    const float* shift;
    const void* residual;
    int32_t relu;
} twn_epilogue;

const char* twn_status_str(int32_t status);   /* host; static string */
/* The library's tuning overrides (environment variables TWN_*: tile and kernel
 * choices for sweeps, none needed for normal use) are read once each, at their
 * first use.  A process that changes one afterwards calls twn_reload_env to
 * have it read again (host; thread-safe against launches on other threads). */
void twn_reload_env(void);
int32_t twn_abi_version(void);                 /* host */

/* ---- packed format helpers (host, pure) --------------------------------- */
int64_t twn_packed_words_per_row(int64_t K);           /* 8*ceil(K/128); 0 if K <= 0 */
size_t  twn_packed_bytes(int32_t rows, int64_t K);     /* rows * words_per_row * 4 */

/* ---- 1. ternarization (Sec. 2.3; Alg. 1 steps 3-7) ------------------------
 * W: float32 [rows][C][R][S], 16-byte aligned.  The tensor is split into
 * `groups` equal groups of consecutive filters (groups must divide rows):
 * groups = 1 is one (Delta, alpha) per layer, groups = rows is one per filter
 * as Alg. 1 prints it.  Per group g, with n the number of weights in it:
 *     Delta_g = (float)((double)delta_factor * sum|W_i| / n)      (rule of thumb)
 *     code_i  = +1 if W_i > Delta_g, -1 if W_i < -Delta_g, else 0  (Eq. 3)
 *     nnz_g   = |{i : |W_i| > Delta_g}|
 *     alpha_g = (float)(sum_{|W_i|>Delta_g} |W_i| / nnz_g), 0 when nnz_g = 0  (Eq. 5)
 * Sums are accumulated in float64 in a fixed order (results are bit-identical
 * run to run); comparisons are float32.
 * Outputs: packed [rows][words_per_row(R*S*C)] (twn2 format above);
 * packed_T [C][words_per_row(R*S*rows)] or NULL; delta, alpha: float32[groups];
 * nnz: uint64[groups].  delta_factor must be in (0, 1]. */
size_t  twn_ternarize_workspace_bytes(const twn_weight_desc* wd, int32_t groups);
int32_t twn_ternarize(const float* W, const twn_weight_desc* wd, int32_t groups,
                      float delta_factor,
                      uint32_t* packed, uint32_t* packed_T,
                      float* delta, float* alpha, uint64_t* nnz,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- 1a. twn_ternarize for callers that cannot allocate ---------------------
 * For code under HIP graph capture, tight serving loops and harnesses that
 * forbid allocation: the same computation, outputs and validation as
 * twn_ternarize, without the workspace argument.  The per-block partial sums
 * live in a fixed array of twn_ternarize_static_scratch_bytes() bytes (98304)
 * inside the library's device image, one copy per GPU, held until the process
 * ends; the call allocates and frees nothing.  The array serves every tensor
 * twn_ternarize accepts (fewer than 2^40 weights; larger: TWN_ERR_SHAPE); the
 * device ordinal must be below 64 (else TWN_ERR_UNSUPPORTED).  The first call
 * on a device looks the array's address up (host-side, no allocation).  All
 * calls on one GPU share that array: two calls that overlap on one GPU (two
 * streams, two threads) race; calls on one stream are ordered and safe. */
size_t  twn_ternarize_static_scratch_bytes(void);
int32_t twn_ternarize_static(const float* W, const twn_weight_desc* wd, int32_t groups,
                             float delta_factor,
                             uint32_t* packed, uint32_t* packed_T,
                             float* delta, float* alpha, uint64_t* nnz, void* stream);

/* ---- 1b. several tensors per call (same passages as above) ------------------
 * twn_ternarize for `count` <= 32 weight tensors at once, in three launches in
 * total for the tensors with one group and two more for those with several
 * (per-filter) groups: meant for the weight tensors of a network, which are too
 * small to fill the chip one at a time.  `items` is a
 * host array (read during the call, not retained); the pointers inside are
 * device pointers with the meaning and alignment of twn_ternarize's arguments
 * (packed_T may be NULL).  Results equal those of `count` separate calls up to
 * the order of the float64 partial sums.  Workspace: device memory, 8-byte
 * aligned, at least twn_ternarize_batch_workspace_bytes(count) bytes. */
typedef struct {
    const float* W;
    twn_weight_desc wd;
    uint32_t* packed;
    uint32_t* packed_T;
    float* delta;
    float* alpha;
    uint64_t* nnz;
    int32_t groups;     /* 1: one Delta, alpha for the tensor; rows: one per filter (Alg. 1 as printed); must divide rows;
                           delta, alpha, nnz then hold `groups` values each */
    int32_t reserved;   /* 0 */
} twn_ternarize_item;
size_t  twn_ternarize_batch_workspace_bytes(int32_t count);
int32_t twn_ternarize_batch(const twn_ternarize_item* items, int32_t count, float delta_factor,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Expand a packed matrix [rows][words_per_row(K)] to int8 codes [rows][K]
 * (the input of TWN_VAR_I8_STORED_POSTSCALE; also lets a caller inspect codes). */
int32_t twn_unpack_i8(const uint32_t* packed, int32_t rows, int64_t K, int8_t* codes, void* stream);

/* ---- 2a. inner product forward (Eq. 2; Alg. 1 step 8) ---------------------
 * X: [M][ldx] of x_dtype; `weights`: packed twn2 [N][words_per_row(K)]
 * (for TWN_VAR_I8_STORED_POSTSCALE: int8 [N][K]); alpha: float32[alpha_groups];
 * ep may be NULL; Y: [M][ldy] of y_dtype.  bf16 variants need x_dtype = BF16,
 * X 16-byte aligned and ldx % 8 == 0; TWN_VAR_FP32 needs x_dtype = F32.
 * Alignment of the outputs (all entry points of section 2): when the channel
 * count N and ldy are multiples of 8, Y (dX) and ep->residual must be 16-byte
 * aligned (rows are written with 16-byte stores); otherwise aligned to their
 * element size.  Violations return TWN_ERR_ALIGN before anything is launched. */
size_t  twn_gemm_fwd_workspace_bytes(const twn_gemm_desc* d);
int32_t twn_gemm_fwd(const twn_gemm_desc* d, const void* X, const void* weights,
                     const float* alpha, const twn_epilogue* ep, void* Y,
                     void* workspace, size_t workspace_bytes, void* stream);

/* ---- 2b. convolution forward (Eq. 2; Alg. 1 step 8) -----------------------
 * Cross-correlation (no kernel flip), zero padding.  X NHWC of x_dtype,
 * `weights` as for the GEMM with rows = O and K = R*S*C, Y NHWC of y_dtype. */
size_t  twn_conv2d_fwd_workspace_bytes(const twn_conv_desc* d);
int32_t twn_conv2d_fwd(const twn_conv_desc* d, const void* X, const void* weights,
                       const float* alpha, const twn_epilogue* ep, void* Y,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Two convolutions over the SAME input X in one call: the first convolution of a
 * residual block and its projection shortcut (the ResNet-18 of Sec. 3.1 has three
 * such block heads).  Results are those of two twn_conv2d_fwd calls (each problem
 * has its own filters, alpha, geometry, epilogue and output); when both problems
 * get the same tile shape and short reductions (K <= 1536) they run in ONE
 * launch, else one after the other.
 * Product variant, bf16 in and out, C % 8 == 0 (else TWN_ERR_UNSUPPORTED); d0 and
 * d1 must agree in N, H, W, C (else TWN_ERR_SHAPE); no workspace is used. */
int32_t twn_conv2d_fwd_pair(const twn_conv_desc* d0, const twn_conv_desc* d1, const void* X,
                            const void* weights0, const float* alpha0, const twn_epilogue* ep0, void* Y0,
                            const void* weights1, const float* alpha1, const twn_epilogue* ep1, void* Y1,
                            void* stream);

/* ---- 2c. straight-through backward (Alg. 1 steps 9-10) --------------------
 * Ordinary back-propagation with T = alpha W~ in place of W:
 *   dX[n,h,w,c]   = sum_{o,r,s} alpha_o * dY[n,p,q,o] * W~[o,c,r,s]   over the (p,q) that read (h,w)
 *   dW[o,c,r,s]   = dW_beta * dW[o,c,r,s] + sum_{n,p,q} X[n,ih,iw,c] * dY[n,p,q,o]
 *   dbias[o]      = sum_{n,p,q} dY[n,p,q,o]
 * dW is dL/dT, delivered unchanged as the gradient of the float32 master
 * weights (identity straight-through estimator: no clipping, no alpha, no
 * codes), float32 in [O][C][R][S] order.  X, dY of x_dtype (bf16), dX of
 * y_dtype.  packed_T is the transposed copy from twn_ternarize.  Any of dX
 * (with packed_T/alpha), dW (with X), dbias may be NULL to skip that part.
 * dW_beta is 0 (overwrite) or 1 (accumulate).  A fully-connected layer is the
 * case H=W=R=S=1.  d->variant may be TWN_VAR_BF16_POSTSCALE or
 * TWN_VAR_BF16_ALPHA_LDS (it only affects dX); others: TWN_ERR_UNSUPPORTED.
 * Strided layers with dilation 1 and O % 64 == 0 compute dX as one stride-1
 * problem per residue class of the output pixels when the workspace of
 * twn_conv2d_bwd_ste_workspace_bytes is passed (otherwise, and for other
 * shapes, by the generic gather: same result, slower).
 * With alpha_groups > 1 (one alpha per filter group, Alg. 1) alpha_o is a
 * factor inside the sum over o: dX then needs a workspace, where alpha_o*dY is
 * formed in float32 and kept as two bf16 terms (high part and remainder, about
 * 17 significant bits together); the contraction runs over each term, the
 * second pass adding onto the first, so no rounding of the inputs is added
 * (twice the contraction time on this path only). */
size_t  twn_conv2d_bwd_ste_workspace_bytes(const twn_conv_desc* d);
int32_t twn_conv2d_bwd_ste(const twn_conv_desc* d, const void* X, const void* dY,
                           const uint32_t* packed_T, const float* alpha,
                           void* dX, float* dW, float* dbias, float dW_beta,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ---- 1c. sign binarization of the binary-weight comparison (Sec. 3) ----------
 * The counterpart the paper measures ternary weights against: codes are the
 * sign of the weight (+1 for W >= 0, the zero included; -1 for W < 0) and the
 * scale is alpha_g = (float)(sum|W_i| / n) per group, i.e. Eq. 5 with no weight
 * set to zero.  Groups as in twn_ternarize.
 * twn1 format: the matrix view of the twn2 format ([rows][K], k = (r*S+s)*C + c,
 * rows padded to a multiple of 128 weights), one bit per weight, 1 = negative:
 * word j of a row holds k = 32j .. 32j+31, the code of k = 32j+2i in bit i and
 * that of k = 32j+2i+1 in bit 16+i (i = 0..15); padding bits are 0 (the
 * contraction never multiplies them: activations beyond K read as zero).
 * packed1: [rows][twn_packed1_words_per_row(R*S*C)], 16-byte aligned; alpha:
 * float32[groups].  Workspace: device memory, 8-byte aligned, at least
 * twn_binarize_workspace_bytes bytes. */
int64_t twn_packed1_words_per_row(int64_t K);          /* host: 4 * ceil(K / 128) */
size_t  twn_binarize_workspace_bytes(const twn_weight_desc* wd, int32_t groups);
int32_t twn_binarize(const float* W, const twn_weight_desc* wd, int32_t groups,
                     uint32_t* packed1, float* alpha,
                     void* workspace, size_t workspace_bytes, void* stream);

/* ---- 3. parameter update (Alg. 1 step 10; Sec. 2.4; Table 1) -----------------
 * SGD with momentum and L2 weight decay on the float32 weights that are kept
 * across iterations, with the gradient of twn_conv2d_bwd_ste (taken with respect
 * to the ternary weights) applied to them unchanged:
 *     g = dW[i] + weight_decay * W[i];  V[i] = momentum * V[i] + g;  W[i] -= lr * V[i]
 * in float32, each line one fused multiply-add.  W, V (velocity, zero before the
 * first step) and dW are device arrays of n floats, 16-byte aligned; W and V
 * are updated in place, dW is only read.
 * Fused with it is pass 1 of the next ternarization of this tensor as one
 * group: the per-block float64 sums of |W[i]| after the update are left in
 * `tern_workspace` (device memory, 8-byte aligned, at least
 * twn_ternarize_workspace_bytes bytes: the workspace of the twn_ternarize call
 * that follows), in the block partition and order twn_ternarize itself uses.
 * twn_ternarize_presummed is twn_ternarize with groups = 1 that trusts those
 * sums instead of reading W once more; its results are bit-identical to
 * twn_ternarize's on the updated tensor.  It must be given the workspace of
 * the twn_sgd_update call for the same W (n = rows*C*R*S), with no other use
 * of that workspace in between.  tern_workspace may be NULL (no sums). */
int32_t twn_sgd_update(float* W, float* V, const float* dW, int64_t n,
                       float lr, float momentum, float weight_decay,
                       void* tern_workspace, size_t workspace_bytes, void* stream);
int32_t twn_ternarize_presummed(const float* W, const twn_weight_desc* wd, float delta_factor,
                                uint32_t* packed, uint32_t* packed_T,
                                float* delta, float* alpha, uint64_t* nnz,
                                void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TWN_H */
