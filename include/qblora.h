/*
 * qblora.h -- C ABI of the MI355X (gfx950) adapted quantized linear layer.
 *
 * The layer is the Q-BLoRA / QA-BLoRA one: a frozen 4-bit block-wise quantized
 * base weight (the triplet (w^, alpha, beta) of Eq. 1) is dequantized and
 * contracted with bf16 activations, and the balanced adapter of Sec. 3.2
 * (AvgPool(lambda) on the input, a rank lambda*D_rank product A B,
 * repeat_interleave(lambda) on the output, scaled by s) is added.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller unless stated
 *     otherwise.  The library never allocates, frees or keeps a pointer after
 *     the call returns; scratch memory is the caller's `workspace`.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream); no call synchronises the device.
 *   - Storage layout of the base weight is [d_out, d_in] row-major (the paper
 *     writes W as D_in x D_out with y = W^T x; Sec. 3.1), so Y = X W~^T.
 *   - A quantization block is `block` contiguous input indices k inside one
 *     output row n.  Block b of row n has index n*(d_in/block)+b.
 *   - 4-bit codes are packed two per byte: element (n,k) is in byte
 *     (n*d_in+k)/2, even k in the low nibble.
 *   - bf16 tensors are raw 16-bit patterns (qblora_bf16).
 *   - Return value: QBLORA_OK (0) or a negative QBLORA_ERR_* code.  Arguments
 *     are validated on the host before anything is enqueued; an invalid call
 *     enqueues nothing.  No entry point throws or aborts.
 */
#ifndef QBLORA_H
#define QBLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t qblora_bf16;

enum {
    QBLORA_OK = 0,
    QBLORA_ERR_NULL = -1,        /* a required pointer is NULL */
    QBLORA_ERR_SHAPE = -2,       /* a size is non-positive or not divisible as the method requires */
    QBLORA_ERR_UNSUPPORTED = -3, /* valid by the paper, not implemented by these kernels */
    QBLORA_ERR_WORKSPACE = -4,   /* workspace missing or smaller than *_workspace_bytes() */
    QBLORA_ERR_ALIGNMENT = -5,   /* beta-shift merge asked for tiles that do not cover whole blocks */
    QBLORA_ERR_LAUNCH = -6       /* the HIP runtime refused a launch */
};

enum { QBLORA_QUANT_ABSMAX_CODEBOOK = 0, QBLORA_QUANT_MINMAX_INT4 = 1 };
enum { QBLORA_SCALES_FP32 = 0, QBLORA_SCALES_E4M3_GROUPED = 1 };
enum { QBLORA_MERGE_BETA_SHIFT = 0, QBLORA_MERGE_REQUANT_MINMAX = 1 };

/*
 * The quantized weight: the triplet (w^, alpha, beta) of Eq. 1, w~ = alpha*c[w^] + beta.
 * The struct itself lives in host memory; the pointers in it are device pointers.
 *   codebook   16 ascending code values c_j (host values, copied by value into launches).
 *              Absmax/codebook quantizer (the NF4-style base of Sec. 3.2): any 16 ascending
 *              values in [-1,1].  Min-max INT4: 0,1,...,15.
 *   codes      [d_out*d_in/2] bytes.
 *   scales     alpha, fp32 [d_out*d_in/block].
 *   beta       beta,  fp32 [d_out*d_in/block], or NULL meaning beta = 0 (absmax quantizer).
 *   scale_mode QBLORA_SCALES_FP32: `scales` is what consumers read.
 *              QBLORA_SCALES_E4M3_GROUPED: consumers reconstruct the block scale i as
 *              fma(e4m3(scale_codes[i]), scale_step[i/scale_group], scale_mid[i/scale_group]);
 *              `scales` is then only written by the quantizer (the unquantized absmax values
 *              the codes were chosen against) and may be NULL for consumers.
 *   scale_codes [d_out*d_in/block] bytes, OCP E4M3 bit patterns.
 *   scale_step, scale_mid  fp32 [ceil(nblocks/scale_group)].
 *   block_rows 8 selects two-dimensional 8 x 8 quantization blocks (Sec. 3.3; Sec. 4.3 pairs block size 64
 *              with lambda1 = lambda2 = 8):
 *              block (i, j) covers output rows [8i, 8i+8) and inputs [8j, 8j+8), its scale / offset has
 *              index i*(d_in/8) + j; `codes` keeps the [d_out, d_in/2] packing.  Then every block lies in
 *              one (lambda1 x lambda2) adapter tile when 8 | lambda1 and 8 | lambda2, and the offset-shift
 *              merge (Alg. 2 get_new_beta) is exact.  Needs d_out % 8 == 0 and fp32 scales.  The caller sets
 *              the field before qblora_quantize_blockwise.  Taken by the quantizers, qblora_prepack_codes,
 *              qblora_dequantize_bf16, the forward / backward calls of both adapter forms, the
 *              merges (QBLORA_MERGE_BETA_SHIFT with the alignment rule 8 | lambda1 and 8 | lambda2; the
 *              requantizing merge and qblora_merge_bf16 for any lambdas, the former writing 8 x 8 blocks again)
 *              and the small-batch inference calls (which then contract bf16(fma(c, alpha, beta)) like the
 *              training forward).
 *              block = 32 with block_rows = 8 selects blocks of 8 output rows x 4 inputs, the other block shape
 *              Sec. 3.3 names ("4 x 8": lambda1 = 4 inputs by lambda2 = 8 outputs); scale / offset index
 *              i*(d_in/4) + j.  Taken by the quantizers, qblora_dequantize_bf16, the forward / backward calls of both
 *              adapter forms at any token count (they dequantize the weight once per call into the workspace, as
 *              calls on many tokens do -- the workspace sizes say so), the three merges (offset shift: 4 | lambda1
 *              and 8 | lambda2) and qblora_linear_decode (at every token count the kernel of the mid-batch form,
 *              i.e. bf16(fma(c, alpha, beta)) contracted; workspace from qblora_linear_decode_tokens_workspace_bytes).
 *              qblora_linear_fwd_noalloc returns QBLORA_ERR_UNSUPPORTED for them.
 *   codes_tiled optional second copy of the codes (NULL = absent) in the order the forward kernel
 *              streams them, qblora_codes_tiled_bytes() bytes: output rows in tiles of 256, and for
 *              tile i and 64-wide input step j one contiguous 8 KiB block at ((i*(d_in/64) + j)*256 + r)*32
 *              holding the 32 code bytes of row 256*i + r, inputs [64j, 64j+64) (runs of rows past d_out
 *              are never used for a result; qblora_prepack_codes zeroes them).  The base weight is frozen (Sec. 3.1), so this is a one-off re-layout: written by
 *              qblora_quantize_blockwise when the pointer is set, or by qblora_prepack_codes.  `codes`
 *              stays the reference layout; qblora_linear_fwd reads `codes_tiled` when it is present and
 *              `codes` otherwise, with identical results.
 */
typedef struct qblora_qweight {
    int32_t d_out;
    int32_t d_in;
    int32_t block;        /* 64 */
    int32_t scale_mode;
    int32_t scale_group;  /* 256 when scale_mode = E4M3_GROUPED, ignored otherwise */
    float codebook[16];
    uint8_t* codes;
    float* scales;
    float* beta;
    uint8_t* scale_codes;
    float* scale_step;
    float* scale_mid;
    uint8_t* codes_tiled;
    int32_t block_rows;   /* 1 (or 0): a block is `block` consecutive inputs of one output row;
                             8: a block is 8 output rows x 8 inputs (see below) */
} qblora_qweight;

/*
 * The balanced adapter (Sec. 3.2): A is [d_in/lambda1, R], B is [R, d_out/lambda2], both bf16
 * row-major; Q-BLoRA uses lambda1 = lambda2 = lambda and R = lambda*D_rank.  `s` is the
 * non-learned scaling of Sec. 3.1 and multiplies the adapter term only.
 * A = NULL, B = NULL or R = 0 means "no adapter" (base layer).
 */
typedef struct qblora_adapter {
    int32_t lambda1;
    int32_t lambda2;
    int32_t R;
    float s;
    const qblora_bf16* A;
    const qblora_bf16* B;
    int32_t scale_op;     /* QBLORA_OP_*; 0 = the method's AvgPool & repeat_interleave */
} qblora_adapter;

/*
 * Non-parametric scale operators around the adapter (Sec. 4.3 "The scale operators", Table 6).
 * With C the compress operator on the d_in input features and E the expand operator on the
 * d_out/lambda2 adapter outputs, the adapter term is s * E((C(x) A) B):
 *   QBLORA_OP_AVGPOOL_REPEAT   C(x)[m] = mean_i x[lambda1*m+i];  E(v)[n] = v[n / lambda2]   (Sec. 3.2)
 *   QBLORA_OP_TRUNCATE_PAD0    C(x)[m] = x[m] (front part kept); E(v)[n] = v[n] for n < d_out/lambda2, else 0
 *   QBLORA_OP_SAMPLE_ZEROFILL  C(x)[m] = x[lambda1*m];           E(v)[n] = v[n / lambda2] where lambda2 | n, else 0
 * The backward applies the transposed operators.  The two alternatives are the ablation's variants:
 * qblora_linear_fwd / _bwd (and their _save / _saved forms) take them; they additionally need
 * (d_in/lambda1) % 8 == 0 and (d_out/lambda2) % 8 == 0.  Their delta weight is not constant on
 * (lambda1 x lambda2) tiles, so qblora_tile_product and the merges refuse them (QBLORA_ERR_UNSUPPORTED).
 */
enum {
    QBLORA_OP_AVGPOOL_REPEAT = 0,
    QBLORA_OP_TRUNCATE_PAD0 = 1,
    QBLORA_OP_SAMPLE_ZEROFILL = 2
};

/*
 * Block-wise quantization of an fp32 weight (Eq. 1; Sec. 3.1 for the min-max and absmax
 * factors; Sec. 3.2 for the codebook base).
 *   W         fp32 [d_out, d_in], device.
 *   quantizer QBLORA_QUANT_ABSMAX_CODEBOOK: alpha = max|w| of the block, beta = 0,
 *             code = #{ j : w > ((c_j + c_{j+1}) * 0.5) * alpha } (nearest codebook entry,
 *             a value on a threshold takes the lower index).
 *             QBLORA_QUANT_MINMAX_INT4: alpha = (max-min)/15, beta = min,
 *             code = rint((w - min) * (15/(max-min))) (ties to even), all codes 0 when max = min;
 *             `codebook` is ignored and out->codebook is set to 0..15; out->beta must be non-NULL.
 *   scale_mode E4M3_GROUPED (absmax quantizer only): after the codes are chosen against the
 *             fp32 absmax scales, groups of 256 consecutive scales are re-encoded as
 *             mid = (min+max)*0.5, step = max|scale - mid|/448, code = E4M3 nearest-even of
 *             (scale - mid)/step saturating at 448 (step = 0 and codes 0 when all equal).
 *   out       host struct whose device pointers the caller has filled in (codes, scales, and
 *             beta or scale_codes/scale_step/scale_mid as the mode needs, codes_tiled or NULL); the
 *             call fills the scalar fields and the codebook and overwrites the device buffers.  The
 *             absmax quantizer sets out->beta to NULL (beta = 0).
 * All fp32 arithmetic is single IEEE operations in the order written above, so the outputs
 * are reproducible bit for bit.  d_in must be a multiple of `block`; block must be 64.
 */
int qblora_quantize_blockwise(const float* W, int32_t d_out, int32_t d_in, int32_t block,
                              int32_t quantizer, const float* codebook /* host, 16 values */,
                              int32_t scale_mode, qblora_qweight* out, void* stream);

/*
 * Size of the tiled code copy of a [d_out, d_in] weight, and the one-off re-layout itself
 * (qw->codes -> qw->codes_tiled, both device buffers of the caller).
 */
size_t qblora_codes_tiled_bytes(int32_t d_out, int32_t d_in);
int qblora_prepack_codes(const qblora_qweight* qw, void* stream);

/*
 * Dequantize (Eq. 1) to the 16-bit compute weight: Wt[n,k] = bf16(c[code]*alpha) or
 * bf16(fma(c[code], alpha, beta)), fp32 arithmetic then round-to-nearest-even.  This is the
 * weight the forward/backward kernels build on the fly in LDS; the standalone call exists
 * for inspection and tests.  Wt is bf16 [d_out, d_in], device.
 */
int qblora_dequantize_bf16(const qblora_qweight* qw, qblora_bf16* Wt, void* stream);

/*
 * How qblora_linear_fwd / _bwd build the 16-bit compute weight of Eq. 1 (Alg. 1: W_tilde = dequantize(...), then
 * x @ W_tilde).  Below qblora_dense_min_tokens() tokens every 256-token tile of the contraction kernel rebuilds
 * the weight tiles it needs from codes and scales in LDS; from that many tokens on, the call first dequantizes
 * the whole weight once into a bf16 buffer inside its workspace (d_out*d_in*2 bytes; transposed for the
 * backward) and the contraction kernel copies weight tiles from there, because rebuilding a tile for each of
 * T/256 token tiles costs more than one sweep over the weight.  The values are the same bf16 numbers either
 * way (qblora_dequantize_bf16's), and so are the results bit for bit.  The buffer is scratch: nothing is kept
 * between calls, and the *_workspace_bytes() queries include it.
 */
int64_t qblora_dense_min_tokens(void);

/* Bytes of workspace the forward / backward calls need for T tokens (0 is possible). */
size_t qblora_linear_fwd_workspace_bytes(const qblora_qweight* qw, const qblora_adapter* ad, int64_t T);
size_t qblora_linear_bwd_workspace_bytes(const qblora_qweight* qw, const qblora_adapter* ad, int64_t T);

/*
 * Adapted forward (Sec. 3.2, Alg. 1 qblora_forward, scaling on the adapter term only):
 *   Y[t,n] = sum_k X[t,k] * w~[n,k]  +  s * V[t, n / lambda2],
 *   V = (AvgPool_lambda1(X) A) B.
 *   X bf16 [T, d_in]; Y bf16 [T, d_out] (fully overwritten); accumulation in fp32.
 *   workspace: device scratch of at least qblora_linear_fwd_workspace_bytes(), 256-byte aligned.
 * Requires d_in % 64 == 0, d_out % 64 == 0, d_in % lambda1 == 0, d_out % lambda2 == 0,
 * R % 8 == 0.  T = 0 is a no-op.
 */
int qblora_linear_fwd(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X, int64_t T,
                      qblora_bf16* Y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of the forward above with respect to X, A and B (the base weight is frozen, Sec. 3.1):
 *   dV[t,j] = s * sum_{i<lambda2} dY[t, lambda2*j+i];  dB = U^T dV;  dU = dV B^T;
 *   dA = P^T dU;  dX[t,k] = sum_n dY[t,n] * w~[n,k] + (1/lambda1) * (dU A^T)[t, k / lambda1],
 * with P = AvgPool_lambda1(X), U = P A recomputed from X.
 *   dX bf16 [T, d_in]; dA fp32 [d_in/lambda1, R]; dB fp32 [R, d_out/lambda2]; all fully
 *   overwritten (not accumulated).  dA/dB may be NULL together (then only dX is produced);
 *   dX may be NULL (then only dA/dB).  Same shape requirements as the forward.
 */
int qblora_linear_bwd(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X,
                      const qblora_bf16* dY, int64_t T, qblora_bf16* dX, float* dA, float* dB,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same forward and backward with the adapter's inner activation kept in between, as a training
 * step does (the forward of Sec. 3.2 computes s*U = s * AvgPool_lambda1(X) A anyway; dB = U^T dV of
 * the backward needs it again).  `saved` is a device buffer of qblora_saved_bytes() bytes, 16-byte
 * aligned, owned by the caller: qblora_linear_fwd_save fills it (bf16 [T, R] high part of s*U
 * followed by bf16 [T, R] residual), qblora_linear_bwd_saved reads it instead of recomputing s*U from
 * X and must be given the buffer a forward call filled for the same X, adapter and T.  Results are
 * those of qblora_linear_fwd / qblora_linear_bwd bit for bit; everything else (arguments, workspace
 * sizes, errors) is as for those calls.  Without an adapter `saved` is ignored and may be NULL;
 * with one, NULL is QBLORA_ERR_NULL (the backward only needs it when dA/dB are asked for).
 */
size_t qblora_saved_bytes(const qblora_adapter* ad, int64_t T);
int qblora_linear_fwd_save(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X, int64_t T,
                           qblora_bf16* Y, qblora_bf16* saved, void* workspace, size_t workspace_bytes,
                           void* stream);
int qblora_linear_bwd_saved(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X,
                            const qblora_bf16* dY, int64_t T, const qblora_bf16* saved, qblora_bf16* dX,
                            float* dA, float* dB, void* workspace, size_t workspace_bytes, void* stream);

/*
 * qblora_linear_fwd for callers that cannot allocate device memory or hold a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks and results (bit
 * for bit) as qblora_linear_fwd, but the scratch is an array of QBLORA_NOALLOC_SCRATCH_BYTES bytes inside the
 * library's device image (each GPU the library runs on holds it until the process ends) instead of a caller
 * workspace; the call allocates nothing.  It always takes the form that rebuilds weight tiles in LDS (whose
 * scratch is the adapter operands, s*U and the re-ordered block scales: 4.5 MiB for the LLaMA-7B attention
 * projection at T = 8192, rank 64); a problem whose scratch in that form exceeds qblora_noalloc_scratch_bytes()
 * is rejected with QBLORA_ERR_WORKSPACE and nothing is enqueued.  All calls on one GPU share that GPU's array:
 * calls that overlap on one GPU (two streams, two host threads) race; calls on one stream do not.  The first
 * call on a device looks the array's address up (hipGetSymbolAddress); make it outside graph capture.
 */
#define QBLORA_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
size_t qblora_noalloc_scratch_bytes(void);
int qblora_linear_fwd_noalloc(const qblora_qweight* qw, const qblora_adapter* ad, const qblora_bf16* X, int64_t T,
                              qblora_bf16* Y, void* stream);

/*
 * Single-matrix adapter (QA-BLoRA, Sec. 3.3, Alg. 2 qablora_forward with the scaling on the adapter
 * term only): the trainable adapter is one matrix H, bf16 [d_in/lambda1, d_out/lambda2] row-major,
 * device memory, whose tiles can later be folded into the block offsets (qablora_merge_quantize).
 *   forward   Y[t,n] = sum_k X[t,k] * w~[n,k] + s * (AvgPool_lambda1(X) H)[t, n / lambda2]
 *   backward  dV[t,j] = s * sum_{i<lambda2} dY[t, lambda2*j+i];  dH = AvgPool_lambda1(X)^T dV;
 *             dX[t,k] = sum_n dY[t,n] * w~[n,k] + (1/lambda1) * (dV H^T)[t, k / lambda1]
 *   X bf16 [T, d_in]; Y, dY bf16 [T, d_out]; dX bf16 [T, d_in]; dH fp32 [d_in/lambda1, d_out/lambda2];
 *   outputs fully overwritten.  dX or dH may be NULL (not both); X may be NULL when dH is.
 *   The pooled input and the pooled output gradient are rounded to bf16 where they feed the MFMA
 *   kernels; accumulation is fp32.
 * Requires d_in % 64 == 0, d_out % 64 == 0, d_in % lambda1 == 0, d_out % lambda2 == 0 and
 * (d_in/lambda1) % 8 == 0, (d_out/lambda2) % 8 == 0.  workspace: device scratch of at least
 * qablora_linear_*_workspace_bytes(), 256-byte aligned.  T = 0: no-op (dH zeroed).
 */
size_t qablora_linear_fwd_workspace_bytes(const qblora_qweight* qw, int32_t lambda1, int32_t lambda2, int64_t T);
size_t qablora_linear_bwd_workspace_bytes(const qblora_qweight* qw, int32_t lambda1, int32_t lambda2, int64_t T);
int qablora_linear_fwd(const qblora_qweight* qw, const qblora_bf16* H, int32_t lambda1, int32_t lambda2, float s,
                       const qblora_bf16* X, int64_t T, qblora_bf16* Y, void* workspace, size_t workspace_bytes,
                       void* stream);
int qablora_linear_bwd(const qblora_qweight* qw, const qblora_bf16* H, int32_t lambda1, int32_t lambda2, float s,
                       const qblora_bf16* X, const qblora_bf16* dY, int64_t T, qblora_bf16* dX, float* dH,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Tile matrix of a two-matrix adapter, H = A B, fp32 [d_in/lambda1, d_out/lambda2] (Alg. 1
 * get_delta_weight before the expansion; the equivalent full-size delta weight is
 * dW[k,n] = H[k/lambda1, n/lambda2]/lambda1, Sec. 3.2 "Merging Q-BLoRA").
 * workspace: at least qblora_tile_product_workspace_bytes().
 */
size_t qblora_tile_product_workspace_bytes(const qblora_adapter* ad, int32_t d_in, int32_t d_out);
int qblora_tile_product(const qblora_adapter* ad, int32_t d_in, int32_t d_out, float* H,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * QA-BLoRA merge (Sec. 3.3, Alg. 2 get_new_beta): fold the adapter, given as its tile matrix
 * H fp32 [d_in/lambda1, d_out/lambda2] (a QA-BLoRA single-matrix adapter is already in this
 * form; a Q-BLoRA adapter goes through qblora_tile_product), into block-wise INT4 parameters.
 * The shift of element (n,k) is delta = (s * H[k/lambda1, n/lambda2]) / lambda1 in fp32.
 *   QBLORA_MERGE_BETA_SHIFT      needs every quantization block inside one (lambda1 x lambda2)
 *                                tile (lambda1 % block == 0), else QBLORA_ERR_ALIGNMENT.
 *                                out->beta[b] = base beta[b] + delta (delta alone when the base
 *                                has no beta); codes and alpha are copied to out unless out
 *                                aliases base's buffers.  out keeps base's codebook; its scales
 *                                are fp32 (reconstructed when the base has grouped scales).
 *   QBLORA_MERGE_REQUANT_MINMAX  per block, w' = w~ + delta with w~ = c*alpha or fma(c,alpha,beta)
 *                                in fp32, then the min-max INT4 quantizer of
 *                                qblora_quantize_blockwise; out gets codes, alpha, beta and
 *                                the codebook 0..15, scale_mode FP32.
 * `out` is a host struct with caller-filled device pointers (codes, scales, beta), as for the
 * quantizer; the merge does not write a tiled code copy and sets out->codes_tiled to NULL.  Outputs are reproducible bit for bit given H.
 */
int qablora_merge_quantize(const qblora_qweight* base, const float* H, int32_t lambda1, int32_t lambda2,
                           float s, int32_t mode, qblora_qweight* out, void* stream);

/*
 * The same merge for `count` weights with common lambdas, scale and mode -- the projections of a layer (Sec. 3.3 merges
 * every adapted matrix of the model).  bases / H / outs are host arrays of `count` pointers, entry m as the arguments
 * of qablora_merge_quantize.  Requantizing merges of row-segment weights that share the scale format and the presence
 * of offsets go out as one launch per 8 weights (no idle tail and no launch gap between them); anything else is
 * merged one weight after the other.  Same outputs, bit for bit, as `count` single calls.  All weights are validated
 * before anything is written or launched; count = 0 is a no-op.
 */
int qablora_merge_quantize_batch(int32_t count, const qblora_qweight* const* bases, const float* const* H,
                                 int32_t lambda1, int32_t lambda2, float s, int32_t mode, qblora_qweight* const* outs,
                                 void* stream);

/*
 * Merge into a 16-bit weight (Sec. 3.2 "Merging Q-BLoRA", Alg. 1 get_delta_weight):
 *   W16[n,k] = bf16( w~[n,k] + (s * H[k/lambda1, n/lambda2]) / lambda1 ),
 * w~ = c*alpha or fma(c, alpha, beta) and the sum in fp32 (the arithmetic of the requantizing merge), one
 * rounding to bf16 (ties to even); reproducible bit for bit.  H fp32 [d_in/lambda1, d_out/lambda2] as for
 * qablora_merge_quantize (qblora_tile_product for a two-matrix adapter); W16 bf16 [d_out, d_in], device,
 * 16-byte aligned, fully overwritten.  X * W16^T then equals the adapted layer up to that one rounding.
 */
int qblora_merge_bf16(const qblora_qweight* base, const float* H, int32_t lambda1, int32_t lambda2, float s,
                      qblora_bf16* W16, void* stream);

/*
 * Small-batch forward of a quantized layer without adapter -- inference on the INT4 model that
 * qablora_merge_quantize produces (Sec. 3.3: the fine-tuned model is deployed in 4 bits), or on any
 * other qblora_qweight, for 1 <= T <= 256 tokens.
 * 1 <= T <= 16 (decode batches), bound by the weight stream from HBM:
 *   Y[t,n] = sum_b ( alpha[n,b] * sum_{k in block b} X[t,k] * bf16(c[code[n,k]]) + beta[n,b] * sum_{k in b} X[t,k] ),
 * fp32 accumulation.  Scale and offset act on the block sums, so the weight itself is never rounded to
 * 16 bits; for the integer codebook of INT4 models bf16(c) = c and the result is Eq. 1 contracted in
 * fp32.  It differs from qblora_linear_fwd without adapter (which contracts the bf16-rounded weight)
 * by that rounding only.
 * 16 < T <= 256 (mid batch: prefill chunks, batched decode), in chunks of at most 128 tokens:
 *   Y[t,n] = sum_k X[t,k] * bf16( c[code[n,k]] * alpha (+ beta) ),
 * the arithmetic of qblora_linear_fwd without adapter (Eq. 1 rounded once to the bf16 compute weight, fp32
 * accumulation), on token tiles of 32 / 64 / 128 with the input dimension split over workgroups; the fp32
 * partial tiles of the splits are added in a fixed order (reproducible bit for bit).
 *   X bf16 [T, d_in], 16-byte aligned; Y bf16 [T, d_out], fully overwritten.
 *   workspace: T <= 16: qblora_linear_decode_workspace_bytes() bytes (non-zero only for grouped scales, and
 *   not needed with a pack); T > 16: qblora_linear_decode_tokens_workspace_bytes(qw, T) bytes, 16-byte aligned
 *   (the former plus the partial tiles).
 * T = 0 is a no-op; T > 256 is QBLORA_ERR_SHAPE (use qblora_linear_fwd).  With T <= 16 a weight whose codes take
 * 2 GB or more (d_out rounded up to 256, times d_in / 2) is QBLORA_ERR_UNSUPPORTED: the kernel addresses them with
 * 32-bit offsets.
 */
size_t qblora_linear_decode_workspace_bytes(const qblora_qweight* qw);
size_t qblora_linear_decode_tokens_workspace_bytes(const qblora_qweight* qw, int32_t T);
int qblora_linear_decode(const qblora_qweight* qw, const void* pack, const qblora_bf16* X, int32_t T, qblora_bf16* Y,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * One-off re-layout of a (frozen) quantized weight for qblora_linear_decode: `pack` is a device buffer of
 * qblora_decode_pack_bytes() bytes, 256-byte aligned, owned by the caller, that receives the codes, the
 * fp32 block scales (grouped scales are reconstructed) and the offsets in tile order (rows in tiles of
 * 256; the values of one block for the rows of a tile are adjacent), so that a wave's load of one block
 * for 16 rows touches 5 cache lines instead of 32.  qblora_linear_decode with pack = NULL reads the
 * row-major arrays of `qw` (the same sums, 2-3 times slower on large layers); with a pack a call of at most
 * 16 tokens needs no workspace.
 * A pack belongs to the description it was made from: pass the same `qw` (codebook, offsets, block shape)
 * to qblora_linear_decode.  For an INT4 model -- codebook exactly 0, 1, ..., 15 with offsets, 64-blocks, the
 * output of the min-max quantizer and of qablora_merge_quantize -- the pack also regroups the nibbles of
 * every code dword and the kernel contracts the codes as the bf16 values 128 + c, taking the 128 off through
 * the block's activation sum (alpha*sum x(128+c) + (beta - 128 alpha)*sum x): the same sums in another
 * rounding order, equal to the unpacked result to about 1e-5 of the output scale, not bit for bit.
 */
size_t qblora_decode_pack_bytes(const qblora_qweight* qw);
int qblora_decode_pack(const qblora_qweight* qw, void* pack, void* stream);

/*
 * Measurement hook.  Registers a pair of caller-created hipEvent_t (passed as void*) that the next
 * calls record on their stream immediately before and after ONE kernel launch, so that a
 * benchmark can time that kernel alone while running the whole path:
 *   QBLORA_PROFILE_FWD_GEMM   the dequantize-and-contract kernel of qblora_linear_fwd
 *   QBLORA_PROFILE_BWD_GEMM   the transposed dequantize-and-contract kernel of qblora_linear_bwd
 *   QBLORA_PROFILE_MERGE      the requantizing (or beta-shift) kernel of qablora_merge_quantize
 *   QBLORA_PROFILE_QUANTIZE   the code-selection kernel of qblora_quantize_blockwise
 *   QBLORA_PROFILE_ADAPTER_FWD    the narrow GEMM s*U = s * AvgPool(X) A of the forward
 *   QBLORA_PROFILE_ADAPTER_BWD    the narrow GEMM dU = dV B^T of the backward
 *   QBLORA_PROFILE_ADAPTER_GRADS  the token contractions behind dA and dB (partial sums, both in one launch)
 *   QBLORA_PROFILE_GRAD_REDUCE    the fixed-order reduction of those partial sums into dA and dB
 *   QBLORA_PROFILE_PREP           the per-call re-layout launch of the forward (adapter operands, block scales)
 *   QBLORA_PROFILE_TILE_PRODUCT   the kernel of qblora_tile_product
 *   QBLORA_PROFILE_DEQUANT        the one-off dequantize pass of a forward / backward call on many tokens
 * Passing NULL for both events unregisters the slot.  The registration is per host thread: it applies to
 * calls made by the thread that registered it, so concurrent callers do not see each other's events.  Has
 * no effect on results.
 */
enum { QBLORA_PROFILE_FWD_GEMM = 0, QBLORA_PROFILE_BWD_GEMM = 1, QBLORA_PROFILE_MERGE = 2,
       QBLORA_PROFILE_QUANTIZE = 3, QBLORA_PROFILE_ADAPTER_FWD = 4, QBLORA_PROFILE_ADAPTER_BWD = 5,
       QBLORA_PROFILE_ADAPTER_GRADS = 6, QBLORA_PROFILE_GRAD_REDUCE = 7, QBLORA_PROFILE_PREP = 8,
       QBLORA_PROFILE_TILE_PRODUCT = 9, QBLORA_PROFILE_DEQUANT = 10, QBLORA_PROFILE_SLOTS = 11 };
int qblora_profile_events(int32_t which, void* start_event, void* stop_event);

/* Static description of an error code. */
const char* qblora_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* QBLORA_H */
