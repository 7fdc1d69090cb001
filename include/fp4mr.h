/*
 * fp4mr — micro-rotated FP4 linear-layer hot path for AMD MI355X (gfx950).
 *
 * C ABI of libfp4mr.so.  The library computes, for a linear layer with activations X [M,K] and weights
 * W [N,K] (both bf16, row-major),
 *
 *        Y = Q(X H_b) * Q(W H_b)^T            (arXiv 2509.23202, Section 4.1 "Ingredient 3", Section 4.2)
 *
 * where H_b is the block-diagonal normalised Hadamard rotation with b x b Sylvester blocks along K and Q
 * is round-to-nearest microscaling FP4 quantization with abs-max group scales (Section 2; Section 3,
 * definition "Scales"):
 *     MXFP4: groups of 32, E2M1 elements, E8M0 scale 2^(floor(log2 amax) - 2)     (OCP MX rule)
 *     NVFP4: groups of 16, E2M1 elements, E4M3 group scale s_G and one fp32 tensor scale s_T,
 *            Xhat = s_T * s_G * Q(X / (s_T * s_G))                                (Section 4.1 "Ingredient 1")
 *            with s_T = amax_T / 2688, s_G = E4M3(amax_g / (6 s_T)), all in binary32.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a parameter says "host".  The caller owns every
 *     buffer, including the workspace; the library allocates, frees and retains nothing.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *     Outputs are valid once the caller has synchronised with the stream.
 *   - Every argument is validated on the host before anything is launched: on any status other than
 *     FP4MR_OK and FP4MR_ERR_DEVICE nothing was launched and nothing was written.  FP4MR_ERR_DEVICE
 *     reports a launch that the HIP runtime refused; an entry point that launches several kernels may
 *     then have written part of its outputs or workspace.  No exception or abort crosses this boundary.
 *   - Data pointers must be 16-byte aligned.
 *   - Behaviour for NaN / Inf inputs is unspecified.
 *
 * Canonical layouts
 *   codes  [rows, K/2] bytes, row-major: byte j of a row holds element k=2j in bits 3:0 and k=2j+1 in
 *          bits 7:4.  A code is  s e1 e0 m : magnitudes 0..7 -> {0, 0.5, 1, 1.5, 2, 3, 4, 6}, bit 3 = sign.
 *   scales [rows, K/G] bytes, row-major.  MXFP4: byte e means 2^(e-127), 0xFF is never produced.
 *          NVFP4: E4M3 ("fn": bias 7, max 448, no infinities), sign bit always 0.
 * GEMM layout (FP4MR_LAYOUT_GEMM): an opaque tiled order produced by the two quantize calls and consumed
 *   by fp4_gemm; sizes come from fp4_packed_bytes (rows are padded to a multiple of 16, K to 128/512).
 *   Padding bytes are never read into a stored result and need not be initialised.
 */
#ifndef FP4MR_H
#define FP4MR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FP4MR_MXFP4 = 0, FP4MR_NVFP4 = 1 } fp4mr_fmt_t;

typedef enum {
    FP4MR_OK = 0,
    FP4MR_ERR_NULL = 1,       /* a required pointer is NULL */
    FP4MR_ERR_SHAPE = 2,      /* M, N or K <= 0, or K not a multiple of what the format/layout needs */
    FP4MR_ERR_HAD_BLOCK = 3,  /* had_block not in {1, 16, 32, 64, 128} */
    FP4MR_ERR_FMT = 4,        /* fmt is neither FP4MR_MXFP4 nor FP4MR_NVFP4, or unknown flag bits */
    FP4MR_ERR_ALIGN = 5,      /* a data pointer is not 16-byte aligned */
    FP4MR_ERR_WORKSPACE = 6,  /* workspace is NULL or smaller than fp4_workspace_bytes() says */
    FP4MR_ERR_DEVICE = 7      /* the HIP runtime reported an error at launch */
} fp4mr_status_t;

/* flags (bit field) */
enum {
    FP4MR_LAYOUT_CANONICAL = 0u,
    FP4MR_LAYOUT_GEMM = 1u << 0,          /* quantize calls: write codes and scales in GEMM layout           */
    FP4MR_INPUT_F32 = 1u << 1,            /* quantize calls: input is fp32 [rows,K]; requires had_block == 1  */
    FP4MR_STATIC_TENSOR_SCALE = 1u << 2,  /* NVFP4 quantize: *tensor_scale already holds s_T; do not derive it */
    FP4MR_A_LAYOUT_GEMM = 1u << 3,        /* fp4_gemm: A codes/scales are in GEMM layout (else canonical)     */
    FP4MR_W_LAYOUT_GEMM = 1u << 4,        /* fp4_gemm: W codes/scales are in GEMM layout (else canonical)     */
    FP4MR_OUT_F32 = 1u << 5,              /* fp4_gemm: write the fp32 accumulator instead of bf16             */
    FP4MR_SCALE_MSE = 1u << 6,            /* quantize ops: group scale by squared-error search (below)        */
    FP4MR_SCALE_ROUND43 = 1u << 7,        /* MXFP4 quantize ops: rounded exponent, scale (4/3) 2^k (below)    */
    FP4MR_A_SCALE43 = 1u << 8,            /* MXFP4 products: the A operand was quantized with SCALE_ROUND43   */
    FP4MR_W_SCALE43 = 1u << 9,            /* MXFP4 products: the W operand was quantized with SCALE_ROUND43   */
    FP4MR_SCALE_FIT_TENSOR = 1u << 10,    /* NVFP4 quantize ops, with SCALE_MSE: also fit the tensor scale    */
    FP4MR_SCALE_FIT_RANGE = 1u << 11      /* MXFP4 quantize ops: scale byte fitted to the tensor's range (below) */
};

/* operation selector for fp4_workspace_bytes */
enum { FP4MR_OP_ROTATE_QUANTIZE = 0, FP4MR_OP_QUANTIZE_WEIGHTS = 1, FP4MR_OP_GEMM = 2, FP4MR_OP_GPTQ = 3, FP4MR_OP_GPTQ_PREPARE = 4, FP4MR_OP_GPTQ_HESSIAN = 5,
       FP4MR_OP_GEMM_SPLIT_K = 6 /* fp4_gemm with room for split-K partials: see fp4_gemm's workspace */ };

/*
 * Online rotation + quantization of activations: codes, scales = Q(X H_b)   (Section 4.2 item 1: rotation
 * with quantization and scale calculation fused behind it; replaces the separate scale re-layout step of
 * Section 4.2 item 2 by writing GEMM layout directly when FP4MR_LAYOUT_GEMM is set).
 *   x            [M,K] bf16 (fp32 with FP4MR_INPUT_F32), row-major
 *   had_block    b in {1,16,32,64,128}; 1 = no rotation.  K must be a multiple of lcm(b, G) (and of 128 for
 *                GEMM layout).
 *   codes_out    canonical: M*K/2 bytes;  scales_out: M*K/G bytes (see fp4_packed_bytes for GEMM layout)
 *   tensor_scale NVFP4 only (NULL for MXFP4): one device float; written with s_T, or read if
 *                FP4MR_STATIC_TENSOR_SCALE is set.  (FP4MR_SCALE_FIT_RANGE: FP4MR_FIT_RANGE_FLOATS floats, see below.)
 *   workspace    device scratch of at least fp4_workspace_bytes(FP4MR_OP_ROTATE_QUANTIZE, ...) bytes
 *                (0 for MXFP4: may be NULL).
 */
fp4mr_status_t fp4_rotate_quantize(const void* x, int64_t M, int64_t K, int had_block, fp4mr_fmt_t fmt,
                                   void* codes_out, void* scales_out, float* tensor_scale,
                                   void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * fp4_rotate_quantize for callers that cannot allocate or pass device scratch -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: the same operation, same kernels and bit-identical results, with the
 * tensor-scale pass's scratch (FP4MR_STATIC_SCRATCH_BYTES: the per-wave partial maxima and the reduced maximum of an NVFP4
 * call with a dynamic tensor scale) in a device array that lives inside the library, one copy per GPU, held until the
 * process ends.  The call allocates nothing and frees nothing; its first use on a device asks the HIP runtime for the
 * array's address (make that first call outside a graph capture).  Arguments as fp4_rotate_quantize without the
 * workspace pair; M * K <= FP4MR_STATIC_MAX_ELEMENTS, beyond which the call returns FP4MR_ERR_SHAPE and launches
 * nothing.  Every call on a GPU shares that GPU's array: two NVFP4 calls without FP4MR_STATIC_TENSOR_SCALE that overlap
 * in time on one GPU (different streams, or different host threads) race on it and may return each other's tensor scale;
 * calls on one stream, MXFP4 calls (other than FP4MR_SCALE_FIT_RANGE ones, whose range pass uses it the same way) and
 * static-scale calls do not touch it.  Nothing in the array needs clearing
 * between calls: every word a call reads was written by that call's own first pass.
 */
#define FP4MR_STATIC_SCRATCH_BYTES (256 + 4096 * 4)
#define FP4MR_STATIC_MAX_ELEMENTS (1ll << 36)
fp4mr_status_t fp4_rotate_quantize_static(const void* x, int64_t M, int64_t K, int had_block, fp4mr_fmt_t fmt,
                                          void* codes_out, void* scales_out, float* tensor_scale, uint32_t flags,
                                          void* stream);

/*
 * Scale policy.  By default a group's scale is the abs-max one (Section 3 "Scales").  With FP4MR_SCALE_MSE the
 * scale code is chosen to minimise the group's squared error sum_i (xhat_i - x_i)^2 (the objective of Section 4.1
 * "Ingredient 1"; the "MSE" method of Section 4.2 item 1) inside a window around the abs-max code c0, a candidate
 * winning only with a strictly smaller error (evaluated in fp32), tried in this order:
 *     MXFP4: E8M0 byte c0, c0+1, c0-1;
 *     NVFP4: E4M3 code c0, c0+1, c0-1, c0+2, c0-2, c0+3, c0+4, c0+5, c0+6, c0+7, with the abs-max tensor scale.
 * The windows hold the minimiser over ALL scale codes in all but about 1e-4 of the groups of heavy-tailed inputs
 * (for NVFP4 it sits either next to c0 or about half an octave above it).  Hardware codec only.  Costs about twice
 * (MXFP4) / four times (NVFP4) the vector-ALU work of abs-max.
 *
 * With FP4MR_SCALE_MSE | FP4MR_SCALE_FIT_TENSOR (NVFP4 only, not with FP4MR_STATIC_TENSOR_SCALE: FP4MR_ERR_FMT) the tensor
 * scale is fitted too -- the alternating optimisation over the block scales and the per-tensor scale of Section 4.1
 * "Ingredient 1", meant for weights (offline): starting from the abs-max tensor scale, three times { group search as
 * above with s_T fixed; s_T = sum_i x_i v_i / sum_i v_i^2 with v_i = s_G * E2M1(code_i), the least-squares factor for
 * fixed codes and group scales, sums in fp64, one rounding to binary32 }, then the quantization proper with the final
 * s_T.  Eight passes over the input instead of two; workspace per fp4_workspace_bytes (about 80 KB).  Deterministic;
 * the fp64 sums are added in a fixed order that differs from a sequential one, so s_T can differ from a sequential
 * evaluation in its last bit.
 *
 * With FP4MR_SCALE_ROUND43 (MXFP4 only; not together with FP4MR_SCALE_MSE: FP4MR_ERR_FMT) the scale follows the
 * first equation of the appendix on MXFP scale fitting: s = (4/3) 2^k with k = clamp(round(log2(amax / 6)), -127, 127).
 * The scale byte stores k + 127; elements are E2M1(x / s), correctly rounded.  The factor 4/3 is not representable in
 * E8M0: it is a constant of the whole tensor, and the products take it as a flag -- FP4MR_A_SCALE43 / FP4MR_W_SCALE43
 * multiply the result by 4/3 for each operand so quantized (in fp32, before the output is rounded).
 *
 * With FP4MR_SCALE_FIT_RANGE (MXFP4 only, no other scale policy beside it: FP4MR_ERR_FMT) the scale byte is re-mapped
 * onto the range of scales the tensor actually has -- the modified format of the appendix on MXFP scale fitting,
 * s = 2^(alpha q + beta):
 *     alpha = (log2 a_max - log2 a_min) / 255,  beta = log2(a_min / 6),   a_min / a_max = the smallest non-zero / the largest
 *     group abs-max of the (rotated) tensor;   q = clamp(round((log2(amax / 6) - beta) / alpha), 0, 255) per group;
 *     elements = E2M1(x / s(q)), saturating (s(q) can lie below amax / 6 by half a step, 2^(alpha / 2)).
 * An all-zero group gets q = 0 and zero codes; one distinct scale gives alpha = 0; an all-zero tensor alpha = beta = 0.
 * tensor_scale must then point to FP4MR_FIT_RANGE_FLOATS device floats (FP4MR_ERR_NULL otherwise):
 *     [0] alpha, [1] beta, [2 + q] = s(q) for q = 0 .. 255, the binary32 scale values the elements were divided by
 * (log2 and exp2 are the GPU's binary32 instructions: decode with these 256 numbers, not by re-evaluating the formula).
 * With FP4MR_STATIC_TENSOR_SCALE the caller's alpha and beta in [0], [1] are used (weights and activations of a layer
 * sharing alpha, last paragraph of that appendix), the byte clamps to 0 .. 255, and [2 ..] is still written.
 * Three launches, two passes over the input; workspace per fp4_workspace_bytes (none when static).  The converting
 * instructions are used whatever the software-codec option says.  scales_out holds q
 * in the place and layout of the E8M0 bytes.  Such operands are NOT inputs of fp4_gemm, fp4_fused_linear or
 * fp4_w4a16_linear: their bytes are not E8M0 exponents and the scaled matrix instruction cannot take a fractional
 * alpha (the paper evaluates this format in emulation); the decoded tensor is E2M1(code) * s(q).
 */
#define FP4MR_FIT_RANGE_FLOATS 258

/*
 * The same with a caller-supplied rotation instead of the Hadamard: codes, scales = Q(X R) with R block-diagonal,
 * every diagonal block equal to rot (Section 4.2 item 1: for k < 256 a dense k x k transform stays memory-bound,
 * so any rotation -- DCT, DST, learned -- costs what the Hadamard costs; appendix tables on other transforms).
 *   block        k in {16,32,64,128}
 *   rot_bf16     device pointer, [block, block] bf16 row-major, 16-byte aligned; y[m, j*k + c] = sum_r x[m, j*k + r] *
 *                rot[r][c], accumulated in fp32.  The matrix carries its own normalisation.  Not retained after the
 *                call returns to the stream (the kernels read it; the caller keeps it alive until they finish).
 * Everything else as fp4_rotate_quantize (FP4MR_INPUT_F32 is not accepted).  Weights are prepared with the same
 * call (rows = N): the GEMM needs both operands rotated by the same matrix.
 */
fp4mr_status_t fp4_rotate_quantize_dense(const void* x, int64_t M, int64_t K, int block, const void* rot_bf16,
                                         fp4mr_fmt_t fmt, void* codes_out, void* scales_out, float* tensor_scale,
                                         void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Offline weight preparation: codes, scales = Q(W H_b) by round-to-nearest (Section 4.2 item 1: the weight-side
 * rotation is folded into the stored weights ahead of time; RTN + HT row of Section 5's method list).  Same
 * arguments as fp4_rotate_quantize with rows = N.  The calibrated alternative is fp4_gptq_quantize_weights below.
 */
fp4mr_status_t fp4_quantize_weights(const void* w, int64_t N, int64_t K, int had_block, fp4mr_fmt_t fmt,
                                    void* codes_out, void* scales_out, float* tensor_scale,
                                    void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * W4A4 product of two quantized operands: out[m,n] = sum_k Ahat[m,k] * What[n,k]  (Section 4.2 item 2),
 * fp32 accumulation, bf16 round-to-nearest-even output (fp32 with FP4MR_OUT_F32).  K % 128 == 0.
 *   a_codes/a_scales  [M,K] operand, w_codes/w_scales [N,K] operand, layouts per flags
 *   a_tensor_scale, w_tensor_scale   NVFP4: device floats s_T of each operand; MXFP4: NULL
 *   out          [M,N] row-major
 *   flags        layouts, FP4MR_OUT_F32, and for MXFP4 FP4MR_A_SCALE43 / FP4MR_W_SCALE43 (FP4MR_ERR_FMT with NVFP4)
 *   workspace    fp4_workspace_bytes(FP4MR_OP_GEMM, M, N, K, fmt, flags) bytes: room for operands handed over in
 *                row-major layout (they are re-tiled first), and, for NVFP4 with M > 64 on the shapes that the
 *                many-token kernel takes, 2 bytes per element of the activation operand (its exact fp16 values
 *                code * s_G are written once, so that the product kernel converts only W).  May be NULL when that size
 *                is 0 (MXFP4 with both operands in GEMM layout).
 *                Optional: with at least fp4_workspace_bytes(FP4MR_OP_GEMM_SPLIT_K, ...) bytes (the same plus room for
 *                fp32 partial results; equal to the former where the shape has nothing to gain) a product with few
 *                output tiles and a long K -- 65 to a few hundred tokens against a narrow layer -- is split along K
 *                over otherwise idle compute units and the partial results are added in a fixed order (deterministic;
 *                the fp32 sums are grouped per split, so the result can differ from the unsplit one in its last bits).
 */
fp4mr_status_t fp4_gemm(const void* a_codes, const void* a_scales, const float* a_tensor_scale,
                        const void* w_codes, const void* w_scales, const float* w_tensor_scale,
                        int64_t M, int64_t N, int64_t K, fp4mr_fmt_t fmt, void* out,
                        void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Few tokens in one launch: out = Q(X H_b) Q(W H_b)^T with the activations rotated and quantized inside the GEMM
 * (Section 4.2 items 1 and 2 fused; the paper's appendix on inference regimes: at small batch its separate kernels give
 * little).  Result bit-identical to fp4_rotate_quantize followed by fp4_gemm for had_block <= 32.
 *   x            [M,K] bf16 row-major, 1 <= M <= 4, K % 128 == 0.  Every workgroup (one per 16 rows of W) repeats the
 *                rotation and quantization of all M tokens, which hides under its weight stream up to four tokens;
 *                from five tokens on the two calls (fp4_rotate_quantize, fp4_gemm) are faster, so M > 4 is
 *                rejected with FP4MR_ERR_SHAPE
 *   had_block    b in {16,32,64,128}
 *   w_codes, w_scales   [N,K] operand in GEMM layout (flags must contain FP4MR_W_LAYOUT_GEMM)
 *   fmt          FP4MR_MXFP4 only (NVFP4's tensor scale needs a pass over all of X first: FP4MR_ERR_FMT)
 *   out          [M,N] bf16 (fp32 with FP4MR_OUT_F32)
 *   flags        FP4MR_W_LAYOUT_GEMM (required), FP4MR_OUT_F32, FP4MR_W_SCALE43 (weights quantized with
 *                FP4MR_SCALE_ROUND43; the activations are always quantized with the abs-max rule here)
 * No workspace.
 */
fp4mr_status_t fp4_fused_linear(const void* x, int64_t M, int64_t K, int had_block, const void* w_codes, const void* w_scales,
                                int64_t N, fp4mr_fmt_t fmt, void* out, uint32_t flags, void* stream);

/*
 * Weight-only variant of the same (W4A16): out = bf16(X H_b) Q(W H_b)^T.  The rotated activations are rounded to bf16
 * (round-to-nearest-even) instead of quantized; the weights' E2M1 codes are decoded with their E8M0 scales and the
 * product accumulates in fp32 (appendix on inference regimes: where the layer is memory-bound, weight-only
 * quantization loses no speed and keeps the activations' accuracy).  Arguments as fp4_fused_linear, except
 * 1 <= M <= 16 (the library has no other weight-only path; above four tokens it falls behind a bf16 GEMM on wide layers).
 */
fp4mr_status_t fp4_w4a16_linear(const void* x, int64_t M, int64_t K, int had_block, const void* w_codes, const void* w_scales,
                                int64_t N, fp4mr_fmt_t fmt, void* out, uint32_t flags, void* stream);

/*
 * Offline MR-GPTQ weight quantizer, the part that runs over the weight matrix (Section 4: all rows are quantized in one
 * fixed column order, each rounded column's error is pushed onto the columns still to come by the optimal-brain update;
 * Section 4.1: on the rotated weights W H_b, with the scales fixed beforehand in the original column order -- abs-max,
 * or FP4MR_SCALE_MSE / FP4MR_SCALE_ROUND43 -- and the columns visited in a static activation order).  Accumulating
 * the Hessian of the rotated calibration inputs comes from fp4_gptq_accumulate_hessian, and fp4_gptq_prepare turns it
 * into the two inputs taken here (both below):
 *   w            [N,K] bf16 row-major, K % 64 == 0, K % lcm(b, G) == 0, K <= 24576
 *   had_block    b in {1,16,32,64,128}
 *   hinv_u       [K,K] fp32 row-major, device: upper-triangular U with U^T U = (H[perm][:,perm] + lambda I)^-1, rows and
 *                columns in visiting order; only the upper triangle is read; the diagonal must be non-zero
 *   perm         [K] int32, device: perm[j] = original index of the column visited j-th (NULL: 0, 1, 2, ...).  Must be a
 *                permutation; entries outside [0,K) are clamped (garbage codes, no fault)
 *   codes_out, scales_out   canonical layout, as fp4_quantize_weights writes them (scales_out equals its output bit for
 *                bit: the sweep changes codes only); tensor_scale as there (NVFP4)
 *   workspace    fp4_workspace_bytes(FP4MR_OP_GPTQ, N, 0, K, fmt, flags) bytes
 *   flags        FP4MR_SCALE_MSE, FP4MR_SCALE_MSE | FP4MR_SCALE_FIT_TENSOR (NVFP4), FP4MR_SCALE_ROUND43 or
 *                FP4MR_SCALE_FIT_RANGE (MXFP4; tensor_scale then receives the FP4MR_FIT_RANGE_FLOATS floats and the sweep
 *                takes each group's scale from its 256 scale values), all optional: how the fixed grid is found;
 *                anything else: FP4MR_ERR_FMT
 * Per column j (visiting order), for every row:  q = E2M1(w_j / s),  e = (w_j - q s) / U[j,j],  w_k -= e U[j,k] (k > j),
 * in fp32; s is the fixed scale of the group the column belongs to in the ORIGINAL order.
 */
fp4mr_status_t fp4_gptq_quantize_weights(const void* w, int64_t N, int64_t K, int had_block, fp4mr_fmt_t fmt,
                                         const float* hinv_u, const int32_t* perm, void* codes_out, void* scales_out,
                                         float* tensor_scale, void* workspace, size_t workspace_bytes, uint32_t flags,
                                         void* stream);

/*
 * Hessian of a layer from calibration inputs (Section 4 "Standard GPTQ": the second-order information of
 * ||X What - X W||^2 is X^T X; Section 4.1 "Ingredient 3": of the ROTATED inputs):  H (+)= (X H_b)^T (X H_b), fp32.
 *   x          [T,K] bf16 row-major, device (T calibration rows; rows = M in fp4_workspace_bytes), K <= 24576
 *   hessian    [K,K] fp32 row-major, device; overwritten, or added to when accumulate != 0 (batches of rows)
 *   workspace  fp4_workspace_bytes(FP4MR_OP_GPTQ_HESSIAN, T, 0, K, fmt ignored, 0) = 4 T K bytes
 */
fp4mr_status_t fp4_gptq_accumulate_hessian(const void* x, int64_t T, int64_t K, int had_block, float* hessian, int accumulate,
                                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * From a layer's Hessian to the two inputs of fp4_gptq_quantize_weights (Section 4 "Standard GPTQ"; Section 4.1
 * "Ingredient 2": static activation order; Section 5 "Algorithms": dampening 1e-2):
 *   perm_out    [K] int32, device: columns by descending Hessian diagonal, equal entries in ascending index order
 *               (the identity when act_order == 0)
 *   hinv_u_out  [K,K] fp32 row-major, device: upper-triangular U with U^T U = (H[perm][:,perm] + damp mean(diag H) I)^-1,
 *               zero below the diagonal.  Computed in fp32 as the inverse of the upper factor R of A = R R^T (blocked
 *               Cholesky of the index-reversed matrix, triangular inversion by recursive doubling); no inverse of A is formed.
 *   hessian     [K,K] fp32 row-major, device, symmetric positive semi-definite: X'^T X' of the ROTATED calibration inputs
 *               (only read); K <= 24576; damp > 0 makes the dampened matrix positive definite
 *   workspace   fp4_workspace_bytes(FP4MR_OP_GPTQ_PREPARE, 0, 0, K, fmt ignored, 0) bytes (about 2.5 K^2 floats)
 * A Hessian that is not positive definite after dampening yields NaNs in hinv_u_out (no fault).
 */
fp4mr_status_t fp4_gptq_prepare(const float* hessian, int64_t K, float damp, int act_order, int32_t* perm_out, float* hinv_u_out,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The decoding side of the formats (Section 2: scale times element per group; Section 4.1 "Ingredient 1": NVFP4 with its
 * tensor scale; appendix on MXFP scale fitting): out[m, k] = E2M1(code) * scale of its group -- what an emulated
 * evaluation multiplies, and the consumer of FP4MR_SCALE_FIT_RANGE tensors.
 *   codes, scales   device pointers, as written by the quantize calls: canonical, or GEMM layout with FP4MR_LAYOUT_GEMM
 *   tensor_scale    NVFP4: one device float; FP4MR_SCALE_FIT_RANGE: the FP4MR_FIT_RANGE_FLOATS floats of the quantize call
 *                   (its 256 scale values are used); NULL otherwise
 *   out             device pointer, [rows, K] row-major bf16 (fp32 with FP4MR_OUT_F32), 16-byte aligned, written in full
 *   flags           FP4MR_LAYOUT_GEMM, FP4MR_OUT_F32, FP4MR_SCALE_ROUND43 (MXFP4: times the tensor-level 4/3),
 *                   FP4MR_SCALE_FIT_RANGE (MXFP4: the byte indexes the scale values); others: FP4MR_ERR_FMT
 * Binary32 arithmetic: MXFP4 exact; 4/3 rule, fitted range and NVFP4 (element times group scale is exact, then the tensor
 * scale) one rounding; bf16 output rounds that value to nearest even.  No workspace.  Errors as the quantize calls.
 */
fp4mr_status_t fp4_dequantize(const void* codes, const void* scales, const float* tensor_scale, int64_t rows, int64_t K,
                              fp4mr_fmt_t fmt, void* out, uint32_t flags, void* stream);

/*
 * Process-wide switches for tuning sweeps and cross-checks (none is needed for normal use; not thread-safe: set them
 * before calls are issued concurrently).  Returns FP4MR_ERR_FMT for an unknown option or a value out of range.
 *   FP4MR_OPT_GEMM_VARIANT  0 (default): fp4_gemm picks the tile shape from M, N, K; 1..18 (MXFP4) / 1..3 (NVFP4): force
 *                           one tile configuration (fp4_gemm returns FP4MR_ERR_FMT if the value is not valid for its format)
 *   FP4MR_OPT_GEMM_GRID     0 (default): one persistent workgroup per compute unit; n > 0: at most n workgroups
 *   FP4MR_OPT_SW_CODEC      1: the quantizers encode E2M1 / E4M3 with integer arithmetic instead of the converting
 *                           instructions (same results bit for bit; abs-max and 4/3 policies only)
 */
enum { FP4MR_OPT_GEMM_VARIANT = 0, FP4MR_OPT_GEMM_GRID = 1, FP4MR_OPT_SW_CODEC = 2 };
fp4mr_status_t fp4_set_option(int option, int value);

/*
 * Measured ceilings for a roofline report (the datasheet peaks assume a clock the chip does not hold under matrix load).
 * Each call launches one kernel on `stream`; the caller times it with events.
 *   FP4MR_PROBE_MFMA_FP4   register-resident issue loop of the block-scaled FP4 MFMA (16x16x128, E2M1 x E2M1) the MXFP4
 *                          product is built on: one workgroup of eight waves per compute unit, sixteen independent
 *                          accumulators per wave, no memory traffic.  flops = CUs * 8 * iters * 32 * 65536
 *   FP4MR_PROBE_MFMA_F16   the same with the fp16 MFMA (16x16x32) of the NVFP4 product.  flops = CUs * 8 * iters * 32 * 16384
 *     buf: device, at least 24 * CUs bytes; receives per compute unit three uint64: the raw differences of the two
 *     shader-readable counters (s_memtime, s_memrealtime) over the loop, and a checksum.  The counters' rates are
 *     machine-dependent (measured against host time on an MI355X: about half the shader clock and about 52 MHz), so
 *     rates are to be computed from the caller's event timing, not from them.  iters >= 1.
 *   FP4MR_PROBE_COPY       streaming copy of the first half of buf to the second half (16 bytes per lane, non-temporal):
 *                          bytes / 2 read + bytes / 2 written
 *   FP4MR_PROBE_READ       streaming read of the first half of buf: bytes / 2 read
 *     buf: device, 16-byte aligned, bytes >= 32; iters ignored.
 * Returns FP4MR_ERR_SHAPE for an unknown probe, a buffer that is too small or iters < 1, FP4MR_ERR_NULL / _ALIGN as usual.
 */
enum { FP4MR_PROBE_MFMA_FP4 = 0, FP4MR_PROBE_MFMA_F16 = 1, FP4MR_PROBE_COPY = 2, FP4MR_PROBE_READ = 3 };
fp4mr_status_t fp4_probe(int which, void* buf, size_t bytes, int iters, void* stream);

/* Bytes of device scratch the given operation needs (0 = none).  rows = M for the quantize ops. */
size_t fp4_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, fp4mr_fmt_t fmt, uint32_t flags);

/* Buffer sizes for an operand of `rows` x K in the layout selected by flags & FP4MR_LAYOUT_GEMM.
 * Returns FP4MR_OK and fills both outputs (host pointers). */
fp4mr_status_t fp4_packed_bytes(int64_t rows, int64_t K, fp4mr_fmt_t fmt, uint32_t flags,
                                size_t* codes_bytes, size_t* scales_bytes);

const char* fp4_status_string(fp4mr_status_t status);
int fp4_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FP4MR_H */
