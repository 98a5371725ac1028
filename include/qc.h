/*
 * libqc -- the quantized-linear hot path of QuantCache (arxiv 2503.06545) for one
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes, no C++ or framework types.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers unless a parameter says "host".  Buffers
 *     are owned by the caller; the library never allocates, frees or synchronises.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work on that stream and return; they are asynchronous.
 *   - Tensors are dense and row major: X [M, K] (token major), W [N, K] (output
 *     channel major, the nn.Linear convention), Y [M, N];  Y = X * W^T + bias.
 *   - Data pointers must be 16-byte aligned.
 *   - Errors are return codes.  Argument errors are found before anything is
 *     launched, so a failed call has no side effect.  NaN / Inf in inputs are not
 *     detected; results are then unspecified.
 *
 * Quantizer (Section 3.1, Eq. (3) and Eq. (4) of the paper, in symmetric signed
 * form; Section 4.1 "Quantization Scheme": per-channel weights, activation scales
 * computed online).  For a row x (a token of X, or an output channel of W) and
 * qmax = 2^(bits-1) - 1 (127 or 7):
 *      a   = max_k |x_k|
 *      s   = max(a, 2^-64) / qmax              IEEE binary32 division
 *      q_k = clamp(rne(x_k / s), -qmax, qmax)  IEEE binary32 division, ties to even
 * Scales are binary32 and are part of the bit-exact contract.
 */
#ifndef QC_H
#define QC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QC_OK = 0,
    QC_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bad enum, misaligned pointer */
    QC_ERR_UNSUPPORTED = 2, /* a size or combination this library does not implement */
    QC_ERR_WORKSPACE = 3,   /* workspace_bytes smaller than the matching *_workspace_bytes() */
    QC_ERR_DEVICE = 4       /* the HIP runtime refused a launch */
} qc_status;

typedef enum { QC_F32 = 0, QC_BF16 = 1 } qc_dtype;

/* Activation applied after dequantization and bias (the STDiT MLP's fc1 uses GELU). */
typedef enum { QC_EPI_NONE = 0, QC_EPI_GELU_TANH = 1, QC_EPI_GELU_ERF = 2 } qc_epilogue;

/* Output element type.  QC_OUT_I32_ACC is a test hook: the raw int32 accumulators
 * (no scales, no bias, no activation), Y then is int32 [M, N]. */
typedef enum { QC_OUT_F32 = 0, QC_OUT_BF16 = 1, QC_OUT_I32_ACC = 2 } qc_out;

/* Largest reduction length: 127 * 127 * K must stay below 2^31. */
#define QC_MAX_K 131072
/* Largest number of output channels (the GEMM addresses a row of Y with 32-bit lane offsets). */
#define QC_MAX_N 67108864
/* Most earlier tensors one qc_cumulative_variation call compares against. */
#define QC_MAX_PREV 8

const char *qc_status_string(qc_status status);
/* Library version (major * 1000 + minor).  The packed-weight blob and the workspaces are
 * opaque and belong to the version that wrote them: the minor number changes whenever their
 * internal order does (the blob's header carries a layout tag of its own). */
int qc_version(void);

/* ---- sizes (host, pure functions) ------------------------------------------------ */

/* Bytes of the opaque packed-weight blob for W [N, K] at `bits` (8 or 4).
 * 0 if the combination is unsupported (bits not 4/8, N or K < 1, K > QC_MAX_K, N > QC_MAX_N,
 * bits == 4 with odd K). */
size_t qc_packed_weight_bytes(int64_t N, int64_t K, int bits);

/* Bytes of scratch qc_qlinear needs: the int8 codes of X in the GEMM's tiled
 * order plus one scale per token.  0 if M or K is out of range. */
size_t qc_qlinear_workspace_bytes(int64_t M, int64_t K, int64_t N);

/* Bytes of scratch qc_latent_delta needs for n elements (does not depend on n
 * beyond a fixed cap on the number of partial sums). */
size_t qc_latent_delta_workspace_bytes(int64_t n);

/* ---- S1: offline weight quantization and packing ----------------------------------
 * Section 4.1 "Quantization Scheme" (per-channel weight quantization) and Section
 * 3.2 AIGQ (1) (the bit-width is fixed per layer by the importance assignment, here
 * an argument).
 *   W        device, float [N, K]
 *   bits     8 or 4; bits == 4 needs an even K
 *   packed   device, qc_packed_weight_bytes(N, K, bits) bytes, 256-byte aligned.
 *            Opaque: a 256-byte header (layout tag, N, K, bits) then the codes in the
 *            order the GEMM consumes them.  It can be saved and restored as bytes.
 *   w_scale  device, float [N]: s of each output channel
 * Errors: INVALID_ARG (null, N/K < 1, alignment), UNSUPPORTED (bits, odd K with
 * bits 4, K > QC_MAX_K), DEVICE. */
qc_status qc_pack_weight(const float *W, int64_t N, int64_t K, int bits, void *packed,
                         float *w_scale, void *stream);

/* Test hook: expand a packed blob back to canonical codes, int8 [N, K] row major
 * (4-bit codes sign-extended to int8). */
qc_status qc_unpack_weight_codes(const void *packed, int64_t N, int64_t K, int bits,
                                 int8_t *codes, void *stream);

/* ---- S2: per-token dynamic activation quantization --------------------------------
 * Section 4.1 "Quantization Scheme" (activation parameters computed online), Eq. (3)
 * and Eq. (4) with one scale per token row.
 *   X        device, [M, K] of `xdt` (float or bf16), leading dimension K
 *   qx       device, int8 [M, K] row major: the codes
 *   x_scale  device, float [M]
 * Errors: INVALID_ARG, UNSUPPORTED (K > QC_MAX_K), DEVICE. */
qc_status qc_quant_act(const void *X, qc_dtype xdt, int64_t M, int64_t K, int8_t *qx,
                       float *x_scale, void *stream);

/* ---- S2+S3+S4: fused quantized linear ----------------------------------------------
 * Section 4.1 "Hardware Implementation": the DiT linear as a low-bit GEMM with the
 * quantization and dequantization fused around it.
 *   Y[m, n] = act( acc[m, n] * x_scale[m] * w_scale[n] + bias[n] ),
 *   acc[m, n] = sum_k qx[m, k] * qw[n, k]   exactly, in int32
 * where qx / x_scale are what qc_quant_act computes for X, and qw / w_scale what
 * qc_pack_weight stored.
 *   X          device, [M, K] of `xdt`
 *   packed     device, blob written by qc_pack_weight(.., N, K, bits, ..)
 *   w_scale    device, float [N]
 *   bias       device, float [N], or NULL for no bias
 *   Y          device, [M, N] of float (QC_OUT_F32), bf16 (QC_OUT_BF16) or int32
 *              (QC_OUT_I32_ACC; bias and epi are then ignored)
 *   workspace  device, >= qc_qlinear_workspace_bytes(M, K, N) bytes, 256-byte aligned;
 *              contents on entry are irrelevant, on exit it holds the activation codes
 *              in tiled order (see qc_debug_workspace_act)
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, DEVICE. */
qc_status qc_qlinear(const void *X, qc_dtype xdt, int64_t M, int64_t K, const void *packed,
                     const float *w_scale, int bits, int64_t N, const float *bias,
                     qc_epilogue epi, void *Y, qc_out ydt, void *workspace,
                     size_t workspace_bytes, void *stream);

/* The two halves of qc_qlinear as calls of their own: qc_qlinear(..) is exactly
 * qc_qlinear_quant(..) followed by qc_qlinear_gemm(..) on the same stream.  They serve a
 * caller that feeds one activation tensor to several linears (quantize once, multiply
 * several times) and the benchmark, which times the halves separately.
 *   qc_qlinear_quant  X [M, K] -> workspace (codes in the GEMM's tiled order + scales)
 *   qc_qlinear_gemm   workspace written by qc_qlinear_quant for the same M, K -> Y [M, N]
 * Arguments, sizes and errors as for qc_qlinear. */
qc_status qc_qlinear_quant(const void *X, qc_dtype xdt, int64_t M, int64_t K, void *workspace,
                           size_t workspace_bytes, void *stream);
qc_status qc_qlinear_gemm(const void *workspace, size_t workspace_bytes, int64_t M, int64_t K,
                          const void *packed, const float *w_scale, int bits, int64_t N,
                          const float *bias, qc_epilogue epi, void *Y, qc_out ydt, void *stream);

/* ---- activation bit-width as an argument ----------------------------------------------
 * Section 3.2 AIGQ (2), Eq. (8): the activation bit-width is switched per timestep between
 * a maximum, a middle and a minimum value; Table 1 reports the W4A6 operating point.  These
 * variants take it as `act_bits` = 8, 6 or 4: the same quantizer with qmax = 2^(act_bits-1) - 1
 * (127, 31, 7), codes still stored one per int8, so the GEMM is unchanged.  The calls without
 * the argument are these with act_bits = 8.  Other values: QC_ERR_UNSUPPORTED. */
qc_status qc_quant_act_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                            int8_t *qx, float *x_scale, void *stream);
qc_status qc_qlinear_quant_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                                void *workspace, size_t workspace_bytes, void *stream);
qc_status qc_qlinear_act_bits(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                              const void *packed, const float *w_scale, int bits, int64_t N,
                              const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                              void *workspace, size_t workspace_bytes, void *stream);

/* ---- rotation fused into the quantization ------------------------------------------------
 * Section 3.2 AIGQ (1): a lightweight rotation evens out the channels before quantization;
 * Section 4.1 "Hardware Implementation": the rotation is fused with the quantization kernel.
 * The paper does not give the matrix.  Here it is block diagonal over the reduction axis:
 * every run of `rot_block` consecutive columns (16, 32, 64 or 128; K a multiple of it) is
 * multiplied by the Walsh-Hadamard matrix H of that size (entries +1/-1, natural order).
 * Activations become X H before their absmax and cast, inside the quantization kernel;
 * qc_pack_weight_rot stores the codes of W H / rot_block, so that the product is unchanged:
 * (X H)(W H / rot_block)^T = X W^T.  H is applied as a butterfly network in binary32 with
 * strides 1, 2, 4, .. in ascending order (one rounding per output per stage); that order is
 * part of the bit-exact contract.
 *   qc_pack_weight_rot    qc_pack_weight on the counter-rotated weights
 *   qc_quant_act_rot      qc_quant_act_bits on the rotated activations
 *   qc_qlinear_quant_rot  qc_qlinear_quant_bits on the rotated activations
 *   qc_qlinear_rot        qc_qlinear_quant_rot then qc_qlinear_gemm; `packed` / `w_scale` must
 *                         come from qc_pack_weight_rot with the same rot_block (not checked)
 * Other arguments and errors as for the calls they extend.  UNSUPPORTED: rot_block not one of
 * 16/32/64/128, K not a multiple of it, or K > 9216. */
qc_status qc_pack_weight_rot(const float *W, int64_t N, int64_t K, int bits, int rot_block,
                             void *packed, float *w_scale, void *stream);
qc_status qc_quant_act_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                           int rot_block, int8_t *qx, float *x_scale, void *stream);
qc_status qc_qlinear_quant_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                               int rot_block, void *workspace, size_t workspace_bytes,
                               void *stream);
qc_status qc_qlinear_rot(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                         int rot_block, const void *packed, const float *w_scale, int bits,
                         int64_t N, const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                         void *workspace, size_t workspace_bytes, void *stream);

/* ---- asymmetric activation quantization ---------------------------------------------------
 * Section 3.1, Eq. (3) and Eq. (4) as printed: unsigned codes with a zero point, here one scale
 * and one zero point per token.  With levels = 2^act_bits - 1 (255, 63, 15), lo / hi the
 * minimum / maximum of the token's row, every step one IEEE binary32 operation:
 *      s = max(hi - lo, 2^-64) / levels
 *      z = -rne(lo / s)                              (the zero point the paper leaves open:
 *                                                     the row minimum gets code 0)
 *      q = clamp(rne(x / s) + z, 0, levels)          dequantized value  s * (q - z)
 * Weights stay symmetric, so
 *      Y[m, n] = act( s[m] w_scale[n] * sum_k (q[m, k] - z[m]) qw[n, k] + bias[n] ).
 * The GEMM runs on the signed bytes q - h, with h = 128 for act_bits 8 and h = 0 for 6 and 4
 * (those codes fit a signed byte as they are); the epilogue adds (h - z[m]) * w_row_sums[n] in
 * binary32.  One-sided inputs (the post-GELU input
 * of the MLP's second linear) gain about one bit over the symmetric form.
 *
 *   qc_weight_row_sums   w_row_sums[n] = sum_k qw[n, k] (int32 [N], device, 16-byte aligned),
 *                        computed once from a blob written by qc_pack_weight / _rot.
 *   qc_quant_act_asym    stand-alone quantizer: qx uint8 [M, K] row major, x_scale float [M],
 *                        x_zero float [M] (integer valued; a float because a row far from zero
 *                        with a narrow range has a zero point beyond int32).
 *   qc_qlinear_asym      quantize + GEMM + epilogue.  workspace >=
 *                        qc_qlinear_asym_workspace_bytes(M, K, N) bytes.  With QC_OUT_I32_ACC, Y
 *                        is sum_k (q[m, k] - h) qw[n, k], the sum the MFMA loop forms on the
 *                        stored bytes.
 *   qc_qlinear_asym_quant, qc_qlinear_asym_gemm   the two halves of qc_qlinear_asym as calls
 *                        of their own, as qc_qlinear_quant / qc_qlinear_gemm are of qc_qlinear.
 *   qc_debug_workspace_act_asym   test hook: the codes, scales and zero points
 *                        qc_qlinear_asym left in its workspace, in canonical form.
 * act_bits 8, 6 or 4.  K must be a multiple of 16 and at most 9216 (UNSUPPORTED otherwise).
 * Other arguments and errors as for qc_qlinear. */
size_t qc_qlinear_asym_workspace_bytes(int64_t M, int64_t K, int64_t N);
qc_status qc_weight_row_sums(const void *packed, int64_t N, int64_t K, int bits,
                             int32_t *w_row_sums, void *stream);
qc_status qc_quant_act_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                            uint8_t *qx, float *x_scale, float *x_zero, void *stream);
qc_status qc_qlinear_asym(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                          const void *packed, const float *w_scale, const int32_t *w_row_sums,
                          int bits, int64_t N, const float *bias, qc_epilogue epi, void *Y,
                          qc_out ydt, void *workspace, size_t workspace_bytes, void *stream);
qc_status qc_qlinear_asym_quant(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                                void *workspace, size_t workspace_bytes, void *stream);
qc_status qc_qlinear_asym_gemm(const void *workspace, size_t workspace_bytes, int64_t M, int64_t K,
                               const void *packed, const float *w_scale,
                               const int32_t *w_row_sums, int bits, int64_t N, const float *bias,
                               qc_epilogue epi, void *Y, qc_out ydt, void *stream);
qc_status qc_debug_workspace_act_asym(const void *workspace, int64_t M, int64_t K, int act_bits,
                                      uint8_t *qx, float *x_scale, float *x_zero, void *stream);

/* ---- one activation scale per layer input ----------------------------------------------------
 * Section 4.1 "Quantization Scheme" speaks of dynamic per-layer activation quantization with
 * parameters computed online.  The calls above take the finer reading (one scale per token);
 * these take the sentence literally: ONE scale for the whole activation tensor X [M, K],
 *      s = max(max_{m,k} |X[m,k]|, 2^-64) / qmax,   q = clamp(rne(X / s), -qmax, qmax),
 * computed online by a reduction over X before the cast (X is read twice).
 *   qc_quant_act_tensor   qx int8 [M, K] row major, x_scale float [1]; workspace >=
 *                         qc_quant_act_tensor_workspace_bytes(M, K) bytes (slab maxima)
 *   qc_qlinear_tensor     quantize + GEMM + epilogue as qc_qlinear_act_bits; workspace >=
 *                         qc_qlinear_tensor_workspace_bytes(M, K, N) bytes, 256-byte aligned.  Its
 *                         first part has the layout of qc_qlinear's workspace (the scale is
 *                         repeated per token), so qc_qlinear_gemm and qc_debug_workspace_act
 *                         work on it.
 * Deterministic.  Errors as for the per-token calls. */
size_t qc_quant_act_tensor_workspace_bytes(int64_t M, int64_t K);
qc_status qc_quant_act_tensor(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                              int8_t *qx, float *x_scale, void *workspace, size_t workspace_bytes,
                              void *stream);
size_t qc_qlinear_tensor_workspace_bytes(int64_t M, int64_t K, int64_t N);
qc_status qc_qlinear_tensor(const void *X, qc_dtype xdt, int64_t M, int64_t K, int act_bits,
                            const void *packed, const float *w_scale, int bits, int64_t N,
                            const float *bias, qc_epilogue epi, void *Y, qc_out ydt,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Test hook: after qc_qlinear(.., M, K, .., workspace, ..) returned QC_OK, copy the
 * activation codes and scales it used out of the workspace in canonical order:
 * qx int8 [M, K] row major, x_scale float [M]. */
qc_status qc_debug_workspace_act(const void *workspace, int64_t M, int64_t K, int8_t *qx,
                                 float *x_scale, void *stream);

/* Test hooks for the GEMM stage, host only (no device is touched).  The GEMM (Section 4.1
 * "Hardware Implementation") exists as two kernels: one streams the weight tile of a block through
 * a ring in LDS, the other keeps a whole 128-channel weight tile resident in LDS and is taken for
 * short reductions (K <= 1152 with 8-bit weights, <= 2304 with 4-bit ones) on problems large
 * enough for its static schedule.
 *   qc_debug_gemm_kernel    which one qc_qlinear_gemm takes for (M, K, N, bits): 1 the ring,
 *                           2 the resident one, 0 if the shape is unsupported
 *   qc_debug_gemm_schedule  the rounds of block `block` (0 .. 255) of the resident kernel for an
 *                           [M, N] output, in the order the block runs them: pairs[2 i] is the
 *                           128-channel tile, pairs[2 i + 1] the 512-token chunk of round i.
 *                           Returns the number of rounds and fills at most `cap` pairs (host
 *                           memory; may be NULL with cap 0); -1 for bad arguments.  Over all
 *                           blocks every (tile, chunk) appears exactly once. */
int qc_debug_gemm_kernel(int64_t M, int64_t K, int64_t N, int bits);
int qc_debug_gemm_schedule(int64_t M, int64_t N, int block, int32_t *pairs, int cap);

/* ---- S5: latent change reduction ----------------------------------------------------
 * Section 3.2 HLC, Eq. (5): the L1 norm of the change between the current latent and
 * the cached one, with the L1 norm of the cached one to make it relative.
 *   cur, prev  device, float [n]
 *   out3       device, float [3]: { sum|cur-prev|, sum|prev|, ratio }.
 *              ratio = +inf if the second sum is 0 and the first is not, 0 if both are.
 *   workspace  device, >= qc_latent_delta_workspace_bytes(n) bytes, 256-byte aligned;
 *              contents on entry are irrelevant (per-block partial sums).  Two calls that
 *              overlap in time need two buffers.
 * The result is deterministic: the same inputs give the same bits on every run.
 * Errors: INVALID_ARG, WORKSPACE, DEVICE. */
qc_status qc_latent_delta(const float *cur, const float *prev, int64_t n, float *out3,
                          void *workspace, size_t workspace_bytes, void *stream);

/* ---- qc_latent_delta without a workspace ------------------------------------------------------
 * For callers that cannot allocate device memory or have none to hand over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same result, bit for bit, as
 * qc_latent_delta; the per-block partial sums go to a fixed array inside the library
 * (4 KiB of device memory per GPU, held until the process ends) instead of a workspace.  The
 * call allocates and frees nothing.  Its first call on a device asks the runtime for that
 * device's address of the array (no allocation, no synchronisation).
 *   n          at most QC_LATENT_DELTA_STATIC_MAX_N, else UNSUPPORTED
 * All calls on one GPU share the array: two calls that overlap in time on one GPU (different
 * streams) race and give undefined results; calls on one stream are ordered by the stream.
 * Nothing has to be cleared between calls: every partial sum the combine reads is written by
 * the same call first.  Other arguments and errors as for qc_latent_delta (no WORKSPACE). */
#define QC_LATENT_DELTA_STATIC_MAX_N ((int64_t)1 << 30)
qc_status qc_latent_delta_static(const float *cur, const float *prev, int64_t n, float *out3,
                                 void *stream);

/* ---- cosine similarity of the features of consecutive layers -----------------------------
 * Section 3.3 SRAP, Eq. (9): S = <a, b> / (||a|| ||b||), the score the layer-pruning rule of
 * Eq. (10) thresholds.
 *   a, b       device, [n] of `dt` (float or bf16)
 *   out4       device, float [4]: { <a,b>, <a,a>, <b,b>, S };  S = 0 if either norm is 0
 *   workspace  device, >= qc_layer_similarity_workspace_bytes(n) bytes, 256-byte aligned,
 *              contents irrelevant on entry
 * Deterministic like qc_latent_delta.  Errors: INVALID_ARG, WORKSPACE, DEVICE. */
size_t qc_layer_similarity_workspace_bytes(int64_t n);
qc_status qc_layer_similarity(const void *a, const void *b, qc_dtype dt, int64_t n, float *out4,
                              void *workspace, size_t workspace_bytes, void *stream);

/* ---- inter-frame gradient norm of a feature map -------------------------------------------
 * Section 3.2 HLC, Eq. (5), second factor.  The paper names this factor without defining it;
 * this library takes the forward difference along the frame axis and the Euclidean norm:
 *   g[f, j] = m[f+1, j] - m[f, j]  (f < frames-1),   out2 = { sum g^2, sqrt(sum g^2) }.
 *   m          device, [frames, inner] of `dt` (float or bf16), dense.  inner a multiple of 8
 *              takes the vectorised path; any inner >= 1 is accepted.  frames = 1 gives zeros.
 *   out2       device, float [2]
 *   workspace  device, >= qc_frame_gradient_norm_workspace_bytes(frames, inner) bytes, 256-byte
 *              aligned, contents irrelevant on entry
 * Deterministic like qc_latent_delta.  Errors: INVALID_ARG, WORKSPACE, DEVICE. */
size_t qc_frame_gradient_norm_workspace_bytes(int64_t frames, int64_t inner);
qc_status qc_frame_gradient_norm(const void *m, qc_dtype dt, int64_t frames, int64_t inner,
                                 float *out2, void *workspace, size_t workspace_bytes,
                                 void *stream);

/* ---- cumulative feature variation over the previous steps ---------------------------------
 * Section 3.3 SRAP, Eq. (11): V = sum_i ||p_t - p_{t-i}||_1 over the kept earlier steps (the
 * i = 0 term is zero and has no input here).  One pass reads `cur` once for all distances.
 *   cur        device, float [n]
 *   prevs      HOST array of `count` device pointers, each float [n]; read during the call
 *              only.  1 <= count <= QC_MAX_PREV, else UNSUPPORTED
 *   out        device, float [count + 1]: the L1 distance to each prevs[i], then V, their sum
 *              in index order
 *   workspace  device, >= qc_cumulative_variation_workspace_bytes(n, count) bytes, 256-byte
 *              aligned, contents irrelevant on entry
 * Deterministic like qc_latent_delta.  out[i] agrees with qc_latent_delta's first output for
 * (cur, prevs[i]) to binary32 rounding; identical bits are not promised (the summation order
 * differs).  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, DEVICE. */
size_t qc_cumulative_variation_workspace_bytes(int64_t n, int count);
qc_status qc_cumulative_variation(const float *cur, const float *const *prevs, int count,
                                  int64_t n, float *out, void *workspace, size_t workspace_bytes,
                                  void *stream);

/* ---- decision rules (host, pure functions) ------------------------------------------------
 * The scalar rules that turn the reductions above into the method's decisions.  All
 * arguments and results are host values; nothing touches the GPU.  A NaN argument, or
 * thresholds given in the wrong order (low > high), is an error: the integer rules then
 * return -1, the floating-point rules NaN.
 *
 * qc_divergence_score   Section 3.2 HLC, Eq. (5): D = l1_change / k * grad_norm, with
 *                       l1_change = qc_latent_delta's first output, k >= 1 the number of steps
 *                       since the cached one, grad_norm = qc_frame_gradient_norm's second.
 * qc_cache_interval     Eq. (6): tau_max if D < delta1, tau_mid if delta1 <= D < delta2,
 *                       tau_min if D >= delta2.
 * qc_activation_bits    Section 3.2 AIGQ (2), Eq. (8), the same three-way rule on the
 *                       timestep's redundancy metric: bit_max below theta1, bit_mid from theta1
 *                       up to theta2, bit_min from theta2 on.
 * qc_prune_probability  Section 3.3 SRAP, Eq. (10): 1 if S > tau_high, 0 if S < tau_low,
 *                       p_base on the closed interval between. */
float qc_divergence_score(float l1_change, int k, float grad_norm);
int qc_cache_interval(float D, float delta1, float delta2, int tau_max, int tau_mid, int tau_min);
int qc_activation_bits(float D, float theta1, float theta2, int bit_max, int bit_mid, int bit_min);
float qc_prune_probability(float S, float tau_low, float tau_high, float p_base);

#ifdef __cplusplus
}
#endif
#endif /* QC_H */
