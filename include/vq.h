/*
 * vq.h - C ABI of the MI355X (gfx950) quantized linear layer of ViDiT-Q
 * (arxiv 2406.02540).
 *
 * The layer: dynamic per-token symmetric int8 quantization of the activations
 * with the per-input-channel balancing factor folded in, an int8 x int8 -> int32
 * contraction along the input channels against per-output-channel int8 (W8A8)
 * or 4-bit (W4A8) weights, and a dequantization epilogue that multiplies the
 * integer sum by the token's scale and the output channel's scale, adds the
 * bias and writes fp16.
 *
 * Conventions for every entry point
 *   - Every pointer is a DEVICE pointer (HIP global memory) unless it says
 *     "host".  The library never allocates, frees or keeps a pointer: the caller
 *     owns every buffer.  Outputs must not overlap inputs.
 *   - Matrices are dense row-major: X[M,K], W[N,K] (the K input channels are
 *     contiguous), Y[M,N].  fp16 data is IEEE binary16.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  A call validates its arguments on the host, enqueues its
 *     kernels on that stream and returns without synchronising; outputs are
 *     valid once the stream has reached that point.
 *   - Return value: VQ_OK (0) or a vq_status error.  On any error nothing was
 *     enqueued and no output byte was written.  M == 0 or N == 0 is not an
 *     error: nothing is enqueued and VQ_OK is returned.
 *   - Not checked on the device: X and chan_mul finite, chan_mul > 0 and within
 *     [2^-20, 2^20]; 4-bit weights in [-7, 7].  Violations give unspecified
 *     values in the outputs, never a fault.
 *   - Limits: K <= VQ_MAX_K so that |sum| <= K * 127 * 127 fits int32 (also with
 *     the 4-bit path, which accumulates 16 * w internally).
 */
#ifndef VQ_H_
#define VQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum vq_status {
    VQ_OK = 0,
    VQ_ERR_NULL = 1,      /* a required pointer is NULL                               */
    VQ_ERR_SHAPE = 2,     /* negative size, K == 0, K too large, or K not a multiple
                             of what the entry point requires                         */
    VQ_ERR_ALIGN = 3,     /* a base pointer is not 16-byte aligned                    */
    VQ_ERR_WORKSPACE = 4, /* workspace smaller than vq_linear_workspace_bytes(), or that
                             size beyond VQ_LINEAR_STATIC_SCRATCH_BYTES (vq_linear_static) */
    VQ_ERR_LAUNCH = 5,    /* the HIP runtime refused the launch                       */
    VQ_ERR_ARCH = 6,      /* the current device is not gfx950 (or there is no device) */
    VQ_ERR_BITS = 7       /* w_bits is neither 8 nor 4                                */
} vq_status;

#define VQ_MAX_K 131072
#define VQ_MAX_FUSED_K 8192 /* the fused quantizers keep a token in registers */
#define VQ_HADAMARD_BLOCK 128 /* block size of the rotation */

/*
 * Dynamic per-token activation quantizer (Sec. 4.1 "Fine-grained Grouping and
 * Dynamic Quantization"; quantizer of Sec. 3.1 Eq. 2 in its symmetric form; the
 * activation half of the channel balancing of Sec. 4.2 Eq. 3).
 *
 * For every token m:  t[k] = float(x[m,k]) * chan_mul[k];  amax = max_k |t[k]|;
 * x_scale[m] = amax / 127;  xq[m,k] = clamp(rne(t[k] * (127 / amax)), -127, 127),
 * all in fp32, one reciprocal per token, halves rounded to even.  A token of
 * zeros gives x_scale = 0 and xq = 0.
 *
 *   x_f16    in  fp16 [M,K]
 *   chan_mul in  fp32 [K], the reciprocal 1/s_k of the balancing mask, or NULL
 *                for no balancing (same as all ones)
 *   xq       out int8 [M,K]
 *   x_scale  out fp32 [M]
 * Any K >= 1 is accepted; rows are processed fastest when K is a multiple of 8.
 */
int vq_quantize_per_token(const void* x_f16, const float* chan_mul, int8_t* xq, float* x_scale,
                          int M, int K, void* hip_stream);

/*
 * The same quantizer fused behind the operation that produces its input (Sec. 5.1
 * "Hardware Implementation Settings": the quantization is integrated into the
 * preceding LayerNorm, GELU and residual operations; Sec. 4.1: the dynamic
 * parameters only need the extrema of the token and can be fused with the previous
 * operation).  The producer's fp32 result t[m,k] takes the place of float(x[m,k]) in
 * vq_quantize_per_token and is never written to memory.  The paper gives no formulas
 * for the producers; the textbook ones are used.  All three need K % 8 == 0 and
 * K <= VQ_MAX_FUSED_K (VQ_ERR_SHAPE otherwise) and 16-byte aligned pointers.
 * "Sample" b of token m is m / tokens_per_sample (the images or videos of a batch,
 * e.g. the two halves of a classifier-free-guidance pair); per-sample arrays are fp32
 * [ceil(M / tokens_per_sample), K].  chan_mul, xq, x_scale, M, K, hip_stream: as above.
 *
 * vq_gelu_quantize:       t = GELU(float(h[m,k])) = x Phi(x); approximate = 0 evaluates
 *                         Phi with erf, 1 uses the tanh form
 *                         Phi(x) ~ (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) / 2.
 * vq_layernorm_quantize:  y = (x - mean) / sqrt(var + eps) over the K channels of the
 *                         token (biased variance, no learned affine), then the feature
 *                         modulation t = (1 + mod_scale[b,k]) y + mod_shift[b,k]; either
 *                         array may be NULL (no scaling / no shift).
 * vq_residual_quantize:   r = x + gate[b,k] * y (gate NULL = 1), product and sum each
 *                         rounded in fp32; r is written to r_f16 [M,K] as fp16 (the new
 *                         residual stream) and t = float(r_f16[m,k]).
 * The integer outputs of vq_residual_quantize are fully determined by this; those of the
 * other two depend on the fp32 evaluation order of the reductions and on the device's
 * exp / erf, within a few fp32 ulps of the exact t.
 */
int vq_gelu_quantize(const void* h_f16, int approximate, const float* chan_mul, int8_t* xq,
                     float* x_scale, int M, int K, void* hip_stream);
int vq_layernorm_quantize(const void* x_f16, const float* mod_scale, const float* mod_shift,
                          int tokens_per_sample, float eps, const float* chan_mul, int8_t* xq,
                          float* x_scale, int M, int K, void* hip_stream);
int vq_residual_quantize(const void* x_f16, const void* y_f16, const float* gate, int tokens_per_sample,
                         void* r_f16, const float* chan_mul, int8_t* xq, float* x_scale, int M, int K,
                         void* hip_stream);

/*
 * Offline calibration of the scaling mask of Sec. 4.2, Eq. 3:
 *     s_i = max|X_i|^alpha / max|W_i|^(1 - alpha)     for every input channel i.
 *
 * vq_channel_absmax: amax[k] = max over the R rows of |a[r,k]| for a dense [R,K] matrix of
 *                    fp16 (is_f32 = 0: activations of a calibration batch) or fp32
 *                    (is_f32 = 1: a weight [N,K]).  accumulate = 0 overwrites amax [K];
 *                    accumulate != 0 combines with the non-negative values already there
 *                    (the running maximum over several batches or denoising steps).
 * vq_balance_mask:   s [K] from the two statistics and alpha in [0,1], and chan_mul = 1/s [K],
 *                    the factor the quantizers take.  Statistics below 1e-5 count as 1e-5 and
 *                    s is kept within [1e-5, 1e5] (an all-zero channel must not give 0 or inf).
 *                    The weight side multiplies W[n,k] by s[k] (vq_quantize_weight, chan_s).
 */
int vq_channel_absmax(const void* a, int is_f32, float* amax, int R, int K, int accumulate, void* hip_stream);
int vq_balance_mask(const float* amax_x, const float* amax_w, float alpha, float* s, float* chan_mul, int K,
                    void* hip_stream);

/*
 * Rotation-based channel balancing, the "dynamic" half of the static-dynamic balancing of
 * Sec. 4.2 (Y = X W^T = (X Q)(W Q)^T for an orthogonal Q; the scaling of Eq. 3 comes first),
 * with the Hadamard transform fused into the quantizer as in Sec. 5.1.  Q is block diagonal
 * with blocks H_128 / sqrt(128), H_128 the Sylvester Hadamard matrix in natural order
 * (H[k][c] = (-1)^popcount(k & c)); the paper does not say how channel counts that are not a
 * power of two (1152, 4608) are rotated, blocks of 128 are this library's reading.
 *
 * vq_hadamard_quantize: t[m,:] = (float(x[m,:]) * chan_mul) Q, then the per-token quantizer
 *                       of vq_quantize_per_token on t.  K % 128 == 0, K <= VQ_MAX_FUSED_K.
 *                       fp32 butterflies: as for the fused LayerNorm and GELU the codes are
 *                       determined up to the rounding of t (a few fp32 ulps).
 * vq_rotate_weight:     the weight side, offline: w_rot[n,:] = (w[n,:] * chan_s) Q in fp32, to
 *                       be quantized with vq_quantize_weight (chan_s = NULL there).  w_f32 and
 *                       w_rot_f32 are fp32 [N,K] and may be the same buffer.
 */
int vq_hadamard_quantize(const void* x_f16, const float* chan_mul, int8_t* xq, float* x_scale, int M, int K,
                         void* hip_stream);
int vq_rotate_weight(const float* w_f32, const float* chan_s, float* w_rot_f32, int N, int K, void* hip_stream);

/*
 * The two comparison points of the paper's hardware evaluation (Sec. 5.3 "Hardware
 * Resource Savings": the INT8 layers against FP16 layers, and against a "naive" W8A8
 * baseline without dynamic token-wise parameters), on the same device and with the same
 * tiling as vq_gemm_w8a8.  They are measured next to the quantized layer, not part of it.
 *
 * vq_gemm_f16:        y[m,n] = fp16(sum_k x[m,k] * w[n,k] + bias[n]), fp16 operands,
 *                     products exact, sums in fp32 (matrix-core order), the bias added to
 *                     the fp32 sum exactly and the result rounded once.  x_f16 [M,K],
 *                     w_f16 [N,K], bias_f16 [N] or NULL, y_f16 [M,N]; K % 8 == 0.
 * vq_quantize_static: xq[m,k] = clamp(rne(float(x[m,k]) * chan_mul[k] * (1 / scale)),
 *                     -127, 127) with one `scale` (host value, > 0) for the whole tensor
 *                     and one fp32 reciprocal; values beyond 127 * scale are clipped.
 *                     The caller passes the same scale for every token to vq_gemm_w8a8.
 */
int vq_gemm_f16(const void* x_f16, const void* w_f16, const void* bias_f16, void* y_f16, int M, int N, int K,
                void* hip_stream);
int vq_quantize_static(const void* x_f16, const float* chan_mul, float scale, int8_t* xq, int M, int K,
                       void* hip_stream);

/*
 * W8A8 integer GEMM with the dequantization epilogue (appendix "Hardware
 * implementation of quantized linear layers": the integer products are summed
 * along the input channels, the token-wise and output-channel-wise scales
 * multiply the sum afterwards; Sec. 5.3 "Hardware Resource Savings").
 *
 *   acc[m,n] = sum_k xq[m,k] * wq[n,k]                       (exact, int32)
 *   y[m,n]   = fp16(float(acc[m,n]) * x_scale[m] * w_scale[n] + float(bias[n]))
 * evaluated as: s = x_scale[m] * w_scale[n] rounded to fp32, then float(acc) * s + bias
 * exactly, rounded once (to nearest even) to fp16; whichever kernel the library picks.
 *
 *   xq       in  int8 [M,K]          x_scale in fp32 [M]
 *   wq       in  int8 [N,K]          w_scale in fp32 [N]
 *   bias_f16 in  fp16 [N] or NULL (no bias)
 *   y_f16    out fp16 [M,N]
 *   acc_out  out int32 [M,N] or NULL: a copy of the integer sums, for checking
 * Requires K % 16 == 0.  Any M, N >= 1; N % 8 == 0 takes the vectorised store path.
 */
int vq_gemm_w8a8(const int8_t* xq, const float* x_scale, const int8_t* wq, const float* w_scale,
                 const void* bias_f16, void* y_f16, int32_t* acc_out,
                 int M, int N, int K, void* hip_stream);

/*
 * W4A8: the same contraction and epilogue with 4-bit weights that are widened
 * to 8 bits on chip before the int8 product (appendix "Performance of ViDiT-Q
 * under lower bitwidth": 4-bit storage, 8-bit compute).
 *
 *   wq4  in uint8 [N,K/2]: byte j of row n holds w[n,2j] in bits 0..3 and
 *        w[n,2j+1] in bits 4..7, two's-complement nibbles in [-7,7].
 * Requires K % 32 == 0.  Other arguments as vq_gemm_w8a8; acc_out holds the sums
 * of the widened weights, i.e. the same integers as the W8A8 routine would give.
 */
int vq_gemm_w4a8(const int8_t* xq, const float* x_scale, const uint8_t* wq4, const float* w_scale,
                 const void* bias_f16, void* y_f16, int32_t* acc_out,
                 int M, int N, int K, void* hip_stream);

/*
 * The whole quantized linear layer as the paper deploys it, a composition of the calls
 * above: the dynamic token-wise quantizer with the balancing factor (Sec. 4.1; Sec. 4.2
 * Eq. 3) into the workspace, then the integer GEMM with its dequantization (appendix
 * "Hardware implementation of quantized linear layers") that w_bits selects (8: w is
 * int8 [N,K]; 4: w is uint8 [N,K/2] packed as above, appendix "Performance of ViDiT-Q
 * under lower bitwidth").
 *
 *   workspace  device scratch of at least vq_linear_workspace_bytes(M,N,K,w_bits)
 *              bytes, 16-byte aligned; holds xq and x_scale between the two
 *              kernels; contents are unspecified afterwards.
 */
int vq_linear(const void* x_f16, const float* chan_mul, const void* w, int w_bits,
              const float* w_scale, const void* bias_f16, void* y_f16,
              void* workspace, size_t workspace_bytes, int M, int N, int K, void* hip_stream);

/* Bytes of workspace vq_linear needs (0 if a size is invalid): the int8 activations and
 * the token scales the quantizer of Sec. 4.1 hands to the GEMM.  Host-only, no HIP call. */
size_t vq_linear_workspace_bytes(int M, int N, int K, int w_bits);

/*
 * The layer behind one of the producers (Sec. 5.1 "Hardware Implementation Settings": the
 * quantizer is merged into the LayerNorm, GELU or residual operation that precedes the linear
 * layer; Sec. 4.2 for the rotation): the fused quantizer of the same name into the workspace,
 * then the GEMM that w_bits selects.  The producer's arguments are those of
 * vq_layernorm_quantize / vq_gelu_quantize / vq_residual_quantize / vq_hadamard_quantize, the
 * rest those of vq_linear (same workspace size), and the results are bit for bit those of the
 * two separate calls.  K as the fused quantizers need it (K % 8 == 0, K <= VQ_MAX_FUSED_K,
 * K % 128 == 0 for the rotation) and as the GEMM needs it (K % 16, K % 32 for 4-bit weights).
 * vq_residual_linear also writes the new residual stream r_f16 [M,K].  For
 * vq_hadamard_linear the weights must have been rotated (vq_rotate_weight) before they
 * were quantized.
 */
int vq_layernorm_linear(const void* x_f16, const float* mod_scale, const float* mod_shift,
                        int tokens_per_sample, float eps, const float* chan_mul, const void* w, int w_bits,
                        const float* w_scale, const void* bias_f16, void* y_f16,
                        void* workspace, size_t workspace_bytes, int M, int N, int K, void* hip_stream);
int vq_gelu_linear(const void* h_f16, int approximate, const float* chan_mul, const void* w, int w_bits,
                   const float* w_scale, const void* bias_f16, void* y_f16,
                   void* workspace, size_t workspace_bytes, int M, int N, int K, void* hip_stream);
int vq_residual_linear(const void* x_f16, const void* y_in_f16, const float* gate, int tokens_per_sample,
                       void* r_f16, const float* chan_mul, const void* w, int w_bits, const float* w_scale,
                       const void* bias_f16, void* y_f16,
                       void* workspace, size_t workspace_bytes, int M, int N, int K, void* hip_stream);
int vq_hadamard_linear(const void* x_f16, const float* chan_mul, const void* w, int w_bits,
                       const float* w_scale, const void* bias_f16, void* y_f16,
                       void* workspace, size_t workspace_bytes, int M, int N, int K, void* hip_stream);

/*
 * vq_linear without a workspace argument, for callers that cannot allocate device memory
 * around the call (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc).  The int8 activations and token scales live in a scratch array built into the
 * library, VQ_LINEAR_STATIC_SCRATCH_BYTES per device, held until the process ends; the call
 * itself allocates and frees nothing.  Same kernels, same results as vq_linear.
 *
 *   - VQ_ERR_WORKSPACE if vq_linear_workspace_bytes(M,N,K,w_bits) exceeds
 *     VQ_LINEAR_STATIC_SCRATCH_BYTES (e.g. 32768 x 1152 and 8192 x 4608 activations fit,
 *     32768 x 4608 do not); VQ_ERR_LAUNCH if the scratch array cannot be located.
 *   - Every call on a device uses that device's one array: calls that may overlap in time
 *     on one device (different streams, different threads) race on it and must be ordered
 *     by the caller.  Nothing in the array has to start at zero; it keeps the last call's
 *     contents.
 *   - The first call on a device looks the array's address up (once per device); make that
 *     call outside any stream capture.
 */
#define VQ_LINEAR_STATIC_SCRATCH_BYTES (40u << 20)
int vq_linear_static(const void* x_f16, const float* chan_mul, const void* w, int w_bits,
                     const float* w_scale, const void* bias_f16, void* y_f16,
                     int M, int N, int K, void* hip_stream);

/*
 * Offline side: per-output-channel symmetric weight quantizer (Sec. 4.1: one
 * parameter set per output channel; Sec. 4.2 Eq. 3: the weight half of the
 * channel balancing, W[n,k] * s_k, applied before quantization).
 *
 *   w_f32   in  fp32 [N,K]
 *   chan_s  in  fp32 [K] balancing mask s, or NULL
 *   w_bits  8: wq_out is int8 [N,K] in [-127,127]
 *           4: wq_out is uint8 [N,K/2], nibbles in [-7,7] packed as for
 *              vq_gemm_w4a8 (K must be even)
 *   w_scale out fp32 [N] = max_k |w[n,k] * s_k| / (127 or 7)
 */
int vq_quantize_weight(const float* w_f32, const float* chan_s, int w_bits, void* wq_out,
                       float* w_scale, int N, int K, void* hip_stream);

/* Static, host-side description of a vq_status value (no passage of the paper: the error
 * reporting of this boundary). */
const char* vq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* VQ_H_ */
