/*
 * dirotq.h -- C ABI of the MI355X (gfx950) implementation of the rotation-aware
 * W4A4 linear layer of DiRotQ ("PCA-guided rotated quantization", Section 4.2 of
 * the paper; forward-computation equation at the end of that section).
 *
 * The layer replaces  y = W x  (W in R^{N x K}) by
 *
 *     x_hat = x Q                                   online rotation into the PCA basis
 *     x_h   = bf16(x_hat[:, 0:r])                   top-r coefficients, kept in 16 bit
 *     x_l   = int4(x_hat[:, r:K]) with fp16 scales  per token, per group of g channels
 *     y     = x_h W'_h^T + sum_j s_x[:,j] s_w[:,j]^T * (q_x,j q_w,j^T)
 *
 * where W' = W Q is fused, split at r and quantized offline.  Names: M tokens,
 * K input channels, N output channels, r = rank of the 16-bit subspace (the
 * paper's k), g = group size, G = (K - r) / g.  The paper writes Y = X W with
 * W in R^{m x n}; this header uses the nn.Linear convention, W' = (V^T W_paper)^T.
 *
 * The quantizer is the symmetric form of the paper's quantizer equation
 * (Section 3): s = max|v| / 7 over a group, stored as IEEE fp16; code =
 * clip(round-half-even(v / s), -7, 7).  In detail, in IEEE fp32:
 * amax = max|v|; s = fp16_rne(min(amax / 7, 65504)); s == 0 -> all codes 0; else
 * inv = 1 / float(s), code = clip(rint(v * inv), -7, 7).
 *
 * Where this header departs from the plainest reading of the paper's problem statement
 * (all of it layout, none of it arithmetic):
 *  - the online rotation operand is Qt = bf16(Q^T), one basis direction per row, made
 *    once per layer by dirotq_prepare_rotation (both GEMM operands then stream
 *    K-contiguous rows); Q itself is only an argument of the offline calls;
 *  - activation scales (and zero-points) are group-major, [G][M], not [M][G];
 *  - an activation nibble is sign-magnitude (bit 3 sign, bits 0-2 |q|), not two's
 *    complement: that form expands to the fp8 operand of the matrix pipe in two
 *    bit operations; the weight blob is private (dirotq_export_weights gives the
 *    canonical int8 codes back);
 *  - K and r must be multiples of 32 (one 16-byte chunk of packed codes);
 *  - dirotq_linear takes its intermediates in a caller-supplied workspace
 *    (dirotq_linear_static keeps them in the library's own fixed array instead).
 *
 * General conventions
 *  - Every pointer is a DEVICE pointer unless marked "host".  The caller owns all
 *    memory; the library never allocates or frees device memory.
 *  - All matrices are dense row-major.  Device pointers must be 16-byte aligned.
 *  - 16-bit floats are passed as uint16_t bit patterns (bfloat16 or IEEE half).
 *  - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = the
 *    default stream) and return without synchronizing.
 *  - Return value: DIROTQ_OK or a negative dirotq_status.  Argument errors are
 *    detected on the host before anything is enqueued; nothing is written then.
 *  - Supported shapes: M >= 0 (M == 0 is a no-op), N >= 1, K a multiple of 32,
 *    0 <= r <= K with r a multiple of 32, g in {32, 64, 128}, (K - r) % g == 0.
 *    Upper limits: M, N <= 2^24, K <= 2^20, ceil(M/128) * ceil(N/128) <= 2^30; element
 *    offsets are 64-bit, so M*K, M*N and N*K may exceed 2^31.
 *  - INT4 packing (activations): byte i of a row holds channel 2i of the 4-bit part
 *    in bits 0-3 and channel 2i+1 in bits 4-7.  A nibble is the code q in [-7, 7] in
 *    sign-magnitude form: bit 3 = sign, bits 0-2 = |q|; zero is always 0x0.
 *  - Activation scales are group-major: s_x[j * M + m] for group j, token m.
 *  - The GEMM calls pick one of several schedules of the same arithmetic from the problem
 *    size (few tokens: K split over the waves of a workgroup; medium: 128 x 128 tiles;
 *    large: persistent wave-specialised workgroups; asymmetric layers use the last two).  The fp32 additions of an output are
 *    ordered differently in each, so a token's result is deterministic for a given
 *    (M, N, K, r, g) but not bit-identical across different M.  For testing, the
 *    environment variables DIROTQ_W4A4_KERNEL (ws | tile | skinny) and
 *    DIROTQ_W4A16_KERNEL (tile) are read at every launch and force a schedule wherever
 *    it applies; they are not needed in normal use.
 */
#ifndef DIROTQ_H
#define DIROTQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DIROTQ_OK = 0,
  DIROTQ_ERR_NULL = -1,        /* a required pointer is NULL */
  DIROTQ_ERR_SHAPE = -2,       /* M<0, N<1, K<32, K%32, r<0, r>K, r%32, g not in {32,64,128}, (K-r)%g, too large */
  DIROTQ_ERR_ALIGN = -3,       /* a device pointer is not 16-byte aligned */
  DIROTQ_ERR_WORKSPACE = -4,   /* workspace / scratch / blob buffer too small */
  DIROTQ_ERR_UNSUPPORTED = -5, /* valid request this build does not implement */
  DIROTQ_ERR_HIP = -6,         /* a HIP call failed; see dirotq_last_hip_error() */
  DIROTQ_ERR_STATIC_LIMIT = -7 /* dirotq_linear_static: intermediates exceed its fixed scratch */
} dirotq_status;

/* Static description of a status code (never freed; host). */
const char* dirotq_strerror(int status);

/* hipError_t (as int) of the last DIROTQ_ERR_HIP on this host thread, else 0. */
int dirotq_last_hip_error(void);

/* ---- size queries (host, pure) ------------------------------------------------ */

/* Bytes of the prepared-weight blob for an N x K layer split at r with groups of g. */
int dirotq_weights_bytes(int N, int K, int r, int g, size_t* bytes /*host out*/);

/* Bytes of scratch dirotq_prepare_weights needs (the fp32 fused weight W Q). */
int dirotq_prepare_scratch_bytes(int N, int K, size_t* bytes /*host out*/);

/* Bytes of workspace dirotq_linear needs (x_h, packed x_l and s_x of one call). */
int dirotq_workspace_bytes(int M, int K, int r, int g, size_t* bytes /*host out*/);

/* ---- offline ------------------------------------------------------------------- */

/*
 * Rotation operand for the online kernel: Qt[c * K + k] = bf16_rne(Q[k * K + c]).
 * Q is the orthogonal basis V = [U_h, U_l R] of Section 4.2, fp32 [K,K], column c =
 * c-th basis direction (eigenvalues descending).  Qt is bf16 [K,K], one basis
 * direction per row, which is the layout the rotation GEMM streams.
 */
int dirotq_prepare_rotation(const float* Q, int K, uint16_t* Qt_bf16 /*out*/, void* stream);

/*
 * Offline weight fusion (the step of Section 4.2 that folds the transposed rotation into
 * the weights, just before the forward-computation equation):
 * W' = W Q with fp64 accumulation rounded to fp32; W'_h = bf16_rne(W'[:, 0:r]);
 * W'[:, r:K] quantized per output channel and per group of g with the quantizer
 * above (round-to-nearest stands in for GPTQ).  W fp32 [N,K], Q fp32 [K,K] as in
 * dirotq_prepare_rotation.  `blob` receives dirotq_weights_bytes bytes in a layout
 * private to this library (read it back with dirotq_export_weights).  `scratch`:
 * dirotq_prepare_scratch_bytes bytes, contents undefined afterwards.  Shapes with more than
 * 2^31 - 1 tiles of 64 x 64 in W (N K > 2^43) return DIROTQ_ERR_SHAPE.
 */
int dirotq_prepare_weights(const float* W, const float* Q, int N, int K, int r, int g,
                           void* blob /*out*/, void* scratch, size_t scratch_bytes, void* stream);

/*
 * Build a blob from already-quantized weights: Wh bf16 [N,r], codes int8 [N,K-r]
 * with values in [-7,7] (anything outside is clamped to that range: -8 is not a code of
 * the symmetric quantizer), sw fp16 [N,G] (channel-major).  Wh may be NULL when r == 0,
 * codes and sw may be NULL when r == K.
 */
int dirotq_import_weights(const uint16_t* Wh_bf16, const int8_t* codes, const uint16_t* sw_fp16,
                          int N, int K, int r, int g, void* blob /*out*/, void* stream);

/* Inverse of dirotq_import_weights (outputs may be NULL to skip them). */
int dirotq_export_weights(const void* blob, int N, int K, int r, int g,
                          uint16_t* Wh_bf16 /*out [N,r]*/, int8_t* codes /*out [N,K-r]*/,
                          uint16_t* sw_fp16 /*out [N,G]*/, void* stream);

/* ---- online -------------------------------------------------------------------- */

/*
 * Rotation, split and activation quantization (rotation/split equation of Section
 * 4.2 and the quantizer of Section 3) in one kernel: x_hat = x Q accumulated in fp32
 * from bf16 operands; channels [0,r) are rounded to bf16, channels [r,K) are
 * quantized per token and per group from the fp32 accumulator.
 *   x_bf16   [M,K]          activations
 *   Qt_bf16  [K,K]          from dirotq_prepare_rotation
 *   xh_bf16  [M,r]    out   (may be NULL when r == 0)
 *   xl_packed[M,(K-r)/2] out  packed INT4 codes (may be NULL when r == K)
 *   sx_fp16  [G,M]    out   group-major scales (may be NULL when r == K)
 */
int dirotq_rotate_quantize(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int M, int K, int r, int g,
                           uint16_t* xh_bf16, uint8_t* xl_packed, uint16_t* sx_fp16, void* stream);

/*
 * Mixed-precision product (forward-computation equation of Section 4.2):
 *   y[m,n] = sum_{k<r} xh[m,k] W'_h[n,k]
 *          + sum_j float(sx[j,m]) float(sw[n,j]) * I[m,n,j]  (+ bias[n])
 * with I[m,n,j] the exact integer dot product of the INT4 codes of group j,
 * everything accumulated in fp32.  Inputs as produced by dirotq_rotate_quantize and
 * dirotq_prepare_weights / dirotq_import_weights.  bias_bf16 [N] may be NULL.
 * y_dtype 0: y is bf16 [M,N] (round to nearest even); 1: y is fp32 [M,N].
 */
int dirotq_w4a4_gemm(const uint16_t* xh_bf16, const uint8_t* xl_packed, const uint16_t* sx_fp16,
                     const void* blob, const uint16_t* bias_bf16, int M, int N, int K, int r, int g,
                     void* y /*out*/, int y_dtype, void* stream);

/*
 * The fused layer: dirotq_rotate_quantize into `workspace`, then dirotq_w4a4_gemm,
 * both on `stream`.  y_bf16 [M,N].  workspace: dirotq_workspace_bytes bytes, 256-byte
 * aligned; its contents afterwards are the intermediates of this call.
 */
int dirotq_linear(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob,
                  const uint16_t* bias_bf16, int M, int N, int K, int r, int g,
                  uint16_t* y_bf16 /*out*/, void* workspace, size_t workspace_bytes, void* stream);

/*
 * dirotq_linear for callers that cannot allocate or pass device memory for intermediates
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same two kernels, with x_h, packed x_l and s_x kept in a fixed 64 MiB array in device
 * memory that belongs to the library (one copy per GPU, held until the process ends).  The
 * call allocates and frees nothing.  DIROTQ_STATIC_SCRATCH_BYTES bounds what
 * dirotq_workspace_bytes(M, K, r, g) may return (FLUX-shaped fc2, M = 4608, K = 12288:
 * 31.2 MiB); a larger request returns DIROTQ_ERR_STATIC_LIMIT and enqueues nothing.  All
 * calls on one GPU share the array: calls that may overlap in time (different streams,
 * different host threads) race on it, and so does a dirotq_linear_static still running when
 * another is enqueued on another stream.  Results are bit-identical to dirotq_linear.
 */
#define DIROTQ_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int dirotq_linear_static(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob,
                         const uint16_t* bias_bf16, int M, int N, int K, int r, int g,
                         uint16_t* y_bf16 /*out*/, void* stream);

/*
 * Several layers that read the same activations (fused QKV next to the MLP's first
 * projection in a block whose branches share their input, Section 5.1's FLUX blocks):
 * one dirotq_rotate_quantize into `workspace`, then one dirotq_w4a4_gemm per output.
 * All outputs share K, r, g and the rotation; output i has N = Ns[i], weights blobs[i],
 * bias biases[i] (the array or any entry may be NULL) and result ys[i] bf16 [M, Ns[i]].
 * blobs, biases, Ns, ys are HOST arrays of n_out entries (1 <= n_out <= 16) holding
 * device pointers.  Results are bit-identical to n_out dirotq_linear calls.
 */
int dirotq_linear_shared(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int n_out,
                         const void* const* blobs /*host*/, const uint16_t* const* biases /*host*/,
                         const int* Ns /*host*/, uint16_t* const* ys /*host, out*/, int M, int K, int r,
                         int g, void* workspace, size_t workspace_bytes, void* stream);

/* ---- online, asymmetric activations ------------------------------------------- */
/*
 * The same three calls with the asymmetric form of the Section 3 quantizer for the
 * activations (the form the paper's experiments use for them; weights stay
 * symmetric): per token and group z = min, s = (max - min) / 15, code =
 * clip(round-half-even((v - z) / s), 0, 15).  In IEEE fp32: z16 = fp16_rne(clamp(min,
 * +-65504)), s32 = (max - min) / 15, s16 = fp16_rne(min(s32, 65504)), inv = 1 / float(s16)
 * (0 when s16 == 0), code = clip(rint((v - float(z16)) * inv), 0, 15).
 * The dequantized activation is code * s + z, so the product gains the zero-point term
 *   y[m,n] += sum_j float(zx[j,m]) * float(sw[n,j]) * sum_{k in group j} q_w[n,k];
 * the per-group sums of the weight codes are part of every prepared blob.
 *   xl_packed[M,(K-r)/2]  two unsigned nibbles per byte, even channel in bits 0-3
 *   sx_fp16, zx_fp16 [G,M]  group-major scales and zero-points
 * Pointer, shape and error rules are those of the symmetric calls.
 */
int dirotq_rotate_quantize_asym(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int M, int K, int r, int g,
                                uint16_t* xh_bf16, uint8_t* xl_packed, uint16_t* sx_fp16,
                                uint16_t* zx_fp16, void* stream);

int dirotq_w4a4_gemm_asym(const uint16_t* xh_bf16, const uint8_t* xl_packed, const uint16_t* sx_fp16,
                          const uint16_t* zx_fp16, const void* blob, const uint16_t* bias_bf16, int M, int N,
                          int K, int r, int g, void* y /*out*/, int y_dtype, void* stream);

/* workspace: dirotq_workspace_bytes bytes (it has room for the zero-points). */
int dirotq_linear_asym(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob,
                       const uint16_t* bias_bf16, int M, int N, int K, int r, int g,
                       uint16_t* y_bf16 /*out*/, void* workspace, size_t workspace_bytes, void* stream);

/* ---- online, 8-bit per-token activations (W4A8) --------------------------------- */
/*
 * The paper's 8-bit activation setting (implementation details of Section 5: per-token
 * dynamic activation quantization) on top of the same 4-bit per-group weights: channels
 * [r, K) of x Q get one symmetric INT8 scale per token,
 *   s32 = max|v| / 127, s16 = fp16_rne(min(s32, 65504)), inv = 1 / float(s16) (0 when
 *   s16 == 0), code = clip(rint(v * inv), -127, 127), all IEEE fp32,
 * and   y[m,n] = sum_{k<r} xh[m,k] Wh[n,k]
 *              + float(sx[m]) * sum_j float(sw[n,j]) * I[m,n,j]  (+ bias[n]),
 * I the exact integer dot product of the INT8 and INT4 codes of weight group j
 * (per-channel weight scales are the case of equal group scales, via
 * dirotq_import_weights).
 *   x8[M,K-r]   one sign-magnitude byte per channel (bit 7 sign, bits 0-6 magnitude; zero is
 *               0x00).  Within each block of 32 channels the 16 even channels come first,
 *               then the 16 odd ones: channel c of the block sits at byte (c & 1) * 16 + c / 2.
 *   sx_fp16[M]  one scale per token
 * scratch: dirotq_a8_scratch_bytes bytes of device memory, 256-byte aligned (the fp32
 * rotated channels before the token's maximum is known); contents undefined afterwards.
 * Shape rules as above (g only constrains K - r here).  Pointer and error rules as above.
 */
int dirotq_a8_scratch_bytes(int M, int K, int r, size_t* bytes /*host out*/);

int dirotq_rotate_quantize_a8(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int M, int K, int r,
                              uint16_t* xh_bf16 /*out*/, uint8_t* x8 /*out*/, uint16_t* sx_fp16 /*out*/,
                              void* scratch, size_t scratch_bytes, void* stream);

int dirotq_w4a8_gemm(const uint16_t* xh_bf16, const uint8_t* x8, const uint16_t* sx_fp16, const void* blob,
                     const uint16_t* bias_bf16, int M, int N, int K, int r, int g, void* y /*out*/,
                     int y_dtype, void* stream);

/* Bytes of workspace dirotq_linear_a8 needs (x_h, x8, s_x and the scratch above). */
int dirotq_a8_workspace_bytes(int M, int K, int r, size_t* bytes /*host out*/);

/* The fused 8-bit layer: dirotq_rotate_quantize_a8 into `workspace`, then dirotq_w4a8_gemm. */
int dirotq_linear_a8(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob,
                     const uint16_t* bias_bf16, int M, int N, int K, int r, int g,
                     uint16_t* y_bf16 /*out*/, void* workspace, size_t workspace_bytes, void* stream);

/* ---- W4A16 layers ----------------------------------------------------------------- */
/*
 * Layers whose input activations stay in 16 bits (the paper's appendix on quantization
 * details): weight-only quantization, no rotation,
 *   y[m,n] = sum_j float(sw[n,j]) * sum_{k in group j} x[m,k] * q_w[n,k]  (+ bias[n]),
 * products exact, sums in fp32.  x_bf16 [M,K] row-major.  blob: a prepared-weight blob
 * with r = 0 (dirotq_import_weights, or dirotq_prepare_weights with Q the identity).
 * bias_bf16 [N] may be NULL.  y_dtype 0: y is bf16 [M,N]; 1: fp32 [M,N].  No workspace.
 * Shape, pointer and error rules as for dirotq_w4a4_gemm.
 */
int dirotq_w4a16_gemm(const uint16_t* x_bf16, const void* blob, const uint16_t* bias_bf16, int M, int N,
                      int K, int g, void* y /*out*/, int y_dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DIROTQ_H */
