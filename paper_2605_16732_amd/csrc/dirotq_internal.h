// Internal declarations shared by the translation units of libdirotq (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dirotq.h"

namespace dirotq {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

// Layout of the prepared-weight blob.  Three sections, each 256-byte aligned:
//   wh    bf16 [N][r]            16-bit branch of W' = W Q
//   codes u8   [N][(K-r)/2]      INT4 codes of W'[:, r:], two per byte (even channel low)
//   sw    fp16 [G][N]            group-major scales
//   wsum  i16  [G][N]            sum of the codes of each group (zero-point term of the
//                                asymmetric-activation product)
struct BlobLayout {
  size_t off_wh, off_codes, off_sw, off_wsum, bytes;
};
inline BlobLayout blob_layout(int N, int K, int r, int g) {
  BlobLayout L;
  const size_t G = (size_t)(K - r) / g;
  L.off_wh = 0;
  L.off_codes = align_up((size_t)N * r * 2);
  L.off_sw = L.off_codes + align_up((size_t)N * (K - r) / 2);
  L.off_wsum = L.off_sw + align_up(G * N * 2);
  L.bytes = L.off_wsum + align_up(G * N * 2);
  if (L.bytes == 0) L.bytes = kAlign;
  return L;
}

// Workspace of dirotq_linear[_asym]: xh bf16 [M][r] | xl u8 [M][(K-r)/2] | sx fp16 [G][M] | zx fp16 [G][M].
struct WorkspaceLayout {
  size_t off_xh, off_xl, off_sx, off_zx, bytes;
};
inline WorkspaceLayout workspace_layout(int M, int K, int r, int g) {
  WorkspaceLayout L;
  const size_t G = (size_t)(K - r) / g;
  L.off_xh = 0;
  L.off_xl = align_up((size_t)M * r * 2);
  L.off_sx = L.off_xl + align_up((size_t)M * (K - r) / 2);
  L.off_zx = L.off_sx + align_up(G * M * 2);
  L.bytes = L.off_zx + align_up(G * M * 2);
  if (L.bytes == 0) L.bytes = kAlign;
  return L;
}

// Workspace of dirotq_linear_a8: xh bf16 [M][r] | x8 u8 [M][K-r] | sx fp16 [M] | xf fp32 [M][K-r] |
// pmax fp32 [ceil((K-r)/128)][M].
struct WorkspaceA8Layout {
  size_t off_xh, off_x8, off_sx, off_xf, off_pmax, bytes;
};
inline WorkspaceA8Layout workspace_a8_layout(int M, int K, int r) {
  WorkspaceA8Layout L;
  const size_t KL = (size_t)(K - r);
  L.off_xh = 0;
  L.off_x8 = align_up((size_t)M * r * 2);
  L.off_sx = L.off_x8 + align_up((size_t)M * KL);
  L.off_xf = L.off_sx + align_up((size_t)M * 2);
  L.off_pmax = L.off_xf + align_up((size_t)M * KL * 4);
  L.bytes = L.off_pmax + align_up((KL + 127) / 128 * (size_t)M * 4);
  if (L.bytes == 0) L.bytes = kAlign;
  return L;
}

int check_shape(long M, long N, long K, long r, long g);   // DIROTQ_OK or DIROTQ_ERR_SHAPE
inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }
int hip_failed(hipError_t e);                               // records e, returns DIROTQ_ERR_HIP

// kernel launchers (arguments already validated)
// Outputs of the rotation kernel.  xf != nullptr: channels [r, K) are written unquantized (fp32, with
// the per-wave-tile absolute maxima in pmax); else zx != nullptr selects the asymmetric 4-bit
// quantizer, zx == nullptr the symmetric one.
struct RqOut {
  uint16_t* xh = nullptr;
  uint8_t* xl = nullptr;
  uint16_t* sx = nullptr;
  uint16_t* zx = nullptr;
  float* xf = nullptr;
  float* pmax = nullptr;
};
int launch_rotate_quantize(const uint16_t* x, const uint16_t* Qt, int M, int K, int r, int g, const RqOut& out,
                           hipStream_t s);
// per-token INT8 quantization of xf [M][KL] given pmax [ceil(KL/128)][M] -> x8 [M][KL], sx [M]
int launch_quantize_tokens(const float* xf, const float* pmax, int M, int KL, uint8_t* x8, uint16_t* sx,
                           hipStream_t s);
int launch_w4a8_gemm(const uint16_t* xh, const uint8_t* x8, const uint16_t* sx, const void* blob,
                     const uint16_t* bias, int M, int N, int K, int r, int g, void* y, int y_dtype,
                     hipStream_t s);
int launch_w4a16_gemm(const uint16_t* x, const void* blob, const uint16_t* bias, int M, int N, int K, int g, void* y,
                      int y_dtype, hipStream_t s);
int launch_w4a4_gemm(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const uint16_t* zx,
                     const void* blob, const uint16_t* bias, int M, int N, int K, int r, int g, void* y,
                     int y_dtype, hipStream_t s);
// 4-bit part not empty (wave-specialised schedule of the same arithmetic); zx: zero-points of asymmetric
// activation codes, or NULL for symmetric ones
int launch_w4a4_gemm_ws(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const uint16_t* zx, const void* blob,
                        const uint16_t* bias, int M, int N, int K, int r, int g, void* y, int y_dtype, hipStream_t s);
// symmetric activation codes, few tokens: the K axis split over the waves of a workgroup (64 x 64 outputs each)
int launch_w4a4_gemm_skinny(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const void* blob,
                            const uint16_t* bias, int M, int N, int K, int r, int g, void* y, int y_dtype,
                            hipStream_t s);
int launch_prepare_rotation(const float* Q, int K, uint16_t* Qt, hipStream_t s);
int launch_prepare_weights(const float* W, const float* Q, int N, int K, int r, int g, void* blob,
                           float* scratch, hipStream_t s);
int launch_import_weights(const uint16_t* Wh, const int8_t* codes, const uint16_t* sw, int N, int K,
                          int r, int g, void* blob, hipStream_t s);
int launch_export_weights(const void* blob, int N, int K, int r, int g, uint16_t* Wh, int8_t* codes,
                          uint16_t* sw, hipStream_t s);

#if defined(__HIPCC__)
// ---- device helpers ---------------------------------------------------------

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  // round to nearest even; inputs are finite in this library
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// two floats -> two bf16 in one dword (lo | hi << 16), round to nearest even: the packed hardware conversion
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_bits(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}
__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) {
  return (float)__builtin_bit_cast(_Float16, b);
}

// Scale of one quantization group from its absolute maximum (symmetric form of the
// paper's quantizer equation, q_max = 7): fp16_rne(min(amax / 7, 65504)).
// Returns the stored scale as float and its bit pattern.
__device__ __forceinline__ float group_scale(float amax, uint16_t& bits) {
  float s32 = fminf(amax / 7.0f, 65504.0f);      // IEEE-rounded division
  _Float16 h = (_Float16)s32;                     // round to nearest even
  bits = __builtin_bit_cast(uint16_t, h);
  return (float)h;
}
// Reciprocal used for the codes: 1 / s, IEEE-rounded; 0 for an all-zero group.
__device__ __forceinline__ float group_inv(float sf) { return sf == 0.0f ? 0.0f : 1.0f / sf; }
// 4-bit code of v: clip(rint(v * inv), -7, 7), ties to even.
__device__ __forceinline__ int quant_code(float v, float inv) {
  float t = rintf(v * inv);
  t = fminf(fmaxf(t, -7.0f), 7.0f);
  return (int)t;
}
// Stored form of a code q in [-7, 7]: sign-magnitude nibble, bit 3 = sign, bits 0-2 = |q|
// (zero is always 0x0).  Zero-extended to a byte with the sign moved to bit 7 this is the
// fp8 (E4M3) number q * 2^-9, which is how the GEMM kernel feeds codes to the matrix pipe.
__device__ __forceinline__ uint32_t code_nibble(int q) { return (uint32_t)(q < 0 ? (8 - q) : q) & 15u; }
__device__ __forceinline__ uint32_t quant_nibble(float v, float inv) { return code_nibble(quant_code(v, inv)); }
// Asymmetric form of the same quantizer (q_min = 0, q_max = 15): stored zero-point
// fp16_rne(clamp(min, +-65504)) and stored scale fp16_rne(min((max - min) / 15, 65504)).
__device__ __forceinline__ float group_zero(float mn, uint16_t& bits) {
  _Float16 h = (_Float16)fminf(fmaxf(mn, -65504.0f), 65504.0f);
  bits = __builtin_bit_cast(uint16_t, h);
  return (float)h;
}
__device__ __forceinline__ float group_scale_asym(float mn, float mx, uint16_t& bits) {
  float s32 = fminf((mx - mn) / 15.0f, 65504.0f);
  _Float16 h = (_Float16)s32;
  bits = __builtin_bit_cast(uint16_t, h);
  return (float)h;
}
// Unsigned 4-bit code of v: clip(rint((v - z) * inv), 0, 15); stored as the plain nibble.
__device__ __forceinline__ uint32_t quant_nibble_asym(float v, float zf, float inv) {
  float t = rintf((v - zf) * inv);
  t = fminf(fmaxf(t, 0.0f), 15.0f);
  return (uint32_t)(int)t;
}
__device__ __forceinline__ int nibble_code(uint32_t nib) { return (nib & 8u) ? -(int)(nib & 7u) : (int)(nib & 7u); }
#endif

}  // namespace dirotq
