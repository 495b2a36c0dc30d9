// Kernel A: online rotation x_hat = x Q (bf16 MFMA, fp32 accumulate) with the
// split / per-group quantize / pack fused into the GEMM epilogue (rotation/split
// equation of Section 4.2 and the quantizer of Section 3 of the paper).
//
// Orientation.  The product is computed transposed, D[channel][token] =
// sum_k Qt[channel][k] x[token][k], so both operands stream K-contiguous rows.
// Rotated channels are tiled relative to the split point r: tiles [0, n_hi) cover the
// bf16 channels [0, r), the rest cover [r, K) starting at r, so a quantization group
// (g | 128) never straddles a tile.
#include "dirotq_internal.h"

namespace dirotq {

constexpr int BC = 128;        // rotated channels per workgroup tile
constexpr int BT = 128;        // tokens per workgroup tile
constexpr int BK = 64;         // contraction step staged in LDS
constexpr int NTHREADS = 256;  // 4 waves as 2 (channels) x 2 (tokens), 64x64 each
constexpr int STAGE_LD = BC + 4;  // floats per token row of the epilogue staging tile
constexpr int OPER_BYTES = BC * BK * 2;                      // one operand tile, bf16
constexpr int SMEM_LOOP = 4 * OPER_BYTES;                    // A,B double-buffered
constexpr int SMEM_EPI = BT * STAGE_LD * 4;
constexpr int SMEM_BYTES = SMEM_LOOP > SMEM_EPI ? SMEM_LOOP : SMEM_EPI;

// Tiles are [128 rows][64 bf16] = 8 chunks of 16 B per row; chunk c of row r lives at
// slot c ^ (r & 7) so that the 16-B MFMA operand reads of 16 consecutive rows hit 16
// different bank groups.
__device__ __forceinline__ int tile_off(int row, int chunk) {  // in bf16 elements
  return row * BK + ((chunk ^ (row & 7)) << 3);
}

__global__ __launch_bounds__(NTHREADS, 2) void rotate_quantize_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ Qt, int M, int K, int r, int g,
    uint16_t* __restrict__ xh, uint8_t* __restrict__ xl, uint16_t* __restrict__ sx, int n_hi, int n_ct,
    int n_tt, int per_xcd) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* As = (uint16_t*)smem;                       // [2][BC*BK]
  uint16_t* Bs = (uint16_t*)(smem + 2 * OPER_BYTES);    // [2][BT*BK]

  // consecutive workgroup ids go to different XCDs; give each XCD a contiguous run of tiles
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= n_ct * n_tt) return;
  const int tt = logical % n_tt, ct = logical / n_tt;
  const bool hi = ct < n_hi;
  const int c0 = hi ? ct * BC : r + (ct - n_hi) * BC;
  const int c_lim = hi ? r : K;
  const int m0 = tt * BT;

  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int wc = w & 1, wt = w >> 1;

  // global -> register staging: 4 chunks of 16 B per operand per thread
  const int lrow = t >> 3, lchunk = t & 7;
  const uint16_t* ga[4];
  const uint16_t* gb[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int c = min(c0 + lrow + 32 * i, c_lim - 1);
    int m = min(m0 + lrow + 32 * i, M - 1);
    ga[i] = Qt + (size_t)c * K + lchunk * 8;
    gb[i] = x + (size_t)m * K + lchunk * 8;
  }
  uint4 ra[4], rb[4];
  auto gload = [&](int k0) {
    const bool ok = k0 + lchunk * 8 < K;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      ra[i] = ok ? *(const uint4*)(ga[i] + k0) : make_uint4(0, 0, 0, 0);
      rb[i] = ok ? *(const uint4*)(gb[i] + k0) : make_uint4(0, 0, 0, 0);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int row = lrow + 32 * i;
      *(uint4*)(As + buf * (BC * BK) + tile_off(row, lchunk)) = ra[i];
      *(uint4*)(Bs + buf * (BT * BK) + tile_off(row, lchunk)) = rb[i];
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  const int nk = (K + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; kt++) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * BK);
    const uint16_t* Ab = As + buf * (BC * BK);
    const uint16_t* Bb = Bs + buf * (BT * BK);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ks++) {
      bf16x8 a[2], b[2];
      const int chunk = 2 * ks + (l >> 5);
#pragma unroll
      for (int i = 0; i < 2; i++) {
        int ra_ = wc * 64 + i * 32 + (l & 31);
        int rb_ = wt * 64 + i * 32 + (l & 31);
        a[i] = *(const bf16x8*)(Ab + tile_off(ra_, chunk));
        b[i] = *(const bf16x8*)(Bb + tile_off(rb_, chunk));
      }
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: accumulators -> LDS as [token][channel] fp32 --------------------
  float* stage = (float*)smem;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int token = wt * 64 + j * 32 + (l & 31);
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int ch = wc * 64 + i * 32 + 8 * q + 4 * (l >> 5);
        float4 v = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                               acc[i][j][4 * q + 3]);
        *(float4*)(stage + token * STAGE_LD + ch) = v;
      }
    }
  __syncthreads();

  if (hi) {
    // bf16 part: one unit = (token, 32 channels) -> 64 contiguous bytes of xh
    for (int u = t; u < BT * (BC / 32); u += NTHREADS) {
      const int token = u & (BT - 1), chk = u >> 7;
      const int c = c0 + chk * 32, m = m0 + token;
      if (c >= c_lim || m >= M) continue;
      const float* src = stage + token * STAGE_LD + chk * 32;
      uint16_t* dst = xh + (size_t)m * r + c;
#pragma unroll
      for (int p = 0; p < 4; p++) {
        float4 v0 = *(const float4*)(src + 8 * p), v1 = *(const float4*)(src + 8 * p + 4);
        uint4 o;
        o.x = f32_to_bf16_bits(v0.x) | ((uint32_t)f32_to_bf16_bits(v0.y) << 16);
        o.y = f32_to_bf16_bits(v0.z) | ((uint32_t)f32_to_bf16_bits(v0.w) << 16);
        o.z = f32_to_bf16_bits(v1.x) | ((uint32_t)f32_to_bf16_bits(v1.y) << 16);
        o.w = f32_to_bf16_bits(v1.z) | ((uint32_t)f32_to_bf16_bits(v1.w) << 16);
        *(uint4*)(dst + 8 * p) = o;
      }
    }
  } else {
    // INT4 part: one unit = (token, group of g channels)
    const int ng = BC / g;
    const size_t xl_ld = (size_t)(K - r) / 2;
    for (int u = t; u < BT * ng; u += NTHREADS) {
      const int token = u & (BT - 1), grp = u >> 7;
      const int cl = (c0 - r) + grp * g;   // first 4-bit channel of the group
      const int m = m0 + token;
      if (c0 + grp * g >= c_lim || m >= M) continue;
      const float* src = stage + token * STAGE_LD + grp * g;
      float amax = 0.0f;
      for (int p = 0; p < g; p += 4) {
        float4 v = *(const float4*)(src + p);
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
      }
      uint16_t sbits;
      const float sf = group_scale(amax, sbits);
      const float inv = group_inv(sf);
      sx[(size_t)(cl / g) * M + m] = sbits;
      uint8_t* dst = xl + (size_t)m * xl_ld + cl / 2;
      for (int p = 0; p < g; p += 32) {
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; d++) {
          float4 v0 = *(const float4*)(src + p + 8 * d), v1 = *(const float4*)(src + p + 8 * d + 4);
          uint32_t wv = 0;
          wv |= (uint32_t)(quant_code(v0.x, inv) & 0xF);
          wv |= (uint32_t)(quant_code(v0.y, inv) & 0xF) << 4;
          wv |= (uint32_t)(quant_code(v0.z, inv) & 0xF) << 8;
          wv |= (uint32_t)(quant_code(v0.w, inv) & 0xF) << 12;
          wv |= (uint32_t)(quant_code(v1.x, inv) & 0xF) << 16;
          wv |= (uint32_t)(quant_code(v1.y, inv) & 0xF) << 20;
          wv |= (uint32_t)(quant_code(v1.z, inv) & 0xF) << 24;
          wv |= (uint32_t)(quant_code(v1.w, inv) & 0xF) << 28;
          o[d] = wv;
        }
        *(uint4*)(dst + p / 2) = make_uint4(o[0], o[1], o[2], o[3]);
      }
    }
  }
}

int launch_rotate_quantize(const uint16_t* x, const uint16_t* Qt, int M, int K, int r, int g, uint16_t* xh,
                           uint8_t* xl, uint16_t* sx, hipStream_t s) {
  const int n_hi = (r + BC - 1) / BC;
  const int n_lo = (K - r + BC - 1) / BC;
  const int n_ct = n_hi + n_lo;
  const int n_tt = (M + BT - 1) / BT;
  const long n_blocks = (long)n_ct * n_tt;
  const int per_xcd = (int)((n_blocks + 7) / 8);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)rotate_quantize_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
    if (e != hipSuccess) return hip_failed(e);
    attr_done = true;
  }
  hipLaunchKernelGGL(rotate_quantize_kernel, dim3(per_xcd * 8), dim3(NTHREADS), SMEM_BYTES, s, x, Qt, M, K,
                     r, g, xh, xl, sx, n_hi, n_ct, n_tt, per_xcd);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

}  // namespace dirotq
