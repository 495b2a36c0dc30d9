// Shared tail of the GEMM kernels (128 x 128 workgroup tile, 4 waves as 2 (n) x 2 (tokens),
// each 64 n x 64 tokens = 2 x 2 accumulators of 32 x 32): the 16-bit branch
// acc += W'_h x_h^T (forward-computation equation of Section 4.2, first term) through bf16
// MFMAs, then bias and the store of y.  D[n][token] orientation: a lane owns one token and 4
// consecutive output channels per register quad.
#pragma once

#include "dirotq_internal.h"

namespace dirotq {

constexpr int TN = 128;         // output channels per workgroup tile
constexpr int TM = 128;         // tokens per workgroup tile
constexpr int NTHREADS = 256;   // 4 waves as 2 (n) x 2 (tokens), 64 n x 64 tokens each

// [rows][128 B] tiles, 16-B chunk c of row r stored at slot c ^ ((r >> 1) & 7): LDS has
// 64 banks and serves 16-byte accesses 16 lanes per cycle, so 16 consecutive rows must
// fall into 16 different 16-byte slots of a 256-byte bank line.
__device__ __forceinline__ int tile_off_bytes(int row, int chunk) {
  return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
}

// Bias and store of a wave's 64 n x 64 token block (2 x 2 accumulators of 32 x 32 in the D[n][token]
// orientation: a lane owns one token and 4 consecutive output channels per register quad -> 8-byte bf16
// stores).  n_base / m_base: first output channel / token of the block.
template <bool OUT_F32>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[2][2], const uint16_t* __restrict__ bias,
                                           void* __restrict__ y, int M, int N, int m_base, int n_base) {
  int l = threadIdx.x & 63;
  asm volatile("" : "+v"(l));   // (a caller that loops over tiles forms these addresses per tile, not once in registers)
  const int h = l >> 5;
  const bool vec_ok = (N % 4) == 0;
  if (vec_ok && n_base + 64 <= N) {
    // The block's 64 output channels all exist and rows are 8-byte aligned: straight-line code, one row
    // pointer per token, the channel offsets as immediates.
    float bv[2][4][4];
    if (bias) {
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const uint2 bb = *(const uint2*)(bias + n_base + i * 32 + 8 * q + 4 * h);
          bv[i][q][0] = bf16_bits_to_f32((uint16_t)(bb.x & 0xFFFF));
          bv[i][q][1] = bf16_bits_to_f32((uint16_t)(bb.x >> 16));
          bv[i][q][2] = bf16_bits_to_f32((uint16_t)(bb.y & 0xFFFF));
          bv[i][q][3] = bf16_bits_to_f32((uint16_t)(bb.y >> 16));
        }
    }
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int m = m_base + j * 32 + (l & 31);
      if (m >= M) continue;
      const size_t row = (size_t)m * N + n_base + 4 * h;
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          if (bias) {
#pragma unroll
            for (int e = 0; e < 4; e++) v[e] += bv[i][q][e];
          }
          if (OUT_F32) {
            *(float4*)((float*)y + row + i * 32 + 8 * q) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            uint2 o;
            o.x = f32x2_to_bf16x2_bits(v[0], v[1]);
            o.y = f32x2_to_bf16x2_bits(v[2], v[3]);
            *(uint2*)((uint16_t*)y + row + i * 32 + 8 * q) = o;
          }
        }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < 2; j++) {
    const int m = m_base + j * 32 + (l & 31);
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int n = n_base + i * 32 + 8 * q + 4 * h;
        if (n >= N) continue;
        float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        const bool full = vec_ok && n + 4 <= N;
        if (bias) {
          if (full) {
            const uint2 bb = *(const uint2*)(bias + n);
            v[0] += bf16_bits_to_f32((uint16_t)(bb.x & 0xFFFF));
            v[1] += bf16_bits_to_f32((uint16_t)(bb.x >> 16));
            v[2] += bf16_bits_to_f32((uint16_t)(bb.y & 0xFFFF));
            v[3] += bf16_bits_to_f32((uint16_t)(bb.y >> 16));
          } else {
#pragma unroll
            for (int e = 0; e < 4; e++)
              if (n + e < N) v[e] += bf16_bits_to_f32(bias[n + e]);
          }
        }
        if (OUT_F32) {
          float* dst = (float*)y + (size_t)m * N + n;
          if (full) {
            *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
          } else {
#pragma unroll
            for (int e = 0; e < 4; e++)
              if (n + e < N) dst[e] = v[e];
          }
        } else {
          uint16_t* dst = (uint16_t*)y + (size_t)m * N + n;
          if (full) {
            uint2 o;
            o.x = f32x2_to_bf16x2_bits(v[0], v[1]);
            o.y = f32x2_to_bf16x2_bits(v[2], v[3]);
            *(uint2*)dst = o;
          } else {
#pragma unroll
            for (int e = 0; e < 4; e++)
              if (n + e < N) dst[e] = f32_to_bf16_bits(v[e]);
          }
        }
      }
  }
}

// smem: at least 32 KB, free for reuse (the caller's main loop is over; a barrier is taken
// here before the first store).  rowA / rowB: this lane's operand rows of the two n tiles
// and the two token tiles within a [256 rows] stage (weights 0..127, tokens 128..255).
template <bool OUT_F32>
__device__ __forceinline__ void gemm_tail(f32x16 (&acc)[2][2], unsigned char* smem, const uint16_t* __restrict__ xh,
                                          const uint16_t* __restrict__ wh, const uint16_t* __restrict__ bias,
                                          void* __restrict__ y, int M, int N, int r, int m0, int n0,
                                          const int (&rowA)[2], const int (&rowB)[2]) {
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int wn = w & 1, wt = w >> 1;
  const int h = l >> 5;
  const int swz = ((l & 31) >> 1) & 7;                 // tile bases are multiples of 32 rows
  // ---- 16-bit branch: acc += W'_h x_h^T, bf16 MFMA, 64 channels per pass ----------
  if (r > 0) {
    const int lrow = t >> 3, lchunk = t & 7;   // 8 rows (stride 32) x one 16-B chunk per thread
    const uint16_t* src[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const int row = lrow + 32 * i;
      src[i] = (row < TN ? wh + (size_t)min(n0 + row, N - 1) * r : xh + (size_t)min(m0 + row - TN, M - 1) * r) +
               lchunk * 8;
    }
    // the next pass is loaded into registers while the current one is multiplied; channels past r
    // re-read the row's last chunk and are zeroed (unconditional loads, no control flow between them)
    uint4 v[8];
    auto fetch = [&](int k0) {
      const int off = min(k0 + lchunk * 8, r - 8) - lchunk * 8;
#pragma unroll
      for (int i = 0; i < 8; i++) v[i] = *(const uint4*)(src[i] + off);
    };
    fetch(0);
    for (int k0 = 0; k0 < r; k0 += 64) {
      const bool ok = k0 + lchunk * 8 < r;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 8; i++)
        *(uint4*)(smem + tile_off_bytes(lrow + 32 * i, lchunk)) = ok ? v[i] : make_uint4(0, 0, 0, 0);
      fetch(min(k0 + 64, r - 8));                // past the end: a harmless re-read, never used
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        bf16x8 a[2], b[2];
        const int chunk = 2 * ks + h;
#pragma unroll
        for (int i = 0; i < 2; i++) a[i] = *(const bf16x8*)(smem + rowA[i] * 128 + ((chunk ^ swz) << 4));
#pragma unroll
        for (int j = 0; j < 2; j++) b[j] = *(const bf16x8*)(smem + rowB[j] * 128 + ((chunk ^ swz) << 4));
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
          for (int j = 0; j < 2; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    }
  }

  store_tile<OUT_F32>(acc, bias, y, M, N, m0 + wt * 64, n0 + wn * 64);
}

}  // namespace dirotq
