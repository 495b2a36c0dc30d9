// Kernel B: y = x_h W'_h^T + sum_j s_x[:,j] s_w[:,j]^T * (q_x,j q_w,j^T)
// (forward-computation equation of Section 4.2 of the paper).
//
// The INT4 codes are unpacked once per workgroup on their way into LDS: a nibble is
// moved to the high half of a byte, so the i8 MFMA operand holds 16 q and the int32
// group dot is 256 I exactly (|256 I| <= 256 * 49 * 128 < 2^31); the factor 2^-8 is
// folded into the fp32 weight scale (exact).  Even and odd channels of an 8-channel
// dword land in different operand registers; both operands use the same permutation,
// so the dot product is unchanged.
#include "dirotq_internal.h"

namespace dirotq {

constexpr int BM = 128;         // tokens per workgroup tile
constexpr int BN = 128;         // output channels per workgroup tile
constexpr int BKQ = 128;        // 4-bit channels per LDS stage (one 128-byte i8 row)
constexpr int NTHREADS = 256;   // 4 waves as 2 (tokens) x 2 (outputs), 64x64 each
constexpr int STAGE_LD = BN + 4;
constexpr int OPER_BYTES = BM * BKQ;                 // one i8 operand tile (= one bf16 [128][64] tile)
constexpr int SCALE_BYTES = 4 * 128 * 4;             // up to 4 groups x 128 rows, fp32
constexpr int SMEM_LOOP = 4 * OPER_BYTES + 4 * SCALE_BYTES;
constexpr int SMEM_EPI = BM * STAGE_LD * 4;
constexpr int SMEM_BYTES = SMEM_LOOP > SMEM_EPI ? SMEM_LOOP : SMEM_EPI;

// [128 rows][128 B] tiles, 16-B chunk c of row r stored at slot c ^ (r & 7)
__device__ __forceinline__ int tile_off_bytes(int row, int chunk) {
  return row * 128 + ((chunk ^ (row & 7)) << 4);
}

// 8 nibbles of a dword -> two dwords of i8 holding 16*q: even channels, odd channels
__device__ __forceinline__ void unpack8(uint32_t p, uint32_t& even, uint32_t& odd) {
  even = (p << 4) & 0xF0F0F0F0u;
  odd = p & 0xF0F0F0F0u;
}

template <int GS, bool OUT_F32>
__global__ __launch_bounds__(NTHREADS, 2) void w4a4_gemm_kernel(
    const uint16_t* __restrict__ xh, const uint8_t* __restrict__ xl, const uint16_t* __restrict__ sx,
    const uint16_t* __restrict__ wh, const uint8_t* __restrict__ wq, const uint16_t* __restrict__ sw,
    const uint16_t* __restrict__ bias, int M, int N, int K, int r, void* __restrict__ y, int n_mt, int n_nt,
    int per_xcd) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* As = smem;                      // [2][OPER_BYTES]
  unsigned char* Bs = smem + 2 * OPER_BYTES;     // [2][OPER_BYTES]
  float* sxs = (float*)(smem + 4 * OPER_BYTES);  // [2][4][128]
  float* sws = sxs + 2 * 4 * 128;                // [2][4][128]

  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= n_mt * n_nt) return;
  const int mt = logical % n_mt, nt = logical / n_mt;
  const int m0 = mt * BM, n0 = nt * BN;

  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int wm = w & 1, wn = w >> 1;
  const int KL = K - r;            // number of 4-bit channels
  const int G = KL / GS;
  constexpr int GPS = BKQ / GS;    // groups per stage
  constexpr int MPG = GS / 32;     // MFMAs (k = 32) per group

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  // ---- 16-bit branch: acc = x_h W'_h^T, bf16 MFMA, 64 channels per stage ---------
  if (r > 0) {
    const int lrow = t >> 3, lchunk = t & 7;
    for (int k0 = 0; k0 < r; k0 += 64) {
      const bool ok = k0 + lchunk * 8 < r;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int row = lrow + 32 * i;
        const int m = min(m0 + row, M - 1), n = min(n0 + row, N - 1);
        uint4 va = ok ? *(const uint4*)(xh + (size_t)m * r + k0 + lchunk * 8) : make_uint4(0, 0, 0, 0);
        uint4 vb = ok ? *(const uint4*)(wh + (size_t)n * r + k0 + lchunk * 8) : make_uint4(0, 0, 0, 0);
        *(uint4*)(As + tile_off_bytes(row, lchunk)) = va;
        *(uint4*)(Bs + tile_off_bytes(row, lchunk)) = vb;
      }
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        bf16x8 a[2], b[2];
        const int chunk = 2 * ks + (l >> 5);
#pragma unroll
        for (int i = 0; i < 2; i++) {
          a[i] = *(const bf16x8*)(As + tile_off_bytes(wm * 64 + i * 32 + (l & 31), chunk));
          b[i] = *(const bf16x8*)(Bs + tile_off_bytes(wn * 64 + i * 32 + (l & 31), chunk));
        }
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
          for (int j = 0; j < 2; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      }
      __syncthreads();
    }
  }

  // ---- 4-bit branch ---------------------------------------------------------------
  if (KL > 0) {
    const size_t ldq = (size_t)KL / 2;       // packed bytes per row
    const int prow = t >> 2, pchunk = t & 3; // 2 rows x one 16-B packed chunk per operand per thread
    const uint8_t* ga[2];
    const uint8_t* gb[2];
#pragma unroll
    for (int i = 0; i < 2; i++) {
      ga[i] = xl + (size_t)min(m0 + prow + 64 * i, M - 1) * ldq + pchunk * 16;
      gb[i] = wq + (size_t)min(n0 + prow + 64 * i, N - 1) * ldq + pchunk * 16;
    }
    // scale staging: threads 0..127 own a token, 128..255 an output channel
    const bool is_x = t < 128;
    const int srow = t & 127;
    const uint16_t* gs = is_x ? sx + min(m0 + srow, M - 1) : sw + min(n0 + srow, N - 1);
    const size_t s_ld = is_x ? (size_t)M : (size_t)N;
    const float s_mul = is_x ? 1.0f : 0.00390625f;   // 2^-8 undoes the two 16x operand factors

    uint4 ra[2], rb[2];
    uint16_t rs[GPS];
    auto gload = [&](int st) {
      const bool ok = st * BKQ + pchunk * 32 < KL;
#pragma unroll
      for (int i = 0; i < 2; i++) {
        ra[i] = ok ? *(const uint4*)(ga[i] + (size_t)st * (BKQ / 2)) : make_uint4(0, 0, 0, 0);
        rb[i] = ok ? *(const uint4*)(gb[i] + (size_t)st * (BKQ / 2)) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int jj = 0; jj < GPS; jj++) {
        const int j = st * GPS + jj;
        rs[jj] = j < G ? gs[(size_t)j * s_ld] : (uint16_t)0;
      }
    };
    auto sstore = [&](int buf) {
#pragma unroll
      for (int i = 0; i < 2; i++) {
        const int row = prow + 64 * i;
        uint4 e, o;
        unpack8(ra[i].x, e.x, o.x);
        unpack8(ra[i].y, e.y, o.y);
        unpack8(ra[i].z, e.z, o.z);
        unpack8(ra[i].w, e.w, o.w);
        *(uint4*)(As + buf * OPER_BYTES + tile_off_bytes(row, 2 * pchunk)) = e;
        *(uint4*)(As + buf * OPER_BYTES + tile_off_bytes(row, 2 * pchunk + 1)) = o;
        unpack8(rb[i].x, e.x, o.x);
        unpack8(rb[i].y, e.y, o.y);
        unpack8(rb[i].z, e.z, o.z);
        unpack8(rb[i].w, e.w, o.w);
        *(uint4*)(Bs + buf * OPER_BYTES + tile_off_bytes(row, 2 * pchunk)) = e;
        *(uint4*)(Bs + buf * OPER_BYTES + tile_off_bytes(row, 2 * pchunk + 1)) = o;
      }
      float* sdst = (is_x ? sxs : sws) + buf * (4 * 128);
#pragma unroll
      for (int jj = 0; jj < GPS; jj++) sdst[jj * 128 + srow] = f16_bits_to_f32(rs[jj]) * s_mul;
    };

    const int nst = (KL + BKQ - 1) / BKQ;
    gload(0);
    sstore(0);
    __syncthreads();
    for (int st = 0; st < nst; st++) {
      const int buf = st & 1;
      if (st + 1 < nst) gload(st + 1);
      const unsigned char* Ab = As + buf * OPER_BYTES;
      const unsigned char* Bb = Bs + buf * OPER_BYTES;
      const float* sxb = sxs + buf * (4 * 128);
      const float* swb = sws + buf * (4 * 128);
#pragma unroll 1
      for (int jj = 0; jj < GPS; jj++) {
        i32x16 I[2][2];
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
          for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++) I[i][j][v] = 0;
#pragma unroll
        for (int kk = 0; kk < MPG; kk++) {
          const int chunk = 2 * (jj * MPG + kk) + (l >> 5);
          i32x4 a[2], b[2];
#pragma unroll
          for (int i = 0; i < 2; i++) {
            a[i] = *(const i32x4*)(Ab + tile_off_bytes(wm * 64 + i * 32 + (l & 31), chunk));
            b[i] = *(const i32x4*)(Bb + tile_off_bytes(wn * 64 + i * 32 + (l & 31), chunk));
          }
#pragma unroll
          for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++)
              I[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], I[i][j], 0, 0, 0);
        }
        // dequantize-accumulate: acc += float(256 I) * s_x[m] * (s_w[n] 2^-8)
        float swl[2];
#pragma unroll
        for (int j = 0; j < 2; j++) swl[j] = swb[jj * 128 + wn * 64 + j * 32 + (l & 31)];
#pragma unroll
        for (int i = 0; i < 2; i++) {
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const float4 s4 = *(const float4*)(sxb + jj * 128 + wm * 64 + i * 32 + 8 * q + 4 * (l >> 5));
            const float sv[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
            for (int e = 0; e < 4; e++)
#pragma unroll
              for (int j = 0; j < 2; j++)
                acc[i][j][4 * q + e] = fmaf((float)I[i][j][4 * q + e], sv[e] * swl[j], acc[i][j][4 * q + e]);
          }
        }
      }
      if (st + 1 < nst) sstore(buf ^ 1);
      __syncthreads();
    }
  }

  // ---- epilogue: [token][n] fp32 through LDS, 16-byte stores ----------------------
  float* stage = (float*)smem;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int n = wn * 64 + j * 32 + (l & 31);
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int token = wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (l >> 5) + (v & 3);
        stage[token * STAGE_LD + n] = acc[i][j][v];
      }
    }
  __syncthreads();
  const bool vec_ok = OUT_F32 ? (N % 4 == 0) : (N % 8 == 0);
  for (int pass = 0; pass < BM / 16; pass++) {
    const int row = pass * 16 + (t >> 4), nn = (t & 15) * 8;
    const int m = m0 + row, n = n0 + nn;
    if (m >= M || n >= N) continue;
    const float* src = stage + row * STAGE_LD + nn;
    float v[8];
    *(float4*)(v) = *(const float4*)(src);
    *(float4*)(v + 4) = *(const float4*)(src + 4);
    if (bias) {
#pragma unroll
      for (int e = 0; e < 8; e++)
        if (n + e < N) v[e] += bf16_bits_to_f32(bias[n + e]);
    }
    if (OUT_F32) {
      float* dst = (float*)y + (size_t)m * N + n;
      if (vec_ok && n + 8 <= N) {
        *(float4*)dst = *(float4*)v;
        *(float4*)(dst + 4) = *(float4*)(v + 4);
      } else {
        for (int e = 0; e < 8 && n + e < N; e++) dst[e] = v[e];
      }
    } else {
      uint16_t* dst = (uint16_t*)y + (size_t)m * N + n;
      if (vec_ok && n + 8 <= N) {
        uint4 o;
        o.x = f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
        o.y = f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
        o.z = f32_to_bf16_bits(v[4]) | ((uint32_t)f32_to_bf16_bits(v[5]) << 16);
        o.w = f32_to_bf16_bits(v[6]) | ((uint32_t)f32_to_bf16_bits(v[7]) << 16);
        *(uint4*)dst = o;
      } else {
        for (int e = 0; e < 8 && n + e < N; e++) dst[e] = f32_to_bf16_bits(v[e]);
      }
    }
  }
}

template <int GS, bool OUT_F32>
static int launch_one(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const void* blob,
                      const uint16_t* bias, int M, int N, int K, int r, void* y, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, GS);
  const char* bp = (const char*)blob;
  const int n_mt = (M + BM - 1) / BM, n_nt = (N + BN - 1) / BN;
  const long n_blocks = (long)n_mt * n_nt;
  const int per_xcd = (int)((n_blocks + 7) / 8);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)w4a4_gemm_kernel<GS, OUT_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
    if (e != hipSuccess) return hip_failed(e);
    attr_done = true;
  }
  hipLaunchKernelGGL((w4a4_gemm_kernel<GS, OUT_F32>), dim3(per_xcd * 8), dim3(NTHREADS), SMEM_BYTES, s, xh,
                     xl, sx, (const uint16_t*)(bp + L.off_wh), (const uint8_t*)(bp + L.off_codes),
                     (const uint16_t*)(bp + L.off_sw), bias, M, N, K, r, y, n_mt, n_nt, per_xcd);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

int launch_w4a4_gemm(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const void* blob,
                     const uint16_t* bias, int M, int N, int K, int r, int g, void* y, int y_dtype,
                     hipStream_t s) {
#define DIROTQ_CASE(GS)                                                                        \
  case GS:                                                                                     \
    return y_dtype ? launch_one<GS, true>(xh, xl, sx, blob, bias, M, N, K, r, y, s)            \
                   : launch_one<GS, false>(xh, xl, sx, blob, bias, M, N, K, r, y, s);
  switch (g) {
    DIROTQ_CASE(32)
    DIROTQ_CASE(64)
    DIROTQ_CASE(128)
  }
#undef DIROTQ_CASE
  return DIROTQ_ERR_SHAPE;
}

}  // namespace dirotq
