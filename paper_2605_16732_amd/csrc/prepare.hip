// Offline side of the layer (weight-fusion step of Section 4.2 of the paper, just before
// its forward-computation equation): W' = W Q in fp64, split at r, round-to-nearest
// INT4 with fp16 group scales; plus import/export of the prepared-weight blob and the
// bf16 transposed rotation operand.  None of this is on the per-step hot path.
#include "dirotq_internal.h"

namespace dirotq {

// ---- Qt[c][k] = bf16(Q[k][c]) ---------------------------------------------------
__global__ __launch_bounds__(256) void transpose_to_bf16_kernel(const float* __restrict__ Q, int K,
                                                                uint16_t* __restrict__ Qt) {
  __shared__ float tile[32][33];
  const int bx = blockIdx.x * 32, by = blockIdx.y * 32;   // bx: c block, by: k block
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5; // 32 x 8
  for (int i = ty; i < 32; i += 8) tile[i][tx] = Q[(size_t)(by + i) * K + bx + tx];   // tile[k][c]
  __syncthreads();
  for (int i = ty; i < 32; i += 8) Qt[(size_t)(bx + i) * K + by + tx] = f32_to_bf16_bits(tile[tx][i]);
}

int launch_prepare_rotation(const float* Q, int K, uint16_t* Qt, hipStream_t s) {
  hipLaunchKernelGGL(transpose_to_bf16_kernel, dim3(K / 32, K / 32), dim3(256), 0, s, Q, K, Qt);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

// ---- Wp[n][c] = fp32( sum_k W[n][k] Q[k][c] ) with fp64 accumulation ------------
// 64 x 64 output tile per workgroup, 4 x 4 outputs per thread, 16 k per LDS stage.
__global__ __launch_bounds__(256) void fuse_rotation_fp64_kernel(const float* __restrict__ W,
                                                                 const float* __restrict__ Q, int N, int K,
                                                                 float* __restrict__ Wp) {
  __shared__ double Ws[16][64 + 2];
  __shared__ double Qs[16][64 + 2];
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  // one workgroup per 64 x 64 tile, tiles numbered row-major over (n tile, c tile) on a 1-D grid
  const int n_ct = (K + 63) / 64;
  const int n0 = (int)(blockIdx.x / n_ct) * 64, c0 = (int)(blockIdx.x % n_ct) * 64;
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = 0.0;
  const int wrow = t >> 2, wk = (t & 3) * 4;    // W tile: 64 rows x 16 k
  const int qk = t >> 4, qc = (t & 15) * 4;     // Q tile: 16 k x 64 c
  const int wn = min(n0 + wrow, N - 1);
  const bool qok = c0 + qc < K;
  for (int k0 = 0; k0 < K; k0 += 16) {
    const float4 wv = *(const float4*)(W + (size_t)wn * K + k0 + wk);
    const float4 qv = qok ? *(const float4*)(Q + (size_t)(k0 + qk) * K + c0 + qc) : make_float4(0, 0, 0, 0);
    __syncthreads();
    Ws[wk + 0][wrow] = wv.x;
    Ws[wk + 1][wrow] = wv.y;
    Ws[wk + 2][wrow] = wv.z;
    Ws[wk + 3][wrow] = wv.w;
    Qs[qk][qc + 0] = qv.x;
    Qs[qk][qc + 1] = qv.y;
    Qs[qk][qc + 2] = qv.z;
    Qs[qk][qc + 3] = qv.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = Ws[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) b[j] = Qs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fma(a[i], b[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int n = n0 + ty * 4 + i, c = c0 + tx * 4;
    if (n < N && c < K)
      *(float4*)(Wp + (size_t)n * K + c) =
          make_float4((float)acc[i][0], (float)acc[i][1], (float)acc[i][2], (float)acc[i][3]);
  }
}

// ---- split + quantize rows of an fp32 matrix -------------------------------------
// unit u < rows * (r/32): (row, 32-channel chunk of the bf16 part)
// else: (row, group).  Consecutive threads take consecutive rows.
__global__ __launch_bounds__(256) void split_quantize_rows_kernel(const float* __restrict__ src, int rows,
                                                                  int K, int r, int g,
                                                                  uint16_t* __restrict__ hi,
                                                                  uint8_t* __restrict__ codes,
                                                                  uint16_t* __restrict__ scales,
                                                                  int16_t* __restrict__ wsum) {
  const long u = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long n_hi = (long)rows * (r / 32);
  const int G = (K - r) / g;
  if (u < n_hi) {
    const int row = (int)(u % rows), chk = (int)(u / rows);
    const float* s = src + (size_t)row * K + chk * 32;
    uint16_t* d = hi + (size_t)row * r + chk * 32;
    for (int p = 0; p < 32; p++) d[p] = f32_to_bf16_bits(s[p]);
    return;
  }
  const long v = u - n_hi;
  if (v >= (long)rows * G) return;
  const int row = (int)(v % rows), j = (int)(v / rows);
  const float* s = src + (size_t)row * K + r + j * g;
  float amax = 0.0f;
  for (int p = 0; p < g; p++) amax = fmaxf(amax, fabsf(s[p]));
  uint16_t sbits;
  const float sf = group_scale(amax, sbits);
  const float inv = group_inv(sf);
  scales[(size_t)j * rows + row] = sbits;
  uint8_t* d = codes + (size_t)row * ((K - r) / 2) + j * (g / 2);
  int sum = 0;
  for (int p = 0; p < g; p += 2) {
    const int q0 = quant_code(s[p], inv), q1 = quant_code(s[p + 1], inv);
    d[p / 2] = (uint8_t)(code_nibble(q0) | (code_nibble(q1) << 4));
    sum += q0 + q1;
  }
  wsum[(size_t)j * rows + row] = (int16_t)sum;     // |sum| <= 7 * 128
}

int launch_prepare_weights(const float* W, const float* Q, int N, int K, int r, int g, void* blob,
                           float* scratch, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, g);
  char* bp = (char*)blob;
  // 1-D grids: both launches must stay within 2^31 - 1 workgroups (only shapes whose fp32 scratch alone
  // would exceed 2^44 bytes get there)
  const long n_tiles = (long)((K + 63) / 64) * (long)((N + 63) / 64);
  const long n_units = (long)N * (r / 32) + (long)N * ((K - r) / g);
  if (n_tiles > 0x7FFFFFFFL || (n_units + 255) / 256 > 0x7FFFFFFFL) return DIROTQ_ERR_SHAPE;
  hipLaunchKernelGGL(fuse_rotation_fp64_kernel, dim3((unsigned)n_tiles), dim3(256), 0, s, W, Q, N, K, scratch);
  hipError_t e0 = hipGetLastError();
  if (e0 != hipSuccess) return hip_failed(e0);      // nothing else is enqueued on an unwritten scratch
  hipLaunchKernelGGL(split_quantize_rows_kernel, dim3((unsigned)((n_units + 255) / 256)), dim3(256), 0, s,
                     scratch, N, K, r, g, (uint16_t*)(bp + L.off_wh), (uint8_t*)(bp + L.off_codes),
                     (uint16_t*)(bp + L.off_sw), (int16_t*)(bp + L.off_wsum));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

// ---- import / export of the blob -------------------------------------------------
__global__ __launch_bounds__(256) void import_kernel(const uint16_t* __restrict__ Wh,
                                                     const int8_t* __restrict__ codes,
                                                     const uint16_t* __restrict__ sw, int N, int K, int r,
                                                     int g, uint16_t* __restrict__ bwh,
                                                     uint8_t* __restrict__ bq, uint16_t* __restrict__ bsw,
                                                     int16_t* __restrict__ bwsum) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long n_wh = (long)N * r, n_q = (long)N * (K - r) / 2;
  const int G = (K - r) / g;
  if (i < n_wh) bwh[i] = Wh[i];
  // (codes outside [-7, 7] are clamped: the symmetric 4-bit quantizer never produces -8)
  auto clamp7 = [](int q) { return min(max(q, -7), 7); };
  if (i < n_q) bq[i] = (uint8_t)(code_nibble(clamp7(codes[2 * i])) | (code_nibble(clamp7(codes[2 * i + 1])) << 4));
  if (i < (long)N * G) {
    const int n = (int)(i / G), j = (int)(i % G);
    bsw[(size_t)j * N + n] = sw[i];
    const int8_t* c = codes + (size_t)n * (K - r) + (size_t)j * g;
    int sum = 0;
    for (int p = 0; p < g; p++) sum += clamp7(c[p]);
    bwsum[(size_t)j * N + n] = (int16_t)sum;
  }
}

__global__ __launch_bounds__(256) void export_kernel(const uint16_t* __restrict__ bwh,
                                                     const uint8_t* __restrict__ bq,
                                                     const uint16_t* __restrict__ bsw, int N, int K, int r,
                                                     int g, uint16_t* __restrict__ Wh,
                                                     int8_t* __restrict__ codes, uint16_t* __restrict__ sw) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long n_wh = (long)N * r, n_q = (long)N * (K - r) / 2;
  const int G = (K - r) / g;
  if (Wh && i < n_wh) Wh[i] = bwh[i];
  if (codes && i < n_q) {
    const int b = bq[i];
    codes[2 * i] = (int8_t)nibble_code(b & 15);
    codes[2 * i + 1] = (int8_t)nibble_code(b >> 4);
  }
  if (sw && i < (long)N * G) {
    const int n = (int)(i / G), j = (int)(i % G);
    sw[i] = bsw[(size_t)j * N + n];
  }
}

static long max3(long a, long b, long c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }

int launch_import_weights(const uint16_t* Wh, const int8_t* codes, const uint16_t* sw, int N, int K, int r,
                          int g, void* blob, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, g);
  char* bp = (char*)blob;
  const long n = max3((long)N * r, (long)N * (K - r) / 2, (long)N * ((K - r) / g));
  if (n == 0) return DIROTQ_OK;
  hipLaunchKernelGGL(import_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, Wh, codes, sw, N, K,
                     r, g, (uint16_t*)(bp + L.off_wh), (uint8_t*)(bp + L.off_codes),
                     (uint16_t*)(bp + L.off_sw), (int16_t*)(bp + L.off_wsum));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

int launch_export_weights(const void* blob, int N, int K, int r, int g, uint16_t* Wh, int8_t* codes,
                          uint16_t* sw, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, g);
  const char* bp = (const char*)blob;
  const long n = max3((long)N * r, (long)N * (K - r) / 2, (long)N * ((K - r) / g));
  if (n == 0) return DIROTQ_OK;
  hipLaunchKernelGGL(export_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                     (const uint16_t*)(bp + L.off_wh), (const uint8_t*)(bp + L.off_codes),
                     (const uint16_t*)(bp + L.off_sw), N, K, r, g, Wh, codes, sw);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

}  // namespace dirotq
