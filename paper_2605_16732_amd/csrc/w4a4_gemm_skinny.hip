// Kernel B for few tokens (symmetric activation codes): the same sum as w4a4_gemm.hip,
//   y = x_h W'_h^T + sum_j s_x[:,j] s_w[:,j]^T * (q_x,j q_w,j^T)
// (forward-computation equation of Section 4.2 of the paper), scheduled for latency.
//
// With a few hundred tokens the tiled kernels put a handful of workgroups on a 256-CU chip, and each walks the
// whole K axis stage by stage (global load -> LDS -> barrier -> MFMA) alone on its CU: the time is a sum of
// memory latencies.  Here the K axis is split over the 8 waves of a workgroup instead.  A workgroup owns 64
// output channels x 64 tokens; wave w takes the work items w, w + 8, ... of the K axis (an item = 16 channels of
// the 16-bit branch or one 64-channel piece of the 4-bit part; a 32-channel group when g = 32).  Nothing is
// shared between waves, so operands go from global memory straight into registers in the MFMA operand layout
// (a lane loads the 16 bytes of its row and k-half), one item ahead; there is no LDS staging and no barrier
// in the loop.  The eight partial 64 x 64 accumulators then meet in LDS and are summed in a fixed order.
// Arithmetic per item as in the other schedules: fp8 MFMA on the codes (block scale 2^9 on both operands: the
// group dot comes back as the integer), fp16 MFMA for the scale product, one fma per accumulator.
#include <atomic>

#include "gemm_tail.h"

namespace dirotq {

namespace skinny {

constexpr int TS = 64;                       // output channels and tokens per workgroup
constexpr int NW = 8, NT = NW * 64;
constexpr int SMEM = NW * 16 * 64 * 16;      // partial sums: [wave][register quad 0..15][lane] float4 = 128 KB

typedef __attribute__((ext_vector_type(8))) int i32x8;

__device__ __forceinline__ void unpack8(uint32_t p, uint32_t& even, uint32_t& odd) {
  even = (p & 0x07070707u) | ((p & 0x08080808u) << 4);
  odd = ((p >> 4) & 0x07070707u) | (p & 0x80808080u);
}

// registers of one work item: the lane's operand bytes for 2 weight tiles and 2 token tiles, and their scales
struct Item {
  uint4 a[2], b[2];
  uint16_t sa[2], sb[2];
};

template <int GS, bool OUT_F32>
__global__ __launch_bounds__(NT, 2) void w4a4_gemm_skinny_kernel(
    const uint16_t* __restrict__ xh, const uint8_t* __restrict__ xl, const uint16_t* __restrict__ sx,
    const uint16_t* __restrict__ wh, const uint8_t* __restrict__ wq, const uint16_t* __restrict__ sw,
    const uint16_t* __restrict__ bias, int M, int N, int K, int r, void* __restrict__ y, int n_nt) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int nt = blockIdx.x % n_nt, mt = blockIdx.x / n_nt;
  const int n0 = nt * TS, m0 = mt * TS;
  const int t = threadIdx.x, l = t & 63, h = l >> 5;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int KL = K - r;
  constexpr int ICH = GS == 32 ? 32 : 64;    // 4-bit channels per item
  const int nb = r / 16, nq = KL / ICH, items = nb + nq;
  const size_t ldq = (size_t)KL / 2;

  // the lane's rows (clamped at the edges: those results are not stored)
  size_t rowA[2], rowB[2];
#pragma unroll
  for (int i = 0; i < 2; i++) rowA[i] = (size_t)min(n0 + i * 32 + (l & 31), N - 1);
#pragma unroll
  for (int j = 0; j < 2; j++) rowB[j] = (size_t)min(m0 + j * 32 + (l & 31), M - 1);

  // Loads of one shape whatever the item's kind (16 bytes per operand row, two scale halfwords), unconditional
  // (an index past the end re-reads the last item, unused): straight-line code, so a wait covers its own item
  // only and the next item's loads stay in flight.
  const uint8_t* whb = (const uint8_t*)wh;
  const uint8_t* xhb = (const uint8_t*)xh;
  auto load = [&](Item& it, int idx) {
    idx = min(idx, items - 1);
    const bool is_b = idx < nb;
    const int qi = max(idx - nb, 0);
    // 16 bf16 channels: this lane's 8 (k = 8 h ..); 64 4-bit channels: this lane's 32 = 16 packed bytes;
    // a 32-channel group: its 16 packed bytes, of which the lane uses the half h
    const size_t offq = GS == 32 ? (size_t)qi * 16 : (size_t)qi * 32 + h * 16;
    const size_t offb = (size_t)idx * 32 + h * 16;
#pragma unroll
    for (int i = 0; i < 2; i++)
      it.a[i] = *(const uint4*)(is_b ? whb + rowA[i] * (size_t)(2 * r) + offb : wq + rowA[i] * ldq + offq);
#pragma unroll
    for (int j = 0; j < 2; j++)
      it.b[j] = *(const uint4*)(is_b ? xhb + rowB[j] * (size_t)(2 * r) + offb : xl + rowB[j] * ldq + offq);
    const size_t grp = (size_t)(qi * ICH) / GS;         // (group 0 for an item of the 16-bit branch: unused)
#pragma unroll
    for (int i = 0; i < 2; i++) it.sa[i] = sw[grp * N + rowA[i]];
#pragma unroll
    for (int j = 0; j < 2; j++) it.sb[j] = sx[grp * M + rowB[j]];
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  auto compute = [&](const Item& it, int idx) {
    if (idx < nb) {
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, it.a[i]),
                                                              __builtin_bit_cast(bf16x8, it.b[j]), acc[i][j], 0, 0, 0);
      return;
    }
    // nibbles -> fp8 bytes [s 0000 mmm]; even channels of a dword to one register, odd ones to another (the same
    // permutation on both operands)
    i32x8 av[2], bv[2];
    auto expand = [&](const uint4& p) -> i32x8 {
      uint32_t e[4], o[4];
      if (GS == 32) {                                  // the lane's 8 bytes of the group's 16; upper k half empty
        unpack8(h ? p.z : p.x, e[0], o[0]);
        unpack8(h ? p.w : p.y, e[1], o[1]);
        return i32x8{(int)e[0], (int)o[0], (int)e[1], (int)o[1], 0, 0, 0, 0};
      }
      unpack8(p.x, e[0], o[0]);
      unpack8(p.y, e[1], o[1]);
      unpack8(p.z, e[2], o[2]);
      unpack8(p.w, e[3], o[3]);
      return i32x8{(int)e[0], (int)o[0], (int)e[1], (int)o[1], (int)e[2], (int)o[2], (int)e[3], (int)o[3]};
    };
#pragma unroll
    for (int i = 0; i < 2; i++) av[i] = expand(it.a[i]);
#pragma unroll
    for (int j = 0; j < 2; j++) bv[j] = expand(it.b[j]);
    // scale vectors {s, 0, 0, 0} in lanes 0..31 (k-slot 0 of the fp16 MFMA), zeros in lanes 32..63
    f16x4 sa[2], sb[2];
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const uint32_t lo = h ? 0u : (uint32_t)it.sa[i];
      sa[i] = __builtin_bit_cast(f16x4, make_uint2(lo, 0u));
    }
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const uint32_t lo = h ? 0u : (uint32_t)it.sb[j];
      sb[j] = __builtin_bit_cast(f16x4, make_uint2(lo, 0u));
    }
    const int sc9 = 127 + 9;                           // E8M0 block scale 2^9: (q 2^-9 2^9)(q' 2^-9 2^9) = q q'
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++) {
        f32x16 z, p;
#pragma unroll
        for (int v = 0; v < 16; v++) z[v] = p[v] = 0.0f;
        const f32x16 I = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av[i], bv[j], z, 0, 0, 0, sc9, 0, sc9);
        const f32x16 P = __builtin_amdgcn_mfma_f32_32x32x8f16(sa[i], sb[j], p, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] = fmaf(I[v], P[v], acc[i][j][v]);
      }
  };

  // two register sets, alternately: the loads of the next item are in flight while this one is multiplied
  Item A, B;
  load(A, w);
  for (int idx = w; idx < items; idx += 2 * NW) {
    load(B, idx + NW);
    compute(A, idx);
    load(A, idx + 2 * NW);
    if (idx + NW < items) compute(B, idx + NW);
  }

  // ---- the eight partial sums meet in LDS; thread t sums quads t and t + 512 over the waves, in wave order ----
  float4* part = (float4*)smem;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int q = 0; q < 4; q++)
        part[((w * 16) + (i * 2 + j) * 4 + q) * 64 + l] =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
  __syncthreads();
#pragma unroll
  for (int s = 0; s < 2; s++) {
    const int slot = t + s * NT;                       // 0..1023 = (register quad, lane)
    const int tq = slot >> 6, lane = slot & 63;
    float4 v = part[tq * 64 + lane];
#pragma unroll
    for (int ww = 1; ww < NW; ww++) {
      const float4 u = part[(ww * 16 + tq) * 64 + lane];
      v.x += u.x;
      v.y += u.y;
      v.z += u.z;
      v.w += u.w;
    }
    const int i = tq >> 3, j = (tq >> 2) & 1, q = tq & 3;
    const int m = m0 + j * 32 + (lane & 31), n = n0 + i * 32 + 8 * q + 4 * (lane >> 5);
    if (m >= M || n >= N) continue;
    float o[4] = {v.x, v.y, v.z, v.w};
    const bool full = (N % 4) == 0 && n + 4 <= N;
    if (bias) {
#pragma unroll
      for (int e = 0; e < 4; e++)
        if (n + e < N) o[e] += bf16_bits_to_f32(bias[n + e]);
    }
    if (OUT_F32) {
      float* dst = (float*)y + (size_t)m * N + n;
      if (full) {
        *(float4*)dst = make_float4(o[0], o[1], o[2], o[3]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; e++)
          if (n + e < N) dst[e] = o[e];
      }
    } else {
      uint16_t* dst = (uint16_t*)y + (size_t)m * N + n;
      if (full) {
        *(uint2*)dst = make_uint2(f32x2_to_bf16x2_bits(o[0], o[1]), f32x2_to_bf16x2_bits(o[2], o[3]));
      } else {
#pragma unroll
        for (int e = 0; e < 4; e++)
          if (n + e < N) dst[e] = f32_to_bf16_bits(o[e]);
      }
    }
  }
}

template <int GS, bool OUT_F32>
static int launch_one(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const void* blob,
                      const uint16_t* bias, int M, int N, int K, int r, void* y, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, GS);
  const char* bp = (const char*)blob;
  const int n_mt = (M + TS - 1) / TS, n_nt = (N + TS - 1) / TS;
  const long n_blocks = (long)n_mt * n_nt;
  if (n_blocks > 0x7FFFFFFFL) return DIROTQ_ERR_SHAPE;
  // (idempotent: two threads racing here would both set the same attribute)
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)w4a4_gemm_skinny_kernel<GS, OUT_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return hip_failed(e);
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((w4a4_gemm_skinny_kernel<GS, OUT_F32>), dim3((unsigned)n_blocks), dim3(NT), SMEM, s, xh, xl, sx,
                     (const uint16_t*)(bp + L.off_wh), (const uint8_t*)(bp + L.off_codes),
                     (const uint16_t*)(bp + L.off_sw), bias, M, N, K, r, y, n_nt);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

}  // namespace skinny

int launch_w4a4_gemm_skinny(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const void* blob,
                            const uint16_t* bias, int M, int N, int K, int r, int g, void* y, int y_dtype,
                            hipStream_t s) {
  switch (g) {
    case 32:
      return y_dtype ? skinny::launch_one<32, true>(xh, xl, sx, blob, bias, M, N, K, r, y, s)
                     : skinny::launch_one<32, false>(xh, xl, sx, blob, bias, M, N, K, r, y, s);
    case 64:
      return y_dtype ? skinny::launch_one<64, true>(xh, xl, sx, blob, bias, M, N, K, r, y, s)
                     : skinny::launch_one<64, false>(xh, xl, sx, blob, bias, M, N, K, r, y, s);
    case 128:
      return y_dtype ? skinny::launch_one<128, true>(xh, xl, sx, blob, bias, M, N, K, r, y, s)
                     : skinny::launch_one<128, false>(xh, xl, sx, blob, bias, M, N, K, r, y, s);
  }
  return DIROTQ_ERR_SHAPE;
}

}  // namespace dirotq
