// W4A8 variant: 8-bit per-token activations against 4-bit per-group weights
// (the paper's implementation details for 8-bit settings: per-token dynamic activation
// quantization; the forward-computation equation of Section 4.2 with one activation scale
// per token):  y = x_h W'_h^T + s_x[m] * sum_j s_w[n,j] * (q8_x,j q4_w,j^T).
//
// quantize_tokens_kernel.  The rotation kernel leaves the channels [r, K) as fp32 together
// with the absolute maximum of every 128-channel tile; this kernel reduces those maxima per
// token, applies the Section 3 quantizer with q_max = 127 and stores sign-magnitude bytes.
// Within each 32-channel block the 16 even channels come first, then the 16 odd ones: the
// order in which the GEMM's weight unpacking produces them.
//
// w4a8_gemm_kernel.  An INT8 code is sign * (16 a + b) with a in 0..7, b in 0..15.  The bytes
// [s 0000 aaa] and [s 000 bbbb] are exact fp8 (E4M3) numbers a 2^-9 and b 2^-9, so the code
// runs on the fp8 matrix pipe as two planes.  The 32x32x64 MFMA takes 32 channels per step:
// the first 16 bytes of a lane's operand belong to k-block 0, the last 16 to k-block 1, and
// the block-scaled form of the instruction multiplies block 0 of the activations by 2^4: one
// MFMA returns 2^-18 * sum_k (16 a_k + b_k) w_k, exactly.  The weight operand carries the
// same 16 bytes in both blocks.  Everything downstream is the W4A4 kernel: scale product by an
// fp16 MFMA (s_w[n,j] x s_x[m]), one fma per accumulator and group, 16-bit branch, store.
//
// Stage = 64 channels: weights [128 rows][64 B], activations [128 rows][64 B a-plane | 64 B
// b-plane]; two stages in LDS; global loads run one stage ahead through registers.
#include <atomic>

#include "gemm_tail.h"

namespace dirotq {

// ---- per-token quantizer -----------------------------------------------------------------
__global__ __launch_bounds__(256) void quantize_tokens_kernel(const float* __restrict__ xf,
                                                              const float* __restrict__ pmax, int M, int KL,
                                                              uint8_t* __restrict__ x8, uint16_t* __restrict__ sx) {
  __shared__ float red[4];
  const int m = blockIdx.x, t = threadIdx.x;
  const int n_tiles = (KL + 127) / 128;
  float a = 0.0f;
  for (int i = t; i < n_tiles; i += 256) a = fmaxf(a, pmax[(size_t)i * M + m]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a = fmaxf(a, __shfl_xor(a, o));
  if ((t & 63) == 0) red[t >> 6] = a;
  __syncthreads();
  const float amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  // quantizer equation, symmetric, q_max = 127: stored scale fp16_rne(min(amax / 127, 65504))
  const float s32 = fminf(amax / 127.0f, 65504.0f);
  const _Float16 s16 = (_Float16)s32;
  if (t == 0) sx[m] = __builtin_bit_cast(uint16_t, s16);
  const float sf = (float)s16;
  const float inv = group_inv(sf);
  const float* src = xf + (size_t)m * KL;
  uint8_t* dst = x8 + (size_t)m * KL;
  for (int b = t; b < KL / 32; b += 256) {                  // one 32-channel block per thread
    uint32_t w[8];                                           // 16 even channels, then 16 odd
#pragma unroll
    for (int k = 0; k < 8; k++) w[k] = 0;
#pragma unroll
    for (int q = 0; q < 8; q++) {
      const float4 v = *(const float4*)(src + b * 32 + 4 * q);
      const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; e++) {
        float c = rintf(vv[e] * inv);
        c = fminf(fmaxf(c, -127.0f), 127.0f);
        const int qi = (int)c;
        const uint32_t byte = (uint32_t)(qi < 0 ? (0x80 - qi) : qi) & 0xFFu;   // sign-magnitude
        const int ch = 4 * q + e, pos = (ch & 1) * 16 + (ch >> 1);
        w[pos >> 2] |= byte << (8 * (pos & 3));
      }
    }
    *(uint4*)(dst + b * 32) = make_uint4(w[0], w[1], w[2], w[3]);
    *(uint4*)(dst + b * 32 + 16) = make_uint4(w[4], w[5], w[6], w[7]);
  }
}

int launch_quantize_tokens(const float* xf, const float* pmax, int M, int KL, uint8_t* x8, uint16_t* sx,
                           hipStream_t s) {
  hipLaunchKernelGGL(quantize_tokens_kernel, dim3(M), dim3(256), 0, s, xf, pmax, M, KL, x8, sx);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

// ---- GEMM ----------------------------------------------------------------------------------
constexpr int BK8 = 64;                               // channels per LDS stage
constexpr int W_BYTES = TN * 64;                      // weights: [128 rows][64 B]
constexpr int T_BYTES = TM * 128;                     // activations: [128 rows][a-plane 64 B | b-plane 64 B]
constexpr int STAGE8 = W_BYTES + T_BYTES;             // 24 KB
constexpr int SCALE8_OFF = 2 * STAGE8;                // u64 [2 bufs][groups per stage][128 rows]: {fp16 s_w, 0, 0, 0}
constexpr int scale8_buf_bytes(int gs) { return (BK8 / gs) * TN * 8; }
constexpr int zero8_off(int gs) { return SCALE8_OFF + 2 * scale8_buf_bytes(gs); }
constexpr int smem8_bytes(int gs) { return zero8_off(gs) + 256; }
static_assert(2 * STAGE8 >= 32768, "the 16-bit branch reuses the stages as a [256 rows][128 B] tile");

// weights: 16-B chunk c (0..3) of 64-byte row r at slot c ^ ((r >> 2) & 3) (4 rows share a 256-byte bank line)
__device__ __forceinline__ int w_off_bytes(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4); }

// 8 sign-magnitude nibbles of a dword -> fp8 bytes [s 0000 mmm]: even channels, odd channels
__device__ __forceinline__ void unpack8_sm(uint32_t p, uint32_t& even, uint32_t& odd) {
  even = (p & 0x07070707u) | ((p & 0x08080808u) << 4);
  odd = ((p >> 4) & 0x07070707u) | (p & 0x80808080u);
}

typedef __attribute__((ext_vector_type(8))) int i32x8_t;

template <int GS, bool OUT_F32>
__global__ __launch_bounds__(NTHREADS, 2) void w4a8_gemm_kernel(
    const uint16_t* __restrict__ xh, const uint8_t* __restrict__ x8, const uint16_t* __restrict__ sx,
    const uint16_t* __restrict__ wh, const uint8_t* __restrict__ wq, const uint16_t* __restrict__ sw,
    const uint16_t* __restrict__ bias, int M, int N, int K, int r, void* __restrict__ y, int n_mt, int n_nt,
    int per_xcd, int sw_shift) {
  // GS = channels per scale application; the stored weight groups hold GS << sw_shift channels
  // (128-channel groups run as two 64-channel halves with the same scale: the same sum)
  extern __shared__ __align__(16) unsigned char smem[];
  static_assert(GS == 32 || GS == 64, "scale granularity of the 8-bit path");

  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= n_mt * n_nt) return;
  constexpr int GN = 4;
  const int grp = logical / (GN * n_mt), in_grp = logical % (GN * n_mt);
  const int gn = min(n_nt - grp * GN, GN);
  const int nt = grp * GN + in_grp % gn, mt = in_grp / gn;
  const int m0 = mt * TM, n0 = nt * TN;

  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int wn = w & 1, wt = w >> 1;
  const int h = l >> 5;
  const int KL = K - r;
  const int G = KL / GS;
  constexpr int GPS = BK8 / GS;    // groups per stage: 1 or 2
  constexpr int MPG = GS / 32;     // 32-channel MFMA steps per group: 2 or 1
  constexpr int SBUF = scale8_buf_bytes(GS), ZERO_OFF = zero8_off(GS);

  if (t < 64) ((uint32_t*)(smem + ZERO_OFF))[t] = 0u;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  // rows of this lane within the tail's [256 rows] tile: weights 0..127, tokens 128..255
  int rowA[2], rowB[2];
#pragma unroll
  for (int i = 0; i < 2; i++) rowA[i] = wn * 64 + i * 32 + (l & 31);
#pragma unroll
  for (int j = 0; j < 2; j++) rowB[j] = TN + wt * 64 + j * 32 + (l & 31);

  if (KL > 0) {
    // ---- staging: thread t owns one 16-B packed weight chunk (row t/2, 32-channel block t%2)
    // and two 16-B activation chunks (rows t/4 and t/4 + 64, chunk t%4) of every stage
    const int wrow = t >> 1, wblk = t & 1;
    const int trow = t >> 2, tchk = t & 3;
    // Loads are unconditional (straight-line code keeps the outstanding-load count exact): a chunk
    // past the end of a row (KL an odd multiple of 32) is re-read from inside the row and belongs to
    // a group >= G, whose weight scale is forced to zero, so it contributes exactly nothing.
    const int wbase = min(wblk * 16, KL / 2 - 16), wlast = KL / 2 - 16 - wbase;
    const int tbase = min(tchk * 16, KL - 16), tlast = KL - 16 - tbase;
    const uint8_t* gw = wq + (size_t)min(n0 + wrow, N - 1) * (KL / 2) + wbase;
    const uint8_t* gt[2];
#pragma unroll
    for (int i = 0; i < 2; i++) gt[i] = x8 + (size_t)min(m0 + trow + 64 * i, M - 1) * KL + tbase;
    const uint16_t* gs = sw + min(n0 + (t & 127), N - 1);        // threads 0..127 stage the weight scales
    const int nst = (KL + BK8 - 1) / BK8;
    uint4 rw, rt[2];
    uint16_t rs[GPS];
    // one stage = 4 pieces (weights, two activation rows, scales); piece p is reloaded for stage s+2 right
    // after it has been unpacked into LDS for stage s+1, so a global load has a whole stage to complete
    auto gload_piece = [&](int st, int p) {
      if (p == 0) {
        rw = *(const uint4*)(gw + min(st * (BK8 / 2), wlast));
      } else if (p < 3) {
        rt[p - 1] = *(const uint4*)(gt[p - 1] + min(st * BK8, tlast));
      } else {
#pragma unroll
        for (int jj = 0; jj < GPS; jj++) {
          const int j = st * GPS + jj;
          const uint16_t v = gs[(size_t)(min(j, G - 1) >> sw_shift) * N];
          rs[jj] = (uint16_t)(v & (j < G ? 0xFFFFu : 0u));
        }
      }
    };
    auto sstore_piece = [&](int buf, int p) {
      unsigned char* sb = smem + buf * STAGE8;
      if (p == 0) {
        uint4 e, o;
        unpack8_sm(rw.x, e.x, o.x);
        unpack8_sm(rw.y, e.y, o.y);
        unpack8_sm(rw.z, e.z, o.z);
        unpack8_sm(rw.w, e.w, o.w);
        *(uint4*)(sb + w_off_bytes(wrow, 2 * wblk)) = e;
        *(uint4*)(sb + w_off_bytes(wrow, 2 * wblk + 1)) = o;
      } else if (p < 3) {
        const int i = p - 1, row = trow + 64 * i;
        uint4 a, b;                                              // planes: [s 0000 aaa] and [s 000 bbbb]
        a.x = (rt[i].x & 0x80808080u) | ((rt[i].x >> 4) & 0x07070707u);
        a.y = (rt[i].y & 0x80808080u) | ((rt[i].y >> 4) & 0x07070707u);
        a.z = (rt[i].z & 0x80808080u) | ((rt[i].z >> 4) & 0x07070707u);
        a.w = (rt[i].w & 0x80808080u) | ((rt[i].w >> 4) & 0x07070707u);
        b.x = rt[i].x & 0x8F8F8F8Fu;
        b.y = rt[i].y & 0x8F8F8F8Fu;
        b.z = rt[i].z & 0x8F8F8F8Fu;
        b.w = rt[i].w & 0x8F8F8F8Fu;
        *(uint4*)(sb + W_BYTES + tile_off_bytes(row, tchk)) = a;
        *(uint4*)(sb + W_BYTES + tile_off_bytes(row, 4 + tchk)) = b;
      } else if (t < TN) {
        uint2* sdst = (uint2*)(smem + SCALE8_OFF + buf * SBUF);
#pragma unroll
        for (int jj = 0; jj < GPS; jj++) sdst[jj * TN + t] = make_uint2(rs[jj], 0u);
      }
    };

    // per-lane LDS addresses.  MFMA step s2 (0 or 1) of a stage covers its 32-channel block s2:
    // lane half h takes 16-byte chunk 2 s2 + h (even channels for h = 0, odd ones for h = 1) of the
    // weight row and of both activation planes (a zero magnitude with the sign bit set is fp8 -0)
    const int wswz = ((l & 31) >> 2) & 3, tswz = ((l & 31) >> 1) & 7;
    int adW[2][2], adTa[2][2], adTb[2][2];
#pragma unroll
    for (int s2 = 0; s2 < 2; s2++) {
      const int c = 2 * s2 + h;
#pragma unroll
      for (int i = 0; i < 2; i++) adW[i][s2] = (wn * 64 + i * 32 + (l & 31)) * 64 + ((c ^ wswz) << 4);
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const int row = wt * 64 + j * 32 + (l & 31);
        adTa[j][s2] = W_BYTES + row * 128 + ((c ^ tswz) << 4);
        adTb[j][s2] = W_BYTES + row * 128 + (((4 + c) ^ tswz) << 4);
      }
    }
    int soffA[2];
#pragma unroll
    for (int i = 0; i < 2; i++) soffA[i] = h ? ZERO_OFF : SCALE8_OFF + (wn * 64 + i * 32 + (l & 31)) * 8;
    const int sstep = h ? 0 : TN * 8, sbufstep = h ? 0 : SBUF;
    // the token's scale sits in k-slot 0 of the scale-product MFMA (lanes 0..31), constant over the groups
    f16x4 sxv[2];
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const uint16_t bits = h ? (uint16_t)0 : sx[min(m0 + wt * 64 + j * 32 + (l & 31), M - 1)];
      sxv[j] = f16x4{__builtin_bit_cast(_Float16, bits), (_Float16)0, (_Float16)0, (_Float16)0};
    }
    const int scale_b = h ? 127 : 131;    // E8M0: k-block 0 (the a-plane, lanes 0..31 hold its scale) x 2^4
    const int scale_a = 127;

#pragma unroll
    for (int p = 0; p < 4; p++) gload_piece(0, p);
#pragma unroll
    for (int p = 0; p < 4; p++) {
      sstore_piece(0, p);
      gload_piece(min(1, nst - 1), p);
    }
    __syncthreads();
    for (int st = 0; st < nst; st++) {
      const int buf = st & 1;
      const int st2 = min(st + 2, nst - 1);     // past the end: harmless re-load, never used
      const unsigned char* sb = smem + buf * STAGE8;
      const unsigned char* ssb = smem + buf * sbufstep;
      f32x16 I[2], P[2];
      i32x4 aw[2][MPG], ta[2][MPG], tb[2][MPG];
      f16x4 sa[2];
      auto load_ops = [&](int jj) {
#pragma unroll
        for (int kk = 0; kk < MPG; kk++) {
          const int s2 = jj * MPG + kk;
#pragma unroll
          for (int i = 0; i < 2; i++) aw[i][kk] = *(const i32x4*)(sb + adW[i][s2]);
#pragma unroll
          for (int j = 0; j < 2; j++) {
            ta[j][kk] = *(const i32x4*)(sb + adTa[j][s2]);
            tb[j][kk] = *(const i32x4*)(sb + adTb[j][s2]);
          }
        }
#pragma unroll
        for (int i = 0; i < 2; i++) sa[i] = *(const f16x4*)(ssb + soffA[i] + jj * sstep);
      };
      auto issue = [&](int i, int j, int slot) {
        f32x16 z, p;
#pragma unroll
        for (int v = 0; v < 16; v++) z[v] = p[v] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < MPG; kk++) {
          const i32x8_t a = __builtin_shufflevector(aw[i][kk], aw[i][kk], 0, 1, 2, 3, 4, 5, 6, 7);
          const i32x8_t b = __builtin_shufflevector(ta[j][kk], tb[j][kk], 0, 1, 2, 3, 4, 5, 6, 7);
          z = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, z, 0, 0, 0, scale_a, 0, scale_b);
          if (kk == 0) P[slot] = __builtin_amdgcn_mfma_f32_32x32x8f16(sa[i], sxv[j], p, 0, 0, 0);
        }
        I[slot] = z;
      };
      auto sweep = [&](int i, int j, int slot) {
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] = fmaf(I[slot][v], P[slot][v], acc[i][j][v]);
        asm volatile("" : "+v"(acc[i][j]));
      };
      // the next stage's unpack work is spread over the tile sweeps of this stage
      constexpr int NSTEP = GPS * 4;
      auto stage_piece = [&](int step) {
        if ((step + 1) % (NSTEP / 4) == 0) {
          const int p = (step + 1) / (NSTEP / 4) - 1;
          sstore_piece(buf ^ 1, p);
          gload_piece(st2, p);
        }
      };
      // one pipeline step = the MFMAs of the next tile interleaved with the fma sweep of the current one
      auto interleave = [&](bool valu_first) {
        constexpr int NM = MPG + 1, PER = 16 / NM;
        if (valu_first) __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);
#pragma unroll
        for (int q = 0; q < NM; q++) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);    // PER VALU instructions
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      load_ops(0);
      issue(0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jj = 0; jj < GPS; jj++) {
        const bool more = jj + 1 < GPS;
        issue(0, 1, 1);
        sweep(0, 0, 0);
        stage_piece(jj * 4 + 0);
        interleave(false);
        issue(1, 0, 0);
        sweep(0, 1, 1);
        stage_piece(jj * 4 + 1);
        interleave(false);
        issue(1, 1, 1);
        sweep(1, 0, 0);
        stage_piece(jj * 4 + 2);
        interleave(false);
        asm volatile("" ::: "memory");
        if (more) {
          load_ops(jj + 1);
          __builtin_amdgcn_sched_barrier(0);
          issue(0, 0, 0);
        }
        sweep(1, 1, 1);
        stage_piece(jj * 4 + 3);
        interleave(true);
      }
      __syncthreads();
    }
    // undo the two 2^-9 operand factors (exact power of two)
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] *= 262144.0f;
  }

  gemm_tail<OUT_F32>(acc, smem, xh, wh, bias, y, M, N, r, m0, n0, rowA, rowB);
}

template <int GS, bool OUT_F32>
static int launch_one8(const uint16_t* xh, const uint8_t* x8, const uint16_t* sx, const void* blob,
                       const uint16_t* bias, int M, int N, int K, int r, int g, void* y, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, g);
  const int sw_shift = g == 2 * GS ? 1 : 0;
  const char* bp = (const char*)blob;
  const int n_mt = (M + TM - 1) / TM, n_nt = (N + TN - 1) / TN;
  const long n_blocks = (long)n_mt * n_nt;
  const int per_xcd = (int)((n_blocks + 7) / 8);
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)w4a8_gemm_kernel<GS, OUT_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem8_bytes(GS));
    if (e != hipSuccess) return hip_failed(e);
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((w4a8_gemm_kernel<GS, OUT_F32>), dim3(per_xcd * 8), dim3(NTHREADS), smem8_bytes(GS), s, xh, x8,
                     sx, (const uint16_t*)(bp + L.off_wh), (const uint8_t*)(bp + L.off_codes),
                     (const uint16_t*)(bp + L.off_sw), bias, M, N, K, r, y, n_mt, n_nt, per_xcd, sw_shift);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

int launch_w4a8_gemm(const uint16_t* xh, const uint8_t* x8, const uint16_t* sx, const void* blob,
                     const uint16_t* bias, int M, int N, int K, int r, int g, void* y, int y_dtype,
                     hipStream_t s) {
  if (g == 32)
    return y_dtype ? launch_one8<32, true>(xh, x8, sx, blob, bias, M, N, K, r, g, y, s)
                   : launch_one8<32, false>(xh, x8, sx, blob, bias, M, N, K, r, g, y, s);
  if (g == 64 || g == 128)
    return y_dtype ? launch_one8<64, true>(xh, x8, sx, blob, bias, M, N, K, r, g, y, s)
                   : launch_one8<64, false>(xh, x8, sx, blob, bias, M, N, K, r, g, y, s);
  return DIROTQ_ERR_UNSUPPORTED;
}

}  // namespace dirotq
