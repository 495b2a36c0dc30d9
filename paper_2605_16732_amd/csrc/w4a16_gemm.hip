// W4A16 layers: 16-bit activations against 4-bit per-group weights, no rotation (the paper's
// appendix on quantization details keeps the input activations of some layers in 16 bits):
//   y[m,n] = sum_j s_w[n,j] * sum_{k in group j} x[m,k] q_w[n,k]   (+ bias[n]).
//
// A 4-bit code is a small integer and therefore an exact bf16 number, so the group sums run on
// the bf16 matrix pipe with nothing rounded before the fp32 accumulator; the per-group weight
// scale is applied afterwards, as in the W4A4 kernel: one fp16 MFMA spreads s_w[n,j] over the
// accumulator layout (token operand = 1), one fma per accumulator and group applies it.
//
// Codes become bf16 on their way into LDS (once per workgroup): the sign-magnitude nibble
// [s mmm] indexes an 8-entry byte table through v_perm_b32 (high and low byte of bf16(m)), the
// sign moves to bit 15, and two more rounds of byte permutes restore the channel order.
//
// Tile 128 n x 128 tokens, 4 waves as 2 x 2, stage = 64 channels as a [256 rows][128 B] tile
// (weights rows 0..127, tokens 128..255), two stages in LDS, global loads one stage ahead
// through registers.
#include <atomic>

#include "gemm_tail.h"

namespace dirotq {

constexpr int BK16 = 64;                               // channels per LDS stage
constexpr int STAGE16 = (TN + TM) * 128;               // 32 KB
constexpr int SCALE16_OFF = 2 * STAGE16;               // u64 [2 bufs][groups per stage][128 rows]: {fp16 s_w, 0, 0, 0}
constexpr int scale16_buf_bytes(int gs) { return (BK16 / gs) * TN * 8; }
constexpr int zero16_off(int gs) { return SCALE16_OFF + 2 * scale16_buf_bytes(gs); }
constexpr int smem16_bytes(int gs) { return zero16_off(gs) + 256; }

// 8 sign-magnitude nibbles (channels c0..c7, c0 lowest) -> 8 bf16 numbers in channel order
__device__ __forceinline__ uint4 nibbles_to_bf16(uint32_t p) {
  const uint32_t sel_e = p & 0x07070707u, sel_o = (p >> 4) & 0x07070707u;   // magnitudes of c0 c2 c4 c6 / c1 c3 c5 c7
  // bf16(m), m = 0..7: 0000 3F80 4000 4040 4080 40A0 40C0 40E0 (selectors 0..3 read the second operand)
  const uint32_t lo_e = __builtin_amdgcn_perm(0xE0C0A080u, 0x40008000u, sel_e);
  const uint32_t lo_o = __builtin_amdgcn_perm(0xE0C0A080u, 0x40008000u, sel_o);
  uint32_t hi_e = __builtin_amdgcn_perm(0x40404040u, 0x40403F00u, sel_e);
  uint32_t hi_o = __builtin_amdgcn_perm(0x40404040u, 0x40403F00u, sel_o);
  hi_e |= (p & 0x08080808u) << 4;                                            // sign -> bit 7 of the high byte
  hi_o |= p & 0x80808080u;
  const uint32_t e01 = __builtin_amdgcn_perm(hi_e, lo_e, 0x05010400u);        // bf16(c0), bf16(c2)
  const uint32_t e23 = __builtin_amdgcn_perm(hi_e, lo_e, 0x07030602u);        // c4, c6
  const uint32_t o01 = __builtin_amdgcn_perm(hi_o, lo_o, 0x05010400u);        // c1, c3
  const uint32_t o23 = __builtin_amdgcn_perm(hi_o, lo_o, 0x07030602u);        // c5, c7
  uint4 r;
  r.x = __builtin_amdgcn_perm(o01, e01, 0x05040100u);                         // c0, c1
  r.y = __builtin_amdgcn_perm(o01, e01, 0x07060302u);                         // c2, c3
  r.z = __builtin_amdgcn_perm(o23, e23, 0x05040100u);                         // c4, c5
  r.w = __builtin_amdgcn_perm(o23, e23, 0x07060302u);                         // c6, c7
  return r;
}

template <int GS, bool OUT_F32>
__global__ __launch_bounds__(NTHREADS, 2) void w4a16_gemm_kernel(
    const uint16_t* __restrict__ x, const uint8_t* __restrict__ wq, const uint16_t* __restrict__ sw,
    const uint16_t* __restrict__ bias, int M, int N, int K, void* __restrict__ y, int n_mt, int n_nt, int per_xcd,
    int sw_shift) {
  // GS = channels per scale application; the stored weight groups hold GS << sw_shift channels
  // (128-channel groups run as two 64-channel halves with the same scale: the same sum)
  extern __shared__ __align__(16) unsigned char smem[];
  static_assert(GS == 32 || GS == 64, "scale granularity");

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
  const int G = K / GS;
  constexpr int GPS = BK16 / GS;   // groups per stage: 1 or 2
  constexpr int KPG = GS / 16;     // 16-channel MFMA steps per group: 4 or 2
  constexpr int SBUF = scale16_buf_bytes(GS), ZERO_OFF = zero16_off(GS);

  if (t < 64) ((uint32_t*)(smem + ZERO_OFF))[t] = 0u;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  int rowA[2], rowB[2];
#pragma unroll
  for (int i = 0; i < 2; i++) rowA[i] = wn * 64 + i * 32 + (l & 31);
#pragma unroll
  for (int j = 0; j < 2; j++) rowB[j] = TN + wt * 64 + j * 32 + (l & 31);
  const int swz = ((l & 31) >> 1) & 7;

  // ---- staging: thread t owns one 16-B packed weight chunk (row t/2, 32-channel half t%2) and four
  // 16-B activation chunks (token rows t/8 + 32 i, chunk t%8) of every stage.
  // Loads are unconditional: a chunk past the end of a row (K an odd multiple of 32) is re-read from
  // inside the row and belongs to a group >= G, whose weight scale is forced to zero.
  const int wrow = t >> 1, whalf = t & 1;
  const int xrow = t >> 3, xchk = t & 7;
  const int wbase = min(whalf * 16, K / 2 - 16), wlast = K / 2 - 16 - wbase;        // bytes
  const int xbase = min(xchk * 8, K - 8), xlast = K - 8 - xbase;                    // bf16 elements
  const uint8_t* gw = wq + (size_t)min(n0 + wrow, N - 1) * (K / 2) + wbase;
  const uint16_t* gx[4];
#pragma unroll
  for (int i = 0; i < 4; i++) gx[i] = x + (size_t)min(m0 + xrow + 32 * i, M - 1) * K + xbase;
  const uint16_t* gs = sw + min(n0 + (t & 127), N - 1);        // threads 0..127 stage the weight scales
  const int nst = (K + BK16 - 1) / BK16;
  uint4 rw;
  i32x4 rx[4];                        // (a native vector type: an array of it stays in registers)
  uint16_t rs[GPS];
  auto gload = [&](int st) {
    rw = *(const uint4*)(gw + min(st * (BK16 / 2), wlast));
#pragma unroll
    for (int i = 0; i < 4; i++) rx[i] = *(const i32x4*)(gx[i] + min(st * BK16, xlast));
#pragma unroll
    for (int jj = 0; jj < GPS; jj++) {
      const int j = st * GPS + jj;
      const uint16_t v = gs[(size_t)(min(j, G - 1) >> sw_shift) * N];
      rs[jj] = (uint16_t)(v & (j < G ? 0xFFFFu : 0u));
    }
  };
  auto sstore = [&](int buf) {
    unsigned char* sb = smem + buf * STAGE16;
    *(uint4*)(sb + tile_off_bytes(wrow, 4 * whalf + 0)) = nibbles_to_bf16(rw.x);
    *(uint4*)(sb + tile_off_bytes(wrow, 4 * whalf + 1)) = nibbles_to_bf16(rw.y);
    *(uint4*)(sb + tile_off_bytes(wrow, 4 * whalf + 2)) = nibbles_to_bf16(rw.z);
    *(uint4*)(sb + tile_off_bytes(wrow, 4 * whalf + 3)) = nibbles_to_bf16(rw.w);
#pragma unroll
    for (int i = 0; i < 4; i++) *(i32x4*)(sb + tile_off_bytes(TN + xrow + 32 * i, xchk)) = rx[i];
    if (t < TN) {
      uint2* sdst = (uint2*)(smem + SCALE16_OFF + buf * SBUF);
#pragma unroll
      for (int jj = 0; jj < GPS; jj++) sdst[jj * TN + t] = make_uint2(rs[jj], 0u);
    }
  };

  // per-lane LDS addresses: 16-channel step k (0..3) of a stage reads chunk 2k + h of the row
  int adA[2][4], adB[2][4];
#pragma unroll
  for (int k = 0; k < 4; k++) {
    const int off = ((2 * k + h) ^ swz) << 4;
#pragma unroll
    for (int i = 0; i < 2; i++) adA[i][k] = rowA[i] * 128 + off;
#pragma unroll
    for (int j = 0; j < 2; j++) adB[j][k] = rowB[j] * 128 + off;
  }
  int soffA[2];
#pragma unroll
  for (int i = 0; i < 2; i++) soffA[i] = h ? ZERO_OFF : SCALE16_OFF + rowA[i] * 8;
  const int sstep = h ? 0 : TN * 8, sbufstep = h ? 0 : SBUF;
  // token operand of the scale MFMA: 1 in k-slot 0 (lanes 0..31), zeros elsewhere
  const f16x4 ones = f16x4{h ? (_Float16)0 : (_Float16)1, (_Float16)0, (_Float16)0, (_Float16)0};

  gload(0);
  sstore(0);
  gload(min(1, nst - 1));
  __syncthreads();
  for (int st = 0; st < nst; st++) {
    const int buf = st & 1;
    const unsigned char* sb = smem + buf * STAGE16;
    const unsigned char* ssb = smem + buf * sbufstep;
    f32x16 I[2], P[2];
    bf16x8 a[2][KPG], b[2][KPG];
    f16x4 sa[2];
    auto load_ops = [&](int jj) {
#pragma unroll
      for (int kk = 0; kk < KPG; kk++) {
#pragma unroll
        for (int i = 0; i < 2; i++) a[i][kk] = *(const bf16x8*)(sb + adA[i][jj * KPG + kk]);
#pragma unroll
        for (int j = 0; j < 2; j++) b[j][kk] = *(const bf16x8*)(sb + adB[j][jj * KPG + kk]);
      }
#pragma unroll
      for (int i = 0; i < 2; i++) sa[i] = *(const f16x4*)(ssb + soffA[i] + jj * sstep);
    };
    auto issue = [&](int i, int j, int slot) {
      f32x16 z, p;
#pragma unroll
      for (int v = 0; v < 16; v++) z[v] = p[v] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < KPG; kk++) {
        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i][kk], b[j][kk], z, 0, 0, 0);
        if (kk == 0) P[slot] = __builtin_amdgcn_mfma_f32_32x32x8f16(sa[i], ones, p, 0, 0, 0);
      }
      I[slot] = z;
    };
    auto sweep = [&](int i, int j, int slot) {
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = fmaf(I[slot][v], P[slot][v], acc[i][j][v]);
      asm volatile("" : "+v"(acc[i][j]));
    };
    load_ops(0);
    issue(0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int jj = 0; jj < GPS; jj++) {
      issue(0, 1, 1);
      sweep(0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      issue(1, 0, 0);
      sweep(0, 1, 1);
      __builtin_amdgcn_sched_barrier(0);
      issue(1, 1, 1);
      sweep(1, 0, 0);
      if (jj == GPS - 1) {                      // the next stage: registers -> LDS, then reload for stage st + 2
        sstore(buf ^ 1);
        gload(min(st + 2, nst - 1));
      }
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("" ::: "memory");
      if (jj + 1 < GPS) {
        load_ops(jj + 1);
        __builtin_amdgcn_sched_barrier(0);
        issue(0, 0, 0);
      }
      sweep(1, 1, 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  }

  gemm_tail<OUT_F32>(acc, smem, nullptr, nullptr, bias, y, M, N, 0, m0, n0, rowA, rowB);
}


// ---- few tokens (M <= 32): every weight is used once, so the kernel is a stream over the packed
// weights (HBM-bound) and skips LDS for the operands.  One workgroup = 32 output channels; its NW waves
// split the K axis into NW contiguous runs of scale groups and add their partial sums through LDS in a
// fixed order.
// Orientation D[token][n]: the activations are the row operand (tokens padded to 32 by re-reading the
// last one), a lane owns one output channel, so the group's weight scale is a per-lane scalar.
// Lane half h holds channels [h GS/2, (h + 1) GS/2) of the group: GS/2 bytes of codes, one load.
template <int GS, bool OUT_F32, int NW>
__global__ __launch_bounds__(NW * 64) void w4a16_skinny_kernel(
    const uint16_t* __restrict__ x, const uint8_t* __restrict__ wq, const uint16_t* __restrict__ sw,
    const uint16_t* __restrict__ bias, int M, int N, int K, void* __restrict__ y, int sw_shift) {
  static_assert(GS == 32 || GS == 64, "scale granularity");
  constexpr int STEPS = GS / 16;          // MFMA steps (16 channels over the lane pair) per group
  constexpr int CW = STEPS;               // code dwords per lane and group
  static_assert(NW == 4 || NW == 8, "waves per workgroup");
  __shared__ float red[NW][16][64];
  const int t = threadIdx.x, l = t & 63, w = t >> 6, h = l >> 5, c = l & 31;
  const int n = blockIdx.x * 32 + c, nc = min(n, N - 1);
  const int mrow = min(c, M - 1);
  const int nkb = K / GS;
  const uint8_t* gw = wq + (size_t)nc * (K / 2) + h * (GS / 4);
  const uint16_t* gx = x + (size_t)mrow * K + h * (GS / 2);
  const uint16_t* gs = sw + nc;

  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; v++) acc[v] = 0.0f;

  // A ring of DEPTH group fetches per wave keeps enough bytes in flight to cover the memory latency
  // (one wave per SIMD is typical for these launches).  The loop is branch-free: a fetch past the end
  // re-reads the last group and its scale is replaced by zero.
  constexpr int DEPTH = 4;
  uint32_t cw[DEPTH][CW];
  bf16x8 xa[DEPTH][STEPS];
  uint32_t sc[DEPTH];                      // raw scale bits: nothing is computed on a load until it is used
  // wave w owns the contiguous run of groups [kb0, kb1): it walks along its 32 weight rows
  const int per = (nkb + NW - 1) / NW, kb0 = w * per, kb1 = min(kb0 + per, nkb);
  auto fetch = [&](int u, int kb_raw) {
    const int kb = min(kb_raw, nkb - 1);
    if constexpr (CW == 4) {
      const uint4 v = *(const uint4*)(gw + (size_t)kb * (GS / 2));
      cw[u][0] = v.x, cw[u][1] = v.y, cw[u][2] = v.z, cw[u][3] = v.w;
    } else {
      const uint2 v = *(const uint2*)(gw + (size_t)kb * (GS / 2));
      cw[u][0] = v.x, cw[u][1] = v.y;
    }
#pragma unroll
    for (int s2 = 0; s2 < STEPS; s2++) xa[u][s2] = *(const bf16x8*)(gx + (size_t)kb * GS + 8 * s2);
    sc[u] = gs[(size_t)(kb >> sw_shift) * N];
  };
  auto block = [&](int u, bool live) {
    f32x16 z;
#pragma unroll
    for (int v = 0; v < 16; v++) z[v] = 0.0f;
#pragma unroll
    for (int s2 = 0; s2 < STEPS; s2++) {
      const uint4 wv = nibbles_to_bf16(cw[u][s2]);
      z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[u][s2], __builtin_bit_cast(bf16x8, wv), z, 0, 0, 0);
    }
    const float sf = f16_bits_to_f32((uint16_t)(live ? sc[u] : 0u));
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] = fmaf(z[v], sf, acc[v]);
  };
  // (the scheduling fences keep each refill where it is written: right after the group it replaces)
#pragma unroll
  for (int d = 0; d < DEPTH; d++) {
    fetch(d, kb0 + d);
    __builtin_amdgcn_sched_barrier(0);
  }
  for (int kb = kb0; kb < kb1; kb += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; d++) {
      block(d, kb + d < kb1);
      __builtin_amdgcn_sched_barrier(0);
      fetch(d, kb + d + DEPTH);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int v = 0; v < 16; v++) red[w][v][l] = acc[v];
  __syncthreads();
  // wave w finishes 16 / NW accumulator registers (register v holds token 8 (v / 4) + 4 h + v % 4);
  // partial sums are added in wave order
  if (n < N) {
    const float b = bias ? bf16_bits_to_f32(bias[n]) : 0.0f;
    constexpr int RPW = 16 / NW;
#pragma unroll
    for (int e = 0; e < RPW; e++) {
      const int v = RPW * w + e, m = 8 * (v >> 2) + 4 * h + (v & 3);
      if (m < M) {
        float r = red[0][v][l];
#pragma unroll
        for (int p = 1; p < NW; p++) r += red[p][v][l];
        r += b;
        if (OUT_F32) ((float*)y)[(size_t)m * N + n] = r;
        else ((uint16_t*)y)[(size_t)m * N + n] = f32_to_bf16_bits(r);
      }
    }
  }
}


// ---- very few tokens (M <= 8): the same stream over the weights with the loads fully coalesced.
// One workgroup (8 waves) = 32 output channels.  K is walked in chunks of 1024 channels: the chunk's codes
// (32 rows x 512 B), activations (M rows x 2 KB) and scales go through registers into one of two LDS
// buffers, every thread loading consecutive 16-byte pieces of a row, while the waves multiply the
// previous chunk (wave w takes scale groups w, w + 8, ...).  LDS rows are padded by 16 bytes so that
// the 32 lanes of an operand read hit different banks.  Within each run of 8 channels both operands
// are kept in the order c0 c2 c4 c6 c1 c3 c5 c7 (the activations are permuted once when they are
// staged), which saves the last round of byte permutes of the weight decode.
constexpr int FEW_KC = 1024;                     // channels per chunk
constexpr int FEW_WROW = FEW_KC / 2 + 16;        // bytes per LDS row of codes
constexpr int FEW_XROW = FEW_KC * 2 + 16;        // bytes per LDS row of activations
constexpr int FEW_CODES_B = 32 * FEW_WROW;
constexpr int FEW_X_B = 8 * FEW_XROW;
constexpr int few_buf_bytes(int gs) { return FEW_CODES_B + FEW_X_B + (FEW_KC / gs) * 32 * 2; }

// 8 sign-magnitude nibbles -> bf16 in the order c0 c2 c4 c6 c1 c3 c5 c7
__device__ __forceinline__ uint4 nibbles_to_bf16_eo(uint32_t p) {
  const uint32_t sel_e = p & 0x07070707u, sel_o = (p >> 4) & 0x07070707u;
  const uint32_t lo_e = __builtin_amdgcn_perm(0xE0C0A080u, 0x40008000u, sel_e);
  const uint32_t lo_o = __builtin_amdgcn_perm(0xE0C0A080u, 0x40008000u, sel_o);
  uint32_t hi_e = __builtin_amdgcn_perm(0x40404040u, 0x40403F00u, sel_e);
  uint32_t hi_o = __builtin_amdgcn_perm(0x40404040u, 0x40403F00u, sel_o);
  hi_e |= (p & 0x08080808u) << 4;
  hi_o |= p & 0x80808080u;
  uint4 r;
  r.x = __builtin_amdgcn_perm(hi_e, lo_e, 0x05010400u);   // c0, c2
  r.y = __builtin_amdgcn_perm(hi_e, lo_e, 0x07030602u);   // c4, c6
  r.z = __builtin_amdgcn_perm(hi_o, lo_o, 0x05010400u);   // c1, c3
  r.w = __builtin_amdgcn_perm(hi_o, lo_o, 0x07030602u);   // c5, c7
  return r;
}

template <int GS, bool OUT_F32>
__global__ __launch_bounds__(512) void w4a16_few_kernel(
    const uint16_t* __restrict__ x, const uint8_t* __restrict__ wq, const uint16_t* __restrict__ sw,
    const uint16_t* __restrict__ bias, int M, int N, int K, void* __restrict__ y, int sw_shift) {
  static_assert(GS == 32 || GS == 64, "scale granularity");
  constexpr int STEPS = GS / 16, GPC = FEW_KC / GS, BUF = few_buf_bytes(GS);
  extern __shared__ __align__(16) unsigned char smem[];
  const int t = threadIdx.x, l = t & 63, w = t >> 6, h = l >> 5, c = l & 31;
  const int n0 = blockIdx.x * 32, n = n0 + c;
  const int mrow = min(c, M - 1);
  const int nch = (K + FEW_KC - 1) / FEW_KC;

  // staging roles of this thread within a chunk
  const int crow = t >> 5, cpiece = t & 31;              // codes: rows crow and crow + 16, 16-byte piece cpiece
  const uint8_t* gc[2];
#pragma unroll
  for (int i = 0; i < 2; i++) gc[i] = wq + (size_t)min(n0 + crow + 16 * i, N - 1) * (K / 2) + cpiece * 16;
  const int xrow[2] = {t >> 7, (t >> 7) + 4};            // activations: token rows t / 128 and t / 128 + 4
  const int xpiece = t & 127;
  const uint16_t* gx[2];
#pragma unroll
  for (int i = 0; i < 2; i++) gx[i] = x + (size_t)min(xrow[i], M - 1) * K + xpiece * 8;
  constexpr int SPT = GPC / 16;                          // scales per thread: groups t / 32 (+ 16), channel t % 32
  const int sgrp = t >> 5;
  const uint16_t* gsc = sw + min(n0 + (t & 31), N - 1);

  uint4 rc[2], rx[2];
  uint32_t rs[SPT] = {};
  auto gload = [&](int ch) {
    const int k0 = ch * FEW_KC;
    const bool cok = k0 + cpiece * 32 < K, xok = k0 + xpiece * 8 < K;
#pragma unroll
    for (int i = 0; i < 2; i++) {
      rc[i] = cok ? *(const uint4*)(gc[i] + k0 / 2) : make_uint4(0, 0, 0, 0);
      rx[i] = (xok && xrow[i] < M) ? *(const uint4*)(gx[i] + k0) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < SPT; i++) {
      const int j = ch * GPC + sgrp + 16 * i;
      if (j < K / GS) rs[i] = gsc[(size_t)(j >> sw_shift) * N];
    }
  };
  auto sstore = [&](int buf) {
    unsigned char* sb = smem + buf * BUF;
#pragma unroll
    for (int i = 0; i < 2; i++) {
      *(uint4*)(sb + (crow + 16 * i) * FEW_WROW + cpiece * 16) = rc[i];
      uint4 v;                                            // c0c1 c2c3 c4c5 c6c7 -> c0c2 c4c6 c1c3 c5c7
      v.x = __builtin_amdgcn_perm(rx[i].y, rx[i].x, 0x05040100u);
      v.y = __builtin_amdgcn_perm(rx[i].w, rx[i].z, 0x05040100u);
      v.z = __builtin_amdgcn_perm(rx[i].y, rx[i].x, 0x07060302u);
      v.w = __builtin_amdgcn_perm(rx[i].w, rx[i].z, 0x07060302u);
      *(uint4*)(sb + FEW_CODES_B + xrow[i] * FEW_XROW + xpiece * 16) = v;
    }
#pragma unroll
    for (int i = 0; i < SPT; i++)
      ((uint16_t*)(sb + FEW_CODES_B + FEW_X_B))[(sgrp + 16 * i) * 32 + (t & 31)] = (uint16_t)rs[i];
  };

  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; v++) acc[v] = 0.0f;

  gload(0);
  sstore(0);
  __syncthreads();
  for (int ch = 0; ch < nch; ch++) {
    const bool more = ch + 1 < nch;
    if (more) gload(ch + 1);                              // in flight while this chunk is multiplied
    const unsigned char* sb = smem + (ch & 1) * BUF;
    const int groups = min(GPC, (K - ch * FEW_KC) / GS);
    for (int gi = w; gi < groups; gi += 8) {
      uint32_t cw[STEPS];
      if constexpr (GS == 64) {
        const uint4 v = *(const uint4*)(sb + c * FEW_WROW + gi * 32 + h * 16);
        cw[0] = v.x, cw[1] = v.y, cw[2] = v.z, cw[3] = v.w;
      } else {
        const uint2 v = *(const uint2*)(sb + c * FEW_WROW + gi * 16 + h * 8);
        cw[0] = v.x, cw[1] = v.y;
      }
      const unsigned char* xs = sb + FEW_CODES_B + mrow * FEW_XROW + (gi * GS + h * (GS / 2)) * 2;
      f32x16 z;
#pragma unroll
      for (int v = 0; v < 16; v++) z[v] = 0.0f;
#pragma unroll
      for (int s2 = 0; s2 < STEPS; s2++) {
        const bf16x8 xa = *(const bf16x8*)(xs + s2 * 16);
        const uint4 wv = nibbles_to_bf16_eo(cw[s2]);
        z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, __builtin_bit_cast(bf16x8, wv), z, 0, 0, 0);
      }
      const float sf = f16_bits_to_f32(((const uint16_t*)(sb + FEW_CODES_B + FEW_X_B))[gi * 32 + c]);
      // tokens 0..7 live in accumulator registers 0..3 (token 4 h + v); the others are padding
#pragma unroll
      for (int v = 0; v < 4; v++) acc[v] = fmaf(z[v], sf, acc[v]);
    }
    if (more) sstore((ch + 1) & 1);
    __syncthreads();
  }
  // partial sums of the 8 waves, added in wave order: red[wave][register][lane]
  float* red = (float*)smem;
#pragma unroll
  for (int v = 0; v < 4; v++) red[(w * 4 + v) * 64 + l] = acc[v];
  __syncthreads();
  if (w < 4 && n < N) {
    const int m = 4 * h + w;
    if (m < M) {
      float r = red[w * 64 + l];
#pragma unroll
      for (int p2 = 1; p2 < 8; p2++) r += red[(p2 * 4 + w) * 64 + l];
      if (bias) r += bf16_bits_to_f32(bias[n]);
      if (OUT_F32) ((float*)y)[(size_t)m * N + n] = r;
      else ((uint16_t*)y)[(size_t)m * N + n] = f32_to_bf16_bits(r);
    }
  }
}

template <int GS, bool OUT_F32>
static int launch_few16(const uint16_t* x, const void* blob, const uint16_t* bias, int M, int N, int K, int g, void* y,
                        hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, 0, g);
  const char* bp = (const char*)blob;
  constexpr int SMEM = 2 * few_buf_bytes(GS);
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)w4a16_few_kernel<GS, OUT_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return hip_failed(e);
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((w4a16_few_kernel<GS, OUT_F32>), dim3((N + 31) / 32), dim3(512), SMEM, s, x,
                     (const uint8_t*)(bp + L.off_codes), (const uint16_t*)(bp + L.off_sw), bias, M, N, K, y,
                     g == 2 * GS ? 1 : 0);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

template <int GS, bool OUT_F32>
static int launch_skinny16(const uint16_t* x, const void* blob, const uint16_t* bias, int M, int N, int K, int g,
                           void* y, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, 0, g);
  const char* bp = (const char*)blob;
  const uint8_t* wq = (const uint8_t*)(bp + L.off_codes);
  const uint16_t* sw = (const uint16_t*)(bp + L.off_sw);
  const int sw_shift = g == 2 * GS ? 1 : 0;
  // 8 waves per workgroup when there are few workgroups and enough scale groups to split further
  if (K / GS >= 16 && (N + 31) / 32 < 256)
    hipLaunchKernelGGL((w4a16_skinny_kernel<GS, OUT_F32, 8>), dim3((N + 31) / 32), dim3(512), 0, s, x, wq, sw, bias, M,
                       N, K, y, sw_shift);
  else
    hipLaunchKernelGGL((w4a16_skinny_kernel<GS, OUT_F32, 4>), dim3((N + 31) / 32), dim3(256), 0, s, x, wq, sw, bias, M,
                       N, K, y, sw_shift);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

template <int GS, bool OUT_F32>
static int launch_one16(const uint16_t* x, const void* blob, const uint16_t* bias, int M, int N, int K, int g, void* y,
                        hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, 0, g);
  const int sw_shift = g == 2 * GS ? 1 : 0;
  const char* bp = (const char*)blob;
  const int n_mt = (M + TM - 1) / TM, n_nt = (N + TN - 1) / TN;
  const long n_blocks = (long)n_mt * n_nt;
  const int per_xcd = (int)((n_blocks + 7) / 8);
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)w4a16_gemm_kernel<GS, OUT_F32>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem16_bytes(GS));
    if (e != hipSuccess) return hip_failed(e);
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((w4a16_gemm_kernel<GS, OUT_F32>), dim3(per_xcd * 8), dim3(NTHREADS), smem16_bytes(GS), s, x,
                     (const uint8_t*)(bp + L.off_codes), (const uint16_t*)(bp + L.off_sw), bias, M, N, K, y, n_mt, n_nt,
                     per_xcd, sw_shift);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

int launch_w4a16_gemm(const uint16_t* x, const void* blob, const uint16_t* bias, int M, int N, int K, int g, void* y,
                      int y_dtype, hipStream_t s) {
  if (M <= 8) {                       // a handful of tokens: activations fit in LDS next to the weight chunks
    if (g == 32)
      return y_dtype ? launch_few16<32, true>(x, blob, bias, M, N, K, g, y, s)
                     : launch_few16<32, false>(x, blob, bias, M, N, K, g, y, s);
    if (g == 64 || g == 128)
      return y_dtype ? launch_few16<64, true>(x, blob, bias, M, N, K, g, y, s)
                     : launch_few16<64, false>(x, blob, bias, M, N, K, g, y, s);
    return DIROTQ_ERR_UNSUPPORTED;
  }
  if (M <= 32) {                      // few tokens: the weight stream, not the matrix pipe, is the bound
    if (g == 32)
      return y_dtype ? launch_skinny16<32, true>(x, blob, bias, M, N, K, g, y, s)
                     : launch_skinny16<32, false>(x, blob, bias, M, N, K, g, y, s);
    if (g == 64 || g == 128)
      return y_dtype ? launch_skinny16<64, true>(x, blob, bias, M, N, K, g, y, s)
                     : launch_skinny16<64, false>(x, blob, bias, M, N, K, g, y, s);
    return DIROTQ_ERR_UNSUPPORTED;
  }
  if (g == 32)
    return y_dtype ? launch_one16<32, true>(x, blob, bias, M, N, K, g, y, s)
                   : launch_one16<32, false>(x, blob, bias, M, N, K, g, y, s);
  if (g == 64 || g == 128)
    return y_dtype ? launch_one16<64, true>(x, blob, bias, M, N, K, g, y, s)
                   : launch_one16<64, false>(x, blob, bias, M, N, K, g, y, s);
  return DIROTQ_ERR_UNSUPPORTED;
}

}  // namespace dirotq
