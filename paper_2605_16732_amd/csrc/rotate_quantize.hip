// Kernel A: online rotation x_hat = x Q (bf16 MFMA, fp32 accumulate) with the
// split / per-group quantize / pack fused into the GEMM epilogue (rotation/split
// equation of Section 4.2 and the quantizer of Section 3 of the paper).
//
// Orientation.  The product is computed transposed, D[channel][token] =
// sum_k Qt[channel][k] x[token][k]: both operands stream K-contiguous rows, and in the
// 32x32 MFMA accumulator layout a lane then owns ONE token and 4 consecutive rotated
// channels per register quad.  A wave computes 128 channels x 64 tokens, so every
// quantization group (32, 64 or 128 channels of one token) lives in one lane pair
// (l, l^32): the absmax is an in-lane max plus one cross-lane exchange, the codes are
// packed in registers, and nothing is staged through LDS after the main loop.
//
// Channel tiling.  Waves own 128 "virtual" channels: the bf16 part [0, r), then the 4-bit part
// [r, K) from virtual channel r_pad on, placed so that groups never straddle a wave: r_pad = r when
// r is a multiple of the group size (the wave that holds the split point then stores both kinds),
// else r rounded up to 128.
//
// Main loop.  Operand tiles are staged HBM -> registers -> LDS (two LDS stages) with an
// XOR swizzle applied on the global side, so that the 16-byte MFMA operand reads of 16
// consecutive rows are bank-conflict free.  While stage kt is multiplied, the registers
// holding stage kt+1 (loaded during stage kt-1) are written to the other LDS stage and
// refilled with stage kt+2; every store/load pair sits between MFMAs.  (On gfx950 this
// beats the direct global_load_lds path: those instructions hold up the matrix pipe of the
// issuing SIMD far longer than a register load plus an LDS store.)
#include <atomic>

#include "dirotq_internal.h"

namespace dirotq {

// KSP = 2: the workgroup holds two such sets of waves, each with LDS stages of its own, and each walks one half of
// K; the halves' accumulators are added through LDS before the epilogue (small launches: half as long a chain of
// stage latencies).
template <int WGC, int WGT, int BK, int WVT = 64, int KSP = 1>
struct RQ {
  static constexpr int WAVE_C = 128, WAVE_T = WVT;         // wave tile: channels x tokens (64, or 32 for the
                                                           // small launches: half the arithmetic per wave and stage)
  static constexpr int TC = WGC * WAVE_C, TT = WGT * WAVE_T;
  static constexpr int NW = WGC * WGT, NT = NW * KSP * 64; // waves per k-part, threads per workgroup
  static constexpr int ROWB = BK * 2;                      // bytes per LDS row
  static constexpr int CPR = ROWB / 16;                    // 16-B chunks per row
  static constexpr int STAGE_BYTES = (TC + TT) * ROWB;
  static constexpr int IPW = (TC + TT) * CPR / 64 / NW;    // 16-B loads per lane per stage
  static constexpr int KS = BK / 16;                       // MFMA k-steps per stage
  static constexpr int PP = IPW / KS;                      // store/load pairs per k-step
  static constexpr int SMEM = KSP * 2 * STAGE_BYTES;
  // register budget: two waves per SIMD unless LDS (160 KB per CU) admits only one 4-wave workgroup
  static constexpr int WAVES_PER_SIMD = (NW * KSP <= 4 && 2 * SMEM > 160 * 1024) ? 1 : 2;
  static_assert(KSP == 1 || (KSP == 2 && SMEM >= NW * 64 * (WAVE_C * WAVE_T / 64) * 4), "the second part's accumulators pass through the stage buffers");
  static_assert((TC + TT) * CPR % (64 * NW) == 0, "loads must divide evenly over waves");
  static_assert(BK == 32 || BK == 64, "BK");
  static_assert(IPW % KS == 0 && PP >= 1 && PP <= 4, "store/load pairs are spread over the 4 MFMA rows of a k-step");

  // chunk c of row `row` is stored in 16-B slot c ^ swz(row)
  // (LDS has 64 banks: a 16-byte read is served 16 lanes per cycle, so 16 consecutive rows
  // must land in 16 different 16-byte slots of a 256-byte bank line)
  // 128-byte rows (BK = 64): row&1 picks the half line, (row>>1)&7 permutes the 8 chunks;
  // 64-byte rows (BK = 32): row&3 picks the quarter line, (row>>2)&3 permutes the 4 chunks.
  __device__ static __forceinline__ int swz(int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
};

// Epilogue of a wave whose accumulators are 4 x WT tiles of 32 channels x 32 tokens (32x32 MFMA layout: a lane
// owns one token and 4 consecutive channels per register quad): the split at r, the per-group quantizer and the
// packing, all in registers.  vb: the wave's first virtual channel (the 16-bit part, then the 4-bit part from
// r_pad on); tok_base: its first token.
template <int QM, int WT>
__device__ __forceinline__ void rq_epilogue32(const f32x16 (&acc)[4][WT], int vb, int tok_base, int M, int K, int r,
                                              int g, int r_pad, int Kv, uint16_t* __restrict__ xh,
                                              uint8_t* __restrict__ xl, uint16_t* __restrict__ sx,
                                              uint16_t* __restrict__ zx, float* __restrict__ xf,
                                              float* __restrict__ pmax, int sx_ld) {
  constexpr bool ASYM = QM == 1;
  const int l = threadIdx.x & 63;
  if (vb >= Kv) return;
  const int h = l >> 5;
  if (vb < r_pad) {
    // 16-bit part: 4 consecutive channels per register quad -> one 8-byte store
#pragma unroll
    for (int j = 0; j < WT; j++) {
      const int m = tok_base + j * 32 + (l & 31);
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const int c = vb + i * 32 + 8 * q + 4 * h;
          if (c < r && m < M) {
            uint2 o;
            o.x = f32_to_bf16_bits(acc[i][j][4 * q]) | ((uint32_t)f32_to_bf16_bits(acc[i][j][4 * q + 1]) << 16);
            o.y = f32_to_bf16_bits(acc[i][j][4 * q + 2]) | ((uint32_t)f32_to_bf16_bits(acc[i][j][4 * q + 3]) << 16);
            *(uint2*)(xh + (size_t)m * r + c) = o;
          }
        }
    }
    if (vb + 128 <= r_pad) return;                          // (else the split point lies inside this wave's channels)
  }
  const int cl0 = vb - r_pad;                               // first 4-bit channel of this wave (negative: see above)
  const int KL = K - r;
  if constexpr (QM == 2) {
    // raw fp32 values (16-byte stores) and the wave tile's absolute maximum per token
#pragma unroll
    for (int j = 0; j < WT; j++) {
      const int m = tok_base + j * 32 + (l & 31);
      float a = 0.0f;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int cl = cl0 + i * 32;
        if (cl < KL) {
#pragma unroll
          for (int v = 0; v < 16; v++) a = fmaxf(a, fabsf(acc[i][j][v]));
          if (m < M) {
#pragma unroll
            for (int q = 0; q < 4; q++)
              *(float4*)(xf + (size_t)m * KL + cl + 8 * q + 4 * h) =
                  make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
          }
        }
      }
      a = fmaxf(a, __shfl_xor(a, 32));
      if (h == 0 && m < M) pmax[(size_t)(cl0 >> 7) * sx_ld + m] = a;
    }
    return;
  }
  const size_t xl_ld = (size_t)KL / 2;
  const int gi_tiles = g >> 5;                              // 32-channel MFMA tiles per group: 1, 2, 4
#pragma unroll
  for (int j = 0; j < WT; j++) {
    const int m = tok_base + j * 32 + (l & 31);
    // absmax (symmetric) or min and max (asymmetric) of each 32-channel tile over the lane
    // pair, then combined per group
    float tmax[4], tmin[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if constexpr (ASYM) {
        float lo = acc[i][j][0], hi = acc[i][j][0];
#pragma unroll
        for (int v = 1; v < 16; v++) {
          lo = fminf(lo, acc[i][j][v]);
          hi = fmaxf(hi, acc[i][j][v]);
        }
        tmin[i] = fminf(lo, __shfl_xor(lo, 32));
        tmax[i] = fmaxf(hi, __shfl_xor(hi, 32));
      } else {
        float a = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; v++) a = fmaxf(a, fabsf(acc[i][j][v]));
        tmax[i] = fmaxf(a, __shfl_xor(a, 32));
        tmin[i] = 0.0f;
      }
    }
    if (gi_tiles == 2) {
      tmax[0] = tmax[1] = fmaxf(tmax[0], tmax[1]);
      tmax[2] = tmax[3] = fmaxf(tmax[2], tmax[3]);
      tmin[0] = tmin[1] = fminf(tmin[0], tmin[1]);
      tmin[2] = tmin[3] = fminf(tmin[2], tmin[3]);
    } else if (gi_tiles == 4) {
      tmax[0] = tmax[1] = tmax[2] = tmax[3] = fmaxf(fmaxf(tmax[0], tmax[1]), fmaxf(tmax[2], tmax[3]));
      tmin[0] = tmin[1] = tmin[2] = tmin[3] = fminf(fminf(tmin[0], tmin[1]), fminf(tmin[2], tmin[3]));
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int cl = cl0 + i * 32;                          // first 4-bit channel of this tile
      const bool valid = cl >= 0 && cl < KL && m < M;
      uint16_t sbits, zbits = 0;
      float sf, zf = 0.0f;
      if constexpr (ASYM) {
        zf = group_zero(tmin[i], zbits);
        sf = group_scale_asym(tmin[i], tmax[i], sbits);
      } else {
        sf = group_scale(tmax[i], sbits);
      }
      const float inv = group_inv(sf);
      if (valid && h == 0 && (i % gi_tiles) == 0) {
        sx[(size_t)(cl / g) * sx_ld + m] = sbits;
        if constexpr (ASYM) zx[(size_t)(cl / g) * sx_ld + m] = zbits;
      }
      auto nib = [&](float v) { return ASYM ? quant_nibble_asym(v, zf, inv) : quant_nibble(v, inv); };
      // this lane's 16 codes: quad q covers channels cl + 8q + 4h .. +3 -> one 16-bit piece
      uint32_t piece[4];
#pragma unroll
      for (int q = 0; q < 4; q++) {
        piece[q] = nib(acc[i][j][4 * q]) | nib(acc[i][j][4 * q + 1]) << 4 | nib(acc[i][j][4 * q + 2]) << 8 |
                   nib(acc[i][j][4 * q + 3]) << 12;
      }
      const uint32_t P0 = piece[0] | (piece[1] << 16), P1 = piece[2] | (piece[3] << 16);
      // lane h=0 keeps dwords 0,1 of the tile's 16 bytes, lane h=1 dwords 2,3
      const uint32_t recv = __shfl_xor(h ? P0 : P1, 32);
      const uint32_t lo = h ? recv : P0, hi = h ? P1 : recv;
      uint2 o;
      o.x = (lo & 0xFFFFu) | (hi << 16);
      o.y = (lo >> 16) | (hi & 0xFFFF0000u);
      if (valid) *(uint2*)(xl + (size_t)m * xl_ld + cl / 2 + 8 * h) = o;
    }
  }
}

// QM selects what happens to the channels [r, K): 0 = symmetric 4-bit per-group quantizer,
// 1 = asymmetric one (zero-point min, 16 unsigned levels; zx receives the zero-points, laid out
// like sx), 2 = no quantizer here: the fp32 values go to xf [M][K-r] and the absolute maximum of
// every 128-channel wave tile to pmax [ceil((K-r)/128)][M] (per-token 8-bit quantization needs the
// maximum over all channels of a token, which no single workgroup sees).
template <int WGC, int WGT, int BK, int MI, int QM, int WVT, int KSP>
__global__ __launch_bounds__(WGC* WGT* KSP * 64, (RQ<WGC, WGT, BK, WVT, KSP>::WAVES_PER_SIMD)) void rotate_quantize_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ Qt, int M, int K, int r, int g,
    uint16_t* __restrict__ xh, uint8_t* __restrict__ xl, uint16_t* __restrict__ sx, uint16_t* __restrict__ zx,
    float* __restrict__ xf, float* __restrict__ pmax, int r_pad, int Kv, int n_ct, int n_tt, int per_xcd, int sx_ld) {
  using C = RQ<WGC, WGT, BK, WVT, KSP>;
  static_assert(WVT == 64 || (WVT == 32 && MI == 32), "32-token wave tiles are written for the 32x32 loop only");
  static_assert(KSP == 1 || MI == 32, "the K split is written for the 32x32 loop only");
  constexpr bool ASYM = QM == 1;
  extern __shared__ __align__(16) unsigned char smem_all[];

  // consecutive workgroup ids go to different XCDs; give each XCD a contiguous run of tiles
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= n_ct * n_tt) return;
  // within an XCD's run, sweep GC channel tiles per token tile so that co-resident
  // workgroups share both operands through the XCD's L2
  constexpr int GC = 4;
  const int grp = logical / (GC * n_tt), in_grp = logical % (GC * n_tt);
  const int gc = min(n_ct - grp * GC, GC);
  const int ct = grp * GC + in_grp % gc, tt = in_grp / gc;
  const int m0 = tt * C::TT;

  const int t = threadIdx.x, l = t & 63;
  const int w = (t >> 6) % C::NW, kp = (t >> 6) / C::NW;    // wave within its k-part, k-part
  const int wc = w % WGC, wt = w / WGC;
  unsigned char* const smem = smem_all + kp * (2 * C::STAGE_BYTES);   // the k-part's own two stages

  // ---- per-lane source pointers of this wave's loads ---------------------------------
  // load q of wave w fills LDS bytes [(w*IPW+q)*1024, +1024) of a stage: rows are the TC
  // channel rows followed by the TT token rows.  Rows past the edge re-read a valid row; their
  // results are discarded in the epilogue.
  const uint16_t* gsrc[C::IPW];
#pragma unroll
  for (int i = 0; i < C::IPW; i++) {
    const int ci = (w * C::IPW + i) * 64 + l;               // chunk index within the stage
    const int row = ci / C::CPR, phys = ci % C::CPR;
    const int logical_chunk = phys ^ C::swz(row);
    const uint16_t* base;
    if (row < C::TC) {
      const int v = ct * C::TC + row;                       // virtual channel
      int ch = v < r_pad ? min(v, r - 1) : min(r + (v - r_pad), K - 1);
      ch = max(ch, 0);
      base = Qt + (size_t)ch * K;
    } else {
      base = x + (size_t)min(m0 + row - C::TC, M - 1) * K;
    }
    gsrc[i] = base + logical_chunk * 8 + kp * (K / KSP);
  }
  i32x4 staged[C::IPW];
  auto gload = [&](int q, int kt) { staged[q] = *(const i32x4*)(gsrc[q] + kt * BK); };
  auto swrite = [&](int q, int buf) {
    *(i32x4*)(smem + buf * C::STAGE_BYTES + (w * C::IPW + q) * 1024 + l * 16) = staged[q];
  };

  const int nk = K / (BK * KSP);                            // the launcher guarantees K % (BK KSP) == 0, nk >= 1

  // prologue: stage 0 into LDS, stage 1 into the registers.  Loads past the last stage re-read
  // it: unconditional loads keep the outstanding-load count the same in every iteration, so
  // the waits the compiler derives are exact.
#pragma unroll
  for (int q = 0; q < C::IPW; q++) gload(q, 0);
#pragma unroll
  for (int q = 0; q < C::IPW; q++) swrite(q, 0);
  __syncthreads();
  // the loads must be issued in the order the main loop consumes them: its waits count the loads
  // issued after the one needed
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int q = 0; q < C::IPW; q++) {
    gload(q, min(1, nk - 1));
    __builtin_amdgcn_sched_barrier(0);
  }

  if constexpr (MI == 32) {
    // ======== 32x32x16 MFMA: wave tile = 4 x 2 tiles of 32 channels x 32 tokens ========
    constexpr int WT = C::WAVE_T / 32;                        // 32-token MFMA tiles per wave
    f32x16 acc[4][WT];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < WT; j++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

    // operand read offsets (bytes within a stage) for k-step 0; k-step ks flips chunk bits
    int offA[4], offB[WT];
#pragma unroll
    for (int i = 0; i < 4; i++) offA[i] = (wc * 128 + i * 32 + (l & 31)) * C::ROWB;
#pragma unroll
    for (int j = 0; j < WT; j++) offB[j] = (C::TC + wt * C::WAVE_T + j * 32 + (l & 31)) * C::ROWB;
    const int swzA = C::swz(l & 31), swzB = C::swz(l & 31);   // tile bases are multiples of 32 rows

    bf16x8 a[2][4], b[2][WT];
    int kt = 0;
    do {                                                      // nk >= 1
      const unsigned char* sb = smem + (kt & 1) * C::STAGE_BYTES;
      const int wbuf = (kt + 1) & 1, kt_load = min(kt + 2, nk - 1);
      // operands of k-step ks+1 are fetched from LDS while the MFMAs of k-step ks run
      auto lds_fetch = [&](int ks, int slot) {
        const int chunk = 2 * ks + (l >> 5);
#pragma unroll
        for (int i = 0; i < 4; i++) a[slot][i] = *(const bf16x8*)(sb + offA[i] + ((chunk ^ swzA) << 4));
#pragma unroll
        for (int j = 0; j < WT; j++) b[slot][j] = *(const bf16x8*)(sb + offB[j] + ((chunk ^ swzB) << 4));
      };
      lds_fetch(0, 0);
#pragma unroll
      for (int ks = 0; ks < C::KS; ks++) {
        const int cur = ks & 1;
        int pair = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) {
#pragma unroll
          for (int j = 0; j < WT; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (i == 0 && ks + 1 < C::KS) lds_fetch(ks + 1, cur ^ 1);
          // the PP store/load pairs of this k-step, spread over its four MFMA rows
          if (pair < C::PP && i >= (pair * 4) / C::PP) {
            const int q = ks * C::PP + pair;
            swrite(q, wbuf);
            gload(q, kt_load);
            pair++;
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __syncthreads();   // stage kt+1 is complete in LDS; stage kt may be overwritten
    } while (++kt < nk);

    if constexpr (KSP == 2) {
      // the second k-part hands its sums to the first through the stage buffers (every wave has passed the
      // loop's last barrier, so nothing reads them any more); the first adds them and goes on alone
      float4* red = (float4*)smem_all + (size_t)w * (4 * WT * 4 * 64) + l;
      if (kp == 1) {
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
          for (int j = 0; j < WT; j++)
#pragma unroll
            for (int q = 0; q < 4; q++)
              red[((i * WT + j) * 4 + q) * 64] =
                  make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
      }
      __syncthreads();
      if (kp == 1) return;
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < WT; j++)
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const float4 v = red[((i * WT + j) * 4 + q) * 64];
            acc[i][j][4 * q] += v.x;
            acc[i][j][4 * q + 1] += v.y;
            acc[i][j][4 * q + 2] += v.z;
            acc[i][j][4 * q + 3] += v.w;
          }
    }

    // ---- epilogue, in registers ------------------------------------------------------
    rq_epilogue32<QM, WT>(acc, ct * C::TC + wc * 128, m0 + wt * C::WAVE_T, M, K, r, g, r_pad, Kv, xh, xl, sx, zx, xf,
                          pmax, sx_ld);
  } else {
    // ======== 16x16x32 MFMA: wave tile = 8 x 4 tiles of 16 channels x 16 tokens =========
    // Accumulator layout of a 16x16 tile: lane l holds channels 4*(l/16) .. +3 of token l%16, so
    // the 16 channels of one token sit in the four lanes {t, t+16, t+32, t+48}; a quantization
    // group (2, 4 or 8 tiles) is reduced in-lane and then across those four lanes.
    constexpr int NI = 8, NJ = 4;                           // 16-channel x 16-token tiles per wave
    constexpr int KS2 = BK / 32;                            // MFMA k-steps per stage
    constexpr int PPS = C::IPW / KS2;                       // store/load pairs per k-step
    static_assert(MI != 16 || (C::IPW % KS2 == 0 && PPS <= NI), "store/load pairs are spread over the 8 tile rows of a k-step");
    f32x4 acc[NI][NJ];
#pragma unroll
    for (int i = 0; i < NI; i++)
#pragma unroll
      for (int j = 0; j < NJ; j++)
#pragma unroll
        for (int v = 0; v < 4; v++) acc[i][j][v] = 0.0f;

    // operand reads: lane l takes row l%16 of a tile, 16-byte chunk 4*ks + l/16 of the stage's k range
    const int lr = l & 15, hq = l >> 4;
    const int offA = (wc * 128 + lr) * C::ROWB, offB = (C::TC + wt * 64 + lr) * C::ROWB;
    const int sw = C::swz(lr);                                // tile bases are multiples of 16 rows

    bf16x8 a[3], b[2][NJ];
    int kt = 0;
    do {                                                      // nk >= 1
      const unsigned char* sb = smem + (kt & 1) * C::STAGE_BYTES;
      const int wbuf = (kt + 1) & 1, kt_load = min(kt + 2, nk - 1);
      // flat index f = ks*NI + i over the stage's (k-step, channel tile) pairs; A tiles are fetched two
      // ahead of their MFMAs, the B tiles of the next k-step during the current one
      auto fetch_a = [&](int f) {
        const int ks = f / NI, i = f % NI;
        a[f % 3] = *(const bf16x8*)(sb + offA + i * 16 * C::ROWB + (((4 * ks + hq) ^ sw) << 4));
      };
      auto fetch_b = [&](int ks, int j) {
        b[ks & 1][j] = *(const bf16x8*)(sb + offB + j * 16 * C::ROWB + (((4 * ks + hq) ^ sw) << 4));
      };
#pragma unroll
      for (int j = 0; j < NJ; j++) fetch_b(0, j);
      fetch_a(0);
      fetch_a(1);
#pragma unroll
      for (int f = 0; f < KS2 * NI; f++) {
        const int ks = f / NI, i = f % NI;
        if (f + 2 < KS2 * NI) fetch_a(f + 2);
        if (ks + 1 < KS2 && i >= 2 && i < 2 + NJ) fetch_b(ks + 1, i - 2);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NJ; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[f % 3], b[ks & 1][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // the PPS store/load pairs of this k-step, spread over its tile rows
#pragma unroll
        for (int p = 0; p < PPS; p++)
          if (i == (p * NI) / PPS) {
            const int q = ks * PPS + p;
            swrite(q, wbuf);
            gload(q, kt_load);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();   // stage kt+1 is complete in LDS; stage kt may be overwritten
    } while (++kt < nk);

    // ---- epilogue, in registers ------------------------------------------------------
    const int vb = ct * C::TC + wc * 128;                     // first virtual channel of this wave
    if (vb >= Kv) return;
    if (vb < r_pad) {
      // 16-bit part: the lane's 4 consecutive channels of a tile -> one 8-byte store
#pragma unroll
      for (int j = 0; j < NJ; j++) {
        const int m = m0 + wt * 64 + j * 16 + lr;
#pragma unroll
        for (int i = 0; i < NI; i++) {
          const int c = vb + i * 16 + 4 * hq;
          if (c < r && m < M) {
            uint2 o;
            o.x = f32_to_bf16_bits(acc[i][j][0]) | ((uint32_t)f32_to_bf16_bits(acc[i][j][1]) << 16);
            o.y = f32_to_bf16_bits(acc[i][j][2]) | ((uint32_t)f32_to_bf16_bits(acc[i][j][3]) << 16);
            *(uint2*)(xh + (size_t)m * r + c) = o;
          }
        }
      }
      if (vb + 128 <= r_pad) return;                          // (else the split point lies inside this wave's channels)
    }
    const int cl0 = vb - r_pad;                               // first 4-bit channel of this wave (negative: see above)
    const int KL = K - r;
    if constexpr (QM == 2) {
#pragma unroll
      for (int j = 0; j < NJ; j++) {
        const int m = m0 + wt * 64 + j * 16 + lr;
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < NI; i++) {
          const int cl = cl0 + i * 16;
          if (cl < KL) {
#pragma unroll
            for (int e = 0; e < 4; e++) a = fmaxf(a, fabsf(acc[i][j][e]));
            if (m < M)
              *(float4*)(xf + (size_t)m * KL + cl + 4 * hq) =
                  make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
          }
        }
        a = fmaxf(a, __shfl_xor(a, 16));
        a = fmaxf(a, __shfl_xor(a, 32));
        if (hq == 0 && m < M) pmax[(size_t)(cl0 >> 7) * sx_ld + m] = a;
      }
      return;
    }
    const size_t xl_ld = (size_t)KL / 2;
    const int gu = g >> 5;                                    // 32-channel units per group: 1, 2, 4
    // The four lanes of a token are the four 16-lane rows of the wave; data moves between them with
    // the row-swap instructions of gfx950 (4 swaps transpose a 4x4 block of dwords over rows x registers).
    auto swap16 = [](uint32_t& x, uint32_t& y) {              // rows (x1 <-> y0), (x3 <-> y2)
      auto v = __builtin_amdgcn_permlane16_swap(x, y, false, false);
      x = v[0];
      y = v[1];
    };
    auto swap32 = [](uint32_t& x, uint32_t& y) {              // rows (x2 <-> y0), (x3 <-> y1)
      auto v = __builtin_amdgcn_permlane32_swap(x, y, false, false);
      x = v[0];
      y = v[1];
    };
    auto transpose4 = [&](uint32_t (&v)[4]) {                 // afterwards v[h] on row q = old v[q] on row h
      swap16(v[0], v[1]);
      swap16(v[2], v[3]);
      swap32(v[0], v[2]);
      swap32(v[1], v[3]);
    };
#pragma unroll
    for (int j = 0; j < NJ; j++) {
      const int m = m0 + wt * 64 + j * 16 + lr;
      // absmax (symmetric) or min and max (asymmetric) per 32-channel unit (two tiles) in-lane;
      // after the transpose row q holds unit q's four partial results, so row q finishes unit q
      uint32_t um[4], un[4];
#pragma unroll
      for (int u = 0; u < 4; u++) {
        if constexpr (ASYM) {
          float lo = acc[2 * u][j][0], hi = acc[2 * u][j][0];
#pragma unroll
          for (int e = 0; e < 4; e++) {
            lo = fminf(lo, fminf(acc[2 * u][j][e], acc[2 * u + 1][j][e]));
            hi = fmaxf(hi, fmaxf(acc[2 * u][j][e], acc[2 * u + 1][j][e]));
          }
          um[u] = __builtin_bit_cast(uint32_t, hi);
          un[u] = __builtin_bit_cast(uint32_t, lo);
        } else {
          float v = 0.0f;
#pragma unroll
          for (int e = 0; e < 4; e++) v = fmaxf(v, fmaxf(fabsf(acc[2 * u][j][e]), fabsf(acc[2 * u + 1][j][e])));
          um[u] = __builtin_bit_cast(uint32_t, v);
        }
      }
      auto f = [](uint32_t b) { return __builtin_bit_cast(float, b); };
      auto bits = [](float v) { return __builtin_bit_cast(uint32_t, v); };
      transpose4(um);
      float gm = fmaxf(fmaxf(f(um[0]), f(um[1])), fmaxf(f(um[2]), f(um[3]))), gn = 0.0f;
      if constexpr (ASYM) {
        transpose4(un);
        gn = fminf(fminf(f(un[0]), f(un[1])), fminf(f(un[2]), f(un[3])));
      }
      if (gu > 1) {                                           // groups of 2 or 4 units: combine rows
        uint32_t e0 = bits(gm), e1 = e0;
        swap16(e0, e1);                                       // e0 = rows (0,0,2,2), e1 = rows (1,1,3,3)
        gm = fmaxf(f(e0), f(e1));
        if constexpr (ASYM) {
          uint32_t d0 = bits(gn), d1 = d0;
          swap16(d0, d1);
          gn = fminf(f(d0), f(d1));
        }
        if (gu > 2) {
          uint32_t f0 = bits(gm), f1 = f0;
          swap32(f0, f1);                                     // f0 = rows (0,1,0,1), f1 = rows (2,3,2,3)
          gm = fmaxf(f(f0), f(f1));
          if constexpr (ASYM) {
            uint32_t c0 = bits(gn), c1 = c0;
            swap32(c0, c1);
            gn = fminf(f(c0), f(c1));
          }
        }
      }
      // row q: scale (and zero-point) of the group that unit q belongs to
      uint16_t sbits, zbits = 0;
      float sf, zf_q = 0.0f;
      if constexpr (ASYM) {
        zf_q = group_zero(gn, zbits);
        sf = group_scale_asym(gn, gm, sbits);
      } else {
        sf = group_scale(gm, sbits);
      }
      const float inv_q = group_inv(sf);
      const int clu = cl0 + 32 * hq;                          // first channel of unit hq
      const bool valid = clu >= 0 && clu < KL && m < M;
      if (valid && (hq % gu) == 0) {
        sx[(size_t)(clu / g) * sx_ld + m] = sbits;
        if constexpr (ASYM) zx[(size_t)(clu / g) * sx_ld + m] = zbits;
      }
      // broadcast the four rows' values to all rows: b[u] = row u's value everywhere
      auto broadcast4 = [&](float v, float (&b)[4]) {
        uint32_t i0 = bits(v), i1 = i0;
        swap16(i0, i1);                                       // i0 = rows (0,0,2,2), i1 = rows (1,1,3,3)
        uint32_t i2 = i0, i3 = i1;
        swap32(i0, i2);                                       // i0 = row 0 everywhere, i2 = row 2 everywhere
        swap32(i1, i3);                                       // i1 = row 1 everywhere, i3 = row 3 everywhere
        b[0] = f(i0);
        b[1] = f(i1);
        b[2] = f(i2);
        b[3] = f(i3);
      };
      float inv[4], zf[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      broadcast4(inv_q, inv);
      if constexpr (ASYM) broadcast4(zf_q, zf);
      // codes: P[u] = the lane's 4 + 4 codes of unit u (tile 2u in the low half, tile 2u+1 in the high half)
      uint32_t P[4];
#pragma unroll
      for (int u = 0; u < 4; u++) {
        uint32_t pc = 0;
#pragma unroll
        for (int half = 0; half < 2; half++)
#pragma unroll
          for (int e = 0; e < 4; e++)
            pc |= (ASYM ? quant_nibble_asym(acc[2 * u + half][j][e], zf[u], inv[u])
                        : quant_nibble(acc[2 * u + half][j][e], inv[u]))
                  << (16 * half + 4 * e);
        P[u] = pc;
      }
      transpose4(P);                                          // P[h] = row h's codes of unit hq
      // unit hq = 16 bytes: tile 2hq (low halves, rows 0..3 in channel order), then tile 2hq+1
      uint4 o;
      o.x = (P[0] & 0xFFFFu) | (P[1] << 16);
      o.y = (P[2] & 0xFFFFu) | (P[3] << 16);
      o.z = (P[0] >> 16) | (P[1] & 0xFFFF0000u);
      o.w = (P[2] >> 16) | (P[3] & 0xFFFF0000u);
      if (valid) *(uint4*)(xl + (size_t)m * xl_ld + clu / 2) = o;
    }
  }
}

// Virtual channel order of the tiling: the 16-bit part [0, r) first, then the 4-bit part from r_pad on.  r_pad is r
// itself when the groups then still fall inside the 128-channel wave tiles (r a multiple of the group size: the
// wave that holds the split point stores both kinds), else r rounded up to 128.  The fp32 output for the 8-bit
// quantizer keeps the rounded form (its per-wave maxima are indexed by whole 128-channel tiles of the 4-bit part).
static void virtual_channels(int K, int r, int g, bool fp32_out, int& r_pad, int& Kv) {
  r_pad = (!fp32_out && r % g == 0) ? r : (r + 127) / 128 * 128;
  Kv = (r_pad + (K - r) + 127) / 128 * 128;
}

template <int WGC, int WGT, int BK, int MI, int QM, int WVT, int KSP>
static int launch_one(const uint16_t* x, const uint16_t* Qt, int M, int K, int r, int g, uint16_t* xh,
                      uint8_t* xl, uint16_t* sx, uint16_t* zx, float* xf, float* pmax, hipStream_t s, int m_off,
                      int sx_ld) {
  // tokens [m_off, m_off + M) of the caller's arrays; sx_ld = total token count (row length of s_x)
  if (sx_ld == 0) sx_ld = M;
  x += (size_t)m_off * K;
  if (xh) xh += (size_t)m_off * r;
  if (xl) xl += (size_t)m_off * ((K - r) / 2);
  if (sx) sx += m_off;
  if (zx) zx += m_off;
  if (xf) xf += (size_t)m_off * (K - r);
  if (pmax) pmax += m_off;
  using C = RQ<WGC, WGT, BK, WVT, KSP>;
  int r_pad, Kv;
  virtual_channels(K, r, g, QM == 2, r_pad, Kv);
  const int n_ct = (Kv + C::TC - 1) / C::TC;
  const int n_tt = (M + C::TT - 1) / C::TT;
  const long n_blocks = (long)n_ct * n_tt;
  const int per_xcd = (int)((n_blocks + 7) / 8);
  // (idempotent: two threads racing here would both set the same attribute)
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)rotate_quantize_kernel<WGC, WGT, BK, MI, QM, WVT, KSP>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM);
    if (e != hipSuccess) return hip_failed(e);
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((rotate_quantize_kernel<WGC, WGT, BK, MI, QM, WVT, KSP>), dim3(per_xcd * 8), dim3(C::NT), C::SMEM, s, x,
                     Qt, M, K, r, g, xh, xl, sx, zx, xf, pmax, r_pad, Kv, n_ct, n_tt, per_xcd, sx_ld);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

template <int WGC, int WGT, int BK, int MI, int WVT = 64, int KSP = 1>
static int launch_cfg(const RqOut& o, const uint16_t* x, const uint16_t* Qt, int M, int K, int r, int g,
                      hipStream_t s, int m_off = 0, int sx_ld = 0) {
  if (o.xf) return launch_one<WGC, WGT, BK, MI, 2, WVT, KSP>(x, Qt, M, K, r, g, o.xh, o.xl, o.sx, o.zx, o.xf, o.pmax, s, m_off, sx_ld);
  if (o.zx) return launch_one<WGC, WGT, BK, MI, 1, WVT, KSP>(x, Qt, M, K, r, g, o.xh, o.xl, o.sx, o.zx, o.xf, o.pmax, s, m_off, sx_ld);
  return launch_one<WGC, WGT, BK, MI, 0, WVT, KSP>(x, Qt, M, K, r, g, o.xh, o.xl, o.sx, o.zx, o.xf, o.pmax, s, m_off, sx_ld);
}

int launch_rotate_quantize(const uint16_t* x, const uint16_t* Qt, int M, int K, int r, int g, const RqOut& o,
                           hipStream_t s) {
  // Large problems: 256 x 256 workgroup tiles (8 waves); medium: 256 channels x 128 tokens
  // (4 waves); small: 128 x 128 as 4 waves of 128 channels x 32 tokens, or 128 x 64 with K split over two
  // sets of such waves (below).  A small launch is a chain of latencies (a few dozen workgroups, each alone
  // on its CU, walk K stage by stage), so its waves carry half the arithmetic per stage: 13 instead of 20 us
  // at M = 256, K = 1152.
  // The large tiles run long enough to be limited by power (the shader clock drops under
  // sustained MFMA work on random data); there the 16x16x32 MFMA, which moves half the
  // accumulator bytes per multiply-add, is the faster one.  The smaller, latency-bound
  // launches are faster with the 32x32x16 MFMA and its shorter epilogue.
  int r_pad, Kv;
  virtual_channels(K, r, g, o.xf != nullptr, r_pad, Kv);
  const long n_tc256 = (Kv + 255) / 256;
  const long big_tiles = n_tc256 * ((M + 255) / 256);    // 256 channels x 256 tokens
  const long mid_tiles = n_tc256 * ((M + 127) / 128);    // 256 channels x 128 tokens
  if (K % 64 != 0) {
    if (mid_tiles >= 100) return launch_cfg<2, 2, 32, 32>(o, x, Qt, M, K, r, g, s);
    return launch_cfg<1, 4, 32, 32, 32>(o, x, Qt, M, K, r, g, s);
  }
  // A launch this small is held back by what one CU can load per cycle (each workgroup streams its 128 basis rows
  // over all of K) and by the chain of stage latencies: with 128 x 64 tiles and the two halves of K on two sets
  // of waves per workgroup it has twice the workgroups and half the stages (11 instead of 13 us at M = 256,
  // K = 1152; 21 instead of 26 at K = 3072), as long as that is still a single round of workgroups.
  const long n_tc128 = (Kv + 127) / 128;
  const long small_tiles = n_tc128 * ((M + 63) / 64);      // 128 channels x 64 tokens
  if (K % 128 == 0 && small_tiles <= 256) return launch_cfg<1, 2, 64, 32, 32, 2>(o, x, Qt, M, K, r, g, s);
  // 128 x 128 tiles (two such workgroups fit a CU) while they are resident all at once, or nearly: 14.6 instead
  // of 22.7 us at M = 3072, K = 1152 (216 workgroups against 120 of 256 x 128); K = 3072 prefers the larger tile
  // from one full round on (M = 1536: 44 against 49 us)
  const long tiles128 = n_tc128 * ((M + 127) / 128);
  if (tiles128 <= 256 || (K <= 2048 && tiles128 <= 320)) return launch_cfg<1, 4, 64, 32, 32>(o, x, Qt, M, K, r, g, s);
  // Beyond that: rounds of 256 workgroups.  A round of 256 x 128 tiles takes about 0.62 of a round of 256 x 256
  // ones (K = 3072: 53 against 81 us, K = 12288: 186 against 300-320), so the plans compared are: all big, all
  // half-size, or k full rounds of big tiles and the remaining tokens in a second launch of half-size ones.
  int cus = 0;
  {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_failed(e);
    if (cus < 1) cus = 1;
  }
  auto rounds = [&](long tiles) { return (double)((tiles + cus - 1) / cus); };
  constexpr double MID = 0.62, SECOND_LAUNCH = 0.03;
  double best = rounds(big_tiles);                          // plan: one launch of big tiles
  int plan_tt = -1;                                         // -1: all big, 0: all half-size, > 0: token tiles in the big launch
  if (rounds(mid_tiles) * MID < best) {
    best = rounds(mid_tiles) * MID;
    plan_tt = 0;
  }
  for (long k = 1; k * cus < big_tiles; k++) {
    const long tt = k * cus / n_tc256;                      // token tiles of 256 that k rounds hold
    if (tt <= 0 || tt * 256 >= M) continue;
    const long rest = n_tc256 * ((M - tt * 256 + 127) / 128);
    const double c = rounds(tt * n_tc256) + rounds(rest) * MID + SECOND_LAUNCH;
    if (c < best) {
      best = c;
      plan_tt = (int)tt;
    }
  }
  if (plan_tt < 0) return launch_cfg<2, 4, 64, 16>(o, x, Qt, M, K, r, g, s);
  if (plan_tt == 0) return launch_cfg<2, 2, 64, 32>(o, x, Qt, M, K, r, g, s);
  const int st = launch_cfg<2, 4, 64, 16>(o, x, Qt, plan_tt * 256, K, r, g, s, 0, M);
  if (st) return st;
  return launch_cfg<2, 2, 64, 32>(o, x, Qt, M - plan_tt * 256, K, r, g, s, plan_tt * 256, M);
}

}  // namespace dirotq
