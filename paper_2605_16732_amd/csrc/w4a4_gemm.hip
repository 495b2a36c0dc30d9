// Kernel B: y = x_h W'_h^T + sum_j s_x[:,j] s_w[:,j]^T * (q_x,j q_w,j^T)
// (forward-computation equation of Section 4.2 of the paper).
//
// Orientation.  D[n][token]: output channels on the MFMA row axis, tokens on the column
// axis, so a lane owns one token and 4 consecutive output channels per register quad
// (one 8-byte bf16 store).  Workgroup tile 128 n x 128 tokens, 4 waves as 2 (n) x 2
// (tokens), each 64 n x 64 tokens = 2 x 2 MFMA tiles; two workgroups share a CU so that
// one's barrier / staging phase overlaps the other's arithmetic.
//
// Integer part.  A stored code is a sign-magnitude nibble.  On its way into LDS (once per
// workgroup) it becomes the byte [sign 0000 magnitude], which read as fp8 (E4M3) is the
// subnormal q * 2^-9: the fp8 matrix pipe then multiplies and adds the codes exactly
// (products and sums of small integers times 2^-18, far inside fp32) and hands back the
// group dot as a float, so no integer-to-float conversion is left for the vector ALU.
// Even and odd channels of an 8-channel dword land in different operand registers; both
// operands use the same permutation, so the dot product is unchanged.  One 32x32x64 MFMA
// covers a 64-channel group (two for 128, a half-empty one for 32).
//
// Dequantisation.  The per-group scale product P[n][token] = s_w[n,j] * s_x[token,j] is an
// outer product of fp16 vectors: it is produced exactly (fp16 x fp16 fits fp32) by one
// fp16 MFMA whose operands carry the scales in k-slot 0 and zeros elsewhere, which
// leaves the vector ALU one fma per accumulator and group: acc += (2^-18 I) * P.  The
// common factor 2^18 is applied once at the end (exact), before the 16-bit branch is
// accumulated on top by bf16 MFMAs.
//
// Asymmetric activations (ASYM).  Codes are then unsigned nibbles, whose zero-extended byte
// is again an exact fp8 number (u * 2^-9 for u in 0..15: the first binade continues the
// subnormals linearly), so the main loop is unchanged.  The zero-point term
// sum_j z[m,j] * (s_w[n,j] * sum_k q_w[n,k]) is a small GEMM over the groups; it is added
// after the main loop by bf16 MFMAs on exact bf16 splits of its factors (z = z1 + z2,
// c = b1 + b2 + b3; every product but z2 b3, which is below 2^-24 of the term, is kept).
//
// Schedule.  The vector ALU is the binding unit (one fma per accumulator and group plus the
// unpacking, against 64 cycles of fp8 MFMA per tile and 64-channel group), so the main loop
// is software-pipelined by hand: the MFMAs of tile s+1 are issued before the fma sweep of
// tile s, and the LDS operand reads of the next group are issued one sweep ahead.
#include <atomic>

#include <cstdlib>
#include <cstring>

#include "gemm_tail.h"

namespace dirotq {

constexpr int BKQ = 128;        // 4-bit channels per LDS stage (one 128-byte fp8 row)
constexpr int ROWS = TN + TM;
constexpr int STAGE_BYTES = ROWS * 128;              // fp8 [256 rows][128 B] (= bf16 [256][64])
constexpr int SCALE_OFF = 2 * STAGE_BYTES;           // u64 [2 bufs][4 groups][256 rows]: {fp16 scale, 0, 0, 0}
// per buffer: (groups per stage) x ROWS x 8 bytes, then 8 zero bytes read by lanes 32..63
constexpr int scale_buf_bytes(int gs) { return (BKQ / gs) * ROWS * 8; }
constexpr int zero_off(int gs) { return SCALE_OFF + 2 * scale_buf_bytes(gs); }
constexpr int smem_bytes(int gs) { return zero_off(gs) + 256; }

// 8 sign-magnitude nibbles of a dword -> two dwords of fp8 (E4M3) bytes [s 0000 mmm], i.e. the
// values +-m * 2^-9 (subnormals, exact): even channels, odd channels
__device__ __forceinline__ void unpack8(uint32_t p, uint32_t& even, uint32_t& odd) {
  even = (p & 0x07070707u) | ((p & 0x08080808u) << 4);
  odd = ((p >> 4) & 0x07070707u) | (p & 0x80808080u);
}

typedef __attribute__((ext_vector_type(8))) int i32x8;
// one 32x32x64 fp8 MFMA step (no block scaling)
__device__ __forceinline__ f32x16 mfma_fp8_k64(i32x4 a_lo, i32x4 a_hi, i32x4 b_lo, i32x4 b_hi, f32x16 c) {
  const i32x8 a = __builtin_shufflevector(a_lo, a_hi, 0, 1, 2, 3, 4, 5, 6, 7);
  const i32x8 b = __builtin_shufflevector(b_lo, b_hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

// 8 unsigned nibbles of a dword -> two dwords of fp8 bytes 0000uuuu = u * 2^-9
__device__ __forceinline__ void unpack8u(uint32_t p, uint32_t& even, uint32_t& odd) {
  even = p & 0x0F0F0F0Fu;
  odd = (p >> 4) & 0x0F0F0F0Fu;
}

template <int GS, bool OUT_F32, bool ASYM>
__global__ __launch_bounds__(NTHREADS, 2) void w4a4_gemm_kernel(
    const uint16_t* __restrict__ xh, const uint8_t* __restrict__ xl, const uint16_t* __restrict__ sx,
    const uint16_t* __restrict__ zx, const uint16_t* __restrict__ wh, const uint8_t* __restrict__ wq,
    const uint16_t* __restrict__ sw, const int16_t* __restrict__ wsum, const uint16_t* __restrict__ bias, int M,
    int N, int K, int r, void* __restrict__ y, int n_mt, int n_nt, int per_xcd) {
  extern __shared__ __align__(16) unsigned char smem[];

  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= n_mt * n_nt) return;
  // within an XCD's run, sweep GN output tiles per token tile (shared operands stay in L2)
  constexpr int GN = 4;
  const int grp = logical / (GN * n_mt), in_grp = logical % (GN * n_mt);
  const int gn = min(n_nt - grp * GN, GN);
  const int nt = grp * GN + in_grp % gn, mt = in_grp / gn;
  const int m0 = mt * TM, n0 = nt * TN;

  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int wn = w & 1, wt = w >> 1;
  const int h = l >> 5;
  const int KL = K - r;            // number of 4-bit channels
  const int G = KL / GS;
  constexpr int GPS = BKQ / GS;    // groups per stage
  constexpr int MPG = GS / 32;     // 16-byte operand chunks (32 channels over the lane pair) per group
  constexpr int SCALE_BUF_BYTES = scale_buf_bytes(GS), ZERO_OFF = zero_off(GS);

  if (t < 64) ((uint32_t*)(smem + ZERO_OFF))[t] = 0u;   // read as the zero operand half

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

  // operand rows of this lane: A = weights (rows 0..127 of a stage), B = tokens (128..255)
  int rowA[2], rowB[2];
#pragma unroll
  for (int i = 0; i < 2; i++) rowA[i] = wn * 64 + i * 32 + (l & 31);
#pragma unroll
  for (int j = 0; j < 2; j++) rowB[j] = TN + wt * 64 + j * 32 + (l & 31);
  const int swz = ((l & 31) >> 1) & 7;                 // tile bases are multiples of 32 rows

  // ---- 4-bit branch ---------------------------------------------------------------
  if (KL > 0) {
    const size_t ldq = (size_t)KL / 2;        // packed bytes per row
    const int prow = t >> 2, pchunk = t & 3;  // 4 rows (stride 64) x one 16-B packed chunk per thread
    const int pc16 = min(pchunk * 16, (int)ldq - 16);   // this thread's chunk, kept inside the row
    const uint8_t* gq[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int row = prow + 64 * i;
      gq[i] = (row < TN ? wq + (size_t)min(n0 + row, N - 1) * ldq : xl + (size_t)min(m0 + row - TN, M - 1) * ldq) +
              pc16;
    }
    // scale staging: thread t owns row t of the stage (weights then tokens)
    const int ts = t;
    const uint16_t* gs = ts < TN ? sw + min(n0 + ts, N - 1) : sx + min(m0 + ts - TN, M - 1);
    const size_t s_ld = t < TN ? (size_t)N : (size_t)M;

    // Staging registers: chunk i (i < 4) / the scales (i == 4) of one stage.  Each piece is
    // reloaded for stage s+2 right after it has been unpacked into LDS for stage s+1, so a
    // global load has a whole stage of arithmetic to complete.
    uint4 rq[4];
    uint16_t rs[GPS];
    // Loads are unconditional (straight-line code keeps the outstanding-load count exact):
    // a chunk past the end of the row is re-read from the row's last chunk and belongs to a
    // group >= G, whose scale is forced to zero, so it contributes exactly nothing.
    const int last_chunk = (int)ldq - 16 - pc16;            // largest in-row offset for this thread (>= 0)
    auto gload_piece = [&](int st, int i) {
      if (i < 4) {
        rq[i] = *(const uint4*)(gq[i] + min(st * (BKQ / 2), last_chunk));
      } else {
#pragma unroll
        for (int jj = 0; jj < GPS; jj++) {
          const int j = st * GPS + jj;
          const uint16_t v = gs[(size_t)min(j, G - 1) * s_ld];
          rs[jj] = (uint16_t)(v & (j < G ? 0xFFFFu : 0u));
        }
      }
    };
    // unpack one staged chunk (or the scales) into the LDS stage `buf`
    auto sstore_piece = [&](int buf, int i) {
      unsigned char* sb = smem + buf * STAGE_BYTES;
      if (i < 4) {
        const int row = prow + 64 * i;
        uint4 e, o;
        if (ASYM && i >= 2) {                 // rows 128..255 of a stage are tokens: unsigned codes
          unpack8u(rq[i].x, e.x, o.x);
          unpack8u(rq[i].y, e.y, o.y);
          unpack8u(rq[i].z, e.z, o.z);
          unpack8u(rq[i].w, e.w, o.w);
        } else {
          unpack8(rq[i].x, e.x, o.x);
          unpack8(rq[i].y, e.y, o.y);
          unpack8(rq[i].z, e.z, o.z);
          unpack8(rq[i].w, e.w, o.w);
        }
        *(uint4*)(sb + tile_off_bytes(row, 2 * pchunk)) = e;
        *(uint4*)(sb + tile_off_bytes(row, 2 * pchunk + 1)) = o;
      } else {
        uint2* sdst = (uint2*)(smem + SCALE_OFF + buf * SCALE_BUF_BYTES);
#pragma unroll
        for (int jj = 0; jj < GPS; jj++)
          sdst[jj * ROWS + t] = make_uint2(rs[jj], 0u);
      }
    };

    // per-lane LDS addresses: operand chunk k (0..3) of each tile row, and the scale words
    // (k-slot 0 of the outer-product MFMA lives in lanes 0..31; lanes 32..63 read zeros)
    int adA[2][4], adB[2][4];
#pragma unroll
    for (int k = 0; k < 4; k++) {
      const int off = ((2 * k + h) ^ swz) << 4;
#pragma unroll
      for (int i = 0; i < 2; i++) adA[i][k] = rowA[i] * 128 + off;
#pragma unroll
      for (int j = 0; j < 2; j++) adB[j][k] = rowB[j] * 128 + off;
    }
    int soffA[2], soffB[2];
#pragma unroll
    for (int i = 0; i < 2; i++) soffA[i] = h ? ZERO_OFF : SCALE_OFF + rowA[i] * 8;
#pragma unroll
    for (int j = 0; j < 2; j++) soffB[j] = h ? ZERO_OFF : SCALE_OFF + rowB[j] * 8;
    const int sstep = h ? 0 : ROWS * 8;       // per group within a stage
    const int sbufstep = h ? 0 : SCALE_BUF_BYTES;

    const int nst = (KL + BKQ - 1) / BKQ;
#pragma unroll
    for (int i = 0; i < 5; i++) gload_piece(0, i);
#pragma unroll
    for (int i = 0; i < 5; i++) {
      sstore_piece(0, i);
      gload_piece(min(1, nst - 1), i);
    }
    __syncthreads();
    for (int st = 0; st < nst; st++) {
      const int buf = st & 1;
      const int st2 = min(st + 2, nst - 1);     // past the end: harmless re-load, never used
      const unsigned char* sb = smem + buf * STAGE_BYTES;
      const unsigned char* ssb = smem + buf * sbufstep;
      // operands of one group: fp8 codes of 2 weight tiles and 2 token tiles, and their scales
      i32x4 a[2][MPG], b[2][MPG];
      f16x4 sa[2], sbv[2];
      auto load_ops = [&](int jj) {
#pragma unroll
        for (int kk = 0; kk < MPG; kk++) {
#pragma unroll
          for (int i = 0; i < 2; i++) a[i][kk] = *(const i32x4*)(sb + adA[i][jj * MPG + kk]);
#pragma unroll
          for (int j = 0; j < 2; j++) b[j][kk] = *(const i32x4*)(sb + adB[j][jj * MPG + kk]);
        }
#pragma unroll
        for (int i = 0; i < 2; i++) sa[i] = *(const f16x4*)(ssb + soffA[i] + jj * sstep);
#pragma unroll
        for (int j = 0; j < 2; j++) sbv[j] = *(const f16x4*)(ssb + soffB[j] + jj * sstep);
      };
      f32x16 I[2], P[2];
      auto issue = [&](int i, int j, int slot) {     // 2^-18 I and the scale product of tile (i, j)
        // (for 128-channel groups the scale-product MFMA sits between the two dependent code
        // MFMAs, so the second one finds its accumulator ready instead of stalling the wave)
        const i32x4 zero4 = {0, 0, 0, 0};
        f32x16 z, p;
#pragma unroll
        for (int v = 0; v < 16; v++) z[v] = p[v] = 0.0f;
        if (MPG == 1) z = mfma_fp8_k64(a[i][0], zero4, b[j][0], zero4, z);     // 32 channels: upper k half empty
        else z = mfma_fp8_k64(a[i][0], a[i][1], b[j][0], b[j][1], z);
        P[slot] = __builtin_amdgcn_mfma_f32_32x32x8f16(sa[i], sbv[j], p, 0, 0, 0);
        if (MPG == 4) z = mfma_fp8_k64(a[i][2], a[i][3], b[j][2], b[j][3], z);
        I[slot] = z;
      };
      auto sweep = [&](int i, int j, int slot) {     // acc += (2^-18 I) * P for tile (i, j)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] = fmaf(I[slot][v], P[slot][v], acc[i][j][v]);
        asm volatile("" : "+v"(acc[i][j]));            // pin the sweep here (keeps I/P live ranges short)
      };
      // the next stage's unpack work is spread over the tile sweeps of this stage
      constexpr int NSTEP = GPS * 4;
      auto stage_piece = [&](int step) {
        // chunk i goes with step (i + 1) * NSTEP / 4 - 1: evenly spread over the stage
        if ((step + 1) % (NSTEP / 4) == 0) {                 // (after the last stage: unused)
          const int i = (step + 1) / (NSTEP / 4) - 1;
          sstore_piece(buf ^ 1, i);
          gload_piece(st2, i);
          if (step == NSTEP - 1) {                           // scales
            sstore_piece(buf ^ 1, 4);
            gload_piece(st2, 4);
          }
        }
      };
      // One pipeline step = the MFMAs of the next tile interleaved with the fma sweep of
      // the current one (so that neither the matrix pipe nor the vector ALU waits for the other
      // inside a wave): 1 MFMA, then a share of the VALU work, repeated.
      auto interleave = [&](bool valu_first) {
        constexpr int NM = (MPG == 4 ? 2 : 1) + 1, PER = 16 / NM;
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
        const bool more = jj + 1 < GPS;              // compile-time after unrolling
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
        asm volatile("" ::: "memory");               // keep the next group's LDS reads below this point
        if (more) {
          load_ops(jj + 1);                          // every MFMA of this group is issued
          __builtin_amdgcn_sched_barrier(0);
          issue(0, 0, 0);
        }
        sweep(1, 1, 1);
        stage_piece(jj * 4 + 3);
        interleave(true);     // the fresh LDS operands get a few VALU slots to arrive
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

    // ---- zero-point term of asymmetric activations: acc += sum_j z[m,j] c[n,j], c = s_w * sum_k q_w
    if constexpr (ASYM) {
      // 12 groups per pass: thread t fills row t of a [256 rows][64 bf16] tile, 5 k-slots per group:
      // weight rows b1 b2 b3 b1 b2, token rows z1 z1 z1 z2 z2 (group-major sources: coalesced over
      // rows).  z = z1 + z2 and c = b1 + b2 + b3 exactly; only z2 b3 (< 2^-24 of the term) is dropped.
      constexpr int GPP = 12;
      const bool is_w = t < TN;                             // uniform per wave
      const size_t ld = is_w ? (size_t)N : (size_t)M;
      const size_t col = is_w ? (size_t)min(n0 + t, N - 1) : (size_t)min(m0 + t - TN, M - 1);
      // Raw factors are fetched two passes ahead (a pass is much shorter than a load's latency).
      // Loads only here, straight-line per wave: the arithmetic on them waits until they are used.
      uint32_t ra[2][GPP];                                  // s_w bits, or z bits
      int rb[2][GPP];                                       // code sums (weight rows only)
      // (token rows read their z twice rather than branch: no control flow between the loads)
      const uint16_t* src_a = is_w ? sw : zx;
      const int16_t* src_b = is_w ? wsum : (const int16_t*)zx;
      auto fetch = [&](int u, int j0) {
#pragma unroll
        for (int gg = 0; gg < GPP; gg++) {
          const size_t idx = (size_t)min(j0 + gg, G - 1) * ld + col;
          ra[u][gg] = src_a[idx];
          rb[u][gg] = src_b[idx];
        }
      };
      // v = p1 + p2 + p3 with each piece a bf16 number: truncating splits (exact, the residuals
      // need no rounding); a piece is kept as fp32 bits with the low half clear
      auto hi16 = [](float v) { return __builtin_bit_cast(uint32_t, v) & 0xFFFF0000u; };
      auto pair = [](uint32_t lo, uint32_t hi) { return (lo >> 16) | hi; };   // two bf16 slots in a dword
      auto pass = [&](int u, int j0) {
        uint32_t slot[64];                                  // fp32-bit pieces, one per k-slot
#pragma unroll
        for (int k = 60; k < 64; k++) slot[k] = 0;
        if (is_w) {
#pragma unroll
          for (int gg = 0; gg < GPP; gg++) {
            const float v = j0 + gg < G ? f16_bits_to_f32((uint16_t)ra[u][gg]) * (float)rb[u][gg] : 0.0f;
            const uint32_t p1 = hi16(v);
            const float r1 = v - __builtin_bit_cast(float, p1);
            const uint32_t p2 = hi16(r1);
            const uint32_t p3 = hi16(r1 - __builtin_bit_cast(float, p2));
            slot[5 * gg + 0] = p1;
            slot[5 * gg + 1] = p2;
            slot[5 * gg + 2] = p3;
            slot[5 * gg + 3] = p1;
            slot[5 * gg + 4] = p2;
          }
        } else {
#pragma unroll
          for (int gg = 0; gg < GPP; gg++) {
            const float v = j0 + gg < G ? f16_bits_to_f32((uint16_t)ra[u][gg]) : 0.0f;   // an fp16 value: two pieces hold it
            const uint32_t p1 = hi16(v);
            const uint32_t p2 = hi16(v - __builtin_bit_cast(float, p1));
            slot[5 * gg + 0] = p1;
            slot[5 * gg + 1] = p1;
            slot[5 * gg + 2] = p1;
            slot[5 * gg + 3] = p2;
            slot[5 * gg + 4] = p2;
          }
        }
        fetch(u, j0 + 2 * GPP);                             // past the end: clamped, never used
        __syncthreads();                                    // the previous use of this LDS tile is over
#pragma unroll
        for (int c8 = 0; c8 < 8; c8++)
          *(uint4*)(smem + tile_off_bytes(t, c8)) =
              make_uint4(pair(slot[8 * c8], slot[8 * c8 + 1]), pair(slot[8 * c8 + 2], slot[8 * c8 + 3]),
                         pair(slot[8 * c8 + 4], slot[8 * c8 + 5]), pair(slot[8 * c8 + 6], slot[8 * c8 + 7]));
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
      };
      fetch(0, 0);
      fetch(1, GPP);
      for (int j0 = 0; j0 < G; j0 += 2 * GPP) {
#pragma unroll
        for (int u = 0; u < 2; u++)
          if (j0 + u * GPP < G) pass(u, j0 + u * GPP);
      }
    }
  }

  gemm_tail<OUT_F32>(acc, smem, xh, wh, bias, y, M, N, r, m0, n0, rowA, rowB);
}

template <int GS, bool OUT_F32, bool ASYM>
static int launch_one(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const uint16_t* zx,
                      const void* blob, const uint16_t* bias, int M, int N, int K, int r, void* y,
                      hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, GS);
  const char* bp = (const char*)blob;
  const int n_mt = (M + TM - 1) / TM, n_nt = (N + TN - 1) / TN;
  const long n_blocks = (long)n_mt * n_nt;
  const int per_xcd = (int)((n_blocks + 7) / 8);
  // (idempotent: two threads racing here would both set the same attribute)
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)w4a4_gemm_kernel<GS, OUT_F32, ASYM>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(GS));
    if (e != hipSuccess) return hip_failed(e);
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((w4a4_gemm_kernel<GS, OUT_F32, ASYM>), dim3(per_xcd * 8), dim3(NTHREADS), smem_bytes(GS), s, xh,
                     xl, sx, zx, (const uint16_t*)(bp + L.off_wh), (const uint8_t*)(bp + L.off_codes),
                     (const uint16_t*)(bp + L.off_sw), (const int16_t*)(bp + L.off_wsum), bias, M, N, K, r, y,
                     n_mt, n_nt, per_xcd);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

// Which of the three schedules runs a symmetric layer.  The wave-specialised kernel (persistent workgroups, one
// per CU, 256 x 128 tiles) is the fastest per tile; the kernel in this file (128 x 128 tiles, two workgroups per
// CU) spreads a medium problem over more CUs; with few tokens both leave most of the chip idle and the split-K
// kernel (64 x 64 outputs per workgroup, the K axis over its 8 waves) is the one with the shortest latency.
// Measured crossovers: about 128 of the 256 x 128 tiles; about 288 of the 64 x 64 ones (512 from K = 2048 on,
// 768 from K = 8192 on: the longer K is, the longer each workgroup of the tiled kernel walks alone).
// DIROTQ_W4A4_KERNEL=ws / tile / skinny in the environment forces one of them wherever it applies (the tests use
// it to run all of them on the same inputs).
enum class W4A4Schedule { kTile, kWs, kSkinny };
static W4A4Schedule w4a4_schedule(int M, int N, int K, int r) {
  if (K - r <= 0) return W4A4Schedule::kTile;
  if (const char* f = getenv("DIROTQ_W4A4_KERNEL")) {
    if (!strcmp(f, "ws")) return W4A4Schedule::kWs;
    if (!strcmp(f, "tile")) return W4A4Schedule::kTile;
    if (!strcmp(f, "skinny")) return W4A4Schedule::kSkinny;
  }
  const long big = (long)((M + 127) / 128) * ((N + 255) / 256);
  if (big >= 128) return W4A4Schedule::kWs;
  const long small = (long)((M + 63) / 64) * ((N + 63) / 64);
  return (small <= 288 || (small <= 512 && K >= 2048) || (small <= 768 && K >= 8192)) ? W4A4Schedule::kSkinny
                                                                                        : W4A4Schedule::kTile;
}

int launch_w4a4_gemm(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const uint16_t* zx,
                     const void* blob, const uint16_t* bias, int M, int N, int K, int r, int g, void* y,
                     int y_dtype, hipStream_t s) {
#define DIROTQ_CASE(GS)                                                                               \
  case GS:                                                                                            \
    if (zx)                                                                                           \
      return y_dtype ? launch_one<GS, true, true>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s)       \
                     : launch_one<GS, false, true>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s);     \
    return y_dtype ? launch_one<GS, true, false>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s)        \
                   : launch_one<GS, false, false>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s);
  {
    // (asymmetric layers: the wave-specialised schedule or this file's kernel; the few-token one has no
    // zero-point term)
    const W4A4Schedule sch = w4a4_schedule(M, N, K, r);
    if (sch == W4A4Schedule::kWs)
      return launch_w4a4_gemm_ws(xh, xl, sx, zx, blob, bias, M, N, K, r, g, y, y_dtype, s);
    if (sch == W4A4Schedule::kSkinny && !zx)
      return launch_w4a4_gemm_skinny(xh, xl, sx, blob, bias, M, N, K, r, g, y, y_dtype, s);
  }
  switch (g) {
    DIROTQ_CASE(32)
    DIROTQ_CASE(64)
    DIROTQ_CASE(128)
  }
#undef DIROTQ_CASE
  return DIROTQ_ERR_SHAPE;
}

}  // namespace dirotq

