// Kernel B, wave-specialised form (symmetric activation codes; the asymmetric ones: see the kernel's comment):
//   y = x_h W'_h^T + sum_j s_x[:,j] s_w[:,j]^T * (q_x,j q_w,j^T)
// (forward-computation equation of Section 4.2 of the paper).  Arithmetic as in w4a4_gemm.hip: codes run on the
// fp8 matrix pipe as exact subnormals, the scale product of a group comes from a small fp16 MFMA, one fma per
// accumulator and group applies it, the 16-bit branch runs on bf16 MFMAs.
//
// Why another schedule.  On this chip a wave issues in order, and two waves of the same kind on a SIMD mostly
// want the same issue port.  When every wave both stages operands (global loads, nibble unpacking, LDS stores)
// and multiplies, the waits of one are rarely covered by the other.  Here the two jobs belong to different
// waves: per SIMD, two "multiplying" waves whose instruction stream is nothing but MFMAs, the fma sweep and LDS
// operand reads, and one "staging" wave whose global loads and LDS stores issue through other ports and whose
// waits hurt nobody.
//
// Workgroup: 12 waves, one workgroup per CU.  Waves 0..7 multiply, as 4 (n) x 2 (tokens) blocks of 64 n x 64
// tokens (2 x 2 MFMA tiles each): tile 256 n x 128 tokens.  Waves 8..11 stage.  K is walked in stages held in a
// ring of four LDS buffers of [384 rows][64 B]: first the 16-bit branch (16 bf16 channels = 32 B of a row per
// stage, copied as they are), then the 4-bit channels (64 per stage: 32 packed bytes of a row, expanded from
// nibbles to 64 fp8 bytes).  Either kind of stage is 32 bytes per row in HBM, so a staging thread's loads have
// one shape: the stage's kind only selects base pointers, and whether the LDS store copies or expands.  The
// multiplying waves' accumulators are in the layer's own units from the start: the block-scaled form of the fp8
// MFMA multiplies both operands by 2^9, so a group dot comes back as the exact integer and both branches add
// into the same registers.  One barrier per stage; in interval s the multiplying waves work on stage s and read
// stage s+1 into operand registers as they fall free, the staging waves fill the slot stage s-1 has left with
// stage s+3 and reload their registers several stages ahead.
#include <algorithm>
#include <atomic>

#include "gemm_tail.h"

namespace dirotq {

namespace ws {

constexpr int TNW = 256, TMW = 128;          // output channels x tokens per workgroup tile
constexpr int ROWS = TNW + TMW;              // rows of a stage: weights, then tokens
constexpr int SB = 64;                       // bytes per row and stage
constexpr int NBUF = 4;                      // stages in the LDS ring
constexpr int nsets(int gs) { return gs == 32 ? 4 : 8; }   // stages of global loads in flight per staging thread
                                                           // (32-channel groups carry twice the scale registers)
constexpr int NMULT = 8, NSTAGE = 4;         // multiplying / staging waves
constexpr int NT = (NMULT + NSTAGE) * 64;
constexpr int STAGE_BYTES = ROWS * SB;       // 24 KB
constexpr int SCALE_OFF = NBUF * STAGE_BYTES;
constexpr int SROWS = ROWS + 8;              // scale rows per (stage, group): the real ones and a zero row (padded)
constexpr int gps(int gs) { return gs == 32 ? 2 : 1; }
constexpr int scale_stage_bytes(int gs) { return gps(gs) * SROWS * 8; }   // u64 {fp16 scale, 0, 0, 0} per row
// behind the rings: per multiplying wave, a [32 tokens][64 channels] bf16 block (rows padded to 144 B) through
// which finished outputs are turned from the accumulator layout (a lane holds one token) into whole rows
constexpr int OUT_ROW = 144, OUT_WAVE_BYTES = 32 * OUT_ROW;
constexpr int out_off(int gs) { return SCALE_OFF + NBUF * scale_stage_bytes(gs); }
constexpr int smem_bytes(int gs) { return out_off(gs) + NMULT * OUT_WAVE_BYTES; }

// 16-B chunk c of row r sits in slot c ^ ((r >> 2) & 3): the 16 rows that a 16-byte LDS access serves per cycle
// fall into 16 different slots of a 256-byte bank line
__device__ __forceinline__ int stage_off(int row, int chunk) { return row * SB + ((chunk ^ ((row >> 2) & 3)) << 4); }

// 8 sign-magnitude nibbles of a dword -> two dwords of fp8 (E4M3) bytes [s 0000 mmm] = +-m * 2^-9: even, odd channels
__device__ __forceinline__ void unpack8(uint32_t p, uint32_t& even, uint32_t& odd) {
  even = (p & 0x07070707u) | ((p & 0x08080808u) << 4);
  odd = ((p >> 4) & 0x07070707u) | (p & 0x80808080u);
}

// 8 unsigned nibbles (asymmetric activations) -> fp8 bytes u * 2^-9, exact for u = 0..15
__device__ __forceinline__ void unpack8u(uint32_t p, uint32_t& even, uint32_t& odd) {
  even = p & 0x0F0F0F0Fu;
  odd = (p >> 4) & 0x0F0F0F0Fu;
}

typedef __attribute__((ext_vector_type(8))) int i32x8;

// bf16 store of a wave's 64 x 64 block whose output channels all exist (N a multiple of 8): in the accumulator
// layout a store instruction would touch 32 rows with 16 bytes each; via the wave's LDS block it writes 8 rows of
// 128 contiguous bytes.  tb: the wave's own LDS block (no other wave touches it: no barrier).
__device__ __forceinline__ void store_block_rows(const f32x16 (&acc)[2][2], const uint16_t* __restrict__ bias,
                                                 uint16_t* __restrict__ y, int M, int N, int m_base, int n_base,
                                                 unsigned char* tb) {
  int l = threadIdx.x & 63;
  asm volatile("" : "+v"(l));   // (addresses below are formed here, per tile: not carried in registers through the loops)
  const int h = l >> 5;
  unsigned char* wr = tb + (l & 31) * OUT_ROW + 8 * h;          // this lane's token row, channel 4 h
  const unsigned char* rd = tb + (l >> 3) * OUT_ROW + (l & 7) * 16;   // row l >> 3 (+ 8 k), channels 8 (l & 7) ..
  uint16_t* dst = y + (size_t)(m_base + (l >> 3)) * N + n_base + 8 * (l & 7);
#pragma unroll
  for (int j = 0; j < 2; j++) {
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        if (bias) {
          const uint2 bb = *(const uint2*)(bias + n_base + i * 32 + 8 * q + 4 * h);
          v[0] += bf16_bits_to_f32((uint16_t)(bb.x & 0xFFFF));
          v[1] += bf16_bits_to_f32((uint16_t)(bb.x >> 16));
          v[2] += bf16_bits_to_f32((uint16_t)(bb.y & 0xFFFF));
          v[3] += bf16_bits_to_f32((uint16_t)(bb.y >> 16));
        }
        uint2 o;
        o.x = f32x2_to_bf16x2_bits(v[0], v[1]);
        o.y = f32x2_to_bf16x2_bits(v[2], v[3]);
        *(uint2*)(wr + (i * 32 + 8 * q) * 2) = o;
      }
#pragma unroll
    for (int k = 0; k < 4; k++) {
      const uint4 d = *(const uint4*)(rd + k * 8 * OUT_ROW);
      if (m_base + j * 32 + k * 8 + (l >> 3) < M) *(uint4*)(dst + (size_t)(j * 32 + k * 8) * N) = d;
    }
  }
}

// first output channel / token of the logical tile `logical`: within an XCD's run of consecutive logical tiles,
// GN output tiles are swept per token tile (shared operands stay in that XCD's L2)
__device__ __forceinline__ void tile_origin(int logical, int n_mt, int n_nt, int& m0, int& n0) {
  constexpr int GN = 2;
  const int grp = logical / (GN * n_mt), in_grp = logical % (GN * n_mt);
  const int gn = min(n_nt - grp * GN, GN);
  n0 = (grp * GN + in_grp % gn) * TNW;
  m0 = (in_grp / gn) * TMW;
}

// Persistent workgroups: gridDim.x = 8 * wpx; workgroup b runs on XCD b & 7 and takes, of that XCD's run of
// per_xcd consecutive logical tiles, the tiles (b >> 3) + it * wpx, it = 0, 1, ...  The stage stream is continuous
// across a workgroup's tiles: the staging waves are loading the next tile while the multiplying waves finish and
// store the current one.
//
// Asymmetric activations (ASYM): the codes of the token rows are unsigned nibbles, and the zero-point term
// sum_j z[m,j] (s_w[n,j] sum_k q_w[n,k]) follows each tile's 4-bit stages as nzp more 16-bit stages whose rows the
// staging waves form on the fly: per group five k-slots, weight rows b1 b2 b3 b1 b2, token rows z1 z1 z1 z2 z2,
// with z = z1 + z2 and s_w sum q_w = b1 + b2 + b3 exact bf16 splits (only z2 b3, below 2^-24 of the term, is
// dropped); six groups per stage (both 16-byte chunks of a lane's operand, two MFMAs per tile).
template <int GS, bool OUT_F32, bool ASYM>
__global__ __launch_bounds__(NT, 1) void w4a4_gemm_ws_kernel(
    const uint16_t* __restrict__ xh, const uint8_t* __restrict__ xl, const uint16_t* __restrict__ sx,
    const uint16_t* __restrict__ zx, const uint16_t* __restrict__ wh, const uint8_t* __restrict__ wq,
    const uint16_t* __restrict__ sw, const int16_t* __restrict__ wsum, const uint16_t* __restrict__ bias, int M, int N,
    int K, int r, void* __restrict__ y, int n_mt, int n_nt, int per_xcd, int wpx) {
  extern __shared__ __align__(16) unsigned char smem[];

  const int run0 = (blockIdx.x & 7) * per_xcd, first = blockIdx.x >> 3;
  const int run_len = min(per_xcd, n_mt * n_nt - run0);
  if (first >= run_len) return;
  const int T = (run_len - first + wpx - 1) / wpx;                    // tiles of this workgroup (>= 1)

  const int w_s = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index as a scalar
  const int KL = K - r;                                               // number of 4-bit channels (> 0)
  const int G = KL / GS;
  constexpr int GPS = gps(GS);
  constexpr int SSB = scale_stage_bytes(GS);
  // stages of a tile: nbf of the 16-bit branch (16 channels each; padded with zero stages to a multiple of 4),
  // then nq of the 4-bit part (64 channels each; padded to a multiple of 4: the extra ones have zero scales)
  const int nbf_real = r / 16, nbf = (nbf_real + 3) / 4 * 4;
  const int nq_real = (KL + 63) / 64, nq = (nq_real + 3) / 4 * 4;
  const int nst = nbf + nq;
  // zero-point stages of a tile (ASYM): 6 groups each, padded to a multiple of 4 (the ring's period, and the
  // period of the staging waves' register sets: the stage stream of the next tile meets them in the same phase)
  const int nzp = ASYM ? ((G + 5) / 6 + 3) / 4 * 4 : 0;

  // ================= staging waves: HBM -> registers -> LDS ring =================
  if (w_s >= NMULT) {
    const int t = threadIdx.x - NMULT * 64;              // 0..255
    // The staging waves are the youngest of the workgroup and would issue last whenever a multiplying wave has
    // an instruction ready, reaching each barrier late with the matrix pipe idle meanwhile: they go first instead.
    __builtin_amdgcn_s_setprio(3);
    // zero rows of the scale ring (read by lanes 32..63: k-slots 4..7 of the scale-product MFMA)
    if (t < NBUF * GPS * 8)
      *(uint2*)(smem + SCALE_OFF + (t >> 3) * (SROWS * 8) + (ROWS + (t & 7)) * 8) = make_uint2(0u, 0u);
    // A stage is 384 rows x 32 B in HBM.  Thread t owns, of every stage, the 16-B half (t & 1) of rows
    // (t >> 1) + 128 u, u = 0..2 (u < 2: weights, u = 2: tokens), and for 4-bit stages the scales of rows t
    // (weights) and 256 + (t & 127) (tokens).
    const int ldq = KL / 2;
    const int half = t & 1;
    int soq[3], sob[3];                                  // LDS offsets within a slot: expanded / copied
#pragma unroll
    for (int u = 0; u < 3; u++) {
      const int row = (t >> 1) + 128 * u;                // 0..383
      soq[u] = stage_off(row, 2 * half);
      sob[u] = stage_off(row, half);
    }
    const int sos_w = SCALE_OFF + t * 8, sos_x = SCALE_OFF + (TNW + (t & 127)) * 8;
    // (a last 4-bit stage of 32 channels, possible for 32-channel groups only: both halves read the one that exists)
    const bool short_last = GS == 32 && (KL % 64) != 0;

    // load cursor: the tile and stage the next load is for.  Uniform bases of the tile; per-lane byte offsets
    // from them (below 2^31: a tile's rows span at most 256 rows of at most 2^19 bytes)
    const uint8_t *wq_b, *xl_b, *wh_b, *xh_b;
    const uint16_t *sw_b, *sx_b;
    uint32_t voq[3], vob[3], vos_w, vos_x;
    int lt = 0, lst = 0;
    auto set_tile = [&](int it) {
      int m0, n0;
      tile_origin(run0 + first + it * wpx, n_mt, n_nt, m0, n0);
      wq_b = wq + (size_t)n0 * ldq;
      xl_b = xl + (size_t)m0 * ldq;
      wh_b = (const uint8_t*)(wh + (size_t)n0 * r);
      xh_b = (const uint8_t*)(xh + (size_t)m0 * r);
      sw_b = sw + n0;
      sx_b = sx + m0;
#pragma unroll
      for (int u = 0; u < 3; u++) {
        const int row = (t >> 1) + 128 * u;
        const uint32_t ro =
            row < TNW ? (uint32_t)(min(n0 + row, N - 1) - n0) : (uint32_t)(min(m0 + row - TNW, M - 1) - m0);
        voq[u] = ro * (uint32_t)ldq + half * 16;
        vob[u] = ro * (uint32_t)(2 * r) + half * 16;
      }
      vos_w = 2u * (uint32_t)(min(n0 + t, N - 1) - n0);
      vos_x = 2u * (uint32_t)(min(m0 + (t & 127), M - 1) - m0);
    };
    set_tile(0);

    // register sets: one stage each.  Loads are straight-line code of one shape, whatever the stage's kind, so
    // that the count of loads in flight is exact and a store waits for its own set only.
    constexpr int NSETS = ASYM ? 4 : nsets(GS);          // (ASYM keeps registers free for the zero-point stages)
    uint4 rg[NSETS][3];
    uint16_t rsw[NSETS][GPS], rsx[NSETS][GPS];
    auto gload = [&](int set) {                          // loads the cursor's stage, then moves the cursor on
      const int st = lst;
      const bool is_b = st < nbf;
      const int sq = max(st - nbf, 0);
      const int sc = is_b ? min(st, max(nbf_real - 1, 0)) : min(sq, nq_real - 1);
      const uint8_t* wb = (is_b ? wh_b : wq_b) + (size_t)sc * 32;
      const uint8_t* xb = (is_b ? xh_b : xl_b) + (size_t)sc * 32;
      const bool last = short_last && !is_b && sq >= nq_real - 1;
#pragma unroll
      for (int u = 0; u < 3; u++) {
        uint32_t off = is_b ? vob[u] : voq[u];
        if (GS == 32) off -= last ? half * 16 : 0;
        rg[set][u] = *(const uint4*)((u < 2 ? wb : xb) + off);
      }
#pragma unroll
      for (int jj = 0; jj < GPS; jj++) {
        const int j = GS == 128 ? sq >> 1 : sq * GPS + jj;          // group of these channels
        const size_t jc = (size_t)min(j, G - 1);
        rsw[set][jj] = *(const uint16_t*)((const uint8_t*)(sw_b + jc * N) + vos_w);
        rsx[set][jj] = *(const uint16_t*)((const uint8_t*)(sx_b + jc * M) + vos_x);
      }
      if (++lst == nst) {                                // (past the last tile: its stages are read again, unused)
        lst = 0;
        if (lt + 1 < T) set_tile(++lt);
      }
    };
    int sst = 0;                                         // store cursor: stage within its tile
    int stiles = 0;                                      // tiles whose regular stages have all been stored
    auto sstore = [&](int slot, int set) {
      const int st = sst;
      unsigned char* sb = smem + slot * STAGE_BYTES;
      if (st < nbf) {
        const bool real = st < nbf_real;                 // padding stages of the 16-bit branch hold zeros
#pragma unroll
        for (int u = 0; u < 3; u++) *(uint4*)(sb + sob[u]) = real ? rg[set][u] : make_uint4(0u, 0u, 0u, 0u);
      } else {
#pragma unroll
        for (int u = 0; u < 3; u++) {
          uint4 e, o;
          if (ASYM && u == 2) {                          // token rows: unsigned codes
            unpack8u(rg[set][u].x, e.x, o.x);
            unpack8u(rg[set][u].y, e.y, o.y);
            unpack8u(rg[set][u].z, e.z, o.z);
            unpack8u(rg[set][u].w, e.w, o.w);
          } else {
            unpack8(rg[set][u].x, e.x, o.x);
            unpack8(rg[set][u].y, e.y, o.y);
            unpack8(rg[set][u].z, e.z, o.z);
            unpack8(rg[set][u].w, e.w, o.w);
          }
          *(uint4*)(sb + soq[u]) = e;
          *(uint4*)(sb + (soq[u] ^ 16)) = o;
        }
        // groups past the end (padding stages, the empty half of a short last stage) get zero scales: their codes
        // are a re-read of real ones and contribute exactly nothing
#pragma unroll
        for (int jj = 0; jj < GPS; jj++) {
          const int sq = st - nbf;
          const int j = GS == 128 ? sq >> 1 : sq * GPS + jj;
          const uint32_t keep = j < G ? 0xFFFFu : 0u;
          *(uint2*)(smem + sos_w + slot * SSB + jj * (SROWS * 8)) = make_uint2(rsw[set][jj] & keep, 0u);
          if (t < TMW) *(uint2*)(smem + sos_x + slot * SSB + jj * (SROWS * 8)) = make_uint2(rsx[set][jj] & keep, 0u);
        }
      }
      if (++sst == nst) {
        sst = 0;
        stiles++;
      }
    };
    // The zero-point stages of tile `it` (ASYM): nzp intervals, each one stage into the ring and one barrier, like
    // the regular intervals around them.  Thread t forms, for its three rows, the 16 k-slots of its half of the
    // row: groups 6 z + 3 half + {0, 1, 2} and a zero slot.  The factors of stage z + 1 are fetched while stage z
    // is formed (two small register sets; the regular stages' sets keep their loads meanwhile).
    int zdone = 0;
    size_t zcol[3];                                      // the thread's rows of the tile: output channels, token
    uint16_t fa[2][3][3];                                // s_w bits (weight rows) or z bits (token row)
    int16_t fb[2][2][3];                                 // code sums (weight rows)
    auto zp_fetch = [&](int buf, int z) {
#pragma unroll
      for (int gg = 0; gg < 3; gg++) {
        const size_t jc = (size_t)min(6 * z + 3 * half + gg, G - 1);
        fa[buf][0][gg] = sw[jc * N + zcol[0]];
        fb[buf][0][gg] = wsum[jc * N + zcol[0]];
        fa[buf][1][gg] = sw[jc * N + zcol[1]];
        fb[buf][1][gg] = wsum[jc * N + zcol[1]];
        fa[buf][2][gg] = zx[jc * M + zcol[2]];
      }
    };
    auto zp_phase = [&](int it) {
      {
        int m0, n0;
        tile_origin(run0 + first + it * wpx, n_mt, n_nt, m0, n0);
#pragma unroll
        for (int u = 0; u < 3; u++) {
          const int row = (t >> 1) + 128 * u;
          zcol[u] = row < TNW ? (size_t)min(n0 + row, N - 1) : (size_t)min(m0 + row - TNW, M - 1);
        }
        zp_fetch(0, 0);
      }
      // v = p1 + p2 + p3 with each piece a bf16 number: truncating splits (exact, the residuals need no rounding)
      auto hi16 = [](float v) { return __builtin_bit_cast(uint32_t, v) & 0xFFFF0000u; };
      auto fill = [&](int slot, int buf, int z) {
        unsigned char* sb = smem + slot * STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < 3; u++) {
          uint32_t k16[16];                              // the 16 k-slots as fp32 bits with the low half clear
          k16[15] = 0u;
#pragma unroll
          for (int gg = 0; gg < 3; gg++) {
            const bool live = 6 * z + 3 * half + gg < G;
            if (u < 2) {
              const float v = live ? f16_bits_to_f32(fa[buf][u][gg]) * (float)fb[buf][u][gg] : 0.0f;
              const uint32_t p1 = hi16(v);
              const float r1 = v - __builtin_bit_cast(float, p1);
              const uint32_t p2 = hi16(r1);
              const uint32_t p3 = hi16(r1 - __builtin_bit_cast(float, p2));
              k16[5 * gg + 0] = p1;
              k16[5 * gg + 1] = p2;
              k16[5 * gg + 2] = p3;
              k16[5 * gg + 3] = p1;
              k16[5 * gg + 4] = p2;
            } else {
              const float v = live ? f16_bits_to_f32(fa[buf][2][gg]) : 0.0f;   // an fp16 value: two pieces hold it
              const uint32_t p1 = hi16(v);
              const uint32_t p2 = hi16(v - __builtin_bit_cast(float, p1));
              k16[5 * gg + 0] = p1;
              k16[5 * gg + 1] = p1;
              k16[5 * gg + 2] = p1;
              k16[5 * gg + 3] = p2;
              k16[5 * gg + 4] = p2;
            }
          }
          auto pair = [&](int a) { return (k16[a] >> 16) | k16[a + 1]; };    // two bf16 slots in a dword
          *(uint4*)(sb + soq[u]) = make_uint4(pair(0), pair(2), pair(4), pair(6));
          *(uint4*)(sb + (soq[u] ^ 16)) = make_uint4(pair(8), pair(10), pair(12), pair(14));
        }
      };
      for (int z0 = 0; z0 < nzp; z0 += 4) {
#pragma unroll
        for (int k = 0; k < 4; k++) {
          zp_fetch((k + 1) & 1, z0 + k + 1);             // (past the end: clamped, unused)
          fill(k, k & 1, z0 + k);
          __syncthreads();
        }
      }
    };
    // stages 0..NSETS-1 into the register sets; stages 0..2 on into ring slots 0..2, their sets reloaded
#pragma unroll
    for (int u = 0; u < NSETS; u++) gload(u);
#pragma unroll
    for (int u = 0; u < 3; u++) {
      sstore(u, u);
      gload(u);
    }
    __syncthreads();
    // interval s: stage s + 3 goes into the slot stage s - 1 has left; its register set takes stage s + 3 + NSETS
    static_assert(NSETS % NBUF == 0, "the unrolled period below serves both rings");
    const int n_intervals = T * nst;                     // (a multiple of NBUF)
    for (int s0 = 0; s0 < n_intervals; s0 += NSETS) {
#pragma unroll
      for (int k = 0; k < NSETS; k++) {
        if (k > 0 && k % NBUF == 0 && s0 + k >= n_intervals) break;
        if constexpr (ASYM) {
          // the store cursor stands at the first stage of a tile: the zero-point stages of the tile before it
          // come first (also behind the last tile: the cursor wraps for the stages that nobody reads)
          if ((k + 3) % NBUF == 0 && sst == 0 && stiles > zdone) zp_phase(zdone++);
        }
        sstore((k + 3) % NBUF, (k + 3) % NSETS);
        gload((k + 3) % NSETS);
        __syncthreads();
      }
    }
    return;
  }

  // ================= multiplying waves: 2 x 2 tiles of 32 n x 32 tokens each =================
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int wn = w & 3, wt = w >> 2;
  const int h = l >> 5;

  // operand registers (refilled in place from the next stage as they fall free): the lane's 32 bytes of its row
  // (lo / hi 16 bytes) for 2 weight tiles and 2 token tiles, and the scales as fp16 vectors {s, 0, 0, 0}
  i32x4 a[2][2], b[2][2];
  f16x4 sa[2][GPS], sb[2][GPS];
  const int rA = wn * 64 + (l & 31), rB = TNW + wt * 64 + (l & 31);
  const int sw4 = ((l & 31) >> 2) & 3;                 // tile bases are multiples of 32 rows
  const int adA_lo = rA * SB + ((h ^ sw4) << 4), adA_hi = rA * SB + (((2 + h) ^ sw4) << 4);
  const int adB_lo = rB * SB + ((h ^ sw4) << 4), adB_hi = rB * SB + (((2 + h) ^ sw4) << 4);
  const int soA = SCALE_OFF + (h ? ROWS : rA) * 8, soB = SCALE_OFF + (h ? ROWS : rB) * 8;
  const int so_step = h ? 0 : 32 * 8;                  // second tile: 32 rows further (the zero row stays)
  auto read_a = [&](int i, int slot) {
    const unsigned char* sp = smem + slot * STAGE_BYTES + i * (32 * SB);
    a[i][0] = *(const i32x4*)(sp + adA_lo);
    a[i][1] = *(const i32x4*)(sp + adA_hi);
#pragma unroll
    for (int jj = 0; jj < GPS; jj++)
      sa[i][jj] = *(const f16x4*)(smem + soA + i * so_step + slot * SSB + jj * (SROWS * 8));
  };
  auto read_b = [&](int j, int slot) {
    const unsigned char* sp = smem + slot * STAGE_BYTES + j * (32 * SB);
    b[j][0] = *(const i32x4*)(sp + adB_lo);
    b[j][1] = *(const i32x4*)(sp + adB_hi);
#pragma unroll
    for (int jj = 0; jj < GPS; jj++)
      sb[j][jj] = *(const f16x4*)(smem + soB + j * so_step + slot * SSB + jj * (SROWS * 8));
  };
  // (In the 16-bit phase the upper halves and the scale words read here are not used: whatever the slot holds.)
  // tile order within a stage alternates so that an operand is refilled at least one tile before its next use:
  // (0,0) (0,1) (1,1) (1,0) in even stages, (0,1) (0,0) (1,0) (1,1) in odd ones
  auto tile_i = [](int u) { return u >> 1; };
  auto tile_j = [](int odd, int u) { return odd ? (u == 0 || u == 3) : (u == 1 || u == 2); };
  // after the MFMAs of tile u (of the stage's last pass) have been issued, these operands are free
  auto refill = [&](int odd, int u, int nslot) {
    if (u == 1) read_a(0, nslot);
    if (u == 2) read_b(odd ? 0 : 1, nslot);
    if (u == 3) {
      read_a(1, nslot);
      read_b(odd ? 1 : 0, nslot);
    }
  };

  __syncthreads();                                     // stages 0..2 are in the ring
  read_a(0, 0);
  read_b(0, 0);
  read_a(1, 0);
  read_b(1, 0);

  for (int it = 0; it < T; it++) {
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] = 0.0f;

    // ---- 16-bit branch: acc += W'_h x_h^T, one bf16 MFMA (16 channels) per tile and stage ----
    for (int s0 = 0; s0 < nbf; s0 += 4) {
#pragma unroll
      for (int k = 0; k < 4; k++) {
        const int odd = k & 1, nslot = (k + 1) % NBUF;
#pragma unroll
        for (int u = 0; u < 4; u++) {
          const int i = tile_i(u), j = tile_j(odd, u);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i][0]),
                                                              __builtin_bit_cast(bf16x8, b[j][0]), acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          refill(odd, u, nslot);
          __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_barrier();
      }
    }

    // ---- 4-bit branch ----
    const int sc9 = 127 + 9;                             // E8M0 block scale 2^9 on both operands: the dot is the integer
    for (int s0 = 0; s0 < nq; s0 += 4) {
#pragma unroll
      for (int k = 0; k < 4; k++) {
        const int odd = k & 1, nslot = (k + 1) % NBUF;
#pragma unroll
        for (int q = 0; q < 4 * GPS; q++) {
          const int u = q & 3, jj = q >> 2;
          const int i = tile_i(u), j = tile_j(odd, u);
          const i32x4 zero4 = {0, 0, 0, 0};
          f32x16 z, p;
#pragma unroll
          for (int v = 0; v < 16; v++) z[v] = p[v] = 0.0f;
          const i32x8 av = GS == 32 ? __builtin_shufflevector(a[i][jj], zero4, 0, 1, 2, 3, 4, 5, 6, 7)
                                    : __builtin_shufflevector(a[i][0], a[i][1], 0, 1, 2, 3, 4, 5, 6, 7);
          const i32x8 bv = GS == 32 ? __builtin_shufflevector(b[j][jj], zero4, 0, 1, 2, 3, 4, 5, 6, 7)
                                    : __builtin_shufflevector(b[j][0], b[j][1], 0, 1, 2, 3, 4, 5, 6, 7);
          const f32x16 I = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, z, 0, 0, 0, sc9, 0, sc9);
          const f32x16 P = __builtin_amdgcn_mfma_f32_32x32x8f16(sa[i][jj], sb[j][jj], p, 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (jj == GPS - 1) refill(odd, u, nslot);            // behind this tile's MFMAs, ahead of their results
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int v = 0; v < 16; v++) acc[i][j][v] = fmaf(I[v], P[v], acc[i][j][v]);
          __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_barrier();
      }
    }

    // ---- zero-point term (ASYM): 32 k-slots per stage, two bf16 MFMAs per tile ----
    if constexpr (ASYM) {
      for (int s0 = 0; s0 < nzp; s0 += 4) {
#pragma unroll
        for (int k = 0; k < 4; k++) {
          const int odd = k & 1, nslot = (k + 1) % NBUF;
#pragma unroll
          for (int u = 0; u < 4; u++) {
            const int i = tile_i(u), j = tile_j(odd, u);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i][0]),
                                                                __builtin_bit_cast(bf16x8, b[j][0]), acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i][1]),
                                                                __builtin_bit_cast(bf16x8, b[j][1]), acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            refill(odd, u, nslot);
            __builtin_amdgcn_sched_barrier(0);
          }
          __builtin_amdgcn_s_barrier();
        }
      }
    }

    int m0, n0;
    tile_origin(run0 + first + it * wpx, n_mt, n_nt, m0, n0);
    if (!OUT_F32 && (N & 7) == 0 && n0 + wn * 64 + 64 <= N)
      store_block_rows(acc, bias, (uint16_t*)y, M, N, m0 + wt * 64, n0 + wn * 64, smem + out_off(GS) + w * OUT_WAVE_BYTES);
    else
      store_tile<OUT_F32>(acc, bias, y, M, N, m0 + wt * 64, n0 + wn * 64);
  }
}

template <int GS, bool OUT_F32, bool ASYM>
static int launch_one(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const uint16_t* zx, const void* blob,
                      const uint16_t* bias, int M, int N, int K, int r, void* y, hipStream_t s) {
  const BlobLayout L = blob_layout(N, K, r, GS);
  const char* bp = (const char*)blob;
  const int n_mt = (M + TMW - 1) / TMW, n_nt = (N + TNW - 1) / TNW;
  const long n_blocks = (long)n_mt * n_nt;
  if (n_blocks > 0x7FFFFFFFL) return DIROTQ_ERR_SHAPE;
  const int per_xcd = (int)((n_blocks + 7) / 8);
  int cus = 0;                                           // workgroups per XCD: one per CU, or fewer tiles than that
  {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_failed(e);
  }
  const int wpx = std::max(1, std::min(cus / 8, per_xcd));
  // (idempotent: two threads racing here would both set the same attribute)
  static std::atomic<bool> attr_done{false};
  if (!attr_done.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)w4a4_gemm_ws_kernel<GS, OUT_F32, ASYM>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(GS));
    if (e != hipSuccess) return hip_failed(e);
    attr_done.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((w4a4_gemm_ws_kernel<GS, OUT_F32, ASYM>), dim3(wpx * 8), dim3(NT), smem_bytes(GS), s, xh, xl, sx,
                     zx, (const uint16_t*)(bp + L.off_wh), (const uint8_t*)(bp + L.off_codes),
                     (const uint16_t*)(bp + L.off_sw), (const int16_t*)(bp + L.off_wsum), bias, M, N, K, r, y, n_mt,
                     n_nt, per_xcd, wpx);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? DIROTQ_OK : hip_failed(e);
}

}  // namespace ws

int launch_w4a4_gemm_ws(const uint16_t* xh, const uint8_t* xl, const uint16_t* sx, const uint16_t* zx, const void* blob,
                        const uint16_t* bias, int M, int N, int K, int r, int g, void* y, int y_dtype, hipStream_t s) {
#define DIROTQ_WS_CASE(GS)                                                                                 \
  case GS:                                                                                                 \
    if (zx)                                                                                                \
      return y_dtype ? ws::launch_one<GS, true, true>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s)        \
                     : ws::launch_one<GS, false, true>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s);      \
    return y_dtype ? ws::launch_one<GS, true, false>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s)         \
                   : ws::launch_one<GS, false, false>(xh, xl, sx, zx, blob, bias, M, N, K, r, y, s);
  switch (g) {
    DIROTQ_WS_CASE(32)
    DIROTQ_WS_CASE(64)
    DIROTQ_WS_CASE(128)
  }
#undef DIROTQ_WS_CASE
  return DIROTQ_ERR_SHAPE;
}

}  // namespace dirotq
