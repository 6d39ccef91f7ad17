// Projections of the attention module (paper App. B.5: "qkv proj", "o proj")
// and of the MLP module: C[M, N] = act(A[M, K] W[N, K]^T + bias[N]),
// activations and weights bf16, fp32 accumulation on the matrix core, one
// rounding to bf16 on the way out; act is nothing or the MLP's GELU.
//
// Both operands are contiguous along K, which is what the MFMA operands want:
// with the weight rows as the A operand and the token rows as the B operand a
// 32x32 tile is C^T[n, m], every lane owns one token and 16 of its outputs.
//
// One workgroup of WM x WN wavefronts computes a BM-token x BN-feature tile,
// each wavefront TM x TN MFMA tiles of it.  The K dimension streams through a
// ring of NST LDS stages of 32 columns: BM token rows and BN weight rows of 64
// bytes each per stage, copied global -> LDS directly (16 bytes per lane)
// NST-1 stages ahead of their use, one barrier per stage.
//
// Rows are 64 bytes, so rows r and r + 4 start in the same bank and the four 16-byte chunks of a
// row are stored permuted: chunk q at position q ^ swz(r).  A 16-byte LDS read is served in four
// cycles of 16 lanes, and these are lanes {0-3, 12-15, 20-23, 24-27}, then {4-7, 8-11, 16-19,
// 28-31}, and the same in the upper half (measured with the bank conflict counter).  With the
// 16 x 16 x 32 operands (lane = 16 chunk + row) a cycle therefore mixes chunk c of rows 0-3 and
// 12-15 with chunk c + 1 of rows 4-11; swz(r) = (r >> 2) & 2 sends the four row quads of a cycle
// to four different bank groups.  With the 32 x 32 x 16 operands (lane = 32 chunk + row) a cycle
// holds one chunk of rows 0-3, 12-15, 20-23, 24-27 and swz(r) = (r >> 2) & 3 does the same.
//
// Workgroup ids go round-robin over the 8 XCDs; an XCD owns every eighth token
// tile and walks its tiles four token tiles at a time across all feature tiles,
// so that the weight rows in flight are shared by four workgroups and a token
// tile's rows by all of its feature tiles inside one L2.  With fewer than eight
// token tiles that order would leave XCDs idle; the tiles are then simply
// numbered feature-major (and the host picks a narrower feature tile so that
// the few token rows still spread over the chip).
#pragma once
#include "mfma_util.hpp"

namespace pab {

struct GemmParams {
  const bf16_t *A;      // [M, K]
  const bf16_t *W;      // [N, K]
  const bf16_t *bias;   // [N] or nullptr
  void *C;              // bf16; feature n of token m goes to C[(n / n_split) * plane_stride + m * ldc + n % n_split]
  int M, N, K;
  long long ldc;        // row pitch of C in elements
  int n_split;          // features per output plane (N: one plane; a multiple of 4)
  long long plane_stride;
  int act;              // 0: none; 1: GELU in its tanh form, applied after the bias
  int n_mt, n_nt;       // token / feature tiles
  int xcd_map;          // 1: the XCD-aware tile order below; 0: tile = blockIdx.x (few token tiles)
};

// NST: ring depth.  WM x WN wavefronts per workgroup, each computing TM x TN MFMA tiles of 32 x 32
// (tokens x features): the workgroup tile is BM = 32 WM TM tokens by BN = 32 WN TN features.
// MF: edge of the MFMA tile, 32 (v_mfma_f32_32x32x16_bf16, two per 32-column slice) or 16
// (v_mfma_f32_16x16x32_bf16, one per slice and 16 x 16 sub-tile; it moves half the accumulator
// data per multiply-add and sustains about 12% more under the power limit).
template <int NST, int WM, int WN, int TM, int TN, int MF>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bias_kernel(const GemmParams p) {
  static_assert(MF == 32 || MF == 16, "MFMA tile edge");
  constexpr int NW = WM * WN;
  constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN, BK = 32;
  constexpr int ROWS = BM + BN;                 // rows per stage: token rows, then weight rows
  constexpr int STAGE_ELEMS = ROWS * BK;
  constexpr int ROUNDS = ROWS * 4 / 64;         // 64-chunk copy rounds per stage (16 rows each)
  constexpr int MYR = ROUNDS / NW;              // per wavefront
  constexpr int MYR_TOK = BM / 16 / NW;         // ... of which token rows (round r = wave + NW i: i < MYR_TOK)
  constexpr int GM = 4;                         // token tiles an XCD keeps in flight together
  static_assert(NST >= 3 && (NST - 2) * MYR < 16, "ring depth / vmcnt immediates");
  static_assert(ROUNDS % NW == 0 && (BM / 16) % NW == 0, "copy rounds must deal evenly to the wavefronts");

  __shared__ __attribute__((aligned(16))) bf16_t smem[NST * STAGE_ELEMS];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31, g = lane >> 5;
  // chunk q of stage row r is stored at position q ^ swz(r) of the row (see the header)
  auto swz = [](int row) { return MF == 32 ? (row >> 2) & 3 : (row >> 2) & 2; };
  const int wm = wave / WN, wn = wave % WN;
  const unsigned smem_addr = (unsigned)(size_t)((__attribute__((address_space(3))) char *)smem);

  // ---- which tile ----
  int mt_id, nt_id;
  if (p.xcd_map) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per_group = GM * p.n_nt;
    const int grp = slot / per_group, rem = slot % per_group;
    nt_id = rem / GM;
    mt_id = 8 * (grp * GM + rem % GM) + xcd;
  } else {
    nt_id = blockIdx.x % p.n_nt;
    mt_id = blockIdx.x / p.n_nt;
  }
  if (mt_id >= p.n_mt) return;
  const int m0 = mt_id * BM, n0 = nt_id * BN;
  const int M = p.M, N = p.N, K = p.K;

  // ---- staging: round r = wave + 4 i covers rows 16 r .. 16 r + 15 of the stage; lane's chunk slot
  //      64 r + lane holds (row, chunk q) with q = (lane & 3) ^ swz(row).  Rows past the
  //      matrix re-read its last row; what they produce is never stored. ----
  unsigned voff[MYR];
#pragma unroll
  for (int i = 0; i < MYR; ++i) {
    const int r = wave + NW * i;
    const int row = 16 * r + (lane >> 2);
    const int q = (lane & 3) ^ swz(row);
    long long grow;
    if (i < MYR_TOK) grow = min(m0 + row, M - 1);    // token rows
    else grow = min(n0 + row - BM, N - 1);           // weight rows
    voff[i] = (unsigned)(2 * (grow * K + 8 * q));
  }
  auto issue = [&](int kt, int stage) {
#pragma unroll
    for (int i = 0; i < MYR; ++i) {
      const int r = wave + NW * i;
      dma16_to_lds((i < MYR_TOK ? p.A : p.W) + (long long)kt * BK, voff[i], smem_addr + 2 * stage * STAGE_ELEMS + 1024 * r);
    }
  };
  auto wait_staged = [&](int stages) {   // at most `stages` of this wavefront's staged K slices still in flight
    if (stages >= 2) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * MYR));
    else if (stages == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | MYR);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
  };

  const int nk = K / BK;
  const int npre = nk < NST - 1 ? nk : NST - 1;
  for (int kt = 0; kt < npre; ++kt) issue(kt, kt);

  f32x16 acc[TM][TN];                 // MF == 32: one 32 x 32 tile each
  f32x4 acc16[2 * TM][2 * TN];        // MF == 16: 16 x 16 sub-tiles
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
#pragma unroll
  for (int a = 0; a < 2 * TM; ++a)
#pragma unroll
    for (int b = 0; b < 2 * TN; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc16[a][b][r] = 0.0f;
  const int l16 = lane & 15, q16 = lane >> 4;   // MF == 16: row inside a sub-tile, 8-column chunk of the slice

  // fragment addresses inside a stage (elements): row * 32 + 8 * (chunk ^ swizzle(row))
  int tok_row[TM], w_row[TN];
#pragma unroll
  for (int a = 0; a < TM; ++a) tok_row[a] = (wm * TM + a) * 32 + j;
#pragma unroll
  for (int b = 0; b < TN; ++b) w_row[b] = BM + (wn * TN + b) * 32 + j;

  for (int kt = 0; kt < nk; ++kt) {
    const int ahead = nk - 1 - kt;                     // staged slices beyond kt
    wait_staged(ahead < NST - 2 ? ahead : NST - 2);    // slice kt has landed (this wavefront's share)
    __syncthreads();                                   // ... everyone's share; all are done with slice kt-1
    if (kt + NST - 1 < nk) issue(kt + NST - 1, (kt + NST - 1) % NST);
    const bf16_t *st = smem + (kt % NST) * STAGE_ELEMS;
    if (MF == 16) {
      // operands of the 16 x 16 x 32 product: lane (l16, q16) holds row l16 of the sub-tile, columns 8 q16 .. + 7
      bf16x8 tf[2 * TM], wf[2 * TN];
#pragma unroll
      for (int a = 0; a < 2 * TM; ++a) {
        const int row = (wm * TM * 2 + a) * 16 + l16;
        tf[a] = *reinterpret_cast<const bf16x8 *>(st + row * BK + 8 * (q16 ^ swz(row)));
      }
#pragma unroll
      for (int b = 0; b < 2 * TN; ++b) {
        const int row = BM + (wn * TN * 2 + b) * 16 + l16;
        wf[b] = *reinterpret_cast<const bf16x8 *>(st + row * BK + 8 * (q16 ^ swz(row)));
      }
#pragma unroll
      for (int a = 0; a < 2 * TM; ++a)
#pragma unroll
        for (int b = 0; b < 2 * TN; ++b)
          acc16[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[b], tf[a], acc16[a][b], 0, 0, 0);
      continue;
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int q = 2 * ks + g;
      bf16x8 tf[TM], wf[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a)
        tf[a] = *reinterpret_cast<const bf16x8 *>(st + tok_row[a] * BK + 8 * (q ^ swz(tok_row[a])));
#pragma unroll
      for (int b = 0; b < TN; ++b)
        wf[b] = *reinterpret_cast<const bf16x8 *>(st + w_row[b] * BK + 8 * (q ^ swz(w_row[b])));
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = mfma32(wf[b], tf[a], acc[a][b]);
    }
  }

  // ---- epilogue: lane (j, g) holds, for token (wm TM + a) 32 + j of the tile, features
  //      (wn TN + b) 32 + 8 rq + 4 g + 0..3 in registers 4 rq .. 4 rq + 3.  Written like that, a store
  //      instruction would scatter 16-byte pieces over 32 rows; instead each wavefront passes its
  //      32 TM x 32 TN block through LDS (the ring is free now) and writes whole row segments. ----
  constexpr int WT = 32 * TN;                   // features of a wavefront's block
  constexpr int PITCH = WT + 8;                 // LDS row pitch (elements): rows 16 bytes apart in bank phase
  constexpr int CHR = WT / 8;                   // 16-byte chunks per row segment
  static_assert(NW * 32 * PITCH <= NST * STAGE_ELEMS, "output staging must fit the ring");
  __syncthreads();                              // everyone is done reading the last K slice
  bf16_t *stg = smem + wave * (32 * PITCH);     // one 32-token block at a time
  bf16_t *C = reinterpret_cast<bf16_t *>(p.C);
  const int nw0 = n0 + wn * WT;                 // first feature of the wavefront's block
#pragma unroll
  for (int a = 0; a < TM; ++a) {
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        // MF == 32: lane (j, g), registers 4 rq .. + 3 of tile (a, b) are features b 32 + 8 rq + 4 g + 0..3 of token j.
        // MF == 16: rq = 2 ua + ub picks sub-tile (2 a + ua, 2 b + ub), whose four registers are features
        //           (2 b + ub) 16 + 4 q16 + 0..3 of token ua 16 + l16.
        const int nl = MF == 32 ? b * 32 + 8 * rq + 4 * g : (2 * b + (rq & 1)) * 16 + 4 * q16;
        const int tl = MF == 32 ? j : (rq >> 1) * 16 + l16;   // token inside the 32-token block
        float bv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (p.bias && nw0 + nl < N) {
          const bf16x4 b4 = *reinterpret_cast<const bf16x4 *>(p.bias + nw0 + nl);
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[e] = (float)b4[e];
        }
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          y[e] = (MF == 32 ? acc[a][b][4 * rq + e] : acc16[2 * a + (rq >> 1)][2 * b + (rq & 1)][e]) + bv[e];
          if (p.act == 1) {   // 0.5 y (1 + tanh u) = y / (1 + exp(-2u)), u = sqrt(2/pi) (y + 0.044715 y^3)
            const float u2 = -2.302208198f * (y[e] + 0.044715f * y[e] * y[e] * y[e]);   // -2 sqrt(2/pi) log2(e) (..)
            y[e] = y[e] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(u2));
          }
        }
        Io<bf16_t>::store4(stg + tl * PITCH + nl, y[0], y[1], y[2], y[3]);
      }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // 32 rows x CHR chunks, consecutive lanes on consecutive chunks of a row
    const int mrow0 = m0 + (wm * TM + a) * 32;
#pragma unroll
    for (int i = 0; i < (32 * CHR + 63) / 64; ++i) {
      const int c = lane + 64 * i, r = c / CHR, ch = c % CHR;
      const int n = nw0 + 8 * ch;
      if (c < 32 * CHR && mrow0 + r < M && n < N) {
        const bf16x8 val = *reinterpret_cast<const bf16x8 *>(stg + r * PITCH + 8 * ch);
        const int plane = n / p.n_split;
        bf16_t *dst = C + plane * p.plane_stride + (long long)(mrow0 + r) * p.ldc + (n - plane * p.n_split);
        if (n + 8 <= N) {
          *reinterpret_cast<bf16x8 *>(dst) = val;
        } else {   // N is a multiple of 4: the last chunk of a row may be half
          bf16x4 half;
          half[0] = val[0]; half[1] = val[1]; half[2] = val[2]; half[3] = val[3];
          *reinterpret_cast<bf16x4 *>(dst) = half;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
}

}  // namespace pab
