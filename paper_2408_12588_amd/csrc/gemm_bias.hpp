// Projections of the attention module (paper App. B.5: "qkv proj", "o proj"):
// C[M, N] = A[M, K] W[N, K]^T + bias[N], activations and weights bf16, fp32
// accumulation on the matrix core, one rounding to bf16 on the way out.
//
// Both operands are contiguous along K, which is what the MFMA operands want:
// with the weight rows as the A operand and the token rows as the B operand a
// 32x32 tile is C^T[n, m], every lane owns one token and 16 of its outputs.
//
// One workgroup = 4 wavefronts (2 x 2) computes a 128-token x 256-feature tile,
// each wavefront 64 x 128 (2 x 4 MFMA tiles, 128 accumulator registers).  The
// K dimension streams through a ring of NST LDS stages of 32 columns: 128 token
// rows and 256 weight rows of 64 bytes each per stage, copied global -> LDS
// directly (16 bytes per lane) two stages ahead of their use, one barrier per
// stage.  Rows are 64 bytes, so row r's four 16-byte chunks are stored at
// position q ^ ((r >> 2) & 3): the 16 lanes that read one chunk column of 16
// consecutive rows then hit 16 different bank groups.
//
// Workgroup ids go round-robin over the 8 XCDs; an XCD owns every eighth token
// tile and walks its tiles four token tiles at a time across all feature tiles,
// so that the weight rows in flight are shared by four workgroups and a token
// tile's rows by all of its feature tiles inside one L2.
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
  int n_mt, n_nt;       // token / feature tiles
};

template <int NST>
__global__ __launch_bounds__(256, 2) void gemm_bias_kernel(const GemmParams p) {
  constexpr int BM = 128, BN = 256, BK = 32;
  constexpr int ROWS = BM + BN;                 // rows per stage: token rows, then weight rows
  constexpr int STAGE_ELEMS = ROWS * BK;        // 24 KB
  constexpr int ROUNDS = ROWS * 4 / 64;         // 64-chunk copy rounds per stage = 24
  constexpr int MYR = ROUNDS / 4;               // per wavefront = 6: two of token rows, four of weight rows
  constexpr int GM = 4;                         // token tiles an XCD keeps in flight together
  static_assert(NST >= 3 && (NST - 2) * MYR < 16, "ring depth / vmcnt immediates");

  __shared__ __attribute__((aligned(16))) bf16_t smem[NST * STAGE_ELEMS];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31, g = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const unsigned smem_addr = (unsigned)(size_t)((__attribute__((address_space(3))) char *)smem);

  // ---- which tile ----
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per_group = GM * p.n_nt;
  const int grp = slot / per_group, rem = slot % per_group;
  const int nt_id = rem / GM;
  const int mt_id = 8 * (grp * GM + rem % GM) + xcd;
  if (mt_id >= p.n_mt) return;
  const int m0 = mt_id * BM, n0 = nt_id * BN;
  const int M = p.M, N = p.N, K = p.K;

  // ---- staging: round r = wave + 4 i covers rows 16 r .. 16 r + 15 of the stage; lane's chunk slot
  //      64 r + lane holds (row, chunk q) with q = (lane & 3) ^ ((row >> 2) & 3).  Rows past the
  //      matrix re-read its last row; what they produce is never stored. ----
  unsigned voff[MYR];
#pragma unroll
  for (int i = 0; i < MYR; ++i) {
    const int r = wave + 4 * i;
    const int row = 16 * r + (lane >> 2);
    const int q = (lane & 3) ^ ((row >> 2) & 3);
    long long grow;
    if (i < 2) grow = min(m0 + row, M - 1);          // token rows (rounds 0..7)
    else grow = min(n0 + row - BM, N - 1);           // weight rows (rounds 8..23)
    voff[i] = (unsigned)(2 * (grow * K + 8 * q));
  }
  auto issue = [&](int kt, int stage) {
#pragma unroll
    for (int i = 0; i < MYR; ++i) {
      const int r = wave + 4 * i;
      dma16_to_lds((i < 2 ? p.A : p.W) + (long long)kt * BK, voff[i], smem_addr + 2 * stage * STAGE_ELEMS + 1024 * r);
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

  f32x16 acc[2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  // fragment addresses inside a stage (elements): row * 32 + 8 * (chunk ^ swizzle(row))
  int tok_row[2], w_row[4];
#pragma unroll
  for (int a = 0; a < 2; ++a) tok_row[a] = wm * 64 + a * 32 + j;
#pragma unroll
  for (int b = 0; b < 4; ++b) w_row[b] = BM + wn * 128 + b * 32 + j;

  for (int kt = 0; kt < nk; ++kt) {
    const int ahead = nk - 1 - kt;                     // staged slices beyond kt
    wait_staged(ahead < NST - 2 ? ahead : NST - 2);    // slice kt has landed (this wavefront's share)
    __syncthreads();                                   // ... everyone's share; all are done with slice kt-1
    if (kt + NST - 1 < nk) issue(kt + NST - 1, (kt + NST - 1) % NST);
    const bf16_t *st = smem + (kt % NST) * STAGE_ELEMS;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int q = 2 * ks + g;
      bf16x8 tf[2], wf[4];
#pragma unroll
      for (int a = 0; a < 2; ++a)
        tf[a] = *reinterpret_cast<const bf16x8 *>(st + tok_row[a] * BK + 8 * (q ^ ((tok_row[a] >> 2) & 3)));
#pragma unroll
      for (int b = 0; b < 4; ++b)
        wf[b] = *reinterpret_cast<const bf16x8 *>(st + w_row[b] * BK + 8 * (q ^ ((w_row[b] >> 2) & 3)));
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = mfma32(wf[b], tf[a], acc[a][b]);
    }
  }

  // ---- epilogue: lane (j, g) holds, for token m0 + wm*64 + a*32 + j, features
  //      n0 + wn*128 + b*32 + 8 rq + 4 g + 0..3 in registers 4 rq .. 4 rq + 3 ----
  bf16_t *C = reinterpret_cast<bf16_t *>(p.C);
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int n = n0 + wn * 128 + b * 32 + 8 * rq + 4 * g;
      if (n >= N) continue;
      const int plane = n / p.n_split;
      bf16_t *Cn = C + plane * p.plane_stride + (n - plane * p.n_split);
      float bv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (p.bias) {
        const bf16x4 b4 = *reinterpret_cast<const bf16x4 *>(p.bias + n);
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[e] = (float)b4[e];
      }
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int m = m0 + wm * 64 + a * 32 + j;
        if (m < M)
          Io<bf16_t>::store4(Cn + (long long)m * p.ldc, acc[a][b][4 * rq] + bv[0], acc[a][b][4 * rq + 1] + bv[1],
                             acc[a][b][4 * rq + 2] + bv[2], acc[a][b][4 * rq + 3] + bv[3]);
      }
    }
}

}  // namespace pab
