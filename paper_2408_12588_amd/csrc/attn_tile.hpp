// Tiled attention kernel for long query sequences (spatial and cross attention,
// paper Sec. 2.1): o = softmax(q k^T / sqrt(D)) v per (batch, head), computed
// with an online softmax over blocks of keys so that scores never reach memory.
//
// Work split: one workgroup = 4 wavefronts = 128*NQT consecutive queries of one
// (batch, head); each wavefront owns NQT tiles of 32 queries whose q fragments
// stay in registers.  Keys and values stream through LDS in blocks of KB keys.
//
// Per key block and query tile the wavefront computes, with bf16 MFMA:
//   S^T[key, query]  = K_blk Q^T            (A = keys, B = queries)
//   P^T              = exp2(c*S^T - c*m)    (in registers, c = log2(e)/sqrt(D))
//   O^T[d, query]   += V_blk^T P^T          (A = values transposed, B = P^T)
// Keeping the query on the lane axis makes every softmax statistic a per-lane
// scalar, and (with the key permutation sigma) the accumulator registers of the
// first product are already the B operand of the second.  Row D of V^T is all
// ones, so row D of O^T accumulates the softmax denominator on the matrix core.
#pragma once
#include "mfma_util.hpp"

namespace pab {

struct TileParams {
  const void *q, *k, *v;
  void *o;
  int n_batch, n_head, sq, sk;
  long long q_bs, q_ss, k_bs, k_ss, v_bs, v_ss, o_bs, o_ss;  // batch / sequence strides, elements
  float c;        // log2(e) / sqrt(D)
  int n_qblk;     // query blocks per (batch, head)
};

template <typename T, int D, int NQT, int KB>
__global__ __launch_bounds__(256) void attn_tile_kernel(const TileParams p) {
  using HD = HeadDim<D>;
  constexpr int DK = HD::DK, KSTEPS = HD::KSTEPS, DV = HD::DV, DT = HD::DT, CH = HD::CH, DKP = HD::DKP;
  constexpr int KBP = KB + 8;      // pitch of the transposed value tile
  constexpr int KT = KB / 32;      // 32-key tiles per block
  constexpr int QBLK = 128 * NQT;  // queries per workgroup
  static_assert(KB % 32 == 0, "key block must be a multiple of 32");

  __shared__ __attribute__((aligned(16))) bf16_t Ks[KB * DKP];   // [key][d], d zero padded to DK
  __shared__ __attribute__((aligned(16))) bf16_t Vt[DV * KBP];   // [d][key], row D = ones, rows > D = 0

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, g = lane >> 5;

  // Workgroup ids are dealt round-robin to the 8 XCDs; give every XCD whole (batch, head)
  // problems so that all query blocks of a problem share that XCD's L2 copy of K and V.
  const int n_bh = p.n_batch * p.n_head;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int bh = (slot / p.n_qblk) * 8 + xcd;
  const int qblk = slot % p.n_qblk;
  if (bh >= n_bh) return;
  const int batch = bh / p.n_head, head = bh % p.n_head;

  const T *qb = reinterpret_cast<const T *>(p.q) + batch * p.q_bs + (long long)head * D;
  const T *kb_ = reinterpret_cast<const T *>(p.k) + batch * p.k_bs + (long long)head * D;
  const T *vb = reinterpret_cast<const T *>(p.v) + batch * p.v_bs + (long long)head * D;
  T *ob = reinterpret_cast<T *>(p.o) + batch * p.o_bs + (long long)head * D;
  const int sq = p.sq, sk = p.sk;

  const int q_wave0 = qblk * QBLK + wave * (32 * NQT);
  const bool wave_active = q_wave0 < sq;

  // ---- q fragments (B operand of the first product), kept for the whole kernel ----
  bf16x8 qf[NQT][KSTEPS];
#pragma unroll
  for (int n = 0; n < NQT; ++n) {
    int qrow = q_wave0 + 32 * n + j;
    qrow = qrow < sq ? qrow : sq - 1;   // tail rows load a valid row and are never stored
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      const int d0 = 16 * s + 8 * g;
      qf[n][s] = (d0 < D) ? Io<T>::load8(qb + qrow * p.q_ss + d0) : zero8();
    }
  }

  // ---- constant parts of the LDS tiles ----
  if (DK > D) {
    constexpr int PADC = (DK - D) / 8;
    for (int idx = tid; idx < KB * PADC; idx += 256) {
      const int row = idx / PADC, cc = idx % PADC;
      *reinterpret_cast<bf16x8 *>(&Ks[row * DKP + D + 8 * cc]) = zero8();
    }
  }
  for (int idx = tid; idx < (DV - D) * (KBP / 8); idx += 256) {
    const int row = D + idx / (KBP / 8), cc = idx % (KBP / 8);
    *reinterpret_cast<bf16x8 *>(&Vt[row * KBP + 8 * cc]) = (row == D) ? splat8(1.0f) : zero8();
  }

  // ---- global -> register staging of one key block ----
  constexpr int NCH = KB * CH;
  constexpr int PER = (NCH + 255) / 256;
  bf16x8 kreg[PER], vreg[PER];
  auto prefetch = [&](int blk) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + 256 * i;
      if (c < NCH) {
        {  // keys: consecutive lanes walk along a row (coalesced)
          const int row = c / CH, cc = c % CH, key = blk * KB + row;
          kreg[i] = key < sk ? Io<T>::load8(kb_ + key * p.k_ss + 8 * cc) : zero8();
        }
        {  // values: consecutive lanes walk down the keys, so that the transposing LDS
           // stores of one instruction fall into consecutive addresses
          const int row = c % KB, cc = c / KB, key = blk * KB + row;
          vreg[i] = key < sk ? Io<T>::load8(vb + key * p.v_ss + 8 * cc) : zero8();
        }
      }
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + 256 * i;
      if (c < NCH) {
        {
          const int row = c / CH, cc = c % CH;
          *reinterpret_cast<bf16x8 *>(&Ks[row * DKP + 8 * cc]) = kreg[i];
        }
        {
          const int row = c % KB, cc = c / KB;
#pragma unroll
          for (int e = 0; e < 8; ++e) Vt[(8 * cc + e) * KBP + row] = vreg[i][e];
        }
      }
    }
  };

  f32x16 oacc[NQT][DT];
  float m_run[NQT];
#pragma unroll
  for (int n = 0; n < NQT; ++n) {
    m_run[n] = -INFINITY;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[n][dt][r] = 0.0f;
  }

  const int nkb = (sk + KB - 1) / KB;
  const float c = p.c;
  prefetch(0);
  for (int blk = 0; blk < nkb; ++blk) {
    __syncthreads();   // every wave is done reading the previous block
    stash();
    __syncthreads();
    if (blk + 1 < nkb) prefetch(blk + 1);
    if (!wave_active) continue;

    // ---- S^T = K Q^T ----
    f32x16 sacc[NQT][KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      bf16x8 kf[KSTEPS];
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s)
        kf[s] = *reinterpret_cast<const bf16x8 *>(&Ks[(32 * kt + sigma(j)) * DKP + 16 * s + 8 * g]);
#pragma unroll
      for (int n = 0; n < NQT; ++n) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[n][kt][r] = 0.0f;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) sacc[n][kt] = mfma32(kf[s], qf[n][s], sacc[n][kt]);
      }
    }
    // keys past the end of the sequence take no probability mass
    if (blk == nkb - 1 && (sk % KB) != 0) {
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = blk * KB + 32 * kt + key_of_reg(r, g);
          if (key >= sk) {
#pragma unroll
            for (int n = 0; n < NQT; ++n) sacc[n][kt][r] = -INFINITY;
          }
        }
    }

    // ---- online softmax, one query per lane (lanes j and j+32 share a query) ----
    bf16x8 pf[NQT][KT][2];
#pragma unroll
    for (int n = 0; n < NQT; ++n) {
      float mx = sacc[n][0][0];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[n][kt][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[n], mx);
      const float alpha = __builtin_amdgcn_exp2f((m_run[n] - m_new) * c);
      m_run[n] = m_new;
      const float mc = m_new * c;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[n][dt][r] *= alpha;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[n][kt][r], c, -mc));
          pf[n][kt][r >> 3][r & 7] = (bf16_t)pr;
        }
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const bf16x8 vf =
              *reinterpret_cast<const bf16x8 *>(&Vt[(32 * dt + j) * KBP + 32 * kt + 16 * m + 8 * g]);
#pragma unroll
          for (int n = 0; n < NQT; ++n) oacc[n][dt] = mfma32(vf, pf[n][kt][m], oacc[n][dt]);
        }
  }

  if (!wave_active) return;

  // ---- epilogue: divide by the denominator held in row D of O^T, store ----
  constexpr int LDT = D / 32, LLOC = D % 32;
  constexpr int LR = 4 * (LLOC / 8) + (LLOC % 4), LG = (LLOC / 4) & 1;
#pragma unroll
  for (int n = 0; n < NQT; ++n) {
    const float denom = __shfl(oacc[n][LDT][LR], j + 32 * LG);
    const float inv = 1.0f / denom;
    const int qrow = q_wave0 + 32 * n + j;
    if (qrow < sq) {
      T *orow = ob + qrow * p.o_ss;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int d0 = 32 * dt + 8 * rq + 4 * g;
          if (d0 < D)
            Io<T>::store4(orow + d0, oacc[n][dt][4 * rq] * inv, oacc[n][dt][4 * rq + 1] * inv,
                          oacc[n][dt][4 * rq + 2] * inv, oacc[n][dt][4 * rq + 3] * inv);
        }
    }
  }
}

}  // namespace pab
