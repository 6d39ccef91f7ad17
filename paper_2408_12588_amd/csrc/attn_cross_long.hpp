// Cross attention (paper Sec. 2.1) against a longer text: 128 < L <= 32*LTMAX
// keys.  Per token there is now several times more matrix-core and exp work
// than memory traffic, but the keys and values of a head (L rows of D) still
// fit in LDS, so unlike the streaming tile kernel nothing is staged twice:
//
// One workgroup = NW wavefronts serves one head: it copies that head's K and V
// rows into LDS once (direct global -> LDS loads, row-major as in memory), and
// then every wavefront walks over 32-query tiles of the head on its own, with
// no further synchronisation.  Per query tile it keeps the q operands in
// registers (those of its next tile are requested before the current one is
// computed) and runs the online softmax of the tile kernel (attn_tile16.hpp:
// 16 x 16 x 32 MFMA sub-tiles, the same lane layouts) over the key tiles:
//   S^T = K Q^T  ->  running max (raised lazily)  ->  P^T = exp2(c (S^T - m))
//   ->  O^T += V^T P^T, the softmax denominator riding along as row D of O^T
// (V rows in LDS carry an extra chunk {1, 0, ..}).  K rows are stored with the
// chunk swizzle of mfma_util.hpp.  K rows past L repeat row L-1 and V rows past
// L are all zero, so padding keys need no masking.
#pragma once
#include "mfma_util.hpp"

namespace pab {

struct CrossLongParams {
  const void *q, *k, *v;
  void *o;
  int n_tok, L, n_head;
  int wg_per_head;     // workgroups that share one head
  float c;             // log2(e) / sqrt(D)
};

// LTMAX: 32-key tiles of LDS capacity.  NW: wavefronts per workgroup.  MINW: wavefronts per SIMD
// the register budget is set for.
template <int D, int LTMAX, int NW, int MINW>
__global__ __launch_bounds__(64 * NW, MINW) void attn_cross_long_kernel(const CrossLongParams p) {
  using HD = HeadDim<D>;
  using T = bf16_t;
  constexpr int CH = HD::CH;
  constexpr int LP = 32 * LTMAX;            // key rows of LDS capacity
  constexpr int RP = D;                     // row pitch: rows packed as in memory
  constexpr int VCH = CH + 1, VP = 8 * VCH; // V rows in LDS: CH data chunks, then the constant chunk
  constexpr int K_ELEMS = LP * RP, V_ELEMS = LP * VP;
  constexpr int SLACK = 64;                 // fragment reads of the last row run past its pitch
  constexpr int KSWZ_CHUNKS = 4 * (D / 32); // chunks of a K row that the 16-byte operand reads cover

  __shared__ __attribute__((aligned(16))) bf16_t smem[K_ELEMS + V_ELEMS + SLACK];
  bf16_t *Ks = smem, *Vs = smem + K_ELEMS;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;   // row / column inside a 16 x 16 sub-tile, 8-element k chunk
  const unsigned smem_addr = (unsigned)(size_t)((__attribute__((address_space(3))) char *)smem);

  // Workgroup ids go round-robin over the 8 XCDs; an XCD takes one contiguous eighth of the tokens
  // for all heads when the host made wg_per_head a multiple of 8, else the split is round-robin.
  const int H = p.n_head;
  const int ntile_q = (p.n_tok + 31) >> 5;
  int head, t_lo, t_hi, part, parts;
  if ((p.wg_per_head & 7) == 0) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    head = slot % H;
    part = slot / H;
    parts = p.wg_per_head >> 3;
    t_lo = (int)((long long)ntile_q * xcd / 8);
    t_hi = (int)((long long)ntile_q * (xcd + 1) / 8);
  } else {
    head = blockIdx.x % H;
    part = blockIdx.x / H;
    parts = p.wg_per_head;
    t_lo = 0;
    t_hi = ntile_q;
  }
  const long long row = (long long)H * D;   // token stride, elements
  const T *qh = reinterpret_cast<const T *>(p.q) + (long long)head * D;
  const T *kh = reinterpret_cast<const T *>(p.k) + (long long)head * D;
  const T *vh = reinterpret_cast<const T *>(p.v) + (long long)head * D;
  T *oh = reinterpret_cast<T *>(p.o) + (long long)head * D;
  const int n_tok = p.n_tok, L = p.L;
  const int ntile = (L + 31) >> 5;          // key tiles in use (<= LTMAX, checked by the host)
  const int rows = 32 * ntile;

  const float c = p.c;
  const float thr = 8.0f / c;   // raise the running maximum only past this margin (raw score units)
  constexpr int REM = D % 32;
  constexpr bool REM16 = REM > 0 && REM <= 16;   // the last columns of the first product as one 16-column step
  constexpr int KS = REM16 ? D / 32 : (D + 31) / 32;
  constexpr int DT16 = (D + 1 + 15) / 16;        // 16-row tiles of O^T incl. the row of the denominator
  const int k_off = l16 * RP + 8 * (g4 ^ k_swizzle<D>(l16));        // + (32 kt + 16 kh) * RP + 32 ks
  const int kr_off = l16 * RP + 32 * KS + 4 * g4;                   // + (32 kt + 16 kh) * RP
  const int v_off = (4 * g4 + (l16 >> 2)) * VP + 4 * (l16 & 3);     // + 32 kt * VP, + 16 * VP for the second key half, + 16 dt

  const int stride = parts * NW;
  // q operands (B) of a tile: query 16 qh + l16, columns 32 ks + 8 g4; tail rows load a valid row, never stored.
  // The rows of the next tile are requested before the current one is computed and arrive meanwhile.
  bf16x8 qf[2][KS], qn[2][KS];
  bf16x4 qr[2], qrn[2];
  auto request_q = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int qh2 = 0; qh2 < 2; ++qh2) {
      int qrow = 32 * t + 16 * qh2 + l16;
      qrow = qrow < n_tok ? qrow : n_tok - 1;
      const T *qp = qh + (long long)qrow * row;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int d0 = 32 * ks + 8 * g4;
        qn[qh2][ks] = (d0 < D) ? Io<T>::load8(qp + d0) : zero8();
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) qrn[qh2][e] = (bf16_t)0.0f;
      if (REM16 && 32 * KS + 4 * g4 < D) qrn[qh2] = Io<T>::load4(qp + 32 * KS + 4 * g4);
    }
  };
  auto take_q = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int qh2 = 0; qh2 < 2; ++qh2) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[qh2][ks] = qn[qh2][ks];
      qr[qh2] = qrn[qh2];
    }
  };
  int t = t_lo + part * NW + wave;
  if (t < t_hi) request_q(t);   // in flight while K and V are staged

  // ---- K and V of the head, 64-chunk rounds dealt round-robin to the wavefronts.  Slots that no
  //      load fills (V rows past L, the constant chunks) are written as ordinary LDS stores. ----
  const int kr = (rows * CH + 63) >> 6, vr = (rows * VCH + 63) >> 6;
  for (int r = wave; r < kr + vr; r += NW) {
    if (r < kr) {
      const int c = r * 64 + lane;
      if (c < rows * CH) {
        const int krow = c / CH;
        int chunk = c % CH;
        if (chunk < KSWZ_CHUNKS) chunk ^= k_swizzle<D>(krow);   // the slot holds the exchanged chunk
        const int key = krow < L ? krow : L - 1;
        dma16_to_lds(kh, (unsigned)(2 * (key * row + 8 * chunk)), smem_addr + 1024 * r);
      }
    } else {
      const int c = (r - kr) * 64 + lane, key = c / VCH, chunk = c % VCH;
      const bool real = c < rows * VCH && key < L && chunk < CH;
      if (real) dma16_to_lds(vh, (unsigned)(2 * (key * row + 8 * chunk)), smem_addr + 2 * K_ELEMS + 1024 * (r - kr));
      if (c < rows * VCH && !real) {
        bf16x8 fill = zero8();
        if (chunk == CH && key < L) fill[0] = (bf16_t)1.0f;
        *reinterpret_cast<bf16x8 *>(Vs + 8 * c) = fill;
      }
    }
  }
  if (tid < SLACK / 2) reinterpret_cast<unsigned *>(smem + K_ELEMS + V_ELEMS)[tid] = 0u;
  // The 16-column operand read of the last K row runs 8 elements past it when D is not a multiple
  // of 16; what it finds there meets zero q columns, but has to be finite.
  if (rows < LP && tid < 4) reinterpret_cast<unsigned *>(Ks + rows * RP)[tid] = 0u;
  __builtin_amdgcn_s_waitcnt(0x0F70);   // this wavefront's share of K and V has landed (and its first q rows)
  __syncthreads();                      // ... everyone's
  if (t >= t_hi) return;

  for (;;) {
    take_q();
    const bool more = t + stride < t_hi;
    if (more) request_q(t + stride);

    f32x4 oacc[DT16][2];
    float m_run[2], m_thr[2], m_negc[2];   // running maximum, m + margin, -m c: the last two change only when m does
#pragma unroll
    for (int qh2 = 0; qh2 < 2; ++qh2) {
      m_run[qh2] = -INFINITY;
      m_thr[qh2] = -INFINITY;
      m_negc[qh2] = 0.0f;
#pragma unroll
      for (int dt = 0; dt < DT16; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) oacc[dt][qh2][r] = 0.0f;
    }

    for (int kt = 0; kt < ntile; ++kt) {
      const bf16_t *ktile = Ks + 32 * kt * RP, *vtile = Vs + 32 * kt * VP;
      // S^T = K Q^T for 32 keys: four 16 x 16 sub-tiles (key half kh, query half); the 32-column steps of
      // all four first, then the 16-column steps (see mfma_shape_change)
      f32x4 S[2][2];
      bf16x4 kr[2];
#pragma unroll
      for (int kh2 = 0; kh2 < 2; ++kh2) {
        bf16x8 kf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(ktile + k_off + 16 * kh2 * RP + 32 * ks);
        // columns past D read on into the next row (finite) and meet zero q columns
        if (REM16) kr[kh2] = *reinterpret_cast<const bf16x4 *>(ktile + kr_off + 16 * kh2 * RP);
#pragma unroll
        for (int qh2 = 0; qh2 < 2; ++qh2) {
#pragma unroll
          for (int r = 0; r < 4; ++r) S[kh2][qh2][r] = 0.0f;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) S[kh2][qh2] = mfma16(kf[ks], qf[qh2][ks], S[kh2][qh2]);
        }
      }
      if (REM16) {
        mfma_shape_change(S[0][0], S[0][1], S[1][0], S[1][1]);
#pragma unroll
        for (int kh2 = 0; kh2 < 2; ++kh2)
#pragma unroll
          for (int qh2 = 0; qh2 < 2; ++qh2) S[kh2][qh2] = mfma16_k16(kr[kh2], qr[qh2], S[kh2][qh2]);
      }

      // tile maximum over this lane's 8 keys per query; the four lanes of a query share m_run, which
      // only moves when one of them exceeds it by the margin
      float mx[2];
      bool grow = false;
#pragma unroll
      for (int qh2 = 0; qh2 < 2; ++qh2) {   // a chain of three-operand maxima over the lane's 8 scores
        float a = fmaxf(fmaxf(S[0][qh2][0], S[0][qh2][1]), S[0][qh2][2]);
        a = fmaxf(fmaxf(a, S[0][qh2][3]), S[1][qh2][0]);
        a = fmaxf(fmaxf(a, S[1][qh2][1]), S[1][qh2][2]);
        mx[qh2] = fmaxf(a, S[1][qh2][3]);
        grow |= mx[qh2] > m_thr[qh2];
      }
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {   // rare after the first tile
#pragma unroll
        for (int qh2 = 0; qh2 < 2; ++qh2) {
          float full = fmaxf(mx[qh2], __shfl_xor(mx[qh2], 16));
          full = fmaxf(full, __shfl_xor(full, 32));
          const float m_new = fmaxf(m_run[qh2], full);
          const float alpha = __builtin_amdgcn_exp2f((m_run[qh2] - m_new) * c);
          m_run[qh2] = m_new;
          m_thr[qh2] = m_new + thr;
          m_negc[qh2] = -m_new * c;
#pragma unroll
          for (int dt = 0; dt < DT16; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) oacc[dt][qh2][r] *= alpha;
        }
      }

      // P^T = exp2(c S^T - c m): the lane's keys of the first half, then of the second, are its B operand
      bf16x8 pf[2];
#pragma unroll
      for (int qh2 = 0; qh2 < 2; ++qh2)
#pragma unroll
        for (int kh2 = 0; kh2 < 2; ++kh2)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            pf[qh2][4 * kh2 + r] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(S[kh2][qh2][r], c, m_negc[qh2]));
      // O^T += V^T P^T
#pragma unroll
      for (int dt = 0; dt < DT16; ++dt) {
        const bf16_t *vp = vtile + v_off + 16 * dt;
        const bf16x4 lo = lds_read_tr4(vp), hi = lds_read_tr4(vp + 16 * VP);
        bf16x8 vf;
        vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
        vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
#pragma unroll
        for (int qh2 = 0; qh2 < 2; ++qh2) oacc[dt][qh2] = mfma16(vf, pf[qh2], oacc[dt][qh2]);
      }
    }

    // ---- divide by the denominator held in row D of O^T (sub-tile D / 16, lane group (D % 16) / 4), store ----
    constexpr int DEN_DT = D / 16, DEN_G = (D % 16) / 4, DEN_R = D % 4;
#pragma unroll
    for (int qh2 = 0; qh2 < 2; ++qh2) {
      const float inv = 1.0f / __shfl(oacc[DEN_DT][qh2][DEN_R], l16 + 16 * DEN_G);
      const int qrow = 32 * t + 16 * qh2 + l16;
      if (qrow < n_tok) {
        T *orow = oh + (long long)qrow * row;
#pragma unroll
        for (int dt = 0; dt < DT16; ++dt) {
          const int d0 = 16 * dt + 4 * g4;
          if (d0 < D)
            Io<T>::store4(orow + d0, oacc[dt][qh2][0] * inv, oacc[dt][qh2][1] * inv, oacc[dt][qh2][2] * inv,
                          oacc[dt][qh2][3] * inv);
        }
      }
    }
    if (!more) break;
    t += stride;
  }
}

}  // namespace pab
