// Cross attention (paper Sec. 2.1) against a longer text: 128 < L <= 32*LTMAX
// keys.  Per token there is now several times more matrix-core and exp work
// than memory traffic, but the keys and values of a head (L rows of D) still
// fit in LDS, so unlike the streaming tile kernel nothing is staged twice:
//
// One workgroup = NW wavefronts serves one head: it copies that head's K and V
// rows into LDS once (direct global -> LDS loads, row-major as in memory), and
// then every wavefront walks over 32-query tiles of the head on its own, with
// no further synchronisation.  Per query tile it keeps the q operands in
// registers and runs the online softmax of the tile kernel over the key tiles:
//   S^T = K Q^T  ->  running max (raised lazily)  ->  P^T = exp2(c (S^T - m))
//   ->  O^T += V^T P^T, the softmax denominator riding along as row D of O^T
// (V rows in LDS carry an extra chunk {1, 0, ..}).  K rows past L repeat row
// L-1 and V rows past L are all zero, so padding keys need no masking.
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
  constexpr int KSTEPS = HD::KSTEPS, DT = HD::DT, CH = HD::CH;
  constexpr int LP = 32 * LTMAX;            // key rows of LDS capacity
  constexpr int RP = D;                     // row pitch: rows packed as in memory
  constexpr int VCH = CH + 1, VP = 8 * VCH; // V rows in LDS: CH data chunks, then the constant chunk
  constexpr int K_ELEMS = LP * RP, V_ELEMS = LP * VP;
  constexpr int SLACK = 64;                 // fragment reads of the last row run past its pitch

  __shared__ __attribute__((aligned(16))) bf16_t smem[K_ELEMS + V_ELEMS + SLACK];
  bf16_t *Ks = smem, *Vs = smem + K_ELEMS;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31, g = lane >> 5;
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

  // ---- K and V of the head, 64-chunk rounds dealt round-robin to the wavefronts.  Slots that no
  //      load fills (V rows past L, the constant chunks) are written as ordinary LDS stores. ----
  const int kr = (rows * CH + 63) >> 6, vr = (rows * VCH + 63) >> 6;
  for (int r = wave; r < kr + vr; r += NW) {
    if (r < kr) {
      const int c = r * 64 + lane;
      if (c < rows * CH) {
        int key = c / CH;
        key = key < L ? key : L - 1;
        dma16_to_lds(kh, (unsigned)(2 * (key * row + 8 * (c % CH))), smem_addr + 1024 * r);
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
  // The operand read of the last K row runs 8 elements past it when D is not a multiple of 16;
  // what it finds there meets zero q columns, but has to be finite.
  if (rows < LP && tid < 4) reinterpret_cast<unsigned *>(Ks + rows * RP)[tid] = 0u;
  __builtin_amdgcn_s_waitcnt(0x0F70);   // this wavefront's share of K and V has landed
  __syncthreads();                      // ... everyone's

  const float c = p.c;
  const float thr = 8.0f / c;   // raise the running maximum only past this margin (raw score units)
  const int k_off = sigma(j) * RP + 8 * g;                                               // + 32 kt * RP + 16 s
  const int i16 = lane & 15, q4 = lane >> 4;
  const int v_off = (8 * (q4 >> 1) + (i16 >> 2)) * VP + 16 * (q4 & 1) + 4 * (i16 & 3);   // + (32 kt + 16 m + 4 hh) * VP + 32 dt
  constexpr int LDT = D / 32, LLOC = D % 32;
  constexpr int LR = 4 * (LLOC / 8) + (LLOC % 4), LG = (LLOC / 4) & 1;

  const int stride = parts * NW;
  for (int t = t_lo + part * NW + wave; t < t_hi; t += stride) {
    // ---- q operands (B): query j, columns 16 s + 8 g; tail rows load a valid row, never stored ----
    int qrow = 32 * t + j;
    const bool q_valid = qrow < n_tok;
    qrow = q_valid ? qrow : n_tok - 1;
    const T *qp = qh + (long long)qrow * row;
    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      const int d0 = 16 * s + 8 * g;
      qf[s] = (d0 < D) ? Io<T>::load8(qp + d0) : zero8();
    }

    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.0f;
    float m_run = -INFINITY;

    for (int kt = 0; kt < ntile; ++kt) {
      // S^T = K Q^T for 32 keys
      const bf16_t *ktile = Ks + 32 * kt * RP, *vtile = Vs + 32 * kt * VP;
      bf16x8 kf[KSTEPS];
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) kf[s] = *reinterpret_cast<const bf16x8 *>(ktile + k_off + 16 * s);
      f32x16 S;
#pragma unroll
      for (int r = 0; r < 16; ++r) S[r] = 0.0f;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) S = mfma32(kf[s], qf[s], S);

      // tile maximum; the running maximum only moves when a score exceeds it by the margin
      float a = fmaxf(fmaxf(S[0], S[1]), S[2]);
      float b = fmaxf(fmaxf(S[3], S[4]), S[5]);
#pragma unroll
      for (int r = 6; r < 14; r += 4) {
        a = fmaxf(fmaxf(a, S[r]), S[r + 1]);
        b = fmaxf(fmaxf(b, S[r + 2]), S[r + 3]);
      }
      a = fmaxf(fmaxf(a, S[14]), S[15]);
      const float mx = fmaxf(a, b);   // this lane's half of the keys; m_run is shared by both lanes of a query
      if (__builtin_amdgcn_ballot_w64(mx > m_run + thr) != 0) {   // rare after the first tile
        const float m_new = fmaxf(m_run, max_pair(mx));
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
      }

      // P^T = exp2(c S^T - c m), already laid out as B operands; O^T += V^T P^T
      const float mc = m_run * c;
      bf16x8 pf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) pf[r >> 3][r & 7] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(S[r], c, -mc));
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const bf16_t *vp = vtile + v_off + 16 * m * VP + 32 * dt;
          const bf16x4 lo = lds_read_tr4(vp), hi = lds_read_tr4(vp + 4 * VP);
          bf16x8 vf;
          vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
          vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
          oacc[dt] = mfma32(vf, pf[m], oacc[dt]);
        }
    }

    // ---- divide by the denominator held in row D of O^T, store ----
    const float inv = 1.0f / __shfl(oacc[LDT][LR], j + 32 * LG);
    if (q_valid) {
      T *orow = oh + (long long)qrow * row;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int d0 = 32 * dt + 8 * rq + 4 * g;
          if (d0 < D)
            Io<T>::store4(orow + d0, oacc[dt][4 * rq] * inv, oacc[dt][4 * rq + 1] * inv,
                          oacc[dt][4 * rq + 2] * inv, oacc[dt][4 * rq + 3] * inv);
        }
    }
  }
}

}  // namespace pab
