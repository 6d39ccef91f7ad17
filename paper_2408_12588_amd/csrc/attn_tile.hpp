// Tiled attention kernel for long query sequences (spatial and cross attention,
// paper Sec. 2.1): o = softmax(q k^T / sqrt(D)) v per (batch, head), computed
// with an online softmax over tiles of keys so that scores never reach memory.
//
// Work split: one workgroup = NWV wavefronts = 32*NQT*NWV consecutive queries of one
// (batch, head); each wavefront owns NQT tiles of 32 queries whose q fragments
// stay in registers.  Keys and values stream through a ring of NST LDS stages,
// one 32-key tile per stage, stored row-major exactly as in memory (for bf16
// inputs the global loads write LDS directly, no registers in between, NST-2
// tiles ahead of their use).  Several workgroups share a CU, so that one
// wavefront's LDS and barrier waits are covered by the others.
//
// Per 32-key tile and 32-query tile the wavefront computes, with bf16 MFMA:
//   S^T[key, query]  = K Q^T                (A = keys, B = queries)
//   P^T              = exp2(c*S^T - c*m)    (in registers, c = log2(e)/sqrt(D))
//   O^T[d, query]   += V^T P^T              (A = values read transposed, B = P^T)
// Keeping the query on the lane axis makes every softmax statistic a per-lane
// scalar, and (with the key permutation sigma) the accumulator registers of the
// first product are already the B operand of the second.  V rows in LDS carry
// one extra 16-byte chunk {1, 0, ..} after their D values (written once; the
// staging loads skip it), so row D of V^T is all ones and row D of O^T
// accumulates the softmax denominator on the matrix core.  The running
// maximum m is only raised when some score exceeds it by more than 8 in the
// exponent (probabilities then stay below 2^8, harmless in fp32 / bf16);
// numerator and denominator always share the same m, so the quotient is
// unaffected.
//
// PIPE selects a variant that is software pipelined inside the wavefront (the
// scores of tile t+1 are issued to the matrix core before the exponentials of
// tile t are taken).  It needs twice the score registers and measured no
// faster than letting the other wavefronts of the SIMD provide the overlap.
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

template <typename T, int D, int NQT, int NWV, int NST, int MINW, bool PIPE, bool DIRECT>
__global__ __launch_bounds__(64 * NWV, MINW) void attn_tile_kernel(const TileParams p) {
  using HD = HeadDim<D>;
  constexpr int KSTEPS = HD::KSTEPS, DT = HD::DT, CH = HD::CH;
  constexpr int KB = 32;             // keys per LDS stage = one MFMA tile
  constexpr int QBLK = 32 * NQT * NWV;   // queries per workgroup
  constexpr int RP = D;              // row pitch of the K tile in LDS: rows packed as in memory
  constexpr int VCH = CH + 1;        // chunks per V row in LDS: CH of data, then the constant chunk {1, 0, ..}
  constexpr int VP = 8 * VCH;        // row pitch of the V tile
  constexpr int TILE_ELEMS = KB * RP;                       // K rows ...
  constexpr int STAGE_ELEMS = TILE_ELEMS + KB * VP;         // ... then V rows
  constexpr int SLACK = 64;          // fragment reads of a tile's last row run past its pitch: finite
                                     // garbage that only meets zero q columns / discarded output rows
  constexpr int PRK = (KB * CH + 63) / 64;   // staging rounds (64 chunk slots each, the last maybe partial) of the K tile
  constexpr int PRV = (KB * VCH + 63) / 64;  // ... of the V tile (the slots of the constant chunks stay idle)
  constexpr int ROUNDS = PRK + PRV;          // K rounds, then V rounds
  constexpr int MYR = (ROUNDS + NWV - 1) / NWV;   // rounds per wavefront (the last may repeat a round)
  static_assert(!DIRECT || sizeof(T) == 2, "direct-to-LDS staging needs bf16 inputs");
  static_assert(NST >= 3 && NST <= 5 && (NST - 2) * MYR < 16, "ring depth / vmcnt immediates");

  __shared__ __attribute__((aligned(16))) bf16_t smem[NST * STAGE_ELEMS + SLACK];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

  // ---- staging of key tile t into LDS stage `stage`.  The ROUNDS rounds are dealt to the
  //      wavefronts round-robin.  Rows past the end of the sequence re-read the last valid row:
  //      their scores are masked, so they carry no weight. ----
  const int ntile = (sk + 31) >> 5;          // 32-key tiles, the last possibly partial
  const unsigned smem_addr = (unsigned)(size_t)((__attribute__((address_space(3))) char *)smem);

  auto my_round = [&](int i) { const int r = wave + NWV * i; return r < ROUNDS ? r : ROUNDS - 1; };
  // round i of this wavefront: chunk slot of this lane inside the K or V tile, and whether it carries data
  auto slot_of = [&](int i) { const int r = my_round(i); return (r < PRK ? r : r - PRK) * 64 + lane; };
  auto live = [&](int i) {
    const int c = slot_of(i);
    return my_round(i) < PRK ? c < KB * CH : (c < KB * VCH && c % VCH < CH);
  };
  auto chunk_off = [&](int i, int t) -> long long {   // element offset of this lane's chunk, round i
    const bool is_k = my_round(i) < PRK;
    const int c = slot_of(i), per = is_k ? CH : VCH;
    int key = t * KB + c / per;
    key = key < sk ? key : sk - 1;
    return key * (is_k ? p.k_ss : p.v_ss) + 8 * (c % per);
  };
  unsigned voff[MYR];   // byte offsets relative to the tile's first K / V row (full tiles)
#pragma unroll
  for (int i = 0; i < MYR; ++i) voff[i] = (unsigned)(2 * chunk_off(i, 0));

  auto issue = [&](int t, int stage) {
    const bool tail = (t + 1) * KB > sk;
#pragma unroll
    for (int i = 0; i < MYR; ++i) {
      const int round = my_round(i);
      const bool is_k = round < PRK;
      const long long t_off = (long long)t * KB * (is_k ? p.k_ss : p.v_ss);
      const int lds_elem = stage * STAGE_ELEMS + (is_k ? 512 * round : TILE_ELEMS + 512 * (round - PRK));
      if (live(i)) {   // idle lanes: past the tile, or on a constant chunk that must survive
        if (DIRECT) {
          const unsigned off = tail ? (unsigned)(2 * (chunk_off(i, t) - t_off)) : voff[i];
          dma16_to_lds((is_k ? kb_ : vb) + t_off, off, smem_addr + 2 * lds_elem);
        } else {   // element types that need conversion go through registers, synchronously
          *reinterpret_cast<bf16x8 *>(smem + lds_elem + 8 * lane) = Io<T>::load8((is_k ? kb_ : vb) + chunk_off(i, t));
        }
      }
    }
  };
  // wait until at most `tiles` of this wavefront's staged tiles are still in flight
  auto wait_staged = [&](int tiles) {
    if (!DIRECT) return;
    if (tiles >= 3) __builtin_amdgcn_s_waitcnt(0x0F70 | (3 * MYR));
    else if (tiles == 2) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * MYR));
    else if (tiles == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | MYR);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
  };

  // ---- prologue: first NST-1 tiles on their way, then the q fragments ----
  if (tid < SLACK / 2) reinterpret_cast<unsigned *>(smem + NST * STAGE_ELEMS)[tid] = 0u;   // the slack is defined
  for (int idx = tid; idx < NST * KB; idx += 64 * NWV) {   // constant chunk of every V row of every stage
    bf16x8 one = zero8();
    one[0] = (bf16_t)1.0f;
    *reinterpret_cast<bf16x8 *>(smem + (idx / KB) * STAGE_ELEMS + TILE_ELEMS + (idx % KB) * VP + D) = one;
  }
  const int npre = ntile < NST - 1 ? ntile : NST - 1;
  for (int t = 0; t < npre; ++t) issue(t, t);

  bf16x8 qf[NQT][KSTEPS];   // B operand of the first product, kept for the whole kernel
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
  // Drain the q loads here, outside the loop.  The compiler cannot see the staging loads, so a
  // wait it placed inside the loop for these registers would also wait for tiles staged ahead.
  __builtin_amdgcn_s_waitcnt(0x0F70);

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

  const float c = p.c;
  const float thr = 8.0f / c;   // raise the running maximum only past this margin (raw score units)

  // per-lane fragment offsets inside a tile of 32 keys
  const int k_off = sigma(j) * RP + 8 * g;                                           // + 16 s
  const int i16 = lane & 15, q4 = lane >> 4;
  const int v_off = (8 * (q4 >> 1) + (i16 >> 2)) * VP + 16 * (q4 & 1) + 4 * (i16 & 3);   // + (16 m + 4 hh) * VP + 32 dt
  constexpr int LDT = D / 32, LLOC = D % 32;   // output tile / row that holds the softmax denominator

  // S^T = K Q^T for one 32-key tile
  auto qk = [&](f32x16(&S)[NQT], const bf16_t *ktile) {
    bf16x8 kf[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) kf[s] = *reinterpret_cast<const bf16x8 *>(ktile + k_off + 16 * s);
#pragma unroll
    for (int n = 0; n < NQT; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) S[n][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
      for (int n = 0; n < NQT; ++n) S[n] = mfma32(kf[s], qf[n][s], S[n]);
  };
  // first half of the online softmax: mask, tile maximum, and (rarely) raising the running maximum
  auto track_max = [&](f32x16(&S)[NQT], int key0, bool masked) {
    if (masked) {   // keys past the end of the sequence take no probability mass
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (key0 + key_of_reg(r, g) >= sk) {
#pragma unroll
          for (int n = 0; n < NQT; ++n) S[n][r] = -INFINITY;
        }
    }
    bool grow = false;
    float mx[NQT];
#pragma unroll
    for (int n = 0; n < NQT; ++n) {
      float a = fmaxf(fmaxf(S[n][0], S[n][1]), S[n][2]);
      float b = fmaxf(fmaxf(S[n][3], S[n][4]), S[n][5]);
#pragma unroll
      for (int r = 6; r < 14; r += 4) {
        a = fmaxf(fmaxf(a, S[n][r]), S[n][r + 1]);
        b = fmaxf(fmaxf(b, S[n][r + 2]), S[n][r + 3]);
      }
      a = fmaxf(fmaxf(a, S[n][14]), S[n][15]);
      mx[n] = fmaxf(a, b);   // over this lane's half of the keys; the other half sits in lane j + 32
      grow |= mx[n] > m_run[n] + thr;
    }
    // m_run is the same in both lanes of a query: if neither lane's half exceeds it by the margin,
    // the tile maximum does not either, and the two halves need not even be combined
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {   // rare after the first tile
#pragma unroll
      for (int n = 0; n < NQT; ++n) {
        const float m_new = fmaxf(m_run[n], max_pair(mx[n]));
        const float alpha = __builtin_amdgcn_exp2f((m_run[n] - m_new) * c);
        m_run[n] = m_new;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[n][dt][r] *= alpha;
      }
    }
  };
  // second half: P^T = exp2(c*S^T - c*m) rounded to bf16, laid out as B operands
  auto probs = [&](const f32x16(&S)[NQT], bf16x8(&pf)[NQT][2]) {
#pragma unroll
    for (int n = 0; n < NQT; ++n) {
      const float mc = m_run[n] * c;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        pf[n][r >> 3][r & 7] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(S[n][r], c, -mc));
    }
  };
  // O^T += V^T P^T; V^T fragments come from the row-major tile via transposing reads
  auto pv = [&](const bf16x8(&pf)[NQT][2], const bf16_t *vtile) {
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const bf16_t *vp = vtile + v_off + 16 * m * VP + 32 * dt;
        const bf16x4 lo = lds_read_tr4(vp), hi = lds_read_tr4(vp + 4 * VP);
        bf16x8 vf;
        vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
        vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
#pragma unroll
        for (int n = 0; n < NQT; ++n) oacc[n][dt] = mfma32(vf, pf[n][m], oacc[n][dt]);
      }
  };
  auto k_tile = [&](int t) { return smem + (t % NST) * STAGE_ELEMS; };
  auto v_tile = [&](int t) { return smem + (t % NST) * STAGE_ELEMS + TILE_ELEMS; };

  f32x16 S0[NQT], S1[NQT];
  bf16x8 pf[NQT][2];

  if (PIPE) {
    // One pipeline step on a full (unmasked) tile t whose scores are in Sc: make tile t+1 visible,
    // refill the stage that tile t-1 occupied, issue the scores of tile t+1 into Sn, finish tile t.
    auto step = [&](int t, f32x16(&Sc)[NQT], f32x16(&Sn)[NQT]) {
      const int ahead = ntile - 2 - t;                 // staged tiles beyond t+1
      wait_staged(ahead < NST - 3 ? ahead : NST - 3);  // tile t+1 has landed (this wavefront's share)
      __syncthreads();                                 // ... everyone's share; all are done with tile t-1
      if (t + NST - 1 < ntile) issue(t + NST - 1, (t + NST - 1) % NST);
      if (wave_active) {
        track_max(Sc, 0, false);
        qk(Sn, k_tile(t + 1));
        probs(Sc, pf);
        pv(pf, v_tile(t));
      }
    };

    wait_staged(npre - 1);   // tile 0 has landed
    __syncthreads();
    if (wave_active) qk(S0, k_tile(0));

    int t = 0;
    for (; t + 2 < ntile; t += 2) {
      step(t, S0, S1);
      step(t + 1, S1, S0);
    }
    // one or two tiles are left; the last of all may be partial
    const bool ragged = (sk & 31) != 0;
    if (t + 1 < ntile) {
      step(t, S0, S1);
      if (wave_active) {
        track_max(S1, 32 * (t + 1), ragged);
        probs(S1, pf);
        pv(pf, v_tile(t + 1));
      }
    } else if (wave_active) {
      track_max(S0, 32 * t, ragged);
      probs(S0, pf);
      pv(pf, v_tile(t));
    }
  } else {
    // Unpipelined variant: each tile is scored, normalised and accumulated in turn; overlap of
    // MFMA and VALU work then comes from the other wavefronts on the SIMD.
    for (int t = 0; t < ntile; ++t) {
      const int ahead = ntile - 1 - t;                 // staged tiles beyond t
      wait_staged(ahead < NST - 2 ? ahead : NST - 2);  // tile t has landed (this wavefront's share)
      __syncthreads();                                 // ... everyone's share; all are done with tile t-1
      if (t + NST - 1 < ntile) issue(t + NST - 1, (t + NST - 1) % NST);
      if (wave_active) {
        qk(S0, k_tile(t));
        track_max(S0, 32 * t, t == ntile - 1 && (sk & 31) != 0);
        probs(S0, pf);
        pv(pf, v_tile(t));
      }
    }
  }

  if (wave_active) {
    // ---- epilogue: divide by the denominator held in row D of O^T, store ----
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
}

}  // namespace pab
