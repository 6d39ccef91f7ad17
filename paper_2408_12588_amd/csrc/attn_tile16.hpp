// Tiled attention kernel for long query sequences (spatial and cross attention,
// paper Sec. 2.1): o = softmax(q k^T / sqrt(D)) v per (batch, head), computed
// with an online softmax over tiles of keys so that scores never reach memory.
//
// Work split: one workgroup = NWV wavefronts = 32 NWV consecutive queries of one
// (batch, head); each wavefront owns 32 queries whose q operands stay in registers.
// Keys and values stream through a ring of NST LDS stages, one 32-key tile per
// stage, rows packed as in memory (for bf16 inputs the global loads write LDS
// directly, no registers in between, NST-2 tiles ahead of their use).  Several
// workgroups share a CU, so that one wavefront's LDS and barrier waits are covered
// by the others.
//
// The products are v_mfma_f32_16x16x32_bf16.  Against 32 x 32 x 16 tiles that instruction moves
// half the accumulator data per multiply-add and sustains about 12% more under the chip's power
// limit, and 16-row output tiles fit the D + 1 = 73 rows of O^T in 80 instead of 96.
// Per 32-key tile a wavefront holds four 16 x 16 score sub-tiles S^T[kh][qh] (key half kh, query
// half qh).  Lane (l16, g4) of a sub-tile owns query l16 and keys 4 g4 .. + 3:
//   S^T[kh][qh]  = K[kh] Q[qh]^T     A = 16 key rows, B = 16 queries, 32 head-dim columns per step
//   P^T[qh]      = exp2(c S^T - c m)  (c = log2(e) / sqrt(D)) the lane's 4 + 4 probabilities of the
//                                     two key halves are the 8 k-slots of its B operand: k-slot
//                                     8 g4 + e is key 4 g4 + e (e < 4) or 16 + 4 g4 + e - 4
//   O^T[dt][qh] += V^T[dt] P^T[qh]    A = 16 rows of V^T read transposed from the row-major tile in
//                                     the same key order, all 32 keys in one instruction
// Keeping the query on the lane axis makes every softmax statistic a per-lane scalar, and the
// accumulator registers of the first product are already the B operand of the second.  V rows in
// LDS carry one extra 16-byte chunk {1, 0, ..} after their D values (written once; the staging
// loads skip it), so row D of V^T is all ones and row D of O^T accumulates the softmax denominator
// on the matrix core.  Four lanes share a query (g4 = 0..3) and hold the same running maximum m;
// m is only raised when some lane's scores exceed it by more than 8 in the exponent
// (probabilities then stay below 2^8, harmless in fp32 / bf16), and only then do the four lanes
// exchange their tile maxima.  Numerator and denominator always share the same m, so the quotient
// is unaffected.  m + margin and -m c are kept beside m (they change only when m does), so the test
// and the exponent's offset cost no arithmetic of their own per tile.
//
// Measured no faster: software pipelining inside the wavefront (scores of tile t + 1 issued
// before the exponentials of tile t), 64 queries per wavefront, wave priorities around the
// matrix or the exponential phases, O^T accumulators in the AGPR half of the register file,
// 10 or 16 wavefronts per workgroup, splitting the ragged last query block of a sequence over
// key groups that combine through LDS.
#pragma once
#include <type_traits>
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


template <typename T, int D, int NWV, int NST, int MINW, bool DIRECT>
__global__ __launch_bounds__(64 * NWV, MINW) void attn_tile16_kernel(const TileParams p) {
  using HD = HeadDim<D>;
  constexpr int CH = HD::CH;
  constexpr int KB = 32;             // keys per LDS stage = one MFMA tile
  constexpr int QBLK = 32 * NWV;   // queries per workgroup
  constexpr int RP = D;              // row pitch of the K tile in LDS: rows packed as in memory
  constexpr int VCH = CH + 1;        // chunks per V row in LDS: CH of data, then the constant chunk {1, 0, ..}
  constexpr int VP = 8 * VCH;        // row pitch of the V tile
  constexpr int TILE_ELEMS = KB * RP;                       // K rows ...
  constexpr int STAGE_ELEMS = TILE_ELEMS + KB * VP;         // ... then V rows
  constexpr int SLACK = 64;          // fragment reads of a tile's last row run past its pitch: finite
                                     // garbage that only meets zero q columns / discarded output rows
  constexpr int KSWZ_CHUNKS = 4 * (D / 32);   // chunks of a K row that the 16-byte operand reads cover
  constexpr int PRK = (KB * CH + 63) / 64;   // staging rounds (64 chunk slots each, the last maybe partial) of the K tile
  constexpr int PRV = (KB * VCH + 63) / 64;  // ... of the V tile (the slots of the constant chunks stay idle)
  constexpr int ROUNDS = PRK + PRV;          // K rounds, then V rounds
  constexpr int MYR = (ROUNDS + NWV - 1) / NWV;   // rounds per wavefront (the last may repeat a round)
  static_assert(!DIRECT || sizeof(T) == 2, "direct-to-LDS staging needs bf16 inputs");
  static_assert(NST >= 3 && NST <= 5 && (NST - 2) * MYR < 16, "ring depth / vmcnt immediates");

  __shared__ __attribute__((aligned(16))) bf16_t smem[NST * STAGE_ELEMS + SLACK];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;   // MFMA 16x16x32: row / column inside a sub-tile, 8-element k chunk

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

  const int q_wave0 = qblk * QBLK + wave * 32;
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
    const int row = c / per;
    int chunk = c % per;
    if (is_k && chunk < KSWZ_CHUNKS) chunk ^= k_swizzle<D>(row);   // the K tile is stored swizzled
    int key = t * KB + row;
    key = key < sk ? key : sk - 1;
    return key * (is_k ? p.k_ss : p.v_ss) + 8 * chunk;
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
  auto issue_full = [&](int t, int stage) {   // the same for a tile known to lie inside the sequence
#pragma unroll
    for (int i = 0; i < MYR; ++i) {
      const int round = my_round(i);
      const bool is_k = round < PRK;
      const long long t_off = (long long)t * KB * (is_k ? p.k_ss : p.v_ss);
      const int lds_elem = stage * STAGE_ELEMS + (is_k ? 512 * round : TILE_ELEMS + 512 * (round - PRK));
      if (live(i)) {
        if (DIRECT) dma16_to_lds((is_k ? kb_ : vb) + t_off, voff[i], smem_addr + 2 * lds_elem);
        else *reinterpret_cast<bf16x8 *>(smem + lds_elem + 8 * lane) = Io<T>::load8((is_k ? kb_ : vb) + chunk_off(i, t));
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

  // ---- prologue: first NST-1 tiles on their way, then the q operands ----
  if (tid < SLACK / 2) reinterpret_cast<unsigned *>(smem + NST * STAGE_ELEMS)[tid] = 0u;   // the slack is defined
  for (int idx = tid; idx < NST * KB; idx += 64 * NWV) {   // constant chunk of every V row of every stage
    bf16x8 one = zero8();
    one[0] = (bf16_t)1.0f;
    *reinterpret_cast<bf16x8 *>(smem + (idx / KB) * STAGE_ELEMS + TILE_ELEMS + (idx % KB) * VP + D) = one;
  }
  const int npre = ntile < NST - 1 ? ntile : NST - 1;
  for (int t = 0; t < npre; ++t) issue(t, t);

  // The first product runs over D head-dim columns: KS steps of 32, then, where at most 16 columns
  // remain, one 16-column step (half the multiply-adds of padding to another 32).
  constexpr int REM = D % 32;
  constexpr bool REM16 = REM > 0 && REM <= 16;
  constexpr int KS = REM16 ? D / 32 : (D + 31) / 32;
  constexpr int DT16 = (D + 1 + 15) / 16;    // 16-row tiles of O^T incl. the row of the denominator
  bf16x8 qf[2][KS];   // B operand of the first product: query 16 qh + l16, columns 32 ks + 8 g4 .. + 7
  bf16x4 qr[2];       // ... of the 16-column step: columns 32 KS + 4 g4 .. + 3
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) {
    int qrow = q_wave0 + 16 * qh + l16;
    qrow = qrow < sq ? qrow : sq - 1;   // tail rows load a valid row and are never stored
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int d0 = 32 * ks + 8 * g4;
      qf[qh][ks] = (d0 < D) ? Io<T>::load8(qb + qrow * p.q_ss + d0) : zero8();
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) qr[qh][e] = (bf16_t)0.0f;
    if (REM16 && 32 * KS + 4 * g4 < D) qr[qh] = Io<T>::load4(qb + qrow * p.q_ss + 32 * KS + 4 * g4);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the q loads outside the loop (the staging loads are invisible to the compiler)

  f32x4 oacc[DT16][2];
  float m_run[2], m_thr[2], m_negc[2];   // running maximum, m + margin, -m c: the last two change only when m does
#pragma unroll
  for (int qh = 0; qh < 2; ++qh) {
    m_run[qh] = -INFINITY;
    m_thr[qh] = -INFINITY;
    m_negc[qh] = 0.0f;
#pragma unroll
    for (int dt = 0; dt < DT16; ++dt)
#pragma unroll
      for (int r = 0; r < 4; ++r) oacc[dt][qh][r] = 0.0f;
  }

  const float c = p.c;
  const float thr = 8.0f / c;   // raise the running maximum only past this margin (raw score units)
  const int k_off = l16 * RP + 8 * (g4 ^ k_swizzle<D>(l16));             // + 16 kh * RP + 32 ks
  const int kr_off = l16 * RP + 32 * KS + 4 * g4;                       // + 16 kh * RP
  const int v_off = (4 * g4 + (l16 >> 2)) * VP + 4 * (l16 & 3);        // + 16 * VP for the second key half, + 16 dt

  // One key tile.  STEADY iterations are those that find the ring full and request another whole
  // tile: their waits and requests need no case distinctions, which keeps scalar work and branches
  // out of the loop that runs almost all of the time.
  auto step = [&](int t, auto steady_tag) {
    constexpr bool STEADY = decltype(steady_tag)::value;
    if (STEADY) {
      wait_staged(NST - 2);
      __syncthreads();
      issue_full(t + NST - 1, (t + NST - 1) % NST);
    } else {
      const int ahead = ntile - 1 - t;                 // staged tiles beyond t
      wait_staged(ahead < NST - 2 ? ahead : NST - 2);  // tile t has landed (this wavefront's share)
      __syncthreads();                                 // ... everyone's share; all are done with tile t-1
      if (t + NST - 1 < ntile) issue(t + NST - 1, (t + NST - 1) % NST);
    }
    if (!wave_active) return;
    const bf16_t *ktile = smem + (t % NST) * STAGE_ELEMS, *vtile = ktile + TILE_ELEMS;

    // ---- S^T = K Q^T, four 16 x 16 sub-tiles: the 32-column steps of all four first, then (after the wait
    //      states that a change of MFMA shape on an accumulator needs, see mfma_util.hpp) the 16-column steps ----
    f32x4 S[2][2];
    bf16x4 kr[2];
#pragma unroll
    for (int kh = 0; kh < 2; ++kh) {
      bf16x8 kf[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(ktile + k_off + 16 * kh * RP + 32 * ks);
      // columns past D (lane groups whose q columns are zero) read on into the next row: finite
      if (REM16) kr[kh] = *reinterpret_cast<const bf16x4 *>(ktile + kr_off + 16 * kh * RP);
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) {
#pragma unroll
        for (int r = 0; r < 4; ++r) S[kh][qh][r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) S[kh][qh] = mfma16(kf[ks], qf[qh][ks], S[kh][qh]);
      }
    }
    if (REM16) {
      mfma_shape_change(S[0][0], S[0][1], S[1][0], S[1][1]);
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int qh = 0; qh < 2; ++qh) S[kh][qh] = mfma16_k16(kr[kh], qr[qh], S[kh][qh]);
    }
    if (!STEADY && t == ntile - 1 && (sk & 31) != 0) {   // keys past the end of the sequence take no probability mass
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (32 * t + 16 * kh + 4 * g4 + r >= sk) {
            S[kh][0][r] = -INFINITY;
            S[kh][1][r] = -INFINITY;
          }
    }

    // ---- running maximum: each lane looks at its own 8 keys per query; the four lanes of a query
    //      hold the same m_run, so as long as none of them exceeds it by the margin nothing moves ----
    float mx[2];
    bool grow = false;
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {   // a chain of three-operand maxima: 3 + 1 instructions for the 8 scores
      float a = fmaxf(fmaxf(S[0][qh][0], S[0][qh][1]), S[0][qh][2]);
      a = fmaxf(fmaxf(a, S[0][qh][3]), S[1][qh][0]);
      a = fmaxf(fmaxf(a, S[1][qh][1]), S[1][qh][2]);
      mx[qh] = fmaxf(a, S[1][qh][3]);
      grow |= mx[qh] > m_thr[qh];
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {   // rare after the first tile
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) {
        float full = fmaxf(mx[qh], __shfl_xor(mx[qh], 16));
        full = fmaxf(full, __shfl_xor(full, 32));
        const float m_new = fmaxf(m_run[qh], full);
        const float alpha = __builtin_amdgcn_exp2f((m_run[qh] - m_new) * c);
        m_run[qh] = m_new;
        m_thr[qh] = m_new + thr;
        m_negc[qh] = -m_new * c;
#pragma unroll
        for (int dt = 0; dt < DT16; ++dt)
#pragma unroll
          for (int r = 0; r < 4; ++r) oacc[dt][qh][r] *= alpha;
      }
    }

    // ---- P^T as B operands: the lane's keys of the first half, then of the second ----
    bf16x8 pf[2];
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          pf[qh][4 * kh + r] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(S[kh][qh][r], c, m_negc[qh]));
    }

    // ---- O^T += V^T P^T: 16 rows of V^T over all 32 keys per instruction ----
#pragma unroll
    for (int dt = 0; dt < DT16; ++dt) {
      const bf16_t *vp = vtile + v_off + 16 * dt;
      const bf16x4 lo = lds_read_tr4(vp), hi = lds_read_tr4(vp + 16 * VP);
      bf16x8 vf;
      vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
      vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) oacc[dt][qh] = mfma16(vf, pf[qh], oacc[dt][qh]);
    }
  };
  // the last NST - 1 tiles request nothing, and a ragged last tile is requested lane by lane
  const int n_steady = ntile - (NST - 1) - ((sk & 31) != 0 ? 1 : 0);
  int t = 0;
  for (; t < n_steady; ++t) step(t, std::true_type{});
  for (; t < ntile; ++t) step(t, std::false_type{});

  if (wave_active) {
    // ---- epilogue: row D of O^T is the denominator; it sits in sub-tile D / 16, lane group (D % 16) / 4 ----
    constexpr int DEN_DT = D / 16, DEN_G = (D % 16) / 4, DEN_R = D % 4;
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      const float inv = 1.0f / __shfl(oacc[DEN_DT][qh][DEN_R], l16 + 16 * DEN_G);
      const int qrow = q_wave0 + 16 * qh + l16;
      if (qrow < sq) {
        T *orow = ob + qrow * p.o_ss;
#pragma unroll
        for (int dt = 0; dt < DT16; ++dt) {
          const int d0 = 16 * dt + 4 * g4;
          if (d0 < D)
            Io<T>::store4(orow + d0, oacc[dt][qh][0] * inv, oacc[dt][qh][1] * inv, oacc[dt][qh][2] * inv,
                          oacc[dt][qh][3] * inv);
        }
      }
    }
  }
}

}  // namespace pab
