// Tiled attention kernel for long query sequences (spatial and cross attention,
// paper Sec. 2.1): o = softmax(q k^T / sqrt(D)) v per (batch, head), computed
// with an online softmax over tiles of keys so that scores never reach memory.
//
// Work split: one workgroup = NWV wavefronts works on one item of one (batch, head).
//   plain item:  32 NWV consecutive queries, one 32-query tile per wavefront, every wavefront walks
//                over all key tiles.
//   split item:  32 NWV / G consecutive queries.  The wavefronts form G key groups per query tile;
//                group g takes the key tiles t = g (mod G), so the item is done in 1/G of the steps,
//                and the partial results (running maximum, O^T with its denominator row) are combined
//                through LDS at the end.  The host turns the (batch, head) problems of a nearly empty
//                last round of workgroups into split items: four times as many workgroups, each a
//                quarter as long, fill the chip where a few long ones would leave most of it idle.
// Each wavefront keeps the q operands of its 32 queries in registers.  Keys and values stream through
// a ring of NRING LDS stages, one 32-key tile per stage, rows packed as in memory (for bf16 inputs the
// global loads write LDS directly, no registers in between).  A step of the loop publishes G tiles with
// one barrier; the tiles of the next AHEAD steps are in flight meanwhile.  Several workgroups share a
// CU, so that one wavefront's LDS and barrier waits are covered by the others.
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
// is unaffected.  m + margin and -m c are kept beside m, so that the test and the exponent cost no
// arithmetic of their own in the common case.
//
// Measured no faster: software pipelining inside the wavefront (scores of tile t + 1 issued
// before the exponentials of tile t), 64 queries per wavefront, wave priorities around the
// matrix or the exponential phases, accumulators in the AGPR half of the register file, 10 or 16
// wavefronts per workgroup, split items for the ragged last query block of every sequence.
#pragma once
#include <type_traits>
#include "mfma_util.hpp"

namespace pab {

struct TileParams {
  const void *q, *k, *v;
  void *o;
  int n_batch, n_head, sq, sk;
  long long q_bs, q_ss, k_bs, k_ss, v_bs, v_ss, o_bs, o_ss;  // batch / sequence strides, elements
  float c;          // log2(e) / sqrt(D)
  int n_item;       // plain items per (batch, head): 32 NWV queries each, the last possibly ragged
  int bh_plain;     // (batch, head) problems done as plain items: [0, bh_plain); the rest as split items
  int plain_wgs;    // workgroups of the plain class: n_item x bh_plain rounded up to a multiple of 8
  int n_split;      // split items per (batch, head) of the second class: 32 NWV / split_g queries each
  int split_g;      // their key groups (4)
};

constexpr int TILE_NRING = 8;   // LDS stages of the K/V ring

template <typename T, int D, int NWV, int MINW, bool DIRECT>
__global__ __launch_bounds__(64 * NWV, MINW) void attn_tile16_kernel(const TileParams p) {
  using HD = HeadDim<D>;
  constexpr int CH = HD::CH;
  constexpr int KB = 32;             // keys per LDS stage = one MFMA tile
  constexpr int NRING = TILE_NRING;
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
  static_assert(!DIRECT || sizeof(T) == 2, "direct-to-LDS staging needs bf16 inputs");
  static_assert(NWV == 8 || NWV == 4, "wavefronts split into 1 or 4 key groups");

  // 16-row tiles of O^T incl. the row of the denominator; words of one wavefront's O^T as its lanes hold it
  constexpr int DT16 = (D + 1 + 15) / 16, ACC_WORDS = 8 * DT16 * 64;
  // the ring, or (split items, after the loop) the running maxima of all wavefronts and the accumulators of the
  // key groups 1 .. G - 1, whichever is larger
  constexpr int RING_ELEMS = NRING * STAGE_ELEMS + SLACK, COMBINE_ELEMS = 2 * (32 * NWV + (NWV - 2) * ACC_WORDS);
  __shared__ __attribute__((aligned(16))) bf16_t smem[RING_ELEMS > COMBINE_ELEMS ? RING_ELEMS : COMBINE_ELEMS];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, g4 = lane >> 4;   // MFMA 16x16x32: row / column inside a sub-tile, 8-element k chunk

  // Workgroup ids are dealt round-robin to the 8 XCDs; give every XCD whole (batch, head)
  // problems so that all items of a problem share that XCD's L2 copy of K and V.  The plain items
  // come first in the grid, the short split items last, where they fill the end of the launch.
  const int n_bh = p.n_batch * p.n_head;
  int bh, q_item0, G;
  {
    const bool plain = (int)blockIdx.x < p.plain_wgs;
    const int b = plain ? (int)blockIdx.x : (int)blockIdx.x - p.plain_wgs;
    const int per = plain ? p.n_item : p.n_split;
    const int xcd = b & 7, slot = b >> 3;
    bh = (slot / per) * 8 + xcd + (plain ? 0 : p.bh_plain);
    const int idx = slot % per;
    G = plain ? 1 : p.split_g;
    q_item0 = plain ? idx * (32 * NWV) : idx * (32 * NWV / p.split_g);
    if (bh >= (plain ? p.bh_plain : n_bh)) return;
  }
  G = __builtin_amdgcn_readfirstlane(G);
  const int batch = bh / p.n_head, head = bh % p.n_head;

  const T *qb = reinterpret_cast<const T *>(p.q) + batch * p.q_bs + (long long)head * D;
  const T *kb_ = reinterpret_cast<const T *>(p.k) + batch * p.k_bs + (long long)head * D;
  const T *vb = reinterpret_cast<const T *>(p.v) + batch * p.v_bs + (long long)head * D;
  T *ob = reinterpret_cast<T *>(p.o) + batch * p.o_bs + (long long)head * D;
  const int sq = p.sq, sk = p.sk;

  const int lg_qt = (NWV == 8 ? 3 : 2) - (G >> 1);   // G = 1, 2, 4 -> log2 of the item's query tiles
  const int n_qt = 1 << lg_qt;
  const int qt = wave & (n_qt - 1), kg = wave >> lg_qt;   // this wavefront's query tile and key group
  const int q_wave0 = q_item0 + qt * 32;
  const bool wave_active = q_wave0 < sq;

  const int ntile = (sk + 31) >> 5;          // 32-key tiles, the last possibly partial
  const unsigned smem_addr = (unsigned)(size_t)((__attribute__((address_space(3))) char *)smem);

  // ---- prologue that does not depend on G: constants in LDS, q operands ----
  if (tid < SLACK / 2) reinterpret_cast<unsigned *>(smem + NRING * STAGE_ELEMS)[tid] = 0u;   // the slack is defined
  for (int idx = tid; idx < NRING * KB; idx += 64 * NWV) {   // constant chunk of every V row of every stage
    bf16x8 one = zero8();
    one[0] = (bf16_t)1.0f;
    *reinterpret_cast<bf16x8 *>(smem + (idx / KB) * STAGE_ELEMS + TILE_ELEMS + (idx % KB) * VP + D) = one;
  }

  // The first product runs over D head-dim columns: KS steps of 32, then, where at most 16 columns
  // remain, one 16-column step (half the multiply-adds of padding to another 32).
  constexpr int REM = D % 32;
  constexpr bool REM16 = REM > 0 && REM <= 16;
  constexpr int KS = REM16 ? D / 32 : (D + 31) / 32;
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

  // ---- one key tile t, staged in ring stage t % NRING ----
  auto compute_tile = [&](int t, bool ragged) {
    const bf16_t *ktile = smem + (t % NRING) * STAGE_ELEMS, *vtile = ktile + TILE_ELEMS;

    // S^T = K Q^T, four 16 x 16 sub-tiles: the 32-column steps of all four first, then (after the wait
    // states that a change of MFMA shape on an accumulator needs, see mfma_util.hpp) the 16-column steps
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
    if (ragged) {   // keys past the end of the sequence take no probability mass
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (32 * t + 16 * kh + 4 * g4 + r >= sk) {
            S[kh][0][r] = -INFINITY;
            S[kh][1][r] = -INFINITY;
          }
    }

    // running maximum: each lane looks at its own 8 keys per query (a chain of three-operand maxima); the
    // four lanes of a query hold the same m_run, so as long as none of them exceeds it by the margin nothing moves
    float mx[2];
    bool grow = false;
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
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

    // P^T as B operands: the lane's keys of the first half, then of the second
    bf16x8 pf[2];
#pragma unroll
    for (int qh = 0; qh < 2; ++qh)
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          pf[qh][4 * kh + r] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(S[kh][qh][r], c, m_negc[qh]));

    // O^T += V^T P^T: 16 rows of V^T over all 32 keys per instruction
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

  // ---- the loop over steps of GG key tiles each.  Staging: the ROUNDS rounds of each of the GG tiles
  //      of a step are dealt to the wavefronts round-robin (the last round of a wavefront may repeat one,
  //      so that every wavefront issues the same number of loads per step and vmcnt can count them).
  //      Rows past the end of the sequence re-read the last valid row: their scores are masked or their
  //      tile is not computed at all. ----
  auto run = [&](auto g_tag) {
    constexpr int GG = decltype(g_tag)::value;
    constexpr int SROUNDS = ROUNDS * GG;                // rounds per step
    constexpr int MYR = (SROUNDS + NWV - 1) / NWV;      // ... per wavefront
    constexpr int AHEAD = GG == 4 ? 1 : 3;              // steps in flight beyond the one being computed
    static_assert((AHEAD + 1) * GG <= NRING && AHEAD * MYR < 64, "ring depth / vmcnt immediates");
    const int nstep = (ntile + GG - 1) / GG;

    auto my_round = [&](int i) { const int r = wave + NWV * i; return r < SROUNDS ? r : SROUNDS - 1; };
    auto tile_of = [&](int i) { return my_round(i) / ROUNDS; };          // tile of the step, 0 .. GG - 1
    auto tround = [&](int i) { return my_round(i) % ROUNDS; };           // round inside that tile
    // chunk slot of this lane inside the K or V tile, and whether it carries data
    auto slot_of = [&](int i) { const int r = tround(i); return (r < PRK ? r : r - PRK) * 64 + lane; };
    auto live = [&](int i) {
      const int cs = slot_of(i);
      return tround(i) < PRK ? cs < KB * CH : (cs < KB * VCH && cs % VCH < CH);
    };
    auto chunk_off = [&](int i, int t) -> long long {   // element offset of this lane's chunk of tile t
      const bool is_k = tround(i) < PRK;
      const int cs = slot_of(i), per = is_k ? CH : VCH;
      const int row = cs / per;
      int chunk = cs % per;
      if (is_k && chunk < KSWZ_CHUNKS) chunk ^= k_swizzle<D>(row);   // the K tile is stored swizzled
      int key = t * KB + row;
      key = key < sk ? key : sk - 1;
      return key * (is_k ? p.k_ss : p.v_ss) + 8 * chunk;
    };
    unsigned voff[MYR];   // byte offsets relative to the first K / V row of the step's first tile (whole tiles)
#pragma unroll
    for (int i = 0; i < MYR; ++i) voff[i] = (unsigned)(2 * chunk_off(i, tile_of(i)));

    // request the GG tiles of step s; WHOLE: all of them lie inside the sequence
    auto issue = [&](int s, auto whole_tag) {
      constexpr bool WHOLE = decltype(whole_tag)::value;
#pragma unroll
      for (int i = 0; i < MYR; ++i) {
        const int tr = tround(i);
        const bool is_k = tr < PRK;
        const int t = s * GG + tile_of(i);
        const long long s_off = (long long)s * GG * KB * (is_k ? p.k_ss : p.v_ss);
        const int lds_elem = (t % NRING) * STAGE_ELEMS + (is_k ? 512 * tr : TILE_ELEMS + 512 * (tr - PRK));
        if (live(i)) {   // idle lanes: past the tile, or on a constant chunk that must survive
          if (DIRECT) {
            const unsigned off = WHOLE ? voff[i] : (unsigned)(2 * (chunk_off(i, t) - s_off));
            dma16_to_lds((is_k ? kb_ : vb) + s_off, off, smem_addr + 2 * lds_elem);
          } else {   // element types that need conversion go through registers, synchronously
            *reinterpret_cast<bf16x8 *>(smem + lds_elem + 8 * lane) = Io<T>::load8((is_k ? kb_ : vb) + chunk_off(i, t));
          }
        }
      }
    };
    // wait until at most `steps` of this wavefront's staged steps are still in flight
    auto wait_staged = [&](int steps) {
      if (!DIRECT) return;
      if (steps >= 3 && AHEAD >= 3) __builtin_amdgcn_s_waitcnt(0x0F70 | ((3 * MYR) & 15) | (((3 * MYR) >> 4) << 14));
      else if (steps == 2 && AHEAD >= 2) __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * MYR) & 15) | (((2 * MYR) >> 4) << 14));
      else if (steps >= 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (MYR & 15) | ((MYR >> 4) << 14));
      else __builtin_amdgcn_s_waitcnt(0x0F70);
    };

    const int npre = nstep < AHEAD ? nstep : AHEAD;
    for (int s = 0; s < npre; ++s) issue(s, std::false_type{});
    // drain the q loads here, outside the loop: the staging loads are invisible to the compiler, so its own
    // count of outstanding loads must not be relied on once they are mixed in
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // STEADY steps find the ring full and request another step of whole tiles: their waits and requests
    // need no case distinctions, which keeps scalar work and branches out of the loop that runs almost
    // all of the time.
    auto step = [&](int s, auto steady_tag) {
      constexpr bool STEADY = decltype(steady_tag)::value;
      if (STEADY) {
        wait_staged(AHEAD - 1);
        __syncthreads();
        issue(s + AHEAD, std::true_type{});
      } else {
        const int ahead = nstep - 1 - s;                     // staged steps beyond s
        wait_staged(ahead < AHEAD - 1 ? ahead : AHEAD - 1);  // step s has landed (this wavefront's share)
        __syncthreads();                                     // ... everyone's share; all are done with step s-1
        if (s + AHEAD < nstep) issue(s + AHEAD, std::false_type{});
      }
      const int t = s * GG + kg;
      if (!wave_active || (GG > 1 && t >= ntile)) return;
      compute_tile(t, !STEADY && t == ntile - 1 && (sk & 31) != 0);
    };
    // the last AHEAD steps request nothing, and steps that touch a ragged last tile are requested lane by lane
    const int n_steady = (sk >> 5) / GG - AHEAD;
    int s = 0;
    for (; s < n_steady; ++s) step(s, std::true_type{});
    for (; s < nstep; ++s) step(s, std::false_type{});
  };
  if (G == 1) run(std::integral_constant<int, 1>{});
  else run(std::integral_constant<int, 4>{});

  // ---- split items: combine the key groups of a query tile through LDS (the ring is free now).
  //      Layout: maxima [wave][32 queries] floats, then per query tile 16 DT16 x 64 lanes of floats
  //      (register-major, so a wavefront's 64 lanes touch 64 consecutive words). ----
  if (G > 1) {
    float *red_m = reinterpret_cast<float *>(smem);
    float *red_o = red_m + 32 * NWV;
    __syncthreads();                       // every wavefront is done reading the ring
    if (g4 == 0) {
      red_m[wave * 32 + l16] = m_run[0];
      red_m[wave * 32 + 16 + l16] = m_run[1];
    }
    __syncthreads();
    float scale[2];
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      float m_all = m_run[qh];
      for (int g = 0; g < G; ++g) m_all = fmaxf(m_all, red_m[(g * n_qt + qt) * 32 + 16 * qh + l16]);
      // a group that saw no key has m = -inf and nothing accumulated: its factor is 0, not NaN
      scale[qh] = m_run[qh] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((m_run[qh] - m_all) * c);
    }
    // groups 1 .. G - 1 leave their rescaled accumulators in LDS (register-major: a wavefront's 64 lanes touch 64
    // consecutive words), group 0 adds them to its own
    if (kg != 0) {
      float *dst = red_o + (wave - n_qt) * ACC_WORDS + lane;
#pragma unroll
      for (int dt = 0; dt < DT16; ++dt)
#pragma unroll
        for (int qh = 0; qh < 2; ++qh)
#pragma unroll
          for (int r = 0; r < 4; ++r) dst[((2 * dt + qh) * 4 + r) * 64] = oacc[dt][qh][r] * scale[qh];
    }
    __syncthreads();
    if (kg != 0) return;
#pragma unroll
    for (int dt = 0; dt < DT16; ++dt)
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 4; ++r) oacc[dt][qh][r] *= scale[qh];
    for (int g = 1; g < G; ++g) {
      const float *src = red_o + (g * n_qt + qt - n_qt) * ACC_WORDS + lane;
#pragma unroll
      for (int dt = 0; dt < DT16; ++dt)
#pragma unroll
        for (int qh = 0; qh < 2; ++qh)
#pragma unroll
          for (int r = 0; r < 4; ++r) oacc[dt][qh][r] += src[((2 * dt + qh) * 4 + r) * 64];
    }
  }

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
