// Tiled attention kernel for long query sequences (spatial and cross attention,
// paper Sec. 2.1): o = softmax(q k^T / sqrt(D)) v per (batch, head), computed
// with an online softmax over blocks of keys so that scores never reach memory.
//
// Work split: one workgroup = 4 wavefronts = 128*NQT consecutive queries of one
// (batch, head); each wavefront owns NQT tiles of 32 queries whose q fragments
// stay in registers.  Keys and values stream through a double-buffered LDS
// stage in blocks of KB keys, both stored row-major exactly as in memory (for
// bf16 inputs the global loads write LDS directly, no registers in between).
//
// Per 32-key tile and 32-query tile the wavefront computes, with bf16 MFMA:
//   S^T[key, query]  = K Q^T                (A = keys, B = queries)
//   P^T              = exp2(c*S^T - c*m)    (in registers, c = log2(e)/sqrt(D))
//   O^T[d, query]   += V^T P^T              (A = values read transposed, B = P^T)
// Keeping the query on the lane axis makes every softmax statistic a per-lane
// scalar, and (with the key permutation sigma) the accumulator registers of the
// first product are already the B operand of the second.  Row D of the V^T
// operand (a padding row of the 32-row output tile) is forced to 1.0, so row D
// of O^T accumulates the softmax denominator on the matrix core.  The running maximum m is only raised when some score exceeds it
// by more than 8 in the exponent (probabilities then stay below 2^8, harmless
// in fp32 / bf16); numerator and denominator always share the same m, so the
// quotient is unaffected.
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

// One wavefront-wide 16-byte-per-lane copy from global memory straight into LDS: lane i's 16 bytes
// at base + voff land at LDS byte address lds_addr + 16*i (lds_addr and base are wavefront-uniform).
// Completion is tracked by vmcnt; the compiler does not see this instruction, so the caller waits
// (s_waitcnt vmcnt(0)) before the barrier that publishes the data.
__device__ __forceinline__ void dma16_to_lds(const void *base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(base), "s"(lds_addr)
               : "memory");
}

__device__ __forceinline__ bf16x4 lds_read_tr4(const bf16_t *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3))) *)(p));
}

template <typename T, int D, int NQT, int KB, bool DIRECT>
__global__ __launch_bounds__(256, 2) void attn_tile_kernel(const TileParams p) {
  using HD = HeadDim<D>;
  constexpr int KSTEPS = HD::KSTEPS, DT = HD::DT, CH = HD::CH;
  constexpr int KT = KB / 32;        // 32-key tiles per block
  constexpr int QBLK = 128 * NQT;    // queries per workgroup
  constexpr int RP = D;              // row pitch of the K and V tiles in LDS: rows packed as in memory
  constexpr int TILE_ELEMS = KB * RP, STAGE_ELEMS = 2 * TILE_ELEMS;   // K tile, then V tile
  constexpr int SLACK = 64;          // fragment reads of a tile's last row run past its pitch: finite
                                     // garbage that only meets zero q columns / discarded output rows
  constexpr int NTC = KB * CH;       // 16-byte chunks per tile; chunk c = (row c / CH, chunk c % CH)
  static_assert(KB % 32 == 0, "key block must be a multiple of 32");
  static_assert(!DIRECT || sizeof(T) == 2, "direct-to-LDS staging needs bf16 inputs");
  static_assert(NTC % 64 == 0, "staging works in whole-wavefront rounds of 64 chunks");

  __shared__ __attribute__((aligned(16))) bf16_t smem[2 * STAGE_ELEMS + SLACK];

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

  // ---- staging of one key block into LDS stage `stage`.  The 2*NTC/64 rounds of 64 chunks (K tile
  //      first, then V tile) are dealt to the 4 wavefronts round-robin.  Rows past the end of the
  //      sequence re-read the last valid row: their scores are masked, so they carry no weight. ----
  constexpr int ROUNDS = 2 * NTC / 64;
  constexpr int MYR = (ROUNDS + 3) / 4;
  const int nkb = (sk + KB - 1) / KB;
  const unsigned smem_addr = (unsigned)(size_t)((__attribute__((address_space(3))) char *)smem);

  auto chunk_off = [&](int i, int blk) -> long long {   // element offset of this lane's chunk in round wave + 4 i
    const int round = wave + 4 * i;
    const int c = (round % (ROUNDS / 2)) * 64 + lane;
    int key = blk * KB + c / CH;
    key = key < sk ? key : sk - 1;
    return key * (round < ROUNDS / 2 ? p.k_ss : p.v_ss) + 8 * (c % CH);
  };

  bf16x8 stage_reg[DIRECT ? 1 : MYR];
  unsigned voff[DIRECT ? MYR : 1];   // byte offsets relative to the block's first K / V row
  if (DIRECT) {
#pragma unroll
    for (int i = 0; i < MYR; ++i) voff[i] = (unsigned)(2 * chunk_off(i, 0));
  }
  auto issue = [&](int blk, int stage) {
    const bool tail = (blk + 1) * KB > sk;
#pragma unroll
    for (int i = 0; i < MYR; ++i) {
      const int round = wave + 4 * i;
      if (round < ROUNDS) {
        const bool is_k = round < ROUNDS / 2;
        if (DIRECT) {
          const T *base = is_k ? kb_ + (long long)blk * KB * p.k_ss : vb + (long long)blk * KB * p.v_ss;
          const unsigned off = tail ? (unsigned)(2 * (chunk_off(i, blk) - (long long)blk * KB * (is_k ? p.k_ss : p.v_ss)))
                                    : voff[i];
          dma16_to_lds(base, off, smem_addr + 2 * stage * STAGE_ELEMS + 1024 * round);
        } else {
          stage_reg[i] = Io<T>::load8((is_k ? kb_ : vb) + chunk_off(i, blk));
        }
      }
    }
  };
  auto commit = [&](int stage) {
    if (DIRECT) {
      __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's share of the block has landed
    } else {
#pragma unroll
      for (int i = 0; i < MYR; ++i) {
        const int round = wave + 4 * i;
        if (round < ROUNDS)
          *reinterpret_cast<bf16x8 *>(smem + stage * STAGE_ELEMS + 512 * round + 8 * lane) = stage_reg[i];
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

  const float c = p.c;
  const float thr = 8.0f / c;   // raise the running maximum only past this margin (raw score units)

  // per-lane fragment offsets inside a stage
  const int k_off = sigma(j) * RP + 8 * g;                                   // + (32 kt) * RP + 16 s
  const int i16 = lane & 15, q4 = lane >> 4;
  const int v_off = TILE_ELEMS + (8 * (q4 >> 1) + (i16 >> 2)) * RP + 16 * (q4 & 1) + 4 * (i16 & 3);
                                                                             // + (32 kt + 16 m + 4 hh) * RP + 32 dt
  constexpr int LDT = D / 32, LLOC = D % 32;   // output tile / row that holds the softmax denominator
  const bool ones_lane = j == LLOC;

  if (tid < SLACK / 2) reinterpret_cast<unsigned *>(smem + 2 * STAGE_ELEMS)[tid] = 0u;   // the slack is defined

  issue(0, 0);
  commit(0);
  __syncthreads();

  for (int blk = 0; blk < nkb; ++blk) {
    const int stage = blk & 1;
    if (blk + 1 < nkb) issue(blk + 1, stage ^ 1);

    if (wave_active) {
      const bf16_t *st = smem + stage * STAGE_ELEMS;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        if (blk * KB + 32 * kt >= sk) break;   // tile entirely past the end of the sequence
        // ---- S^T = K Q^T for this 32-key tile ----
        f32x16 sacc[NQT];
        bf16x8 kf[KSTEPS];
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
          kf[s] = *reinterpret_cast<const bf16x8 *>(st + k_off + (32 * kt) * RP + 16 * s);
#pragma unroll
        for (int n = 0; n < NQT; ++n)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[n][r] = 0.0f;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
          for (int n = 0; n < NQT; ++n) sacc[n] = mfma32(kf[s], qf[n][s], sacc[n]);

        // keys past the end of the sequence take no probability mass
        if (blk == nkb - 1 && blk * KB + 32 * (kt + 1) > sk) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = blk * KB + 32 * kt + key_of_reg(r, g);
            if (key >= sk) {
#pragma unroll
              for (int n = 0; n < NQT; ++n) sacc[n][r] = -INFINITY;
            }
          }
        }

        // ---- online softmax, one query per lane (lanes j and j+32 share a query) ----
        bf16x8 pf[NQT][2];
#pragma unroll
        for (int n = 0; n < NQT; ++n) {
          float mx = fmaxf(sacc[n][0], sacc[n][1]);
#pragma unroll
          for (int r = 2; r < 16; r += 2) mx = fmaxf(mx, fmaxf(sacc[n][r], sacc[n][r + 1]));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          if (__builtin_amdgcn_ballot_w64(mx > m_run[n] + thr) != 0) {   // rare after the first tile
            const float m_new = fmaxf(m_run[n], mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run[n] - m_new) * c);
            m_run[n] = m_new;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
              for (int r = 0; r < 16; ++r) oacc[n][dt][r] *= alpha;
          }
          const float mc = m_run[n] * c;
#pragma unroll
          for (int r = 0; r < 16; ++r)
            pf[n][r >> 3][r & 7] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(sacc[n][r], c, -mc));
        }

        // ---- O^T += V^T P^T; V^T fragments come from the row-major tile via transposing reads ----
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const bf16_t *vp = st + v_off + (32 * kt + 16 * m) * RP + 32 * dt;
            const bf16x4 lo = lds_read_tr4(vp), hi = lds_read_tr4(vp + 4 * RP);
            bf16x8 vf;
            vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
            vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
            if (dt == LDT) vf = ones_lane ? splat8(1.0f) : vf;   // row D of V^T := 1 (rows past D: don't care)
#pragma unroll
            for (int n = 0; n < NQT; ++n) oacc[n][dt] = mfma32(vf, pf[n][m], oacc[n][dt]);
          }
      }
    }

    if (blk + 1 < nkb) commit(stage ^ 1);
    __syncthreads();   // next block visible to all; everyone is done with this one
  }

  if (!wave_active) return;

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

}  // namespace pab
