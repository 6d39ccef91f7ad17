// Cross attention (paper Sec. 2.1): every video token attends to the L text
// tokens of the conditioning input.  L is short (<= 128 here), so per head the
// keys and values fit in LDS once and for all and the softmax needs a single
// pass; what is left per token is streaming q in and o out of HBM, and a fixed
// amount of matrix-core and exp work per 32-token tile.
//
// One workgroup = NW wavefronts serves one head: it stages that head's K and V
// rows ([L, D], row-major as in memory) into LDS once, then each wavefront walks
// over 32-query tiles of the head with a stride of all wavefronts serving it.
// The wavefronts never synchronise with each other after the K/V load.
//
// A wavefront owns two LDS tile buffers: X receives q tiles (direct global ->
// LDS loads, 16 bytes per lane, consecutive lanes on consecutive chunks of a
// row), Y holds the finished output tile until it is written out, whole rows
// per instruction.  The loop over tiles is software pipelined so that the
// matrix core always has work while the softmax runs on the vector ALU:
//
//   iteration for tile t (its scores S^T = K Q^T are already in registers):
//     wait for all outstanding memory operations (all one iteration old)
//     write tile t-1 from Y to global memory
//     fetch the q operands of tile t+1 from X, then request tile t+2 into X
//     row max of S; for each 32-key tile kt:
//         P^T = exp2(c (S^T - max))            (vector ALU)
//         O^T += V^T P^T                       (matrix core)
//         S^T[kt] of tile t+1 = K[kt] Q^T      (matrix core, reuses the registers)
//     normalise O and stage it in Y
//
// Keys are permuted so that the accumulator registers of the first product are
// the B operand of the second.  V rows in LDS carry an extra chunk {1, 0, ..}:
// row D of O^T is then the softmax denominator.  K rows past L repeat row L-1
// (so the row max is unchanged) while V rows past L are all zero, constant
// chunk included: such keys add nothing to numerator or denominator and no
// score has to be masked.
#pragma once
#include <type_traits>
#include "mfma_util.hpp"

namespace pab {

struct CrossParams {
  const void *q, *k, *v;
  void *o;
  int n_tok, L, n_head;
  int wg_per_head;     // workgroups that share one head
  float c;             // log2(e) / sqrt(D)
};

// LT: 32-key tiles that hold L (1..4).  NW: wavefronts per workgroup.
template <int D, int LT, int NW>
__global__ __launch_bounds__(64 * NW) void attn_cross_kernel(const CrossParams p) {
  using HD = HeadDim<D>;
  using T = bf16_t;
  constexpr int KSTEPS = HD::KSTEPS, DT = HD::DT, CH = HD::CH;
  constexpr int LP = 32 * LT;               // key rows held in LDS
  constexpr int RP = D;                     // row pitch: rows packed as in memory
  // V rows in LDS: CH data chunks, the constant chunk, then zero chunks up to a pitch of 96 elements = 48 banks.
  // A transposed 8-byte read takes 64 bytes from each of four consecutive rows per half wavefront; with rows
  // 48 banks apart these four stretches are the four quarters of the 64 banks (0, 48, 32, 16), with the 40 banks
  // of the minimal pitch the fourth overlapped the first (every such read took twice as long).
  constexpr int VCH = 12, VP = 8 * VCH;
  static_assert(CH + 1 <= VCH, "head dim too long for the V row pitch");
  constexpr int K_ELEMS = LP * RP, V_ELEMS = LP * VP, KV_ELEMS = K_ELEMS + V_ELEMS;
  constexpr int QB_ELEMS = 32 * RP;         // one tile buffer
  constexpr int NCHUNK = 32 * CH;           // 16-byte chunks of a tile
  constexpr int KR = (LP * CH + 63) / 64;   // staging rounds (64 chunk slots) for K
  constexpr int VR = (LP * VCH + 63) / 64;  // ... for V
  constexpr int QR = (NCHUNK + 63) / 64;    // rounds for a q / o tile (the last may be partial)
  constexpr int ZERO_ELEMS = 64;            // zeros behind the buffers (operand columns past D)
  static_assert(LT >= 1 && LT <= 4, "keys must fit four 32-key tiles");

  __shared__ __attribute__((aligned(16))) bf16_t smem[KV_ELEMS + NW * 2 * QB_ELEMS + ZERO_ELEMS];
  bf16_t *Ks = smem, *Vs = smem + K_ELEMS;
  bf16_t *zeros = smem + KV_ELEMS + NW * 2 * QB_ELEMS;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31, g = lane >> 5;
  const unsigned smem_addr = (unsigned)(size_t)((__attribute__((address_space(3))) char *)smem);

  // Workgroup ids go round-robin over the 8 XCDs.  An XCD takes one contiguous eighth of the tokens
  // for all heads, so that the cache lines shared by neighbouring heads (rows are D elements, not
  // a multiple of the line) are used up inside one L2.  The host makes wg_per_head a multiple of 8
  // whenever there are enough tiles; otherwise the split is plain round-robin.
  const int H = p.n_head;
  const int ntile = (p.n_tok + 31) >> 5;
  int head, t_lo, t_hi, part, parts;
  if ((p.wg_per_head & 7) == 0) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    head = slot % H;
    part = slot / H;
    parts = p.wg_per_head >> 3;
    t_lo = (int)((long long)ntile * xcd / 8);
    t_hi = (int)((long long)ntile * (xcd + 1) / 8);
  } else {
    head = blockIdx.x % H;
    part = blockIdx.x / H;
    parts = p.wg_per_head;
    t_lo = 0;
    t_hi = ntile;
  }
  const long long row = (long long)H * D;   // token stride, elements
  const T *qh = reinterpret_cast<const T *>(p.q) + (long long)head * D;
  const T *kh = reinterpret_cast<const T *>(p.k) + (long long)head * D;
  const T *vh = reinterpret_cast<const T *>(p.v) + (long long)head * D;
  T *oh = reinterpret_cast<T *>(p.o) + (long long)head * D;
  const int n_tok = p.n_tok, L = p.L;
  const int stride = parts * NW;
  bf16_t *X = smem + KV_ELEMS + wave * (2 * QB_ELEMS), *Y = X + QB_ELEMS;
  const unsigned x_addr = smem_addr + 2 * (unsigned)(X - smem);

  // ---- K and V of the head, rounds dealt round-robin to the wavefronts.  Slots that no load
  //      fills (V rows past L, the constant chunks) are written as ordinary LDS stores. ----
  for (int r = wave; r < KR + VR; r += NW) {
    if (r < KR) {
      const int c = r * 64 + lane;
      if (c < LP * CH) {
        int key = c / CH;
        key = key < L ? key : L - 1;
        dma16_to_lds(kh, (unsigned)(2 * (key * row + 8 * (c % CH))), smem_addr + 1024 * r);
      }
    } else {
      const int c = (r - KR) * 64 + lane, key = c / VCH, chunk = c % VCH;
      const bool real = c < LP * VCH && key < L && chunk < CH;
      if (real) dma16_to_lds(vh, (unsigned)(2 * (key * row + 8 * chunk)), smem_addr + 2 * K_ELEMS + 1024 * (r - KR));
      if (c < LP * VCH && !real) {
        bf16x8 fill = zero8();
        if (chunk == CH && key < L) fill[0] = (bf16_t)1.0f;
        *reinterpret_cast<bf16x8 *>(Vs + 8 * c) = fill;
      }
    }
  }
  if (tid < ZERO_ELEMS / 2) reinterpret_cast<unsigned *>(zeros)[tid] = 0u;

  // ---- lane constants of the tile copies: chunk c = 64 r + lane of a tile is row c / CH, chunk
  //      c % CH of that row; in LDS the tile is packed, so the chunk sits at element 8 c. ----
  int trow[QR];
  unsigned voff[QR];   // byte offset of the chunk from the tile's first row in global memory
#pragma unroll
  for (int r = 0; r < QR; ++r) {
    const int c = r * 64 + lane;
    trow[r] = c / CH;
    voff[r] = (unsigned)(2 * (trow[r] * row + 8 * (c % CH)));
  }

  // q tile t -> X.  Rows past the last token repeat the last one (their results are never stored).
  // Token offsets can exceed 32 bits: the base moves with the tile, the lane offset stays small.
  auto stage_q = [&](int t) {
    const int tok0 = 32 * t;
    const T *base = qh + (long long)tok0 * row;
    const bool whole = tok0 + 32 <= n_tok;
#pragma unroll
    for (int r = 0; r < QR; ++r) {
      const int c = r * 64 + lane;
      if (c < NCHUNK) {
        unsigned off = voff[r];
        if (!whole) {
          const int tr = min(trow[r], n_tok - 1 - tok0);
          off = (unsigned)(2 * (tr * row + 8 * (c - CH * trow[r])));
        }
        dma16_to_lds(base, off, x_addr + 1024 * r);
      }
    }
  };

  // finished tile t: Y -> global memory, whole rows per instruction
  auto store_tile = [&](int t) {
    char *ot = reinterpret_cast<char *>(oh + (long long)(32 * t) * row);
    bf16x8 val[QR];
#pragma unroll
    for (int r = 0; r < QR; ++r) val[r] = *reinterpret_cast<const bf16x8 *>(Y + 8 * min(r * 64 + lane, NCHUNK - 1));
#pragma unroll
    for (int r = 0; r < QR; ++r)
      if (r * 64 + lane < NCHUNK && 32 * t + trow[r] < n_tok) *reinterpret_cast<bf16x8 *>(ot + voff[r]) = val[r];
  };

  int t = t_lo + part * NW + wave;
  if (t < t_hi) stage_q(t);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // K, V (this wavefront's share) and the first q tile have landed
  __syncthreads();                      // ... everyone's share of K and V
  if (t >= t_hi) return;

  const float c = p.c;
  const int k_off = sigma(j) * RP + 8 * g;                                             // + 32 kt * RP + 16 s
  const int i16 = lane & 15, q4 = lane >> 4;
  const int v_off = (8 * (q4 >> 1) + (i16 >> 2)) * VP + 16 * (q4 & 1) + 4 * (i16 & 3);   // + (32 kt + 16 m + 4 hh) * VP + 32 dt
  constexpr int LDT = D / 32, LLOC = D % 32;
  constexpr int LR = 4 * (LLOC / 8) + (LLOC % 4), LG = (LLOC / 4) & 1;
  // q operand (B): query j, columns 16 s + 8 g; a chunk past D is read from the zeros
  const bf16_t *q_src = X + j * RP + 8 * g;
  const bf16_t *q_last = (16 * (KSTEPS - 1) + 8 * g < D) ? q_src + 16 * (KSTEPS - 1) : zeros;

  bf16x8 qn[KSTEPS];   // q operands of the tile whose scores are computed next
  auto fetch_q = [&]() {
#pragma unroll
    for (int s = 0; s < KSTEPS - 1; ++s) qn[s] = *reinterpret_cast<const bf16x8 *>(q_src + 16 * s);
    qn[KSTEPS - 1] = *reinterpret_cast<const bf16x8 *>(q_last);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // the reads of X are done before a later load may overwrite it
  };
  f32x16 S[LT];
  auto scores = [&](int kt) {
#pragma unroll
    for (int r = 0; r < 16; ++r) S[kt][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(Ks + k_off + 32 * kt * RP + 16 * s);
      S[kt] = mfma32(kf, qn[s], S[kt]);
    }
  };

  // softmax and second product of the tile in S; with MORE, the scores of the next tile replace S
  auto tile_body = [&](auto more_tag) {
    constexpr bool MORE = decltype(more_tag)::value;
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < LT; ++kt) {
      float a = fmaxf(fmaxf(S[kt][0], S[kt][1]), S[kt][2]);
      float b2 = fmaxf(fmaxf(S[kt][3], S[kt][4]), S[kt][5]);
#pragma unroll
      for (int r = 6; r < 14; r += 4) {
        a = fmaxf(fmaxf(a, S[kt][r]), S[kt][r + 1]);
        b2 = fmaxf(fmaxf(b2, S[kt][r + 2]), S[kt][r + 3]);
      }
      a = fmaxf(fmaxf(a, S[kt][14]), S[kt][15]);
      mx = fmaxf(mx, fmaxf(a, b2));
    }
    mx = max_pair(mx);
    const float mc = mx * c;

    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.0f;
#pragma unroll
    for (int kt = 0; kt < LT; ++kt) {
      bf16x8 pf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r)
        pf[r >> 3][r & 7] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(S[kt][r], c, -mc));
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const bf16_t *vp = Vs + v_off + (32 * kt + 16 * m) * VP + 32 * dt;
          const bf16x4 lo = lds_read_tr4(vp), hi = lds_read_tr4(vp + 4 * VP);
          bf16x8 vf;
          vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
          vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
          oacc[dt] = mfma32(vf, pf[m], oacc[dt]);
        }
      if (MORE) scores(kt);
    }

    // normalise and stage the tile [token][d] in Y
    const float inv = 1.0f / __shfl(oacc[LDT][LR], j + 32 * LG);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int d0 = 32 * dt + 8 * rq + 4 * g;
        if (d0 < D)
          Io<T>::store4(Y + j * RP + d0, oacc[dt][4 * rq] * inv, oacc[dt][4 * rq + 1] * inv,
                        oacc[dt][4 * rq + 2] * inv, oacc[dt][4 * rq + 3] * inv);
      }
  };

  // ---- prologue: scores of the first tile, second tile requested ----
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  fetch_q();
  if (t + stride < t_hi) stage_q(t + stride);
#pragma unroll
  for (int kt = 0; kt < LT; ++kt) scores(kt);

  int t_prev = -1;
  for (;;) {
    const bool more = t + stride < t_hi;
    // Everything still in flight (the q tile for the next iteration, the stores of the tile before
    // the previous one) was issued an iteration ago.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (t_prev >= 0) store_tile(t_prev);
    if (more) {
      fetch_q();
      if (t + 2 * stride < t_hi) stage_q(t + 2 * stride);
      tile_body(std::true_type{});
    } else {
      tile_body(std::false_type{});
    }
    t_prev = t;
    t += stride;
    if (!more) break;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  store_tile(t_prev);
}

}  // namespace pab
