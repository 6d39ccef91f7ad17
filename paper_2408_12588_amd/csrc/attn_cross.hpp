// Cross attention (paper Sec. 2.1): every video token attends to the L text
// tokens of the conditioning input.  L is short (<= 128 here), so per head the
// keys and values fit in LDS once and for all, the softmax needs a single pass,
// and the operation is bound by streaming q in and o out of HBM.
//
// One workgroup = NW wavefronts serves one head: it stages that head's K and V
// rows ([L, D], row-major as in memory) into LDS once, then each wavefront walks
// over 32-query tiles of the head with a stride of all wavefronts serving it.
// The wavefronts never synchronise with each other after the K/V load.
//
// Per tile a wavefront
//   - has the tile's 32 q rows copied global -> LDS by direct loads that were
//     issued two tiles ahead (three per-wavefront buffers), 16 bytes per lane
//     with consecutive lanes on consecutive chunks of a row.  Two tiles, not
//     one: loads and stores share one in-order-per-kind counter, and with two
//     tiles of loads behind it a tile can be waited for without also waiting
//     for the stores of the tile before it;
//   - computes S^T = K Q^T for all keys (bf16 MFMA, keys x queries, so the
//     softmax statistics are per-lane scalars), one max, P^T = exp2(c(S^T - m))
//     in registers, O^T = V^T P^T with V^T read transposed from LDS; V rows in
//     LDS carry an extra chunk {1, 0, ..}, so row D of O^T is the softmax
//     denominator, accumulated on the matrix core;
//   - writes the normalised tile into the LDS buffer its q rows came from and
//     from there to global memory, again whole rows per instruction.
#pragma once
#include "mfma_util.hpp"

namespace pab {

struct CrossParams {
  const void *q, *k, *v;
  void *o;
  int n_tok, L, n_head;
  int wg_per_head;     // workgroups that share one head
  float c;             // log2(e) / sqrt(D)
};

// LT: 32-key tiles that hold L (1..4).  NW: wavefronts per workgroup.  NB: q/o tile buffers per
// wavefront (2 or 3); q tiles are requested NB-1 tiles ahead.
template <int D, int LT, int NW, int NB>
__global__ __launch_bounds__(64 * NW) void attn_cross_kernel(const CrossParams p) {
  using HD = HeadDim<D>;
  using T = bf16_t;
  constexpr int KSTEPS = HD::KSTEPS, DT = HD::DT, CH = HD::CH;
  constexpr int LP = 32 * LT;               // key rows held in LDS (rows past L repeat row L-1, masked)
  constexpr int RP = D;                     // row pitch: rows packed as in memory
  constexpr int VCH = CH + 1, VP = 8 * VCH; // V rows in LDS: CH data chunks, then the constant chunk {1, 0, ..}
  constexpr int K_ELEMS = LP * RP, V_ELEMS = LP * VP, KV_ELEMS = K_ELEMS + V_ELEMS;
  constexpr int QB_ELEMS = 32 * RP;         // one q / o tile buffer
  constexpr int KR = (LP * CH + 63) / 64;   // staging rounds (64 chunk slots) for K
  constexpr int VR = (LP * VCH + 63) / 64;  // ... for V (the slots of the constant chunks stay idle)
  constexpr int QR = (32 * CH + 63) / 64;   // staging rounds for a q tile (the last may be partial)
  constexpr int SLACK = 64;
  static_assert(LT >= 1 && LT <= 4, "keys must fit four 32-key tiles");
  static_assert((NB == 2 || NB == 3) && 2 * QR < 16, "buffers / vmcnt immediate");

  __shared__ __attribute__((aligned(16))) bf16_t smem[KV_ELEMS + NW * NB * QB_ELEMS + SLACK];
  bf16_t *Ks = smem, *Vs = smem + K_ELEMS;

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
  bf16_t *qbuf = smem + KV_ELEMS + wave * (NB * QB_ELEMS);

  // ---- K and V of the head, rounds dealt round-robin to the wavefronts ----
  for (int r = wave; r < KR + VR; r += NW) {
    const bool is_k = r < KR;
    const int c = (is_k ? r : r - KR) * 64 + lane, per = is_k ? CH : VCH;
    if (c < LP * per && c % per < CH) {
      int key = c / per;
      key = key < L ? key : L - 1;
      dma16_to_lds(is_k ? kh : vh, (unsigned)(2 * (key * row + 8 * (c % per))),
                   smem_addr + 2 * (is_k ? 512 * r : K_ELEMS + 512 * (r - KR)));
    }
  }
  for (int idx = tid; idx < LP; idx += 64 * NW) {   // constant chunk of every V row
    bf16x8 one = zero8();
    one[0] = (bf16_t)1.0f;
    *reinterpret_cast<bf16x8 *>(Vs + idx * VP + D) = one;
  }
  if (tid < SLACK / 2) reinterpret_cast<unsigned *>(smem + KV_ELEMS + NB * NW * QB_ELEMS)[tid] = 0u;

  // ---- q tile t -> this wavefront's buffer `b`: QR direct loads, rows past the end repeat the last.
  //      Token offsets can exceed 32 bits: the base moves with the tile, the lane offset stays small. ----
  auto stage_q = [&](int t, int b) {
    const int tok0 = 32 * t;
    const T *base = qh + (long long)tok0 * row;
#pragma unroll
    for (int r = 0; r < QR; ++r) {
      const int c = r * 64 + lane;
      if (c < 32 * CH) {
        int tr = c / CH;
        tr = tok0 + tr < n_tok ? tr : n_tok - 1 - tok0;
        dma16_to_lds(base, (unsigned)(2 * (tr * row + 8 * (c % CH))), smem_addr + 2 * (int)(qbuf - smem) + 2 * b * QB_ELEMS + 1024 * r);
      }
    }
  };

  constexpr int PD = NB - 1;   // prefetch distance in tiles
  int t = t_lo + part * NW + wave;
#pragma unroll
  for (int d = 0; d < PD; ++d)
    if (t + d * stride < t_hi) stage_q(t + d * stride, d);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // K, V (this wavefront's share) and the first q tiles have landed
  __syncthreads();                      // ... everyone's share of K and V

  const float c = p.c;
  const int k_off = sigma(j) * RP + 8 * g;                                             // + 32 kt * RP + 16 s
  const int i16 = lane & 15, q4 = lane >> 4;
  const int v_off = (8 * (q4 >> 1) + (i16 >> 2)) * VP + 16 * (q4 & 1) + 4 * (i16 & 3);   // + (32 kt + 16 m + 4 hh) * VP + 32 dt
  constexpr int LDT = D / 32, LLOC = D % 32;
  constexpr int LR = 4 * (LLOC / 8) + (LLOC % 4), LG = (LLOC / 4) & 1;

  int cur = 0;   // ring position of tile t's buffer
  for (; t < t_hi; t += stride, cur = cur == NB - 1 ? 0 : cur + 1) {
    bf16_t *qb = qbuf + cur * QB_ELEMS;
    // Request the tile PD tiles ahead into the buffer the previous tile was written out from, then
    // wait for tile t.  Loads complete in order among themselves (so do stores, but not against
    // loads): tile t's loads are followed by those of the `later` tiles already requested, so once at
    // most later*QR operations are in flight tile t has landed, whatever earlier stores are doing.
    if (t + PD * stride < t_hi) stage_q(t + PD * stride, cur == 0 ? NB - 1 : cur - 1);
    const int left = (t_hi - 1 - t) / stride;
    const int later = left < PD ? left : PD;
    if (later >= 2) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * QR));
    else if (later == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | QR);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- q fragments (B operand): query j, columns 16 s + 8 g; columns past D are zero ----
    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
      qf[s] = *reinterpret_cast<const bf16x8 *>(qb + j * RP + 16 * s + 8 * g);
      if (16 * s + 8 >= D) qf[s] = (16 * s + 8 * g < D) ? qf[s] : zero8();
    }

    // ---- S^T = K Q^T over all keys ----
    f32x16 S[LT];
#pragma unroll
    for (int kt = 0; kt < LT; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) S[kt][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(Ks + k_off + 32 * kt * RP + 16 * s);
        S[kt] = mfma32(kf, qf[s], S[kt]);
      }
    }
    // keys past L take no probability mass (only the last tile can hold any)
    if ((L & 31) != 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (32 * (LT - 1) + key_of_reg(r, g) >= L) S[LT - 1][r] = -INFINITY;
    }

    // ---- single-pass softmax of lane j's query ----
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
    mx = max_pair(mx);   // key 0 is always valid, so mx is finite
    const float mc = mx * c;

    // ---- O^T = V^T P^T, tile by tile of keys ----
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
    }

    // ---- normalise, stage the tile [token][d] in the buffer its q rows came from, write whole rows ----
    const float inv = 1.0f / __shfl(oacc[LDT][LR], j + 32 * LG);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // all q fragment reads are done
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int d0 = 32 * dt + 8 * rq + 4 * g;
        if (d0 < D)
          Io<T>::store4(qb + j * RP + d0, oacc[dt][4 * rq] * inv, oacc[dt][4 * rq + 1] * inv,
                        oacc[dt][4 * rq + 2] * inv, oacc[dt][4 * rq + 3] * inv);
      }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    T *ot = oh + (long long)(32 * t) * row;
#pragma unroll
    for (int r = 0; r < QR; ++r) {
      const int cidx = r * 64 + lane;
      const int tr = cidx / CH, cc = cidx % CH;
      if (cidx < 32 * CH && 32 * t + tr < n_tok)
        *reinterpret_cast<bf16x8 *>(ot + tr * row + 8 * cc) = *reinterpret_cast<const bf16x8 *>(qb + tr * RP + 8 * cc);
    }
  }
}

}  // namespace pab
