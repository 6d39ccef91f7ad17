// Temporal attention (paper Sec. 2.1): for every spatial position and head, the
// T frames attend to each other.  Sequences are tiny (T <= 32) and the batch is
// huge (S * H problems), so the op is bound by HBM traffic, not by arithmetic.
//
// One wavefront owns one (position, head) problem at a time and never talks to
// the other wavefronts of its workgroup (no workgroup barrier anywhere).  The
// activations stay in their [T, S, H, D] layout: frame t of a problem is the
// D-element row at t * (S*H*D) + (position*H + head) * D, so a problem is T
// rows far apart in memory; each is read with consecutive lanes on consecutive
// 16-byte chunks, staged in the wavefront's own LDS region, and turned into
// MFMA operands there.  The whole T x T score tile lives in one 32x32
// accumulator; the softmax is single pass.  Outputs go back through LDS so
// that every global store again covers whole rows.
#pragma once
#include "mfma_util.hpp"

namespace pab {

struct TemporalParams {
  const void *q, *k, *v;
  void *o;
  int T;              // frames = sequence length, 1..32
  int n_head;
  int n_prob;         // S * H problems
  long long ss;       // sequence (frame) stride in elements = S*H*D
  float c;            // log2(e) / sqrt(D)
};

// TP: 16 or 32, the power-of-two tile edge that holds T.  RT: rows of LDS staging per tensor
// (T <= RT <= TP); fewer rows let more workgroups share a CU.  QDIRECT: the q operands are loaded
// from global memory in MFMA operand layout instead of being staged in LDS like k and v.
template <typename T_, int D, int TP, int RT, bool QDIRECT>
__global__ __launch_bounds__(256) void attn_temporal_kernel(const TemporalParams p) {
  using HD = HeadDim<D>;
  constexpr int DK = HD::DK, KSTEPS = HD::KSTEPS, DT = HD::DT, CH = HD::CH, DKP = HD::DKP;
  constexpr int CHZ = DK / 8;             // chunks per staged row incl. the zero padding chunk(s)
  constexpr int NR = TP / 2;              // live accumulator registers (keys 16..31 unused when TP == 16)
  constexpr int NM = TP / 16;             // 16-key steps of the second product
  constexpr int OP = D + 8;               // pitch of the output staging rows (elements of T_)
  constexpr int QK_BYTES = (QDIRECT ? 1 : 2) * RT * DKP * 2;   // k (and q) staging
  constexpr int O_BYTES = RT * OP * (int)sizeof(T_);
  constexpr int A_BYTES = QK_BYTES > O_BYTES ? QK_BYTES : O_BYTES;   // q/k staging, reused for o
  constexpr int VP = 96;                  // pitch of the V rows: 48 banks, so that the four rows of a transposed read do not meet
  static_assert(D + 8 <= VP, "head dim too long for the V row pitch");
  constexpr int V_BYTES = RT * VP * 2;
  constexpr int WAVE_BYTES = A_BYTES + V_BYTES;

  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * WAVE_BYTES];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 31, g = lane >> 5;
  unsigned char *base = smem + wave * WAVE_BYTES;
  bf16_t *Qs = reinterpret_cast<bf16_t *>(base);                   // [RT][DKP] (unused with QDIRECT)
  bf16_t *Ks = QDIRECT ? Qs : Qs + RT * DKP;                       // [RT][DKP]
  T_ *Os = reinterpret_cast<T_ *>(base);                           // [RT][OP], aliases Qs/Ks
  bf16_t *Vs = reinterpret_cast<bf16_t *>(base + A_BYTES);         // [RT][VP], rows >= T stay zero; column D is 1

  const int T = p.T;
  const float c = p.c;

  // value rows of frames that do not exist must be finite: zero the tile once
  // and column D of every row is 1, so that row D of V^T sums the probabilities (the softmax denominator)
  for (int idx = lane; idx < RT * VP / 8; idx += 64) {
    bf16x8 fill = zero8();
    if (idx % (VP / 8) == D / 8) fill[D % 8] = (bf16_t)1.0f;
    reinterpret_cast<bf16x8 *>(Vs)[idx] = fill;
  }

  // Workgroup ids go round-robin over the 8 XCDs.  Give every XCD a contiguous run of problems:
  // four neighbouring heads are 4.5 cache lines, so neighbouring workgroups share a line, and this
  // way they find it in the same L2.  (The host launches a multiple of 8 workgroups.)
  const int wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  const int waves_total = gridDim.x * 4;
  for (int prob = wg * 4 + wave; prob < p.n_prob; prob += waves_total) {
    const long long off = (long long)prob * D;   // (position*H + head) * D
    const T_ *qg = reinterpret_cast<const T_ *>(p.q) + off;
    const T_ *kg = reinterpret_cast<const T_ *>(p.k) + off;
    const T_ *vg = reinterpret_cast<const T_ *>(p.v) + off;
    T_ *og = reinterpret_cast<T_ *>(p.o) + off;

    // ---- global -> registers -> LDS, whole rows per instruction; the padding chunk of q and k
    //      rows is written as zeros.  All loads are issued before the first LDS store. ----
    constexpr int NLD = (RT * CHZ + 63) / 64;
    bf16x8 q8[NLD], k8[NLD], v8[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int cidx = lane + 64 * i, t = cidx / CHZ, cc = cidx % CHZ;
      q8[i] = zero8(); k8[i] = zero8(); v8[i] = zero8();
      if (cidx < T * CHZ && cc < CH) {
        if (!QDIRECT) q8[i] = Io<T_>::load8(qg + t * p.ss + 8 * cc);
        k8[i] = Io<T_>::load8(kg + t * p.ss + 8 * cc);
        v8[i] = Io<T_>::load8(vg + t * p.ss + 8 * cc);
      }
    }
    // with QDIRECT the q operands (B: query j = frame j, columns 16 st + 8 g) come straight from memory
    bf16x8 qd[KSTEPS];
    if (QDIRECT) {
      const T_ *qrow_p = qg + (long long)min(j & (TP - 1), T - 1) * p.ss;
#pragma unroll
      for (int st = 0; st < KSTEPS; ++st) qd[st] = (16 * st + 8 * g < D) ? Io<T_>::load8(qrow_p + 16 * st + 8 * g) : zero8();
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // previous problem's reads of Os are done
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int cidx = lane + 64 * i, t = cidx / CHZ, cc = cidx % CHZ;
      if (cidx < T * CHZ) {
        if (!QDIRECT) *reinterpret_cast<bf16x8 *>(&Qs[t * DKP + 8 * cc]) = q8[i];
        *reinterpret_cast<bf16x8 *>(&Ks[t * DKP + 8 * cc]) = k8[i];
        if (cc < CH) *reinterpret_cast<bf16x8 *>(&Vs[t * VP + 8 * cc]) = v8[i];
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    // ---- S^T = K Q^T (rows: keys permuted by sigma, columns: queries) ----
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.0f;
    // rows past the staging area alias a staged row: such keys are masked, such queries never stored
    const int krow = min(sigma(j) & (TP - 1), RT - 1), qrow = min(j & (TP - 1), RT - 1);
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&Ks[krow * DKP + 16 * st + 8 * g]);
      const bf16x8 qf = QDIRECT ? qd[st] : *reinterpret_cast<const bf16x8 *>(&Qs[qrow * DKP + 16 * st + 8 * g]);
      s = mfma32(kf, qf, s);
    }

    // ---- single-pass softmax over the keys of lane j's query ----
    float mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      if (key_of_reg(r, g) >= T) s[r] = -INFINITY;
      mx = fmaxf(mx, s[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));   // T >= 1: key 0 is valid, so mx is finite for valid queries
    const float mc = mx * c;
    bf16x8 pf[NM];
#pragma unroll
    for (int r = 0; r < NR; ++r)
      pf[r >> 3][r & 7] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -mc));

    // ---- O^T = V^T P^T; the A operand is gathered column-wise from the row-major tile ----
    f32x16 o[DT];
    // Two transposed 8-byte reads give lane (j, g) row 32 dt + j of V^T over keys 16 m + 8 g .. + 7: within 16
    // lanes, lane i receives element i of the rows that lanes 4 e .. 4 e + 3 address (e = 0 .. 3).  Rows past the
    // staging area alias its last row: such keys weigh 0.
    const int i16 = lane & 15, q4 = lane >> 4;
    const int vcol = 16 * (q4 & 1) + 4 * (i16 & 3);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const int row = 16 * m + 8 * (q4 >> 1) + (i16 >> 2);
        const bf16x4 lo = lds_read_tr4(Vs + min(row, RT - 1) * VP + vcol + 32 * dt);
        const bf16x4 hi = lds_read_tr4(Vs + min(row + 4, RT - 1) * VP + vcol + 32 * dt);
        bf16x8 vf;
        vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
        vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
        o[dt] = mfma32(vf, pf[m], o[dt]);
      }
    }

    // ---- normalise, stage [t][d] in LDS, write whole rows ----
    constexpr int LDT = D / 32, LLOC = D % 32;
    constexpr int LR = 4 * (LLOC / 8) + (LLOC % 4), LG = (LLOC / 4) & 1;
    const float inv = 1.0f / __shfl(o[LDT][LR], j + 32 * LG);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // Qs / Ks are dead from here on
    if (j < RT) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int d0 = 32 * dt + 8 * rq + 4 * g;
          if (d0 < D)
            Io<T_>::store4(&Os[j * OP + d0], o[dt][4 * rq] * inv, o[dt][4 * rq + 1] * inv,
                           o[dt][4 * rq + 2] * inv, o[dt][4 * rq + 3] * inv);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    for (int cidx = lane; cidx < T * CH; cidx += 64) {
      const int t = cidx / CH, cc = cidx % CH;
      const T_ *src = &Os[t * OP + 8 * cc];
      T_ *dst = og + t * p.ss + 8 * cc;
      if (sizeof(T_) == 2) {
        *reinterpret_cast<bf16x8 *>(dst) = *reinterpret_cast<const bf16x8 *>(src);
      } else {
        *reinterpret_cast<f32x4 *>(dst) = *reinterpret_cast<const f32x4 *>(src);
        *reinterpret_cast<f32x4 *>(dst + 4) = *reinterpret_cast<const f32x4 *>(src + 4);
      }
    }
  }
}

}  // namespace pab
