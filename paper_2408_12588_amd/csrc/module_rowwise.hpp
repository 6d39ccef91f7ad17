// The row-wise parts of the attention module (paper App. B.5: "layernorm1",
// "modulate", "layernorm2", "pos emb"), the ones the paper finds slow because
// they touch every element once with almost no arithmetic: both kernels here
// are bound by HBM traffic and fuse what the paper lists as separate steps.
//
//   ln_modulate_kernel : h = LayerNorm(x) * (1 + scale) + shift over the hidden
//                        size C, one wavefront per token, the row held in
//                        registers between the two reduction passes.
//   qk_norm_rope_kernel: in place on the projected q and k, LayerNorm over the
//                        head dimension D with a learned scale and shift, then
//                        (temporal attention only) the rotary position
//                        embedding by frame index.  A few lanes per (token,
//                        head) row, so that a wavefront reads and writes one
//                        contiguous stretch of memory and a row fits in a
//                        handful of registers.
#pragma once
#include "mfma_util.hpp"

namespace pab {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

struct LnModParams {
  const bf16_t *x;       // [n_tok, C]
  const bf16_t *shift;   // [C]
  const bf16_t *scale;   // [C]
  bf16_t *h;             // [n_tok, C]
  int n_tok, C;
  float eps;
};

// NCH: 8-element chunks a lane holds (ceil(C / 512)).
template <int NCH>
__global__ __launch_bounds__(256) void ln_modulate_kernel(const LnModParams p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tok = blockIdx.x * 4 + wave;
  if (tok >= p.n_tok) return;
  const int C = p.C, nchunk = C >> 3;
  const bf16_t *xr = p.x + (long long)tok * C;
  float v[NCH][8];
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    bf16x8 t = zero8();
    if (c < nchunk) t = *reinterpret_cast<const bf16x8 *>(xr + 8 * c);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      v[i][e] = (float)t[e];
      s += v[i][e];
    }
  }
  const float mean = wave_sum(s) / (float)C;
  float ss = 0.0f;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
    if (lane + 64 * i < nchunk) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = v[i][e] - mean;
        ss += d * d;
      }
    }
  const float rstd = 1.0f / sqrtf(wave_sum(ss) / (float)C + p.eps);
  bf16_t *hr = p.h + (long long)tok * C;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nchunk) {
      const bf16x8 sh = *reinterpret_cast<const bf16x8 *>(p.shift + 8 * c);
      const bf16x8 sc = *reinterpret_cast<const bf16x8 *>(p.scale + 8 * c);
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (bf16_t)((v[i][e] - mean) * rstd * (1.0f + (float)sc[e]) + (float)sh[e]);
      *reinterpret_cast<bf16x8 *>(hr + 8 * c) = o;
    }
  }
}

struct QkNormParams {
  bf16_t *q, *k;                   // [n_tok, H, D] each, normalised in place
  const bf16_t *gq, *bq, *gk, *bk; // [D]
  int n_tok, H, S;                 // S: tokens per frame (frame index = token / S)
  int rope;                        // 1: rotate by the frame index afterwards
  float eps;
  float log2_base;                 // log2 of the rotary base
};

// LPR lanes share one (token, head) row, D / LPR consecutive elements each (a multiple of 8 and
// of 2); a wavefront covers 64 / LPR consecutive rows of q or of k (blockIdx.y picks which), i.e.
// one contiguous stretch of memory that its lanes read and write in order.  The two row sums are
// combined across the lanes of a row by lane permutes.
template <int D, int LPR>
__global__ __launch_bounds__(256) void qk_norm_rope_kernel(const QkNormParams p) {
  constexpr int EPL = D / LPR;              // elements per lane
  constexpr int CPL = EPL / 8;              // 16-byte chunks per lane
  constexpr int RPW = 64 / LPR;             // rows per wavefront
  static_assert(D % LPR == 0 && EPL % 8 == 0, "a lane holds whole chunks");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  bf16_t *base = blockIdx.y == 0 ? p.q : p.k;
  const bf16_t *gamma = blockIdx.y == 0 ? p.gq : p.gk, *beta = blockIdx.y == 0 ? p.bq : p.bk;
  const long long n_rows = (long long)p.n_tok * p.H;
  const int r_in_wave = lane / LPR, part = lane % LPR;
  const long long row = ((long long)blockIdx.x * 4 + wave) * RPW + r_in_wave;
  const bool live = r_in_wave < RPW && row < n_rows;
  bf16_t *g0 = base + row * D + part * EPL;

  float v[EPL];
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    bf16x8 t = zero8();
    if (live) t = *reinterpret_cast<const bf16x8 *>(g0 + 8 * i);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      v[8 * i + e] = (float)t[e];
      s += v[8 * i + e];
    }
  }
  const int first = lane - part;            // first lane of this row
  float tot = 0.0f;
#pragma unroll
  for (int l = 0; l < LPR; ++l) tot += __shfl(s, first + l);
  const float mean = tot / (float)D;
  float ss = 0.0f;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const float d = v[e] - mean;
    ss += d * d;
  }
  tot = 0.0f;
#pragma unroll
  for (int l = 0; l < LPR; ++l) tot += __shfl(ss, first + l);
  const float rstd = 1.0f / sqrtf(tot / (float)D + p.eps);
  if (!live) return;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const bf16x8 gm = *reinterpret_cast<const bf16x8 *>(gamma + part * EPL + 8 * i);
    const bf16x8 bt = *reinterpret_cast<const bf16x8 *>(beta + part * EPL + 8 * i);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[8 * i + e] = (v[8 * i + e] - mean) * rstd * (float)gm[e] + (float)bt[e];
  }
  if (p.rope) {
    const float pos = (float)(int)(row / p.H / p.S);   // frame index of this row's token
#pragma unroll
    for (int i = 0; i < EPL / 2; ++i) {
      const float pair = (float)(part * (EPL / 2) + i);          // index of the feature pair inside the head
      const float theta = __builtin_amdgcn_exp2f(-(2.0f * pair / (float)D) * p.log2_base);
      float sn, cs;
      sincosf(pos * theta, &sn, &cs);
      const float a = v[2 * i], b = v[2 * i + 1];
      v[2 * i] = a * cs - b * sn;
      v[2 * i + 1] = a * sn + b * cs;
    }
  }
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16_t)v[8 * i + e];
    *reinterpret_cast<bf16x8 *>(g0 + 8 * i) = o;
  }
}

}  // namespace pab
