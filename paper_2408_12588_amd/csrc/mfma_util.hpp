// Shared device helpers for the gfx950 attention kernels: vector types, the
// bf16 MFMA wrapper with its operand / accumulator lane layouts, loads that
// round to bf16 on the way in, and stores that round once on the way out.
#pragma once
#include <hip/hip_runtime.h>

namespace pab {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32], one wavefront.
//   lane l, j = l % 32, g = l / 32
//   A operand: row j of A, columns 8g .. 8g+7       (8 bf16 per lane)
//   B operand: column j of B, rows 8g .. 8g+7       (8 bf16 per lane)
//   D / C:     column j, rows 8*(r/4) + 4g + r%4    (r = 0..15, fp32)
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row permutation used for the "keys" operand of the first product: lane row i
// of A is fed key sigma(i) (bits 2 and 3 of i swapped).  With it, accumulator
// register r of lane (j, g) holds key 16*(r/8) + 8g + r%8, i.e. registers
// 8m .. 8m+7 are exactly the B operand (8 consecutive keys 16m + 8g ..) of the
// second product, so probabilities never leave registers.
__device__ __forceinline__ int sigma(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }
__device__ __forceinline__ int key_of_reg(int r, int g) { return 16 * (r >> 3) + 8 * g + (r & 7); }

template <typename T> struct Io;  // element type of q, k, v, o in memory

template <> struct Io<bf16_t> {
  static __device__ __forceinline__ bf16x8 load8(const bf16_t *p) { return *reinterpret_cast<const bf16x8 *>(p); }
  static __device__ __forceinline__ bf16x4 load4(const bf16_t *p) { return *reinterpret_cast<const bf16x4 *>(p); }
  static __device__ __forceinline__ void store4(bf16_t *p, float a, float b, float c, float d) {
    bf16x4 v;
    v[0] = (bf16_t)a; v[1] = (bf16_t)b; v[2] = (bf16_t)c; v[3] = (bf16_t)d;
    *reinterpret_cast<bf16x4 *>(p) = v;
  }
};

template <> struct Io<float> {
  static __device__ __forceinline__ bf16x8 load8(const float *p) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(p);
    const f32x4 b = *reinterpret_cast<const f32x4 *>(p + 4);
    bf16x8 v;
    v[0] = (bf16_t)a[0]; v[1] = (bf16_t)a[1]; v[2] = (bf16_t)a[2]; v[3] = (bf16_t)a[3];
    v[4] = (bf16_t)b[0]; v[5] = (bf16_t)b[1]; v[6] = (bf16_t)b[2]; v[7] = (bf16_t)b[3];
    return v;
  }
  static __device__ __forceinline__ bf16x4 load4(const float *p) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(p);
    bf16x4 v;
    v[0] = (bf16_t)a[0]; v[1] = (bf16_t)a[1]; v[2] = (bf16_t)a[2]; v[3] = (bf16_t)a[3];
    return v;
  }
  static __device__ __forceinline__ void store4(float *p, float a, float b, float c, float d) {
    f32x4 v = {a, b, c, d};
    *reinterpret_cast<f32x4 *>(p) = v;
  }
};

// v_mfma_f32_16x16x32_bf16: D[16x16] += A[16x32] * B[32x16].  lane l, i = l % 16, g = l / 16
//   A operand: row i, columns 8g .. 8g+7;  B operand: column i, rows 8g .. 8g+7;  D / C: column i, rows 4g .. 4g+3
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// v_mfma_f32_16x16x16_bf16: the same with 16 columns of A / rows of B, lane (i, g) holding 4g .. 4g+3.
__device__ __forceinline__ f32x4 mfma16_k16(bf16x4 a, bf16x4 b, f32x4 c) {
  typedef __attribute__((ext_vector_type(4))) short s16x4;
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
}

// On gfx950 a 16 x 16 x 16 MFMA that takes the result of a 16 x 16 x 32 one as its C operand (or the other way
// round) needs more wait states than hipcc 7.2 leaves between the two: with the instructions in source order
// (-mllvm -enable-misched=0) every such chain returned wrong sums, and in scheduled builds it depended on what the
// scheduler happened to put in between.  About ten wait states are enough (four on top of the compiler's passed
// every test).  Call this between the last 16 x 16 x 32 MFMA and the first 16 x 16 x 16 one on the given
// accumulators: the s_nop is tied to them by a data dependence, so no schedule can move it away.
__device__ __forceinline__ void mfma_shape_change(f32x4 &a, f32x4 &b, f32x4 &c, f32x4 &d) {
  asm volatile("s_nop 7" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16_t)0.0f;
  return z;
}

__device__ __forceinline__ bf16x8 splat8(float x) {
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16_t)x;
  return z;
}

// One wavefront-wide 16-byte-per-lane copy from global memory straight into LDS: lane i's 16 bytes
// at base + voff land at LDS byte address lds_addr + 16*i (lds_addr and base are wavefront-uniform).
// Completion is tracked by vmcnt; the compiler does not see this instruction, so the caller waits
// (s_waitcnt vmcnt) before the barrier that publishes the data.
__device__ __forceinline__ void dma16_to_lds(const void *base, unsigned voff, unsigned lds_addr) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);   // uniform by contract; tell the compiler
  // The LDS address travels in M0.  It is bound to that register as an operand, so the compiler writes M0 itself and
  // knows that this statement reads it; the s_nop is the wait state between a write of M0 and the instruction using it.
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(base), "{m0}"(lds_addr)
               : "memory");
}

__device__ __forceinline__ bf16x4 lds_read_tr4(const bf16_t *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3))) *)(p));
}

// max over lanes j and j+32 (the two lanes that share a query), result in both
__device__ __forceinline__ float max_pair(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

// A 16-byte LDS read is served in four cycles of 16 lanes, and the lanes of a cycle are not
// consecutive: lanes {0-3, 12-15, 20-23, 24-27} go together, then {4-7, 8-11, 16-19, 28-31}, and
// the same in the upper half (measured with the bank conflict counter, two lane quads at a time).
// With 16 x 16 x 32 operands, lane (l16, g4) reads chunk 4 ks + g4 of K row l16, so a cycle mixes chunk g4
// of rows 0-3 and 12-15 with chunk g4 + 1 of rows 4-11 (or the other way round), which collide in
// a plain row-major tile.  Storing chunk c of tile row r at position c ^ k_swizzle(r) of that row
// makes every cycle hit all 64 banks once (checked by enumeration for both row lengths).  The
// staging lanes apply the same exchange to the global address they fetch, so rows stay contiguous.
template <int D> __device__ __forceinline__ int k_swizzle(int row) {
  static_assert(D == 72 || D == 32, "swizzle derived for 9 and 4 chunks per row");
  return D == 72 ? ((row >> 2) ^ (row >> 3)) & 1 : ((row >> 3) & 1) << 1;
}

// Head-dim dependent tile constants.
template <int D> struct HeadDim {
  static_assert(D % 8 == 0, "head dim must be a multiple of 8");
  static constexpr int DK = (D + 15) / 16 * 16;       // contraction length of q.k, zero padded
  static constexpr int KSTEPS = DK / 16;              // MFMA steps of the first product
  static constexpr int DV = (D + 1 + 31) / 32 * 32;   // output rows incl. the all-ones row at index D
  static constexpr int DT = DV / 32;                  // 32-row output tiles
  static constexpr int CH = D / 8;                    // 8-element chunks per head row
  static constexpr int DKP = DK + 8;                  // LDS row pitch (elements) of row-major tiles
};

}  // namespace pab
