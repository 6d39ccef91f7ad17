// libpab: C-ABI entry points (declared in include/pab.h), the host-side
// broadcast schedule and cache bookkeeping, and the kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <mutex>
#include <vector>

#include "../../include/pab.h"
#include "attn_cross.hpp"
#include "attn_cross_long.hpp"
#include "attn_temporal.hpp"
#include "attn_tile16.hpp"
#include "gemm_bias.hpp"
#include "module_rowwise.hpp"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

bool kind_ok(int kind) { return kind == PAB_SPATIAL || kind == PAB_TEMPORAL || kind == PAB_CROSS; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t elem_size(int dtype) { return dtype == PAB_BF16 ? 2 : 4; }

// ---- launches -----------------------------------------------------------------

constexpr int TILE_NWV = 8;    // wavefronts per workgroup: 256 queries share each staged K/V tile (4: 1.5-2% slower)
constexpr int TILE_MINW = 4;   // wavefronts per SIMD the register budget is sized for
constexpr int TILE_SPLIT_G = 4;   // key groups of a split item
constexpr int TILE_SLOTS = 512;   // workgroups the chip holds at once: 2 per CU (16 wavefronts) x 256 CUs

template <typename T, int D>
int launch_tile(int n_batch, int n_head, int sq, int sk, long long q_bs, long long q_ss, long long kv_bs,
                long long kv_ss, const void *q, const void *k, const void *v, void *o, hipStream_t st) {
  pab::TileParams p;
  p.q = q; p.k = k; p.v = v; p.o = o;
  p.n_batch = n_batch; p.n_head = n_head; p.sq = sq; p.sk = sk;
  p.q_bs = q_bs; p.q_ss = q_ss; p.k_bs = kv_bs; p.k_ss = kv_ss; p.v_bs = kv_bs; p.v_ss = kv_ss;
  p.o_bs = q_bs; p.o_ss = q_ss;
  p.c = (float)(1.4426950408889634 / std::sqrt((double)D));
  constexpr int QBLK = 32 * TILE_NWV;
  p.n_item = (sq + QBLK - 1) / QBLK;
  // staging addresses the key tiles of one step with 32-bit byte offsets
  if (32 * TILE_SPLIT_G * kv_ss * (long long)sizeof(T) >= (1LL << 32)) return fail(PAB_EINVAL, "sequence stride too large");
  const long long n_bh = (long long)n_batch * n_head;
  if (n_bh > 0x3fffffffLL) return fail(PAB_EINVAL, "problem too large for one launch");
  // Workgroups all take about the same time, so a launch runs in rounds of TILE_SLOTS.  When the last round
  // would be at most a quarter full, the (batch, head) problems it would hold are done as split items
  // instead (a quarter of the queries, four key groups each): four times the workgroups, a quarter of the steps.
  p.bh_plain = (int)n_bh;
  p.n_split = 0;
  p.split_g = TILE_SPLIT_G;
  const long long total = n_bh * p.n_item, rest = total % TILE_SLOTS;
  const int ntile = (sk + 31) / 32;
  if (total > TILE_SLOTS && rest >= p.n_item && rest * 4 <= TILE_SLOTS && ntile >= 4 * TILE_SPLIT_G) {
    p.bh_plain = (int)(n_bh - rest / p.n_item);
    p.n_split = (sq + QBLK / TILE_SPLIT_G - 1) / (QBLK / TILE_SPLIT_G);
  }
  const long long plain_wgs = (long long)(p.bh_plain + 7) / 8 * 8 * p.n_item;
  const long long grid = plain_wgs + (n_bh - p.bh_plain + 7) / 8 * 8 * p.n_split;
  if (grid > 0x7fffffffLL) return fail(PAB_EINVAL, "problem too large for one launch (%lld workgroups)", grid);
  p.plain_wgs = (int)plain_wgs;
  constexpr bool DIRECT = sizeof(T) == 2;   // bf16 rows go from global memory straight into LDS
  hipLaunchKernelGGL((pab::attn_tile16_kernel<T, D, TILE_NWV, TILE_MINW, DIRECT>), dim3((unsigned)grid),
                     dim3(64 * TILE_NWV), 0, st, p);
  return PAB_OK;
}

template <typename T, int D>
int launch_temporal(int T_, int S, int H, const void *q, const void *k, const void *v, void *o, hipStream_t st) {
  const long long row = (long long)H * D;
  if (T_ > 32) {
    // long clips: frames become the sequence of the tiled kernel, positions its batch
    return launch_tile<T, D>(S, H, T_, T_, row, (long long)S * row, row, (long long)S * row, q, k, v, o, st);
  }
  pab::TemporalParams p;
  p.q = q; p.k = k; p.v = v; p.o = o;
  p.T = T_; p.n_head = H;
  const long long n_prob = (long long)S * H;
  if (n_prob > 0x7fffffffLL) return fail(PAB_EINVAL, "too many temporal problems");
  p.n_prob = (int)n_prob;
  p.ss = (long long)S * row;
  p.c = (float)(1.4426950408889634 / std::sqrt((double)D));
  long long grid = (n_prob + 3) / 4;
  // one problem per wavefront measured faster than fewer workgroups that loop; the kernel still
  // loops, so any grid is correct
  grid = (grid + 7) / 8 * 8;      // the kernel deals whole eighths of the grid to the XCDs
  // Clips of more than 16 frames read their q operands straight from memory: the smaller LDS footprint
  // lets four (24 staged rows) or three (32) workgroups share a CU; at 16 rows staging q measured faster.
  if (T_ <= 16)
    hipLaunchKernelGGL((pab::attn_temporal_kernel<T, D, 16, 16, false>), dim3((unsigned)grid), dim3(256), 0, st, p);
  else if (T_ <= 24)
    hipLaunchKernelGGL((pab::attn_temporal_kernel<T, D, 32, 24, true>), dim3((unsigned)grid), dim3(256), 0, st, p);
  else
    hipLaunchKernelGGL((pab::attn_temporal_kernel<T, D, 32, 32, true>), dim3((unsigned)grid), dim3(256), 0, st, p);
  return PAB_OK;
}

// Cross attention with few keys and bf16 rows: K and V stay in LDS, q and o stream.
constexpr int CROSS_NW = 4;    // wavefronts per workgroup

template <int D>
int launch_cross(int n_tok, int L, int H, const void *q, const void *k, const void *v, void *o, hipStream_t st) {
  pab::CrossParams p;
  p.q = q; p.k = k; p.v = v; p.o = o;
  p.n_tok = n_tok; p.L = L; p.n_head = H;
  p.c = (float)(1.4426950408889634 / std::sqrt((double)D));
  const int ntile = (n_tok + 31) / 32;
  // about two workgroups per CU in total; a multiple of 8 per head lets every XCD take its own
  // eighth of the tokens; never more wavefronts than tiles
  int per_head = (512 / H + 7) / 8 * 8;
  if (ntile < per_head * CROSS_NW) per_head = (ntile + CROSS_NW - 1) / CROSS_NW;
  if (per_head < 1) per_head = 1;
  p.wg_per_head = per_head;
  const dim3 grid((unsigned)(H * per_head)), block(64 * CROSS_NW);
  switch ((L + 31) / 32) {
    case 1: hipLaunchKernelGGL((pab::attn_cross_kernel<D, 1, CROSS_NW>), grid, block, 0, st, p); break;
    case 2: hipLaunchKernelGGL((pab::attn_cross_kernel<D, 2, CROSS_NW>), grid, block, 0, st, p); break;
    case 3: hipLaunchKernelGGL((pab::attn_cross_kernel<D, 3, CROSS_NW>), grid, block, 0, st, p); break;
    default: hipLaunchKernelGGL((pab::attn_cross_kernel<D, 4, CROSS_NW>), grid, block, 0, st, p); break;
  }
  return PAB_OK;
}

// Cross attention with up to 512 keys and bf16 rows: K and V of a head still fit in LDS, the
// online softmax runs over its key tiles.  One workgroup per CU.
constexpr int CROSSL_NW = 16;   // wavefronts per workgroup
constexpr int CROSSL_MINW = 4;  // ... per SIMD
constexpr int CROSSL_MAX_L = 512;

template <int D>
int launch_cross_long(int n_tok, int L, int H, const void *q, const void *k, const void *v, void *o, hipStream_t st) {
  pab::CrossLongParams p;
  p.q = q; p.k = k; p.v = v; p.o = o;
  p.n_tok = n_tok; p.L = L; p.n_head = H;
  p.c = (float)(1.4426950408889634 / std::sqrt((double)D));
  const int ntile = (n_tok + 31) / 32;
  int per_head = (256 / H + 7) / 8 * 8;
  if (ntile < per_head * CROSSL_NW) per_head = (ntile + CROSSL_NW - 1) / CROSSL_NW;
  if (per_head < 1) per_head = 1;
  p.wg_per_head = per_head;
  const dim3 grid((unsigned)(H * per_head)), block(64 * CROSSL_NW);
  const int lt = (L + 31) / 32;
  if (lt <= 6) hipLaunchKernelGGL((pab::attn_cross_long_kernel<D, 6, CROSSL_NW, CROSSL_MINW>), grid, block, 0, st, p);
  else if (lt <= 8) hipLaunchKernelGGL((pab::attn_cross_long_kernel<D, 8, CROSSL_NW, CROSSL_MINW>), grid, block, 0, st, p);
  else if (lt <= 10) hipLaunchKernelGGL((pab::attn_cross_long_kernel<D, 10, CROSSL_NW, CROSSL_MINW>), grid, block, 0, st, p);
  else hipLaunchKernelGGL((pab::attn_cross_long_kernel<D, 16, CROSSL_NW, CROSSL_MINW>), grid, block, 0, st, p);
  return PAB_OK;
}

template <typename T, int D>
int launch_kind(int kind, int T_, int S, int L, int H, const void *q, const void *k, const void *v, void *o,
                hipStream_t st) {
  const long long row = (long long)H * D;
  switch (kind) {
    case PAB_SPATIAL:   // batch = frames, sequence = tokens of the frame
      return launch_tile<T, D>(T_, H, S, S, (long long)S * row, row, (long long)S * row, row, q, k, v, o, st);
    case PAB_TEMPORAL:  // batch = positions, sequence = frames
      return launch_temporal<T, D>(T_, S, H, q, k, v, o, st);
    default: {          // cross: every video token against the L text tokens
      const long long tok = (long long)T_ * S;
      if (tok > 0x7fffffffLL) return fail(PAB_EINVAL, "too many tokens");
      if (sizeof(T) == 2 && L <= 128 && H <= 512) return launch_cross<D>((int)tok, L, H, q, k, v, o, st);
      if (sizeof(T) == 2 && L <= CROSSL_MAX_L && H <= 512) return launch_cross_long<D>((int)tok, L, H, q, k, v, o, st);
      return launch_tile<T, D>(1, H, (int)tok, L, 0, row, 0, row, q, k, v, o, st);
    }
  }
}

int check_shape(int kind, int dtype, int T_, int S, int L, int H, int D) {
  if (!kind_ok(kind)) return fail(PAB_EINVAL, "kind %d is not spatial(0)/temporal(1)/cross(2)", kind);
  if (dtype != PAB_BF16 && dtype != PAB_F32) return fail(PAB_EINVAL, "dtype %d is not bf16(0)/f32(1)", dtype);
  if (D != 32 && D != 72) return fail(PAB_EINVAL, "head_dim %d unsupported (32 or 72)", D);
  if (T_ < 1 || S < 1 || H < 1) return fail(PAB_EINVAL, "T=%d S=%d heads=%d must all be >= 1", T_, S, H);
  if (kind == PAB_CROSS && L < 1) return fail(PAB_EINVAL, "cross attention needs L >= 1 text tokens (L=%d)", L);
  if ((long long)T_ * S * H * D > (1LL << 40)) return fail(PAB_EINVAL, "tensor too large");
  return PAB_OK;
}

int launch_checked(int kind, int dtype, int T_, int S, int L, int H, int D, const void *q, const void *k,
                   const void *v, void *o, hipStream_t st) {
  int rc;
  if (dtype == PAB_BF16)
    rc = (D == 72) ? launch_kind<pab::bf16_t, 72>(kind, T_, S, L, H, q, k, v, o, st)
                   : launch_kind<pab::bf16_t, 32>(kind, T_, S, L, H, q, k, v, o, st);
  else
    rc = (D == 72) ? launch_kind<float, 72>(kind, T_, S, L, H, q, k, v, o, st)
                   : launch_kind<float, 32>(kind, T_, S, L, H, q, k, v, o, st);
  if (rc != PAB_OK) return rc;
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PAB_EDEVICE, "kernel launch failed: %s", hipGetErrorString(e));
  return PAB_OK;
}

size_t slot_bytes_of(const pab_config &c) {
  const size_t raw = (size_t)c.T * c.S * c.heads * c.head_dim * elem_size(c.dtype);
  return (raw + 255) / 256 * 256;
}

int check_config(const pab_config *c) {
  if (!c) return fail(PAB_EINVAL, "config is NULL");
  if (c->n_blocks < 1) return fail(PAB_EINVAL, "n_blocks=%d must be >= 1", c->n_blocks);
  if (c->n_steps < 1) return fail(PAB_EINVAL, "n_steps=%d must be >= 1", c->n_steps);
  int present = 0;
  for (int k = 0; k < 3; ++k) {
    if (c->interval[k] < 0) return fail(PAB_EINVAL, "interval[%d]=%d must be >= 0", k, c->interval[k]);
    present += c->interval[k] > 0;
  }
  if (!present) return fail(PAB_EINVAL, "no attention kind present (all intervals 0)");
  if (c->range_lo < 0 || c->range_lo > c->range_hi)
    return fail(PAB_EINVAL, "window [%d, %d] must satisfy 0 <= lo <= hi", c->range_lo, c->range_hi);
  if (c->block_kinds)
    for (int b = 0; b < c->n_blocks; ++b) {
      if (c->block_kinds[b] > 7) return fail(PAB_EINVAL, "block_kinds[%d]=%d has bits beyond the three kinds", b, c->block_kinds[b]);
      for (int k = 0; k < 3; ++k)
        if (((c->block_kinds[b] >> k) & 1) && c->interval[k] == 0)
          return fail(PAB_EINVAL, "block_kinds[%d] names kind %d, which has interval 0", b, k);
    }
  const int kind_for_shape = c->interval[PAB_CROSS] > 0 ? PAB_CROSS : PAB_SPATIAL;
  return check_shape(kind_for_shape, c->dtype, c->T, c->S, c->L, c->heads, c->head_dim);
}

// kinds that block b has: the caller's mask, else every kind with a broadcast range
unsigned kinds_of_block(const pab_config &c, int b) {
  if (c.block_kinds) return c.block_kinds[b];
  unsigned m = 0;
  for (int k = 0; k < 3; ++k) m |= (unsigned)(c.interval[k] > 0) << k;
  return m;
}

}  // namespace

struct pab_ctx {
  pab_config cfg;        // block_kinds is NULL here: the mask is copied into slot_index
  unsigned char *workspace;
  size_t slot_bytes;
  std::vector<long long> slot_index;   // per (block, kind): slot number in the slab (block-major, kind-minor), -1 if absent
  std::vector<int> last_step;      // per (block, kind): last step seen since reset, -1 if none
  std::vector<int> computed_step;  // per (block, kind): step whose output the slot holds, -1 if none
  long long launches;
};

namespace {

// ---- what the two cached entry points share: validate the cell, take the decision of Eq. 1,
//      find the slot; after a successful launch (or on reuse) record the step ----
int schedule_cell(pab_ctx *ctx, int block, int kind, int step, void **slot) {
  const pab_config &c = ctx->cfg;
  if (!kind_ok(kind)) return fail(PAB_EINVAL, "kind %d is not spatial(0)/temporal(1)/cross(2)", kind);
  if (c.interval[kind] == 0) return fail(PAB_EINVAL, "kind %d is absent from this config (interval 0)", kind);
  if (block < 0 || block >= c.n_blocks) return fail(PAB_EINVAL, "block %d outside [0, %d)", block, c.n_blocks);
  if (ctx->slot_index[(size_t)block * 3 + kind] < 0)
    return fail(PAB_EINVAL, "block %d has no attention of kind %d (block_kinds)", block, kind);
  if (step < 0 || step >= c.n_steps) return fail(PAB_EINVAL, "step %d outside [0, %d)", step, c.n_steps);
  const size_t cell = (size_t)block * 3 + kind;
  if (step < ctx->last_step[cell])
    return fail(PAB_ESTATE, "step %d after step %d for block %d kind %d without pab_reset", step,
                ctx->last_step[cell], block, kind);
  const int decision = pab_schedule(kind, step, c.range_lo, c.range_hi, c.interval[kind]);
  if (decision < 0) return decision;
  if (decision == PAB_REUSE) {   // the slot must hold the step that Eq. 1 broadcasts from
    const int src = pab_source_step(kind, step, c.range_lo, c.range_hi, c.interval[kind]);
    if (ctx->computed_step[cell] != src)
      return fail(PAB_ESTATE, "reuse at step %d needs the output of step %d, block %d kind %d holds step %d", step, src,
                  block, kind, ctx->computed_step[cell]);
  }
  *slot = const_cast<void *>(pab_slot_ptr(ctx, block, kind));
  return decision;
}

void commit_cell(pab_ctx *ctx, int block, int kind, int step, int decision) {
  const size_t cell = (size_t)block * 3 + kind;
  if (decision == PAB_COMPUTE) {
    ctx->computed_step[cell] = step;
    ctx->launches++;
  }
  ctx->last_step[cell] = step;
}

// ---- the attention module (paper App. B.5 / B.6) ----
size_t module_plane_bytes(int T, int S, int L, int H, int D) {
  const long long rows = (long long)T * S > L ? (long long)T * S : L;
  return ((size_t)rows * H * D * 2 + 255) / 256 * 256;
}

// projection kernel shape: 4 x 2 wavefronts of 1 x 4 MFMA tiles = 128 tokens x 256 features per workgroup
// (eight wavefronts measured 3% faster than four with twice the tiles each)
constexpr int GEMM_NST = 3, GEMM_WM = 4, GEMM_WN = 2, GEMM_TM = 1, GEMM_TN = 4;
constexpr int GEMM_MF = 16;   // 16 x 16 x 32 MFMA tiles
constexpr int GEMM_BM = 32 * GEMM_WM * GEMM_TM, GEMM_BN = 32 * GEMM_WN * GEMM_TN;

int launch_gemm(int M, int N, int K, const void *A, const void *W, const void *bias, void *C, long long ldc,
                int n_split, long long plane_stride, hipStream_t st, int act = 0) {
  if (!A || !W || !C) return fail(PAB_EINVAL, "A, W and C must not be NULL");
  if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(C) |
       reinterpret_cast<uintptr_t>(bias)) & 15u)
    return fail(PAB_EINVAL, "A, W, bias and C must be 16-byte aligned");
  if (M < 1 || N < 1) return fail(PAB_EINVAL, "M=%d N=%d must be >= 1", M, N);
  if (K < 32 || K % 32) return fail(PAB_EINVAL, "K=%d must be a positive multiple of 32", K);
  if (N % 4 || ldc % 4 || plane_stride % 4 || (n_split != N && n_split % 8))
    return fail(PAB_EINVAL, "N=%d and ldc=%lld must be multiples of 4", N, ldc);
  if ((long long)M * K > 0x7fffffffLL || (long long)N * K > 0x7fffffffLL)
    return fail(PAB_EINVAL, "matrix too large");
  pab::GemmParams p;
  p.A = static_cast<const pab::bf16_t *>(A);
  p.W = static_cast<const pab::bf16_t *>(W);
  p.bias = static_cast<const pab::bf16_t *>(bias);
  p.C = C;
  p.M = M; p.N = N; p.K = K; p.ldc = ldc;
  p.n_split = n_split; p.plane_stride = plane_stride; p.act = act;
  // Few token rows (the text of a cross-attention module): 128 x 64 tiles, four wavefronts stacked along the
  // tokens, plain tile order: four times the workgroups, spread over all XCDs.
  const bool skinny = (long long)((M + GEMM_BM - 1) / GEMM_BM) * ((N + GEMM_BN - 1) / GEMM_BN) < 512 && (M + GEMM_BM - 1) / GEMM_BM < 8;
  const int bm = GEMM_BM, bn = skinny ? 64 : GEMM_BN;
  p.n_mt = (M + bm - 1) / bm;
  p.n_nt = (N + bn - 1) / bn;
  p.xcd_map = skinny ? 0 : 1;
  long long grid;
  if (skinny) {
    grid = (long long)p.n_mt * p.n_nt;
  } else {   // an XCD owns every eighth token tile and takes them four at a time over all feature tiles
    const long long owned = (p.n_mt + 7) / 8, groups = (owned + 3) / 4;
    grid = 8 * groups * 4 * p.n_nt;
  }
  if (grid > 0x7fffffffLL) return fail(PAB_EINVAL, "matrix too large");
  if (skinny)
    hipLaunchKernelGGL((pab::gemm_bias_kernel<GEMM_NST, 4, 1, 1, 2, GEMM_MF>), dim3((unsigned)grid), dim3(256), 0, st, p);
  else
    hipLaunchKernelGGL((pab::gemm_bias_kernel<GEMM_NST, GEMM_WM, GEMM_WN, GEMM_TM, GEMM_TN, GEMM_MF>), dim3((unsigned)grid),
                       dim3(64 * GEMM_WM * GEMM_WN), 0, st, p);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PAB_EDEVICE, "kernel launch failed: %s", hipGetErrorString(e));
  return PAB_OK;
}

int launch_ln_modulate(int n_tok, int C, const void *x, const void *shift, const void *scale, void *h, hipStream_t st) {
  pab::LnModParams p;
  p.x = static_cast<const pab::bf16_t *>(x);
  p.shift = static_cast<const pab::bf16_t *>(shift);
  p.scale = static_cast<const pab::bf16_t *>(scale);
  p.h = static_cast<pab::bf16_t *>(h);
  p.n_tok = n_tok; p.C = C; p.eps = 1e-6f;
  const dim3 grid((unsigned)((n_tok + 3) / 4)), block(256);
  switch ((C + 511) / 512) {
    case 1: hipLaunchKernelGGL((pab::ln_modulate_kernel<1>), grid, block, 0, st, p); break;
    case 2: hipLaunchKernelGGL((pab::ln_modulate_kernel<2>), grid, block, 0, st, p); break;
    case 3: hipLaunchKernelGGL((pab::ln_modulate_kernel<3>), grid, block, 0, st, p); break;
    case 4: hipLaunchKernelGGL((pab::ln_modulate_kernel<4>), grid, block, 0, st, p); break;
    default: return fail(PAB_EINVAL, "hidden size %d beyond 2048", C);
  }
  return PAB_OK;
}

int launch_qk_norm(int n_tok, int H, int D, int S, int rope, void *q, void *k, const pab_module_weights *w, hipStream_t st) {
  pab::QkNormParams p;
  p.q = static_cast<pab::bf16_t *>(q);
  p.k = static_cast<pab::bf16_t *>(k);
  p.gq = static_cast<const pab::bf16_t *>(w->gamma_q); p.bq = static_cast<const pab::bf16_t *>(w->beta_q);
  p.gk = static_cast<const pab::bf16_t *>(w->gamma_k); p.bk = static_cast<const pab::bf16_t *>(w->beta_k);
  p.n_tok = n_tok; p.H = H; p.S = S; p.rope = rope; p.eps = 1e-6f;
  p.log2_base = 13.287712379549449f;   // log2(10000)
  // three lanes per 72-element row (21 rows per wavefront), two per 32-element row (32 rows)
  const int rows_per_wave = D == 72 ? 21 : 32;
  const long long waves = ((long long)n_tok * H + rows_per_wave - 1) / rows_per_wave;
  const dim3 grid((unsigned)((waves + 3) / 4), 2), block(256);
  if (D == 72) hipLaunchKernelGGL((pab::qk_norm_rope_kernel<72, 3>), grid, block, 0, st, p);
  else hipLaunchKernelGGL((pab::qk_norm_rope_kernel<32, 2>), grid, block, 0, st, p);
  return PAB_OK;
}

int launch_module(int kind, int T, int S, int L, int H, int D, const void *x, const void *text,
                  const pab_module_weights *w, void *scratch, size_t scratch_bytes, void *out, hipStream_t st) {
  const int C = H * D;
  const long long tok = (long long)T * S;
  if (C % 32) return fail(PAB_EINVAL, "hidden size heads*head_dim=%d must be a multiple of 32", C);
  if (tok > 0x7fffffffLL / C) return fail(PAB_EINVAL, "too many tokens");
  if (!x || !w || !scratch) return fail(PAB_EINVAL, "x, weights and scratch must be non-NULL on a computed step");
  if (!aligned16(x) || (reinterpret_cast<uintptr_t>(scratch) & 255u)) return fail(PAB_EINVAL, "x must be 16-byte, scratch 256-byte aligned");
  const size_t plane = module_plane_bytes(T, S, L, H, D);
  if (scratch_bytes < 4 * plane) return fail(PAB_ENOMEM, "scratch of %zu bytes, need %zu", scratch_bytes, 4 * plane);
  unsigned char *s0 = static_cast<unsigned char *>(scratch);
  void *p_ho = s0, *p_q = s0 + plane, *p_k = s0 + 2 * plane, *p_v = s0 + 3 * plane;
  const long long plane_elems = (long long)(plane / 2);
  int rc;
  if (kind == PAB_CROSS) {
    if (!text || !aligned16(text)) return fail(PAB_EINVAL, "cross attention needs the text tokens, 16-byte aligned");
    if (!w->w_qkv || !w->w_kv || !w->w_o) return fail(PAB_EINVAL, "cross module needs w_qkv (queries), w_kv and w_o");
    if ((rc = launch_gemm((int)tok, C, C, x, w->w_qkv, w->b_qkv, p_q, C, C, 0, st)) != PAB_OK) return rc;
    if ((rc = launch_gemm(L, 2 * C, C, text, w->w_kv, w->b_kv, p_k, C, C, plane_elems, st)) != PAB_OK) return rc;
  } else {
    if (!w->shift || !w->scale || !w->w_qkv || !w->gamma_q || !w->beta_q || !w->gamma_k || !w->beta_k || !w->w_o)
      return fail(PAB_EINVAL, "self-attention module needs shift, scale, w_qkv, gamma/beta of q and k, w_o");
    if ((rc = launch_ln_modulate((int)tok, C, x, w->shift, w->scale, p_ho, st)) != PAB_OK) return rc;
    if ((rc = launch_gemm((int)tok, 3 * C, C, p_ho, w->w_qkv, w->b_qkv, p_q, C, C, plane_elems, st)) != PAB_OK) return rc;
    if ((rc = launch_qk_norm((int)tok, H, D, S, kind == PAB_TEMPORAL, p_q, p_k, w, st)) != PAB_OK) return rc;
  }
  if ((rc = launch_checked(kind, PAB_BF16, T, S, L, H, D, p_q, p_k, p_v, p_ho, st)) != PAB_OK) return rc;
  if ((rc = launch_gemm((int)tok, C, C, p_ho, w->w_o, w->b_o, out, C, C, 0, st)) != PAB_OK) return rc;
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PAB_EDEVICE, "kernel launch failed: %s", hipGetErrorString(e));
  return PAB_OK;
}

// ---- module scratch inside the library, for callers that cannot allocate.  One array per GPU the library is
//      loaded on, held until the process ends; its device address is looked up once per device.  Every plane of
//      it is written in full before it is read within a call, so nothing has to be cleared between calls. ----
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)16 << 20;
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static __device__ __align__(256) __attribute__((used)) unsigned char g_static_scratch[STATIC_SCRATCH_BYTES];
void *g_static_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES];   // device address per device ordinal, NULL until looked up
std::mutex g_static_scratch_mutex;

// device address of the scratch array on the current device (host code never uses the array's name for that)
int static_scratch_of_current_device(void **ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(PAB_EDEVICE, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return fail(PAB_EDEVICE, "device ordinal %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
  if (!g_static_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess || !p) return fail(PAB_EDEVICE, "hipGetSymbolAddress failed: %s", hipGetErrorString(e));
    g_static_scratch_ptr[dev] = p;
  }
  *ptr = g_static_scratch_ptr[dev];
  return PAB_OK;
}

// ---- the MLP module (paper Sec. 2.3, last sentence; App. A.2.2 MLP table) ----
size_t mlp_scratch_bytes_of(long long n_tok, int C, int F) {
  const size_t h = ((size_t)n_tok * C * 2 + 255) / 256 * 256, u = ((size_t)n_tok * F * 2 + 255) / 256 * 256;
  return h + u;
}

int launch_mlp(long long n_tok, int C, int F, const void *x, const pab_mlp_weights *w, void *scratch,
               size_t scratch_bytes, void *out, hipStream_t st) {
  if (n_tok < 1 || C < 32 || C % 32 || C > 2048 || F < 32 || F % 32)
    return fail(PAB_EINVAL, "n_tok=%lld, C=%d (multiple of 32, <= 2048), F=%d (multiple of 32)", n_tok, C, F);
  if (n_tok > 0x7fffffffLL / (F > C ? F : C)) return fail(PAB_EINVAL, "too many tokens");
  if (!x || !w || !scratch || !out) return fail(PAB_EINVAL, "x, weights, scratch and out must be non-NULL");
  if (!w->shift || !w->scale || !w->w1 || !w->w2) return fail(PAB_EINVAL, "MLP needs shift, scale, w1 and w2");
  if (!aligned16(x) || !aligned16(out) || (reinterpret_cast<uintptr_t>(scratch) & 255u))
    return fail(PAB_EINVAL, "x and out must be 16-byte, scratch 256-byte aligned");
  const size_t need = mlp_scratch_bytes_of(n_tok, C, F);
  if (scratch_bytes < need) return fail(PAB_ENOMEM, "scratch of %zu bytes, need %zu", scratch_bytes, need);
  unsigned char *h = static_cast<unsigned char *>(scratch);
  unsigned char *u = h + ((size_t)n_tok * C * 2 + 255) / 256 * 256;
  int rc;
  if ((rc = launch_ln_modulate((int)n_tok, C, x, w->shift, w->scale, h, st)) != PAB_OK) return rc;
  if ((rc = launch_gemm((int)n_tok, F, C, h, w->w1, w->b1, u, F, F, 0, st, 1)) != PAB_OK) return rc;
  if ((rc = launch_gemm((int)n_tok, C, F, u, w->w2, w->b2, out, C, C, 0, st)) != PAB_OK) return rc;
  return PAB_OK;
}

}  // namespace

// context of the MLP broadcast: one slot per participating block
struct pab_mlp_ctx {
  pab_mlp_config cfg;
  std::vector<int> starts;
  unsigned char *workspace;
  size_t slot_bytes;
  std::vector<int> last_step;       // per block
  std::vector<int> computed_step;   // per participating block: step whose output the slot holds
  long long launches;
};

extern "C" {

int pab_mlp_schedule(int step, int block, const int *start_steps, int n_starts, int range, int block_lo,
                     int block_hi) {
  if (step < 0 || block < 0) return fail(PAB_EINVAL, "step %d and block %d must be >= 0", step, block);
  if (range < 1) return fail(PAB_EINVAL, "range %d must be >= 1", range);
  if (n_starts < 0 || (n_starts > 0 && !start_steps)) return fail(PAB_EINVAL, "bad list of starting steps");
  for (int i = 0; i < n_starts; ++i)
    if (start_steps[i] < 0) return fail(PAB_EINVAL, "starting step %d is negative", start_steps[i]);
  if (block < block_lo || block > block_hi) return PAB_COMPUTE;
  for (int i = 0; i < n_starts; ++i)
    if (step - start_steps[i] >= 1 && step - start_steps[i] <= range - 1) return PAB_REUSE;
  return PAB_COMPUTE;
}

int pab_mlp_source_step(int step, int block, const int *start_steps, int n_starts, int range, int block_lo,
                        int block_hi) {
  const int d = pab_mlp_schedule(step, block, start_steps, n_starts, range, block_lo, block_hi);
  if (d < 0) return d;
  if (d == PAB_COMPUTE) return step;
  for (int i = 0; i < n_starts; ++i)
    if (step - start_steps[i] >= 1 && step - start_steps[i] <= range - 1) return start_steps[i];
  return step;
}

int pab_steps_from_timesteps(const double *timesteps, int n_steps, const double *start_timesteps, int n_starts,
                             int *start_steps) {
  if (!timesteps || n_steps < 1 || n_starts < 0 || (n_starts > 0 && (!start_timesteps || !start_steps)))
    return fail(PAB_EINVAL, "bad arguments");
  for (int s = 1; s < n_steps; ++s)
    if (timesteps[s] > timesteps[s - 1]) return fail(PAB_EINVAL, "timesteps increase at step %d", s);
  int found = 0;
  for (int i = 0; i < n_starts; ++i) {
    int s = 0;
    while (s < n_steps && timesteps[s] > start_timesteps[i]) ++s;
    start_steps[i] = s < n_steps ? s : -1;
    found += s < n_steps;
  }
  return found;
}

size_t pab_mlp_scratch_bytes(long long n_tok, int hidden, int inner) {
  if (n_tok < 1 || hidden < 1 || inner < 1) return 0;
  return mlp_scratch_bytes_of(n_tok, hidden, inner);
}

int pab_mlp_compute(long long n_tok, int hidden, int inner, const void *x, const pab_mlp_weights *w, void *scratch,
                    size_t scratch_bytes, void *out, void *hip_stream) {
  const int rc = launch_mlp(n_tok, hidden, inner, x, w, scratch, scratch_bytes, out, static_cast<hipStream_t>(hip_stream));
  if (rc != PAB_OK) return rc;
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PAB_EDEVICE, "kernel launch failed: %s", hipGetErrorString(e));
  return PAB_OK;
}

size_t pab_mlp_workspace_bytes(const pab_mlp_config *c) {
  if (!c || c->n_blocks < 1 || c->n_tok < 1 || c->hidden < 1 || c->block_lo < 0 || c->block_hi < c->block_lo) return 0;
  const int hi = c->block_hi < c->n_blocks - 1 ? c->block_hi : c->n_blocks - 1;
  if (hi < c->block_lo) return 0;
  const size_t slot = ((size_t)c->n_tok * c->hidden * 2 + 255) / 256 * 256;
  return slot * (size_t)(hi - c->block_lo + 1);
}

int pab_mlp_create(const pab_mlp_config *c, const int *start_steps, void *workspace, size_t workspace_bytes,
                   pab_mlp_ctx **out) {
  if (!out) return fail(PAB_EINVAL, "out is NULL");
  *out = nullptr;
  if (!c) return fail(PAB_EINVAL, "config is NULL");
  if (c->n_blocks < 1 || c->n_steps < 1 || c->n_tok < 1) return fail(PAB_EINVAL, "n_blocks, n_steps, n_tok must be >= 1");
  if (c->hidden < 32 || c->hidden % 32 || c->hidden > 2048 || c->inner < 32 || c->inner % 32)
    return fail(PAB_EINVAL, "hidden=%d (multiple of 32, <= 2048), inner=%d (multiple of 32)", c->hidden, c->inner);
  if (c->range < 1 || c->n_starts < 0 || (c->n_starts > 0 && !start_steps)) return fail(PAB_EINVAL, "bad range or starts");
  if (c->block_lo < 0 || c->block_hi < c->block_lo) return fail(PAB_EINVAL, "bad block range [%d, %d]", c->block_lo, c->block_hi);
  for (int i = 0; i < c->n_starts; ++i)
    if (start_steps[i] < 0 || start_steps[i] >= c->n_steps) return fail(PAB_EINVAL, "starting step %d outside the run", start_steps[i]);
  // two broadcasts must not overlap: a start inside another start's reused steps would itself be reused,
  // and the steps after it would then name a source that was never computed
  for (int i = 0; i < c->n_starts; ++i)
    for (int j = 0; j < c->n_starts; ++j)
      if (i != j && start_steps[j] != start_steps[i] && start_steps[j] - start_steps[i] >= 1 &&
          start_steps[j] - start_steps[i] <= c->range - 1)
        return fail(PAB_EINVAL, "starting steps %d and %d are closer than the broadcast range %d", start_steps[i],
                    start_steps[j], c->range);
  const size_t need = pab_mlp_workspace_bytes(c);
  if (need > 0) {
    if (!workspace) return fail(PAB_EINVAL, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(PAB_EINVAL, "workspace must be 256-byte aligned");
    if (workspace_bytes < need) return fail(PAB_ENOMEM, "workspace of %zu bytes, need %zu", workspace_bytes, need);
  }
  pab_mlp_ctx *ctx = new (std::nothrow) pab_mlp_ctx;
  if (!ctx) return fail(PAB_ENOMEM, "out of host memory");
  ctx->cfg = *c;
  ctx->starts.assign(start_steps, start_steps + c->n_starts);
  ctx->workspace = static_cast<unsigned char *>(workspace);
  ctx->slot_bytes = ((size_t)c->n_tok * c->hidden * 2 + 255) / 256 * 256;
  ctx->last_step.assign(c->n_blocks, -1);
  ctx->computed_step.assign(c->n_blocks, -1);
  ctx->launches = 0;
  *out = ctx;
  return PAB_OK;
}

int pab_mlp_reset(pab_mlp_ctx *ctx) {
  if (!ctx) return fail(PAB_EINVAL, "ctx is NULL");
  std::fill(ctx->last_step.begin(), ctx->last_step.end(), -1);
  std::fill(ctx->computed_step.begin(), ctx->computed_step.end(), -1);
  ctx->launches = 0;
  return PAB_OK;
}

int pab_mlp(pab_mlp_ctx *ctx, int block, int step, const void *x, const pab_mlp_weights *w, void *scratch,
            size_t scratch_bytes, void *y, void *hip_stream, const void **out) {
  if (!ctx) return fail(PAB_EINVAL, "ctx is NULL");
  if (!out) return fail(PAB_EINVAL, "out is NULL");
  *out = nullptr;
  const pab_mlp_config &c = ctx->cfg;
  if (block < 0 || block >= c.n_blocks) return fail(PAB_EINVAL, "block %d outside [0, %d)", block, c.n_blocks);
  if (step < 0 || step >= c.n_steps) return fail(PAB_EINVAL, "step %d outside [0, %d)", step, c.n_steps);
  if (step < ctx->last_step[block])
    return fail(PAB_ESTATE, "step %d after step %d for block %d without pab_mlp_reset", step, ctx->last_step[block], block);
  const int decision = pab_mlp_schedule(step, block, ctx->starts.data(), c.n_starts, c.range, c.block_lo, c.block_hi);
  if (decision < 0) return decision;
  const bool cached = block >= c.block_lo && block <= c.block_hi;
  void *dst = cached ? const_cast<void *>(pab_mlp_slot_ptr(ctx, block)) : y;
  if (decision == PAB_REUSE) {
    const int src = pab_mlp_source_step(step, block, ctx->starts.data(), c.n_starts, c.range, c.block_lo, c.block_hi);
    if (ctx->computed_step[block] != src)
      return fail(PAB_ESTATE, "reuse at step %d needs the output of step %d, block %d holds step %d", step, src, block,
                  ctx->computed_step[block]);
  } else {
    if (!dst) return fail(PAB_EINVAL, "block %d is not cached: y must be given", block);
    const int rc = launch_mlp(c.n_tok, c.hidden, c.inner, x, w, scratch, scratch_bytes, dst, static_cast<hipStream_t>(hip_stream));
    if (rc != PAB_OK) return rc;
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PAB_EDEVICE, "kernel launch failed: %s", hipGetErrorString(e));
    ctx->computed_step[block] = step;
    ctx->launches++;
  }
  ctx->last_step[block] = step;
  *out = dst;
  return decision;
}

long long pab_mlp_launch_count(const pab_mlp_ctx *ctx) { return ctx ? ctx->launches : -1; }

const void *pab_mlp_slot_ptr(const pab_mlp_ctx *ctx, int block) {
  if (!ctx || block < ctx->cfg.block_lo || block > ctx->cfg.block_hi || block >= ctx->cfg.n_blocks) return nullptr;
  return ctx->workspace + ctx->slot_bytes * (size_t)(block - ctx->cfg.block_lo);
}

int pab_mlp_destroy(pab_mlp_ctx *ctx) {
  delete ctx;
  return PAB_OK;
}

int pab_schedule(int kind, int step, int range_lo, int range_hi, int interval) {
  if (!kind_ok(kind)) return fail(PAB_EINVAL, "kind %d is not spatial(0)/temporal(1)/cross(2)", kind);
  if (step < 0) return fail(PAB_EINVAL, "step %d is negative", step);
  if (interval < 1) return fail(PAB_EINVAL, "interval %d must be >= 1", interval);
  if (range_lo < 0 || range_lo > range_hi)
    return fail(PAB_EINVAL, "window [%d, %d] must satisfy 0 <= lo <= hi", range_lo, range_hi);
  if (step < range_lo || step > range_hi) return PAB_COMPUTE;
  return ((step - range_lo) % interval == 0) ? PAB_COMPUTE : PAB_REUSE;
}

int pab_source_step(int kind, int step, int range_lo, int range_hi, int interval) {
  const int d = pab_schedule(kind, step, range_lo, range_hi, interval);
  if (d < 0) return d;
  if (d == PAB_COMPUTE) return step;
  return step - (step - range_lo) % interval;
}

int pab_window_from_timesteps(const double *timesteps, int n_steps, double t_start, double t_end,
                              int *range_lo, int *range_hi) {
  if (!timesteps || !range_lo || !range_hi) return fail(PAB_EINVAL, "NULL pointer");
  if (n_steps < 1) return fail(PAB_EINVAL, "n_steps=%d must be >= 1", n_steps);
  if (!(t_start >= t_end)) return fail(PAB_EINVAL, "window [%g - %g] starts below its end", t_start, t_end);
  for (int s = 1; s < n_steps; ++s)
    if (timesteps[s] > timesteps[s - 1])
      return fail(PAB_EINVAL, "timesteps increase at step %d (%g after %g)", s, timesteps[s], timesteps[s - 1]);
  // the list never increases: the steps inside form one run; find its two ends
  int lo = 0;
  while (lo < n_steps && timesteps[lo] > t_start) ++lo;
  int hi = n_steps - 1;
  while (hi >= 0 && timesteps[hi] < t_end) --hi;
  if (lo > hi) return 0;
  *range_lo = lo;
  *range_hi = hi;
  return hi - lo + 1;
}

int pab_preset(int model, int level, int interval[3], double *t_start, double *t_end) {
  // App. A.2.1: {spatial, temporal, cross} per level, and the window of the model
  static const int ranges[3][3][3] = {
      {{2, 4, 6}, {3, 5, 7}, {5, 7, 9}},   // Open-Sora
      {{2, 4, 6}, {3, 5, 7}, {5, 7, 9}},   // Open-Sora-Plan
      {{2, 3, 5}, {3, 4, 7}, {4, 6, 9}},   // Latte
  };
  static const double window[3][2] = {{930, 450}, {850, 100}, {800, 100}};
  if (model < 0 || model > 2) return fail(PAB_EINVAL, "model %d is not open_sora(0)/open_sora_plan(1)/latte(2)", model);
  if (level < 0 || level > 2) return fail(PAB_EINVAL, "level %d outside 0..2", level);
  if (!interval || !t_start || !t_end) return fail(PAB_EINVAL, "NULL pointer");
  for (int k = 0; k < 3; ++k) interval[k] = ranges[model][level][k];
  *t_start = window[model][0];
  *t_end = window[model][1];
  return PAB_OK;
}

size_t pab_workspace_bytes(const pab_config *cfg) {
  if (check_config(cfg) != PAB_OK) return 0;
  size_t slots = 0;
  for (int b = 0; b < cfg->n_blocks; ++b) slots += (size_t)__builtin_popcount(kinds_of_block(*cfg, b));
  return slot_bytes_of(*cfg) * slots;
}

int pab_create(const pab_config *cfg, void *workspace, size_t workspace_bytes, pab_ctx **out) {
  if (!out) return fail(PAB_EINVAL, "out is NULL");
  *out = nullptr;
  const int rc = check_config(cfg);
  if (rc != PAB_OK) return rc;
  if (!workspace) return fail(PAB_EINVAL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(PAB_EINVAL, "workspace must be 256-byte aligned");
  const size_t need = pab_workspace_bytes(cfg);
  if (workspace_bytes < need)
    return fail(PAB_ENOMEM, "workspace has %zu bytes, the cache needs %zu", workspace_bytes, need);
  pab_ctx *ctx = new (std::nothrow) pab_ctx;
  if (!ctx) return fail(PAB_ENOMEM, "out of host memory");
  ctx->cfg = *cfg;
  ctx->workspace = static_cast<unsigned char *>(workspace);
  ctx->slot_bytes = slot_bytes_of(*cfg);
  ctx->slot_index.assign((size_t)cfg->n_blocks * 3, -1);
  long long next = 0;
  for (int b = 0; b < cfg->n_blocks; ++b)
    for (int k = 0; k < 3; ++k)
      if ((kinds_of_block(*cfg, b) >> k) & 1) ctx->slot_index[(size_t)b * 3 + k] = next++;
  ctx->cfg.block_kinds = nullptr;   // the caller's array is not kept
  ctx->last_step.assign((size_t)cfg->n_blocks * 3, -1);
  ctx->computed_step.assign((size_t)cfg->n_blocks * 3, -1);
  ctx->launches = 0;
  *out = ctx;
  return PAB_OK;
}

int pab_reset(pab_ctx *ctx) {
  if (!ctx) return fail(PAB_EINVAL, "ctx is NULL");
  std::fill(ctx->last_step.begin(), ctx->last_step.end(), -1);
  std::fill(ctx->computed_step.begin(), ctx->computed_step.end(), -1);
  ctx->launches = 0;
  return PAB_OK;
}

const void *pab_slot_ptr(const pab_ctx *ctx, int block, int kind) {
  if (!ctx || !kind_ok(kind) || block < 0 || block >= ctx->cfg.n_blocks) return nullptr;
  const long long slot = ctx->slot_index[(size_t)block * 3 + kind];
  return slot < 0 ? nullptr : ctx->workspace + (size_t)slot * ctx->slot_bytes;
}

int pab_attention(pab_ctx *ctx, int block, int kind, int step, const void *q, const void *k, const void *v,
                  void *hip_stream, const void **out) {
  if (!ctx) return fail(PAB_EINVAL, "ctx is NULL");
  if (!out) return fail(PAB_EINVAL, "out is NULL");
  *out = nullptr;
  const pab_config &c = ctx->cfg;
  void *slot = nullptr;
  const int decision = schedule_cell(ctx, block, kind, step, &slot);
  if (decision < 0) return decision;
  if (decision == PAB_COMPUTE) {
    if (!q || !k || !v) return fail(PAB_EINVAL, "q, k, v must be non-NULL on a computed step");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v)) return fail(PAB_EINVAL, "q, k, v must be 16-byte aligned");
    const int rc = launch_checked(kind, c.dtype, c.T, c.S, c.L, c.heads, c.head_dim, q, k, v, slot,
                                  static_cast<hipStream_t>(hip_stream));
    if (rc != PAB_OK) return rc;
  }
  commit_cell(ctx, block, kind, step, decision);
  *out = slot;
  return decision;
}

int pab_attention_compute(int kind, int dtype, int T, int S, int L, int heads, int head_dim, const void *q,
                          const void *k, const void *v, void *o, void *hip_stream) {
  const int rc = check_shape(kind, dtype, T, S, L, heads, head_dim);
  if (rc != PAB_OK) return rc;
  if (!q || !k || !v || !o) return fail(PAB_EINVAL, "q, k, v, o must be non-NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
    return fail(PAB_EINVAL, "q, k, v, o must be 16-byte aligned");
  return launch_checked(kind, dtype, T, S, L, heads, head_dim, q, k, v, o, static_cast<hipStream_t>(hip_stream));
}

int pab_linear(int M, int N, int K, const void *A, const void *W, const void *bias, void *C, long long ldc,
               void *hip_stream) {
  if (ldc < N) return fail(PAB_EINVAL, "ldc=%lld must be >= N=%d", ldc, N);
  return launch_gemm(M, N, K, A, W, bias, C, ldc, N, 0, static_cast<hipStream_t>(hip_stream));
}

size_t pab_module_scratch_bytes(const pab_config *cfg) {
  if (check_config(cfg) != PAB_OK) return 0;
  return 4 * module_plane_bytes(cfg->T, cfg->S, cfg->L, cfg->heads, cfg->head_dim);
}

int pab_module_compute(int kind, int T, int S, int L, int heads, int head_dim, const void *x, const void *text,
                       const pab_module_weights *w, void *scratch, size_t scratch_bytes, void *out,
                       void *hip_stream) {
  const int rc = check_shape(kind, PAB_BF16, T, S, L, heads, head_dim);
  if (rc != PAB_OK) return rc;
  if (!out || !aligned16(out)) return fail(PAB_EINVAL, "out must be non-NULL and 16-byte aligned");
  return launch_module(kind, T, S, L, heads, head_dim, x, text, w, scratch, scratch_bytes, out,
                       static_cast<hipStream_t>(hip_stream));
}

size_t pab_module_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int pab_module_compute_static(int kind, int T, int S, int L, int heads, int head_dim, const void *x, const void *text,
                              const pab_module_weights *w, void *out, void *hip_stream) {
  const int rc = check_shape(kind, PAB_BF16, T, S, L, heads, head_dim);
  if (rc != PAB_OK) return rc;
  if (!out || !aligned16(out)) return fail(PAB_EINVAL, "out must be non-NULL and 16-byte aligned");
  const size_t need = 4 * module_plane_bytes(T, S, L, heads, head_dim);
  if (need > STATIC_SCRATCH_BYTES)
    return fail(PAB_ENOMEM, "this shape needs %zu bytes of scratch, the built-in scratch holds %zu: use pab_module_compute",
                need, STATIC_SCRATCH_BYTES);
  void *scratch = nullptr;
  const int rs = static_scratch_of_current_device(&scratch);
  if (rs != PAB_OK) return rs;
  return launch_module(kind, T, S, L, heads, head_dim, x, text, w, scratch, STATIC_SCRATCH_BYTES, out,
                       static_cast<hipStream_t>(hip_stream));
}

int pab_module_attention(pab_ctx *ctx, int block, int kind, int step, const void *x, const void *text,
                         const pab_module_weights *w, void *scratch, size_t scratch_bytes, void *hip_stream,
                         const void **out) {
  if (!ctx) return fail(PAB_EINVAL, "ctx is NULL");
  if (!out) return fail(PAB_EINVAL, "out is NULL");
  *out = nullptr;
  const pab_config &c = ctx->cfg;
  if (c.dtype != PAB_BF16) return fail(PAB_EINVAL, "the module path takes bf16 configs only");
  void *slot = nullptr;
  const int decision = schedule_cell(ctx, block, kind, step, &slot);
  if (decision < 0) return decision;
  if (decision == PAB_COMPUTE) {
    const int rc = launch_module(kind, c.T, c.S, c.L, c.heads, c.head_dim, x, text, w, scratch, scratch_bytes, slot,
                                 static_cast<hipStream_t>(hip_stream));
    if (rc != PAB_OK) return rc;
  }
  commit_cell(ctx, block, kind, step, decision);
  *out = slot;
  return decision;
}

long long pab_launch_count(const pab_ctx *ctx) { return ctx ? ctx->launches : -1; }

int pab_destroy(pab_ctx *ctx) {
  if (!ctx) return fail(PAB_EINVAL, "ctx is NULL");
  delete ctx;
  return PAB_OK;
}

const char *pab_last_error(void) { return g_err; }

}  // extern "C"
