/*
 * pab.h -- C ABI of libpab: the attention hot path of Pyramid Attention
 * Broadcast (PAB) for one MI355X (gfx950).
 *
 * PAB (paper Sec. 2.3) speeds up a video diffusion transformer by computing
 * each attention kind only at some diffusion steps and handing the output of
 * the last computed step to the following steps unchanged.  This library holds
 * exactly that path: the compute-or-reuse schedule (Eq. 1), a device-resident
 * cache of the broadcast outputs keyed by (block, kind), and the three
 * attention kernels (Sec. 2.1: spatial, temporal, cross).
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers owned by the caller, 16-byte
 *     aligned, dense, in the layouts given below.  The library never allocates,
 *     frees or copies device memory and never synchronises a stream (the one
 *     piece of device memory of its own is the fixed array behind
 *     pab_module_compute_static, part of its code object).
 *   - Activations are laid out [T, S, H, D]: T latent frames, S tokens per
 *     frame, H heads, D head dim, D contiguous.  Spatial and temporal attention
 *     read the same buffers (batch = T / sequence = S, resp. batch = S /
 *     sequence = T); no transposed copy is ever made.  Cross-attention keys and
 *     values are [L, H, D] for L text tokens.
 *   - Element type is bf16 (PAB_BF16) or fp32 (PAB_F32) for q, k, v and the
 *     output alike.  Arithmetic: operands rounded to bf16, products and softmax
 *     accumulated in fp32, output rounded once to the element type.
 *   - Supported head dims: 32 and 72.
 *   - Every function returns PAB_OK (0) or a negative pab_status; nothing
 *     aborts or throws across this boundary.  pab_last_error() gives the text
 *     of the calling thread's last failure.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Kernels are launched on it asynchronously.
 */
#ifndef PAB_H
#define PAB_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* attention kinds (paper Sec. 2.1) */
enum pab_kind { PAB_SPATIAL = 0, PAB_TEMPORAL = 1, PAB_CROSS = 2 };
/* schedule decisions (paper Eq. 1: F(X_t) computed, Y*_t reused) */
enum pab_decision { PAB_COMPUTE = 0, PAB_REUSE = 1 };
enum pab_status {
  PAB_OK = 0,
  PAB_EINVAL = -1,  /* bad argument: kind, step, block, shape, dtype, alignment, NULL */
  PAB_ESTATE = -2,  /* reuse of a slot that does not hold its source step; step went backwards */
  PAB_ENOMEM = -3,  /* workspace smaller than pab_workspace_bytes()                  */
  PAB_EDEVICE = -4  /* a HIP call failed                                             */
};
enum pab_dtype { PAB_BF16 = 0, PAB_F32 = 1 };

/*
 * One video-generation run.  interval[kind] is the paper's "broadcast range" n
 * of that kind (App. A.2.1: e.g. 2 / 4 / 6 for spatial / temporal / cross):
 * one computed step, then n-1 reused steps.  1 = never reuse (the no-PAB
 * baseline), 0 = the model has no attention of that kind (no cache slot).
 * [range_lo, range_hi] is the inclusive, 0-based window of diffusion steps
 * (denoising order, 0 = first / noisiest) in which broadcasting is active
 * (the paper's "diffusion timesteps" column, the stable middle segment of
 * Sec. 2.2); outside it every step is computed.
 */
typedef struct pab_config {
  int n_blocks;   /* transformer blocks; cache slots are keyed (block, kind) */
  int T, S;       /* latent frames, tokens per frame                          */
  int L;          /* text tokens for cross attention (ignored if interval[2]==0) */
  int heads, head_dim;
  int dtype;      /* enum pab_dtype */
  int n_steps;    /* diffusion steps of the run */
  int interval[3];
  int range_lo, range_hi;
  /* Optional, n_blocks entries or NULL: bit k of block_kinds[b] set = block b has attention of kind k.
   * Models whose blocks alternate (one spatial, the next temporal) get one cache slot per block this way
   * instead of one per kind and block.  NULL = every block has every kind with interval > 0.  A set bit
   * for a kind with interval 0 is PAB_EINVAL.  Host memory, read during the call only. */
  const unsigned char *block_kinds;
} pab_config;

typedef struct pab_ctx pab_ctx;

/*
 * Eq. 1 as a pure function (host, no device access, no state).
 * Inside [range_lo, range_hi] step s is computed iff (s - range_lo) is a
 * multiple of interval (the period is anchored at the first step of the
 * window); outside the window it is always computed.
 * Returns PAB_COMPUTE or PAB_REUSE; PAB_EINVAL if kind is not a pab_kind,
 * step < 0, interval < 1, range_lo < 0 or range_lo > range_hi.  `kind` does not change the
 * decision (the per-kind range is the caller's `interval`); it is validated.
 */
int pab_schedule(int kind, int step, int range_lo, int range_hi, int interval);

/*
 * Step whose computed output is delivered at `step` under the same schedule:
 * `step` itself if it computes, else the computed step that opened the current
 * broadcast run.  Negative pab_status on the errors of pab_schedule.
 */
int pab_source_step(int kind, int step, int range_lo, int range_hi, int interval);

/*
 * The paper states its broadcast windows as diffusion timesteps, e.g.
 * [930-450] on a scale where 1000 is the beginning of denoising and 0 its end
 * (App. A.2.1, table of attention broadcast configurations).  This maps such a
 * window onto the steps of a sampler (host, pure): timesteps[s] is the
 * timestep the sampler visits at step s, n_steps values that never increase.
 * Step s is inside iff t_end <= timesteps[s] <= t_start (both ends inclusive).
 * Returns the number of steps inside and, if that is >= 1, writes the first
 * and last of them to *range_lo / *range_hi (the values pab_config and
 * pab_schedule take).  0 means no step of this sampler falls in the window:
 * nothing is to be broadcast (use interval 1); *range_lo / *range_hi are then
 * left alone.  PAB_EINVAL: NULL pointer, n_steps < 1, t_start < t_end, or a
 * timestep list that increases somewhere.
 */
int pab_window_from_timesteps(const double *timesteps, int n_steps, double t_start, double t_end,
                              int *range_lo, int *range_hi);

/*
 * The settings the paper evaluates (App. A.2.1, same table): broadcast ranges
 * for spatial / temporal / cross attention and the timestep window, per model
 * and per level (0 = the best-quality setting PAB_246 / PAB_235, 1 and 2 the
 * faster ones).  Writes interval[0..2], *t_start and *t_end.
 * PAB_EINVAL: model not a pab_model, level outside 0..2, NULL pointer.
 */
enum pab_model { PAB_OPEN_SORA = 0, PAB_OPEN_SORA_PLAN = 1, PAB_LATTE = 2 };
int pab_preset(int model, int level, int interval[3], double *t_start, double *t_end);

/*
 * Bytes of device memory the broadcast cache of `cfg` needs: one output tensor
 * [T, S, H, D] per (block, kind that the block has), each slot rounded up to 256
 * bytes, laid out block-major, kind-minor.
 * Returns 0 if cfg is NULL or invalid (pab_last_error says why).
 */
size_t pab_workspace_bytes(const pab_config *cfg);

/*
 * Create a context over a caller-owned device workspace (paper Sec. 2.3: the
 * retained outputs Y*).  `workspace` must be 256-byte aligned, at least
 * pab_workspace_bytes(cfg) long, and must outlive the context.  The library
 * owns only the small host-side pab_ctx.  All slots start invalid.
 * Errors: PAB_EINVAL (NULL, bad shape / dtype / head_dim / interval / window,
 * misaligned workspace), PAB_ENOMEM (workspace too small).
 */
int pab_create(const pab_config *cfg, void *workspace, size_t workspace_bytes, pab_ctx **out);

/* Start a new video: every slot invalid again, step history cleared. */
int pab_reset(pab_ctx *ctx);

/*
 * One attention call of the denoising loop (paper Sec. 2.3, Eq. 1).
 * Looks up the schedule for (kind, step).  On PAB_COMPUTE it launches the
 * kernel of that kind on `hip_stream`, writing straight into cache slot
 * (block, kind); on PAB_REUSE it launches nothing and reads nothing (q, k, v
 * may be NULL or hold anything).  Either way *out receives the device pointer
 * of the slot, which holds -- once the stream reaches this point -- the
 * output [T, S, H, D] of the last computed step.  *out is borrowed and
 * read-only: valid until the next computed step of the same (block, kind),
 * pab_reset or pab_destroy.
 *   q: [T, S, H, D];  k, v: [T, S, H, D] (spatial, temporal) or [L, H, D] (cross).
 * Returns the decision taken (PAB_COMPUTE / PAB_REUSE) or a negative status:
 * PAB_EINVAL (NULL ctx/out, block or kind or step out of range, kind absent
 * from the config, NULL or misaligned q/k/v on a computed step), PAB_ESTATE
 * (reuse at a step whose source step, pab_source_step, is not the step the
 * slot holds -- never written, or the caller skipped that computed step -- or
 * a step smaller than the last step seen for this (block, kind) since the
 * last reset), PAB_EDEVICE (launch failed).
 * Never synchronises.
 */
int pab_attention(pab_ctx *ctx, int block, int kind, int step, const void *q, const void *k,
                  const void *v, void *hip_stream, const void **out);

/*
 * The attention operation alone (paper Sec. 2.1), no schedule and no cache:
 * o = softmax(q k^T / sqrt(D)) v of the given kind, written to `o`
 * ([T, S, H, D], same dtype), one kernel launch on `hip_stream`.  This is the
 * launch pab_attention performs on a computed step.
 * Errors: PAB_EINVAL (NULL / misaligned pointers, T, S, heads < 1, L < 1 for
 * cross, unsupported head_dim or dtype), PAB_EDEVICE.
 */
int pab_attention_compute(int kind, int dtype, int T, int S, int L, int heads, int head_dim,
                          const void *q, const void *k, const void *v, void *o, void *hip_stream);

/*
 * A projection of the attention module (paper App. B.5: "qkv proj", "o proj";
 * the first and the last step of the workflow of App. B.6): C = A W^T + bias, one kernel launch
 * on `hip_stream`.  A: [M, K] activations, W: [N, K] weights (row n produces
 * feature n), bias: [N] or NULL, C: [M, N] written with a row pitch of `ldc`
 * elements (ldc >= N; ldc > N lets several projections write side by side).
 * All bf16, dense along their last axis, device pointers, 16-byte aligned;
 * products accumulate in fp32 and are rounded once.
 * PAB_EINVAL: NULL or misaligned A / W / C, M or N < 1, K not a positive
 * multiple of 32, N or ldc not a multiple of 4, ldc < N, or a matrix of more
 * than 2^31 elements.  PAB_EDEVICE: launch failed.
 */
int pab_linear(int M, int N, int K, const void *A, const void *W, const void *bias, void *C, long long ldc,
               void *hip_stream);

/*
 * The paper broadcasts the output of the whole attention MODULE, so that a
 * reused step also skips what surrounds the attention operation (the workflow
 * of App. B.6: the hidden states are projected to queries, keys and values,
 * queries and keys are normalised and given their position embedding, the
 * attention operation runs, and its result goes through the output
 * projection; App. B.5 lists the parts it times: layernorm1, modulate, qkv
 * proj, layernorm2, pos emb, attn, o proj).  The three calls below are that module
 * with its output as the cached object; they use the same context, schedule
 * and cache slots as pab_attention (a slot holds [T, S, C], C = heads *
 * head_dim, the same bytes as an attention output).  bf16 only.
 *
 * Weights of one module: device pointers, bf16, dense.
 *   spatial / temporal:  h = LayerNorm_C(x) * (1 + scale) + shift          shift, scale [C]
 *                        [q | k | v] = h w_qkv^T + b_qkv                    w_qkv [3C, C], b_qkv [3C] or NULL,
 *                                                                           each of q, k, v laid out [heads, D]
 *                        q, k = LayerNorm_D(.) * gamma + beta               gamma_q, beta_q, gamma_k, beta_k [D]
 *                        temporal only: rotary embedding of q, k by the frame index (pairs (2i, 2i+1),
 *                        angle t * 10000^(-2i/D))
 *                        y = attention(q, k, v) w_o^T + b_o                 w_o [C, C], b_o [C] or NULL
 *   cross:               q = x w_qkv^T + b_qkv                              w_qkv [C, C], b_qkv [C] or NULL
 *                        [k | v] = text w_kv^T + b_kv                       w_kv [2C, C], b_kv [2C] or NULL
 *                        y = attention(q, k, v) w_o^T + b_o                 (shift .. beta_k unused)
 * LayerNorms use the biased variance and eps = 1e-6.  C must be a multiple
 * of 32 and at most 2048.
 */
typedef struct pab_module_weights {
  const void *shift, *scale;
  const void *w_qkv, *b_qkv;
  const void *gamma_q, *beta_q, *gamma_k, *beta_k;
  const void *w_kv, *b_kv;
  const void *w_o, *b_o;
} pab_module_weights;

/*
 * Bytes of device scratch a computed module call of `cfg` needs (four planes
 * of max(T*S, L) * C bf16 elements, each rounded up to 256 bytes): the
 * modulated input / attention output, q, k and v.  The caller allocates it
 * once; calls on one stream may share it.  0 if cfg is NULL or invalid.
 */
size_t pab_module_scratch_bytes(const pab_config *cfg);

/*
 * One module, no schedule and no cache: x [T, S, C] (and text [L, C] for
 * cross attention) -> out [T, S, C], five kernel launches (four for cross)
 * on `hip_stream`.  `scratch` must be 256-byte aligned and at least
 * pab_module_scratch_bytes() of the same shape long.
 * PAB_EINVAL: bad kind / shape / head_dim, C not a multiple of 32 or > 2048,
 * NULL or misaligned x / out / scratch / a weight the kind needs, text missing
 * for cross.  PAB_ENOMEM: scratch too small.  PAB_EDEVICE: a launch failed.
 */
int pab_module_compute(int kind, int T, int S, int L, int heads, int head_dim, const void *x, const void *text,
                       const pab_module_weights *w, void *scratch, size_t scratch_bytes, void *out,
                       void *hip_stream);

/*
 * pab_module_compute for callers that cannot allocate device memory (code
 * under HIP graph capture, serving loops and harnesses that forbid it): the
 * same module with the same kernels, its scratch taken from an array inside
 * the library (pab_module_static_scratch_bytes() = 16 MiB per GPU that the
 * library runs on, held until the process ends) instead of from the caller.
 * Allocates nothing and frees nothing; x, text, weights and out are still the
 * caller's.  Shapes whose four scratch planes (each max(T*S, L) * heads *
 * head_dim bf16 elements, rounded up to 256 bytes) exceed the array are
 * refused with PAB_ENOMEM: use pab_module_compute for those.  All calls on one
 * GPU share that GPU's array, whose planes are written in full before they
 * are read within a call: calls that follow each other on one stream need no
 * clearing in between, calls that overlap on one GPU (two streams, two
 * threads) race.  Other errors as pab_module_compute, plus PAB_EDEVICE if the
 * array's address cannot be obtained.
 */
size_t pab_module_static_scratch_bytes(void);
int pab_module_compute_static(int kind, int T, int S, int L, int heads, int head_dim, const void *x,
                              const void *text, const pab_module_weights *w, void *out, void *hip_stream);

/*
 * pab_attention at module level (paper Sec. 2.3, Eq. 1 with the module output
 * as Y): on a computed step runs the module into cache slot (block, kind), on
 * a reused step launches nothing and reads nothing (x, text, w, scratch may be
 * NULL).  *out, return value and errors as pab_attention, plus those of
 * pab_module_compute; PAB_EINVAL if the context's dtype is not bf16.
 */
int pab_module_attention(pab_ctx *ctx, int block, int kind, int step, const void *x, const void *text,
                         const pab_module_weights *w, void *scratch, size_t scratch_bytes, void *hip_stream,
                         const void **out);

/*
 * MLP broadcast.  The paper applies the same idea to the MLP modules of a few
 * blocks (Sec. 2.3, last sentence; App. A.2.2, table of MLP broadcast
 * configurations; App. B.2): the output computed at each listed starting
 * step is retained and handed to the following range-1 steps; only blocks
 * block_lo..block_hi take part; every other (block, step) is computed.
 *
 * pab_mlp_schedule / pab_mlp_source_step: the decision and the step whose
 * output is delivered (host, pure).  start_steps: n_starts step indices
 * (0-based, denoising order).  PAB_EINVAL: negative step / block / start,
 * range < 1, NULL list with n_starts > 0.
 */
int pab_mlp_schedule(int step, int block, const int *start_steps, int n_starts, int range, int block_lo,
                     int block_hi);
int pab_mlp_source_step(int step, int block, const int *start_steps, int n_starts, int range, int block_lo,
                        int block_hi);

/*
 * The table gives the starting points as diffusion timesteps (1000 = start of
 * denoising).  Maps them onto a sampler's timestep list (n_steps values that
 * never increase): start_steps[i] = first step whose timestep is not above
 * start_timesteps[i], or -1 if there is none.  Returns how many were found.
 */
int pab_steps_from_timesteps(const double *timesteps, int n_steps, const double *start_timesteps, int n_starts,
                             int *start_steps);

/*
 * The MLP module: h = LayerNorm_C(x) * (1 + scale) + shift; u = gelu(h w1^T +
 * b1) with GELU in its tanh form; y = u w2^T + b2.  Device pointers, bf16,
 * dense: shift, scale [hidden]; w1 [inner, hidden]; b1 [inner] or NULL;
 * w2 [hidden, inner]; b2 [hidden] or NULL.
 */
typedef struct pab_mlp_weights {
  const void *shift, *scale;
  const void *w1, *b1;
  const void *w2, *b2;
} pab_mlp_weights;

/* Scratch of one MLP call: h [n_tok, hidden] and u [n_tok, inner], each rounded up to 256 bytes. */
size_t pab_mlp_scratch_bytes(long long n_tok, int hidden, int inner);

/*
 * One MLP module, no schedule and no cache: x [n_tok, hidden] -> out
 * [n_tok, hidden], three kernel launches on `hip_stream`.
 * PAB_EINVAL: NULL / misaligned pointers (x, out 16 bytes; scratch 256),
 * hidden not a multiple of 32 or > 2048, inner not a multiple of 32, a missing
 * weight.  PAB_ENOMEM: scratch too small.  PAB_EDEVICE: launch failed.
 */
int pab_mlp_compute(long long n_tok, int hidden, int inner, const void *x, const pab_mlp_weights *w, void *scratch,
                    size_t scratch_bytes, void *out, void *hip_stream);

/* One run of MLP broadcasting: shapes, the schedule above, and a cache slot
 * [n_tok, hidden] for each participating block. */
typedef struct pab_mlp_config {
  int n_blocks, n_steps;
  long long n_tok;
  int hidden, inner;
  int n_starts, range;
  int block_lo, block_hi;
} pab_mlp_config;
typedef struct pab_mlp_ctx pab_mlp_ctx;

/* Bytes of the caller-owned cache: one slot per block in [block_lo, min(block_hi, n_blocks-1)]; 0 if invalid or none. */
size_t pab_mlp_workspace_bytes(const pab_mlp_config *cfg);
/* As pab_create: workspace 256-byte aligned, at least pab_mlp_workspace_bytes long (may be NULL if that is 0).
 * PAB_EINVAL also when two different starting steps are closer than `range`: the later one would fall among the
 * reused steps of the earlier one, and the steps after it would name a source that is never computed. */
int pab_mlp_create(const pab_mlp_config *cfg, const int *start_steps, void *workspace, size_t workspace_bytes,
                   pab_mlp_ctx **out);
int pab_mlp_reset(pab_mlp_ctx *ctx);
/*
 * One MLP call of the denoising loop.  Computed: runs the module; the output
 * goes to the block's cache slot if the block takes part, else to `y` (which
 * must then be given).  Reused: launches nothing, reads nothing.  *out is the
 * device pointer of the output either way.  Returns the decision or a
 * negative status: as pab_attention, plus PAB_ESTATE if the slot does not hold
 * the step the schedule wants to reuse.
 */
int pab_mlp(pab_mlp_ctx *ctx, int block, int step, const void *x, const pab_mlp_weights *w, void *scratch,
            size_t scratch_bytes, void *y, void *hip_stream, const void **out);
long long pab_mlp_launch_count(const pab_mlp_ctx *ctx);
/* Device pointer of the cache slot of a participating block (block_lo <= block
 * <= block_hi), NULL for any other block or a NULL ctx.  Borrowed, read-only. */
const void *pab_mlp_slot_ptr(const pab_mlp_ctx *ctx, int block);
int pab_mlp_destroy(pab_mlp_ctx *ctx);

/* Computed calls issued through ctx since pab_create / the last pab_reset: one
 * per call of pab_attention / pab_module_attention that the schedule decided
 * to compute (an operation-level call is one kernel launch, a module-level
 * call four or five); equals the schedule's number of computed steps.  -1 if
 * ctx is NULL. */
long long pab_launch_count(const pab_ctx *ctx);

/* Device pointer of slot (block, kind) without touching any state; NULL if the block has no such kind. */
const void *pab_slot_ptr(const pab_ctx *ctx, int block, int kind);

/* Free the host-side context (the workspace stays the caller's). */
int pab_destroy(pab_ctx *ctx);

/* Text of the calling thread's last error ("" if none).  Never NULL. */
const char *pab_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PAB_H */
