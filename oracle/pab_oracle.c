/*
 * pab_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 CPU statement of what the Pyramid Attention Broadcast hot
 * path computes.  It exists so that the GPU library can be checked against
 * something that is obviously the definition; nothing in the product path may
 * call it.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * link or load this file.  It shares no code with the HIP library.
 *
 * Two things are defined here:
 *
 *  1. The broadcast schedule (paper Sec. 2.3, Eq. 1): an attention kind is
 *     computed at a step t, its output Y*_t is repeated for the rest of the
 *     "broadcast range", then computed again at t-n, and so on; broadcasting
 *     happens only inside the stable middle segment of the diffusion process
 *     (Sec. 2.2, Sec. 2.3; App. A.2.1 gives the segment per model).
 *     Readings taken where the paper is silent: the range n is a period (one
 *     compute followed by n-1 repeats, as the subscripts t -> t-n of Eq. 1
 *     say); the period is anchored at the first step of the segment (every
 *     run of Eq. 1 opens with F(X_t)); the segment [lo, hi] is inclusive and
 *     steps are counted 0-based in denoising order; outside it every step is
 *     computed.
 *
 *  2. The attention operation whose output is broadcast (Sec. 2.1: spatial
 *     attention among tokens of one frame, temporal attention across frames
 *     at one position, cross attention from video tokens to text tokens).
 *     The paper uses the standard transformer attention, so this is the plain
 *     definition softmax(Q K^T / sqrt(D)) V, no mask, written with the usual
 *     max subtraction.  One strided routine serves the three kinds: the kind
 *     only decides which axis of the activation tensor is "batch" and which
 *     is "sequence".
 *
 *  3. The mapping of a broadcast window given in diffusion timesteps
 *     (App. A.2.1) onto the step indices of a sampler's timestep list.
 *
 * parity unpinned: nothing the paper prints fixes the phase of the period,
 * the inclusiveness of the segment ends, or the inclusiveness of a timestep
 * window's ends (readings above and at pab_oracle_window); everything else
 * here is pinned by the CPU tests.
 */
#include <math.h>
#include <stdlib.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* decision codes */
#define ORACLE_COMPUTE 0
#define ORACLE_REUSE 1
#define ORACLE_BAD (-1)

/*
 * Eq. 1.  step: 0-based index in denoising order.  [lo, hi]: inclusive
 * segment in which broadcasting is active.  n: broadcast range (period).
 * Returns ORACLE_COMPUTE, ORACLE_REUSE, or ORACLE_BAD for arguments that have
 * no meaning (negative step, n < 1, lo > hi).
 */
int pab_oracle_schedule(long step, long lo, long hi, long n)
{
    if (step < 0 || n < 1 || lo > hi) return ORACLE_BAD;
    if (step < lo) return ORACLE_COMPUTE;      /* before the stable segment */
    if (step > hi) return ORACLE_COMPUTE;      /* after the stable segment  */
    if ((step - lo) % n == 0) return ORACLE_COMPUTE; /* F(X_t) opens a run  */
    return ORACLE_REUSE;                       /* Y*_t repeated             */
}

/*
 * The step whose output is delivered at `step`: the step itself when it is a
 * computed one, else the computed step that opened the current run of Eq. 1.
 * Returns -1 on meaningless arguments.
 */
long pab_oracle_source_step(long step, long lo, long hi, long n)
{
    int dec = pab_oracle_schedule(step, lo, hi, n);
    if (dec == ORACLE_BAD) return -1;
    if (dec == ORACLE_COMPUTE) return step;
    return lo + n * ((step - lo) / n);
}

/*
 * The paper gives broadcast windows as diffusion timesteps, written
 * [t_start - t_end] on a scale where 1000 is the beginning of denoising and 0
 * its end (App. A.2.1, table of attention broadcast configurations).  A
 * sampler visits a list of timesteps, one per step, that never increases.
 * Step s lies in the window iff t_end <= timesteps[s] <= t_start (both ends
 * taken as inclusive: the paper does not say).  Marks every step, then
 * reports how many are inside and the first and last of them.
 * Returns the count (0: *lo and *hi untouched), or -1 on meaningless
 * arguments (n_steps < 1, t_start < t_end, a timestep list that increases).
 */
long pab_oracle_window(const double *timesteps, long n_steps, double t_start,
                       double t_end, long *lo, long *hi)
{
    long s, count = 0, first = -1, last = -1;
    if (!timesteps || n_steps < 1 || t_start < t_end) return -1;
    for (s = 1; s < n_steps; ++s)
        if (timesteps[s] > timesteps[s - 1]) return -1;
    for (s = 0; s < n_steps; ++s) {
        int inside = timesteps[s] <= t_start && timesteps[s] >= t_end;
        if (!inside) continue;
        if (first < 0) first = s;
        last = s;
        ++count;
    }
    if (count > 0) { *lo = first; *hi = last; }
    return count;
}

/*
 * Broadcast schedule of the MLP modules (App. A.2.2, table of MLP broadcast
 * configurations; App. B.2 for the reason): the output computed at each of a
 * few listed starting steps is retained and handed to the following steps of
 * its broadcast range n, i.e. to the n-1 steps after the starting step; only
 * blocks block_lo..block_hi take part.  Everything else is computed.
 * `starts` are step indices (0-based, denoising order).  Written as the
 * definition: look at every start in turn.
 * Returns ORACLE_COMPUTE / ORACLE_REUSE and, through *src (may be NULL), the
 * step whose output is delivered; ORACLE_BAD on meaningless arguments.
 */
int pab_oracle_mlp_schedule(long step, long block, const long *starts, long n_starts,
                            long n, long block_lo, long block_hi, long *src)
{
    long i;
    if (step < 0 || block < 0 || n < 1 || n_starts < 0 || (n_starts > 0 && !starts))
        return ORACLE_BAD;
    if (src) *src = step;
    if (block < block_lo || block > block_hi) return ORACLE_COMPUTE;
    for (i = 0; i < n_starts; ++i) {
        if (starts[i] < 0) return ORACLE_BAD;
        if (step > starts[i] && step <= starts[i] + (n - 1)) {
            if (src) *src = starts[i];
            return ORACLE_REUSE;
        }
    }
    return ORACLE_COMPUTE;
}

/*
 * softmax(Q K^T / sqrt(D)) V for n_batch x n_head independent problems.
 *
 * q, o: sq query rows; k, v: sk key rows; each row has d contiguous fp64
 * values.  Element (b, i, h, e) of a tensor lives at
 *     base[b * st[0] + i * st[1] + h * st[2] + e]
 * with st given in elements.  For each query row i:
 *     s_j = (q_i . k_j) / sqrt(d)
 *     m   = max_j s_j
 *     p_j = exp(s_j - m)
 *     o_i = (sum_j p_j v_j) / (sum_j p_j)
 * sk == 0 or sq == 0 or d == 0 writes nothing and returns 0.
 * n_threads <= 0 means "whatever OpenMP picks".  Returns the number of
 * threads used, or -1 if scratch memory cannot be had.
 */
int pab_oracle_attention(const double *q, const double *k, const double *v,
                         double *o, long n_batch, long n_head, long sq,
                         long sk, long d, const long *q_st, const long *k_st,
                         const long *v_st, const long *o_st, int n_threads)
{
    int used = 1;
    int failed = 0;
    if (n_batch <= 0 || n_head <= 0 || sq <= 0 || sk <= 0 || d <= 0) return 0;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const long n_prob = n_batch * n_head;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif

#pragma omp parallel
    {
        double *p = (double *)malloc((size_t)sk * sizeof(double));
        if (!p) {
#pragma omp atomic write
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (long bh = 0; bh < n_prob; ++bh) {
            for (long i = 0; i < sq; ++i) {
                if (!p) continue;
                const long b = bh / n_head, h = bh % n_head;
                const double *qi = q + b * q_st[0] + i * q_st[1] + h * q_st[2];
                double m = -INFINITY;
                for (long j = 0; j < sk; ++j) {
                    const double *kj = k + b * k_st[0] + j * k_st[1] + h * k_st[2];
                    double dot = 0.0;
                    for (long e = 0; e < d; ++e) dot += qi[e] * kj[e];
                    p[j] = dot * inv_sqrt_d;
                    if (p[j] > m) m = p[j];
                }
                double denom = 0.0;
                for (long j = 0; j < sk; ++j) {
                    p[j] = exp(p[j] - m);
                    denom += p[j];
                }
                double *oi = o + b * o_st[0] + i * o_st[1] + h * o_st[2];
                for (long e = 0; e < d; ++e) oi[e] = 0.0;
                for (long j = 0; j < sk; ++j) {
                    const double *vj = v + b * v_st[0] + j * v_st[1] + h * v_st[2];
                    for (long e = 0; e < d; ++e) oi[e] += p[j] * vj[e];
                }
                for (long e = 0; e < d; ++e) oi[e] /= denom;
            }
        }
        free(p);
    }
    return failed ? -1 : used;
}
