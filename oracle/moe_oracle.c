/*
 * CPU oracle for one GPU's share of a tile-granular MoE layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or
 * call this file; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.  It shares no code with the HIP library.
 *
 * Every function is the plain definition written out: no blocking, no fusion,
 * no reordering.  Inputs arrive as fp32 or as raw bf16 bit patterns (the very
 * values the GPU sees); every dot product is accumulated in double and rounded
 * once on output.
 *
 * What is computed (paper section 2.1: gate -> dispatch -> expert compute ->
 * combine; section 2.3: tiles and ready flags; section 4.1 / Algorithm 1:
 * one fence per group of signals):
 *
 *   route     l[t,e] = sum_i x[t,i] Wg[i,e] + bias[e]; the k largest l[t,.]
 *             in descending order (equal scores: lower expert id first);
 *             w[t,j] = exp(l_j - m) / sum_j' exp(l_j' - m) over the k chosen.
 *   dispatch  stable counting sort of slots s = t*k + j by expert id.
 *   experts   y = (silu(x W1[e]) * (x W3[e])) W2[e], silu(g) = g / (1 + e^-g)
 *             (gated MLP, three matrices: the x6 FLOP factor of section 3.1's
 *             footnote).
 *   combine   out[t] = sum_j w[t,j] * staging[t*k + j].
 *   publish   which (expert, destination, row block, column block) tiles exist,
 *             the flag index of each, and how many fences each signaling mode
 *             issues.
 *
 * Pins (tests/test_oracle_*.py): brute force over all C(E,k) subsets for
 * T <= 8, textbook softmax at k = E, numpy bincount / stable argsort for the
 * permutation, a dense numpy SwiGLU MLP at E = 1, identity experts returning
 * x, and the transfer / fence / message-size / FLOP figures the paper prints.
 * The bf16-faithful mode (section 6.2, "Correctness": the rounding points a
 * bf16 pipeline cannot avoid) is pinned bit for bit by a numpy rebuild that
 * rounds with its own integer arithmetic at each point, and round_bf16 by a
 * table of hand-derived cases (ties to even, carry into the exponent,
 * negative values).
 * End-to-end numeric values of a whole layer: parity unpinned by the paper (it
 * prints no worked example); pinned only through the special cases above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };

/* element i of a tensor stored as fp32 or as raw bf16 bits, as a double */
static inline double ld(const void *p, size_t i, int dt)
{
    if (dt == ORC_F32)
        return (double)((const float *)p)[i];
    uint32_t u = ((uint32_t)((const uint16_t *)p)[i]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* round a float to the nearest bf16 (ties to even), returned as a float */
static inline float round_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) /* inf / nan: truncate */
        u &= 0xffff0000u;
    else
        u = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

/* round_bf16 as tests call it (so that a table of hand-derived cases can pin it) */
float orc_round_bf16(float f)
{
    return round_bf16(f);
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ route */
/*
 * Section 2.1: the gate scores every expert and keeps the top k; the layer
 * output weights the chosen experts.  Scores are softmax-normalised over the k
 * chosen (same as a full softmax renormalised over them: the denominator
 * cancels).  logits / margin may be NULL.  margin[t] is the smallest gap
 * between neighbours among the k+1 largest scores (k if k == E): how far the
 * token is from a different routing decision.
 */
void orc_route(int T, int d, int E, int k, int dt, const void *x, const void *Wg,
               const float *bias, int32_t *idx, float *w, double *logits,
               double *margin)
{
#pragma omp parallel
    {
        double *l = (double *)malloc(sizeof(double) * (size_t)E);
        char *taken = (char *)malloc((size_t)E);
        double *sel = (double *)malloc(sizeof(double) * (size_t)(k + 1));
#pragma omp for schedule(static)
        for (int t = 0; t < T; ++t) {
            for (int e = 0; e < E; ++e) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i)
                    acc += ld(x, (size_t)t * d + i, dt) * ld(Wg, (size_t)i * E + e, dt);
                if (bias)
                    acc += (double)bias[e];
                l[e] = acc;
                if (logits)
                    logits[(size_t)t * E + e] = acc;
            }
            memset(taken, 0, (size_t)E);
            int nsel = (k < E) ? k + 1 : k;
            for (int j = 0; j < nsel; ++j) {
                int best = -1;
                for (int e = 0; e < E; ++e)
                    if (!taken[e] && (best < 0 || l[e] > l[best]))
                        best = e; /* strict >: lower id wins ties */
                taken[best] = 1;
                sel[j] = l[best];
                if (j < k)
                    idx[(size_t)t * k + j] = best;
            }
            double m = sel[0], den = 0.0;
            for (int j = 0; j < k; ++j)
                den += exp(sel[j] - m);
            for (int j = 0; j < k; ++j)
                w[(size_t)t * k + j] = (float)(exp(sel[j] - m) / den);
            if (margin) {
                double g = INFINITY;
                for (int j = 0; j + 1 < nsel; ++j)
                    if (sel[j] - sel[j + 1] < g)
                        g = sel[j] - sel[j + 1];
                margin[t] = g;
            }
        }
        free(l);
        free(taken);
        free(sel);
    }
}

/* --------------------------------------------------------------- dispatch */
/*
 * Section 2.1 step (2) in its local form: group the N = T*k slots by expert.
 * counts[e] = number of slots routed to e; offsets = exclusive scan
 * (offsets[E] = N); perm[p] = slot at sorted position p, slots of one expert
 * in increasing slot order (stable); inv_perm[perm[p]] = p.
 */
void orc_dispatch(int N, int E, const int32_t *idx, int32_t *counts, int32_t *offsets,
                  int32_t *perm, int32_t *inv_perm)
{
    if (E <= 0 || N < 0)
        return;
    for (int e = 0; e < E; ++e)
        counts[e] = 0;
    for (int s = 0; s < N; ++s)
        counts[idx[s]] += 1;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e)
        offsets[e + 1] = offsets[e] + counts[e];
    int32_t *fill = (int32_t *)calloc((size_t)E, sizeof(int32_t));
    for (int s = 0; s < N; ++s) {
        int e = idx[s];
        int p = offsets[e] + fill[e]++;
        perm[p] = s;
        inv_perm[s] = p;
    }
    free(fill);
}

/* x_perm[p,:] = x[perm[p] / k, :] (raw element copy, either dtype) */
void orc_gather(int N, int k, int d, int dt, const void *x, const int32_t *perm, void *x_perm)
{
    size_t esz = (dt == ORC_F32) ? 4 : 2;
    for (int p = 0; p < N; ++p)
        memcpy((char *)x_perm + (size_t)p * d * esz,
               (const char *)x + (size_t)(perm[p] / k) * d * esz, (size_t)d * esz);
}

/* ---------------------------------------------------------------- experts */
/*
 * One row through expert e (section 2.1 step (3), gated form):
 *   g = xrow W1[e], u = xrow W3[e], h = silu(g) * u, y = h W2[e].
 * faithful != 0 mirrors where a bf16 pipeline must round: g, u to fp32,
 * h to bf16, y to fp32 then bf16 -- still in this file's own arithmetic.
 * g, u, h are caller scratch of f doubles; y receives d doubles.
 */
static void expert_row(int d, int f, int dt, const void *x, size_t xrow, const void *W1,
                       const void *W3, const void *W2, int e, int faithful, double *g,
                       double *u, double *h, double *y)
{
    const size_t wbase = (size_t)e * d * f;
    for (int j = 0; j < f; ++j)
        g[j] = u[j] = 0.0;
    for (int i = 0; i < d; ++i) {
        double xi = ld(x, xrow * d + i, dt);
        size_t r = wbase + (size_t)i * f;
        for (int j = 0; j < f; ++j) {
            g[j] += xi * ld(W1, r + j, dt);
            u[j] += xi * ld(W3, r + j, dt);
        }
    }
    for (int j = 0; j < f; ++j) {
        double gj = g[j], uj = u[j];
        if (faithful) {
            gj = (double)(float)gj;
            uj = (double)(float)uj;
        }
        double hj = gj / (1.0 + exp(-gj)) * uj;
        if (faithful)
            hj = (double)round_bf16((float)hj);
        h[j] = hj;
    }
    for (int c = 0; c < d; ++c)
        y[c] = 0.0;
    for (int j = 0; j < f; ++j) {
        double hj = h[j];
        size_t r = (size_t)e * f * d + (size_t)j * d;
        for (int c = 0; c < d; ++c)
            y[c] += hj * ld(W2, r + c, dt);
    }
    if (faithful)
        for (int c = 0; c < d; ++c)
            y[c] = (double)round_bf16((float)y[c]);
}

/*
 * Expert outputs in sorted order: y[p,:] for every sorted position p in
 * [0, N), where row p holds token perm[p] / k and belongs to the expert whose
 * offsets range contains p.  y is fp32 [N, d].
 */
void orc_experts_sorted(int N, int k, int d, int E, int f, int dt, const void *x,
                        const void *W1, const void *W3, const void *W2,
                        const int32_t *offsets, const int32_t *perm, int faithful, float *y)
{
#pragma omp parallel
    {
        double *g = (double *)malloc(sizeof(double) * (size_t)f * 3);
        double *u = g + f, *h = u + f;
        double *yr = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
        for (int p = 0; p < N; ++p) {
            int e = 0;
            while (!(offsets[e] <= p && p < offsets[e + 1]))
                ++e;
            expert_row(d, f, dt, x, (size_t)(perm[p] / k), W1, W3, W2, e, faithful, g, u, h, yr);
            for (int c = 0; c < d; ++c)
                y[(size_t)p * d + c] = (float)yr[c];
        }
        free(g);
        free(yr);
    }
}

/* staging[s,:] = y[inv_perm[s],:]: every expert output row lands in the slot
 * of the token that asked for it (the combine-side layout, section 2.1 (4)) */
void orc_stage(int N, int d, const float *y, const int32_t *inv_perm, float *staging)
{
    for (int s = 0; s < N; ++s)
        memcpy(staging + (size_t)s * d, y + (size_t)inv_perm[s] * d, sizeof(float) * (size_t)d);
}

/* out[t,:] = sum_j w[t,j] * staging[t*k+j,:]  (section 2.1: weighted
 * combination of the selected experts' outputs) */
void orc_combine(int T, int k, int d, const float *staging, const float *w, int faithful,
                 float *out)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j)
                acc += (double)w[(size_t)t * k + j] * (double)staging[((size_t)t * k + j) * d + c];
            out[(size_t)t * d + c] = faithful ? round_bf16((float)acc) : (float)acc;
        }
}

/*
 * The same layer restricted to chosen tokens (for full-size workloads where
 * the whole layer would take minutes): for each listed token t, its k expert
 * outputs (rows of staging, [n_tok*k, d]) and the combined row ([n_tok, d]),
 * straight from the definitions; the permutation cancels out of both.
 */
void orc_forward_tokens(int k, int d, int f, int dt, const void *x, const void *W1,
                        const void *W3, const void *W2, const int32_t *idx, const float *w,
                        int n_tok, const int32_t *tok, int faithful, float *staging_rows,
                        float *out_rows)
{
    int n_rows = n_tok * k;
#pragma omp parallel
    {
        double *g = (double *)malloc(sizeof(double) * (size_t)f * 3);
        double *u = g + f, *h = u + f;
        double *yr = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r) {
            int t = tok[r / k], j = r % k;
            int e = idx[(size_t)t * k + j];
            expert_row(d, f, dt, x, (size_t)t, W1, W3, W2, e, faithful, g, u, h, yr);
            for (int c = 0; c < d; ++c)
                staging_rows[(size_t)r * d + c] = (float)yr[c];
        }
        free(g);
        free(yr);
    }
    for (int n = 0; n < n_tok; ++n) {
        int t = tok[n];
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j)
                acc += (double)w[(size_t)t * k + j] *
                       (double)staging_rows[((size_t)n * k + j) * d + c];
            out_rows[(size_t)n * d + c] = faithful ? round_bf16((float)acc) : (float)acc;
        }
    }
}

/* ---------------------------------------------------------------- publish */
/*
 * Which output tiles get published, and under which flag (sections 2.3 and
 * 4.1).  Token t belongs to destination r = t / (T/R).  Inside expert e the
 * rows of destination r are the contiguous expert-local range [a, b) (the
 * sort is stable and r is monotone in t).  A publish tile is (e, r, row block
 * i, column block c): expert-local rows [i*tile_m, (i+1)*tile_m) cut to
 * [a, b), columns [c*tile_n, (c+1)*tile_n) cut to d.  Flags are numbered
 * destination-major, then expert, then row block, then column block.
 *
 * Outputs: seg_begin[e*R + r] = a (expert-local, 0 for an empty segment) and
 * seg_cnt[e*R + r] = b - a; flag_base[r*E + e]; slot_flag[s] = flag of column
 * block 0 of the tile holding slot s; dest_flag_begin[R+1]; returns the
 * number of flags in use.  fences_per_tile / fences_per_dest: fences issued by the
 * coupled mode (one per publish tile) and by the decoupled mode with one
 * group per destination (one per destination that receives anything).
 */
int64_t orc_publish_plan(int T, int k, int E, int R, int d, int tile_m, int tile_n,
                         const int32_t *idx, const int32_t *offsets, const int32_t *inv_perm,
                         int32_t *seg_begin, int32_t *seg_cnt, int32_t *flag_base,
                         int32_t *slot_flag, int32_t *dest_flag_begin, int64_t *fences_per_tile,
                         int64_t *fences_per_dest)
{
    const int per = T / R;
    const int ncb = (d + tile_n - 1) / tile_n;
    for (int i = 0; i < E * R; ++i) {
        seg_begin[i] = 0x7fffffff;
        seg_cnt[i] = 0;
    }
    for (int s = 0; s < T * k; ++s) {
        int e = idx[s], r = (s / k) / per;
        int q = inv_perm[s] - offsets[e];
        if (q < seg_begin[e * R + r])
            seg_begin[e * R + r] = q;
        seg_cnt[e * R + r] += 1;
    }
    int64_t nflags = 0, nd = 0;
    for (int r = 0; r < R; ++r) {
        dest_flag_begin[r] = (int32_t)nflags;
        for (int e = 0; e < E; ++e) {
            flag_base[r * E + e] = (int32_t)nflags;
            int c = seg_cnt[e * R + r];
            if (c > 0) {
                int a = seg_begin[e * R + r], b = a + c;
                nflags += (int64_t)((b - 1) / tile_m - a / tile_m + 1) * ncb;
            } else {
                seg_begin[e * R + r] = 0;
            }
        }
        if (nflags > dest_flag_begin[r])
            nd += 1;
    }
    dest_flag_begin[R] = (int32_t)nflags;
    for (int s = 0; s < T * k; ++s) {
        int e = idx[s], r = (s / k) / per;
        int q = inv_perm[s] - offsets[e];
        int a = seg_begin[e * R + r];
        slot_flag[s] = flag_base[r * E + e] + (q / tile_m - a / tile_m) * ncb;
    }
    if (fences_per_tile)
        *fences_per_tile = nflags;
    if (fences_per_dest)
        *fences_per_dest = nd;
    return nflags;
}
