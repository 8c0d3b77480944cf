/*
 * gaf_oracle.c -- reference (CPU, fp64) implementation of Gradient Agreement
 * Filtering's aggregation step.
 *
 * THIS IS TEST INFRASTRUCTURE. It is slow on purpose, shares no code with the
 * HIP library, and must never be reached from the product path. Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What it follows:
 *   - cosine distance between two vectors: Eq. 4 of the paper (Sec. 3.1),
 *     D_c(x, y) = 1 - x.y / (|x| |y|), range [0, 2] (Sec. 1).
 *   - the filter: Algorithm 1, the part from "g <- seed gradient, c <- 1" to
 *     "g_GAF <- g / c" (Sec. 3.1 prose: distance is taken against the running
 *     SUM of accepted micro-gradients; accept iff D_c <= tau; an accepted
 *     gradient is added to the sum and the counter is incremented).
 *   - the result: Eq. 5, g_GAF = g / c.
 *   - plain averaging (Eq. 2) is what the filter must reduce to when every
 *     gradient is admitted (tau = 2, Sec. 4.1).
 *
 * Readings taken where the paper is silent (all restated in the design notes):
 *   - the seed is the FIRST gradient of the sequence handed in; the remaining
 *     ones are visited in array order (the paper samples the seed at random and
 *     leaves the order open; both are the caller's choice here);
 *   - the seed's own distance is reported as 0 and its mask entry as 1;
 *   - the normalisation g / c happens once, after all gradients were visited
 *     (the listing's indentation would put it inside the loop; the prose and
 *     Eq. 5 put it after);
 *   - if either vector has zero norm the distance is defined as exactly 1
 *     ("no agreement information");
 *   - no clamping of D to [0, 2]; a NaN distance fails "D <= tau" and is
 *     therefore rejected;
 *   - |x| |y| is formed as sqrt(x.x) * sqrt(y.y), two square roots.
 *
 * All sums are plain left-to-right fp64 sums. With OpenMP the index range is
 * split statically between threads (a "reduction(+)" clause); this changes
 * the summation order at the 1e-16 level only and nothing else.
 *
 * Input element types: 0 = IEEE binary32, 1 = bfloat16 (upper 16 bits of a
 * binary32). Both widen to fp64 exactly.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static inline double widen(const void *v, size_t p, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)v)[p];
    uint32_t bits = (uint32_t)((const uint16_t *)v)[p] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. 4 from the three inner products. */
double oracle_distance_from_sums(double xy, double xx, double yy)
{
    if (xx == 0.0 || yy == 0.0)
        return 1.0;
    return 1.0 - xy / (sqrt(xx) * sqrt(yy));
}

/* Eq. 4 between two stored vectors x and y of length P. */
double oracle_cosine_distance(const void *x, const void *y, size_t P, int dtype)
{
    double xy = 0.0, xx = 0.0, yy = 0.0;
#pragma omp parallel for reduction(+ : xy, xx, yy) schedule(static)
    for (size_t p = 0; p < P; ++p) {
        double a = widen(x, p, dtype), b = widen(y, p, dtype);
        xy += a * b;
        xx += a * a;
        yy += b * b;
    }
    return oracle_distance_from_sums(xy, xx, yy);
}

/*
 * One visit of Algorithm 1's inner loop. (g, *c) is the running sum and the
 * counter, carried by the caller. *c == 0 means "nothing seen yet": g_i then
 * becomes the seed (g <- g_i, c <- 1, distance 0, accepted).
 * tau is compared in fp64.
 */
int oracle_gaf_step(double *g, int32_t *c, const void *g_i, size_t P, int dtype,
                    double tau, double *dist, uint8_t *accepted)
{
    if (!g || !c || !g_i || !dist || !accepted || *c < 0)
        return 1;
    if (*c == 0) {
#pragma omp parallel for schedule(static)
        for (size_t p = 0; p < P; ++p)
            g[p] = widen(g_i, p, dtype);
        *c = 1;
        *dist = 0.0;
        *accepted = 1;
        return 0;
    }
    double gig = 0.0, gg = 0.0, gigi = 0.0;
#pragma omp parallel for reduction(+ : gig, gg, gigi) schedule(static)
    for (size_t p = 0; p < P; ++p) {
        double a = g[p], b = widen(g_i, p, dtype);
        gig += b * a;
        gg += a * a;
        gigi += b * b;
    }
    double D = oracle_distance_from_sums(gig, gg, gigi);
    *dist = D;
    if (D <= tau) {
#pragma omp parallel for schedule(static)
        for (size_t p = 0; p < P; ++p)
            g[p] += widen(g_i, p, dtype);
        *c += 1;
        *accepted = 1;
    } else {
        *accepted = 0;
    }
    return 0;
}

/*
 * The whole aggregation of one macrobatch: grads[0] seeds, grads[1..N-1] are
 * visited in order, out = g / c (Eq. 5). out has P doubles; mask and dist
 * have N entries; *count receives c.
 */
int oracle_gaf_aggregate(const void *const *grads, int N, size_t P, int dtype,
                         double tau, double *out, uint8_t *mask, double *dist,
                         int32_t *count)
{
    if (!grads || N < 1 || !out || !mask || !dist || !count)
        return 1;
    int32_t c = 0;
    for (int i = 0; i < N; ++i) {
        int rc = oracle_gaf_step(out, &c, grads[i], P, dtype, tau, &dist[i], &mask[i]);
        if (rc)
            return rc;
    }
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < P; ++p)
        out[p] = out[p] / (double)c;
    *count = c;
    return 0;
}

/* Eq. 2: the unfiltered mean of all N micro-gradients. */
int oracle_plain_average(const void *const *grads, int N, size_t P, int dtype, double *out)
{
    if (!grads || N < 1 || !out)
        return 1;
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < P; ++p) {
        double s = 0.0;
        for (int i = 0; i < N; ++i)
            s += widen(grads[i], p, dtype);
        out[p] = s / (double)N;
    }
    return 0;
}

/*
 * All-pairs cosine distances (Eq. 4 applied to every pair), the diagnostic the
 * paper logs between micro-gradients (Fig. 1c/d). D is N x N row-major,
 * symmetric, with an exactly zero diagonal. G (nullable) receives the N x N
 * matrix of inner products.
 */
int oracle_gaf_pairwise(const void *const *grads, int N, size_t P, int dtype, double *D, double *G)
{
    if (!grads || N < 1 || !D)
        return 1;
    double *gram = (double *)malloc(sizeof(double) * (size_t)N * (size_t)N);
    if (!gram)
        return 2;
    for (int i = 0; i < N; ++i) {
        for (int j = i; j < N; ++j) {
            double s = 0.0;
            const void *x = grads[i], *y = grads[j];
#pragma omp parallel for reduction(+ : s) schedule(static)
            for (size_t p = 0; p < P; ++p)
                s += widen(x, p, dtype) * widen(y, p, dtype);
            gram[(size_t)i * N + j] = s;
            gram[(size_t)j * N + i] = s;
        }
    }
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j)
            D[(size_t)i * N + j] = (i == j) ? 0.0
                : oracle_distance_from_sums(gram[(size_t)i * N + j], gram[(size_t)i * N + i],
                                            gram[(size_t)j * N + j]);
    if (G)
        memcpy(G, gram, sizeof(double) * (size_t)N * (size_t)N);
    free(gram);
    return 0;
}

/*
 * Order-indifferent variant (Sec. 3.1, last paragraph; the item on order
 * indifference under future research): every micro-gradient acts as the seed in turn, the
 * others are visited in ring order behind it (s, s+1, .., N-1, 0, .., s-1),
 * and the run with the largest agreement is the one that is kept.
 * Readings: "agreement" = number of accepted gradients c; ties go to the
 * lowest seed index. Outputs are indexed by ORIGINAL gradient index: mask[i],
 * and dist[i] = the distance of g_i when it was visited in the winning run
 * (0 for the seed). counts_all (nullable, N entries) receives c of every run.
 */
int oracle_gaf_best_seed(const void *const *grads, int N, size_t P, int dtype, double tau,
                         double *out, uint8_t *mask, double *dist, int32_t *count, int32_t *seed,
                         int32_t *counts_all)
{
    if (!grads || N < 1 || !out || !mask || !dist || !count || !seed)
        return 1;
    const void **ring = (const void **)malloc(sizeof(void *) * (size_t)N);
    double *tmp = (double *)malloc(sizeof(double) * P);
    uint8_t *m = (uint8_t *)malloc((size_t)N);
    double *d = (double *)malloc(sizeof(double) * (size_t)N);
    int best = -1, rc = (!ring || !tmp || !m || !d) ? 2 : 0;
    int32_t best_c = 0;
    for (int s = 0; s < N && !rc; ++s) {
        for (int k = 0; k < N; ++k)
            ring[k] = grads[(s + k) % N];
        int32_t c = 0;
        rc = oracle_gaf_aggregate(ring, N, P, dtype, tau, tmp, m, d, &c);
        if (rc)
            break;
        if (counts_all)
            counts_all[s] = c;
        if (c > best_c) {
            best = s;
            best_c = c;
            memcpy(out, tmp, sizeof(double) * P);
            for (int k = 0; k < N; ++k) {
                mask[(s + k) % N] = m[k];
                dist[(s + k) % N] = d[k];
            }
        }
    }
    *count = best_c;
    *seed = best;
    free(ring);
    free(tmp);
    free(m);
    free(d);
    return rc;
}

/*
 * GAF-SGD step: Eq. 6 with the optimizer the experiments name (Sec. 4.1: SGD
 * with momentum, L2 regularisation through a weight decay), and Algorithm 1's
 * skip: if c == 1 neither the parameters nor the optimizer state are touched.
 * Readings: the momentum form is the common heavy-ball one with the decay
 * folded into the gradient,
 *     d = g_GAF + wd * theta;   v <- mu * v + d;   theta <- theta - lr * v,
 * no dampening, no Nesterov look-ahead; v starts at zero.
 * g_gaf is the output of the aggregation, c its count.
 */
int oracle_sgd_step(double *theta, double *v, const double *g_gaf, int32_t c, size_t P, double lr,
                    double mu, double wd)
{
    if (!theta || !v || !g_gaf)
        return 1;
    if (c <= 1)
        return 0;
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < P; ++p) {
        double d = g_gaf[p] + wd * theta[p];
        v[p] = mu * v[p] + d;
        theta[p] = theta[p] - lr * v[p];
    }
    return 0;
}

/*
 * Bucketed GAF (the per-bucket form of the distance listed under future research): the
 * parameter vector is cut into B contiguous buckets [off[b], off[b+1]) and
 * Algorithm 1 runs independently inside each bucket. mask and dist are B x N
 * row-major, count has B entries, out has P entries.
 */
int oracle_gaf_bucketed(const void *const *grads, int N, size_t P, int dtype, double tau, int B,
                        const size_t *off, double *out, uint8_t *mask, double *dist, int32_t *count)
{
    if (!grads || N < 1 || B < 1 || !off || off[0] != 0 || off[B] != P)
        return 1;
    const size_t es = dtype == ORACLE_F32 ? 4 : 2;
    const void **sl = (const void **)malloc(sizeof(void *) * (size_t)N);
    if (!sl)
        return 2;
    int rc = 0;
    for (int b = 0; b < B && !rc; ++b) {
        if (off[b + 1] <= off[b]) {
            rc = 1;
            break;
        }
        for (int i = 0; i < N; ++i)
            sl[i] = (const char *)grads[i] + off[b] * es;
        rc = oracle_gaf_aggregate(sl, N, off[b + 1] - off[b], dtype, tau, out + off[b],
                                  mask + (size_t)b * N, dist + (size_t)b * N, &count[b]);
    }
    free(sl);
    return rc;
}
