/*
 * CPU oracle for the SAR aggregation path -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct fp64 loops written from the paper's
 * equations.  Nothing here is shared with the HIP path and nothing in the
 * product may link or call it; only tests, the smoke check and the bench's
 * cpu_baseline leg use it.
 *
 * Conventions (the paper's notation): an edge j->i carries a message from
 * source j to destination i.  A block is the edge set E_{p,q} of Sec. 3.2 in
 * destination-major CSR: row i of the block lists the partition-local ids j
 * of the sources in V_q that point at destination i in V_p.
 *   indptr  [n_dst+1] int64, indices [nnz] int32
 * Features are row-major doubles; heads are independent and concatenated:
 * Z[n][H][D].  a_r multiplies the destination's z_i, a_l the source's z_j
 * (the vector a of Eq. 3 is [a_r ; a_l] in the order the equation writes
 * z_i || z_j).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/* ---------------------------------------------------------------- Eq. 2 */

/* acc[i,:] += sum over edges j->i of the block of Zq[j,:]   (Alg. 1, the
 * per-block accumulation; the mean's division by |N(i)| happens once, after
 * the last block, in the caller). */
void oracle_spmm_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                       const double* Zq, int64_t F, double* acc)
{
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            const double* z = Zq + (int64_t)indices[e] * F;
            for (int64_t f = 0; f < F; ++f) acc[i * F + f] += z[f];
        }
}

/* Case 1 of Sec. 3.2: the gradient of a sum needs no features.
 * dZq[j,:] += sum over edges j->i of Gs[i,:]  where Gs is the upstream
 * gradient already divided by |N(i)| for the mean. */
void oracle_spmm_bwd_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                           const double* Gs, int64_t F, double* dZq)
{
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            double* d = dZq + (int64_t)indices[e] * F;
            for (int64_t f = 0; f < F; ++f) d[f] += Gs[i * F + f];
        }
}

/* ---------------------------------------------------------------- Eq. 3 */

static double leaky(double u, double slope) { return u > 0.0 ? u : slope * u; }

/* score[n,h] = <a[h,:], Z[n,h,:]> : one half of a^T (z_i || z_j). */
void oracle_gat_scores(int64_t n, int64_t H, int64_t D, const double* Z, const double* a,
                       double* score)
{
    for (int64_t v = 0; v < n; ++v)
        for (int64_t h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int64_t d = 0; d < D; ++d) acc += a[h * D + d] * Z[(v * H + h) * D + d];
            score[v * H + h] = acc;
        }
}

/* Pass 1 of the plain softmax: M[i,h] = max over the block's edges of
 * e_{j->i} = LeakyReLU(s_i + t_j); call once per block, M starts at -inf. */
void oracle_gat_rowmax_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                             int64_t H, const double* s, const double* t, double slope, double* M)
{
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            int64_t j = indices[e];
            for (int64_t h = 0; h < H; ++h) {
                double ev = leaky(s[i * H + h] + t[j * H + h], slope);
                if (ev > M[i * H + h]) M[i * H + h] = ev;
            }
        }
}

/* Pass 2: den[i,h] += exp(e - M), num[i,h,:] += exp(e - M) z_j. */
void oracle_gat_sums_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                           int64_t H, int64_t D, const double* Zq, const double* s,
                           const double* t, double slope, const double* M, double* den,
                           double* num)
{
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            int64_t j = indices[e];
            for (int64_t h = 0; h < H; ++h) {
                double ev = leaky(s[i * H + h] + t[j * H + h], slope);
                double w = exp(ev - M[i * H + h]);
                den[i * H + h] += w;
                for (int64_t d = 0; d < D; ++d)
                    num[(i * H + h) * D + d] += w * Zq[(j * H + h) * D + d];
            }
        }
}

/* Chain rule through Eq. 3 for one block (Alg. 2, the per-block body).
 * With alpha = exp(e - L_i) the softmax weight (L = log-sum-exp of e over
 * ALL in-edges of i, every block), G the error w.r.t. the aggregate and
 * delta[i,h] = <G[i,h,:], out[i,h,:]>:
 *   d e   = alpha (<G_i, z_j> - delta_i)
 *   d u   = d e * (1 if u > 0 else slope)
 *   dZq[j]   += alpha G_i + du a_l      (the error E_{p->q} sent to worker q)
 *   dZdst[i] += du a_r
 *   da_l     += du z_j ,  da_r += du z_i        (theta.grad, summed over edges)
 * dZq is this block's own array; dZdst, da_l, da_r accumulate across blocks.
 * ds[i,h] += du and dt[j,h] += du (the gradients of the two score halves)
 * are also returned when the pointers are non-null.
 */
void oracle_gat_bwd_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                          int64_t H, int64_t D, const double* Zdst, const double* Zq,
                          const double* G, const double* s, const double* t, const double* L,
                          const double* delta, const double* a_l, const double* a_r,
                          double slope, double* dZq, double* dZdst, double* da_l, double* da_r,
                          double* ds, double* dt)
{
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            int64_t j = indices[e];
            for (int64_t h = 0; h < H; ++h) {
                const double* gi = G + (i * H + h) * D;
                const double* zj = Zq + (j * H + h) * D;
                const double* zi = Zdst + (i * H + h) * D;
                double u = s[i * H + h] + t[j * H + h];
                double alpha = exp(leaky(u, slope) - L[i * H + h]);
                double c = 0.0;
                for (int64_t d = 0; d < D; ++d) c += gi[d] * zj[d];
                double de = alpha * (c - delta[i * H + h]);
                double du = de * (u > 0.0 ? 1.0 : slope);
                if (ds) ds[i * H + h] += du;
                if (dt) dt[j * H + h] += du;
                for (int64_t d = 0; d < D; ++d) {
                    dZq[(j * H + h) * D + d] += alpha * gi[d] + du * a_l[h * D + d];
                    dZdst[(i * H + h) * D + d] += du * a_r[h * D + d];
                    da_l[h * D + d] += du * zj[d];
                    da_r[h * D + d] += du * zi[d];
                }
            }
        }
}

/* ------------------------------------------------- Sec. 3.2 / Sec. 3.4 */

/* The method itself, step by step: one block arrives, every destination that
 * has an edge in it folds the block's messages into its running state.  The
 * running maximum m is the largest e seen so far; when it grows, the
 * accumulated numerator (acc) and denominator (l) are multiplied by
 * exp(old_max - new_max) before the new terms are added.  State starts at
 * m = -inf, l = 0, acc = 0; destinations with no edge in the block are left
 * untouched.  After the last block the caller divides acc by l. */
void oracle_gat_online_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                             int64_t H, int64_t D, const double* Zq, const double* s,
                             const double* t, double slope, double* m, double* l, double* acc)
{
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            int64_t j = indices[e];
            for (int64_t h = 0; h < H; ++h) {
                double ev = leaky(s[i * H + h] + t[j * H + h], slope);
                double old_max = m[i * H + h];
                if (ev > old_max) {
                    double corr = (old_max == -INFINITY) ? 0.0 : exp(old_max - ev);
                    l[i * H + h] *= corr;
                    for (int64_t d = 0; d < D; ++d) acc[(i * H + h) * D + d] *= corr;
                    m[i * H + h] = ev;
                }
                double w = exp(ev - m[i * H + h]);
                l[i * H + h] += w;
                for (int64_t d = 0; d < D; ++d)
                    acc[(i * H + h) * D + d] += w * Zq[(j * H + h) * D + d];
            }
        }
}

/* ------------------------------------------- the same loops on all host cores
 *
 * For the timed CPU baseline only: the loops above with an OpenMP `parallel
 * for` over the rows that own the results, so that no two threads write the
 * same element.  Forward: over destination rows (each owns its M, den, num).
 * Backward: one loop over destination rows for what a destination owns (ds,
 * dZdst, its share of da_r) and one over the source rows of the transposed
 * index for what a source owns (dZq, dt, its share of da_l); the per-edge
 * coefficient is recomputed in both.  The parameter gradients are summed per
 * thread and added up in thread order.  tests/test_oracle_gat.py holds these
 * against the serial loops.  Without OpenMP the pragmas vanish and the loops
 * run on one core.
 */
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_par_gat_rowmax_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                                 int64_t H, const double* s, const double* t, double slope,
                                 double* M)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            int64_t j = indices[e];
            for (int64_t h = 0; h < H; ++h) {
                double ev = leaky(s[i * H + h] + t[j * H + h], slope);
                if (ev > M[i * H + h]) M[i * H + h] = ev;
            }
        }
}

void oracle_par_gat_sums_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                               int64_t H, int64_t D, const double* Zq, const double* s,
                               const double* t, double slope, const double* M, double* den,
                               double* num)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_dst; ++i)
        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
            int64_t j = indices[e];
            for (int64_t h = 0; h < H; ++h) {
                double ev = leaky(s[i * H + h] + t[j * H + h], slope);
                double w = exp(ev - M[i * H + h]);
                den[i * H + h] += w;
                for (int64_t d = 0; d < D; ++d)
                    num[(i * H + h) * D + d] += w * Zq[(j * H + h) * D + d];
            }
        }
}

/* du of one edge and head, and alpha through *alpha_out (the body of oracle_gat_bwd_block). */
static double edge_du(const double* gi, const double* zj, int64_t D, double u, double Lih,
                      double delta_ih, double slope, double* alpha_out)
{
    double alpha = exp(leaky(u, slope) - Lih);
    double c = 0.0;
    for (int64_t d = 0; d < D; ++d) c += gi[d] * zj[d];
    *alpha_out = alpha;
    return alpha * (c - delta_ih) * (u > 0.0 ? 1.0 : slope);
}

/* What the destinations own: ds[i] += du, dZdst[i] += du a_r, da_r += du z_i. */
void oracle_par_gat_bwd_dst_block(int64_t n_dst, const int64_t* indptr, const int32_t* indices,
                                  int64_t H, int64_t D, const double* Zdst, const double* Zq,
                                  const double* G, const double* s, const double* t,
                                  const double* L, const double* delta, const double* a_r,
                                  double slope, double* dZdst, double* da_r, double* ds)
{
    const int nt = oracle_threads();
    double* part = (double*)calloc((size_t)nt * H * D, sizeof(double));
#pragma omp parallel
    {
#ifdef _OPENMP
        double* mine = part + (size_t)omp_get_thread_num() * H * D;
#else
        double* mine = part;
#endif
#pragma omp for schedule(dynamic, 256)
        for (int64_t i = 0; i < n_dst; ++i)
            for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {
                int64_t j = indices[e];
                for (int64_t h = 0; h < H; ++h) {
                    const double* zi = Zdst + (i * H + h) * D;
                    double alpha;
                    double du = edge_du(G + (i * H + h) * D, Zq + (j * H + h) * D, D,
                                        s[i * H + h] + t[j * H + h], L[i * H + h],
                                        delta[i * H + h], slope, &alpha);
                    ds[i * H + h] += du;
                    for (int64_t d = 0; d < D; ++d) {
                        dZdst[(i * H + h) * D + d] += du * a_r[h * D + d];
                        mine[h * D + d] += du * zi[d];
                    }
                }
            }
    }
    for (int k = 0; k < nt; ++k)
        for (int64_t x = 0; x < H * D; ++x) da_r[x] += part[(size_t)k * H * D + x];
    free(part);
}

/* What the sources own, over the transposed (source-major) index of the block:
 * dZq[j] += alpha G_i + du a_l, dt[j] += du, da_l += du z_j. */
void oracle_par_gat_bwd_src_block(int64_t n_src, const int64_t* t_indptr, const int32_t* t_indices,
                                  int64_t H, int64_t D, const double* Zq, const double* G,
                                  const double* s, const double* t, const double* L,
                                  const double* delta, const double* a_l, double slope,
                                  double* dZq, double* da_l, double* dt)
{
    const int nt = oracle_threads();
    double* part = (double*)calloc((size_t)nt * H * D, sizeof(double));
#pragma omp parallel
    {
#ifdef _OPENMP
        double* mine = part + (size_t)omp_get_thread_num() * H * D;
#else
        double* mine = part;
#endif
#pragma omp for schedule(dynamic, 256)
        for (int64_t j = 0; j < n_src; ++j)
            for (int64_t e = t_indptr[j]; e < t_indptr[j + 1]; ++e) {
                int64_t i = t_indices[e];
                for (int64_t h = 0; h < H; ++h) {
                    const double* gi = G + (i * H + h) * D;
                    const double* zj = Zq + (j * H + h) * D;
                    double alpha;
                    double du = edge_du(gi, zj, D, s[i * H + h] + t[j * H + h], L[i * H + h],
                                        delta[i * H + h], slope, &alpha);
                    dt[j * H + h] += du;
                    for (int64_t d = 0; d < D; ++d) {
                        dZq[(j * H + h) * D + d] += alpha * gi[d] + du * a_l[h * D + d];
                        mine[h * D + d] += du * zj[d];
                    }
                }
            }
    }
    for (int k = 0; k < nt; ++k)
        for (int64_t x = 0; x < H * D; ++x) da_l[x] += part[(size_t)k * H * D + x];
    free(part);
}
