/*
 * CPU oracle for DynLP in plain C, float64.  TEST INFRASTRUCTURE ONLY: it exists so that
 * tests, the smoke check and the benchmark's cpu_baseline leg can evaluate the definitions on
 * graphs that are too large for the Python loops.  It shares no code with the GPU library.
 *
 * What each function states:
 *   oracle_itlp_sweep    one Jacobi sweep of Eq. (1): every unlabelled row with d(u) > 0 becomes
 *                        (1/d(u)) sum_v w(u,v) F_v, read from F_in, written to F_out; seed rows
 *                        and isolated rows are copied.
 *   oracle_itlp_solve    repeat the sweep until max_u max_c |F_new - F| <= tol (ItLP).
 *   oracle_neumann_solve x = (I - P_UU)^{-1} b as the limit of x <- b + P_UU x (the series sum_k P_UU^k b of the
 *                        convergence proof), P = D^{-1} W: error bounds for labels that are not yet converged.
 *   oracle_laplacian_cg  the linear system of Eq. (2) in symmetric form, (D - W)_UU X = B, by conjugate gradients
 *                        (for graphs on which the thousands of sweeps of the two iterations above take too long).
 *   oracle_affected_set  V_aff after Step 1 of Alg. 2 for an insertion batch.
 *   oracle_step3         Step 3 of Alg. 2 in synchronous rounds over V_aff.
 *
 * Graph: CSR over n vertices, row_ptr (int64, n+1), col (int32), w (double).  Parallel edges
 * may appear as separate entries (everything is linear in w).  seed_class[u] >= 0 marks a
 * vertex of V^L and gives its class; -1 marks V^U.  F is n x C row-major.
 * The loops over rows are independent (Jacobi), so the OpenMP pragma changes no result.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* F_out[u,:] for one unlabelled row with at least one edge: the weighted mean of Eq. (1). */
static void weighted_mean_row(const int64_t* row_ptr, const int32_t* col, const double* w, int C,
                              const double* F, int64_t u, double* out) {
    double d = 0.0;
    for (int c = 0; c < C; ++c) out[c] = 0.0;
    for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) {
        const double* Fv = F + (int64_t)col[j] * C;
        d += w[j];
        for (int c = 0; c < C; ++c) out[c] += w[j] * Fv[c];
    }
    for (int c = 0; c < C; ++c) out[c] /= d;
}

double oracle_itlp_sweep(int64_t n, const int64_t* row_ptr, const int32_t* col, const double* w, int C,
                         const int32_t* seed_class, const double* F_in, double* F_out) {
    double change = 0.0;
#pragma omp parallel for schedule(dynamic, 1024) reduction(max : change)
    for (int64_t u = 0; u < n; ++u) {
        double* out = F_out + u * C;
        const double* old = F_in + u * C;
        if (seed_class[u] >= 0 || row_ptr[u + 1] == row_ptr[u]) {
            for (int c = 0; c < C; ++c) out[c] = old[c];
            continue;
        }
        weighted_mean_row(row_ptr, col, w, C, F_in, u, out);
        for (int c = 0; c < C; ++c) {
            double r = fabs(out[c] - old[c]);
            if (r > change) change = r;
        }
    }
    return change;
}

/* F is read and overwritten with the result; tmp is caller-provided scratch of n*C doubles. */
int64_t oracle_itlp_solve(int64_t n, const int64_t* row_ptr, const int32_t* col, const double* w, int C,
                          const int32_t* seed_class, double* F, double* tmp, double tol, int64_t max_iter,
                          double* last_change) {
    double* a = F;
    double* b = tmp;
    int64_t it = 0;
    double change = INFINITY;
    while (it < max_iter) {
        change = oracle_itlp_sweep(n, row_ptr, col, w, C, seed_class, a, b);
        double* t = a;
        a = b;
        b = t;
        ++it;
        if (change <= tol) break;
    }
    if (a != F) memcpy(F, a, (size_t)n * C * sizeof(double));
    if (last_change) *last_change = change;
    return it;
}

/*
 * x = sum_k P_UU^k b, i.e. the solution of (I - P_UU) x = b, by the iteration x <- b + P_UU x over the unlabelled
 * rows with d(u) > 0 (P_uv = w(u,v)/d(u); x is 0 on labelled and isolated vertices, which is how P_UU drops their
 * columns).  This is the matrix of the convergence corollary: a label matrix F with residual r = F - (P_UU F + P_UL Y)
 * differs from the fixed point by exactly (I - P_UU)^{-1} r, so |F - F*| <= (I - P_UU)^{-1} |r| row by row, and
 * with b = 1 the largest x_u is ||(I - P_UU)^{-1}||_inf (the largest expected number of steps of the random walk
 * before it meets a labelled vertex).  x is read as the start (zero it for the plain series) and overwritten; tmp is
 * scratch of n doubles.  Stops when max_u |x_new - x| <= tol or after max_iter sweeps; returns the sweeps done.
 * Only meaningful where every unlabelled vertex reaches a labelled one (elsewhere the series diverges).
 */
int64_t oracle_neumann_solve(int64_t n, const int64_t* row_ptr, const int32_t* col, const double* w,
                             const int32_t* seed_class, const double* b, double* x, double* tmp, double tol,
                             int64_t max_iter, double* last_change) {
    double* cur = x;
    double* nxt = tmp;
    int64_t it = 0;
    double change = INFINITY;
    while (it < max_iter) {
        change = 0.0;
#pragma omp parallel for schedule(dynamic, 1024) reduction(max : change)
        for (int64_t u = 0; u < n; ++u) {
            if (seed_class[u] >= 0 || row_ptr[u + 1] == row_ptr[u]) {
                nxt[u] = 0.0;
                continue;
            }
            double d = 0.0, acc = 0.0;
            for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) {
                const int32_t v = col[j];
                d += w[j];
                if (seed_class[v] < 0 && row_ptr[v + 1] > row_ptr[v]) acc += w[j] * cur[v];
            }
            nxt[u] = b[u] + acc / d;
            const double r = fabs(nxt[u] - cur[u]);
            if (r > change) change = r;
        }
        double* t = cur;
        cur = nxt;
        nxt = t;
        ++it;
        if (change <= tol) break;
    }
    if (cur != x) memcpy(x, cur, (size_t)n * sizeof(double));
    if (last_change) *last_change = change;
    return it;
}

/*
 * Solve (D - W)_UU X = B for k right-hand sides at once (X, B: n x k row-major; rows outside U are ignored in B and
 * left untouched in X, which holds the start on entry).  in_U[u] != 0 marks the rows of U; the caller passes the
 * unlabelled vertices that have an edge and are connected to a labelled vertex, on which the matrix is symmetric
 * positive definite.  With B = W_UL Y_L the solution is the harmonic labelling of Eq. (2); with B = D_U b it is
 * (I - P_UU)^{-1} b.  Method: the textbook conjugate-gradient iteration with the diagonal as preconditioner, the k
 * systems advancing in lockstep (each has its own step lengths); a system stops changing once its residual norm
 * is <= rtol times the norm of its right-hand side.  Returns the iterations done; *worst (may be NULL) = the
 * largest relative residual norm left.  Callers check the result with one sweep of the defining iteration.
 */
static void lap_apply(int64_t n, const int64_t* row_ptr, const int32_t* col, const double* w, const uint8_t* in_U,
                      int k, const double* P, double* out) {
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t u = 0; u < n; ++u) {
        if (!in_U[u]) continue;
        double d = 0.0;
        double* o = out + u * k;
        for (int c = 0; c < k; ++c) o[c] = 0.0;
        for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) {
            const int32_t v = col[j];
            d += w[j];
            if (in_U[v])
                for (int c = 0; c < k; ++c) o[c] -= w[j] * P[(int64_t)v * k + c];
        }
        for (int c = 0; c < k; ++c) o[c] += d * P[u * k + c];
    }
}

/* dots[c] = sum over U of a[u][c] * b[u][c] */
static void col_dots(int64_t n, const uint8_t* in_U, int k, const double* a, const double* b, double* dots) {
    for (int c = 0; c < k; ++c) dots[c] = 0.0;
#pragma omp parallel
    {
        double loc[64];
        for (int c = 0; c < k; ++c) loc[c] = 0.0;
#pragma omp for schedule(static)
        for (int64_t u = 0; u < n; ++u) {
            if (!in_U[u]) continue;
            for (int c = 0; c < k; ++c) loc[c] += a[u * k + c] * b[u * k + c];
        }
#pragma omp critical
        for (int c = 0; c < k; ++c) dots[c] += loc[c];
    }
}

int64_t oracle_laplacian_cg(int64_t n, const int64_t* row_ptr, const int32_t* col, const double* w,
                            const uint8_t* in_U, int k, const double* B, double* X, double rtol, int64_t max_iter,
                            double* worst) {
    if (k < 1 || k > 64) return -1;
    const size_t sz = (size_t)(n > 0 ? n : 1) * k;
    double* r = (double*)calloc(sz, sizeof(double));
    double* z = (double*)calloc(sz, sizeof(double));
    double* p = (double*)calloc(sz, sizeof(double));
    double* Ap = (double*)calloc(sz, sizeof(double));
    double* diag = (double*)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
    double rz[64], rz_new[64], pAp[64], bb[64], rr[64], alpha[64], beta[64];
    int live[64];
    for (int64_t u = 0; u < n; ++u)
        for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) diag[u] += w[j];
    /* a system whose right-hand side is zero has the solution zero (the matrix is positive definite): take it
       at once, the relative stopping rule has nothing to measure against there */
    col_dots(n, in_U, k, B, B, bb);
    for (int64_t u = 0; u < n; ++u)
        if (in_U[u])
            for (int c = 0; c < k; ++c)
                if (bb[c] == 0.0) X[u * k + c] = 0.0;
    /* r = B - A X on U; z = r / diag; p = z */
    for (int64_t u = 0; u < n; ++u)
        if (in_U[u])
            for (int c = 0; c < k; ++c) p[u * k + c] = X[u * k + c];
    lap_apply(n, row_ptr, col, w, in_U, k, p, Ap);
    for (int64_t u = 0; u < n; ++u) {
        for (int c = 0; c < k; ++c) {
            const int64_t i = u * k + c;
            if (in_U[u]) {
                r[i] = B[i] - Ap[i];
                z[i] = r[i] / diag[u];
                p[i] = z[i];
            } else {
                r[i] = z[i] = p[i] = 0.0;
            }
        }
    }
    col_dots(n, in_U, k, r, z, rz);
    col_dots(n, in_U, k, r, r, rr);
    int64_t it = 0;
    double left = 0.0;
    for (;;) {
        int any = 0;
        left = 0.0;
        for (int c = 0; c < k; ++c) {
            const double rel = bb[c] > 0.0 ? sqrt(rr[c] / bb[c]) : (rr[c] > 0.0 ? INFINITY : 0.0);
            live[c] = rel > rtol && rz[c] > 0.0;
            if (live[c]) any = 1;
            if (rel > left) left = rel;
        }
        if (!any || it >= max_iter) break;
        lap_apply(n, row_ptr, col, w, in_U, k, p, Ap);
        col_dots(n, in_U, k, p, Ap, pAp);
        for (int c = 0; c < k; ++c) alpha[c] = live[c] && pAp[c] > 0.0 ? rz[c] / pAp[c] : 0.0;
#pragma omp parallel for schedule(static)
        for (int64_t u = 0; u < n; ++u) {
            if (!in_U[u]) continue;
            for (int c = 0; c < k; ++c) {
                const int64_t i = u * k + c;
                X[i] += alpha[c] * p[i];
                r[i] -= alpha[c] * Ap[i];
                z[i] = r[i] / diag[u];
            }
        }
        col_dots(n, in_U, k, r, z, rz_new);
        col_dots(n, in_U, k, r, r, rr);
        for (int c = 0; c < k; ++c) {
            beta[c] = live[c] && rz[c] > 0.0 ? rz_new[c] / rz[c] : 0.0;
            if (live[c]) rz[c] = rz_new[c];
        }
#pragma omp parallel for schedule(static)
        for (int64_t u = 0; u < n; ++u) {
            if (!in_U[u]) continue;
            for (int c = 0; c < k; ++c) {
                const int64_t i = u * k + c;
                if (live[c]) p[i] = z[i] + beta[c] * p[i];
            }
        }
        ++it;
    }
    if (worst) *worst = left;
    free(r);
    free(z);
    free(p);
    free(Ap);
    free(diag);
    return it;
}

/*
 * V_aff for an insertion batch applied to a graph that now has n vertices (CSR already
 * updated): inserted vertices n_old..n-1 and their neighbours, both endpoints of every new
 * edge, and the neighbours of every vertex that has just become a seed; minus seeds and
 * isolated vertices.  flag is n bytes of scratch.  Writes ascending ids to out (capacity n);
 * returns the count.
 */
int64_t oracle_affected_set(int64_t n, const int64_t* row_ptr, const int32_t* col, const int32_t* seed_class,
                            int64_t n_old, int64_t m, const int32_t* eu, const int32_t* ev, int64_t s,
                            const int32_t* new_seed_vertex, uint8_t* flag, int32_t* out) {
    memset(flag, 0, (size_t)n);
    for (int64_t u = n_old; u < n; ++u) {
        flag[u] = 1;
        for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) flag[col[j]] = 1;
    }
    for (int64_t e = 0; e < m; ++e) {
        flag[eu[e]] = 1;
        flag[ev[e]] = 1;
    }
    for (int64_t i = 0; i < s; ++i) {
        int64_t u = new_seed_vertex[i];
        for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) flag[col[j]] = 1;
    }
    int64_t cnt = 0;
    for (int64_t u = 0; u < n; ++u)
        if (flag[u] && seed_class[u] < 0 && row_ptr[u + 1] > row_ptr[u]) out[cnt++] = (int32_t)u;
    return cnt;
}

/*
 * Alg. 2 Step 3.  Round t: for every u in V_aff compute F'_u (weighted mean of the round-start
 * F), commit all of them, then V_aff <- union over {u : change(u) > tol} of {u} U N(u), minus
 * seeds and isolated vertices.  change(u) = max_c |F'_u[c] - F_u[c]|; with decide_fp32 the two
 * rows are rounded to binary32 and the subtraction and comparison are done in binary32 (the
 * precision in which the GPU kernel takes the same decision).  Stops when V_aff is empty or
 * after max_iter rounds.  frontier_sizes / max_changes (capacity cap, may be NULL) receive the
 * first cap rounds.  totals[0] = rows updated, totals[1] = CSR entries traversed.
 * Returns the number of rounds; *remaining = |V_aff| at exit (0 if it emptied).
 */
int64_t oracle_step3(int64_t n, const int64_t* row_ptr, const int32_t* col, const double* w, int C,
                     const int32_t* seed_class, double* F, const int32_t* frontier0, int64_t n0, double tol,
                     int64_t max_iter, int decide_fp32, int64_t* frontier_sizes, double* max_changes,
                     int64_t cap, int64_t* totals, int64_t* remaining) {
    int32_t* A = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    uint8_t* flag = (uint8_t*)calloc((size_t)(n > 0 ? n : 1), 1);
    uint8_t* big = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
    double* stage = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * C);
    int64_t na = n0;
    memcpy(A, frontier0, sizeof(int32_t) * (size_t)n0);
    int64_t rounds = 0, rows = 0, edges = 0;
    const float tolf = (float)tol;
    while (na > 0 && rounds < max_iter) {
        double mx = 0.0;
#pragma omp parallel for schedule(dynamic, 256) reduction(max : mx)
        for (int64_t i = 0; i < na; ++i) {
            int64_t u = A[i];
            double* out = stage + i * C;
            weighted_mean_row(row_ptr, col, w, C, F, u, out);
            double r = 0.0;
            if (decide_fp32) {
                float rf = 0.0f;
                for (int c = 0; c < C; ++c) {
                    float df = fabsf((float)out[c] - (float)F[u * C + c]);
                    if (df > rf) rf = df;
                }
                big[i] = rf > tolf;
                r = rf;
            } else {
                for (int c = 0; c < C; ++c) {
                    double dd = fabs(out[c] - F[u * C + c]);
                    if (dd > r) r = dd;
                }
                big[i] = r > tol;
            }
            if (r > mx) mx = r;
        }
        for (int64_t i = 0; i < na; ++i) {
            int64_t u = A[i];
            memcpy(F + u * C, stage + i * C, sizeof(double) * C);
            rows += 1;
            edges += row_ptr[u + 1] - row_ptr[u];
            if (big[i]) {
                flag[u] = 1;
                for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) flag[col[j]] = 1;
            }
        }
        if (rounds < cap) {
            if (frontier_sizes) frontier_sizes[rounds] = na;
            if (max_changes) max_changes[rounds] = mx;
        }
        int64_t nn = 0;
        for (int64_t u = 0; u < n; ++u) {
            if (flag[u]) {
                flag[u] = 0;
                if (seed_class[u] < 0 && row_ptr[u + 1] > row_ptr[u]) A[nn++] = (int32_t)u;
            }
        }
        na = nn;
        ++rounds;
    }
    if (totals) {
        totals[0] = rows;
        totals[1] = edges;
    }
    if (remaining) *remaining = na;
    free(A);
    free(flag);
    free(big);
    free(stage);
    return rounds;
}

/*
 * Alg. 2 Step 1, components of the sparsified batch-internal graph G'(V',E'): V' = the k inserted
 * vertices n_old..n_old+k-1; E' = the batch edges with both endpoints in V' and weight > tau
 * (each listed edge tested on its own weight).  comp[i] (i = batch-local id) = index of i's
 * component, components numbered by ascending smallest member.  Breadth-first search over an
 * adjacency list built by counting.  *kept (may be NULL) = |E'|.  Returns the number of
 * components.
 */
int64_t oracle_components(int64_t n_old, int64_t k, int64_t m, const int32_t* eu, const int32_t* ev,
                          const double* ew, double tau, int32_t* comp, int64_t* kept) {
    int64_t* start = (int64_t*)calloc((size_t)k + 2, sizeof(int64_t));
    int64_t ne = 0;
    for (int64_t e = 0; e < m; ++e) {
        int64_t a = eu[e] - n_old, b = ev[e] - n_old;
        if (a >= 0 && a < k && b >= 0 && b < k && ew[e] > tau) {
            start[a + 1]++;
            start[b + 1]++;
            ne++;
        }
    }
    for (int64_t i = 0; i < k; ++i) start[i + 1] += start[i];
    int32_t* nbr = (int32_t*)malloc(sizeof(int32_t) * (size_t)(2 * ne + 1));
    int64_t* fill = (int64_t*)malloc(sizeof(int64_t) * (size_t)(k + 1));
    memcpy(fill, start, sizeof(int64_t) * (size_t)(k + 1));
    for (int64_t e = 0; e < m; ++e) {
        int64_t a = eu[e] - n_old, b = ev[e] - n_old;
        if (a >= 0 && a < k && b >= 0 && b < k && ew[e] > tau) {
            nbr[fill[a]++] = (int32_t)b;
            nbr[fill[b]++] = (int32_t)a;
        }
    }
    int32_t* queue = (int32_t*)malloc(sizeof(int32_t) * (size_t)(k + 1));
    for (int64_t i = 0; i < k; ++i) comp[i] = -1;
    int64_t count = 0;
    for (int64_t s = 0; s < k; ++s) {
        if (comp[s] >= 0) continue;
        int64_t head = 0, tail = 0;
        queue[tail++] = (int32_t)s;
        comp[s] = (int32_t)count;
        while (head < tail) {
            int64_t u = queue[head++];
            for (int64_t j = start[u]; j < start[u + 1]; ++j) {
                int32_t v = nbr[j];
                if (comp[v] < 0) {
                    comp[v] = (int32_t)count;
                    queue[tail++] = v;
                }
            }
        }
        ++count;
    }
    if (kept) *kept = ne;
    free(start);
    free(nbr);
    free(fill);
    free(queue);
    return count;
}

/*
 * Alg. 2 Step 2 on the updated graph (n vertices, CSR already holds the batch):
 * W[c][j] = sum over members u of component c, over neighbours v of u labelled j, of w(u,v)
 * (W is num_comp x C, zeroed here); then every unlabelled inserted vertex u gets
 * F[u][j] = W[comp(u)][j] / sum_j W[comp(u)][j], or 1/C when that sum is 0.
 */
void oracle_supernode_init(int64_t n, const int64_t* row_ptr, const int32_t* col, const double* w, int C,
                           const int32_t* seed_class, int64_t n_old, const int32_t* comp, int64_t num_comp,
                           double* W, double* F) {
    memset(W, 0, sizeof(double) * (size_t)num_comp * C);
    for (int64_t u = n_old; u < n; ++u) {
        double* Wc = W + (int64_t)comp[u - n_old] * C;
        for (int64_t j = row_ptr[u]; j < row_ptr[u + 1]; ++j) {
            int32_t sc = seed_class[col[j]];
            if (sc >= 0) Wc[sc] += w[j];
        }
    }
    for (int64_t u = n_old; u < n; ++u) {
        if (seed_class[u] >= 0) continue;
        const double* Wc = W + (int64_t)comp[u - n_old] * C;
        double tot = 0.0;
        for (int c = 0; c < C; ++c) tot += Wc[c];
        for (int c = 0; c < C; ++c) F[u * C + c] = tot > 0.0 ? Wc[c] / tot : 1.0 / C;
    }
}
