/*
 * CPU oracle for HAG neighbourhood aggregation.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow and meant to be checked against the paper by eye.  It shares no
 * code, header, table or helper with the HIP library; only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.
 *
 * What it computes
 *   - naive aggregation: Algorithm 1, the Aggregate line, with the set
 *     aggregates of Table 1 (sum, element-wise max) plus mean = sum / |N(v)|;
 *   - aggregation over a HAG: Algorithm 2, the copy loop, the aggregation-node
 *     loop in creation order and the final per-node loop (the Update line is
 *     outside the hot path);
 *   - the transposed pass (vector-Jacobian product of the above), which the
 *     paper names only as an operation (Section 5.1) and which equivalence
 *     (Section 3.2, the definition before Theorem 2) forces to equal the
 *     naive gradient;
 *   - cover(v), Equation 1, expanded as a multiset so that a source feeding a
 *     node twice is detected (Theorem 2 is then checked as multiset equality);
 *   - the greedy search, Algorithm 3 for a set Aggregate, by brute force:
 *     every pair is recounted from scratch in every iteration.
 *
 * Conventions (ours where the paper is silent)
 *   - unified ids: original nodes 0..n-1, aggregation nodes n..n+a-1 in
 *     creation order, so creation order is a valid evaluation order
 *     (Section 3.1: a HAG is acyclic);
 *   - CSR rows are destinations, columns are in-neighbours (Section 3.1: an
 *     edge (u,v) means computing v needs u);
 *   - a node as a source always contributes its own activation, as a
 *     destination it aggregates its HAG in-neighbours (Algorithm 2);
 *   - fp32 inputs are accumulated in fp64; s_abs returns the sum of absolute
 *     values of the aggregated terms, the scale the tolerance is stated in;
 *   - int32 sums wrap modulo 2^32 (exactly associative);
 *   - empty neighbourhood: sum 0, mean 0, max 0 with argmax -1, no gradient;
 *   - max ties go to the smallest original node id; argmax holds original ids
 *     also when the value travelled through aggregation nodes;
 *   - the search stops when the best redundancy is <= 1 (such a merge saves
 *     nothing) and, among pairs of maximal redundancy, takes the
 *     lexicographically smallest (smaller id, larger id).
 *
 * Pins (tests marked "not gpu"): scipy CSR products, numpy segmented max,
 * hand-worked graphs, Theorem 2, the cost identity of Section 4.1, per-merge
 * accounting, capacity monotonicity, exhaustive optimum on tiny graphs.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

enum { OP_SUM = 0, OP_MEAN = 1, OP_MAX = 2, OP_GCN = 3 };
/* OP_GCN: GCN's Update before the weight matrix (Table 1): (sum over N(v) of h_u + h_v) / (|N(v)| + 1) */

/* ------------------------------------------------------------------ */
/* Algorithm 1, Aggregate line: a_v = Aggregate({h_u : u in N(v)})     */
/* ------------------------------------------------------------------ */
void oracle_naive_forward_f32(int64_t n, const int64_t *rowptr, const int32_t *col,
                              int64_t d, int op, const float *x,
                              double *y, double *s_abs, int32_t *argmax)
{
    #pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; ++v) {
        int64_t deg = rowptr[v + 1] - rowptr[v];
        for (int64_t f = 0; f < d; ++f) {
            double acc = 0.0, sa = 0.0;
            int32_t am = -1;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int32_t u = col[e];
                double xv = (double)x[(int64_t)u * d + f];
                if (op == OP_MAX) {
                    if (am < 0 || xv > acc || (xv == acc && u < am)) { acc = xv; am = u; }
                } else {
                    acc += xv;
                }
                sa += fabs(xv);
            }
            if (op == OP_MEAN && deg > 0) { acc /= (double)deg; sa /= (double)deg; }
            if (op == OP_GCN) {
                double xs = (double)x[v * d + f];
                acc = (acc + xs) / (double)(deg + 1);
                sa = (sa + fabs(xs)) / (double)(deg + 1);
            }
            y[v * d + f] = acc;
            if (s_abs) s_abs[v * d + f] = sa;
            if (op == OP_MAX && argmax) argmax[v * d + f] = am;
        }
    }
}

/* Transposed pass of the above: gX[u] = sum over v with u in N(v) of the
 * seed of v; seed = gY[v] (sum), gY[v]/|N(v)| (mean), gY[v] where
 * argmax[v]==u (max). */
void oracle_naive_backward_f32(int64_t n, const int64_t *rowptr, const int32_t *col,
                               int64_t d, int op, const float *gy, const int32_t *argmax,
                               double *gx, double *s_abs)
{
    /* threads own disjoint feature columns, so the scatter has no races */
    #pragma omp parallel for schedule(static)
    for (int64_t f = 0; f < d; ++f) {
        for (int64_t u = 0; u < n; ++u) { gx[u * d + f] = 0.0; if (s_abs) s_abs[u * d + f] = 0.0; }
        for (int64_t v = 0; v < n; ++v) {
            int64_t deg = rowptr[v + 1] - rowptr[v];
            double g = (double)gy[v * d + f];
            if (op == OP_MEAN && deg > 0) g /= (double)deg;
            if (op == OP_GCN) {               /* v also aggregates itself */
                g /= (double)(deg + 1);
                gx[v * d + f] += g;
                if (s_abs) s_abs[v * d + f] += fabs(g);
            }
            if (op == OP_MAX) {
                int32_t u = argmax[v * d + f];
                if (u >= 0) { gx[(int64_t)u * d + f] += g; if (s_abs) s_abs[(int64_t)u * d + f] += fabs(g); }
            } else {
                for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                    int64_t u = col[e];
                    gx[u * d + f] += g;
                    if (s_abs) s_abs[u * d + f] += fabs(g);
                }
            }
        }
    }
}

void oracle_naive_forward_i32(int64_t n, const int64_t *rowptr, const int32_t *col,
                              int64_t d, int op, const int32_t *x, int32_t *y, int32_t *argmax)
{
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f) {
            uint32_t acc = 0; int32_t best = 0, am = -1;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int32_t u = col[e];
                int32_t xv = x[(int64_t)u * d + f];
                if (op == OP_MAX) {
                    if (am < 0 || xv > best || (xv == best && u < am)) { best = xv; am = u; }
                } else acc += (uint32_t)xv;
            }
            y[v * d + f] = (op == OP_MAX) ? best : (int32_t)acc;
            if (op == OP_MAX && argmax) argmax[v * d + f] = am;
        }
}

void oracle_naive_backward_i32(int64_t n, const int64_t *rowptr, const int32_t *col,
                               int64_t d, int op, const int32_t *gy, const int32_t *argmax, int32_t *gx)
{
    uint32_t *g = (uint32_t *)gx;
    memset(g, 0, (size_t)(n * d) * sizeof(uint32_t));
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f) {
            uint32_t gv = (uint32_t)gy[v * d + f];
            if (op == OP_MAX) {
                int32_t u = argmax[v * d + f];
                if (u >= 0) g[(int64_t)u * d + f] += gv;
            } else
                for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
                    g[(int64_t)col[e] * d + f] += gv;
        }
}

/* ------------------------------------------------------------------ */
/* Algorithm 2 over a given HAG.                                       */
/*   left/right[a]: the two in-neighbours of aggregation node n+i      */
/*   hrowptr/hcol : the HAG in-neighbours of every original node       */
/*   deg[v]       : |N(v)| in the input graph (mean divides by it)     */
/* ------------------------------------------------------------------ */
void oracle_hag_forward_f32(int64_t n, int64_t a, const int32_t *left, const int32_t *right,
                            const int64_t *hrowptr, const int32_t *hcol, const int64_t *deg,
                            int64_t d, int op, const float *x,
                            double *y, int32_t *argmax)
{
    int64_t m = n + a;
    double *ahat = (double *)malloc((size_t)(m * d) * sizeof(double));
    int32_t *aid = (int32_t *)malloc((size_t)(m * d) * sizeof(int32_t));
    /* copy loop: ahat_v <- h_v for v in V */
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f) { ahat[v * d + f] = (double)x[v * d + f]; aid[v * d + f] = (int32_t)v; }
    /* aggregation nodes, creation order */
    for (int64_t i = 0; i < a; ++i) {
        int64_t w = n + i, l = left[i], r = right[i];
        for (int64_t f = 0; f < d; ++f) {
            double xl = ahat[l * d + f], xr = ahat[r * d + f];
            if (op == OP_MAX) {
                int32_t il = aid[l * d + f], ir = aid[r * d + f];
                int take_r = (xr > xl) || (xr == xl && ir < il);
                ahat[w * d + f] = take_r ? xr : xl;
                aid[w * d + f] = take_r ? ir : il;
            } else {
                ahat[w * d + f] = xl + xr;
                aid[w * d + f] = -1;
            }
        }
    }
    /* final loop: a_v <- Aggregate({ahat_u : u in Nhat_v}) */
    #pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f) {
            double acc = 0.0; int32_t am = -1;
            for (int64_t e = hrowptr[v]; e < hrowptr[v + 1]; ++e) {
                int64_t u = hcol[e];
                double xv = ahat[u * d + f];
                if (op == OP_MAX) {
                    int32_t iu = aid[u * d + f];
                    if (am < 0 || xv > acc || (xv == acc && iu < am)) { acc = xv; am = iu; }
                } else acc += xv;
            }
            if (op == OP_MEAN && deg[v] > 0) acc /= (double)deg[v];
            if (op == OP_GCN) acc = (acc + ahat[v * d + f]) / (double)(deg[v] + 1);
            y[v * d + f] = acc;
            if (op == OP_MAX && argmax) argmax[v * d + f] = am;
        }
    free(ahat); free(aid);
}

/* Reverse of Algorithm 2 for sum / mean: gradients flow from destinations to
 * their HAG in-neighbours, then down the aggregation nodes in reverse
 * creation order.  (Max uses only argmax: see oracle_naive_backward_f32.) */
void oracle_hag_backward_f32(int64_t n, int64_t a, const int32_t *left, const int32_t *right,
                             const int64_t *hrowptr, const int32_t *hcol, const int64_t *deg,
                             int64_t d, int op, const float *gy, double *gx)
{
    int64_t m = n + a;
    double *ghat = (double *)calloc((size_t)(m * d), sizeof(double));
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f) {
            double g = (double)gy[v * d + f];
            if (op == OP_MEAN && deg[v] > 0) g /= (double)deg[v];
            if (op == OP_GCN) { g /= (double)(deg[v] + 1); ghat[v * d + f] += g; }
            for (int64_t e = hrowptr[v]; e < hrowptr[v + 1]; ++e)
                ghat[(int64_t)hcol[e] * d + f] += g;
        }
    for (int64_t i = a - 1; i >= 0; --i) {
        int64_t w = n + i, l = left[i], r = right[i];
        for (int64_t f = 0; f < d; ++f) {
            ghat[l * d + f] += ghat[w * d + f];
            ghat[r * d + f] += ghat[w * d + f];
        }
    }
    memcpy(gx, ghat, (size_t)(n * d) * sizeof(double));
    free(ghat);
}

void oracle_hag_forward_i32(int64_t n, int64_t a, const int32_t *left, const int32_t *right,
                            const int64_t *hrowptr, const int32_t *hcol,
                            int64_t d, int op, const int32_t *x, int32_t *y, int32_t *argmax)
{
    int64_t m = n + a;
    int32_t *ahat = (int32_t *)malloc((size_t)(m * d) * sizeof(int32_t));
    int32_t *aid = (int32_t *)malloc((size_t)(m * d) * sizeof(int32_t));
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f) { ahat[v * d + f] = x[v * d + f]; aid[v * d + f] = (int32_t)v; }
    for (int64_t i = 0; i < a; ++i) {
        int64_t w = n + i, l = left[i], r = right[i];
        for (int64_t f = 0; f < d; ++f) {
            int32_t xl = ahat[l * d + f], xr = ahat[r * d + f];
            if (op == OP_MAX) {
                int32_t il = aid[l * d + f], ir = aid[r * d + f];
                int take_r = (xr > xl) || (xr == xl && ir < il);
                ahat[w * d + f] = take_r ? xr : xl;
                aid[w * d + f] = take_r ? ir : il;
            } else {
                ahat[w * d + f] = (int32_t)((uint32_t)xl + (uint32_t)xr);
                aid[w * d + f] = -1;
            }
        }
    }
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f) {
            uint32_t acc = 0; int32_t best = 0, am = -1;
            for (int64_t e = hrowptr[v]; e < hrowptr[v + 1]; ++e) {
                int64_t u = hcol[e];
                int32_t xv = ahat[u * d + f];
                if (op == OP_MAX) {
                    int32_t iu = aid[u * d + f];
                    if (am < 0 || xv > best || (xv == best && iu < am)) { best = xv; am = iu; }
                } else acc += (uint32_t)xv;
            }
            y[v * d + f] = (op == OP_MAX) ? best : (int32_t)acc;
            if (op == OP_MAX && argmax) argmax[v * d + f] = am;
        }
    free(ahat); free(aid);
}

void oracle_hag_backward_i32(int64_t n, int64_t a, const int32_t *left, const int32_t *right,
                             const int64_t *hrowptr, const int32_t *hcol,
                             int64_t d, const int32_t *gy, int32_t *gx)
{
    int64_t m = n + a;
    uint32_t *ghat = (uint32_t *)calloc((size_t)(m * d), sizeof(uint32_t));
    for (int64_t v = 0; v < n; ++v)
        for (int64_t f = 0; f < d; ++f)
            for (int64_t e = hrowptr[v]; e < hrowptr[v + 1]; ++e)
                ghat[(int64_t)hcol[e] * d + f] += (uint32_t)gy[v * d + f];
    for (int64_t i = a - 1; i >= 0; --i) {
        int64_t w = n + i, l = left[i], r = right[i];
        for (int64_t f = 0; f < d; ++f) {
            ghat[l * d + f] += ghat[w * d + f];
            ghat[r * d + f] += ghat[w * d + f];
        }
    }
    memcpy(gx, ghat, (size_t)(n * d) * sizeof(uint32_t));
    free(ghat);
}

/* ------------------------------------------------------------------ */
/* Equation 1 as a multiset, then Theorem 2.                           */
/* Returns 0 when, for every v, expanding Nhat_v down to original      */
/* nodes lists every member of N(v) exactly once and nothing else;     */
/* otherwise 1 + the first offending v.  -1: malformed HAG (an         */
/* aggregation node referring to itself or a later node).              */
/* ------------------------------------------------------------------ */
static void expand_cover(int64_t n, const int32_t *left, const int32_t *right,
                         int64_t node, int32_t *count, int64_t *touched, int64_t *n_touched)
{
    if (node < n) {
        if (count[node] == 0) touched[(*n_touched)++] = node;
        count[node] += 1;
        return;
    }
    expand_cover(n, left, right, left[node - n], count, touched, n_touched);
    expand_cover(n, left, right, right[node - n], count, touched, n_touched);
}

int64_t oracle_cover_check(int64_t n, const int64_t *rowptr, const int32_t *col,
                           int64_t a, const int32_t *left, const int32_t *right,
                           const int64_t *hrowptr, const int32_t *hcol)
{
    for (int64_t i = 0; i < a; ++i)
        if (left[i] < 0 || right[i] < 0 || left[i] >= n + i || right[i] >= n + i) return -1;
    int32_t *count = (int32_t *)calloc((size_t)n, sizeof(int32_t));
    int64_t *touched = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    int64_t bad = 0;
    for (int64_t v = 0; v < n && !bad; ++v) {
        int64_t nt = 0;
        for (int64_t e = hrowptr[v]; e < hrowptr[v + 1]; ++e) {
            if (hcol[e] < 0 || hcol[e] >= n + a) { bad = 1 + v; break; }
            expand_cover(n, left, right, hcol[e], count, touched, &nt);
        }
        /* every member of N(v) must have been listed exactly once ... */
        for (int64_t e = rowptr[v]; e < rowptr[v + 1] && !bad; ++e) {
            if (count[col[e]] != 1) bad = 1 + v;
            else count[col[e]] = -1;          /* mark as matched */
        }
        /* ... and nothing else may have been listed */
        for (int64_t t = 0; t < nt; ++t) {
            if (count[touched[t]] != -1 && !bad) bad = 1 + v;
            count[touched[t]] = 0;
        }
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) count[col[e]] = 0;
    }
    free(count); free(touched);
    return bad;
}

/* ------------------------------------------------------------------ */
/* Algorithm 3, set Aggregate, brute force.                            */
/* Every iteration recounts Redundancy(v1, v2) for every pair that     */
/* co-occurs in some Nhat_u, u in V, from scratch in a dense           */
/* (n+capacity)^2 table, picks the maximum with the canonical          */
/* tie-break, and rewrites the lists.  Only for small graphs.          */
/* Outputs: left/right/red[capacity]; hrowptr[n+1]; hcol[|E|] (the     */
/* rewritten lists, each sorted ascending).  Returns |V_A|.            */
/* ------------------------------------------------------------------ */
static int cmp_i32(const void *p, const void *q)
{
    int32_t x = *(const int32_t *)p, y = *(const int32_t *)q;
    return (x > y) - (x < y);
}

int64_t oracle_search(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity,
                      int32_t *left, int32_t *right, int32_t *red,
                      int64_t *hrowptr, int32_t *hcol)
{
    int64_t m = n + capacity;
    int64_t e_total = rowptr[n];
    /* Nhat_u as fixed-capacity slices of one array: a list never grows */
    int32_t *nb = (int32_t *)malloc((size_t)(e_total > 0 ? e_total : 1) * sizeof(int32_t));
    int64_t *len = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    memcpy(nb, col, (size_t)e_total * sizeof(int32_t));
    for (int64_t u = 0; u < n; ++u) len[u] = rowptr[u + 1] - rowptr[u];
    int32_t *cnt = (int32_t *)calloc((size_t)(m * m), sizeof(int32_t));
    int64_t a = 0;
    while (a < capacity) {
        /* count every co-occurring pair, indexed [smaller][larger] */
        for (int64_t u = 0; u < n; ++u) {
            const int32_t *l = nb + rowptr[u];
            for (int64_t i = 0; i < len[u]; ++i)
                for (int64_t j = i + 1; j < len[u]; ++j) {
                    int64_t p = l[i] < l[j] ? l[i] : l[j], q = l[i] < l[j] ? l[j] : l[i];
                    cnt[p * m + q] += 1;
                }
        }
        /* argmax with the canonical tie-break */
        int32_t best = 0; int64_t bp = -1, bq = -1;
        for (int64_t u = 0; u < n; ++u) {
            const int32_t *l = nb + rowptr[u];
            for (int64_t i = 0; i < len[u]; ++i)
                for (int64_t j = i + 1; j < len[u]; ++j) {
                    int64_t p = l[i] < l[j] ? l[i] : l[j], q = l[i] < l[j] ? l[j] : l[i];
                    int32_t c = cnt[p * m + q];
                    if (c > best || (c == best && (p < bp || (p == bp && q < bq)))) { best = c; bp = p; bq = q; }
                }
        }
        /* clear the table for the next iteration */
        for (int64_t u = 0; u < n; ++u) {
            const int32_t *l = nb + rowptr[u];
            for (int64_t i = 0; i < len[u]; ++i)
                for (int64_t j = i + 1; j < len[u]; ++j) {
                    int64_t p = l[i] < l[j] ? l[i] : l[j], q = l[i] < l[j] ? l[j] : l[i];
                    cnt[p * m + q] = 0;
                }
        }
        if (best <= 1) break;
        int32_t w = (int32_t)(n + a);
        left[a] = (int32_t)bp; right[a] = (int32_t)bq; red[a] = best;
        a += 1;
        /* every u in V holding both drops them and takes w instead */
        for (int64_t u = 0; u < n; ++u) {
            int32_t *l = nb + rowptr[u];
            int has_p = 0, has_q = 0;
            for (int64_t i = 0; i < len[u]; ++i) { has_p |= (l[i] == bp); has_q |= (l[i] == bq); }
            if (!(has_p && has_q)) continue;
            int64_t k = 0;
            for (int64_t i = 0; i < len[u]; ++i)
                if (l[i] != bp && l[i] != bq) l[k++] = l[i];
            l[k++] = w;
            len[u] = k;
        }
    }
    hrowptr[0] = 0;
    for (int64_t u = 0; u < n; ++u) {
        memcpy(hcol + hrowptr[u], nb + rowptr[u], (size_t)len[u] * sizeof(int32_t));
        qsort(hcol + hrowptr[u], (size_t)len[u], sizeof(int32_t), cmp_i32);
        hrowptr[u + 1] = hrowptr[u] + len[u];
    }
    free(nb); free(len); free(cnt);
    return a;
}

/* Redundancy(v1, v2) of Algorithm 3 for a set Aggregate, over given lists:
 * the number of u in V whose list holds both. */
int64_t oracle_redundancy(int64_t n, const int64_t *hrowptr, const int32_t *hcol, int32_t v1, int32_t v2)
{
    int64_t r = 0;
    for (int64_t u = 0; u < n; ++u) {
        int h1 = 0, h2 = 0;
        for (int64_t e = hrowptr[u]; e < hrowptr[u + 1]; ++e) { h1 |= (hcol[e] == v1); h2 |= (hcol[e] == v2); }
        r += (h1 && h2);
    }
    return r;
}
