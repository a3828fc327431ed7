/*
 * rama_oracle.c -- plain, slow, single-threaded CPU reference for the primal-dual
 * multicut round of "RAMA: A Rapid Multicut Algorithm on GPU" (arXiv 2109.01838).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
 * check and the benchmark's "cpu_baseline" leg may call it.  It shares no code,
 * header, table or helper with the HIP library; it is written directly from the
 * paper, one function per step, in the paper's order and notation, with no
 * blocking, fusion or reordering.  Every function names the passage it follows.
 *
 * Precision: the per-edge / per-triangle state is held in `real` (float by
 * default, because the reduced costs decide integers -- which edges are
 * attractive, which edge a node prefers in the matching -- and those decisions
 * must be taken in the precision of the GPU path; compile with
 * -DORACLE_REAL=double for an all-fp64 build used to size tolerances).  Scalar
 * results (lower bound, primal cost) are accumulated in double.  Compile with
 * -ffp-contract=off so that no multiply-add is fused.
 *
 * Pins (tests/test_oracle_*.py): the contraction worked example of Fig. 2,
 * brute-force optimal multicuts, brute-force cycle enumeration (lengths 3..7; the
 * shortest-only filter against that set and against scipy's hop distances), dense K^T A K,
 * scipy connected components / duplicate summation, closed-form min-marginals,
 * monotone lower bound, zero min-marginals after a triangle update; for the dual rounds:
 * every multicut keeps its cost under the reparametrisation (edges + kept triangles), the
 * bound grows from round to round and stays below the brute-force optimum.
 * Parity unpinned: the *choice* of triangulation (fan from the repulsive edge's
 * smaller endpoint) and the matching's tie-break order are readings of passages
 * on which the paper is silent; only their invariants are pinned.
 *
 * Conventions used throughout
 *   - a graph is (n, m, i[], j[], c[]); "canonical" means i<j, sorted by (i,j),
 *     no duplicates, no self-loops.
 *   - c>0 attractive, c<0 repulsive, c==0 neither (Sec. 3, eq. 2; Alg. 5 first two lines).
 *   - status: 0 ok, -1 invalid argument, -2 bad graph, -3 capacity, -4 out of memory.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL float
#endif
typedef ORACLE_REAL real;

#define OK 0
#define ERR_ARG (-1)
#define ERR_GRAPH (-2)
#define ERR_CAP (-3)
#define ERR_OOM (-4)

#define MAX_CYCLE_LEN 7            /* longest conflicted cycle the oracle separates */
#define N_LISTS (MAX_CYCLE_LEN - 2) /* one list per length 3..MAX_CYCLE_LEN; list L-3 holds the L-cycles */

/* ------------------------------------------------------------------------------------------ */
/* small helpers                                                                              */
/* ------------------------------------------------------------------------------------------ */

static void *xmalloc(size_t bytes) { return malloc(bytes ? bytes : 1); }

typedef struct {
    int32_t a, b;
    int64_t pos;
    real c;
} keyed_edge;

static int cmp_keyed_edge(const void *pa, const void *pb)
{
    const keyed_edge *x = (const keyed_edge *)pa, *y = (const keyed_edge *)pb;
    if (x->a != y->a) return x->a < y->a ? -1 : 1;
    if (x->b != y->b) return x->b < y->b ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

/* position of the canonical edge (u,v), u<v, or -1 */
static int64_t find_edge(int64_t m, const int32_t *i, const int32_t *j, int32_t u, int32_t v)
{
    int64_t lo = 0, hi = m;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (i[mid] < u || (i[mid] == u && j[mid] < v)) lo = mid + 1; else hi = mid;
    }
    return (lo < m && i[lo] == u && j[lo] == v) ? lo : -1;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a0: problem statement -> canonical edge list                                          */
/* Sec. 3 (graph, cost vector); Lemma 1(b): parallel edges carry the sum of their costs.      */
/* Self-loops can never be cut and are dropped.  Duplicates are summed in input order.        */
/* ------------------------------------------------------------------------------------------ */
int rama_oracle_canonicalise(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                             int32_t *io, int32_t *jo, float *co, int64_t *m_out)
{
    if (n < 0 || m < 0 || !m_out || (m > 0 && (!i || !j || !c || !io || !jo || !co))) return ERR_ARG;
    for (int64_t e = 0; e < m; ++e) {
        if (i[e] < 0 || i[e] >= n || j[e] < 0 || j[e] >= n) return ERR_GRAPH;
        if (!isfinite(c[e])) return ERR_GRAPH;
    }
    keyed_edge *k = (keyed_edge *)xmalloc((size_t)m * sizeof *k);
    if (!k) return ERR_OOM;
    int64_t cnt = 0;
    for (int64_t e = 0; e < m; ++e) {
        if (i[e] == j[e]) continue;
        k[cnt].a = i[e] < j[e] ? i[e] : j[e];
        k[cnt].b = i[e] < j[e] ? j[e] : i[e];
        k[cnt].pos = e;
        k[cnt].c = (real)c[e];
        ++cnt;
    }
    qsort(k, (size_t)cnt, sizeof *k, cmp_keyed_edge);
    int64_t o = 0;
    for (int64_t e = 0; e < cnt;) {
        real acc = k[e].c;
        int64_t f = e + 1;
        while (f < cnt && k[f].a == k[e].a && k[f].b == k[e].b) { acc = acc + k[f].c; ++f; }
        io[o] = k[e].a; jo[o] = k[e].b; co[o] = (float)acc; ++o;
        e = f;
    }
    free(k);
    *m_out = o;
    return OK;
}

/* ------------------------------------------------------------------------------------------ */
/* positive neighbourhoods N+(v) (Sec. 3.2.2 definition of E+; appendix "Conflicted cycles")  */
/* built from a canonical edge list; every row comes out in ascending order.                   */
/* ------------------------------------------------------------------------------------------ */
typedef struct {
    int32_t n;
    int64_t *ptr;  /* n+1 */
    int32_t *nb;   /* 2|E+| */
} posadj;

static int posadj_build(posadj *a, int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c)
{
    a->n = n;
    a->ptr = (int64_t *)calloc((size_t)n + 2, sizeof(int64_t));
    if (!a->ptr) return ERR_OOM;
    for (int64_t e = 0; e < m; ++e)
        if (c[e] > 0.0f) { a->ptr[i[e] + 1]++; a->ptr[j[e] + 1]++; }
    for (int32_t v = 0; v < n; ++v) a->ptr[v + 1] += a->ptr[v];
    a->nb = (int32_t *)xmalloc((size_t)a->ptr[n] * sizeof(int32_t));
    int64_t *fill = (int64_t *)xmalloc(((size_t)n + 1) * sizeof(int64_t));
    if (!a->nb || !fill) return ERR_OOM;
    memcpy(fill, a->ptr, ((size_t)n + 1) * sizeof(int64_t));
    for (int64_t e = 0; e < m; ++e)
        if (c[e] > 0.0f) { a->nb[fill[i[e]]++] = j[e]; a->nb[fill[j[e]]++] = i[e]; }
    free(fill);
    return OK;
}

static void posadj_free(posadj *a) { free(a->ptr); free(a->nb); }

static int posadj_has(const posadj *a, int32_t u, int32_t v)
{
    int64_t lo = a->ptr[u], hi = a->ptr[u + 1];
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (a->nb[mid] < v) lo = mid + 1; else hi = mid;
    }
    return lo < a->ptr[u + 1] && a->nb[lo] == v;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a1: conflicted cycles (Sec. 3.2.2 "Conflicted cycles" definition; Lemma on the search */
/* per repulsive edge; appendix Alg. "Parallel Conf. 5-Cycles"; the paper stops at length 5    */
/* and names longer cycles as future work, Sec. 5 -- the definition is the same for any L).   */
/* Plain definition: every simple cycle of length L in {3,..,Lmax} with exactly one edge of   */
/* E- and L-1 edges of E+.  For the repulsive edge (v0,v_{L-1}), v0<v_{L-1}, that is every    */
/* simple path v0,v1,..,v_{L-1} along E+.  Depth-first enumeration, nothing pruned.           */
/* Stored as the tuple (v0,..,v_{L-1}); lists ordered by (v0, v_{L-1}, v1, .., v_{L-2}).      */
/*                                                                                            */
/* shortest_only (the separation Lemma read literally: per repulsive edge, the shortest paths */
/* w.r.t. hop distance in (V,E+)): with d = hop distance between the endpoints of the         */
/* repulsive edge in (V,E+), only its cycles of length d+1 are kept (all of them), and none   */
/* if d+1 > Lmax.  d comes from a breadth-first search that is independent of the             */
/* enumeration above.                                                                         */
/* ------------------------------------------------------------------------------------------ */
typedef struct {
    int L;
    int64_t cap, cnt;
    int32_t *out;
} cycle_sink;

static void cycles_extend(const posadj *a, int32_t *path, int len, int L, int32_t vlast, cycle_sink *s)
{
    if (len == L - 1) {
        if (posadj_has(a, path[len - 1], vlast)) {
            if (s->cnt < s->cap) {
                for (int q = 0; q < L - 1; ++q) s->out[s->cnt * L + q] = path[q];
                s->out[s->cnt * L + L - 1] = vlast;
            }
            s->cnt++;
        }
        return;
    }
    int32_t tail = path[len - 1];
    for (int64_t p = a->ptr[tail]; p < a->ptr[tail + 1]; ++p) {
        int32_t w = a->nb[p];
        if (w == vlast) continue;
        int seen = 0;
        for (int q = 0; q < len; ++q) if (path[q] == w) seen = 1;
        if (seen) continue;
        path[len] = w;
        cycles_extend(a, path, len + 1, L, vlast, s);
    }
}

/* hop distance src -> dst in (V,E+) by breadth-first search, given up beyond `limit` hops
 * (returns limit+1 then).  seen[] holds the id of the last search that reached a node. */
static int hop_distance(const posadj *a, int32_t src, int32_t dst, int limit, int64_t search_id,
                        int64_t *seen, int32_t *queue, int32_t *depth)
{
    int64_t head = 0, tail = 0;
    queue[tail] = src; depth[tail] = 0; ++tail;
    seen[src] = search_id;
    while (head < tail) {
        int32_t u = queue[head];
        int d = depth[head];
        ++head;
        if (u == dst) return d;
        if (d == limit) continue;
        for (int64_t p = a->ptr[u]; p < a->ptr[u + 1]; ++p) {
            int32_t w = a->nb[p];
            if (seen[w] == search_id) continue;
            seen[w] = search_id;
            queue[tail] = w; depth[tail] = d + 1; ++tail;
        }
    }
    return limit + 1;
}

static int g_cyc_L;
static int cmp_cycle(const void *pa, const void *pb)
{
    const int32_t *x = (const int32_t *)pa, *y = (const int32_t *)pb;
    const int L = g_cyc_L;
    /* repulsive edge first, then the path: v0, v_{L-1}, v1, .., v_{L-2} */
    int order[MAX_CYCLE_LEN];
    order[0] = 0; order[1] = L - 1;
    for (int q = 1; q <= L - 2; ++q) order[q + 1] = q;
    for (int q = 0; q < L; ++q) {
        int32_t xa = x[order[q]], ya = y[order[q]];
        if (xa != ya) return xa < ya ? -1 : 1;
    }
    return 0;
}

/* cap[L-3] / cycles[L-3] / n_out[L-3] belong to the L-cycles, L = 3..max_cycle_len; cap and
 * cycles may be NULL (count only).  n_out gets max_cycle_len-2 entries. */
int rama_oracle_find_conflicted_cycles(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                                       int32_t max_cycle_len, int32_t shortest_only, const int64_t *cap,
                                       int32_t *const *cycles, int64_t *n_out)
{
    if (!n_out || max_cycle_len < 3 || max_cycle_len > MAX_CYCLE_LEN) return ERR_ARG;
    int32_t *ci = (int32_t *)xmalloc((size_t)m * 4), *cj = (int32_t *)xmalloc((size_t)m * 4);
    float *cc = (float *)xmalloc((size_t)m * 4);
    int64_t mc = 0;
    if (!ci || !cj || !cc) return ERR_OOM;
    int st = rama_oracle_canonicalise(n, m, i, j, c, ci, cj, cc, &mc);
    if (st != OK) { free(ci); free(cj); free(cc); return st; }
    posadj a;
    st = posadj_build(&a, n, mc, ci, cj, cc);
    if (st != OK) return st;
    int *dist = NULL;                                    /* per edge: hop distance of its endpoints in (V,E+) */
    if (shortest_only) {
        dist = (int *)xmalloc((size_t)mc * sizeof(int));
        int64_t *seen = (int64_t *)xmalloc(((size_t)n + 1) * 8);
        int32_t *queue = (int32_t *)xmalloc(((size_t)n + 1) * 4), *depth = (int32_t *)xmalloc(((size_t)n + 1) * 4);
        if (!dist || !seen || !queue || !depth) return ERR_OOM;
        for (int32_t v = 0; v < n; ++v) seen[v] = -1;
        for (int64_t e = 0; e < mc; ++e)
            if (cc[e] < 0.0f) dist[e] = hop_distance(&a, ci[e], cj[e], max_cycle_len - 1, e, seen, queue, depth);
        free(seen); free(queue); free(depth);
    }
    int over = 0;
    for (int L = 3; L <= max_cycle_len; ++L) {
        int32_t *out = cycles ? cycles[L - 3] : NULL;
        cycle_sink s = { L, (out && cap) ? cap[L - 3] : 0, 0, out };
        for (int64_t e = 0; e < mc; ++e) {
            if (!(cc[e] < 0.0f)) continue;               /* e in E- */
            if (shortest_only && dist[e] != L - 1) continue;
            int32_t path[MAX_CYCLE_LEN];
            path[0] = ci[e];
            cycles_extend(&a, path, 1, L, cj[e], &s);
        }
        if (s.cnt > s.cap) over = 1;
        else if (s.cnt > 1) { g_cyc_L = L; qsort(s.out, (size_t)s.cnt, (size_t)L * 4, cmp_cycle); }
        n_out[L - 3] = s.cnt;
    }
    posadj_free(&a);
    free(dist);
    free(ci); free(cj); free(cc);
    return over ? ERR_CAP : OK;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a2: triangulation (Sec. 3.2.1: cycles longer than three are triangulated; the paper   */
/* gives no procedure).  Reading: fan from v0 -- triangles {v0,v_m,v_{m+1}}, m=1..L-2, chords */
/* (v0,v_m), m=2..L-2.  A chord that is not an edge yet joins the edge set with cost 0.  The  */
/* augmented edge list stays canonical; T is the sorted set of node triples u<v<w;            */
/* tri_edge[3t+s] is the edge id of slot s, slots ordered (u,v),(u,w),(v,w).                  */
/* Input must be canonical.  cycles[L-3] holds the n_cycles[L-3] cycles of length L,           */
/* L = 3..max_cycle_len.  ia/ja/ca need room for m + sum (L-3)*n_L edges, tri_* for            */
/* sum (L-2)*n_L triangles.                                                                    */
/* ------------------------------------------------------------------------------------------ */
typedef struct { int32_t u, v, w; } tri3;
static int cmp_tri3(const void *pa, const void *pb)
{
    const tri3 *x = (const tri3 *)pa, *y = (const tri3 *)pb;
    if (x->u != y->u) return x->u < y->u ? -1 : 1;
    if (x->v != y->v) return x->v < y->v ? -1 : 1;
    if (x->w != y->w) return x->w < y->w ? -1 : 1;
    return 0;
}
static void sort3(int32_t *p)
{
    int32_t t;
    if (p[0] > p[1]) { t = p[0]; p[0] = p[1]; p[1] = t; }
    if (p[1] > p[2]) { t = p[1]; p[1] = p[2]; p[2] = t; }
    if (p[0] > p[1]) { t = p[0]; p[0] = p[1]; p[1] = t; }
}

int rama_oracle_triangulate(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                            int32_t max_cycle_len, const int32_t *const *cycles, const int64_t *n_cycles,
                            int32_t *ia, int32_t *ja, float *ca, int64_t *m_aug,
                            int32_t *tri_nodes, int32_t *tri_edge, int64_t *n_tri)
{
    if (!m_aug || !n_tri || max_cycle_len < 3 || max_cycle_len > MAX_CYCLE_LEN || !cycles || !n_cycles) return ERR_ARG;
    /* chords */
    int64_t n_chord_max = 0, nch = 0, n_tri_max = 0, nt = 0;
    for (int L = 3; L <= max_cycle_len; ++L) {
        if (n_cycles[L - 3] < 0) return ERR_ARG;
        n_chord_max += (L - 3) * n_cycles[L - 3];
        n_tri_max += (L - 2) * n_cycles[L - 3];
    }
    keyed_edge *ch = (keyed_edge *)xmalloc((size_t)n_chord_max * sizeof *ch);
    tri3 *tr = (tri3 *)xmalloc((size_t)n_tri_max * sizeof *tr);
    if (!ch || !tr) return ERR_OOM;
    for (int L = 3; L <= max_cycle_len; ++L) {
        for (int64_t q = 0; q < n_cycles[L - 3]; ++q) {
            const int32_t *v = cycles[L - 3] + q * L;
            for (int s = 0; s < L; ++s) {
                if (v[s] < 0 || v[s] >= n) { free(ch); free(tr); return ERR_GRAPH; }
                for (int s2 = 0; s2 < s; ++s2) if (v[s2] == v[s]) { free(ch); free(tr); return ERR_GRAPH; }
            }
            for (int s = 0; s < L; ++s) {      /* every cycle edge must exist in the graph */
                int32_t x = v[s], y = v[(s + 1) % L];
                if (find_edge(m, i, j, x < y ? x : y, x < y ? y : x) < 0) { free(ch); free(tr); return ERR_GRAPH; }
            }
            for (int mm = 2; mm <= L - 2; ++mm) {
                ch[nch].a = v[0] < v[mm] ? v[0] : v[mm];
                ch[nch].b = v[0] < v[mm] ? v[mm] : v[0];
                ch[nch].pos = 0; ch[nch].c = 0;
                ++nch;
            }
            for (int mm = 1; mm <= L - 2; ++mm) {
                int32_t p[3] = { v[0], v[mm], v[mm + 1] };
                sort3(p);
                tr[nt].u = p[0]; tr[nt].v = p[1]; tr[nt].w = p[2];
                ++nt;
            }
        }
    }
    qsort(ch, (size_t)nch, sizeof *ch, cmp_keyed_edge);
    /* merge the canonical edges and the new chords */
    int64_t e = 0, o = 0;
    for (int64_t q = 0; q < nch; ++q) {
        if (q > 0 && ch[q].a == ch[q - 1].a && ch[q].b == ch[q - 1].b) continue;
        if (find_edge(m, i, j, ch[q].a, ch[q].b) >= 0) continue;
        while (e < m && (i[e] < ch[q].a || (i[e] == ch[q].a && j[e] < ch[q].b))) {
            ia[o] = i[e]; ja[o] = j[e]; ca[o] = c[e]; ++o; ++e;
        }
        ia[o] = ch[q].a; ja[o] = ch[q].b; ca[o] = 0.0f; ++o;
    }
    while (e < m) { ia[o] = i[e]; ja[o] = j[e]; ca[o] = c[e]; ++o; ++e; }
    *m_aug = o;
    free(ch);
    /* unique triangles */
    qsort(tr, (size_t)nt, sizeof *tr, cmp_tri3);
    int64_t t = 0;
    for (int64_t q = 0; q < nt; ++q) {
        if (q > 0 && cmp_tri3(&tr[q], &tr[q - 1]) == 0) continue;
        tri_nodes[3 * t + 0] = tr[q].u; tri_nodes[3 * t + 1] = tr[q].v; tri_nodes[3 * t + 2] = tr[q].w;
        int64_t e0 = find_edge(o, ia, ja, tr[q].u, tr[q].v);
        int64_t e1 = find_edge(o, ia, ja, tr[q].u, tr[q].w);
        int64_t e2 = find_edge(o, ia, ja, tr[q].v, tr[q].w);
        if (e0 < 0 || e1 < 0 || e2 < 0) { free(tr); return ERR_GRAPH; }
        tri_edge[3 * t + 0] = (int32_t)e0; tri_edge[3 * t + 1] = (int32_t)e1; tri_edge[3 * t + 2] = (int32_t)e2;
        ++t;
    }
    *n_tri = t;
    free(tr);
    return OK;
}

/* ------------------------------------------------------------------------------------------ */
/* Triangle subproblem (Sec. 3.2.1): feasible labelings M_T; cost <c_t, y>.                    */
/* ------------------------------------------------------------------------------------------ */
static const int M_T[5][3] = { { 0, 0, 0 }, { 1, 1, 0 }, { 1, 0, 1 }, { 0, 1, 1 }, { 1, 1, 1 } };

static real tri_cost(const real *ct, const int *y)
{
    real acc = 0;
    for (int s = 0; s < 3; ++s) if (y[s]) acc = acc + ct[s];
    return acc;
}

/* min-marginal of slot s (Sec. 3.2.3, "Marginalization for triangle subproblems") */
static real tri_min_marginal(const real *ct, int s)
{
    real best1 = 0, best0 = 0;
    int have1 = 0, have0 = 0;
    for (int l = 0; l < 5; ++l) {
        real v = tri_cost(ct, M_T[l]);
        if (M_T[l][s]) { if (!have1 || v < best1) best1 = v; have1 = 1; }
        else           { if (!have0 || v < best0) best0 = v; have0 = 1; }
    }
    return best1 - best0;
}

/* triangle term of LB(lambda) (eq. 5) */
static real tri_lower_bound(const real *ct)
{
    real best = tri_cost(ct, M_T[0]);
    for (int l = 1; l < 5; ++l) { real v = tri_cost(ct, M_T[l]); if (v < best) best = v; }
    return best;
}

double rama_oracle_min_marginal(const float *ct3, int32_t slot)
{
    real ct[3] = { (real)ct3[0], (real)ct3[1], (real)ct3[2] };
    return (double)tri_min_marginal(ct, slot);
}
double rama_oracle_triangle_lb(const float *ct3)
{
    real ct[3] = { (real)ct3[0], (real)ct3[1], (real)ct3[2] };
    return (double)tri_lower_bound(ct);
}

/* ------------------------------------------------------------------------------------------ */
/* Step a3: message passing state and the two half-steps of Alg. "Parallel-Message-Passing".  */
/* State: ce[e] = reparametrised edge cost c^lambda_e (eq. 6a), ct[3t+s] = c^lambda_t (eq. 6b, */
/* i.e. minus the multipliers).  Both persist over the k iterations of one round.              */
/* ------------------------------------------------------------------------------------------ */
typedef struct {
    int64_t m, T;
    const int32_t *tri_edge;
    real *ce, *ct;
    int64_t *slot_ptr;   /* m+1 : triangle slots of every edge, ascending triangle id */
    int64_t *slot;       /* 3T */
} mp_state;

/* ct0: triangle costs to start from (3T values), NULL = all zero (no multipliers yet) */
static int mp_init(mp_state *s, int64_t m, const float *c, int64_t T, const int32_t *tri_edge, const real *ct0)
{
    s->m = m; s->T = T; s->tri_edge = tri_edge;
    s->ce = (real *)xmalloc((size_t)m * sizeof(real));
    s->ct = (real *)calloc((size_t)(3 * T) + 1, sizeof(real));
    s->slot_ptr = (int64_t *)calloc((size_t)m + 2, sizeof(int64_t));
    s->slot = (int64_t *)xmalloc((size_t)(3 * T) * sizeof(int64_t));
    if (!s->ce || !s->ct || !s->slot_ptr || !s->slot) return ERR_OOM;
    if (ct0) for (int64_t q = 0; q < 3 * T; ++q) s->ct[q] = ct0[q];
    for (int64_t e = 0; e < m; ++e) s->ce[e] = (real)c[e];
    for (int64_t q = 0; q < 3 * T; ++q) s->slot_ptr[tri_edge[q] + 1]++;
    for (int64_t e = 0; e < m; ++e) s->slot_ptr[e + 1] += s->slot_ptr[e];
    int64_t *fill = (int64_t *)xmalloc(((size_t)m + 1) * sizeof(int64_t));
    if (!fill) return ERR_OOM;
    memcpy(fill, s->slot_ptr, ((size_t)m + 1) * sizeof(int64_t));
    for (int64_t q = 0; q < 3 * T; ++q) s->slot[fill[tri_edge[q]]++] = q;
    free(fill);
    return OK;
}
static void mp_free(mp_state *s) { free(s->ce); free(s->ct); free(s->slot_ptr); free(s->slot); }

/* edges -> triangles: an edge hands its whole reparametrised cost to its triangles in equal
 * shares and ends at zero.  An edge in no triangle keeps its cost. */
static void mp_edges_to_triangles(mp_state *s)
{
    for (int64_t e = 0; e < s->m; ++e) {
        int64_t N = s->slot_ptr[e + 1] - s->slot_ptr[e];
        if (N == 0) continue;
        real alpha = s->ce[e];
        real share = alpha / (real)N;
        for (int64_t p = s->slot_ptr[e]; p < s->slot_ptr[e + 1]; ++p)
            s->ct[s->slot[p]] = s->ct[s->slot[p]] + share;     /* lambda_{t,e} -= alpha/N  <=>  c_t[e] += alpha/N */
        s->ce[e] = 0;
    }
}

/* triangles -> edges: six min-marginal updates per triangle with weights 1/3, 1/2, 1, 1/2, 1, 1
 * on the slots ij, ik, jk, ij, ik, ij; each uses the triangle costs as they stand at that
 * moment.  lambda_{t,e} += w*m  <=>  c_t[e] -= w*m and c^lambda_e += w*m (eq. 6a, 6b).
 * The messages of one edge are added in ascending triangle order. */
static void mp_triangles_to_edges(mp_state *s, real *msg /* 3T scratch */)
{
    static const int order[6] = { 0, 1, 2, 0, 1, 0 };
    const real weight[6] = { (real)1 / (real)3, (real)1 / (real)2, (real)1, (real)1 / (real)2, (real)1, (real)1 };
    for (int64_t t = 0; t < s->T; ++t) {
        real *ct = s->ct + 3 * t;
        real out[3] = { 0, 0, 0 };
        for (int q = 0; q < 6; ++q) {
            int sl = order[q];
            real d = weight[q] * tri_min_marginal(ct, sl);
            ct[sl] = ct[sl] - d;
            out[sl] = out[sl] + d;
        }
        for (int sl = 0; sl < 3; ++sl) msg[3 * t + sl] = out[sl];
    }
    for (int64_t e = 0; e < s->m; ++e) {
        real acc = s->ce[e];
        for (int64_t p = s->slot_ptr[e]; p < s->slot_ptr[e + 1]; ++p) acc = acc + msg[s->slot[p]];
        s->ce[e] = acc;
    }
}

/* LB(lambda), eq. 5 */
static double mp_lower_bound(const mp_state *s)
{
    double lb = 0.0;
    for (int64_t e = 0; e < s->m; ++e) if (s->ce[e] < 0) lb += (double)s->ce[e];
    for (int64_t t = 0; t < s->T; ++t) lb += (double)tri_lower_bound(s->ct + 3 * t);
    return lb;
}

/* Exposed half-steps on caller-held state (for invariant tests).  ce: float[m], ct: float[3T]. */
int rama_oracle_mp_half_step(int64_t m, float *ce, int64_t T, const int32_t *tri_edge, float *ct, int32_t which)
{
    mp_state s;
    int st = mp_init(&s, m, ce, T, tri_edge, NULL);
    if (st != OK) return st;
    for (int64_t q = 0; q < 3 * T; ++q) s.ct[q] = (real)ct[q];
    if (which == 0) mp_edges_to_triangles(&s);
    else {
        real *msg = (real *)xmalloc((size_t)(3 * T) * sizeof(real));
        if (!msg) return ERR_OOM;
        mp_triangles_to_edges(&s, msg);
        free(msg);
    }
    for (int64_t e = 0; e < m; ++e) ce[e] = (float)s.ce[e];
    for (int64_t q = 0; q < 3 * T; ++q) ct[q] = (float)s.ct[q];
    mp_free(&s);
    return OK;
}
double rama_oracle_lower_bound(int64_t m, const float *ce, int64_t T, const float *ct)
{
    double lb = 0.0;
    for (int64_t e = 0; e < m; ++e) if (ce[e] < 0) lb += (double)ce[e];
    for (int64_t t = 0; t < T; ++t) {
        real x[3] = { (real)ct[3 * t], (real)ct[3 * t + 1], (real)ct[3 * t + 2] };
        lb += (double)tri_lower_bound(x);
    }
    return lb;
}

/* The whole dual step of one round (Alg. "Primal-Dual Multicut", inner loop): triangulate the
 * cycles, run k iterations of message passing, hand back the augmented edge list with the
 * reparametrised costs, LB after the k-th iteration and optionally LB after every iteration
 * (lb_trace[0] is LB before the first). */
int rama_oracle_message_passing(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                                int32_t max_cycle_len, const int32_t *const *cycles, const int64_t *n_cycles,
                                int32_t k_iters, int64_t edge_cap,
                                int32_t *io, int32_t *jo, float *co, int64_t *m_out,
                                double *lower_bound, double *lb_trace)
{
    if (k_iters < 0 || !m_out || max_cycle_len < 3 || max_cycle_len > MAX_CYCLE_LEN || !cycles || !n_cycles) return ERR_ARG;
    int32_t *ci = (int32_t *)xmalloc((size_t)m * 4), *cj = (int32_t *)xmalloc((size_t)m * 4);
    float *cc = (float *)xmalloc((size_t)m * 4);
    if (!ci || !cj || !cc) return ERR_OOM;
    int64_t mc = 0;
    int st = rama_oracle_canonicalise(n, m, i, j, c, ci, cj, cc, &mc);
    if (st != OK) { free(ci); free(cj); free(cc); return st; }
    int64_t room = mc, Tmax = 0;
    for (int L = 3; L <= max_cycle_len; ++L) {
        if (n_cycles[L - 3] < 0) { free(ci); free(cj); free(cc); return ERR_ARG; }
        room += (L - 3) * n_cycles[L - 3];
        Tmax += (L - 2) * n_cycles[L - 3];
    }
    int32_t *ia = (int32_t *)xmalloc((size_t)room * 4), *ja = (int32_t *)xmalloc((size_t)room * 4);
    float *ca = (float *)xmalloc((size_t)room * 4);
    int32_t *tn = (int32_t *)xmalloc((size_t)Tmax * 12), *te = (int32_t *)xmalloc((size_t)Tmax * 12);
    if (!ia || !ja || !ca || !tn || !te) return ERR_OOM;
    int64_t ma = 0, T = 0;
    st = rama_oracle_triangulate(n, mc, ci, cj, cc, max_cycle_len, cycles, n_cycles, ia, ja, ca, &ma, tn, te, &T);
    free(ci); free(cj); free(cc);
    if (st == OK && ma > edge_cap) { *m_out = ma; st = ERR_CAP; }
    if (st != OK) { free(ia); free(ja); free(ca); free(tn); free(te); return st; }
    mp_state s;
    st = mp_init(&s, ma, ca, T, te, NULL);
    if (st != OK) return st;
    real *msg = (real *)xmalloc((size_t)(3 * T) * sizeof(real));
    if (!msg) return ERR_OOM;
    if (lb_trace) lb_trace[0] = mp_lower_bound(&s);
    for (int32_t it = 1; it <= k_iters; ++it) {
        mp_edges_to_triangles(&s);
        mp_triangles_to_edges(&s, msg);
        if (lb_trace) lb_trace[it] = mp_lower_bound(&s);
    }
    if (lower_bound) *lower_bound = mp_lower_bound(&s);
    for (int64_t e = 0; e < ma; ++e) { io[e] = ia[e]; jo[e] = ja[e]; co[e] = (float)s.ce[e]; }
    *m_out = ma;
    free(msg); mp_free(&s);
    free(ia); free(ja); free(ca); free(tn); free(te);
    return OK;
}

/* ------------------------------------------------------------------------------------------ */
/* Dual rounds on one graph.  One round = separate the conflicted cycles of the current         */
/* reparametrised costs (step a1), add their triangles to the triangle set, k iterations of     */
/* message passing over the whole set.  With one round this is the dual part of a round of      */
/* Alg. "Primal-Dual Multicut".  More rounds re-separate on the same graph, the cutting-plane   */
/* loop that Sec. 5 points to when it asks for better separation: triangles found earlier stay  */
/* in the relaxation and keep their costs c_t (dropping them would give back what their         */
/* multipliers gained), new ones start at zero, so LB never decreases from round to round.      */
/* The loop ends early when a separation finds nothing.                                         */
/* In/out: a canonical graph (*gi,*gj,*gc of *m edges, malloc'd; replaced by the augmented      */
/* graph with reparametrised costs).  Out: lb (after the last round run; the sum of negative    */
/* costs if none ran), lb_trace[0..rounds] (optional; [0] before the first round, entries of    */
/* rounds that did not run repeat the last value), cycles_first[N_LISTS] (optional, first       */
/* round), and optionally the final triangle set: *tri_nodes_out (3T, sorted triples), *ct_out  */
/* (3T), *T_out.                                                                                */
/* ------------------------------------------------------------------------------------------ */
static int tri_triple_cmp(const int32_t *a, const int32_t *b)
{
    for (int q = 0; q < 3; ++q) if (a[q] != b[q]) return a[q] < b[q] ? -1 : 1;
    return 0;
}

static int dual_block(int32_t n, int64_t *m, int32_t **gi, int32_t **gj, float **gc,
                      int32_t max_cycle_len, int32_t shortest_only, int32_t k_iters, int32_t rounds,
                      double *lb, double *lb_trace, int64_t *cycles_first,
                      int32_t **tri_nodes_out, real **ct_out, int64_t *T_out)
{
    int st = OK;
    int64_t T = 0;
    int32_t *tn = NULL;      /* triangle set so far: sorted node triples */
    real *ct = NULL;         /* their costs */
    double cur = 0.0;
    for (int64_t e = 0; e < *m; ++e) if ((*gc)[e] < 0) cur += (double)(*gc)[e];
    if (lb_trace) lb_trace[0] = cur;
    if (cycles_first) for (int q = 0; q < N_LISTS; ++q) cycles_first[q] = 0;
    int32_t done = 0;
    for (int32_t d = 1; d <= rounds && max_cycle_len >= 3; ++d) {
        int64_t cnt[N_LISTS] = { 0 }, total = 0, chords = 0, fans = 0;
        int32_t *cyc[N_LISTS] = { NULL };
        st = rama_oracle_find_conflicted_cycles(n, *m, *gi, *gj, *gc, max_cycle_len, shortest_only, NULL, NULL, cnt);
        if (st != OK && st != ERR_CAP) break;
        for (int L = 3; L <= max_cycle_len; ++L) {
            /* room for the old triangles behind the new 3-cycles: they re-enter as 3-cycles */
            cyc[L - 3] = (int32_t *)xmalloc((size_t)(cnt[L - 3] + (L == 3 ? T : 0)) * L * 4);
            if (!cyc[L - 3]) return ERR_OOM;
        }
        st = rama_oracle_find_conflicted_cycles(n, *m, *gi, *gj, *gc, max_cycle_len, shortest_only, cnt, cyc, cnt);
        if (st != OK) break;
        for (int L = 3; L <= max_cycle_len; ++L) { total += cnt[L - 3]; chords += (L - 3) * cnt[L - 3]; fans += (L - 2) * cnt[L - 3]; }
        if (d == 1 && cycles_first) for (int q = 0; q < N_LISTS; ++q) cycles_first[q] = cnt[q];
        if (total == 0) { for (int L = 0; L < N_LISTS; ++L) free(cyc[L]); break; }
        if (T > 0) memcpy(cyc[0] + 3 * cnt[0], tn, (size_t)T * 12);
        int64_t with_old[N_LISTS];
        for (int q = 0; q < N_LISTS; ++q) with_old[q] = cnt[q];
        with_old[0] += T;
        int64_t room = *m + chords, ma = 0, Tn = 0;
        int32_t *ia = (int32_t *)xmalloc((size_t)room * 4), *ja = (int32_t *)xmalloc((size_t)room * 4);
        float *ca = (float *)xmalloc((size_t)room * 4);
        int32_t *tnn = (int32_t *)xmalloc((size_t)(fans + T) * 12), *te = (int32_t *)xmalloc((size_t)(fans + T) * 12);
        if (!ia || !ja || !ca || !tnn || !te) return ERR_OOM;
        st = rama_oracle_triangulate(n, *m, *gi, *gj, *gc, max_cycle_len, (const int32_t *const *)cyc, with_old,
                                     ia, ja, ca, &ma, tnn, te, &Tn);
        for (int L = 0; L < N_LISTS; ++L) free(cyc[L]);
        if (st != OK) break;
        /* old triangles keep their costs: both lists are sorted triples, the old one a subset */
        real *ctn = (real *)calloc((size_t)(3 * Tn) + 1, sizeof(real));
        if (!ctn) return ERR_OOM;
        int64_t q = 0;
        for (int64_t t = 0; t < T; ++t) {
            while (q < Tn && tri_triple_cmp(tnn + 3 * q, tn + 3 * t) < 0) ++q;
            if (q >= Tn || tri_triple_cmp(tnn + 3 * q, tn + 3 * t) != 0) return ERR_GRAPH;
            for (int sl = 0; sl < 3; ++sl) ctn[3 * q + sl] = ct[3 * t + sl];
        }
        mp_state s;
        st = mp_init(&s, ma, ca, Tn, te, ctn);
        free(ctn);
        if (st != OK) break;
        real *msg = (real *)xmalloc((size_t)(3 * Tn) * sizeof(real));
        if (!msg) return ERR_OOM;
        for (int32_t it = 1; it <= k_iters; ++it) {
            mp_edges_to_triangles(&s);
            mp_triangles_to_edges(&s, msg);
        }
        free(msg);
        cur = mp_lower_bound(&s);
        for (int64_t e = 0; e < ma; ++e) ca[e] = (float)s.ce[e];
        free(tn); free(ct);
        tn = tnn; T = Tn;
        ct = (real *)xmalloc((size_t)(3 * Tn) * sizeof(real));
        if (!ct) return ERR_OOM;
        memcpy(ct, s.ct, (size_t)(3 * Tn) * sizeof(real));
        mp_free(&s);
        free(te);
        free(*gi); free(*gj); free(*gc);
        *gi = ia; *gj = ja; *gc = ca; *m = ma;
        done = d;
        if (lb_trace) lb_trace[d] = cur;
    }
    if (lb_trace) for (int32_t d = done + 1; d <= rounds; ++d) lb_trace[d] = cur;
    if (lb) *lb = cur;
    if (T_out) *T_out = T;
    if (tri_nodes_out) *tri_nodes_out = tn; else free(tn);
    if (ct_out) *ct_out = ct; else free(ct);
    return st == ERR_CAP ? OK : st;
}

/* The dual block on its own: any edge list in, augmented canonical graph with reparametrised costs
 * out (capacity edge_cap), LB after the last round, optional trace lb_trace[0..dual_rounds], and
 * optionally the final triangles (tri_nodes: 3*tri_cap int32, ct: 3*tri_cap float; n_tri_out always
 * gets the count, nothing is copied if tri_cap is too small). */
int rama_oracle_dual_rounds(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                            int32_t max_cycle_len, int32_t shortest_only, int32_t k_iters, int32_t dual_rounds,
                            int64_t edge_cap, int32_t *io, int32_t *jo, float *co, int64_t *m_out,
                            double *lower_bound, double *lb_trace,
                            int64_t tri_cap, int32_t *tri_nodes, float *ct, int64_t *n_tri_out)
{
    if (!m_out || k_iters < 0 || dual_rounds < 0 || max_cycle_len > MAX_CYCLE_LEN) return ERR_ARG;
    size_t mm = (size_t)(m > 0 ? m : 1);
    int32_t *gi = (int32_t *)xmalloc(mm * 4), *gj = (int32_t *)xmalloc(mm * 4);
    float *gc = (float *)xmalloc(mm * 4);
    if (!gi || !gj || !gc) return ERR_OOM;
    int64_t mc = 0, T = 0;
    int st = rama_oracle_canonicalise(n, m, i, j, c, gi, gj, gc, &mc);
    int32_t *tn = NULL;
    real *ctr = NULL;
    if (st == OK) st = dual_block(n, &mc, &gi, &gj, &gc, max_cycle_len, shortest_only, k_iters, dual_rounds,
                                  lower_bound, lb_trace, NULL, &tn, &ctr, &T);
    if (st == OK) {
        *m_out = mc;
        if (n_tri_out) *n_tri_out = T;
        if (mc > edge_cap) st = ERR_CAP;
        else {
            for (int64_t e = 0; e < mc; ++e) { io[e] = gi[e]; jo[e] = gj[e]; co[e] = gc[e]; }
            if (tri_nodes && ct && T <= tri_cap)
                for (int64_t q = 0; q < 3 * T; ++q) { tri_nodes[q] = tn[q]; ct[q] = (float)ctr[q]; }
        }
    }
    free(tn); free(ctr);
    free(gi); free(gj); free(gc);
    return st;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a4: contraction set S by handshake matching (Sec. 3.1 "Maximum matching"; the paper   */
/* names the scheme but gives no tie-break or round count).  Reading: candidates are edges     */
/* with c > tau; total order "larger cost first, then smaller edge position in the canonical   */
/* list"; in each round every still-unmatched node points at its best candidate edge whose     */
/* other endpoint is unmatched too; an edge both of whose endpoints point at it is matched.    */
/* Rounds repeat until no candidate joins two unmatched nodes or the cap is reached.           */
/* Input canonical.  mate[v] = partner or -1.  Returns the number of matched edges.            */
/* ------------------------------------------------------------------------------------------ */
int64_t rama_oracle_matching(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                             float tau, int32_t rounds_cap, int32_t *mate)
{
    int64_t *best = (int64_t *)xmalloc((size_t)n * sizeof(int64_t));
    int64_t matched = 0;
    if (!best) return ERR_OOM;
    for (int32_t v = 0; v < n; ++v) mate[v] = -1;
    for (int32_t r = 0; r < rounds_cap; ++r) {
        int64_t n_cand = 0;
        for (int32_t v = 0; v < n; ++v) best[v] = -1;
        for (int64_t e = 0; e < m; ++e) {
            if (!(c[e] > tau) || mate[i[e]] != -1 || mate[j[e]] != -1) continue;
            ++n_cand;
            int32_t ends[2] = { i[e], j[e] };
            for (int q = 0; q < 2; ++q) {
                int64_t b = best[ends[q]];
                if (b < 0 || c[e] > c[b]) best[ends[q]] = e;      /* ties keep the earlier edge */
            }
        }
        if (n_cand == 0) break;
        for (int64_t e = 0; e < m; ++e) {
            if (!(c[e] > tau) || mate[i[e]] != -1 || mate[j[e]] != -1) continue;
            if (best[i[e]] == e && best[j[e]] == e) { mate[i[e]] = j[e]; mate[j[e]] = i[e]; ++matched; }
        }
    }
    free(best);
    return matched;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a4, second strategy: maximum spanning forest without conflicts (Sec. 3.1).             */
/* The paper names Boruvka's algorithm and says: for every negative edge ij find the unique    */
/* i-j path in the forest (if there is one) and remove its smallest positive edge.  Reading:   */
/*  - the forest is the maximum spanning forest of the candidate edges (c > tau) under the     */
/*    same total order as the matching (larger cost first, then earlier canonical position);   */
/*    with a strict order it is unique, so Kruskal's algorithm gives the same forest;          */
/*  - all repulsive edges (c < 0) look at the forest as built; each marks the lowest edge of   */
/*    its path; all marked edges are removed together.  Then no repulsive edge has both        */
/*    endpoints in one component, so every join lowers the objective.                          */
/* Input canonical.  in_forest / removed (optional, [m]) flag the forest edges and the marked  */
/* ones; S = forest minus marked is written to si/sj (capacity n).  Returns |S|.               */
/* ------------------------------------------------------------------------------------------ */
static int32_t uf_find(int32_t *p, int32_t v);
typedef struct { float c; int64_t pos; } ranked_edge;
static int cmp_ranked_desc(const void *pa, const void *pb)
{
    const ranked_edge *x = (const ranked_edge *)pa, *y = (const ranked_edge *)pb;
    if (x->c != y->c) return x->c > y->c ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}
/* 1 if edge e ranks below edge f in the contraction order */
static int ranks_below(const float *c, int64_t e, int64_t f) { return c[e] < c[f] || (c[e] == c[f] && e > f); }

int64_t rama_oracle_forest_set(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c, float tau,
                               uint8_t *in_forest, uint8_t *removed, int32_t *si, int32_t *sj)
{
    ranked_edge *cand = (ranked_edge *)xmalloc((size_t)m * sizeof *cand);
    int32_t *uf = (int32_t *)xmalloc(((size_t)n + 1) * 4);
    uint8_t *inf = (uint8_t *)calloc((size_t)m + 1, 1), *rem = (uint8_t *)calloc((size_t)m + 1, 1);
    int64_t *adj_ptr = (int64_t *)calloc((size_t)n + 2, sizeof(int64_t));
    if (!cand || !uf || !inf || !rem || !adj_ptr) return ERR_OOM;
    /* Kruskal on the candidates in descending order */
    int64_t nc = 0;
    for (int64_t e = 0; e < m; ++e) if (c[e] > tau) { cand[nc].c = c[e]; cand[nc].pos = e; ++nc; }
    qsort(cand, (size_t)nc, sizeof *cand, cmp_ranked_desc);
    for (int32_t v = 0; v < n; ++v) uf[v] = v;
    int64_t nf = 0;
    for (int64_t q = 0; q < nc; ++q) {
        int64_t e = cand[q].pos;
        int32_t a = uf_find(uf, i[e]), b = uf_find(uf, j[e]);
        if (a == b) continue;
        if (a < b) uf[b] = a; else uf[a] = b;
        inf[e] = 1; ++nf;
    }
    /* adjacency of the forest */
    for (int64_t e = 0; e < m; ++e) if (inf[e]) { adj_ptr[i[e] + 1]++; adj_ptr[j[e] + 1]++; }
    for (int32_t v = 0; v < n; ++v) adj_ptr[v + 1] += adj_ptr[v];
    int64_t *adj_edge = (int64_t *)xmalloc((size_t)(2 * nf) * sizeof(int64_t));
    int64_t *fillp = (int64_t *)xmalloc(((size_t)n + 1) * sizeof(int64_t));
    int32_t *up = (int32_t *)xmalloc(((size_t)n + 1) * 4), *depth = (int32_t *)xmalloc(((size_t)n + 1) * 4);
    int32_t *tree = (int32_t *)xmalloc(((size_t)n + 1) * 4), *queue = (int32_t *)xmalloc(((size_t)n + 1) * 4);
    int64_t *up_edge = (int64_t *)xmalloc(((size_t)n + 1) * sizeof(int64_t));
    if (!adj_edge || !fillp || !up || !depth || !tree || !queue || !up_edge) return ERR_OOM;
    memcpy(fillp, adj_ptr, ((size_t)n + 1) * sizeof(int64_t));
    for (int64_t e = 0; e < m; ++e) if (inf[e]) { adj_edge[fillp[i[e]]++] = e; adj_edge[fillp[j[e]]++] = e; }
    /* root every tree (breadth first) */
    for (int32_t v = 0; v < n; ++v) depth[v] = -1;
    for (int32_t r = 0; r < n; ++r) {
        if (depth[r] >= 0) continue;
        int64_t head = 0, tail = 0;
        depth[r] = 0; up[r] = r; up_edge[r] = -1; tree[r] = r; queue[tail++] = r;
        while (head < tail) {
            int32_t v = queue[head++];
            for (int64_t p = adj_ptr[v]; p < adj_ptr[v + 1]; ++p) {
                int64_t e = adj_edge[p];
                int32_t w = i[e] == v ? j[e] : i[e];
                if (depth[w] >= 0) continue;
                depth[w] = depth[v] + 1; up[w] = v; up_edge[w] = e; tree[w] = r; queue[tail++] = w;
            }
        }
    }
    /* every repulsive edge inside a tree marks the lowest edge of its forest path */
    for (int64_t e = 0; e < m; ++e) {
        if (!(c[e] < 0.0f)) continue;
        int32_t a = i[e], b = j[e];
        if (tree[a] != tree[b]) continue;
        int64_t low = -1;
        while (a != b) {
            int64_t pe;
            if (depth[a] >= depth[b]) { pe = up_edge[a]; a = up[a]; } else { pe = up_edge[b]; b = up[b]; }
            if (low < 0 || ranks_below(c, pe, low)) low = pe;
        }
        if (low >= 0) rem[low] = 1;
    }
    int64_t ns = 0;
    for (int64_t e = 0; e < m; ++e) if (inf[e] && !rem[e]) { si[ns] = i[e]; sj[ns] = j[e]; ++ns; }
    if (in_forest) memcpy(in_forest, inf, (size_t)m);
    if (removed) memcpy(removed, rem, (size_t)m);
    free(cand); free(uf); free(inf); free(rem); free(adj_ptr); free(adj_edge); free(fillp);
    free(up); free(depth); free(tree); free(queue); free(up_edge);
    return ns;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a5: contraction mapping from S (Lemma 1(a)): f(u)=f(v) iff u,v are joined by a path in */
/* (V,S).  rep[v] = smallest node id of v's component; f'[v] = number of component             */
/* representatives smaller than rep[v].  Union-find with the smaller id as root.               */
/* ------------------------------------------------------------------------------------------ */
static int32_t uf_find(int32_t *p, int32_t v)
{
    while (p[v] != v) { p[v] = p[p[v]]; v = p[v]; }
    return v;
}
int rama_oracle_components(int32_t n, int64_t ns, const int32_t *si, const int32_t *sj,
                           int32_t *rep, int32_t *fmap, int32_t *n_out)
{
    for (int32_t v = 0; v < n; ++v) rep[v] = v;
    for (int64_t e = 0; e < ns; ++e) {
        if (si[e] < 0 || si[e] >= n || sj[e] < 0 || sj[e] >= n) return ERR_GRAPH;
        int32_t a = uf_find(rep, si[e]), b = uf_find(rep, sj[e]);
        if (a == b) continue;
        if (a < b) rep[b] = a; else rep[a] = b;
    }
    for (int32_t v = 0; v < n; ++v) rep[v] = uf_find(rep, v);
    int32_t cnt = 0;
    for (int32_t v = 0; v < n; ++v) if (rep[v] == v) fmap[v] = cnt++;
    for (int32_t v = 0; v < n; ++v) fmap[v] = fmap[rep[v]];
    if (n_out) *n_out = cnt;
    return OK;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a6: contraction of the graph under a mapping (Lemma 1(b); Lemma 3; Alg. "GPU           */
/* Edge-Contraction": relabel the endpoints, sort, add up parallel edges).  One entry per      */
/* undirected edge; entries whose endpoints fall together are the diagonal of K^T A K          */
/* (Lemma 3(b)) and leave the edge list.  Sums run in ascending input edge position.           */
/* Input canonical (only its order matters).  diag may be NULL.                                */
/* ------------------------------------------------------------------------------------------ */
int rama_oracle_contract_with_mapping(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                                      const int32_t *fmap, int32_t n_new,
                                      int32_t *io, int32_t *jo, float *co, int64_t *m_out, float *diag)
{
    keyed_edge *k = (keyed_edge *)xmalloc((size_t)m * sizeof *k);
    if (!k) return ERR_OOM;
    (void)n;
    for (int64_t e = 0; e < m; ++e) {
        int32_t a = fmap[i[e]], b = fmap[j[e]];
        k[e].a = a < b ? a : b; k[e].b = a < b ? b : a; k[e].pos = e; k[e].c = (real)c[e];
    }
    qsort(k, (size_t)m, sizeof *k, cmp_keyed_edge);
    if (diag) for (int32_t v = 0; v < n_new; ++v) diag[v] = 0.0f;
    int64_t o = 0;
    for (int64_t e = 0; e < m;) {
        real acc = k[e].c;
        int64_t f = e + 1;
        while (f < m && k[f].a == k[e].a && k[f].b == k[e].b) { acc = acc + k[f].c; ++f; }
        if (k[e].a == k[e].b) { if (diag) diag[k[e].a] = (float)acc; }
        else { io[o] = k[e].a; jo[o] = k[e].b; co[o] = (float)acc; ++o; }
        e = f;
    }
    free(k);
    *m_out = o;
    return OK;
}

/* One primal update (Alg. "Parallel-Edge-Contraction"): S by matching -- or, when the matching
 * joins fewer than forest_ratio*|V| pairs, by the spanning forest without conflicts (Sec. 3.1,
 * last paragraph of "Finding contraction edge set S"; forest_ratio <= 0 disables the switch) --
 * then f' by components and A' = K^T A K - diag.  Input canonical.  Returns |S| through n_matched. */
static int contract_once(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                         float tau, int32_t rounds_cap, float forest_ratio, int32_t *fmap, int32_t *n_new,
                         int32_t *io, int32_t *jo, float *co, int64_t *m_out, float *diag, int64_t *n_matched)
{
    int32_t *mate = (int32_t *)xmalloc((size_t)n * 4), *rep = (int32_t *)xmalloc((size_t)n * 4);
    int32_t *si = (int32_t *)xmalloc(((size_t)n + 1) * 4), *sj = (int32_t *)xmalloc(((size_t)n + 1) * 4);
    if (!mate || !rep || !si || !sj) return ERR_OOM;
    int64_t ns = rama_oracle_matching(n, m, i, j, c, tau, rounds_cap, mate);
    if (ns < 0) return (int)ns;
    if (ns > 0 && forest_ratio > 0.0f && (double)ns < (double)forest_ratio * (double)n) {
        ns = rama_oracle_forest_set(n, m, i, j, c, tau, NULL, NULL, si, sj);
        if (ns < 0) return (int)ns;
    } else {
        int64_t q = 0;
        for (int32_t v = 0; v < n; ++v) if (mate[v] > v) { si[q] = v; sj[q] = mate[v]; ++q; }
    }
    int st = rama_oracle_components(n, ns, si, sj, rep, fmap, n_new);
    if (st == OK) st = rama_oracle_contract_with_mapping(n, m, i, j, c, fmap, *n_new, io, jo, co, m_out, diag);
    *n_matched = ns;
    free(mate); free(rep); free(si); free(sj);
    return st;
}

/* Boundary-level contraction.  repeat=1: one primal update.  repeat=0: primal updates until no
 * edge with c>tau is left (the purely primal solver "P" of Sec. 4).  mapping: original node ->
 * final node.  diag (optional): diagonal of K^T A K for the composed mapping, i.e. for every
 * final node the sum of the input edges inside it, added in canonical edge order. */
int rama_oracle_contract(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                         float tau, int32_t rounds_cap, float forest_ratio, int32_t repeat,
                         int32_t *mapping, int32_t *io, int32_t *jo, float *co, float *diag,
                         int32_t *n_out, int64_t *m_out)
{
    if (!mapping || !n_out || !m_out) return ERR_ARG;
    size_t mm = (size_t)(m > 0 ? m : 1);
    int32_t *ci = (int32_t *)xmalloc(mm * 4), *cj = (int32_t *)xmalloc(mm * 4);
    float *cc = (float *)xmalloc(mm * 4);
    int32_t *gi = (int32_t *)xmalloc(mm * 4), *gj = (int32_t *)xmalloc(mm * 4);
    float *gc = (float *)xmalloc(mm * 4);
    int32_t *ni = (int32_t *)xmalloc(mm * 4), *nj = (int32_t *)xmalloc(mm * 4);
    float *nc = (float *)xmalloc(mm * 4);
    int32_t *fm = (int32_t *)xmalloc(((size_t)n + 1) * 4);
    if (!ci || !cj || !cc || !gi || !gj || !gc || !ni || !nj || !nc || !fm) return ERR_OOM;
    int64_t mc = 0;
    int st = rama_oracle_canonicalise(n, m, i, j, c, ci, cj, cc, &mc);
    if (st != OK) goto done;
    memcpy(gi, ci, (size_t)mc * 4); memcpy(gj, cj, (size_t)mc * 4); memcpy(gc, cc, (size_t)mc * 4);
    int32_t ncur = n; int64_t mcur = mc;
    for (int32_t v = 0; v < n; ++v) mapping[v] = v;
    for (;;) {
        int32_t nn = 0; int64_t mn = 0, ns = 0;
        st = contract_once(ncur, mcur, gi, gj, gc, tau, rounds_cap, forest_ratio, fm, &nn, ni, nj, nc, &mn, NULL, &ns);
        if (st != OK) goto done;
        if (ns == 0) break;
        for (int32_t v = 0; v < n; ++v) mapping[v] = fm[mapping[v]];       /* f <- f' o f */
        memcpy(gi, ni, (size_t)mn * 4); memcpy(gj, nj, (size_t)mn * 4); memcpy(gc, nc, (size_t)mn * 4);
        ncur = nn; mcur = mn;
        if (repeat) break;
    }
    if (io) memcpy(io, gi, (size_t)mcur * 4);
    if (jo) memcpy(jo, gj, (size_t)mcur * 4);
    if (co) memcpy(co, gc, (size_t)mcur * 4);
    *n_out = ncur; *m_out = mcur;
    if (diag) {
        int64_t dummy = 0;
        st = rama_oracle_contract_with_mapping(n, mc, ci, cj, cc, mapping, ncur, ni, nj, nc, &dummy, diag);
    }
done:
    free(ci); free(cj); free(cc); free(gi); free(gj); free(gc); free(ni); free(nj); free(nc); free(fm);
    return st;
}

/* ------------------------------------------------------------------------------------------ */
/* Objective (eq. 2): cost of the multicut induced by node labels, on the given edge costs.    */
/* ------------------------------------------------------------------------------------------ */
double rama_oracle_multicut_cost(int64_t m, const int32_t *i, const int32_t *j, const float *c, const int32_t *labels)
{
    double acc = 0.0;
    for (int64_t e = 0; e < m; ++e) if (labels[i[e]] != labels[j[e]]) acc += (double)c[e];
    return acc;
}

/* ------------------------------------------------------------------------------------------ */
/* Step a7 + driver: Alg. "Primal-Dual Multicut".                                              */
/* Round r: separate cycles up to length L_r (first round / later rounds, Sec. 4 "PD"), run    */
/* k_r message-passing iterations, contract on the reparametrised costs, compose f.  Stop when */
/* the contraction set is empty.  The lower bound is the one recorded on the original graph    */
/* (round 1).  labels[v] = smallest original node id in v's cluster.                           */
/* shortest_only: the separation keeps, per repulsive edge, only its shortest cycles (step a1). */
/* dual_rounds: separation + k message-passing iterations are repeated that many times on the  */
/* graph of a round before it is contracted (1 = the paper's loop; see dual_block).            */
/* stats (optional, int64[5+N_LISTS]): rounds, clusters, |T|, |E'| of round 1, final edges,     */
/* then the number of 3-,4-,..,MAX_CYCLE_LEN-cycles of round 1                                 */
/* ------------------------------------------------------------------------------------------ */
int rama_oracle_solve(int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                      int32_t max_cycle_len_first, int32_t max_cycle_len_later, int32_t shortest_only,
                      int32_t dual_rounds, int32_t mp_iters_first, int32_t mp_iters_later,
                      int32_t matching_rounds_cap, float tau, float forest_ratio, int32_t max_rounds,
                      int32_t *labels, double *primal_cost, double *lower_bound, int64_t *stats)
{
    if (!labels || n < 0) return ERR_ARG;
    size_t mm = (size_t)(m > 0 ? m : 1);
    int32_t *gi = (int32_t *)xmalloc(mm * 4), *gj = (int32_t *)xmalloc(mm * 4);
    float *gc = (float *)xmalloc(mm * 4);
    int32_t *f = (int32_t *)xmalloc(((size_t)n + 1) * 4), *fm = (int32_t *)xmalloc(((size_t)n + 1) * 4);
    if (!gi || !gj || !gc || !f || !fm) return ERR_OOM;
    int64_t mcur = 0;
    int st = rama_oracle_canonicalise(n, m, i, j, c, gi, gj, gc, &mcur);
    if (st != OK) { free(gi); free(gj); free(gc); free(f); free(fm); return st; }
    int32_t ncur = n;
    for (int32_t v = 0; v < n; ++v) f[v] = v;
    double lb = 0.0;
    int have_lb = 0;
    int64_t st_rounds = 0, st_c[N_LISTS] = { 0 }, st_T = 0, st_ma = 0;
    if (max_cycle_len_first > MAX_CYCLE_LEN || max_cycle_len_later > MAX_CYCLE_LEN) { st = ERR_ARG; goto fail; }
    for (int32_t round = 1; max_rounds <= 0 || round <= max_rounds; ++round) {
        int32_t Lmax = round == 1 ? max_cycle_len_first : max_cycle_len_later;
        int32_t k = round == 1 ? mp_iters_first : mp_iters_later;
        if (Lmax >= 3 && k > 0) {
            /* dual part: separation + message passing, dual_rounds times on this graph */
            double lbr = 0.0;
            st = dual_block(ncur, &mcur, &gi, &gj, &gc, Lmax, shortest_only, k, dual_rounds, &lbr, NULL,
                            round == 1 ? st_c : NULL, NULL, NULL, round == 1 ? &st_T : NULL);
            if (st != OK) goto fail;
            if (round == 1) { lb = lbr; have_lb = 1; st_ma = mcur; }
        }
        if (round == 1 && !have_lb) {
            for (int64_t e = 0; e < mcur; ++e) if (gc[e] < 0) lb += (double)gc[e];
            have_lb = 1; st_ma = mcur;
        }
        /* primal update on the reparametrised costs */
        size_t mq = (size_t)(mcur > 0 ? mcur : 1);
        int32_t *ni = (int32_t *)xmalloc(mq * 4), *nj = (int32_t *)xmalloc(mq * 4);
        float *nc = (float *)xmalloc(mq * 4);
        int32_t nn = 0; int64_t mn = 0, ns = 0;
        if (!ni || !nj || !nc) { st = ERR_OOM; goto fail; }
        st = contract_once(ncur, mcur, gi, gj, gc, tau, matching_rounds_cap, forest_ratio, fm, &nn, ni, nj, nc, &mn, NULL, &ns);
        if (st != OK) goto fail;
        st_rounds = round;
        if (ns == 0) { free(ni); free(nj); free(nc); break; }
        for (int32_t v = 0; v < n; ++v) f[v] = fm[f[v]];
        free(gi); free(gj); free(gc);
        gi = ni; gj = nj; gc = nc; ncur = nn; mcur = mn;
    }
    {   /* labels: smallest original id per cluster */
        int32_t *first = (int32_t *)xmalloc(((size_t)ncur + 1) * 4);
        for (int32_t a = 0; a < ncur; ++a) first[a] = -1;
        for (int32_t v = 0; v < n; ++v) if (first[f[v]] < 0) first[f[v]] = v;
        for (int32_t v = 0; v < n; ++v) labels[v] = first[f[v]];
        free(first);
    }
    if (primal_cost) *primal_cost = rama_oracle_multicut_cost(m, i, j, c, labels);
    if (lower_bound) *lower_bound = lb;
    if (stats) {
        stats[0] = st_rounds; stats[1] = ncur; stats[2] = st_T; stats[3] = st_ma; stats[4] = mcur;
        for (int q = 0; q < N_LISTS; ++q) stats[5 + q] = st_c[q];
    }
    st = OK;
fail:
    free(gi); free(gj); free(gc); free(f); free(fm);
    return st;
}

int32_t rama_oracle_real_bytes(void) { return (int32_t)sizeof(real); }
