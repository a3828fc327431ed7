/*
 * rama.h -- C ABI of the MI355X (gfx950) primal-dual multicut library.
 *
 * The library implements one round -- and the loop over rounds -- of the primal-dual
 * multicut algorithm of "RAMA: A Rapid Multicut Algorithm on GPU" (arXiv 2109.01838):
 * conflicted-cycle separation, edge<->triangle message passing, and parallel edge
 * contraction.  Every step runs in hand-written HIP kernels on one GPU.
 *
 * Problem statement (paper Sec. 3, eq. 2): an undirected graph with `n_nodes` nodes and
 * `n_edges` edges given as endpoint arrays i[], j[] (int32) and costs c[] (fp32).
 * c > 0: attractive (the endpoints want to share a cluster); c < 0: repulsive; c == 0:
 * neither.  The objective is the sum of the costs of the edges whose endpoints end up in
 * different clusters.
 *
 * General conventions
 *   - "device" pointers are HIP device memory valid on the ctx's device; "host" pointers are
 *     ordinary host memory.  All graph arrays are DEVICE pointers; all scalar results are
 *     HOST pointers.
 *   - The caller owns every input and output buffer.  Inputs are never modified.  The
 *     library keeps no reference to caller memory after a call returns.  Workspace is
 *     allocated through the ctx -- with the allocator callbacks given to rama_create, else
 *     with hipMalloc -- cached for reuse, and released by rama_destroy.
 *   - Every call enqueues its kernels on the ctx's stream and synchronises that stream
 *     before it returns (scalar results are on the host when the call returns).
 *   - Any edge list is accepted: either orientation, self-loops (dropped; they can never
 *     be cut) and duplicate / antiparallel edges (their costs are added in input order,
 *     Lemma 1(b)).  A "canonical" edge list has i<j, is sorted by (i,j) and has no
 *     duplicates; all edge lists the library RETURNS are canonical.
 *   - No exception crosses the boundary; every call returns a rama_status.  On failure
 *     outputs are unspecified unless stated otherwise; rama_last_error() describes the
 *     failure.  Endpoints outside [0,n_nodes) and non-finite costs give RAMA_ERR_BAD_GRAPH.
 *   - Element counts of any one array must stay below 2^31 (RAMA_ERR_CAPACITY otherwise).
 *   - One ctx must not be used from two threads at once.
 */
#ifndef RAMA_H
#define RAMA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rama_ctx rama_ctx; /* opaque: device, stream, cached workspace, last error */

/* Longest conflicted cycle the separation can look for.  The paper stops at 5 (Sec. 4) and
 * lists longer cycles as future work (Sec. 5); 6 and 7 come from the same search. */
#define RAMA_MAX_CYCLE_LEN 7

typedef enum {
    RAMA_OK = 0,
    RAMA_ERR_INVALID_ARG = -1, /* null pointer, negative size, cycle length out of range, ... */
    RAMA_ERR_BAD_GRAPH = -2,   /* endpoint out of range, non-finite cost, a cycle that is not in the graph */
    RAMA_ERR_CAPACITY = -3,    /* a caller buffer is too small (needed sizes are written) or a count reaches 2^31 */
    RAMA_ERR_OOM = -4,         /* the workspace allocator (callbacks or hipMalloc) returned no memory */
    RAMA_ERR_HIP = -5          /* any other HIP runtime error */
} rama_status;

/* Parameters of the primal-dual loop (paper Alg. "Primal-Dual Multicut" and Sec. 4, solver
 * variants).  rama_params_default() fills the values of solver "PD". */
typedef struct {
    int32_t max_cycle_len_first;  /* longest conflicted cycle separated on the original graph: 5 (0 = no separation) */
    int32_t max_cycle_len_later;  /* ... on contracted graphs: 3 for "PD", 5 for "PD+" */
    int32_t mp_iters_first;       /* message-passing iterations k in the first round: 10 */
    int32_t mp_iters_later;       /* ... in later rounds: 5 */
    int32_t matching_rounds_cap;  /* upper limit on handshake rounds per matching: 32 */
    float contract_threshold;     /* tau: an edge is a contraction candidate iff c > tau; 0 */
    float forest_ratio;           /* if the matching joins fewer than forest_ratio*|V| pairs, S is the spanning
                                     forest without conflicts instead; 0.1 (<= 0: matching only) */
    int32_t max_rounds;           /* stop after this many rounds; <=0: until no candidate edge is left */
    int32_t shortest_cycles_only; /* != 0: per repulsive edge keep only its shortest conflicted cycles; 0 */
    int32_t dual_rounds;          /* separation + k message-passing iterations are repeated this often on the
                                     graph of a round before it is contracted, see rama_dual_rounds; 1 */
} rama_params;

/* What rama_solve did (all host memory). */
typedef struct {
    int32_t rounds;             /* rounds of the outer loop that ran */
    int32_t n_clusters;         /* clusters in the result */
    int64_t n_cycles_first[RAMA_MAX_CYCLE_LEN - 2]; /* conflicted 3-, 4-, .. cycles found on the original graph */
    int64_t n_triangles_first;  /* triangles after triangulation, first round */
    int64_t n_edges_aug_first;  /* edges after adding chords, first round */
    int64_t n_edges_final;      /* edges of the last contracted graph */
    double ms_total;            /* wall time of the call */
    double ms_cycles, ms_dual, ms_contract, ms_other; /* split by stage: stream time between HIP events recorded at
                                   the stage boundaries (no extra synchronisation), ms_other = the rest of ms_total; with
                                   dual_rounds > 1 separation and message passing interleave and are both booked as ms_cycles */
} rama_stats;

/* One round of the outer loop of rama_solve (all host memory); see rama_round_get. */
typedef struct {
    int32_t n_nodes;            /* nodes of the graph the round started from */
    int32_t used_forest;        /* 1: S came from the spanning forest without conflicts, 0: from the matching */
    int64_t n_edges;            /* its edges */
    int64_t n_attractive;       /* edges with c > 0 / c < 0 when the round started; -1 if the round did not separate */
    int64_t n_repulsive;
    int64_t n_cycles[RAMA_MAX_CYCLE_LEN - 2]; /* conflicted 3-, 4-, .. cycles separated in this round */
    int64_t n_triangles;        /* triangles the message passing ran on */
    int64_t n_edges_aug;        /* edges after adding chords */
    int64_t n_contracted;       /* |S| */
    int64_t workspace_peak;     /* largest number of workspace bytes in use at one time during the round */
    double ms_cycles, ms_dual, ms_contract; /* stream time between stage marks (HIP events) */
} rama_round_stats;

/* Optional source of device workspace (for instance a framework's caching allocator).  alloc returns
 * device memory of at least `bytes` bytes, aligned to 256 bytes, on the ctx's device, or NULL when it
 * has none (the call in progress then ends with RAMA_ERR_OOM and the ctx stays usable); free takes back
 * a block alloc returned.  Both are called from the thread that calls into the library, only while such
 * a call runs; blocks are cached by the ctx and go back in rama_destroy (or earlier, when an allocation
 * fails and the cache is given up before one more attempt). */
typedef struct {
    void *(*alloc)(void *user, size_t bytes);
    void (*free)(void *user, void *ptr);
    void *user;
} rama_alloc;

/* Create a context on the current HIP device.  `hip_stream` is a hipStream_t (may be NULL
 * for the default stream) on which all work is enqueued; the caller keeps ownership of it.
 * `alloc` (may be NULL: hipMalloc / hipFree) is copied; alloc->alloc must then be non-NULL. */
rama_status rama_create(rama_ctx **out, void *hip_stream, const rama_alloc *alloc);
/* Free the workspace and the context.  NULL is allowed. */
rama_status rama_destroy(rama_ctx *ctx);
/* Text for the last failure on this ctx; owned by the ctx, valid until the next call. */
const char *rama_last_error(const rama_ctx *ctx);
/* Defaults of solver "PD" (Sec. 4): cycles up to 5 then 3, k = 10 then 5, tau = 0. */
void rama_params_default(rama_params *p);
/* Bytes of device workspace currently cached by the ctx. */
int64_t rama_workspace_bytes(const rama_ctx *ctx);
/* Per-round record of the last rama_solve on this ctx (metrics, not an operation of the paper):
 * rama_round_count rounds are held, rama_round_get copies round `index` (0-based) to *out. */
int32_t rama_round_count(const rama_ctx *ctx);
rama_status rama_round_get(const rama_ctx *ctx, int32_t index, rama_round_stats *out);

/*
 * Measurement hooks (not operations of the paper): per-kernel timers for roofline reports.
 * While enabled, every kernel launch of the library is bracketed by two HIP events on the ctx
 * stream (the triangle update of the message passing stamps its events from the dispatch itself) and
 * accounted under the kernel's name together with the algorithmic bytes that launch
 * has to move (the launch site computes them from the array sizes).  Enabling resets the
 * accumulators; `only` (may be NULL) restricts the timers to kernels whose name starts with it -- or with
 * one of several prefixes separated by '|' -- which keeps the event overhead out of a timed region.  rama_profile_get returns entry `index` in [0, rama_profile_count): name
 * (owned by the library), number of launches, summed milliseconds, summed algorithmic bytes.
 */
rama_status rama_profile_enable(rama_ctx *ctx, int32_t on, const char *only);
int32_t rama_profile_count(const rama_ctx *ctx);
rama_status rama_profile_get(const rama_ctx *ctx, int32_t index, const char **name, int64_t *launches, double *ms,
                             double *bytes);

/*
 * Tuning hook (not an operation of the paper).  The library sorts with stable 8-bit radix passes.
 * An array of at least `n_min` elements is instead sorted by passes over its top key bits followed
 * by one sort of the remaining bits inside LDS, provided that replaces at least
 * `min_passes_replaced` passes.  Both ways are the same stable sort, so no result depends on the
 * setting.  Defaults: 2^21 and 2.  (0, 0) sends every array that way, (INT64_MAX, any) none.
 * Independently of n_min, an array short enough for one workgroup (8192 keys of up to 32 bits, 4096 wider
 * ones) is sorted inside LDS by a single launch, unless n_min is INT64_MAX.
 */
rama_status rama_set_sort_split(rama_ctx *ctx, int64_t n_min, int32_t min_passes_replaced);

/*
 * Tuning hook (not an operation of the paper).  Three searches produce the same cycle lists:
 *   1  the walk: one thread per repulsive edge (v0,vL) walks v0 -> v1 -> v2 -> .. over attractive edges and
 *      tests every node it reaches against N+(vL); its last level fetches one row per path;
 *   3  the same walk, but its last level closes from vL's side as in the appendix algorithm "Parallel Conf.
 *      5-Cycles" (pairs (v1,v3) of N+(v0) x N+(vL) meeting in a common neighbour): the rows of N+(vL)'s
 *      entries are fetched once per repulsive edge and held in registers (rows of up to 8 entries);
 *   2  the cooperative search for lengths 4 and 5: sixteen lanes per repulsive edge, N+(v0), N+(vL) and
 *      the rows of N+(vL)'s entries staged in LDS (rows of up to 16 entries; edges with longer rows are
 *      walked as in 3), hits placed by ballots and prefix sums over the sixteen lanes.
 * Searches for triangles only (max_cycle_len 3) are row intersections: by one thread per repulsive edge
 * (modes 1 and 3), or by sixteen lanes per edge that bisect the longer row for sixteen entries of the shorter
 * one at a time (mode 2).
 * mode 0 (default) chooses from the sizes of the graph: for lengths 4-5 between 2 and 3, for triangles the
 * sixteen-lane search when the attractive rows hold more than 12 entries on average.
 */
rama_status rama_set_cycle_search(rama_ctx *ctx, int32_t mode);

/*
 * Conflicted-cycle separation (Sec. 3.2.2, definition "Conflicted cycles", and the appendix
 * algorithm "Parallel Conf. 5-Cycles"): every simple cycle of length L in {3,..,max_cycle_len}
 * with exactly one repulsive edge and L-1 attractive edges.  The paper separates up to length 5
 * and names longer cycles as an open improvement (Sec. 5); lengths up to RAMA_MAX_CYCLE_LEN are
 * found by the same depth-first walk.
 *
 * A cycle is stored as the node tuple (v0,...,v_{L-1}) where (v0,v_{L-1}) is its repulsive
 * edge, v0 < v_{L-1}, and v0,v1,...,v_{L-1} is the attractive path.  Each list is ordered by
 * (v0, v_{L-1}, v1, ..., v_{L-2}): grouped by repulsive edge, then lexicographic along the path.
 * List q (q = 0 .. max_cycle_len-3) holds the cycles of length q+3.
 *
 *   i, j, c            device, [n_edges]
 *   max_cycle_len      3 .. RAMA_MAX_CYCLE_LEN
 *   shortest_only      != 0: the separation lemma of Sec. 3.2.2 taken literally -- per repulsive
 *                      edge only the cycles along its shortest attractive paths (hop count) are
 *                      reported, all of them, and none if that length exceeds max_cycle_len
 *   cap                host, [max_cycle_len-2]: capacity of each list, in cycles; NULL = all 0
 *   cycles             host array of max_cycle_len-2 device pointers, list q has room for
 *                      (q+3)*cap[q] int32; an entry may be NULL when its cap is 0; the array
 *                      itself may be NULL when every cap is 0
 *   n_cycles_out       host, [max_cycle_len-2]: number of cycles found per length (always written
 *                      on RAMA_OK and RAMA_ERR_CAPACITY)
 * RAMA_ERR_CAPACITY if any list does not fit; then nothing is written to the lists, and
 * calling again with the reported counts succeeds (calling with cap = NULL is the way to
 * size the buffers).  Also RAMA_ERR_CAPACITY if a list would reach 2^31 entries.
 */
rama_status rama_find_conflicted_cycles(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges,
                                        const int32_t *i, const int32_t *j, const float *c,
                                        int32_t max_cycle_len, int32_t shortest_only, const int64_t *cap,
                                        int32_t *const *cycles, int64_t *n_cycles_out);

/*
 * Dual update of one round (Sec. 3.2.1 Lagrange decomposition, eq. 5 and 6; Sec. 3.2.3,
 * algorithm "Parallel-Message-Passing"; inner loop of "Primal-Dual Multicut"):
 * triangulate the given cycles, run k_iters iterations of edge->triangle and
 * triangle->edge message passing, and return the reparametrised graph.
 *
 * Triangulation (the paper leaves the rule open): a cycle (v0,...,v_{L-1}) becomes the
 * triangles {v0,v_m,v_{m+1}}, m=1..L-2; a chord (v0,v_m) that is not yet an edge is added
 * with cost 0.  The triangle set is the sorted set of distinct node triples.
 *
 *   max_cycle_len      2 .. RAMA_MAX_CYCLE_LEN: max_cycle_len-2 lists follow (2: none)
 *   cycles, n_cycles   host arrays [max_cycle_len-2]: device list q holds n_cycles[q] cycles of
 *                      length q+3 in the format of rama_find_conflicted_cycles (any order);
 *                      every cycle edge must be an edge of the graph, nodes distinct
 *   k_iters            >= 0
 *   edge_cap           capacity of i_out/j_out/c_out; n_edges + sum_q q*n_cycles[q] always suffices
 *   i_out,j_out,c_out  device: canonical edge list incl. new chords, c_out = reduced costs c^lambda (eq. 6a)
 *   n_edges_out        host: number of edges written (needed size on RAMA_ERR_CAPACITY)
 *   lower_bound        host, optional: LB(lambda) of eq. 5 after the last iteration
 *   lb_trace           host, optional, [k_iters+1]: LB before the first and after every iteration
 */
rama_status rama_message_passing(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges,
                                 const int32_t *i, const int32_t *j, const float *c,
                                 int32_t max_cycle_len, const int32_t *const *cycles, const int64_t *n_cycles,
                                 int32_t k_iters, int64_t edge_cap,
                                 int32_t *i_out, int32_t *j_out, float *c_out, int64_t *n_edges_out,
                                 double *lower_bound, double *lb_trace);

/*
 * The dual part of a round, repeated on one graph (Sec. 3.2; with dual_rounds = 1 it is the
 * separation and the inner loop of algorithm "Primal-Dual Multicut" in one call; more rounds are
 * the cutting-plane loop behind the better separation that Sec. 5 asks for): each round separates
 * the conflicted cycles of the *current* reparametrised costs, adds their triangles to the triangle
 * set -- triangles found in earlier rounds stay and keep their costs c_t, new ones start at zero --
 * and runs k_iters message-passing iterations over the whole set.  LB(lambda) never decreases from
 * round to round.  The loop ends early when a separation finds no cycle.
 *
 *   params             used: max_cycle_len_first (cycle length of every round), mp_iters_first
 *                      (k_iters), shortest_cycles_only, dual_rounds (>= 0)
 *   edge_cap, i_out, j_out, c_out, n_edges_out   as in rama_message_passing; the needed size is
 *                      not known beforehand: on RAMA_ERR_CAPACITY it is written to n_edges_out
 *   lower_bound        host, optional: LB(lambda) after the last round (the sum of the negative costs
 *                      if no round found a cycle)
 *   lb_trace           host, optional, [dual_rounds+1]: LB before the first and after every round
 *                      (rounds that did not run repeat the last value)
 *   n_triangles_out    host, optional: size of the triangle set at the end
 */
rama_status rama_dual_rounds(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges,
                             const int32_t *i, const int32_t *j, const float *c, const rama_params *params,
                             int64_t edge_cap, int32_t *i_out, int32_t *j_out, float *c_out, int64_t *n_edges_out,
                             double *lower_bound, double *lb_trace, int64_t *n_triangles_out);

/*
 * Primal update (Sec. 3.1: Lemma 1, Lemma 3, algorithm "Parallel-Edge-Contraction", "Finding
 * contraction edge set S: Maximum matching"; appendix algorithm "GPU Edge-Contraction").
 * S is a handshake matching on the edges with c > params->contract_threshold (larger cost
 * wins, ties go to the edge that comes first in the canonical list).  If it joins fewer than
 * params->forest_ratio * n_nodes pairs, S is instead the maximum spanning forest of those edges
 * (same edge order) minus, for every repulsive edge whose endpoints share a tree, the
 * lowest-ranked edge on its tree path ("Maximum spanning forest without conflicts").  The
 * contraction mapping
 * is the connected-component map of (V,S), numbered by ascending smallest member; the
 * contracted graph is K^T A K without its diagonal.
 *
 *   repeat             1: one primal update.  0: repeat until no edge with c > tau is left
 *                      (the purely primal solver "P" of Sec. 4)
 *   mapping            device, [n_nodes]: node -> node of the contracted graph, in [0,*n_nodes_out)
 *   i_out,j_out,c_out  device, capacity n_edges each: canonical contracted edge list
 *   diag_out           device, optional, [n_nodes]: first *n_nodes_out entries = diagonal of
 *                      K^T A K (Lemma 3(b)): per new node the summed cost of the input edges inside it
 *   n_nodes_out, n_edges_out   host
 * If no edge qualifies the mapping is the identity and the output is the canonical input.
 */
rama_status rama_contract(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges,
                          const int32_t *i, const int32_t *j, const float *c,
                          const rama_params *params, int32_t repeat,
                          int32_t *mapping, int32_t *i_out, int32_t *j_out, float *c_out, float *diag_out,
                          int32_t *n_nodes_out, int64_t *n_edges_out);

/*
 * The whole solver (algorithm "Primal-Dual Multicut"): repeat { separate conflicted cycles;
 * k message-passing iterations; contract on the reduced costs; compose the mapping } until
 * the contraction set is empty.
 *
 *   labels        device, [n_nodes]: label of a node = smallest node id in its cluster
 *   primal_cost   host, optional: cost (eq. 2) of the returned clustering on the input costs
 *   lower_bound   host, optional: LB(lambda) recorded after message passing on the original graph
 *   stats         host, optional
 */
rama_status rama_solve(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges,
                       const int32_t *i, const int32_t *j, const float *c, const rama_params *params,
                       int32_t *labels, double *primal_cost, double *lower_bound, rama_stats *stats);

/*
 * rama_solve for callers that cannot allocate device memory while they run -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result (bit for
 * bit) as rama_solve, but every byte of device workspace is taken from a static array of
 * RAMA_STATIC_SCRATCH_BYTES that the library holds on each GPU it runs on from load time to process end,
 * and the call itself calls no hipMalloc / hipFree, no allocator callback and no allocating library routine.
 *
 * Limits: n_nodes <= RAMA_STATIC_MAX_NODES and n_edges <= RAMA_STATIC_MAX_EDGES, else RAMA_ERR_CAPACITY
 * (nothing is run).  How much workspace a graph inside these limits needs depends on how many conflicted
 * cycles it has; if the array does not suffice the call returns RAMA_ERR_OOM ("static scratch exhausted").
 * All calls on one GPU, from any ctx, share that GPU's array: calls that overlap in time on one GPU race.
 * Nothing is kept in the array between calls.  Per-kernel timers (rama_profile_enable) are not collected
 * during this call.
 */
#define RAMA_STATIC_SCRATCH_BYTES (64u << 20)
#define RAMA_STATIC_MAX_NODES (1 << 17)
#define RAMA_STATIC_MAX_EDGES (1 << 18)
rama_status rama_solve_static(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges,
                              const int32_t *i, const int32_t *j, const float *c, const rama_params *params,
                              int32_t *labels, double *primal_cost, double *lower_bound, rama_stats *stats);

#ifdef __cplusplus
}
#endif
#endif /* RAMA_H */
