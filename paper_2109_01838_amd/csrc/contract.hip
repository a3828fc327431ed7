// Steps a4-a6: one primal update (paper Sec. 3.1: Lemma 1, Lemma 3, algorithm
// "Parallel-Edge-Contraction", "Maximum matching"; appendix algorithm "GPU Edge-Contraction").
//
//   S   : handshake matching on the edges with c > tau.  Edges are ranked by (cost, position in
//         the canonical list) packed into one 64-bit word, so "each node points at its best
//         incident candidate" is an integer atomicMax per endpoint -- order independent, hence
//         deterministic.  An edge both of whose endpoints point at it is matched; rounds repeat
//         on the shrinking list of edges whose endpoints are both still free (two kernels per
//         round: accept, then compaction of the survivors fused with their next proposals); the
//         list carries endpoints and rank word, so a round streams it and touches no edge array.
//   f'  : connected components of (V,S) by min-label hooking + pointer jumping; a component is
//         represented by its smallest node; new ids are the ranks of the representatives.
//   S'  : when the matching joins fewer than forest_ratio*|V| pairs: maximum spanning forest of the
//         candidate edges (Boruvka rounds with the same atomicMax ranks) minus, for every
//         repulsive edge inside a tree, the lowest edge of its tree path (trees rooted breadth
//         first, paths walked up from both ends).
//   A'  : endpoints relabelled through f', re-oriented, sorted by (row, col) with the cost as
//         payload (stable), runs of equal pairs summed in order, loops dropped.
#include "prim.h"

namespace rama {

namespace {

__device__ __forceinline__ uint32_t ordered_bits(float x)
{
    uint32_t u = __float_as_uint(x + 0.0f);   // -0 and +0 rank alike
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ unsigned long long edge_rank(float cost, uint32_t e)
{
    return ((unsigned long long)ordered_bits(cost) << 32) | (unsigned long long)(0xFFFFFFFFu - e);
}

struct CandFlag {
    static constexpr int bytes = 4;   // bytes read per item
    static constexpr const char *tag = "CandFlag";
    const float *c;
    float tau;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return c[e] > tau ? 1u : 0u; }
};

// consumer of the scan over CandFlag: the list of candidate edges
struct CollectEmit {
    static constexpr const char *tag = "Collect";
    uint32_t *act;
    __device__ __forceinline__ void operator()(size_t e, uint32_t cand, uint32_t p) const
    {
        if (cand) act[p] = (uint32_t)e;
    }
};

// Both endpoints of a candidate edge learn its rank.  The candidate list of the first round is
// in canonical order, so neighbouring lanes often share the first endpoint: those lanes combine
// their ranks with shuffles and only the last lane of a run issues the atomic.  (Combining any
// two lanes with the same node is valid whatever the list order; runs only make it pay.)
__device__ __forceinline__ void propose_edge(bool valid, int32_t u, int32_t v, unsigned long long r,
                                             unsigned long long *best)
{
    const int lane = lane_id();
    unsigned long long ru = valid ? r : 0ull;
    const int32_t key = valid ? u : -1 - lane;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        unsigned long long other_r = __shfl_up(ru, off, 64);
        int32_t other_k = __shfl_up(key, off, 64);
        if (lane >= off && other_k == key && other_r > ru) ru = other_r;
    }
    const int32_t next_k = __shfl_down(key, 1, 64);
    if (valid) {
        if (lane == 63 || next_k != key) atomicMax(&best[u], ru);
        atomicMax(&best[v], r);
    }
}

// The matching keeps its candidates packed -- endpoints and rank word, 16 bytes per candidate in three
// arrays -- so that a handshake round reads its list contiguously instead of reaching through the edge
// id into i, j and c of an ever sparser subset of the edges.
struct Cands {
    int32_t *u, *v;
    unsigned long long *r;
};
// consumer of the scan over CandFlag: the packed candidate list; with `best` set, the candidates also make
// the proposals of the first handshake round on the way (the list is then not read once more just for that)
struct PackCandsEmit {
    static constexpr const char *tag = "PackCands";
    static constexpr bool whole_wave = true;
    const int32_t *i, *j;
    const float *c;
    Cands out;
    unsigned long long *best;
    __device__ __forceinline__ void operator()(size_t e, uint32_t cand, uint32_t p) const
    {
        int32_t u = 0, v = 0;
        unsigned long long r = 0ull;
        if (cand) {
            u = i[e]; v = j[e];
            r = edge_rank(c[e], (uint32_t)e);
            out.u[p] = u; out.v[p] = v; out.r[p] = r;
        }
        if (best) propose_edge(cand != 0u, u, v, r, best);   // uniform
    }
};

// first proposals as a launch of their own (short lists, see matching())
__global__ __launch_bounds__(kBlock) void k_propose(size_t na, Cands a, unsigned long long *best)
{
    size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x;
    const bool valid = k < na;
    propose_edge(valid, valid ? a.u[k] : 0, valid ? a.v[k] : 0, valid ? a.r[k] : 0ull, best);
}

// matched edges fix their endpoints
// The length of a round's candidate list is read from device memory (*n_list: the count the previous
// round's compaction left there), so that several handshake rounds can be enqueued without the host
// looking at the counts in between; the grid is sized from an upper bound and surplus workgroups leave.
__global__ __launch_bounds__(kBlock) void k_accept(const uint32_t *n_list, Cands a, const unsigned long long *best, int32_t *mate)
{
    const size_t na = *n_list;
    size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (k >= na) return;
    const int32_t u = a.u[k], v = a.v[k];
    const unsigned long long r = a.r[k];
    if (best[u] == r && best[v] == r) { mate[u] = v; mate[v] = u; }
}

// Survivors (both endpoints still free) move to the next list and at once propose for the next
// round.  Every workgroup compacts 2048 candidates locally and reserves its output range with a
// single atomicAdd; the order of the ranges varies from run to run, which is harmless: proposals
// (atomicMax) and the accept test do not depend on the order of the list.
// Three rank arrays rotate: this round's proposals were read by k_accept, the survivors propose into
// the second, and they clear their endpoints' words in the third, which takes the proposals of the
// round after next -- so only survivors pay for clearing, and nobody clears what somebody else
// is proposing into.
constexpr int kAdvItems = 8;
constexpr uint32_t kMatchBatchMax = 1u << 20;   // candidate lists up to this length run their handshake rounds in batches
constexpr int kMatchBatch = 4;
__global__ __launch_bounds__(kBlock) void k_advance(const uint32_t *n_list, Cands a, const int32_t *mate, Cands next,
                                                    unsigned long long *best_next, unsigned long long *best_after,
                                                    uint32_t *counter)
{
    __shared__ uint32_t s_base, s_wave[4], s_pairs[4];
    const size_t na = *n_list;
    if ((size_t)blockIdx.x * (kBlock * kAdvItems) >= na) return;   // the whole workgroup: nothing left of the list here
    const int w = threadIdx.x >> 6, lane = lane_id();
    const bool short_list = gridDim.x <= 64;
    const size_t base = (size_t)blockIdx.x * (kBlock * kAdvItems) + (size_t)w * (64 * kAdvItems) + lane;
    int32_t u[kAdvItems], v[kAdvItems];
    unsigned long long r[kAdvItems];
    uint32_t where[kAdvItems];
    uint32_t keep = 0, cnt = 0, pairs = 0;
#pragma unroll
    for (int q = 0; q < kAdvItems; ++q) {
        const size_t k = base + (size_t)q * 64;
        u[q] = 0; v[q] = 0; r[q] = 0ull;
        bool ok = false, pair = false;
        if (k < na) {
            u[q] = a.u[k]; v[q] = a.v[k];
            // a short list is all latency: its rank words come in with the endpoints instead of after the test
            // (on a long list that costs more than it saves: most of its candidates do not survive)
            unsigned long long rk = 0ull;
            if (short_list) rk = a.r[k];
            const int32_t mu = mate[u[q]], mv = mate[v[q]];
            ok = mu < 0 && mv < 0;
            pair = mu == v[q];            // this very edge was matched in the round that just ended
            if (ok) r[q] = short_list ? rk : a.r[k];
        }
        pairs += (uint32_t)__popcll(__ballot(pair));
        const unsigned long long vote = __ballot(ok);
        where[q] = cnt + (uint32_t)__popcll(vote & ((1ull << lane) - 1ull));
        cnt += (uint32_t)__popcll(vote);
        if (ok) {
            keep |= 1u << q;
            best_after[u[q]] = 0ull;
            best_after[v[q]] = 0ull;
        }
        propose_edge(ok, u[q], v[q], r[q], best_next);
    }
    if (lane == 0) { s_wave[w] = cnt; s_pairs[w] = pairs; }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        const uint32_t made = s_pairs[0] + s_pairs[1] + s_pairs[2] + s_pairs[3];
        if (gridDim.x == 1) {   // the only workgroup: its range starts at 0, and nobody has to wait for the counters
            s_base = 0u;
            counter[0] = total; counter[1] = made;
        } else {
            s_base = total ? atomicAdd(counter, total) : 0u;
            if (made) atomicAdd(counter + 1, made);     // counter[1]: pairs made in this handshake round
        }
    }
    __syncthreads();
    uint32_t off = s_base;
#pragma unroll
    for (int k = 0; k < 3; ++k)
        if (k < w) off += s_wave[k];
#pragma unroll
    for (int q = 0; q < kAdvItems; ++q)
        if (keep & (1u << q)) {
            const uint32_t p = off + where[q];
            next.u[p] = u[q]; next.v[p] = v[q]; next.r[p] = r[q];
        }
}

__global__ __launch_bounds__(kBlock) void k_pair_rep(size_t n, const int32_t *mate, int32_t *rep)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= n) return;
    const int32_t w = mate[v];
    rep[v] = (w >= 0 && w < (int32_t)v) ? w : (int32_t)v;
}

// ---- connected components of (V,S) -------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_iota(size_t n, int32_t *p)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < n) p[v] = (int32_t)v;
}

__device__ __forceinline__ int32_t root_of(const int32_t *parent, int32_t v)
{
    int32_t p = parent[v];
    while (p != v) { v = p; p = parent[v]; }   // parents only ever decrease: the walk ends
    return v;
}

__global__ __launch_bounds__(kBlock) void k_hook(size_t ns, const int32_t *si, const int32_t *sj, int32_t *parent,
                                                 int32_t *changed)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= ns) return;
    int32_t a = root_of(parent, si[e]), b = root_of(parent, sj[e]);
    if (a == b) return;
    int32_t hi = max(a, b), lo = min(a, b);
    atomicMin(&parent[hi], lo);
    *changed = 1;
}

__global__ __launch_bounds__(kBlock) void k_flatten(size_t n, int32_t *parent)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < n) parent[v] = root_of(parent, (int32_t)v);
}

struct IsRoot {
    static constexpr int bytes = 4;   // bytes read per item
    static constexpr const char *tag = "IsRoot";
    const int32_t *rep;
    __device__ __forceinline__ uint32_t operator()(size_t v) const { return rep[v] == (int32_t)v ? 1u : 0u; }
};

__global__ __launch_bounds__(kBlock) void k_number(size_t n, const int32_t *rep, const uint32_t *rank, int32_t *fmap)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < n) fmap[v] = (int32_t)rank[rep[v]];
}

// ---- contraction ---------------------------------------------------------------------------------
struct InnerFlag {
    static constexpr int bytes = 16;   // bytes read per item
    static constexpr const char *tag = "InnerFlag";
    const int32_t *i, *j, *fmap;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return fmap[i[e]] == fmap[j[e]] ? 1u : 0u; }
};

// Relabelling gathers f' for both endpoints of every edge -- random 4-byte reads, the expensive
// part of the contraction -- so it is done exactly once: the packed pair of every edge is stored
// (loops get an all-ones key), the scan and the compaction then stream over the stored keys.
constexpr uint64_t kLoopKey = ~0ull;
// raw[e] = (lo, hi-lo) in two 32-bit halves; *maxdiff collects the largest hi-lo.  A workgroup takes one tile of
// the scan that follows (kScanTile edges) and leaves the number of edges that are no loops in tile_sums: the scan
// over NotLoopKey then needs no pass of its own to count them.
__global__ __launch_bounds__(kBlock) void k_relabel_keys(size_t m, const int32_t *i, const int32_t *j,
                                                         const int32_t *fmap, uint64_t *raw, uint32_t *maxdiff,
                                                         uint32_t *tile_sums)
{
    const size_t base = (size_t)blockIdx.x * kScanTile + threadIdx.x;
    uint32_t diff = 0, kept = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const size_t e = base + (size_t)q * kBlock;
        if (e < m) {
            const int32_t a = fmap[i[e]], b = fmap[j[e]];
            const uint32_t d = (uint32_t)abs(a - b);
            diff = d > diff ? d : diff;
            kept += a != b ? 1u : 0u;
            raw[e] = (a == b) ? kLoopKey : (((uint64_t)(uint32_t)min(a, b) << 32) | d);
        }
    }
    kept = block_sum(kept);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = kept;
    block_max_into(diff, maxdiff);
}
struct NotLoopKey {
    static constexpr int bytes = 8;   // bytes read per item
    static constexpr const char *tag = "NotLoopKey";
    const uint64_t *raw;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return raw[e] != kLoopKey ? 1u : 0u; }
};
// consumer of the scan over NotLoopKey: edge e that survives goes to place p
struct CompactKeysEmit {
    static constexpr const char *tag = "CompactKeys";
    const uint64_t *raw;
    const float *c;
    int dbits;
    uint64_t *key;
    uint32_t *val;
    __device__ __forceinline__ void operator()(size_t e, uint32_t keep, uint32_t p) const
    {
        if (!keep) return;
        const uint64_t k = raw[e];
        key[p] = ((k >> 32) << dbits) | (k & 0xFFFFFFFFull);
        val[p] = __float_as_uint(c[e]);
    }
};

__global__ __launch_bounds__(kBlock) void k_inner(size_t m, const int32_t *i, const int32_t *j, const float *c,
                                                  const int32_t *fmap, const uint32_t *pos, uint32_t *key, uint32_t *val)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= m) return;
    int32_t a = fmap[i[e]], b = fmap[j[e]];
    if (a != b) return;
    uint32_t p = pos[e];
    key[p] = (uint32_t)a;
    val[p] = __float_as_uint(c[e]);
}

struct HeadFlag {
    static constexpr int bytes = 8;   // bytes read per item
    static constexpr const char *tag = "HeadFlag";
    const uint64_t *key;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return (e == 0 || key[e] != key[e - 1]) ? 1u : 0u; }
};

__global__ __launch_bounds__(kBlock) void k_diag_runs(size_t m, const uint32_t *key, const uint32_t *val, float *diag)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= m) return;
    uint32_t k = key[e];
    if (e > 0 && key[e - 1] == k) return;
    float acc = __uint_as_float(val[e]);
    for (size_t f = e + 1; f < m && key[f] == k; ++f) acc = acc + __uint_as_float(val[f]);
    diag[k] = acc;
}


// ---- maximum spanning forest without conflicts (second strategy for S, Sec. 3.1) ----------------
// Boruvka rounds on the candidate edges under the matching's edge order.  comp[] is kept flat
// (comp[v] = current component root of v).  Every component points at its best outgoing edge by
// atomicMax; the chosen edges join the forest; a component hooks onto the component across its
// edge, except that of two components choosing the same edge the smaller id stays a root.
// With a strict edge order the hook graph has no other cycles, and the forest is the unique
// maximum spanning forest whatever the execution order.
__global__ __launch_bounds__(kBlock) void k_bor_propose(size_t na, const uint32_t *act, const int32_t *i,
                                                        const int32_t *j, const float *c, const int32_t *comp,
                                                        unsigned long long *best)
{
    size_t a = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (a >= na) return;
    uint32_t e = act[a];
    int32_t cu = comp[i[e]], cv = comp[j[e]];
    if (cu == cv) return;
    unsigned long long r = edge_rank(c[e], e);
    atomicMax(&best[cu], r);
    atomicMax(&best[cv], r);
}

__global__ __launch_bounds__(kBlock) void k_bor_select(size_t na, const uint32_t *act, const int32_t *i,
                                                       const int32_t *j, const float *c, const int32_t *comp,
                                                       const unsigned long long *best, int32_t *hook,
                                                       uint8_t *in_forest)
{
    size_t a = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (a >= na) return;
    uint32_t e = act[a];
    int32_t cu = comp[i[e]], cv = comp[j[e]];
    if (cu == cv) return;
    unsigned long long r = edge_rank(c[e], e);
    const bool bu = best[cu] == r, bv = best[cv] == r;
    if (!(bu || bv)) return;
    in_forest[e] = 1;
    if (bu && !(bv && cu < cv)) hook[cu] = cv;
    if (bv && !(bu && cv < cu)) hook[cv] = cu;
}

// comp[v] <- root of comp[v] in the hook forest (roots have hook[r] == r)
__global__ __launch_bounds__(kBlock) void k_bor_flatten(size_t n, const int32_t *hook, int32_t *comp)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= n) return;
    int32_t r = comp[v], h = hook[r];
    while (h != r) { r = h; h = hook[r]; }   // every chain ends in a root: the hook graph is a forest
    comp[v] = r;
}

// edges still joining two components move on; best[] and hook[] of their components are reset
__global__ __launch_bounds__(kBlock) void k_bor_advance(size_t na, const uint32_t *act, const int32_t *i,
                                                        const int32_t *j, const int32_t *comp, uint32_t *act_next,
                                                        unsigned long long *best, int32_t *hook, uint32_t *counter)
{
    __shared__ uint32_t s_base;
    const size_t tile = (size_t)blockIdx.x * (kBlock * kAdvItems);
    uint32_t e[kAdvItems];
    uint32_t keep = 0, cnt = 0;
#pragma unroll
    for (int q = 0; q < kAdvItems; ++q) {
        size_t a = tile + (size_t)threadIdx.x * kAdvItems + q;
        e[q] = 0;
        if (a < na) {
            e[q] = act[a];
            int32_t cu = comp[i[e[q]]], cv = comp[j[e[q]]];
            if (cu != cv) {
                keep |= 1u << q;
                ++cnt;
                best[cu] = 0ull; best[cv] = 0ull;
                hook[cu] = cu; hook[cv] = cv;
            }
        }
    }
    uint32_t total;
    uint32_t off = block_inclusive_scan(cnt, &total) - cnt;
    if (threadIdx.x == 0) s_base = total ? atomicAdd(counter, total) : 0u;
    __syncthreads();
    off += s_base;
#pragma unroll
    for (int q = 0; q < kAdvItems; ++q)
        if (keep & (1u << q)) act_next[off++] = e[q];
}

struct ForestFlag {
    static constexpr int bytes = 1;   // bytes read per item
    static constexpr const char *tag = "ForestFlag";
    const uint8_t *in_forest;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return in_forest[e] ? 1u : 0u; }
};
struct KeptFlag {
    static constexpr int bytes = 2;   // bytes read per item
    static constexpr const char *tag = "KeptFlag";
    const uint8_t *in_forest, *removed;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return (in_forest[e] && !removed[e]) ? 1u : 0u; }
};

__global__ __launch_bounds__(kBlock) void k_collect_flagged(size_t m, const uint8_t *flag, const uint8_t *veto,
                                                            const uint32_t *pos, const int32_t *i, const int32_t *j,
                                                            uint32_t *ids, int32_t *si, int32_t *sj)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= m || !flag[e] || (veto && veto[e])) return;
    uint32_t p = pos[e];
    if (ids) ids[p] = (uint32_t)e;
    if (si) { si[p] = i[e]; sj[p] = j[e]; }
}

// rooting of the forest, one breadth-first level per launch: a node at depth `lvl` adopts its
// still unrooted forest neighbours.  up[v] = parent, up_edge[v] = edge to the parent.
__global__ __launch_bounds__(kBlock) void k_root_init(size_t n, const int32_t *comp, int32_t *depth, int32_t *up)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= n) return;
    bool root = comp[v] == (int32_t)v;
    depth[v] = root ? 0 : -1;
    up[v] = (int32_t)v;
}

__global__ __launch_bounds__(kBlock) void k_root_level(size_t nf, const uint32_t *fe, const int32_t *i, const int32_t *j,
                                                       int32_t lvl, int32_t *depth, int32_t *up, uint32_t *up_edge,
                                                       int32_t *changed)
{
    size_t q = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (q >= nf) return;
    uint32_t e = fe[q];
    int32_t a = i[e], b = j[e];
    int32_t da = depth[a], db = depth[b];
    if (da == lvl && db < 0) { depth[b] = lvl + 1; up[b] = a; up_edge[b] = e; *changed = 1; }
    else if (db == lvl && da < 0) { depth[a] = lvl + 1; up[a] = b; up_edge[a] = e; *changed = 1; }
}

// every repulsive edge whose endpoints share a tree walks the two ends up to their meeting
// point and marks the lowest-ranked edge of the path
__global__ __launch_bounds__(kBlock) void k_mark_conflicts(size_t m, const int32_t *i, const int32_t *j, const float *c,
                                                           const int32_t *comp, const int32_t *depth, const int32_t *up,
                                                           const uint32_t *up_edge, uint8_t *removed)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= m || !(c[e] < 0.0f)) return;
    int32_t a = i[e], b = j[e];
    if (comp[a] != comp[b]) return;
    int32_t da = depth[a], db = depth[b];
    unsigned long long low = ~0ull;
    uint32_t low_e = 0;
    while (a != b) {
        uint32_t pe;
        if (da >= db) { pe = up_edge[a]; a = up[a]; --da; } else { pe = up_edge[b]; b = up[b]; --db; }
        unsigned long long r = edge_rank(c[pe], pe);
        if (r < low) { low = r; low_e = pe; }
    }
    if (low != ~0ull) removed[low_e] = 1;
}

}  // namespace

// handshake matching; mate[v] = partner or -1; returns |S| in n_matched
static rama_status matching(Ctx &ctx, const Graph &g, float tau, int rounds_cap, Buf<int32_t> &mate, int64_t &n_matched)
{
    const size_t m = (size_t)g.m, n = (size_t)g.n;
    n_matched = 0;
    RAMA_TRY(mate.alloc(ctx, n > 0 ? n : 1));
    MultiFill setup;   // mate = -1, rank words and counters = 0: one launch
    setup.add(mate.get(), 0xffffffffu, n);
    if (m == 0) return setup.run(ctx);
    Buf<int32_t> cu[2], cv[2];
    Buf<unsigned long long> cr[2];
    Cands cur{}, nxt{};
    uint32_t na = 0;
    ScanPlan<uint32_t> cand;   // its total -- the length of the first list -- stays on the device for the first round
    RAMA_TRY((scan_plan_alloc<uint32_t>(ctx, m, 0, cand)));
    RAMA_TRY((scan_totals<uint32_t>(ctx, CandFlag{g.c.get(), tau}, cand)));
    na = cand.total;
    if (na == 0) return setup.run(ctx);
    for (int k = 0; k < 2; ++k) {
        RAMA_TRY(cu[k].alloc(ctx, na));
        RAMA_TRY(cv[k].alloc(ctx, na));
        RAMA_TRY(cr[k].alloc(ctx, na));
    }
    cur = Cands{cu[0].get(), cv[0].get(), cr[0].get()};
    nxt = Cands{cu[1].get(), cv[1].get(), cr[1].get()};
    Buf<unsigned long long> best, best_next, best_after;   // rank words of this round, the next, the one after
    RAMA_TRY(best.alloc(ctx, n));
    RAMA_TRY(best_next.alloc(ctx, n));
    RAMA_TRY(best_after.alloc(ctx, n));
    const int cap = rounds_cap > 0 ? rounds_cap : 0;
    Buf<uint32_t> counters;                      // per handshake round: survivors, pairs made
    RAMA_TRY(counters.alloc(ctx, (size_t)(2 * cap + 2)));
    setup.add(best.get(), 0u, n);
    setup.add(best_next.get(), 0u, n);
    setup.add(counters.get(), 0u, (size_t)(2 * cap + 2));
    RAMA_TRY(setup.run(ctx));
    // The list is packed and, on long edge lists, makes the first round's proposals on the way (the packed list is
    // not read once more just for that: -0.5 ms per solve on the 320^3 grid); on short ones the proposals are a
    // launch of their own over the candidates only (the fused kernel shuffles for every edge: +0.1-0.2 ms on the
    // 512^2 grid).
    const bool fused = cap > 0 && m >= (size_t(1) << 21);
    RAMA_TRY((scan_emit<uint32_t>(ctx, CandFlag{g.c.get(), tau},
                                  PackCandsEmit{g.i.get(), g.j.get(), g.c.get(), cur, fused ? best.get() : nullptr}, cand,
                                  (double)((size_t)na * (fused ? 44 : 28)))));
    if (cap > 0 && !fused) {
        ProfScope ps_(ctx, "k_propose", (double)((size_t)na * 32));
        k_propose<<<grid_for(na), kBlock, 0, ctx.stream>>>(na, cur, best.get());
    }
    LAUNCH_TRY(ctx, "propose");
    // Long lists: one round per look at the counts, so that every launch has its exact size.  Short lists
    // (the launches are empty anyway): a batch of rounds is enqueued on the size of its first list, the counts
    // come back together; rounds behind the one that emptied the list find a zero count and do nothing.
    std::vector<uint32_t> back((size_t)(2 * cap + 2), 0u);
    for (int r = 0; r < cap && na > 0;) {
        const int batch = na > kMatchBatchMax ? 1 : (cap - r < kMatchBatch ? cap - r : kMatchBatch);
        for (int b = 0; b < batch; ++b, ++r) {
            const uint32_t *n_list = r == 0 ? cand.offs.get() + cand.nb : counters.get() + 2 * (r - 1);
            {
                ProfScope ps_(ctx, "k_accept", (double)((size_t)na * 40));
                k_accept<<<grid_for(na), kBlock, 0, ctx.stream>>>(n_list, cur, best.get(), mate.get());
            }
            LAUNCH_TRY(ctx, "accept");
            {
                ProfScope ps_(ctx, "k_advance", (double)((size_t)na * 56));
                k_advance<<<grid_for(na, kBlock * kAdvItems), kBlock, 0, ctx.stream>>>(
                    n_list, cur, mate.get(), nxt, best_next.get(), best_after.get(), counters.get() + 2 * r);
            }
            LAUNCH_TRY(ctx, "advance");
            Cands t = cur; cur = nxt; nxt = t;
            best.swap(best_next);          // (this, next, after) <- (next, after, this)
            best_next.swap(best_after);
        }
        RAMA_TRY(read_back(ctx, back.data() + 2 * (r - batch), counters.get() + 2 * (r - batch), (size_t)batch * 8));
        for (int b = r - batch; b < r; ++b) n_matched += back[(size_t)(2 * b + 1)];
        na = back[(size_t)(2 * (r - 1))];
    }
    return RAMA_OK;
}

// S by the spanning forest without conflicts; writes the S edges to si/sj (allocated here)
static rama_status forest_set(Ctx &ctx, const Graph &g, float tau, Buf<int32_t> &si, Buf<int32_t> &sj, int64_t &n_set)
{
    const size_t m = (size_t)g.m, n = (size_t)g.n;
    n_set = 0;
    Buf<uint32_t> pos, act, act2, counters;
    RAMA_TRY(pos.alloc(ctx, m + 1));
    uint32_t na = 0;
    {
        ScanPlan<uint32_t> cand;
        RAMA_TRY((scan_plan_alloc<uint32_t>(ctx, m, 0, cand)));
        RAMA_TRY((scan_totals<uint32_t>(ctx, CandFlag{g.c.get(), tau}, cand)));
        na = cand.total;
        if (na == 0) return RAMA_OK;
        RAMA_TRY(act.alloc(ctx, na));
        RAMA_TRY(act2.alloc(ctx, na));
        RAMA_TRY((scan_emit<uint32_t>(ctx, CandFlag{g.c.get(), tau}, CollectEmit{act.get()}, cand, (double)((size_t)na * 4))));
    }
    Buf<unsigned long long> best;
    Buf<int32_t> comp, hook;
    Buf<uint8_t> in_forest, removed;
    RAMA_TRY(best.alloc(ctx, n));
    RAMA_TRY(comp.alloc(ctx, n));
    RAMA_TRY(hook.alloc(ctx, n));
    RAMA_TRY(in_forest.alloc(ctx, m));
    RAMA_TRY(removed.alloc(ctx, m));
    RAMA_TRY(fill<unsigned long long>(ctx, best.get(), 0ull, n));
    RAMA_TRY(fill<uint8_t>(ctx, in_forest.get(), (uint8_t)0, m));
    RAMA_TRY(fill<uint8_t>(ctx, removed.get(), (uint8_t)0, m));
    {
        ProfScope ps_(ctx, "k_iota", (double)(n * 8));
        k_iota<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, comp.get());
        k_iota<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, hook.get());
    }
    LAUNCH_TRY(ctx, "iota");
    const int max_rounds = 64;   // the number of components with an outgoing edge at least halves per round
    RAMA_TRY(zeroed<uint32_t>(ctx, max_rounds, counters));
    int round = 0;
    for (; round < max_rounds && na > 0; ++round) {
        {
            ProfScope ps_(ctx, "k_bor_propose", (double)((size_t)na * 40));
            k_bor_propose<<<grid_for(na), kBlock, 0, ctx.stream>>>(na, act.get(), g.i.get(), g.j.get(), g.c.get(), comp.get(),
                                                                  best.get());
        }
        LAUNCH_TRY(ctx, "bor_propose");
        {
            ProfScope ps_(ctx, "k_bor_select", (double)((size_t)na * 48));
            k_bor_select<<<grid_for(na), kBlock, 0, ctx.stream>>>(na, act.get(), g.i.get(), g.j.get(), g.c.get(), comp.get(),
                                                                 best.get(), hook.get(), in_forest.get());
        }
        LAUNCH_TRY(ctx, "bor_select");
        {
            ProfScope ps_(ctx, "k_bor_flatten", (double)(n * 12));
            k_bor_flatten<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, hook.get(), comp.get());
        }
        LAUNCH_TRY(ctx, "bor_flatten");
        {
            ProfScope ps_(ctx, "k_bor_advance", (double)((size_t)na * 28));
            k_bor_advance<<<grid_for(na, kBlock * kAdvItems), kBlock, 0, ctx.stream>>>(
                na, act.get(), g.i.get(), g.j.get(), comp.get(), act2.get(), best.get(), hook.get(), counters.get() + round);
        }
        LAUNCH_TRY(ctx, "bor_advance");
        uint32_t nn = 0;
        RAMA_TRY(read_back(ctx, &nn, counters.get() + round, 4));
        act.swap(act2);
        na = nn;
    }
    if (na > 0) return fail(ctx, RAMA_ERR_HIP, "spanning forest did not converge");
    act.reset(); act2.reset(); best.reset();
    // forest edge list
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, ForestFlag{in_forest.get()}, pos.get(), m)));
    uint32_t nf = 0;
    RAMA_TRY(read_back(ctx, &nf, pos.get() + m, 4));
    if (nf == 0) return RAMA_OK;
    Buf<uint32_t> fe, up_edge;
    Buf<int32_t> depth, up, changed;
    RAMA_TRY(fe.alloc(ctx, nf));
    {
        ProfScope ps_(ctx, "k_collect_flagged", (double)(m * 5 + (size_t)nf * 4));
        k_collect_flagged<<<grid_for(m), kBlock, 0, ctx.stream>>>(m, in_forest.get(), (const uint8_t *)nullptr, pos.get(),
                                                                 g.i.get(), g.j.get(), fe.get(), (int32_t *)nullptr,
                                                                 (int32_t *)nullptr);
    }
    LAUNCH_TRY(ctx, "collect_flagged");
    // root the trees at their component representative, level by level
    RAMA_TRY(depth.alloc(ctx, n));
    RAMA_TRY(up.alloc(ctx, n));
    RAMA_TRY(up_edge.alloc(ctx, n));
    {
        ProfScope ps_(ctx, "k_root_init", (double)(n * 12));
        k_root_init<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, comp.get(), depth.get(), up.get());
    }
    LAUNCH_TRY(ctx, "root_init");
    const int levels_per_check = 8;
    for (int32_t lvl = 0;; lvl += levels_per_check) {
        // a tree is at most n-1 levels deep; the sweep after the deepest level reports no change
        if ((size_t)lvl > n + levels_per_check) return fail(ctx, RAMA_ERR_HIP, "forest rooting did not converge");
        RAMA_TRY(zeroed<int32_t>(ctx, 1, changed));   // a fresh word per look
        for (int q = 0; q < levels_per_check; ++q) {
            ProfScope ps_(ctx, "k_root_level", (double)((size_t)nf * 20));
            k_root_level<<<grid_for(nf), kBlock, 0, ctx.stream>>>(nf, fe.get(), g.i.get(), g.j.get(), lvl + q, depth.get(),
                                                                 up.get(), up_edge.get(), changed.get());
        }
        LAUNCH_TRY(ctx, "root_level");
        int32_t h = 0;
        RAMA_TRY(read_back(ctx, &h, changed.get(), 4));
        if (!h) break;
    }
    {
        ProfScope ps_(ctx, "k_mark_conflicts", (double)(m * 12));
        k_mark_conflicts<<<grid_for(m), kBlock, 0, ctx.stream>>>(m, g.i.get(), g.j.get(), g.c.get(), comp.get(), depth.get(),
                                                                up.get(), up_edge.get(), removed.get());
    }
    LAUNCH_TRY(ctx, "mark_conflicts");
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, KeptFlag{in_forest.get(), removed.get()}, pos.get(), m)));
    uint32_t ns = 0;
    RAMA_TRY(read_back(ctx, &ns, pos.get() + m, 4));
    n_set = ns;
    if (ns == 0) return RAMA_OK;
    RAMA_TRY(si.alloc(ctx, ns));
    RAMA_TRY(sj.alloc(ctx, ns));
    {
        ProfScope ps_(ctx, "k_collect_flagged", (double)(m * 6 + (size_t)ns * 8));
        k_collect_flagged<<<grid_for(m), kBlock, 0, ctx.stream>>>(m, in_forest.get(), removed.get(), pos.get(), g.i.get(),
                                                                 g.j.get(), (uint32_t *)nullptr, si.get(), sj.get());
    }
    LAUNCH_TRY(ctx, "collect_flagged");
    return RAMA_OK;
}

// rep[v] = smallest node of v's component in (V,S)
static rama_status components(Ctx &ctx, size_t n, size_t ns, const int32_t *si, const int32_t *sj, Buf<int32_t> &rep)
{
    RAMA_TRY(rep.alloc(ctx, n > 0 ? n : 1));
    {
        ProfScope ps_(ctx, "k_iota", (double)(n * 4));
        k_iota<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, rep.get());
    }
    LAUNCH_TRY(ctx, "iota");
    if (ns == 0) return RAMA_OK;
    Buf<int32_t> changed;
    for (int it = 0; it < 64; ++it) {   // the number of trees at least halves per sweep
        RAMA_TRY(zeroed<int32_t>(ctx, 1, changed));   // a fresh word per sweep
        {
            ProfScope ps_(ctx, "k_hook", (double)(ns * 24));
            k_hook<<<grid_for(ns), kBlock, 0, ctx.stream>>>(ns, si, sj, rep.get(), changed.get());
        }
        LAUNCH_TRY(ctx, "hook");
        {
            ProfScope ps_(ctx, "k_flatten", (double)(n * 12));
            k_flatten<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, rep.get());
        }
        LAUNCH_TRY(ctx, "flatten");
        int32_t h = 0;
        RAMA_TRY(read_back(ctx, &h, changed.get(), 4));
        if (!h) return RAMA_OK;
    }
    return fail(ctx, RAMA_ERR_HIP, "connected components did not converge");
}

// contracted graph of canonical g under fmap (n_new new nodes)
static rama_status contract_edges(Ctx &ctx, const Graph &g, const int32_t *fmap, int32_t n_new, Graph &out)
{
    const size_t m = (size_t)g.m;
    out.n = n_new;
    out.m = 0;
    const int nbits = bits_for((uint64_t)n_new);
    ScanPlan<uint32_t> keep;   // the extra word behind the total: largest hi-lo
    Buf<uint64_t> raw;
    RAMA_TRY((scan_plan_alloc<uint32_t>(ctx, m, 1, keep)));
    RAMA_TRY(raw.alloc(ctx, m));
    {
        ProfScope ps_(ctx, "k_relabel_keys", (double)(m * 24));
        k_relabel_keys<<<keep.nb, kBlock, 0, ctx.stream>>>(m, g.i.get(), g.j.get(), fmap, raw.get(), keep.extra_ptr(),
                                                           keep.sums.get());
    }
    LAUNCH_TRY(ctx, "relabel_keys");
    RAMA_TRY((scan_totals<uint32_t>(ctx, NotLoopKey{raw.get()}, keep, keep.sums.get())));   // tile sums: left by k_relabel_keys
    const uint32_t kept = keep.total;
    const int dbits = bits_for((uint64_t)keep.extra_value[0] + 1);
    if (kept == 0) {
        RAMA_TRY(out.i.alloc(ctx, 1));
        RAMA_TRY(out.j.alloc(ctx, 1));
        RAMA_TRY(out.c.alloc(ctx, 1));
        return RAMA_OK;
    }
    Buf<uint64_t> key;
    Buf<uint32_t> val;
    RAMA_TRY(key.alloc(ctx, kept));
    RAMA_TRY(val.alloc(ctx, kept));
    RAMA_TRY((scan_emit<uint32_t>(ctx, NotLoopKey{raw.get()}, CompactKeysEmit{raw.get(), g.c.get(), dbits, key.get(), val.get()},
                                  keep, (double)(m * 4 + (size_t)kept * 12))));
    keep.offs.reset();
    raw.reset();
    Buf<uint32_t> head_sums;   // heads per scan tile, if the sort's last kernel could count them
    RAMA_TRY((radix_sort_pairs<uint64_t, uint32_t>(ctx, key, val, kept, nbits + dbits, false, &head_sums, (uint64_t)n_new << dbits)));
    ScanPlan<uint32_t> runs;
    RAMA_TRY((scan_plan_alloc<uint32_t>(ctx, kept, 0, runs)));
    RAMA_TRY((scan_totals<uint32_t>(ctx, HeadFlag{key.get()}, runs, head_sums.get())));
    head_sums.reset();
    const uint32_t uniq = runs.total;
    RAMA_TRY(out.i.alloc(ctx, uniq));
    RAMA_TRY(out.j.alloc(ctx, uniq));
    RAMA_TRY(out.c.alloc(ctx, uniq));
    RAMA_TRY(reduce_runs(ctx, runs, key.get(), val.get(), dbits, out.i.get(), out.j.get(), out.c.get(), &out.sign_sums));
    out.m = uniq;
    return RAMA_OK;
}

rama_status contract_once(Ctx &ctx, const Graph &g, float tau, int rounds_cap, float forest_ratio, Buf<int32_t> &fmap,
                          int32_t &n_new, Graph &out, int64_t &n_matched, bool *used_forest)
{
    const size_t n = (size_t)g.n;
    if (used_forest) *used_forest = false;
    RAMA_TRY(zero_page_recycle(ctx));
    Buf<int32_t> mate;
    RAMA_TRY(matching(ctx, g, tau, rounds_cap, mate, n_matched));
    n_new = g.n;
    if (n_matched == 0) return RAMA_OK;
    Buf<uint32_t> npos;
    Buf<int32_t> si, sj, rep;
    RAMA_TRY(npos.alloc(ctx, n + 1));
    bool pairs_only = true;   // S is a matching: every component of (V,S) is a node or a pair
    // too few pairs: switch to the spanning forest without conflicts (Sec. 3.1, "fewer than 0.1|V|")
    if (forest_ratio > 0.0f && (double)n_matched < (double)forest_ratio * (double)g.n) {
        pairs_only = false;
        mate.reset();
        if (used_forest) *used_forest = true;
        RAMA_TRY(forest_set(ctx, g, tau, si, sj, n_matched));
        if (n_matched == 0) return RAMA_OK;
        RAMA_TRY(components(ctx, n, (size_t)n_matched, si.get(), sj.get(), rep));
    } else {
        // the components of a matching are its pairs: the representative (smallest node) is at hand
        RAMA_TRY(rep.alloc(ctx, n));
        ProfScope ps_(ctx, "k_pair_rep", (double)(n * 8));
        k_pair_rep<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, mate.get(), rep.get());
    }
    LAUNCH_TRY(ctx, "pair_rep");
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, IsRoot{rep.get()}, npos.get(), n)));
    if (pairs_only) {
        n_new = (int32_t)((int64_t)g.n - n_matched);   // every pair removes one node: no need to ask the device
    } else {
        uint32_t nn = 0;
        RAMA_TRY(read_back(ctx, &nn, npos.get() + n, 4));
        n_new = (int32_t)nn;
    }
    RAMA_TRY(fmap.alloc(ctx, n));
    {
        ProfScope ps_(ctx, "k_number", (double)(n * 12));
        k_number<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, rep.get(), npos.get(), fmap.get());
    }
    LAUNCH_TRY(ctx, "number");
    RAMA_TRY(contract_edges(ctx, g, fmap.get(), n_new, out));
    return RAMA_OK;
}

rama_status contraction_diagonal(Ctx &ctx, const Graph &g, const int32_t *fmap, int32_t n_new, float *diag)
{
    const size_t m = (size_t)g.m;
    RAMA_TRY(fill<float>(ctx, diag, 0.0f, (size_t)n_new));
    if (m == 0) return RAMA_OK;
    Buf<uint32_t> pos;
    RAMA_TRY(pos.alloc(ctx, m + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, InnerFlag{g.i.get(), g.j.get(), fmap}, pos.get(), m)));
    uint32_t kept = 0;
    RAMA_TRY(read_back(ctx, &kept, pos.get() + m, 4));
    if (kept == 0) return RAMA_OK;
    Buf<uint32_t> key, val;
    RAMA_TRY(key.alloc(ctx, kept));
    RAMA_TRY(val.alloc(ctx, kept));
    {
        ProfScope ps_(ctx, "k_inner", (double)(m * 28 + (size_t)kept * 8));
        k_inner<<<grid_for(m), kBlock, 0, ctx.stream>>>(m, g.i.get(), g.j.get(), g.c.get(), fmap, pos.get(), key.get(), val.get());
    }
    LAUNCH_TRY(ctx, "inner");
    RAMA_TRY((radix_sort_pairs<uint32_t, uint32_t>(ctx, key, val, kept, bits_for((uint64_t)n_new), false, nullptr, (uint64_t)n_new)));
    {
        ProfScope ps_(ctx, "k_diag_runs", (double)((size_t)kept * 12));
        k_diag_runs<<<grid_for(kept), kBlock, 0, ctx.stream>>>(kept, key.get(), val.get(), diag);
    }
    LAUNCH_TRY(ctx, "diag_runs");
    return RAMA_OK;
}

}  // namespace rama
