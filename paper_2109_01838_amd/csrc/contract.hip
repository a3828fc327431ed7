// Steps a4-a6: one primal update (paper Sec. 3.1: Lemma 1, Lemma 3, algorithm
// "Parallel-Edge-Contraction", "Maximum matching"; appendix algorithm "GPU Edge-Contraction").
//
//   S   : handshake matching on the edges with c > tau.  Edges are ranked by (cost, position in
//         the canonical list) packed into one 64-bit word, so "each node points at its best
//         incident candidate" is an integer atomicMax per endpoint -- order independent, hence
//         deterministic.  An edge both of whose endpoints point at it is matched; rounds repeat
//         on the shrinking list of edges whose endpoints are both still free.
//   f'  : connected components of (V,S) by min-label hooking + pointer jumping; a component is
//         represented by its smallest node; new ids are the ranks of the representatives.
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

__global__ __launch_bounds__(kBlock) void k_collect(size_t m, const float *c, float tau, const uint32_t *pos, uint32_t *act)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e < m && c[e] > tau) act[pos[e]] = (uint32_t)e;
}

__global__ __launch_bounds__(kBlock) void k_propose(size_t na, const uint32_t *act, const int32_t *i, const int32_t *j,
                                                    const float *c, unsigned long long *best)
{
    size_t a = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (a >= na) return;
    uint32_t e = act[a];
    unsigned long long r = edge_rank(c[e], e);
    atomicMax(&best[i[e]], r);
    atomicMax(&best[j[e]], r);
}

__global__ __launch_bounds__(kBlock) void k_accept(size_t na, const uint32_t *act, const int32_t *i, const int32_t *j,
                                                   const float *c, const unsigned long long *best, int32_t *mate)
{
    size_t a = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (a >= na) return;
    uint32_t e = act[a];
    unsigned long long r = edge_rank(c[e], e);
    int32_t u = i[e], v = j[e];
    if (best[u] == r && best[v] == r) { mate[u] = v; mate[v] = u; }
}

// Survivors (both endpoints still free) move to the next list and the pointers of their
// endpoints are cleared for the next round.  Every workgroup compacts 2048 candidates locally and
// reserves its output range with a single atomicAdd; the order of the ranges varies from run to
// run, which is harmless: the atomicMax proposals and the accept test do not depend on the order
// of the list.
constexpr int kAdvItems = 8;
__global__ __launch_bounds__(kBlock) void k_advance(size_t na, const uint32_t *act, const int32_t *i, const int32_t *j,
                                                    const int32_t *mate, uint32_t *act_next,
                                                    unsigned long long *best, uint32_t *counter)
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
            int32_t u = i[e[q]], v = j[e[q]];
            if (mate[u] < 0 && mate[v] < 0) {
                keep |= 1u << q;
                ++cnt;
                best[u] = 0ull;
                best[v] = 0ull;
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

struct MatchedLow {
    static constexpr int bytes = 4;   // bytes read per item
    static constexpr const char *tag = "MatchedLow";
    const int32_t *mate;
    __device__ __forceinline__ uint32_t operator()(size_t v) const { return mate[v] > (int32_t)v ? 1u : 0u; }
};

__global__ __launch_bounds__(kBlock) void k_emit_pairs(size_t n, const int32_t *mate, const uint32_t *pos, int32_t *si,
                                                       int32_t *sj)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v >= n) return;
    if (mate[v] > (int32_t)v) { si[pos[v]] = (int32_t)v; sj[pos[v]] = mate[v]; }
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
struct CrossFlag {
    static constexpr int bytes = 16;   // bytes read per item
    static constexpr const char *tag = "CrossFlag";
    const int32_t *i, *j, *fmap;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return fmap[i[e]] != fmap[j[e]] ? 1u : 0u; }
};
struct InnerFlag {
    static constexpr int bytes = 16;   // bytes read per item
    static constexpr const char *tag = "InnerFlag";
    const int32_t *i, *j, *fmap;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return fmap[i[e]] == fmap[j[e]] ? 1u : 0u; }
};

// relabelled, re-oriented cross edges -> (key, cost) in input order
__global__ __launch_bounds__(kBlock) void k_relabel(size_t m, const int32_t *i, const int32_t *j, const float *c,
                                                    const int32_t *fmap, const uint32_t *pos, int nbits, uint64_t *key,
                                                    uint32_t *val)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= m) return;
    int32_t a = fmap[i[e]], b = fmap[j[e]];
    if (a == b) return;
    uint32_t p = pos[e];
    key[p] = ((uint64_t)(uint32_t)min(a, b) << nbits) | (uint32_t)max(a, b);
    val[p] = __float_as_uint(c[e]);
}

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

}  // namespace

// handshake matching; mate[v] = partner or -1; returns |S| in n_matched
static rama_status matching(Ctx &ctx, const Graph &g, float tau, int rounds_cap, Buf<int32_t> &mate, int64_t &n_matched)
{
    const size_t m = (size_t)g.m, n = (size_t)g.n;
    n_matched = 0;
    RAMA_TRY(mate.alloc(ctx, n > 0 ? n : 1));
    RAMA_TRY(fill<int32_t>(ctx, mate.get(), -1, n));
    if (m == 0) return RAMA_OK;
    Buf<uint32_t> pos, act, act2;
    RAMA_TRY(pos.alloc(ctx, m + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, CandFlag{g.c.get(), tau}, pos.get(), m)));
    uint32_t na = 0;
    RAMA_TRY(read_back(ctx, &na, pos.get() + m, 4));
    if (na == 0) return RAMA_OK;
    RAMA_TRY(act.alloc(ctx, na));
    RAMA_TRY(act2.alloc(ctx, na));
    {
        ProfScope ps_(ctx, "k_collect", (double)(m * 8 + (size_t)na * 4));
        k_collect<<<grid_for(m), kBlock, 0, ctx.stream>>>(m, g.c.get(), tau, pos.get(), act.get());
    }
    LAUNCH_TRY(ctx, "collect");
    Buf<unsigned long long> best;
    RAMA_TRY(best.alloc(ctx, n));
    RAMA_TRY(fill<unsigned long long>(ctx, best.get(), 0ull, n));
    Buf<uint32_t> counters;                      // one survivor counter per handshake round
    RAMA_TRY(counters.alloc(ctx, (size_t)(rounds_cap > 0 ? rounds_cap : 1)));
    RAMA_TRY(fill<uint32_t>(ctx, counters.get(), 0u, (size_t)(rounds_cap > 0 ? rounds_cap : 1)));
    for (int r = 0; r < rounds_cap && na > 0; ++r) {
        {
            ProfScope ps_(ctx, "k_propose", (double)((size_t)na * 32));
            k_propose<<<grid_for(na), kBlock, 0, ctx.stream>>>(na, act.get(), g.i.get(), g.j.get(), g.c.get(), best.get());
        }
        LAUNCH_TRY(ctx, "propose");
        {
            ProfScope ps_(ctx, "k_accept", (double)((size_t)na * 40));
            k_accept<<<grid_for(na), kBlock, 0, ctx.stream>>>(na, act.get(), g.i.get(), g.j.get(), g.c.get(), best.get(),
                                                             mate.get());
        }
        LAUNCH_TRY(ctx, "accept");
        {
            ProfScope ps_(ctx, "k_advance", (double)((size_t)na * 20));
            k_advance<<<grid_for(na, kBlock * kAdvItems), kBlock, 0, ctx.stream>>>(na, act.get(), g.i.get(), g.j.get(), mate.get(), act2.get(),
                                                              best.get(), counters.get() + r);
        }
        LAUNCH_TRY(ctx, "advance");
        uint32_t nn = 0;
        RAMA_TRY(read_back(ctx, &nn, counters.get() + r, 4));
        act.swap(act2);
        na = nn;
    }
    Buf<uint32_t> npos;
    RAMA_TRY(npos.alloc(ctx, n + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, MatchedLow{mate.get()}, npos.get(), n)));
    uint32_t ns = 0;
    RAMA_TRY(read_back(ctx, &ns, npos.get() + n, 4));
    n_matched = ns;
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
    RAMA_TRY(changed.alloc(ctx, 1));
    for (int it = 0; it < 64; ++it) {   // the number of trees at least halves per sweep
        RAMA_TRY(fill<int32_t>(ctx, changed.get(), 0, 1));
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
    Buf<uint32_t> pos;
    RAMA_TRY(pos.alloc(ctx, m + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, CrossFlag{g.i.get(), g.j.get(), fmap}, pos.get(), m)));
    uint32_t kept = 0;
    RAMA_TRY(read_back(ctx, &kept, pos.get() + m, 4));
    if (kept == 0) {
        RAMA_TRY(out.i.alloc(ctx, 1));
        RAMA_TRY(out.j.alloc(ctx, 1));
        RAMA_TRY(out.c.alloc(ctx, 1));
        return RAMA_OK;
    }
    const int nbits = bits_for((uint64_t)n_new);
    Buf<uint64_t> key;
    Buf<uint32_t> val;
    RAMA_TRY(key.alloc(ctx, kept));
    RAMA_TRY(val.alloc(ctx, kept));
    {
        ProfScope ps_(ctx, "k_relabel", (double)(m * 28 + (size_t)kept * 12));
        k_relabel<<<grid_for(m), kBlock, 0, ctx.stream>>>(m, g.i.get(), g.j.get(), g.c.get(), fmap, pos.get(), nbits,
                                                      key.get(), val.get());
    }
    LAUNCH_TRY(ctx, "relabel");
    pos.reset();
    RAMA_TRY((radix_sort_pairs<uint64_t, uint32_t>(ctx, key, val, kept, 2 * nbits)));
    Buf<uint32_t> opos;
    RAMA_TRY(opos.alloc(ctx, (size_t)kept + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, HeadFlag{key.get()}, opos.get(), (size_t)kept)));
    uint32_t uniq = 0;
    RAMA_TRY(read_back(ctx, &uniq, opos.get() + kept, 4));
    RAMA_TRY(out.i.alloc(ctx, uniq));
    RAMA_TRY(out.j.alloc(ctx, uniq));
    RAMA_TRY(out.c.alloc(ctx, uniq));
    {
        ProfScope ps_(ctx, "k_reduce_runs", (double)((size_t)kept * 16 + (size_t)uniq * 12));
        k_reduce_runs<<<grid_for(kept), kBlock, 0, ctx.stream>>>(kept, key.get(), val.get(), opos.get(), nbits, out.i.get(),
                                                            out.j.get(), out.c.get());
    }
    LAUNCH_TRY(ctx, "reduce_runs");
    out.m = uniq;
    return RAMA_OK;
}

rama_status contract_once(Ctx &ctx, const Graph &g, float tau, int rounds_cap, Buf<int32_t> &fmap, int32_t &n_new,
                          Graph &out, int64_t &n_matched)
{
    const size_t n = (size_t)g.n;
    Buf<int32_t> mate;
    RAMA_TRY(matching(ctx, g, tau, rounds_cap, mate, n_matched));
    n_new = g.n;
    if (n_matched == 0) return RAMA_OK;
    const size_t ns = (size_t)n_matched;
    Buf<uint32_t> npos;
    Buf<int32_t> si, sj, rep;
    RAMA_TRY(npos.alloc(ctx, n + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, MatchedLow{mate.get()}, npos.get(), n)));
    RAMA_TRY(si.alloc(ctx, ns));
    RAMA_TRY(sj.alloc(ctx, ns));
    {
        ProfScope ps_(ctx, "k_emit_pairs", (double)(n * 8 + ns * 8));
        k_emit_pairs<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, mate.get(), npos.get(), si.get(), sj.get());
    }
    LAUNCH_TRY(ctx, "emit_pairs");
    RAMA_TRY(components(ctx, n, ns, si.get(), sj.get(), rep));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, IsRoot{rep.get()}, npos.get(), n)));
    uint32_t nn = 0;
    RAMA_TRY(read_back(ctx, &nn, npos.get() + n, 4));
    n_new = (int32_t)nn;
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
    RAMA_TRY((radix_sort_pairs<uint32_t, uint32_t>(ctx, key, val, kept, bits_for((uint64_t)n_new))));
    {
        ProfScope ps_(ctx, "k_diag_runs", (double)((size_t)kept * 12));
        k_diag_runs<<<grid_for(kept), kBlock, 0, ctx.stream>>>(kept, key.get(), val.get(), diag);
    }
    LAUNCH_TRY(ctx, "diag_runs");
    return RAMA_OK;
}

}  // namespace rama
