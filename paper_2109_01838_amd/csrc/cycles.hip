// Step a1: conflicted-cycle separation (paper Sec. 3.2.2, definition "Conflicted cycles" and the
// lemma on searching per repulsive edge; appendix algorithm "Parallel Conf. 5-Cycles").
//
// For every repulsive edge (v0,vL), v0<vL, all attractive simple paths of 2, 3 and 4 hops
// between its endpoints are enumerated on the positive neighbourhoods N+ held as a CSR with
// ascending rows:
//   3-cycles: v1 in N+(v0) & N+(vL)
//   4-cycles: v1 in N+(v0), v2 in N+(v1) & N+(vL)
//   5-cycles: v1 in N+(v0), v2 in N+(v1), v3 in N+(v2) & N+(vL); the same set as the appendix
//             algorithm's pairs (v1,v3) in N+(v0) x N+(vL) with common neighbour v2
// A count pass, a scan and a fill pass produce the lists already in their final order
// (v0, vL, then the path v1, v2, v3), because repulsive edges are visited in canonical order
// and every row is ascending.
#include "prim.h"

namespace rama {

namespace {

struct PosFlag {
    static constexpr int bytes = 4;   // bytes read per item
    static constexpr const char *tag = "PosFlag";
    const float *c;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return c[e] > 0.0f ? 1u : 0u; }
};
struct NegFlag {
    static constexpr int bytes = 4;   // bytes read per item
    static constexpr const char *tag = "NegFlag";
    const float *c;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return c[e] < 0.0f ? 1u : 0u; }
};

__global__ __launch_bounds__(kBlock) void k_split_sign(size_t m, const int32_t *i, const int32_t *j, const float *c,
                                                       const uint32_t *ppos, const uint32_t *npos, int32_t *pi,
                                                       int32_t *pj, uint32_t *lkey, uint32_t *lval, int32_t *ri,
                                                       int32_t *rj)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= m) return;
    float w = c[e];
    if (w > 0.0f) {
        uint32_t p = ppos[e];
        pi[p] = i[e]; pj[p] = j[e];
        lkey[p] = (uint32_t)j[e]; lval[p] = (uint32_t)i[e];
    } else if (w < 0.0f) {
        uint32_t p = npos[e];
        ri[p] = i[e]; rj[p] = j[e];
    }
}

__global__ __launch_bounds__(kBlock) void k_add_ptr(int32_t n, const int32_t *a, const int32_t *b, int32_t *out)
{
    int32_t v = blockIdx.x * kBlock + threadIdx.x;
    if (v <= n) out[v] = a[v] + b[v];
}

// row v of N+ = [lower neighbours u<v, ascending][upper neighbours w>v, ascending]
__global__ __launch_bounds__(kBlock) void k_fill_adj(size_t mp, const int32_t *pi, const int32_t *pj,
                                                     const uint32_t *lj, const uint32_t *li, const int32_t *up_ptr,
                                                     const int32_t *low_ptr, const int32_t *rowptr, int32_t *nb)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= mp) return;
    {   // upper entry of edge e: row pi[e]
        int32_t u = pi[e];
        int32_t lowdeg = low_ptr[u + 1] - low_ptr[u];
        nb[rowptr[u] + lowdeg + ((int32_t)e - up_ptr[u])] = pj[e];
    }
    {   // lower entry at sorted position e: row lj[e]
        int32_t v = (int32_t)lj[e];
        nb[rowptr[v] + ((int32_t)e - low_ptr[v])] = (int32_t)li[e];
    }
}

struct Adj {
    const int32_t *ptr;
    const int32_t *nb;
};

// calls f(x) for every x in row a & row b, ascending: walk the shorter row, search the longer
template <typename F>
__device__ __forceinline__ void intersect_rows(const Adj &g, int32_t a, int32_t b, F &&f)
{
    int32_t a0 = g.ptr[a], a1 = g.ptr[a + 1], b0 = g.ptr[b], b1 = g.ptr[b + 1];
    if (a1 - a0 > b1 - b0) { int32_t t = a0; a0 = b0; b0 = t; t = a1; a1 = b1; b1 = t; }
    for (int32_t p = a0; p < a1 && b0 < b1; ++p) {
        int32_t x = g.nb[p];
        int32_t lo = b0, hi = b1;
        while (lo < hi) {
            int32_t mid = lo + ((hi - lo) >> 1);
            if (g.nb[mid] < x) lo = mid + 1; else hi = mid;
        }
        b0 = lo;
        if (lo < b1 && g.nb[lo] == x) { f(x); b0 = lo + 1; }
    }
}

// N+(vL) of the repulsive edge under work: kept in registers when it has at most 8 entries
// (always the case on grid-like inputs), otherwise searched in memory
constexpr int kRowRegs = 8;
struct EndRow {
    int32_t r[kRowRegs];
    int32_t b0, b1;
    const int32_t *nb;
    bool in_regs;
    __device__ __forceinline__ void load(const Adj &g, int32_t vl)
    {
        nb = g.nb; b0 = g.ptr[vl]; b1 = g.ptr[vl + 1];
        in_regs = (b1 - b0) <= kRowRegs;
#pragma unroll
        for (int k = 0; k < kRowRegs; ++k) r[k] = (in_regs && b0 + k < b1) ? nb[b0 + k] : -1;
    }
    __device__ __forceinline__ bool has(int32_t x) const
    {
        if (in_regs) {
            bool f = false;
#pragma unroll
            for (int k = 0; k < kRowRegs; ++k) f |= (r[k] == x);
            return f;
        }
        int32_t lo = b0, hi = b1;
        while (lo < hi) {
            int32_t mid = lo + ((hi - lo) >> 1);
            if (nb[mid] < x) lo = mid + 1; else hi = mid;
        }
        return lo < b1 && nb[lo] == x;
    }
};

// Depth-first walk v0 -> v1 -> v2 -> v3 along N+, closing on N+(vL) at every depth:
//   v1 in N+(vL)                      -> 3-cycle (v0,v1,vL)
//   v2 in N+(vL)                      -> 4-cycle (v0,v1,v2,vL)
//   v3 in N+(vL), v3 != v1            -> 5-cycle (v0,v1,v2,v3,vL)   (the appendix algorithm's
//                                        pairs (v1,v3) with common neighbour v2, visited path-first)
// vL and v0 are never in N+(vL) / N+(v0) of a repulsive edge, which settles the other
// distinctness conditions.  Rows are ascending, so every list comes out in path order.
template <typename Emit>
__device__ __forceinline__ void enumerate_cycles(const Adj &g, int32_t v0, int32_t vl, int max_len, Emit &emit)
{
    if (max_len <= 3) {
        intersect_rows(g, v0, vl, [&](int32_t v1) { emit.c3(v1); });
        return;
    }
    EndRow end;
    end.load(g, vl);
    if (end.b0 == end.b1) return;
    const int32_t r0 = g.ptr[v0], r0e = g.ptr[v0 + 1];
    for (int32_t p = r0; p < r0e; ++p) {
        const int32_t v1 = g.nb[p];
        if (end.has(v1)) emit.c3(v1);
        const int32_t r1 = g.ptr[v1], r1e = g.ptr[v1 + 1];
        for (int32_t q = r1; q < r1e; ++q) {
            const int32_t v2 = g.nb[q];
            if (v2 == v0) continue;
            if (end.has(v2)) emit.c4(v1, v2);
            if (max_len < 5 || v2 == vl) continue;
            const int32_t r2 = g.ptr[v2], r2e = g.ptr[v2 + 1];
            for (int32_t t = r2; t < r2e; ++t) {
                const int32_t v3 = g.nb[t];
                if (v3 != v1 && end.has(v3)) emit.c5(v1, v2, v3);
            }
        }
    }
}

struct CountEmit {
    uint32_t n3 = 0, n4 = 0, n5 = 0;
    __device__ __forceinline__ void c3(int32_t) { ++n3; }
    __device__ __forceinline__ void c4(int32_t, int32_t) { ++n4; }
    __device__ __forceinline__ void c5(int32_t, int32_t, int32_t) { ++n5; }
};

struct FillEmit {
    int32_t v0, vl;
    int32_t *o3, *o4, *o5;
    __device__ __forceinline__ void c3(int32_t v1) { o3[0] = v0; o3[1] = v1; o3[2] = vl; o3 += 3; }
    __device__ __forceinline__ void c4(int32_t v1, int32_t v2) { o4[0] = v0; o4[1] = v1; o4[2] = v2; o4[3] = vl; o4 += 4; }
    __device__ __forceinline__ void c5(int32_t v1, int32_t v2, int32_t v3)
    {
        o5[0] = v0; o5[1] = v1; o5[2] = v2; o5[3] = v3; o5[4] = vl; o5 += 5;
    }
};

__global__ __launch_bounds__(kBlock) void k_count_cycles(size_t nr, const int32_t *ri, const int32_t *rj, Adj g,
                                                         int max_len, uint32_t *c3, uint32_t *c4, uint32_t *c5)
{
    size_t r = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (r >= nr) return;
    CountEmit em;
    enumerate_cycles(g, ri[r], rj[r], max_len, em);
    c3[r] = em.n3; c4[r] = em.n4; c5[r] = em.n5;
}

struct HasCycles {
    static constexpr int bytes = 12;   // bytes read per item
    static constexpr const char *tag = "HasCycles";
    const uint32_t *c3, *c4, *c5;
    __device__ __forceinline__ uint32_t operator()(size_t r) const { return (c3[r] | c4[r] | c5[r]) ? 1u : 0u; }
};

__global__ __launch_bounds__(kBlock) void k_collect_hits(size_t nr, const uint32_t *c3, const uint32_t *c4,
                                                         const uint32_t *c5, const uint32_t *pos, uint32_t *hit)
{
    size_t r = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (r < nr && (c3[r] | c4[r] | c5[r])) hit[pos[r]] = (uint32_t)r;
}

// second walk, only over the repulsive edges that have cycles and only as deep as their
// longest cycle; writes every list at the offsets of the scan
__global__ __launch_bounds__(kBlock) void k_fill_cycles(size_t nh, const uint32_t *hit, const int32_t *ri,
                                                        const int32_t *rj, Adj g, const uint32_t *c4,
                                                        const uint32_t *c5, const uint64_t *off3, const uint64_t *off4,
                                                        const uint64_t *off5, int32_t *out3, int32_t *out4,
                                                        int32_t *out5)
{
    size_t h = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (h >= nh) return;
    const uint32_t r = hit[h];
    const int depth = c5[r] ? 5 : (c4[r] ? 4 : 3);
    FillEmit em{ri[r], rj[r], out3 + 3 * off3[r], out4 + 4 * off4[r], out5 + 5 * off5[r]};
    enumerate_cycles(g, em.v0, em.vl, depth, em);
}

}  // namespace

rama_status find_cycles(Ctx &ctx, const Graph &g, int max_len, bool count_only, CycleLists &out)
{
    for (int k = 0; k < 3; ++k) { out.n[k] = 0; out.v[k].reset(); }
    const size_t m = (size_t)g.m;
    if (m == 0 || max_len < 3) return RAMA_OK;
    // sign partition
    Buf<uint32_t> ppos, npos;
    RAMA_TRY(ppos.alloc(ctx, m + 1));
    RAMA_TRY(npos.alloc(ctx, m + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, PosFlag{g.c.get()}, ppos.get(), m)));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, NegFlag{g.c.get()}, npos.get(), m)));
    uint32_t mp = 0, mr = 0;
    RAMA_TRY(read_back(ctx, &mp, ppos.get() + m, 4));
    RAMA_TRY(read_back(ctx, &mr, npos.get() + m, 4));
    if (mp == 0 || mr == 0) return RAMA_OK;
    if ((uint64_t)2 * mp >= (uint64_t(1) << 31)) return fail(ctx, RAMA_ERR_CAPACITY, "positive adjacency reaches 2^31 entries");
    Buf<int32_t> pi, pj, ri, rj;
    Buf<uint32_t> lkey, lval;
    RAMA_TRY(pi.alloc(ctx, mp));
    RAMA_TRY(pj.alloc(ctx, mp));
    RAMA_TRY(lkey.alloc(ctx, mp));
    RAMA_TRY(lval.alloc(ctx, mp));
    RAMA_TRY(ri.alloc(ctx, mr));
    RAMA_TRY(rj.alloc(ctx, mr));
    {
        ProfScope ps_(ctx, "k_split_sign", (double)(m * 20 + (size_t)mp * 16 + (size_t)mr * 8));
        k_split_sign<<<grid_for(m), kBlock, 0, ctx.stream>>>(m, g.i.get(), g.j.get(), g.c.get(), ppos.get(), npos.get(),
                                                         pi.get(), pj.get(), lkey.get(), lval.get(), ri.get(), rj.get());
    }
    LAUNCH_TRY(ctx, "split_sign");
    ppos.reset();
    npos.reset();
    // positive CSR
    const int32_t n = g.n;
    Buf<int32_t> up_ptr, low_ptr, rowptr, nb;
    RAMA_TRY(up_ptr.alloc(ctx, (size_t)n + 1));
    RAMA_TRY(low_ptr.alloc(ctx, (size_t)n + 1));
    RAMA_TRY(rowptr.alloc(ctx, (size_t)n + 1));
    RAMA_TRY(nb.alloc(ctx, (size_t)2 * mp));
    RAMA_TRY((row_bounds<int32_t, int32_t>(ctx, pi.get(), mp, n, up_ptr.get())));
    RAMA_TRY((radix_sort_pairs<uint32_t, uint32_t>(ctx, lkey, lval, mp, bits_for((uint64_t)n))));
    RAMA_TRY((row_bounds<uint32_t, int32_t>(ctx, lkey.get(), mp, n, low_ptr.get())));
    {
        ProfScope ps_(ctx, "k_add_ptr", (double)(((size_t)n + 1) * 12));
        k_add_ptr<<<grid_for((size_t)n + 1), kBlock, 0, ctx.stream>>>(n, up_ptr.get(), low_ptr.get(), rowptr.get());
    }
    LAUNCH_TRY(ctx, "add_ptr");
    {
        ProfScope ps_(ctx, "k_fill_adj", (double)((size_t)mp * 24 + ((size_t)n + 1) * 12));
        k_fill_adj<<<grid_for(mp), kBlock, 0, ctx.stream>>>(mp, pi.get(), pj.get(), lkey.get(), lval.get(), up_ptr.get(),
                                                        low_ptr.get(), rowptr.get(), nb.get());
    }
    LAUNCH_TRY(ctx, "fill_adj");
    pi.reset(); pj.reset(); lkey.reset(); lval.reset(); up_ptr.reset(); low_ptr.reset();
    Adj adj{rowptr.get(), nb.get()};
    // count, scan, fill
    Buf<uint32_t> cnt[3];
    Buf<uint64_t> off[3];
    for (int k = 0; k < 3; ++k) {
        RAMA_TRY(cnt[k].alloc(ctx, mr));
        RAMA_TRY(off[k].alloc(ctx, (size_t)mr + 1));
    }
    {
        ProfScope ps_(ctx, "k_count_cycles", (double)((size_t)mr * 20 + ((size_t)n + 1) * 4 + (size_t)mp * 8));
        k_count_cycles<<<grid_for(mr), kBlock, 0, ctx.stream>>>(mr, ri.get(), rj.get(), adj, max_len, cnt[0].get(),
                                                           cnt[1].get(), cnt[2].get());
    }
    LAUNCH_TRY(ctx, "count_cycles");
    uint64_t tot[3];
    for (int k = 0; k < 3; ++k) {
        RAMA_TRY((exclusive_scan<uint64_t>(ctx, PtrInput<uint32_t>{cnt[k].get()}, off[k].get(), (size_t)mr)));
        RAMA_TRY(read_back(ctx, &tot[k], off[k].get() + mr, 8));
        out.n[k] = (int64_t)tot[k];
    }
    if (count_only) return RAMA_OK;
    for (int k = 0; k < 3; ++k) {
        if ((uint64_t)(k + 3) * tot[k] >= (uint64_t(1) << 31))
            return fail(ctx, RAMA_ERR_CAPACITY, "cycle list reaches 2^31 entries");
        RAMA_TRY(out.v[k].alloc(ctx, (size_t)(k + 3) * tot[k]));
    }
    if (tot[0] + tot[1] + tot[2] == 0) return RAMA_OK;
    Buf<uint32_t> hpos, hit;
    RAMA_TRY(hpos.alloc(ctx, (size_t)mr + 1));
    RAMA_TRY((exclusive_scan<uint32_t>(ctx, HasCycles{cnt[0].get(), cnt[1].get(), cnt[2].get()}, hpos.get(), (size_t)mr)));
    uint32_t nh = 0;
    RAMA_TRY(read_back(ctx, &nh, hpos.get() + mr, 4));
    RAMA_TRY(hit.alloc(ctx, nh));
    {
        ProfScope ps_(ctx, "k_collect_hits", (double)((size_t)mr * 16 + (size_t)nh * 4));
        k_collect_hits<<<grid_for(mr), kBlock, 0, ctx.stream>>>(mr, cnt[0].get(), cnt[1].get(), cnt[2].get(), hpos.get(),
                                                               hit.get());
    }
    LAUNCH_TRY(ctx, "collect_hits");
    {
        ProfScope ps_(ctx, "k_fill_cycles", (double)((size_t)nh * 44 + ((size_t)n + 1) * 4 + (size_t)mp * 8 + 12.0 * tot[0] + 16.0 * tot[1] + 20.0 * tot[2]));
        k_fill_cycles<<<grid_for(nh), kBlock, 0, ctx.stream>>>(nh, hit.get(), ri.get(), rj.get(), adj, cnt[1].get(),
                                                              cnt[2].get(), off[0].get(), off[1].get(), off[2].get(),
                                                              out.v[0].get(), out.v[1].get(), out.v[2].get());
    }
    LAUNCH_TRY(ctx, "fill_cycles");
    return RAMA_OK;
}

}  // namespace rama
