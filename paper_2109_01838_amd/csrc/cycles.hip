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

// both sign counters in one scan: attractive edges count in the low word, repulsive ones in the high word
struct SignFlags {
    static constexpr int bytes = 4;   // bytes read per item
    static constexpr const char *tag = "SignFlags";
    const float *c;
    __device__ __forceinline__ uint64_t operator()(size_t e) const
    {
        const float w = c[e];
        return w > 0.0f ? 1ull : (w < 0.0f ? (1ull << 32) : 0ull);
    }
};

// consumer of the scan over SignFlags: an attractive edge goes to place low(prefix) of the attractive
// list (the lower half of the adjacency is sorted from its pairs read as (j,i)), a repulsive one
// to place high(prefix) of the repulsive list
struct SplitSignEmit {
    static constexpr const char *tag = "SplitSign";
    const int32_t *i, *j;
    int32_t *pi, *pj;
    int32_t *ri, *rj;
    __device__ __forceinline__ void operator()(size_t e, uint64_t sign, uint64_t prefix) const
    {
        if (sign == 0) return;
        const int32_t a = i[e], b = j[e];
        if (sign == 1ull) {
            const uint32_t p = (uint32_t)prefix;
            pi[p] = a; pj[p] = b;
        } else {
            const uint32_t p = (uint32_t)(prefix >> 32);
            ri[p] = a; rj[p] = b;
        }
    }
};

// row pointers of N+ = lower + upper part; *longest (optional) collects the longest row
__global__ __launch_bounds__(kBlock) void k_add_ptr(int32_t n, const int32_t *a, const int32_t *b, int32_t *out,
                                                    uint32_t *longest)
{
    int32_t v = blockIdx.x * kBlock + threadIdx.x;
    if (v <= n) out[v] = a[v] + b[v];
    if (longest) block_max_into(v < n ? (uint32_t)((a[v + 1] - a[v]) + (b[v + 1] - b[v])) : 0u, longest);
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

// both rows (at most N entries each) are fetched whole with 16-byte loads -- one wait instead of a
// chain of dependent probes -- and compared in registers; f is called for the common entries in
// ascending order.  The array is padded by kWideRow entries; what lies behind a row's end is masked out.
template <int N, typename F>
__device__ __forceinline__ void intersect_in_registers(const Adj &g, int32_t a0, int32_t a1, int32_t b0, int32_t b1, F &&f)
{
    int32_t ra[N], rb[N];
    __builtin_memcpy(ra, g.nb + a0, sizeof(ra));
    __builtin_memcpy(rb, g.nb + b0, sizeof(rb));
#pragma unroll
    for (int k = 0; k < N; ++k) {
        ra[k] = a0 + k < a1 ? ra[k] : -1;
        rb[k] = b0 + k < b1 ? rb[k] : -2;
    }
#pragma unroll
    for (int k = 0; k < N; ++k) {
        bool hit = false;
#pragma unroll
        for (int q = 0; q < N; ++q) hit |= (ra[k] == rb[q]);
        if (hit) f(ra[k]);
    }
}

// calls f(x) for every x in row a & row b, ascending.  Rows of up to kWideRow entries -- nearly all
// rows of the contracted graphs -- are compared in registers; longer ones: walk the shorter row,
// bisect the longer (a chain of dependent loads: measured, this fallback used to take half of the
// triangle search's time when it started at nine entries).
constexpr int kShortRow = 8;
constexpr int kWideRow = 16;
template <typename F>
__device__ __forceinline__ void intersect_rows(const Adj &g, int32_t a, int32_t b, F &&f)
{
    int32_t a0 = g.ptr[a], a1 = g.ptr[a + 1], b0 = g.ptr[b], b1 = g.ptr[b + 1];
    if (a0 == a1 || b0 == b1) return;
    if (a1 - a0 <= kShortRow && b1 - b0 <= kShortRow) {
        intersect_in_registers<kShortRow>(g, a0, a1, b0, b1, f);
        return;
    }
    if (a1 - a0 <= kWideRow && b1 - b0 <= kWideRow) {
        intersect_in_registers<kWideRow>(g, a0, a1, b0, b1, f);
        return;
    }
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
    // The rows of the entries, for closing the last hop from vL's side (the appendix algorithm's meeting
    // in the middle): the walk is at its last inner node `tail`, and instead of fetching N+(tail) and
    // testing its entries against N+(vL), every entry v of N+(vL) tests whether tail is in N+(v).  These
    // rows are the same for the whole search of one repulsive edge, so they are fetched once, where the
    // walk would fetch one row per path that reaches its last level.
    int32_t rows[kRowRegs][kRowRegs];
    bool rows_ok;   // N+(vL) and the rows of all its entries have at most kRowRegs entries and are loaded
    __device__ __forceinline__ void load(const Adj &g, int32_t vl)
    {
        nb = g.nb; b0 = g.ptr[vl]; b1 = g.ptr[vl + 1];
        in_regs = (b1 - b0) <= kRowRegs;
        rows_ok = false;
#pragma unroll
        for (int k = 0; k < kRowRegs; ++k) r[k] = (in_regs && b0 + k < b1) ? nb[b0 + k] : -1;
    }
    __device__ __forceinline__ void load_rows(const Adj &g)
    {
        bool ok = in_regs;
        int32_t p0[kRowRegs], p1[kRowRegs];
#pragma unroll
        for (int k = 0; k < kRowRegs; ++k) {
            p0[k] = 0; p1[k] = 0;
            if (r[k] >= 0) { p0[k] = g.ptr[r[k]]; p1[k] = g.ptr[r[k] + 1]; }
            ok &= (p1[k] - p0[k]) <= kRowRegs;
        }
#pragma unroll
        for (int k = 0; k < kRowRegs; ++k) {
            // two 16-byte loads per row (the array is padded); what lies behind the row's end becomes -1
            int32_t row[kRowRegs];
            __builtin_memcpy(row, nb + p0[k], sizeof(row));
#pragma unroll
            for (int q = 0; q < kRowRegs; ++q) rows[k][q] = (ok && p0[k] + q < p1[k]) ? row[q] : -1;
        }
        rows_ok = ok;
    }
    // entry k of N+(vL) has `x` in its row
    __device__ __forceinline__ bool row_has(int k, int32_t x) const
    {
        bool f = false;
#pragma unroll
        for (int q = 0; q < kRowRegs; ++q) f |= (rows[k][q] == x);
        return f;
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

// Depth-first walk v0 -> v1 -> v2 -> ... along N+, closing on N+(vL) at every depth: a node v_K
// reached over K attractive hops that lies in N+(vL) closes the (K+2)-cycle (v0,..,v_K,vL).  For
// length 5 these are the appendix algorithm's pairs (v1,v3) with common neighbour v2, visited
// path-first.  vL and v0 are never in N+(vL) / N+(v0) of a repulsive edge and a row never holds its
// own node, so a closing node only has to differ from the inner path nodes; a node the walk
// continues through must also differ from v0 and vL.  Rows are ascending, so every list comes out
// in path order.  The recursion is over a compile-time depth: it unrolls into nested loops with
// the path in registers.
// [r0, r1) is the row of path[K-1]: the level above fetched the bounds while it was still busy with
// the previous neighbour, so that a level does not start with a load it has to wait for.
template <int K, int MAXL, typename Emit>
__device__ __forceinline__ void extend_path(const Adj &g, const EndRow &end, int32_t vl, int max_len,
                                            int32_t (&path)[MAXL], Emit &emit, int32_t r0, int32_t r1)
{
    if constexpr (K >= 3) {
        if (K + 3 > max_len && end.rows_ok) {
            // Last level, met from vL's side: no row of the tail is fetched at all.  N+(vL) is ascending,
            // so the closing nodes come in the same order as from the tail's row.
            const int32_t tail = path[K - 1];
#pragma unroll
            for (int k = 0; k < kRowRegs; ++k) {
                const int32_t v = end.r[k];
                bool inner = false;
#pragma unroll
                for (int q = 1; q < K - 1; ++q) inner |= (path[q] == v);
                if (v >= 0 && !inner && end.row_has(k, tail)) { path[K] = v; emit.template cycle<K + 2>(path); }
            }
            return;
        }
    }
    if (K + 3 > max_len && r1 - r0 <= kShortRow) {
        // Last level (nothing continues below) and a short row: its entries come in with two 16-byte
        // loads instead of one dependent load per turn of a loop -- the walk spends most of its time
        // waiting for exactly these loads.  (The array is padded; entries behind the row's end are skipped.)
        int32_t row[kShortRow];
        __builtin_memcpy(row, g.nb + r0, sizeof(row));
#pragma unroll
        for (int k = 0; k < kShortRow; ++k) {
            if (r0 + k < r1) {
                const int32_t v = row[k];
                bool inner = false;
#pragma unroll
                for (int q = 1; q < K - 1; ++q) inner |= (path[q] == v);
                if (!inner && end.has(v)) { path[K] = v; emit.template cycle<K + 2>(path); }
            }
        }
        return;
    }
    // the level below needs its row's bounds -- unless it is the last one and closes from vL's side
    const bool deeper = (K + 3 <= MAXL) && (K + 3 <= max_len) && !(K >= 2 && K + 4 > max_len && end.rows_ok);
    int32_t vn = r0 < r1 ? g.nb[r0] : 0, n0 = 0, n1 = 0;      // the neighbour of the coming turn and its row
    if (deeper && r0 < r1) { n0 = g.ptr[vn]; n1 = g.ptr[vn + 1]; }
    for (int32_t p = r0; p < r1; ++p) {
        const int32_t v = vn, c0 = n0, c1 = n1;
        if (p + 1 < r1) {
            vn = g.nb[p + 1];
            if (deeper) { n0 = g.ptr[vn]; n1 = g.ptr[vn + 1]; }
        }
        bool inner = false;
#pragma unroll
        for (int q = 1; q < K - 1; ++q) inner |= (path[q] == v);
        if (inner) continue;
        if (end.has(v)) { path[K] = v; emit.template cycle<K + 2>(path); }
        if constexpr (K + 3 <= MAXL) {
            if (K + 3 > max_len || v == vl || v == path[0]) continue;
            path[K] = v;
            extend_path<K + 1, MAXL>(g, end, vl, max_len, path, emit, c0, c1);
        }
    }
}
template <int K, int MAXL, typename Emit>
__device__ __forceinline__ void extend_path(const Adj &g, const EndRow &end, int32_t vl, int max_len,
                                            int32_t (&path)[MAXL], Emit &emit)
{
    const int32_t tail = path[K - 1];
    extend_path<K, MAXL>(g, end, vl, max_len, path, emit, g.ptr[tail], g.ptr[tail + 1]);
}

template <int MAXL, bool MEET = false, typename Emit>
__device__ __forceinline__ void enumerate_cycles(const Adj &g, int32_t v0, int32_t vl, int max_len, Emit &emit)
{
    int32_t path[MAXL];
    path[0] = v0;
    if (max_len <= 3) {
        intersect_rows(g, v0, vl, [&](int32_t v1) { path[1] = v1; emit.template cycle<3>(path); });
        return;
    }
    EndRow end;
    end.load(g, vl);
    if (end.b0 == end.b1) return;
    if constexpr (MEET)
        if (max_len >= 5) end.load_rows(g);   // the last level (three or more hops from v0) closes from vL's side
    extend_path<1, MAXL>(g, end, vl, max_len, path, emit);
}

// the walk below one given first hop v1 (what the walk from v0 does for each entry of its row)
template <int MAXL, typename Emit>
__device__ __forceinline__ void walk_from_first(const Adj &g, const EndRow &end, int32_t v0, int32_t v1, int32_t vl,
                                                int max_len, Emit &emit)
{
    int32_t path[MAXL];
    path[0] = v0; path[1] = v1;
    if (end.has(v1)) emit.template cycle<3>(path);
    if constexpr (MAXL >= 4)
        if (max_len >= 4) extend_path<2, MAXL>(g, end, vl, max_len, path, emit);
}

// A repulsive edge whose first endpoint has a long attractive row is "heavy": one thread would walk
// the whole row alone while its wave waits.  The per-thread kernels put such edges on a list
// instead, and a second kernel gives each listed edge to a whole wave, one first hop per lane.
// (Walks of length 3 are row intersections and stay with the per-thread kernels.)
constexpr size_t kListHitsFrom = size_t(1) << 17;
constexpr int kHeavyRow = 128;
constexpr unsigned kHeavyGroups = 512;
__device__ __forceinline__ bool heavy_edge(const Adj &g, int32_t v0, int max_len)
{
    return max_len >= 4 && g.ptr[v0 + 1] - g.ptr[v0] > kHeavyRow;
}

template <int MAXL>
struct CountEmit {
    uint32_t n[MAXL - 2];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int k = 0; k < MAXL - 2; ++k) n[k] = 0;
    }
    template <int L>
    __device__ __forceinline__ void cycle(const int32_t (&)[MAXL])
    {
        n[L - 3] += (n[L - 3] != 0xffffffffu);   // saturates; the host reports it
    }
};

template <int MAXL>
struct FillEmit {
    int32_t vl;
    int32_t *o[MAXL - 2];
    template <int L>
    __device__ __forceinline__ void cycle(const int32_t (&path)[MAXL])
    {
        int32_t *w = o[L - 3];
#pragma unroll
        for (int q = 0; q < L - 1; ++q) w[q] = path[q];
        w[L - 1] = vl;
        o[L - 3] = w + L;
    }
};

// per-list arrays of one repulsive-edge table: list k (the (k+3)-cycles) starts at k*stride
template <typename T, int N>
struct ListPtrs {
    T *p[N];
};

// counts per repulsive edge and length.  shortest_only: deepen the walk one length at a time
// and stop at the first length that closes a cycle (the hop distance in (V,E+) plus one); only
// that length's count is kept.  All lanes of a wave call this together; `valid` says whether the
// lane has an edge r.
template <int MAXL, bool MEET>
__device__ __forceinline__ void count_edge(bool valid, size_t r, const int32_t *ri, const int32_t *rj, const Adj &g,
                                           int max_len, int flags, const ListPtrs<uint32_t, MAXL - 2> &cnt,
                                           uint32_t *heavy, uint32_t *n_heavy, uint32_t *saturated)
{
    const bool shortest_only = flags != 0;
    const bool is_heavy = valid && heavy_edge(g, ri[r], max_len);
    const unsigned long long vote = __ballot(is_heavy);
    if (vote) {   // the wave's heavy edges join the list with one atomic
        const int lane = (int)(threadIdx.x & 63);
        uint32_t base = 0;
        if (lane == __ffsll((long long)vote) - 1) base = atomicAdd(n_heavy, (uint32_t)__popcll(vote));
        base = (uint32_t)__shfl((int)base, __ffsll((long long)vote) - 1, 64);
        if (is_heavy) heavy[base + (uint32_t)__popcll(vote & ((1ull << lane) - 1ull))] = (uint32_t)r;
    }
    if (!valid || is_heavy) return;
    CountEmit<MAXL> em;
    em.clear();
    if (!shortest_only) {
        enumerate_cycles<MAXL, MEET>(g, ri[r], rj[r], max_len, em);
    } else {
        for (int L = 3; L <= max_len; ++L) {
            em.clear();
            enumerate_cycles<MAXL, MEET>(g, ri[r], rj[r], L, em);
            uint32_t any = 0;   // only length L can have closed: shorter ones were tried before
#pragma unroll
            for (int k = 0; k < MAXL - 2; ++k) any |= em.n[k];
            if (any) break;
        }
    }
    bool sat = false;
#pragma unroll
    for (int k = 0; k < MAXL - 2; ++k)
        if (k + 3 <= max_len) { cnt.p[k][r] = em.n[k]; sat |= (em.n[k] == 0xffffffffu); }
    if (sat) *saturated = 1u;   // a count that reached 2^32-1 may have lost cycles: the host turns this into an error
}

template <int MAXL, bool MEET>
__global__ __launch_bounds__(kBlock) void k_count_cycles(size_t nr, const int32_t *ri, const int32_t *rj, Adj g,
                                                         int max_len, int flags,
                                                         ListPtrs<uint32_t, MAXL - 2> cnt, uint32_t *heavy,
                                                         uint32_t *n_heavy, uint32_t *saturated)
{
    const size_t r = (size_t)blockIdx.x * kBlock + threadIdx.x;
    count_edge<MAXL, MEET>(r < nr, r, ri, rj, g, max_len, flags, cnt, heavy, n_heavy, saturated);
}

// the same for the repulsive edges on a list whose length is only known on the device (fixed grid,
// every workgroup strides over the list)
template <int MAXL, bool MEET>
__global__ __launch_bounds__(kBlock) void k_count_cycles_listed(const uint32_t *list, const uint32_t *n_list,
                                                                const int32_t *ri, const int32_t *rj, Adj g, int max_len,
                                                                int flags, ListPtrs<uint32_t, MAXL - 2> cnt,
                                                                uint32_t *heavy, uint32_t *n_heavy, uint32_t *saturated)
{
    const size_t n = *n_list;
    for (size_t base = (size_t)blockIdx.x * kBlock; base < n; base += (size_t)gridDim.x * kBlock) {
        const size_t q = base + threadIdx.x;
        const bool valid = q < n;
        count_edge<MAXL, MEET>(valid, valid ? list[q] : 0, ri, rj, g, max_len, flags, cnt, heavy, n_heavy, saturated);
    }
}

// counts of the listed heavy edges: a wave per edge, lane l takes the first hops l, l+64, ...
template <int MAXL>
__global__ __launch_bounds__(kBlock) void k_count_cycles_heavy(const uint32_t *heavy, const uint32_t *n_heavy,
                                                               const int32_t *ri, const int32_t *rj, Adj g, int max_len,
                                                               int shortest_only, ListPtrs<uint32_t, MAXL - 2> cnt,
                                                               uint32_t *saturated)
{
    const uint32_t nh = *n_heavy;
    const int lane = (int)(threadIdx.x & 63);
    for (uint32_t h = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6); h < nh; h += gridDim.x * (kBlock / 64)) {
        const uint32_t r = heavy[h];
        const int32_t v0 = ri[r], vl = rj[r];
        EndRow end;
        end.load(g, vl);
        const int32_t r0 = g.ptr[v0], r1 = g.ptr[v0 + 1];
        unsigned long long tot[MAXL - 2];
        for (int L = shortest_only ? 3 : max_len; L <= max_len; ++L) {
            CountEmit<MAXL> em;
            em.clear();
            if (end.b0 != end.b1)
                for (int32_t p = r0 + lane; p < r1; p += 64) walk_from_first<MAXL>(g, end, v0, g.nb[p], vl, L, em);
            unsigned long long any = 0;
#pragma unroll
            for (int k = 0; k < MAXL - 2; ++k) {
                tot[k] = wave_sum((unsigned long long)em.n[k]);
                any |= tot[k];
            }
            if (any) break;   // plain search: single pass at full depth; shortest only: first length that closes
        }
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < MAXL - 2; ++k)
                if (k + 3 <= max_len) {
                    cnt.p[k][r] = tot[k] >= 0xffffffffull ? 0xffffffffu : (uint32_t)tot[k];
                    if (tot[k] >= 0xffffffffull) *saturated = 1u;
                }
        }
    }
}

template <int MAXL>
struct HasCycles {
    static constexpr int bytes = 4;   // bytes read per item: at least one count (one per list searched)
    static constexpr const char *tag = MAXL > 5 ? "HasCycles7" : "HasCycles";
    ListPtrs<uint32_t, MAXL - 2> cnt;
    int live;   // bit mask of the lists that hold any cycle
    __device__ __forceinline__ uint32_t operator()(size_t r) const
    {
        uint32_t any = 0;
#pragma unroll
        for (int k = 0; k < MAXL - 2; ++k)
            if (live & (1 << k)) any |= cnt.p[k][r];
        return any ? 1u : 0u;
    }
};

// consumer of the scan over HasCycles: the repulsive edges that close a cycle
struct CollectHitsEmit {
    static constexpr const char *tag = "CollectHits";
    uint32_t *hit;
    __device__ __forceinline__ void operator()(size_t r, uint32_t any, uint32_t p) const
    {
        if (any) hit[p] = (uint32_t)r;
    }
};

// the list totals (last entry of every offset array) and the saturation flag, side by side for one read-back
template <int NL>
__global__ void k_cycle_totals(ListPtrs<uint64_t, NL> off, size_t mr, int lists, const uint32_t *saturated, uint64_t *summary)
{
    const int k = (int)threadIdx.x;
    if (k < lists) summary[k] = off.p[k][mr];
    if (k == NL) summary[NL] = *saturated;
}

// second walk, only over the repulsive edges that have cycles and only as deep as their
// longest cycle; writes every list at the offsets of the scan
template <int MAXL, bool MEET>
__device__ __forceinline__ void fill_edge(uint32_t r, const int32_t *ri, const int32_t *rj, const Adj &g, int live,
                                          int max_len, const ListPtrs<uint32_t, MAXL - 2> &cnt,
                                          const ListPtrs<uint64_t, MAXL - 2> &off, const ListPtrs<int32_t, MAXL - 2> &out)
{
    if (heavy_edge(g, ri[r], max_len)) return;   // written by k_fill_cycles_heavy
    int depth = 0;
    FillEmit<MAXL> em;
    em.vl = rj[r];
#pragma unroll
    for (int k = 0; k < MAXL - 2; ++k) {
        em.o[k] = nullptr;
        if (live & (1 << k)) {   // `live`: bit k set iff list k holds any cycle at all (the arrays of empty lists are not touched)
            if (cnt.p[k][r]) depth = k + 3;
            em.o[k] = out.p[k] + (size_t)(k + 3) * off.p[k][r];
        }
    }
    if (depth) enumerate_cycles<MAXL, MEET>(g, ri[r], em.vl, depth, em);
}

template <int MAXL, bool MEET>
__global__ __launch_bounds__(kBlock) void k_fill_cycles(size_t nh, const uint32_t *hit, const int32_t *ri,
                                                        const int32_t *rj, Adj g, int live, int max_len,
                                                        ListPtrs<uint32_t, MAXL - 2> cnt,
                                                        ListPtrs<uint64_t, MAXL - 2> off,
                                                        ListPtrs<int32_t, MAXL - 2> out)
{
    size_t h = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (h >= nh) return;
    fill_edge<MAXL, MEET>(hit ? hit[h] : (uint32_t)h, ri, rj, g, live, max_len, cnt, off, out);
}

template <int MAXL, bool MEET>
__global__ __launch_bounds__(kBlock) void k_fill_cycles_listed(const uint32_t *list, const uint32_t *n_list,
                                                               const int32_t *ri, const int32_t *rj, Adj g, int live,
                                                               int max_len, ListPtrs<uint32_t, MAXL - 2> cnt,
                                                               ListPtrs<uint64_t, MAXL - 2> off,
                                                               ListPtrs<int32_t, MAXL - 2> out)
{
    const size_t n = *n_list;
    for (size_t q = (size_t)blockIdx.x * kBlock + threadIdx.x; q < n; q += (size_t)gridDim.x * kBlock)
        fill_edge<MAXL, MEET>(list[q], ri, rj, g, live, max_len, cnt, off, out);
}

// ---- cooperative search for cycles of length up to 5 ---------------------------------------------
// The appendix algorithm "Parallel Conf. 5-Cycles" meets in the middle: for a repulsive edge (v0,vL)
// it pairs v1 in N+(v0) with v3 in N+(vL) and intersects N+(v1) with N+(v3).  Only the rows of the two
// endpoints and of their neighbours are touched -- 2d+2 rows instead of the d^2+d+2 rows a walk from v0
// over three hops fetches -- and all of them can be requested at once.  Sixteen lanes share one edge:
// they stage N+(v0), N+(vL) and the rows of N+(vL)'s entries in LDS (every lane fetches one row), then
// take the pairs (v1, v2), v2 in N+(v1), sixteen at a time in list order; a lane tests its v2 against
// N+(vL) (a 4-cycle) and against the staged row of every v3 (5-cycles) out of LDS.  The count kernel
// adds the lanes' hits up; the fill kernel places them with prefix sums over the sixteen lanes, so the
// lists come out in the same order as from the walk: (v0, vL, v1, v2, v3).
// Edges with a row beyond the staged sizes go to a list that the walking kernels work off.
constexpr int kCoopLanes = 16;                     // lanes per repulsive edge (one DPP row)
constexpr int kCoopEdges = kBlock / kCoopLanes;    // edges per workgroup
constexpr int kCoopCap = 16;                       // longest N+(v0), N+(vL) and N+(v3) that are staged
constexpr int kCoopCapA = 64;                      // longest N+(v1) (read from memory, bounds the pairs per edge)
struct alignas(16) CoopStage {
    int32_t rowA[kCoopCap];                   // N+(v0)
    int32_t rowB[kCoopCap];                   // N+(vL), -1 behind its end
    int32_t startA[kCoopCap];                 // where the row of rowA[k] starts in the adjacency array
    int32_t offA[kCoopCap];                   // pairs before the row of rowA[k]; the largest int behind the last row
    int32_t rowsB[kCoopCap][kCoopCap];        // the rows of rowB[k], -1 behind their ends
};
// what every lane of a group keeps in registers once the rows are staged: one wait for eight 16-byte
// LDS reads instead of a wait per entry inside the loops over the pairs
struct CoopRegs {
    int32_t rowB[kCoopCap];
    int32_t offA[kCoopCap];
    __device__ __forceinline__ void load(const CoopStage &S)
    {
        __builtin_memcpy(rowB, S.rowB, sizeof(rowB));
        __builtin_memcpy(offA, S.offA, sizeof(offA));
    }
};

__device__ __forceinline__ uint32_t group_ballot(bool p)
{
    return (uint32_t)(__ballot(p) >> (lane_id() & 48)) & 0xffffu;
}
__device__ __forceinline__ uint32_t group_sum(uint32_t v)
{
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) v += (uint32_t)__shfl_xor((int)v, off, kCoopLanes);
    return v;
}
// exclusive prefix over the sixteen lanes of a group; *total = the group's sum
__device__ __forceinline__ uint32_t group_exclusive_scan(uint32_t v, uint32_t *total)
{
    uint32_t inc = v;
    inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x111, 0xf, 0xf, false);   // row_shr:1
    inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x112, 0xf, 0xf, false);   // row_shr:2
    inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x114, 0xf, 0xf, false);   // row_shr:4
    inc += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)inc, 0x118, 0xf, 0xf, false);   // row_shr:8
    *total = (uint32_t)__shfl((int)inc, kCoopLanes - 1, kCoopLanes);
    return inc - v;
}

// what a group knows about its edge after staging
struct CoopEdge {
    int32_t v0, vl;
    int dA, dB;
    uint32_t pairs;     // number of (v1, v2) pairs
    int32_t my_v1;      // lane k < dA: rowA[k]
    bool live;          // the edge is searched here (valid, both rows non-empty, everything fits)
    bool spilled;       // a row is too long: the walking kernels take this edge
};

// stages the rows of edge (v0, vl) for the calling group; the caller synchronises the workgroup afterwards
__device__ __forceinline__ CoopEdge coop_stage(CoopStage &S, bool valid, int32_t v0, int32_t vl, const Adj &g, int max_len)
{
    const int gl = (int)(threadIdx.x & (kCoopLanes - 1));
    CoopEdge E;
    E.v0 = v0; E.vl = vl; E.my_v1 = -1; E.pairs = 0;
    int32_t pa0 = 0, pa1 = 0, pb0 = 0, pb1 = 0;
    if (valid) { pa0 = g.ptr[v0]; pa1 = g.ptr[v0 + 1]; pb0 = g.ptr[vl]; pb1 = g.ptr[vl + 1]; }
    E.dA = pa1 - pa0; E.dB = pb1 - pb0;
    const bool fits = E.dA <= kCoopCap && E.dB <= kCoopCap;
    const bool search = valid && E.dA > 0 && E.dB > 0;
    bool too_long = false;
    uint32_t lenA = 0;
    if (search && fits) {
        if (gl < E.dA) {
            const int32_t v1 = g.nb[pa0 + gl];
            const int32_t q0 = g.ptr[v1];
            lenA = (uint32_t)(g.ptr[v1 + 1] - q0);
            S.rowA[gl] = v1; S.startA[gl] = q0;
            E.my_v1 = v1;
            too_long |= lenA > (uint32_t)kCoopCapA;
        }
        S.rowB[gl] = -1;
        if (gl < E.dB) {
            const int32_t v3 = g.nb[pb0 + gl];
            S.rowB[gl] = v3;
            if (max_len >= 5) {
                const int32_t s0 = g.ptr[v3];
                const int32_t lb = g.ptr[v3 + 1] - s0;
                if (lb > kCoopCap) {
                    too_long = true;
                } else {
                    // the whole row with four 16-byte loads (the array is padded; what lies behind the row's end becomes -1)
                    int32_t row[kCoopCap];
                    __builtin_memcpy(row, g.nb + s0, sizeof(row));
#pragma unroll
                    for (int q = 0; q < kCoopCap; ++q) row[q] = q < lb ? row[q] : -1;
                    __builtin_memcpy(S.rowsB[gl], row, sizeof(row));
                }
            }
        }
    }
    E.spilled = search && (!fits || group_ballot(too_long) != 0);
    E.live = search && !E.spilled;
    const uint32_t excl = group_exclusive_scan(E.live ? lenA : 0u, &E.pairs);
    S.offA[gl] = gl < E.dA ? (int32_t)excl : 0x7fffffff;
    return E;
}

// pair number w of the staged edge: v1, v2, whether (v0,v1,v2,vl) is a cycle, and -- as a bit mask over
// N+(vL) -- which v3 close the 5-cycle (v0,v1,v2,v3,vl)
__device__ __forceinline__ void coop_pair(const CoopStage &S, const CoopRegs &R, const CoopEdge &E, const Adj &g, uint32_t w,
                                          int max_len, int32_t &v1, int32_t &v2, bool &four, uint32_t &fives)
{
    int a = 0;
#pragma unroll
    for (int k = 1; k < kCoopCap; ++k) a += (R.offA[k] <= (int32_t)w);   // the last row that starts at or before w
    v1 = S.rowA[a];
    v2 = g.nb[S.startA[a] + ((int32_t)w - S.offA[a])];
    four = false;
#pragma unroll
    for (int b = 0; b < kCoopCap; ++b) four |= (R.rowB[b] == v2);
    fives = 0;
    if (max_len >= 5 && v2 != E.v0 && v2 != E.vl) {
#pragma unroll
        for (int b = 0; b < kCoopCap; ++b) {
            if (b < E.dB && R.rowB[b] != v1) {
                int32_t row[kCoopCap];
                __builtin_memcpy(row, S.rowsB[b], sizeof(row));
                bool hit = false;
#pragma unroll
                for (int q = 0; q < kCoopCap; ++q) hit |= (row[q] == v2);
                fives |= hit ? (1u << b) : 0u;
            }
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_count_cycles_coop(size_t nr, const int32_t *ri, const int32_t *rj, Adj g,
                                                              int max_len, int shortest_only, ListPtrs<uint32_t, 3> cnt,
                                                              uint32_t *spill, uint32_t *n_spill)
{
    __shared__ CoopStage stage[kCoopEdges];
    const int gl = (int)(threadIdx.x & (kCoopLanes - 1)), grp = (int)(threadIdx.x / kCoopLanes);
    CoopStage &S = stage[grp];
    const size_t r = (size_t)blockIdx.x * kCoopEdges + grp;
    const bool valid = r < nr;
    const CoopEdge E = coop_stage(S, valid, valid ? ri[r] : 0, valid ? rj[r] : 0, g, max_len);
    __syncthreads();
    uint32_t n3 = 0, n4 = 0, n5 = 0;
    if (E.live) {
        CoopRegs R;
        R.load(S);
        if (gl < E.dA) {
            bool hit = false;
#pragma unroll
            for (int b = 0; b < kCoopCap; ++b) hit |= (R.rowB[b] == E.my_v1);
            n3 = hit ? 1u : 0u;
        }
        for (uint32_t w = (uint32_t)gl; w < E.pairs; w += kCoopLanes) {
            int32_t v1, v2;
            bool four;
            uint32_t fives;
            coop_pair(S, R, E, g, w, max_len, v1, v2, four, fives);
            n4 += four ? 1u : 0u;
            n5 += (uint32_t)__popc(fives);
        }
    }
    n3 = group_sum(n3); n4 = group_sum(n4); n5 = group_sum(n5);
    if (shortest_only) {   // only the shortest length that closes a cycle is kept
        if (n3) { n4 = 0; n5 = 0; }
        else if (n4) n5 = 0;
    }
    if (valid && gl == 0) {
        cnt.p[0][r] = n3;
        if (max_len >= 4) cnt.p[1][r] = n4;
        if (max_len >= 5) cnt.p[2][r] = n5;
        if (E.spilled) spill[atomicAdd(n_spill, 1u)] = (uint32_t)r;   // counted again by the walking kernel
    }
}

__global__ __launch_bounds__(kBlock) void k_fill_cycles_coop(size_t nh, const uint32_t *hit, const int32_t *ri,
                                                             const int32_t *rj, Adj g, int max_len, int live,
                                                             ListPtrs<uint32_t, 3> cnt, ListPtrs<uint64_t, 3> off,
                                                             ListPtrs<int32_t, 3> out)
{
    __shared__ CoopStage stage[kCoopEdges];
    const int gl = (int)(threadIdx.x & (kCoopLanes - 1)), grp = (int)(threadIdx.x / kCoopLanes);
    CoopStage &S = stage[grp];
    const size_t h = (size_t)blockIdx.x * kCoopEdges + grp;
    bool valid = h < nh;
    const uint32_t r = valid ? (hit ? hit[h] : (uint32_t)h) : 0u;
    if (valid && !hit) {   // no list of the edges with cycles was made: look at the counts first
        uint32_t any = 0;   // `live`: bit k set iff list k holds any cycle at all
        if (live & 1) any |= cnt.p[0][r];
        if (live & 2) any |= cnt.p[1][r];
        if (live & 4) any |= cnt.p[2][r];
        valid = any != 0;
    }
    const CoopEdge E = coop_stage(S, valid, valid ? ri[r] : 0, valid ? rj[r] : 0, g, max_len);
    __syncthreads();
    if (!E.live) return;   // nothing to search, or written by the walking kernels; the whole group leaves
    // a list is written iff the count pass kept cycles of that length (with shortest_only: one length only)
    const bool want3 = (live & 1) && cnt.p[0][r] != 0;
    const bool want4 = (live & 2) && cnt.p[1][r] != 0;
    const bool want5 = (live & 4) && cnt.p[2][r] != 0;
    CoopRegs R;
    R.load(S);
    if (want3) {
        bool c3 = false;
        if (gl < E.dA) {
#pragma unroll
            for (int b = 0; b < kCoopCap; ++b) c3 |= (R.rowB[b] == E.my_v1);
        }
        const uint32_t vote = group_ballot(c3);
        if (c3) {
            int32_t *o = out.p[0] + 3 * (off.p[0][r] + (uint64_t)__popc(vote & ((1u << gl) - 1u)));
            o[0] = E.v0; o[1] = E.my_v1; o[2] = E.vl;
        }
    }
    if (!want4 && !want5) return;
    uint64_t at4 = want4 ? off.p[1][r] : 0, at5 = want5 ? off.p[2][r] : 0;
    for (uint32_t base = 0; base < E.pairs; base += kCoopLanes) {   // the same number of turns for every lane of the group
        const uint32_t w = base + (uint32_t)gl;
        int32_t v1 = 0, v2 = 0;
        bool four = false;
        uint32_t fives = 0;
        if (w < E.pairs) coop_pair(S, R, E, g, w, max_len, v1, v2, four, fives);
        if (want4) {
            const uint32_t vote = group_ballot(four);
            if (four) {
                int32_t *o = out.p[1] + 4 * (at4 + (uint64_t)__popc(vote & ((1u << gl) - 1u)));
                o[0] = E.v0; o[1] = v1; o[2] = v2; o[3] = E.vl;
            }
            at4 += (uint64_t)__popc(vote);
        }
        if (want5) {
            uint32_t total;
            const uint32_t before = group_exclusive_scan((uint32_t)__popc(fives), &total);
            int32_t *o = out.p[2] + 5 * (at5 + before);
            while (fives) {
                const int b = __ffs((int)fives) - 1;
                fives &= fives - 1;
                o[0] = E.v0; o[1] = v1; o[2] = v2; o[3] = S.rowB[b]; o[4] = E.vl;
                o += 5;
            }
            at5 += total;
        }
    }
}

// ---- triangles on graphs with long rows ----------------------------------------------------------
// The contracted graphs of later rounds can be dense (rows of 20-40 attractive neighbours and more).  One
// thread per repulsive edge then walks its shorter row alone, a dependent bisection of the longer row per
// entry.  Here sixteen lanes share the edge: they take the shorter row sixteen entries at a time, every lane
// bisects the longer row for its entry, and a ballot counts -- or, in the fill pass, places -- the common
// neighbours.  The shorter row is ascending, so the triangles (v0, v1, vL) come out in list order.
template <bool FILL>
__global__ __launch_bounds__(kBlock) void k_triangles_group(size_t nr, const uint32_t *hit, const int32_t *ri,
                                                            const int32_t *rj, Adj g, uint32_t *cnt0, const uint64_t *off0,
                                                            int32_t *out0)
{
    const int gl = (int)(threadIdx.x & (kCoopLanes - 1));
    const size_t h = (size_t)blockIdx.x * kCoopEdges + threadIdx.x / kCoopLanes;
    if (h >= nr) return;                                   // the whole group
    const uint32_t r = hit ? hit[h] : (uint32_t)h;
    if (FILL && cnt0[r] == 0) return;
    const int32_t v0 = ri[r], vl = rj[r];
    int32_t a0 = g.ptr[v0], a1 = g.ptr[v0 + 1], b0 = g.ptr[vl], b1 = g.ptr[vl + 1];
    if (a1 - a0 > b1 - b0) { int32_t t = a0; a0 = b0; b0 = t; t = a1; a1 = b1; b1 = t; }   // [a0,a1): the shorter row
    uint32_t found = 0;
    uint64_t at = FILL ? off0[r] : 0;
    if (b0 < b1)
        for (int32_t base = a0; base < a1; base += kCoopLanes) {   // the same number of turns for every lane of the group
            const int32_t p = base + gl;
            bool common = false;
            int32_t x = 0;
            if (p < a1) {
                x = g.nb[p];
                int32_t lo = b0, hi = b1;
                while (lo < hi) {
                    const int32_t mid = lo + ((hi - lo) >> 1);
                    if (g.nb[mid] < x) lo = mid + 1; else hi = mid;
                }
                common = lo < b1 && g.nb[lo] == x;
            }
            const uint32_t vote = group_ballot(common);
            if (FILL) {
                if (common) {
                    int32_t *o = out0 + 3 * (at + (uint64_t)__popc(vote & ((1u << gl) - 1u)));
                    o[0] = v0; o[1] = x; o[2] = vl;
                }
                at += (uint64_t)__popc(vote);
            } else {
                found += (uint32_t)__popc(vote);
            }
        }
    if (!FILL && gl == 0) cnt0[r] = found;
}

// cycles of the listed heavy edges: per round of 64 first hops every lane counts what its hop
// closes, a wave scan turns the counts into places, and the lane walks again and writes
template <int MAXL>
__global__ __launch_bounds__(kBlock) void k_fill_cycles_heavy(const uint32_t *heavy, const uint32_t *n_heavy,
                                                              const int32_t *ri, const int32_t *rj, Adj g, int live,
                                                              ListPtrs<uint32_t, MAXL - 2> cnt,
                                                              ListPtrs<uint64_t, MAXL - 2> off,
                                                              ListPtrs<int32_t, MAXL - 2> out)
{
    const uint32_t nh = *n_heavy;
    const int lane = (int)(threadIdx.x & 63);
    for (uint32_t h = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6); h < nh; h += gridDim.x * (kBlock / 64)) {
        const uint32_t r = heavy[h];
        int depth = 0;
        size_t place[MAXL - 2];   // cycles of this edge already written, per length
#pragma unroll
        for (int k = 0; k < MAXL - 2; ++k) {
            place[k] = 0;
            if (live & (1 << k)) {
                if (cnt.p[k][r]) depth = k + 3;
                place[k] = off.p[k][r];
            }
        }
        if (depth == 0) continue;
        const int32_t v0 = ri[r], vl = rj[r];
        EndRow end;
        end.load(g, vl);
        const int32_t r0 = g.ptr[v0], r1 = g.ptr[v0 + 1];
        for (int32_t p0 = r0; p0 < r1; p0 += 64) {
            const int32_t p = p0 + lane;
            const int32_t v1 = p < r1 ? g.nb[p] : -1;
            CountEmit<MAXL> em;
            em.clear();
            if (v1 >= 0) walk_from_first<MAXL>(g, end, v0, v1, vl, depth, em);
            FillEmit<MAXL> fe;
            fe.vl = vl;
#pragma unroll
            for (int k = 0; k < MAXL - 2; ++k) {
                fe.o[k] = nullptr;
                if (live & (1 << k)) {
                    const uint32_t inc = wave_inclusive_scan(em.n[k]);
                    fe.o[k] = out.p[k] + (size_t)(k + 3) * (place[k] + (inc - em.n[k]));
                    place[k] += wave_last(inc);
                }
            }
            if (v1 >= 0) walk_from_first<MAXL>(g, end, v0, v1, vl, depth, fe);
        }
    }
}

// count, scan, fill for walks of at most MAXL nodes
template <int MAXL>
rama_status count_and_fill(Ctx &ctx, size_t mr, const int32_t *ri, const int32_t *rj, Adj adj, int32_t n, size_t mp,
                           int max_len, bool shortest_only, bool count_only, CycleLists &out, uint32_t longest_row = 0xffffffffu)
{
    constexpr int NL = MAXL - 2;
    const int lists = max_len - 2;
    Buf<uint32_t> cnt[NL];
    Buf<uint64_t> off[NL];
    ListPtrs<uint32_t, NL> cp;
    ListPtrs<uint64_t, NL> op;
    ListPtrs<int32_t, NL> vp;
    for (int k = 0; k < NL; ++k) {
        cp.p[k] = nullptr; op.p[k] = nullptr; vp.p[k] = nullptr;
        if (k >= lists) continue;
        RAMA_TRY(cnt[k].alloc(ctx, mr));
        RAMA_TRY(off[k].alloc(ctx, mr + 1));
        cp.p[k] = cnt[k].get(); op.p[k] = off[k].get();
    }
    // heavy edges (only possible for max_len >= 4): listed by the first kernel, counted by the second,
    // which ends at once when the list is empty
    const bool may_be_heavy = max_len >= 4;
    // Lengths 4 and 5.  If every attractive row has at most kRowRegs entries (3-D grids), the walk holds the
    // rows it needs in registers and is the fastest; if rows are longer but still short on average (2-D
    // grids with long-range edges, neighbour graphs), the cooperative search stages them in LDS, and what
    // does not fit its staged sizes is listed and walked; with long rows on average (contracted graphs)
    // everything is walked.  Measured on the 320^3 grid (rows <= 6): walk 4.4 ms, cooperative 12.0 ms; on
    // the 512^2 grid with long-range edges (rows <= 12): 4.0 against 1.0 ms; on the 6-nearest-neighbour
    // graph of 10^6 points (rows of 3..15): 1.5 against 0.55 ms.
    bool coop = false;
    if constexpr (MAXL == 5) {
        const bool short_on_average = 2 * mp <= (size_t)12 * (size_t)n;
        const bool fit_registers = longest_row <= (uint32_t)kRowRegs;
        coop = max_len >= 4 && (ctx.cycle_search == 2 || (ctx.cycle_search == 0 && short_on_average && !fit_registers));
    }
    Buf<uint32_t> heavy, spill, n_heavy;   // n_heavy[0]: length of the heavy list, [1]: a count saturated, [2]: length of the spill list
    RAMA_TRY(heavy.alloc(ctx, may_be_heavy ? mr : 1));
    RAMA_TRY(spill.alloc(ctx, coop ? mr : 1));
    RAMA_TRY(zeroed<uint32_t>(ctx, 3, n_heavy));
    // mode 1 is the walk that fetches a row per path at its last level, kept for comparison; walks of at
    // most three nodes have no such level
    const bool meet = MAXL >= 5 && max_len >= 5 && ctx.cycle_search != 1;
    const int walk_flags = shortest_only ? 1 : 0;
    const double search_bytes = (double)(mr * (8 + 4 * (size_t)lists) + ((size_t)n + 1) * 4 + mp * 8);
    if constexpr (MAXL == 5) {
        if (coop) {
            {
                ProfScope ps_(ctx, "k_count_cycles_coop", search_bytes);
                k_count_cycles_coop<<<grid_for(mr, kCoopEdges), kBlock, 0, ctx.stream>>>(mr, ri, rj, adj, max_len, shortest_only ? 1 : 0,
                                                                                      cp, spill.get(), n_heavy.get() + 2);
            }
            LAUNCH_TRY(ctx, "count_cycles_coop");
            ProfScope ps_(ctx, "k_count_cycles_listed", 0.0);
            k_count_cycles_listed<MAXL, true><<<kHeavyGroups, kBlock, 0, ctx.stream>>>(spill.get(), n_heavy.get() + 2, ri, rj, adj, max_len,
                                                                                     walk_flags, cp, heavy.get(), n_heavy.get(),
                                                                                     n_heavy.get() + 1);
        }
    }
    // triangles only, rows of more than 12 attractive neighbours on average: sixteen lanes per repulsive edge
    bool wide3 = false;
    if constexpr (MAXL == 3)
        wide3 = ctx.cycle_search == 2 || (ctx.cycle_search == 0 && 2 * mp > (size_t)12 * (size_t)n);
    if (wide3) {
        ProfScope ps_(ctx, "k_count_triangles_group", search_bytes);
        k_triangles_group<false><<<grid_for(mr, kCoopEdges), kBlock, 0, ctx.stream>>>(mr, (const uint32_t *)nullptr, ri, rj, adj, cp.p[0],
                                                                                   (const uint64_t *)nullptr, (int32_t *)nullptr);
    } else if (!coop) {
        ProfScope ps_(ctx, MAXL == 3 ? "k_count_cycles<3>" : MAXL == 5 ? "k_count_cycles<5>" : "k_count_cycles<7>", search_bytes);
        if (meet)
            k_count_cycles<MAXL, (MAXL >= 5)><<<grid_for(mr), kBlock, 0, ctx.stream>>>(mr, ri, rj, adj, max_len, walk_flags, cp,
                                                                                      heavy.get(), n_heavy.get(), n_heavy.get() + 1);
        else
            k_count_cycles<MAXL, false><<<grid_for(mr), kBlock, 0, ctx.stream>>>(mr, ri, rj, adj, max_len, walk_flags, cp,
                                                                                heavy.get(), n_heavy.get(), n_heavy.get() + 1);
    }
    LAUNCH_TRY(ctx, "count_cycles");
    if (may_be_heavy) {
        ProfScope ps_(ctx, "k_count_cycles_heavy", 0.0);
        k_count_cycles_heavy<MAXL><<<kHeavyGroups, kBlock, 0, ctx.stream>>>(heavy.get(), n_heavy.get(), ri, rj, adj, max_len,
                                                                          shortest_only ? 1 : 0, cp, n_heavy.get() + 1);
        LAUNCH_TRY(ctx, "count_cycles_heavy");
    }
    uint64_t tot[NL + 1], all = 0;
    for (int k = 0; k < lists; ++k)
        RAMA_TRY((exclusive_scan<uint64_t>(ctx, PtrInput<uint32_t>{cnt[k].get()}, off[k].get(), mr)));
    {
        Buf<uint64_t> summary;
        RAMA_TRY(summary.alloc(ctx, NL + 1));
        k_cycle_totals<NL><<<1, 64, 0, ctx.stream>>>(op, mr, lists, n_heavy.get() + 1, summary.get());
        LAUNCH_TRY(ctx, "cycle_totals");
        RAMA_TRY(read_back(ctx, tot, summary.get(), sizeof(tot)));
    }
    if (tot[NL]) return fail(ctx, RAMA_ERR_CAPACITY, "a repulsive edge closes 2^32 - 1 or more cycles of one length");
    for (int k = 0; k < lists; ++k) {
        out.n[k] = (int64_t)tot[k];
        all += tot[k];
    }
    if (count_only) return RAMA_OK;
    double list_bytes = 0.0;
    for (int k = 0; k < lists; ++k) {
        if ((uint64_t)(k + 3) * tot[k] >= (uint64_t(1) << 31))
            return fail(ctx, RAMA_ERR_CAPACITY, "cycle list reaches 2^31 entries");
        RAMA_TRY(out.v[k].alloc(ctx, (size_t)(k + 3) * tot[k]));
        vp.p[k] = out.v[k].get();
        list_bytes += 4.0 * (k + 3) * (double)tot[k];
    }
    if (all == 0) return RAMA_OK;
    int live = 0;   // the lists that hold any cycle: the fill pass leaves the count and offset arrays of the others alone
    for (int k = 0; k < lists; ++k)
        if (tot[k]) live |= 1 << k;
    // The fill pass visits the repulsive edges that have cycles.  Listing them first pays on long lists; a
    // short one is visited whole (an edge without cycles costs its thread three loads) and the launches and
    // the count read-back of the listing are saved.
    const bool list_hits = mr > kListHitsFrom;
    Buf<uint32_t> hit;
    uint32_t nh = (uint32_t)mr;
    if (list_hits) {
        HasCycles<MAXL> has{cp, live};
        ScanPlan<uint32_t> hits;
        RAMA_TRY((scan_plan_alloc<uint32_t>(ctx, mr, 0, hits)));
        RAMA_TRY((scan_totals<uint32_t>(ctx, has, hits)));
        nh = hits.total;
        RAMA_TRY(hit.alloc(ctx, nh));
        RAMA_TRY((scan_emit<uint32_t>(ctx, has, CollectHitsEmit{hit.get()}, hits, (double)((size_t)nh * 4))));
    }
    const double fill_bytes = (double)((size_t)nh * (12 + 12 * (size_t)lists) + ((size_t)n + 1) * 4 + mp * 8) + list_bytes;
    // without 5-cycles (bipartite inputs) the fill only has to go two hops deep: the walk does that with
    // one row per first hop and needs nothing staged
    bool long_cycles = false;   // is there any cycle of length 5 or more to write?
    for (int k = 2; k < lists; ++k) long_cycles |= tot[k] != 0;
    if (!long_cycles) coop = false;
    if constexpr (MAXL == 5) {
        if (coop) {
            {
                ProfScope ps_(ctx, "k_fill_cycles_coop", fill_bytes);
                k_fill_cycles_coop<<<grid_for(nh, kCoopEdges), kBlock, 0, ctx.stream>>>(nh, list_hits ? hit.get() : nullptr, ri, rj, adj, max_len, live, cp, op, vp);
            }
            LAUNCH_TRY(ctx, "fill_cycles_coop");
            ProfScope ps_(ctx, "k_fill_cycles_listed", 0.0);
            k_fill_cycles_listed<MAXL, true><<<kHeavyGroups, kBlock, 0, ctx.stream>>>(spill.get(), n_heavy.get() + 2, ri, rj, adj, live,
                                                                                    max_len, cp, op, vp);
        }
    }
    if (wide3) {
        ProfScope ps_(ctx, "k_fill_triangles_group", fill_bytes);
        k_triangles_group<true><<<grid_for(nh, kCoopEdges), kBlock, 0, ctx.stream>>>(nh, list_hits ? hit.get() : nullptr, ri, rj, adj, cp.p[0],
                                                                                  op.p[0], vp.p[0]);
    } else if (!coop) {
        ProfScope ps_(ctx, MAXL == 3 ? "k_fill_cycles<3>" : MAXL == 5 ? "k_fill_cycles<5>" : "k_fill_cycles<7>", fill_bytes);
        if (meet && long_cycles)
            k_fill_cycles<MAXL, (MAXL >= 5)><<<grid_for(nh), kBlock, 0, ctx.stream>>>(nh, list_hits ? hit.get() : nullptr, ri, rj, adj, live, max_len, cp, op, vp);
        else
            k_fill_cycles<MAXL, false><<<grid_for(nh), kBlock, 0, ctx.stream>>>(nh, list_hits ? hit.get() : nullptr, ri, rj, adj, live, max_len, cp, op, vp);
    }
    LAUNCH_TRY(ctx, "fill_cycles");
    if (may_be_heavy) {
        ProfScope ps_(ctx, "k_fill_cycles_heavy", 0.0);
        k_fill_cycles_heavy<MAXL><<<kHeavyGroups, kBlock, 0, ctx.stream>>>(heavy.get(), n_heavy.get(), ri, rj, adj, live, cp,
                                                                         op, vp);
        LAUNCH_TRY(ctx, "fill_cycles_heavy");
    }
    return RAMA_OK;
}

}  // namespace

rama_status find_cycles(Ctx &ctx, const Graph &g, int max_len, bool shortest_only, bool count_only, CycleLists &out)
{
    for (int k = 0; k < kCycleLists; ++k) { out.n[k] = 0; out.v[k].reset(); }
    out.n_attractive = 0; out.n_repulsive = 0;
    const size_t m = (size_t)g.m;
    if (m == 0 || max_len < 3) return RAMA_OK;
    RAMA_TRY(zero_page_recycle(ctx));
    if (max_len > kMaxCycleLen) return fail(ctx, RAMA_ERR_INVALID_ARG, "cycle length beyond the supported maximum");
    // sign partition
    ScanPlan<uint64_t> signs;
    RAMA_TRY((scan_plan_alloc<uint64_t>(ctx, m, 0, signs)));
    RAMA_TRY((scan_totals<uint64_t>(ctx, SignFlags{g.c.get()}, signs, g.sign_sums.get())));   // tile sums, if the graph brings them
    const uint32_t mp = (uint32_t)signs.total, mr = (uint32_t)(signs.total >> 32);
    out.n_attractive = mp; out.n_repulsive = mr;
    if (mp == 0 || mr == 0) return RAMA_OK;
    if ((uint64_t)2 * mp >= (uint64_t(1) << 31)) return fail(ctx, RAMA_ERR_CAPACITY, "positive adjacency reaches 2^31 entries");
    Buf<int32_t> pi, pj, ri, rj;
    Buf<uint32_t> lkey, lval;
    RAMA_TRY(pi.alloc(ctx, mp));
    RAMA_TRY(pj.alloc(ctx, mp));
    RAMA_TRY(ri.alloc(ctx, mr));
    RAMA_TRY(rj.alloc(ctx, mr));
    RAMA_TRY((scan_emit<uint64_t>(ctx, SignFlags{g.c.get()},
                                  SplitSignEmit{g.i.get(), g.j.get(), pi.get(), pj.get(), ri.get(), rj.get()},
                                  signs, (double)(m * 8 + (size_t)mp * 8 + (size_t)mr * 8))));
    signs.offs.reset();
    // positive CSR
    const int32_t n = g.n;
    Buf<int32_t> up_ptr, low_ptr, rowptr, nb;
    RAMA_TRY(up_ptr.alloc(ctx, (size_t)n + 1));
    RAMA_TRY(low_ptr.alloc(ctx, (size_t)n + 1));
    RAMA_TRY(rowptr.alloc(ctx, (size_t)n + 1));
    RAMA_TRY(nb.alloc(ctx, (size_t)2 * mp + kWideRow));   // padded: short rows are read eight entries at a time
    // The choice between the two searches for lengths 4 and 5 needs the longest attractive row when the
    // rows are short on average (see count_and_fill).
    const bool want_longest = max_len >= 4 && max_len <= 5 && ctx.cycle_search == 0 && 2 * (size_t)mp <= (size_t)9 * (size_t)n / 2;
    Buf<uint32_t> longest;
    if (want_longest) {
        RAMA_TRY(zeroed<uint32_t>(ctx, 1, longest));
    }
    RAMA_TRY((row_bounds<int32_t, int32_t>(ctx, pi.get(), mp, n, up_ptr.get())));
    // lower neighbours: the attractive pairs read as (j, i), sorted by j (stable: i stays ascending)
    RAMA_TRY((radix_sort_pairs_from<uint32_t, uint32_t>(ctx, (const uint32_t *)pj.get(), (const uint32_t *)pi.get(), lkey, lval, mp,
                                                        bits_for((uint64_t)n), (uint64_t)n)));
    RAMA_TRY((row_bounds<uint32_t, int32_t>(ctx, lkey.get(), mp, n, low_ptr.get())));
    {
        ProfScope ps_(ctx, "k_add_ptr", (double)(((size_t)n + 1) * 12));
        k_add_ptr<<<grid_for((size_t)n + 1), kBlock, 0, ctx.stream>>>(n, up_ptr.get(), low_ptr.get(), rowptr.get(),
                                                                  want_longest ? longest.get() : nullptr);
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
    uint32_t longest_row = 0xffffffffu;   // unknown
    if (want_longest) RAMA_TRY(read_back(ctx, &longest_row, longest.get(), 4));
    // one instantiation per depth class: triangles are row intersections and need no walk state
    if (max_len <= 3)
        return count_and_fill<3>(ctx, (size_t)mr, ri.get(), rj.get(), adj, n, (size_t)mp, max_len, shortest_only, count_only, out);
    if (max_len <= 5)
        return count_and_fill<5>(ctx, (size_t)mr, ri.get(), rj.get(), adj, n, (size_t)mp, max_len, shortest_only, count_only, out,
                                 longest_row);
    return count_and_fill<kMaxCycleLen>(ctx, (size_t)mr, ri.get(), rj.get(), adj, n, (size_t)mp, max_len, shortest_only,
                                        count_only, out);
}

}  // namespace rama
