// Step a0: problem statement -> canonical device graph (paper Sec. 3: graph and cost vector;
// Lemma 1(b): parallel edges carry the sum of their costs).
#include "prim.h"
#include <algorithm>
#include <vector>

namespace rama {

namespace {

// flags[0]: endpoint out of range or non-finite cost; flags[1]: list is not canonical;
// flags[2]: largest |i-j| of a valid edge; flags[3]: number of places where the oriented pair (min, max) is smaller
// than the one before it (few of them: the list is a handful of sorted runs, e.g. one per grid direction).  A workgroup takes one tile of the scan over NotLoop (kScanTile
// edges) and leaves the number of edges that are no self-loops in tile_sums, so that scan needs no counting pass.
__global__ __launch_bounds__(kBlock) void k_validate(int32_t n, size_t m, const int32_t *i, const int32_t *j,
                                                     const float *c, int32_t *flags, uint32_t *tile_sums)
{
    const size_t base = (size_t)blockIdx.x * kScanTile + threadIdx.x;
    uint32_t diff = 0, kept = 0, down = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const size_t e = base + (size_t)q * kBlock;
        if (e >= m) continue;
        int32_t a = i[e], b = j[e];
        float w = c[e];
        kept += a != b ? 1u : 0u;
        bool bad = a < 0 || a >= n || b < 0 || b >= n || !(fabsf(w) <= 3.402823466e+38f);
        if (bad) {
            flags[0] = 1;
        } else {
            const uint32_t d = (uint32_t)abs(a - b);
            diff = d > diff ? d : diff;
            bool canon = a < b;
            if (e > 0) {
                const int32_t pa = i[e - 1], pb = j[e - 1];
                canon = canon && (pa < a || (pa == a && pb < b));
                const int32_t lo = min(a, b), hi = max(a, b), plo = min(pa, pb), phi = max(pa, pb);
                down += (lo < plo || (lo == plo && hi < phi)) ? 1u : 0u;
            }
            if (!canon) flags[1] = 1;
        }
    }
    kept = block_sum(kept);
    down = block_sum(down);
    if (threadIdx.x == 0) {
        tile_sums[blockIdx.x] = kept;
        if (down) atomicAdd((uint32_t *)&flags[3], down);
    }
    block_max_into(diff, (uint32_t *)&flags[2]);
}

struct NotLoop {
    static constexpr int bytes = 8;   // bytes read per item
    static constexpr const char *tag = "NotLoop";
    const int32_t *i, *j;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return i[e] != j[e] ? 1u : 0u; }
};

// consumer of the scan over NotLoop: edge e that is no self-loop goes to place p
struct PackEdgesEmit {
    static constexpr const char *tag = "PackEdges";
    const int32_t *i, *j;
    const float *c;
    int dbits;
    uint64_t *key;
    uint32_t *val;
    __device__ __forceinline__ void operator()(size_t e, uint32_t keep, uint32_t p) const
    {
        if (!keep) return;
        const int32_t a = i[e], b = j[e];
        key[p] = edge_key((uint32_t)min(a, b), (uint32_t)max(a, b), dbits);
        val[p] = __float_as_uint(c[e]);
    }
};

struct HeadFlag {
    static constexpr int bytes = 8;   // bytes read per item
    static constexpr const char *tag = "HeadFlag";
    const uint64_t *key;
    __device__ __forceinline__ uint32_t operator()(size_t e) const { return (e == 0 || key[e] != key[e - 1]) ? 1u : 0u; }
};

// ---- a list that consists of a few sorted runs is merged instead of sorted --------------------------------------
constexpr int kMaxRuns = 8;
constexpr int kMergeTile = 2048;

// places p >= 1 with key[p] < key[p-1]: out[0] counts them, out[1..] takes the first kMaxRuns - 1 (in any order)
__global__ __launch_bounds__(kBlock) void k_find_descents(const uint64_t *key, size_t n, uint32_t *out)
{
    const size_t p = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (p == 0 || p >= n) return;
    if (key[p] < key[p - 1]) {
        const uint32_t k = atomicAdd(out, 1u);
        if (k < (uint32_t)(kMaxRuns - 1)) out[1 + k] = (uint32_t)p;
    }
}

// Merge path: split[t] = how many of the first t * kMergeTile merged elements come from a (a's elements go first among
// equal keys, which keeps the merge stable).
__global__ __launch_bounds__(kBlock) void k_merge_partition(const uint64_t *a, uint32_t na, const uint64_t *b, uint32_t nb,
                                                            uint32_t ntiles, uint32_t *split)
{
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t > ntiles) return;
    const uint64_t d64 = (uint64_t)t * kMergeTile;
    const uint32_t diag = d64 < (uint64_t)na + nb ? (uint32_t)d64 : na + nb;
    uint32_t lo = diag > nb ? diag - nb : 0u, hi = diag < na ? diag : na;
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo) / 2;
        if (a[mid] <= b[diag - 1 - mid]) lo = mid + 1;
        else hi = mid;
    }
    split[t] = lo;
}

// One tile of the merged list: its pieces of a and b go to LDS side by side, every element finds its place by a
// bisection of the other piece, and the tile is written out in order.
__global__ __launch_bounds__(kBlock) void k_merge_pairs(const uint64_t *ak, const uint32_t *av, uint32_t na, const uint64_t *bk,
                                                        const uint32_t *bv, uint32_t nb, const uint32_t *split, uint64_t *ok,
                                                        uint32_t *ov)
{
    __shared__ uint64_t sk[kMergeTile];
    __shared__ uint32_t sv[kMergeTile];
    constexpr int kPer = kMergeTile / kBlock;
    const uint32_t t = blockIdx.x;
    const uint32_t diag0 = t * (uint32_t)kMergeTile;
    const uint32_t diag1 = (uint64_t)diag0 + kMergeTile < (uint64_t)na + nb ? diag0 + kMergeTile : na + nb;
    const uint32_t a0 = split[t], a1 = split[t + 1], b0 = diag0 - a0;
    const uint32_t cnt_a = a1 - a0, total = diag1 - diag0, cnt_b = total - cnt_a;
    for (uint32_t x = threadIdx.x; x < total; x += kBlock) {
        if (x < cnt_a) { sk[x] = ak[a0 + x]; sv[x] = av[a0 + x]; }
        else { sk[x] = bk[b0 + (x - cnt_a)]; sv[x] = bv[b0 + (x - cnt_a)]; }
    }
    __syncthreads();
    uint64_t k[kPer];
    uint32_t v[kPer], r[kPer];
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const uint32_t x = threadIdx.x + (uint32_t)q * kBlock;
        r[q] = 0xffffffffu;
        if (x >= total) continue;
        k[q] = sk[x]; v[q] = sv[x];
        uint32_t lo, hi;
        if (x < cnt_a) {           // elements of b that are smaller
            lo = 0; hi = cnt_b;
            while (lo < hi) { const uint32_t mid = (lo + hi) / 2; if (sk[cnt_a + mid] < k[q]) lo = mid + 1; else hi = mid; }
            r[q] = x + lo;
        } else {                   // elements of a that are smaller or equal
            lo = 0; hi = cnt_a;
            while (lo < hi) { const uint32_t mid = (lo + hi) / 2; if (sk[mid] <= k[q]) lo = mid + 1; else hi = mid; }
            r[q] = (x - cnt_a) + lo;
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kPer; ++q)
        if (r[q] != 0xffffffffu) { sk[r[q]] = k[q]; sv[r[q]] = v[q]; }
    __syncthreads();
    for (uint32_t x = threadIdx.x; x < total; x += kBlock) { ok[diag0 + x] = sk[x]; ov[diag0 + x] = sv[x]; }
}

// key/val consist of the sorted runs [start[r], start[r+1]), r < runs: rounds of pairwise stable merges
rama_status merge_runs(Ctx &ctx, Buf<uint64_t> &key, Buf<uint32_t> &val, size_t n, std::vector<uint32_t> start)
{
    Buf<uint64_t> key2;
    Buf<uint32_t> val2, split;
    RAMA_TRY(key2.alloc(ctx, n));
    RAMA_TRY(val2.alloc(ctx, n));
    RAMA_TRY(split.alloc(ctx, n / kMergeTile + 2));
    while (start.size() > 2) {
        std::vector<uint32_t> next;
        for (size_t r = 0; r + 1 < start.size(); r += 2) {
            const uint32_t s0 = start[r], s1 = start[r + 1];
            next.push_back(s0);
            if (r + 2 >= start.size()) {   // a run without a partner moves over as it is
                HIP_TRY(ctx, hipMemcpyAsync(key2.get() + s0, key.get() + s0, (size_t)(s1 - s0) * 8, hipMemcpyDeviceToDevice, ctx.stream));
                HIP_TRY(ctx, hipMemcpyAsync(val2.get() + s0, val.get() + s0, (size_t)(s1 - s0) * 4, hipMemcpyDeviceToDevice, ctx.stream));
                continue;
            }
            const uint32_t s2 = start[r + 2], na = s1 - s0, nb = s2 - s1;
            const uint32_t ntiles = (na + nb + kMergeTile - 1) / kMergeTile;
            {
                ProfScope ps_(ctx, "k_merge_partition", (double)ntiles * 4);
                k_merge_partition<<<grid_for((size_t)ntiles + 1), kBlock, 0, ctx.stream>>>(key.get() + s0, na, key.get() + s1, nb, ntiles,
                                                                                      split.get());
            }
            LAUNCH_TRY(ctx, "merge_partition");
            {
                ProfScope ps_(ctx, "k_merge_pairs", (double)(na + nb) * 24);
                k_merge_pairs<<<ntiles, kBlock, 0, ctx.stream>>>(key.get() + s0, val.get() + s0, na, key.get() + s1, val.get() + s1, nb,
                                                               split.get(), key2.get() + s0, val2.get() + s0);
            }
            LAUNCH_TRY(ctx, "merge_pairs");
        }
        next.push_back(start.back());
        start.swap(next);
        key.swap(key2);
        val.swap(val2);
    }
    return RAMA_OK;
}

}  // namespace

rama_status canonicalise(Ctx &ctx, int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c, Graph &out)
{
    if (n < 0 || m < 0 || (m > 0 && (!i || !j || !c))) return fail(ctx, RAMA_ERR_INVALID_ARG, "canonicalise: bad arguments");
    if (m >= (int64_t(1) << 31) - 1) return fail(ctx, RAMA_ERR_CAPACITY, "edge count reaches 2^31");
    out.n = n;
    out.m = 0;
    RAMA_TRY(zero_page_recycle(ctx));
    if (m == 0) {
        RAMA_TRY(out.i.alloc(ctx, 1));
        RAMA_TRY(out.j.alloc(ctx, 1));
        RAMA_TRY(out.c.alloc(ctx, 1));
        return RAMA_OK;
    }
    Buf<int32_t> flags;
    RAMA_TRY(zeroed<int32_t>(ctx, 4, flags));
    ScanPlan<uint32_t> keep;
    RAMA_TRY((scan_plan_alloc<uint32_t>(ctx, (size_t)m, 0, keep)));
    {
        ProfScope ps_(ctx, "k_validate", (double)((size_t)m * 12));
        k_validate<<<keep.nb, kBlock, 0, ctx.stream>>>(n, (size_t)m, i, j, c, flags.get(), keep.sums.get());
    }
    LAUNCH_TRY(ctx, "validate");
    int32_t hf[4];
    RAMA_TRY(read_back(ctx, hf, flags.get(), sizeof hf));
    if (hf[0]) return fail(ctx, RAMA_ERR_BAD_GRAPH, "edge endpoint outside [0,n_nodes) or non-finite cost");
    if (!hf[1]) {  // already canonical: plain copy
        RAMA_TRY(out.i.alloc(ctx, m));
        RAMA_TRY(out.j.alloc(ctx, m));
        RAMA_TRY(out.c.alloc(ctx, m));
        HIP_TRY(ctx, hipMemcpyAsync(out.i.get(), i, (size_t)m * 4, hipMemcpyDeviceToDevice, ctx.stream));
        HIP_TRY(ctx, hipMemcpyAsync(out.j.get(), j, (size_t)m * 4, hipMemcpyDeviceToDevice, ctx.stream));
        HIP_TRY(ctx, hipMemcpyAsync(out.c.get(), c, (size_t)m * 4, hipMemcpyDeviceToDevice, ctx.stream));
        out.m = m;
        return RAMA_OK;
    }
    const int nbits = bits_for((uint64_t)n), dbits = bits_for((uint64_t)hf[2] + 1);
    RAMA_TRY((scan_totals<uint32_t>(ctx, NotLoop{i, j}, keep, keep.sums.get())));   // tile sums: left by k_validate
    const uint32_t kept = keep.total;
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
    RAMA_TRY((scan_emit<uint32_t>(ctx, NotLoop{i, j}, PackEdgesEmit{i, j, c, dbits, key.get(), val.get()}, keep,
                                  (double)((size_t)m * 4 + (size_t)kept * 12))));
    keep.offs.reset();
    Buf<uint32_t> head_sums;   // heads per scan tile, if the sort's last kernel could count them
    bool merged = false;
    if ((uint32_t)hf[3] < (uint32_t)kMaxRuns && kept > (uint32_t)LocalSort<uint64_t>::cap) {
        // few places where the order breaks: the packed list is a handful of sorted runs (dropping self-loops cannot
        // add any): find their starts and merge them, one pass per doubling, instead of sorting by all key bits
        Buf<uint32_t> desc;
        RAMA_TRY(zeroed<uint32_t>(ctx, kMaxRuns, desc));
        {
            ProfScope ps_(ctx, "k_find_descents", (double)kept * 8);
            k_find_descents<<<grid_for(kept), kBlock, 0, ctx.stream>>>(key.get(), kept, desc.get());
        }
        LAUNCH_TRY(ctx, "find_descents");
        uint32_t hd[kMaxRuns];
        RAMA_TRY(read_back(ctx, hd, desc.get(), sizeof hd));
        if (hd[0] < (uint32_t)kMaxRuns) {
            std::vector<uint32_t> start(hd + 1, hd + 1 + hd[0]);
            start.push_back(0u);
            start.push_back(kept);
            std::sort(start.begin(), start.end());
            RAMA_TRY(merge_runs(ctx, key, val, kept, start));
            merged = true;
        }
    }
    if (!merged)
        RAMA_TRY((radix_sort_pairs<uint64_t, uint32_t>(ctx, key, val, kept, nbits + dbits, false, &head_sums, (uint64_t)n << dbits)));
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

namespace {
struct NegPart {
    static constexpr int bytes = 4;   // bytes read per item
    static constexpr const char *tag = "NegPart";
    const float *c;
    __device__ __forceinline__ double operator()(size_t e) const { float w = c[e]; return w < 0.0f ? (double)w : 0.0; }
};
}  // namespace

rama_status negative_cost_sum(Ctx &ctx, const float *c, int64_t m, double *out)
{
    Buf<double> d;
    RAMA_TRY(d.alloc(ctx, 1));
    RAMA_TRY(device_sum(ctx, NegPart{c}, (size_t)m, d.get(), false));
    return read_back(ctx, out, d.get(), 8);
}

}  // namespace rama
