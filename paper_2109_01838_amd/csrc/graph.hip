// Step a0: problem statement -> canonical device graph (paper Sec. 3: graph and cost vector;
// Lemma 1(b): parallel edges carry the sum of their costs).
#include "prim.h"

namespace rama {

namespace {

// flags[0]: endpoint out of range or non-finite cost; flags[1]: list is not canonical;
// flags[2]: largest |i-j| of a valid edge.  A workgroup takes one tile of the scan over NotLoop (kScanTile
// edges) and leaves the number of edges that are no self-loops in tile_sums, so that scan needs no counting pass.
__global__ __launch_bounds__(kBlock) void k_validate(int32_t n, size_t m, const int32_t *i, const int32_t *j,
                                                     const float *c, int32_t *flags, uint32_t *tile_sums)
{
    const size_t base = (size_t)blockIdx.x * kScanTile + threadIdx.x;
    uint32_t diff = 0, kept = 0;
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
            if (canon && e > 0) {
                int32_t pa = i[e - 1], pb = j[e - 1];
                canon = pa < a || (pa == a && pb < b);
            }
            if (!canon) flags[1] = 1;
        }
    }
    kept = block_sum(kept);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = kept;
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
    RAMA_TRY(zeroed<int32_t>(ctx, 3, flags));
    ScanPlan<uint32_t> keep;
    RAMA_TRY((scan_plan_alloc<uint32_t>(ctx, (size_t)m, 0, keep)));
    {
        ProfScope ps_(ctx, "k_validate", (double)((size_t)m * 12));
        k_validate<<<keep.nb, kBlock, 0, ctx.stream>>>(n, (size_t)m, i, j, c, flags.get(), keep.sums.get());
    }
    LAUNCH_TRY(ctx, "validate");
    int32_t hf[3];
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
