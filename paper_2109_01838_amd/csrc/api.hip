// C ABI: argument checks, the four entry points, and the primal-dual loop
// (paper algorithm "Primal-Dual Multicut").  Host code here only sequences the stage kernels.
#include <chrono>

#include <vector>

#include "prim.h"

using namespace rama;

// Workspace of rama_solve_static: device memory that exists from the moment the library is loaded, so
// that the call never has to ask anybody for memory.  In host code the array's name is only a handle;
// its device address is looked up once per device (rama_create) and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[RAMA_STATIC_SCRATCH_BYTES];
namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
}  // namespace

namespace {

double now_ms()
{
    using clk = std::chrono::steady_clock;
    return std::chrono::duration<double, std::milli>(clk::now().time_since_epoch()).count();
}

rama_status finish(Ctx &ctx, rama_status st)
{
    hipError_t e = sync_stream(ctx);
    if (st == RAMA_OK && e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, RAMA_ERR_HIP, std::string("stream synchronize: ") + hipGetErrorString(e));
    }
    return st;
}

rama_status copy_out(Ctx &ctx, void *dst, const void *src, size_t bytes)
{
    if (bytes == 0) return RAMA_OK;
    HIP_TRY(ctx, hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, ctx.stream));
    return RAMA_OK;
}

__global__ __launch_bounds__(kBlock) void k_iota32(size_t n, int32_t *p)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < n) p[v] = (int32_t)v;
}

// f <- f' o f  (last line of the loop body of "Primal-Dual Multicut")
__global__ __launch_bounds__(kBlock) void k_compose(size_t n, int32_t *f, const int32_t *fprime)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < n) f[v] = fprime[f[v]];
}

__global__ __launch_bounds__(kBlock) void k_cluster_min(size_t n, const int32_t *f, int32_t *first)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    // nodes ascend with the lanes: a lane whose left neighbour is in the same cluster cannot hold the minimum
    const int32_t mine = v < n ? f[v] : -1;
    const int32_t left = __shfl_up(mine, 1, 64);
    if (v < n && (lane_id() == 0 || left != mine)) atomicMin(&first[mine], (int32_t)v);
}

__global__ __launch_bounds__(kBlock) void k_labels(size_t n, const int32_t *f, const int32_t *first, int32_t *labels)
{
    size_t v = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (v < n) labels[v] = first[f[v]];
}

// objective of eq. 2 on the caller's edge list
struct CutCost {
    static constexpr int bytes = 20;   // bytes read per item
    static constexpr const char *tag = "CutCost";
    const int32_t *i, *j;
    const float *c;
    const int32_t *labels;
    __device__ __forceinline__ double operator()(size_t e) const
    {
        return labels[i[e]] != labels[j[e]] ? (double)c[e] : 0.0;
    }
};

bool bad_graph_args(int32_t n, int64_t m, const void *i, const void *j, const void *c)
{
    return n < 0 || m < 0 || (m > 0 && (!i || !j || !c));
}

// Dual part of a round on graph g (replaced by the augmented graph with reparametrised costs):
// `rounds` times { separate, add triangles to the kept set, k iterations }.  lb: after the last round
// that ran (untouched if none ran: *ran stays false).  trace: optional [rounds+1].
rama_status dual_block(Ctx &ctx, Graph &g, int lmax, bool shortest_only, int k, int rounds, double *lb, bool *ran,
                       double *trace, int64_t *cycles_first, int64_t *n_triangles)
{
    *ran = false;
    if (n_triangles) *n_triangles = 0;
    DualState state;
    double cur = 0.0;
    if (trace) {
        RAMA_TRY(negative_cost_sum(ctx, g.c.get(), g.m, &cur));
        trace[0] = cur;
    }
    int done = 0;
    for (int d = 1; d <= rounds && lmax >= 3; ++d) {
        CycleLists cyc;
        RAMA_TRY(find_cycles(ctx, g, lmax, shortest_only, false, cyc));
        int64_t n_cyc = 0;
        const int32_t *lists[kCycleLists];
        for (int q = 0; q < kCycleLists; ++q) { n_cyc += cyc.n[q]; lists[q] = cyc.v[q].get(); }
        if (d == 1 && cycles_first) for (int q = 0; q < kCycleLists; ++q) cycles_first[q] = cyc.n[q];
        if (n_cyc == 0) break;
        Graph aug;
        DualInfo info;
        DualState next;
        const bool more = d < rounds;   // the last round's triangles are not needed afterwards
        RAMA_TRY(dual_update(ctx, g, kCycleLists, lists, cyc.n, false, k, aug, (lb || trace) ? &cur : nullptr, nullptr, &info,
                             state.T > 0 ? &state : nullptr, more ? &next : nullptr, &g));
        g = std::move(aug);
        state = std::move(next);
        if (n_triangles) *n_triangles = info.n_triangles;
        *ran = true;
        done = d;
        if (trace) trace[d] = cur;
    }
    if (trace) for (int d = done + 1; d <= rounds; ++d) trace[d] = cur;
    if (*ran && lb) *lb = cur;
    return RAMA_OK;
}

// stage clock of the solver: marks on the stream (no synchronisation); read when the stream has drained
struct StageClock {
    Ctx &ctx;
    int used = 0;
    explicit StageClock(Ctx &c) : ctx(c) {}
    // mark `which` (0: round starts, 1: separation done, 2: message passing done, 3: contraction done) of a round
    void mark(int round, int which)
    {
        const int k = 4 * (round - 1) + which;
        if (k >= Ctx::kStageEvents || !ctx.stage_ev[k]) return;
        if (hipEventRecord(ctx.stage_ev[k], ctx.stream) != hipSuccess) { (void)hipGetLastError(); return; }
        if (k + 1 > used) used = k + 1;
    }
    double between(int round, int a, int b) const
    {
        const int ka = 4 * (round - 1) + a, kb = 4 * (round - 1) + b;
        if (kb >= used) return 0.0;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx.stage_ev[ka], ctx.stage_ev[kb]) != hipSuccess) { (void)hipGetLastError(); return 0.0; }
        return (double)ms;
    }
};

rama_status solve_impl(Ctx &ctx, int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c,
                       const rama_params &P, int32_t *labels, double *primal, double *lower_bound, rama_stats *stats)
{
    const double t_begin = now_ms();
    rama_stats S;
    memset(&S, 0, sizeof S);
    ctx.rounds.clear();
    if (n == 0) {   // no nodes: nothing to label (edges would have been rejected as out of range)
        if (m > 0) return fail(ctx, RAMA_ERR_BAD_GRAPH, "edges given for a graph without nodes");
        if (primal) *primal = 0.0;
        if (lower_bound) *lower_bound = 0.0;
        if (stats) *stats = S;
        return RAMA_OK;
    }
    StageClock clock(ctx);
    Graph g;
    RAMA_TRY(canonicalise(ctx, n, m, i, j, c, g));
    // The rounds' node mappings f' are kept and composed at the end, last round first: every
    // composition then runs over the (shrinking) node set of its own round instead of all n nodes.
    std::vector<Buf<int32_t>> maps;
    std::vector<size_t> map_size;
    double lb = 0.0;
    bool have_lb = false;
    int32_t n_cur = n;
    for (int round = 1; P.max_rounds <= 0 || round <= P.max_rounds; ++round) {
        const int lmax = round == 1 ? P.max_cycle_len_first : P.max_cycle_len_later;
        const int k = round == 1 ? P.mp_iters_first : P.mp_iters_later;
        rama_round_stats R;
        memset(&R, 0, sizeof R);
        R.n_nodes = n_cur; R.n_edges = g.m; R.n_attractive = -1; R.n_repulsive = -1;
        ctx.active->reset_peak();
        clock.mark(round, 0);
        bool ran = false;
        double lbr = 0.0;
        int64_t ntri = 0;
        bool dual_marked = false;
        if (lmax >= 3 && k > 0) {
            if (P.dual_rounds == 1) {
                CycleLists cyc;
                RAMA_TRY(find_cycles(ctx, g, lmax, P.shortest_cycles_only != 0, false, cyc));
                clock.mark(round, 1);
                dual_marked = true;
                R.n_attractive = cyc.n_attractive; R.n_repulsive = cyc.n_repulsive;
                int64_t n_cyc = 0;
                const int32_t *lists[kCycleLists];
                for (int q = 0; q < kCycleLists; ++q) { n_cyc += cyc.n[q]; lists[q] = cyc.v[q].get(); R.n_cycles[q] = cyc.n[q]; }
                if (n_cyc > 0) {
                    Graph aug;
                    DualInfo info;
                    RAMA_TRY(dual_update(ctx, g, kCycleLists, lists, cyc.n, false, k, aug, round == 1 ? &lbr : nullptr,
                                         nullptr, &info, nullptr, nullptr, &g));
                    ntri = info.n_triangles;
                    ran = true;
                    g = std::move(aug);
                }
            } else {
                // separations and message-passing blocks interleave: the stage clock books all as cycles
                RAMA_TRY(dual_block(ctx, g, lmax, P.shortest_cycles_only != 0, k, P.dual_rounds, round == 1 ? &lbr : nullptr,
                                    &ran, nullptr, R.n_cycles, &ntri));
            }
        }
        if (!dual_marked) clock.mark(round, 1);
        R.n_triangles = ntri;
        R.n_edges_aug = g.m;
        if (round == 1) {
            for (int q = 0; q < kCycleLists; ++q) S.n_cycles_first[q] = R.n_cycles[q];
            if (ran) { lb = lbr; have_lb = true; S.n_triangles_first = ntri; }
            if (!have_lb) { RAMA_TRY(negative_cost_sum(ctx, g.c.get(), g.m, &lb)); have_lb = true; }
            S.n_edges_aug_first = g.m;
        }
        clock.mark(round, 2);
        Buf<int32_t> fprime;
        Graph gn;
        int32_t n_new = n_cur;
        int64_t ns = 0;
        bool forest = false;
        RAMA_TRY(contract_once(ctx, g, P.contract_threshold, P.matching_rounds_cap, P.forest_ratio, fprime, n_new, gn, ns, &forest));
        S.rounds = round;
        if (ns > 0) {
            maps.push_back(std::move(fprime));
            map_size.push_back((size_t)n_cur);
            g = std::move(gn);
            n_cur = n_new;
        }
        clock.mark(round, 3);
        R.n_contracted = ns;
        R.used_forest = forest ? 1 : 0;
        R.workspace_peak = (int64_t)ctx.active->peak_live();
        ctx.rounds.push_back(R);
        if (ns == 0) break;
    }
    Buf<int32_t> f;    // original node -> final cluster
    for (size_t k = maps.size(); k-- > 1;) {
        ProfScope ps_(ctx, "k_compose", (double)(map_size[k - 1] * 12));
        k_compose<<<grid_for(map_size[k - 1]), kBlock, 0, ctx.stream>>>(map_size[k - 1], maps[k - 1].get(), maps[k].get());
    }
    LAUNCH_TRY(ctx, "compose");
    if (!maps.empty()) {
        f = std::move(maps[0]);
    } else {
        RAMA_TRY(f.alloc(ctx, (size_t)(n > 0 ? n : 1)));
        ProfScope ps_(ctx, "k_iota32", (double)((size_t)n * 4));
        k_iota32<<<grid_for((size_t)n), kBlock, 0, ctx.stream>>>((size_t)n, f.get());
    }
    LAUNCH_TRY(ctx, "iota");
    maps.clear();
    // labels: smallest original node per cluster; primal cost on the caller's costs
    {
        Buf<int32_t> first;
        RAMA_TRY(first.alloc(ctx, (size_t)(n_cur > 0 ? n_cur : 1)));
        RAMA_TRY(fill<int32_t>(ctx, first.get(), 0x7FFFFFFF, (size_t)n_cur));
        if (n > 0) {
            {
                ProfScope ps_(ctx, "k_cluster_min", (double)((size_t)n * 12));
                k_cluster_min<<<grid_for((size_t)n), kBlock, 0, ctx.stream>>>((size_t)n, f.get(), first.get());
            }
            LAUNCH_TRY(ctx, "cluster_min");
            {
                ProfScope ps_(ctx, "k_labels", (double)((size_t)n * 12));
                k_labels<<<grid_for((size_t)n), kBlock, 0, ctx.stream>>>((size_t)n, f.get(), first.get(), labels);
            }
            LAUNCH_TRY(ctx, "labels");
        }
    }
    if (primal) {
        Buf<double> d;
        RAMA_TRY(d.alloc(ctx, 1));
        RAMA_TRY(device_sum(ctx, CutCost{i, j, c, labels}, (size_t)m, d.get(), false));
        RAMA_TRY(read_back(ctx, primal, d.get(), 8));
    }
    if (lower_bound) *lower_bound = lb;
    RAMA_TRY(finish(ctx, RAMA_OK));
    S.n_clusters = n_cur;
    S.n_edges_final = g.m;
    S.ms_total = now_ms() - t_begin;
    for (size_t r = 0; r < ctx.rounds.size(); ++r) {
        rama_round_stats &R = ctx.rounds[r];
        R.ms_cycles = clock.between((int)r + 1, 0, 1);
        R.ms_dual = clock.between((int)r + 1, 1, 2);
        R.ms_contract = clock.between((int)r + 1, 2, 3);
        S.ms_cycles += R.ms_cycles; S.ms_dual += R.ms_dual; S.ms_contract += R.ms_contract;
    }
    S.ms_other = S.ms_total - S.ms_cycles - S.ms_dual - S.ms_contract;
    if (stats) *stats = S;
    return RAMA_OK;
}

}  // namespace

extern "C" {

rama_status rama_create(rama_ctx **out, void *hip_stream, const rama_alloc *alloc)
{
    if (!out) return RAMA_ERR_INVALID_ARG;
    *out = nullptr;
    if (alloc && !alloc->alloc) return RAMA_ERR_INVALID_ARG;
    rama_ctx *ctx = new (std::nothrow) rama_ctx();
    if (!ctx) return RAMA_ERR_OOM;
    ctx->stream = (hipStream_t)hip_stream;
    if (alloc) ctx->pool.set_source(alloc->alloc, alloc->free, alloc->user);
    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) e = hipHostMalloc(&ctx->pinned, rama_ctx::kPinnedBytes, hipHostMallocDefault);
    if (e == hipSuccess) memset(ctx->pinned, 0, rama_ctx::kPinnedBytes);
    if (e == hipSuccess) {   // the ticket word of the fused scans: zero at rest
        void *t = nullptr;
        e = ctx->pool.alloc(sizeof(uint32_t), &t);
        if (e == hipSuccess) {
            ctx->ticket = (uint32_t *)t;
            e = hipMemsetAsync(t, 0, sizeof(uint32_t), ctx->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        }
    }
    if (e == hipSuccess) {   // the page of zeroed words
        void *z = nullptr;
        e = ctx->pool.alloc(rama_ctx::kZeroPageWords * sizeof(uint32_t), &z);
        if (e == hipSuccess) {
            ctx->zero_page = (uint32_t *)z;
            e = hipMemsetAsync(z, 0, rama_ctx::kZeroPageWords * sizeof(uint32_t), ctx->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        }
    }
    for (int k = 0; k < rama_ctx::kStageEvents && e == hipSuccess; ++k) e = hipEventCreate(&ctx->stage_ev[k]);
    if (e == hipSuccess && ctx->device >= 0 && ctx->device < kMaxDevices) {
        // every GPU holds its own copy of the static scratch array at its own address
        if (!g_scratch_ptr[ctx->device]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e == hipSuccess) g_scratch_ptr[ctx->device] = p;
        }
        if (e == hipSuccess) ctx->arena.set_arena(g_scratch_ptr[ctx->device], RAMA_STATIC_SCRATCH_BYTES);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        fprintf(stderr, "rama_create: %s\n", hipGetErrorString(e));
        rama_destroy(ctx);
        return RAMA_ERR_HIP;
    }
    *out = ctx;
    return RAMA_OK;
}

rama_status rama_destroy(rama_ctx *ctx)
{
    if (!ctx) return RAMA_OK;
    (void)hipStreamSynchronize(ctx->stream);
    ctx->prof.destroy();
    ctx->pool.destroy();
    for (hipEvent_t ev : ctx->stage_ev)
        if (ev) (void)hipEventDestroy(ev);
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    delete ctx;
    return RAMA_OK;
}

const char *rama_last_error(const rama_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

void rama_params_default(rama_params *p)
{
    if (!p) return;
    p->max_cycle_len_first = 5;
    p->max_cycle_len_later = 3;
    p->mp_iters_first = 10;
    p->mp_iters_later = 5;
    p->matching_rounds_cap = 32;
    p->contract_threshold = 0.0f;
    p->forest_ratio = 0.1f;
    p->max_rounds = 0;
    p->shortest_cycles_only = 0;
    p->dual_rounds = 1;
}

int64_t rama_workspace_bytes(const rama_ctx *ctx) { return ctx ? (int64_t)ctx->pool.total() : 0; }

int32_t rama_round_count(const rama_ctx *ctx) { return ctx ? (int32_t)ctx->rounds.size() : 0; }

rama_status rama_round_get(const rama_ctx *ctx, int32_t index, rama_round_stats *out)
{
    if (!ctx || !out || index < 0 || index >= (int32_t)ctx->rounds.size()) return RAMA_ERR_INVALID_ARG;
    *out = ctx->rounds[(size_t)index];
    return RAMA_OK;
}

rama_status rama_profile_enable(rama_ctx *ctx, int32_t on, const char *only)
{
    if (!ctx) return RAMA_ERR_INVALID_ARG;
    ctx->prof.only = only ? only : "";
    (void)hipStreamSynchronize(ctx->stream);
    ctx->prof.collect();
    if (on) ctx->prof.reset();
    ctx->prof.on = on != 0;
    return RAMA_OK;
}

rama_status rama_set_sort_split(rama_ctx *ctx, int64_t n_min, int32_t min_passes_replaced)
{
    if (!ctx || n_min < 0 || min_passes_replaced < 0) return RAMA_ERR_INVALID_ARG;
    ctx->sort_split_min = (size_t)n_min;
    ctx->sort_split_gain = min_passes_replaced;
    return RAMA_OK;
}

rama_status rama_set_cycle_search(rama_ctx *ctx, int32_t mode)
{
    if (!ctx || mode < 0 || mode > 3) return RAMA_ERR_INVALID_ARG;
    ctx->cycle_search = mode;
    return RAMA_OK;
}

int32_t rama_profile_count(const rama_ctx *ctx) { return ctx ? (int32_t)ctx->prof.stats.size() : 0; }

rama_status rama_profile_get(const rama_ctx *ctx, int32_t index, const char **name, int64_t *launches, double *ms,
                             double *bytes)
{
    if (!ctx || index < 0 || index >= (int32_t)ctx->prof.stats.size()) return RAMA_ERR_INVALID_ARG;
    const KernelStat &k = ctx->prof.stats[index];
    if (name) *name = k.name;
    if (launches) *launches = (int64_t)k.launches;
    if (ms) *ms = k.ms;
    if (bytes) *bytes = k.bytes;
    return RAMA_OK;
}

rama_status rama_find_conflicted_cycles(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges, const int32_t *i,
                                        const int32_t *j, const float *c, int32_t max_cycle_len, int32_t shortest_only,
                                        const int64_t *cap, int32_t *const *cycles, int64_t *n_cycles_out)
{
    if (!ctx) return RAMA_ERR_INVALID_ARG;
    if (bad_graph_args(n_nodes, n_edges, i, j, c) || !n_cycles_out || max_cycle_len < 3 || max_cycle_len > kMaxCycleLen)
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_find_conflicted_cycles: bad arguments");
    const int lists = max_cycle_len - 2;
    for (int q = 0; q < lists; ++q) {
        const int64_t cq = cap ? cap[q] : 0;
        if (cq < 0 || (cq > 0 && (!cycles || !cycles[q])))
            return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_find_conflicted_cycles: bad capacities or null list");
    }
    auto body = [&]() -> rama_status {
        Graph g;
        RAMA_TRY(canonicalise(*ctx, n_nodes, n_edges, i, j, c, g));
        CycleLists cnt;
        RAMA_TRY(find_cycles(*ctx, g, max_cycle_len, shortest_only != 0, true, cnt));
        bool fits = true;
        int64_t total = 0;
        for (int q = 0; q < lists; ++q) {
            n_cycles_out[q] = cnt.n[q];
            total += cnt.n[q];
            if (cnt.n[q] > (cap ? cap[q] : 0)) fits = false;
        }
        if (!fits)
            return fail(*ctx, RAMA_ERR_CAPACITY, "cycle output lists are too small; needed sizes written to n_cycles_out");
        if (total == 0) return RAMA_OK;
        CycleLists cyc;
        RAMA_TRY(find_cycles(*ctx, g, max_cycle_len, shortest_only != 0, false, cyc));
        for (int q = 0; q < lists; ++q)
            if (cyc.n[q] > 0) RAMA_TRY(copy_out(*ctx, cycles[q], cyc.v[q].get(), (size_t)cyc.n[q] * (q + 3) * 4));
        return finish(*ctx, RAMA_OK);
    };
    return finish(*ctx, body());
}

rama_status rama_message_passing(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges, const int32_t *i, const int32_t *j,
                                 const float *c, int32_t max_cycle_len, const int32_t *const *cycles,
                                 const int64_t *n_cycles, int32_t k_iters, int64_t edge_cap,
                                 int32_t *i_out, int32_t *j_out, float *c_out, int64_t *n_edges_out,
                                 double *lower_bound, double *lb_trace)
{
    if (!ctx) return RAMA_ERR_INVALID_ARG;
    if (bad_graph_args(n_nodes, n_edges, i, j, c) || !n_edges_out || k_iters < 0 || edge_cap < 0 ||
        max_cycle_len < 2 || max_cycle_len > kMaxCycleLen || (max_cycle_len > 2 && (!cycles || !n_cycles)) ||
        (edge_cap > 0 && (!i_out || !j_out || !c_out)))
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_message_passing: bad arguments");
    auto body = [&]() -> rama_status {
        Graph g, out;
        RAMA_TRY(canonicalise(*ctx, n_nodes, n_edges, i, j, c, g));
        RAMA_TRY(dual_update(*ctx, g, max_cycle_len - 2, cycles, n_cycles, true, k_iters, out, lower_bound, lb_trace,
                             nullptr, nullptr, nullptr, &g));
        *n_edges_out = out.m;
        if (out.m > edge_cap)
            return fail(*ctx, RAMA_ERR_CAPACITY, "edge output buffers are too small; needed size written to n_edges_out");
        RAMA_TRY(copy_out(*ctx, i_out, out.i.get(), (size_t)out.m * 4));
        RAMA_TRY(copy_out(*ctx, j_out, out.j.get(), (size_t)out.m * 4));
        RAMA_TRY(copy_out(*ctx, c_out, out.c.get(), (size_t)out.m * 4));
        return finish(*ctx, RAMA_OK);
    };
    return finish(*ctx, body());
}

rama_status rama_contract(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges, const int32_t *i, const int32_t *j,
                          const float *c, const rama_params *params, int32_t repeat, int32_t *mapping, int32_t *i_out,
                          int32_t *j_out, float *c_out, float *diag_out, int32_t *n_nodes_out, int64_t *n_edges_out)
{
    if (!ctx) return RAMA_ERR_INVALID_ARG;
    if (bad_graph_args(n_nodes, n_edges, i, j, c) || !params || !n_nodes_out || !n_edges_out ||
        (n_nodes > 0 && !mapping) || (n_edges > 0 && (!i_out || !j_out || !c_out)))
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_contract: bad arguments");
    auto body = [&]() -> rama_status {
        if (n_nodes == 0) {
            if (n_edges > 0) return fail(*ctx, RAMA_ERR_BAD_GRAPH, "edges given for a graph without nodes");
            *n_nodes_out = 0;
            *n_edges_out = 0;
            return RAMA_OK;
        }
        Graph g0, g;
        RAMA_TRY(canonicalise(*ctx, n_nodes, n_edges, i, j, c, g0));
        {
            ProfScope ps_(*ctx, "k_iota32", (double)((size_t)n_nodes * 4));
            k_iota32<<<grid_for((size_t)n_nodes), kBlock, 0, ctx->stream>>>((size_t)n_nodes, mapping);
        }
        LAUNCH_TRY(*ctx, "iota");
        const Graph *cur = &g0;
        int32_t n_cur = n_nodes;
        for (;;) {
            Buf<int32_t> fprime;
            Graph gn;
            int32_t n_new = n_cur;
            int64_t ns = 0;
            RAMA_TRY(contract_once(*ctx, *cur, params->contract_threshold, params->matching_rounds_cap, params->forest_ratio, fprime,
                                   n_new, gn, ns));
            if (ns == 0) break;
            {
                ProfScope ps_(*ctx, "k_compose", (double)((size_t)n_nodes * 12));
                k_compose<<<grid_for((size_t)n_nodes), kBlock, 0, ctx->stream>>>((size_t)n_nodes, mapping, fprime.get());
            }
            LAUNCH_TRY(*ctx, "compose");
            g = std::move(gn);
            cur = &g;
            n_cur = n_new;
            if (repeat) break;
        }
        *n_nodes_out = n_cur;
        *n_edges_out = cur->m;
        RAMA_TRY(copy_out(*ctx, i_out, cur->i.get(), (size_t)cur->m * 4));
        RAMA_TRY(copy_out(*ctx, j_out, cur->j.get(), (size_t)cur->m * 4));
        RAMA_TRY(copy_out(*ctx, c_out, cur->c.get(), (size_t)cur->m * 4));
        if (diag_out) RAMA_TRY(contraction_diagonal(*ctx, g0, mapping, n_cur, diag_out));
        return finish(*ctx, RAMA_OK);
    };
    return finish(*ctx, body());
}

rama_status rama_dual_rounds(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges, const int32_t *i, const int32_t *j,
                             const float *c, const rama_params *params, int64_t edge_cap, int32_t *i_out,
                             int32_t *j_out, float *c_out, int64_t *n_edges_out, double *lower_bound, double *lb_trace,
                             int64_t *n_triangles_out)
{
    if (!ctx) return RAMA_ERR_INVALID_ARG;
    if (bad_graph_args(n_nodes, n_edges, i, j, c) || !params || !n_edges_out || edge_cap < 0 ||
        (edge_cap > 0 && (!i_out || !j_out || !c_out)) || params->dual_rounds < 0 || params->mp_iters_first < 0 ||
        params->max_cycle_len_first > RAMA_MAX_CYCLE_LEN)
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_dual_rounds: bad arguments");
    auto body = [&]() -> rama_status {
        Graph g;
        RAMA_TRY(canonicalise(*ctx, n_nodes, n_edges, i, j, c, g));
        std::vector<double> trace((size_t)params->dual_rounds + 1, 0.0);
        double lb = 0.0;
        bool ran = false;
        int64_t ntri = 0;
        RAMA_TRY(dual_block(*ctx, g, params->max_cycle_len_first, params->shortest_cycles_only != 0, params->mp_iters_first,
                            params->dual_rounds, &lb, &ran, trace.data(), nullptr, &ntri));
        if (lower_bound) *lower_bound = trace[(size_t)params->dual_rounds];
        if (lb_trace) for (size_t d = 0; d < trace.size(); ++d) lb_trace[d] = trace[d];
        if (n_triangles_out) *n_triangles_out = ntri;
        *n_edges_out = g.m;
        if (g.m > edge_cap)
            return fail(*ctx, RAMA_ERR_CAPACITY, "edge output buffers are too small; needed size written to n_edges_out");
        RAMA_TRY(copy_out(*ctx, i_out, g.i.get(), (size_t)g.m * 4));
        RAMA_TRY(copy_out(*ctx, j_out, g.j.get(), (size_t)g.m * 4));
        RAMA_TRY(copy_out(*ctx, c_out, g.c.get(), (size_t)g.m * 4));
        return finish(*ctx, RAMA_OK);
    };
    return finish(*ctx, body());
}

rama_status rama_solve(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges, const int32_t *i, const int32_t *j,
                       const float *c, const rama_params *params, int32_t *labels, double *primal_cost,
                       double *lower_bound, rama_stats *stats)
{
    if (!ctx) return RAMA_ERR_INVALID_ARG;
    if (bad_graph_args(n_nodes, n_edges, i, j, c) || !params || (n_nodes > 0 && !labels))
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_solve: bad arguments");
    if (params->max_cycle_len_first > RAMA_MAX_CYCLE_LEN || params->max_cycle_len_later > RAMA_MAX_CYCLE_LEN)
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_solve: cycle length beyond RAMA_MAX_CYCLE_LEN");
    if (params->dual_rounds < 1) return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_solve: dual_rounds must be at least 1");
    return finish(*ctx, solve_impl(*ctx, n_nodes, n_edges, i, j, c, *params, labels, primal_cost, lower_bound, stats));
}

rama_status rama_solve_static(rama_ctx *ctx, int32_t n_nodes, int64_t n_edges, const int32_t *i, const int32_t *j,
                              const float *c, const rama_params *params, int32_t *labels, double *primal_cost,
                              double *lower_bound, rama_stats *stats)
{
    if (!ctx) return RAMA_ERR_INVALID_ARG;
    if (bad_graph_args(n_nodes, n_edges, i, j, c) || !params || (n_nodes > 0 && !labels))
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_solve_static: bad arguments");
    if (params->max_cycle_len_first > RAMA_MAX_CYCLE_LEN || params->max_cycle_len_later > RAMA_MAX_CYCLE_LEN)
        return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_solve_static: cycle length beyond RAMA_MAX_CYCLE_LEN");
    if (params->dual_rounds < 1) return fail(*ctx, RAMA_ERR_INVALID_ARG, "rama_solve_static: dual_rounds must be at least 1");
    if (n_nodes > RAMA_STATIC_MAX_NODES || n_edges > RAMA_STATIC_MAX_EDGES)
        return fail(*ctx, RAMA_ERR_CAPACITY,
                    "rama_solve_static: at most " + std::to_string(RAMA_STATIC_MAX_NODES) + " nodes and " +
                        std::to_string(RAMA_STATIC_MAX_EDGES) + " edges (got " + std::to_string(n_nodes) + " and " +
                        std::to_string(n_edges) + "); use rama_solve");
    if (!ctx->arena.is_arena()) return fail(*ctx, RAMA_ERR_HIP, "rama_solve_static: no static scratch on this device");
    // every Buf of the solve now comes out of the static array; the per-kernel timers (they create events) stay off
    const bool prof_was_on = ctx->prof.on;
    ctx->prof.on = false;
    ctx->arena.arena_reset();
    ctx->active = &ctx->arena;
    rama_status st = finish(*ctx, solve_impl(*ctx, n_nodes, n_edges, i, j, c, *params, labels, primal_cost, lower_bound, stats));
    ctx->active = &ctx->pool;
    ctx->arena.arena_reset();
    ctx->prof.on = prof_was_on;
    return st;
}

}  // extern "C"
