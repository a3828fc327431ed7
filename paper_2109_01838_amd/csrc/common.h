// Shared host-side plumbing of the library: context, cached device workspace, status handling.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <chrono>
#include <cstdio>
#include <cstring>
#include <string>
#include <utility>
#include <vector>

#include "../../include/rama.h"

namespace rama {

constexpr int kBlock = 256;  // threads per workgroup everywhere: four wave64

// Device memory cache.  All work of one ctx is enqueued on one stream, so a block released by
// an earlier step can be handed to a later step without synchronisation.
// Blocks come from one of three sources: the caller's allocator callbacks (rama_alloc), hipMalloc,
// or -- in arena mode -- a fixed piece of device memory that is carved up and never grows.
class Pool {
public:
    // where fresh blocks come from when no cached one fits; both null: hipMalloc / hipFree
    void set_source(void *(*alloc_fn)(void *, size_t), void (*free_fn)(void *, void *), void *user)
    {
        alloc_fn_ = alloc_fn; free_fn_ = free_fn; user_ = user;
    }
    // arena mode: every block is a piece of [base, base+bytes); nothing is ever requested from a driver
    void set_arena(void *base, size_t bytes)
    {
        arena_ = (char *)base; arena_bytes_ = bytes;
        arena_reset();
    }
    bool is_arena() const { return arena_ != nullptr; }
    void arena_reset()
    {
        holes_.clear(); used_.clear();
        if (arena_bytes_ > 0) holes_.push_back({arena_, arena_bytes_});
        live_ = 0; peak_live_ = 0;
    }
    hipError_t alloc(size_t bytes, void **out)
    {
        // every block ends with at least 32 readable bytes of slack: kernels fetch short index rows
        // with 16-byte loads and may read (never use) up to 28 bytes behind the last element
        bytes = (bytes + 32 + 255) & ~size_t(255);
        if (arena_) return arena_alloc(bytes, out);
        int best = -1;
        for (int k = 0; k < (int)free_.size(); ++k)
            if (free_[k].bytes >= bytes && (best < 0 || free_[k].bytes < free_[best].bytes)) best = k;
        if (best >= 0 && free_[best].bytes <= 2 * bytes + (size_t(1) << 20)) {
            *out = free_[best].ptr;
            used_.push_back(free_[best]);
            went_live(free_[best].bytes);
            free_.erase(free_.begin() + best);
            return hipSuccess;
        }
        void *p = nullptr;
        hipError_t e = fresh(&p, bytes);
        if (e != hipSuccess) {  // give cached blocks back to their source and retry once
            trim();
            e = fresh(&p, bytes);
            if (e != hipSuccess) return e;
        }
        total_ += bytes;
        went_live(bytes);
        used_.push_back({p, bytes});
        *out = p;
        return hipSuccess;
    }
    void release(void *p)
    {
        for (int k = (int)used_.size() - 1; k >= 0; --k)
            if (used_[k].ptr == p) {
                live_ -= used_[k].bytes;
                if (arena_) arena_release(used_[k]); else free_.push_back(used_[k]);
                used_.erase(used_.begin() + k);
                return;
            }
    }
    void trim()
    {
        if (arena_) return;
        for (auto &b : free_) { give_back(b.ptr); total_ -= b.bytes; }
        free_.clear();
    }
    void destroy()
    {
        if (arena_) { arena_reset(); return; }
        trim();
        for (auto &b : used_) { give_back(b.ptr); total_ -= b.bytes; }
        used_.clear();
        live_ = 0;
    }
    size_t total() const { return arena_ ? arena_bytes_ : total_; }   // bytes held, cached blocks included
    size_t live() const { return live_; }                             // bytes handed out right now
    size_t peak_live() const { return peak_live_; }                   // largest value of live() since reset_peak()
    void reset_peak() { peak_live_ = live_; }

private:
    struct Blk { void *ptr; size_t bytes; };
    void went_live(size_t bytes)
    {
        live_ += bytes;
        if (live_ > peak_live_) peak_live_ = live_;
    }
    hipError_t fresh(void **p, size_t bytes)
    {
        if (alloc_fn_) {
            *p = alloc_fn_(user_, bytes);
            return *p ? hipSuccess : hipErrorOutOfMemory;
        }
        hipError_t e = hipMalloc(p, bytes);
        if (e != hipSuccess) (void)hipGetLastError();
        return e;
    }
    void give_back(void *p)
    {
        if (alloc_fn_) { if (free_fn_) free_fn_(user_, p); }
        else (void)hipFree(p);
    }
    // arena: holes_ is sorted by address; first hole that fits is cut from its front
    hipError_t arena_alloc(size_t bytes, void **out)
    {
        for (size_t k = 0; k < holes_.size(); ++k)
            if (holes_[k].bytes >= bytes) {
                *out = holes_[k].ptr;
                used_.push_back({holes_[k].ptr, bytes});
                if (holes_[k].bytes == bytes) holes_.erase(holes_.begin() + (long)k);
                else { holes_[k].ptr = (char *)holes_[k].ptr + bytes; holes_[k].bytes -= bytes; }
                went_live(bytes);
                return hipSuccess;
            }
        return hipErrorOutOfMemory;
    }
    void arena_release(const Blk &b)
    {
        size_t k = 0;
        while (k < holes_.size() && holes_[k].ptr < b.ptr) ++k;
        holes_.insert(holes_.begin() + (long)k, b);
        if (k + 1 < holes_.size() && (char *)holes_[k].ptr + holes_[k].bytes == holes_[k + 1].ptr) {
            holes_[k].bytes += holes_[k + 1].bytes;
            holes_.erase(holes_.begin() + (long)k + 1);
        }
        if (k > 0 && (char *)holes_[k - 1].ptr + holes_[k - 1].bytes == holes_[k].ptr) {
            holes_[k - 1].bytes += holes_[k].bytes;
            holes_.erase(holes_.begin() + (long)k);
        }
    }
    std::vector<Blk> free_, used_, holes_;
    size_t total_ = 0, live_ = 0, peak_live_ = 0;
    void *(*alloc_fn_)(void *, size_t) = nullptr;
    void (*free_fn_)(void *, void *) = nullptr;
    void *user_ = nullptr;
    char *arena_ = nullptr;
    size_t arena_bytes_ = 0;
};

// Per-kernel timers: when switched on, every instrumented launch is bracketed by two HIP events
// on the ctx stream; elapsed times are collected at the next stream synchronisation.
struct KernelStat {
    const char *name;
    uint64_t launches;
    double ms;
    double bytes;  // algorithmic bytes, summed over launches
};
class Profiler {
public:
    bool on = false;
    std::string only;   // when non-empty: '|'-separated prefixes; only kernels whose name starts with one of them are timed
    std::vector<KernelStat> stats;
    bool wants(const char *name) const
    {
        if (!on) return false;
        if (only.empty()) return true;
        size_t a = 0;
        while (a <= only.size()) {
            size_t b = only.find('|', a);
            if (b == std::string::npos) b = only.size();
            if (b > a && strncmp(name, only.c_str() + a, b - a) == 0) return true;
            a = b + 1;
        }
        return false;
    }
    void begin(hipStream_t s, const char *name, double bytes)
    {
        Pending p{id_of(name), get_event(), get_event(), bytes};
        (void)hipEventRecord(p.a, s);
        pending_.push_back(p);
    }
    void end(hipStream_t s) { (void)hipEventRecord(pending_.back().b, s); }
    // for a launch that stamps its own start and stop events (hipExtLaunchKernelGGL): the times then come
    // from the dispatch itself, nothing extra is put into the queue
    void begin_stamped(const char *name, double bytes, hipEvent_t *a, hipEvent_t *b)
    {
        Pending p{id_of(name), get_event(), get_event(), bytes};
        *a = p.a; *b = p.b;
        pending_.push_back(p);
    }
    // call only when the stream has been synchronised
    void collect()
    {
        for (auto &p : pending_) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
                stats[p.id].launches += 1;
                stats[p.id].ms += ms;
                stats[p.id].bytes += p.bytes;
            } else {
                (void)hipGetLastError();
            }
            free_.push_back(p.a);
            free_.push_back(p.b);
        }
        pending_.clear();
    }
    void reset() { stats.clear(); }
    void destroy()
    {
        collect();
        for (auto e : free_) (void)hipEventDestroy(e);
        free_.clear();
    }

private:
    struct Pending { int id; hipEvent_t a, b; double bytes; };
    int id_of(const char *name)
    {
        for (int k = 0; k < (int)stats.size(); ++k)
            if (stats[k].name == name || strcmp(stats[k].name, name) == 0) return k;
        stats.push_back({name, 0, 0.0, 0.0});
        return (int)stats.size() - 1;
    }
    hipEvent_t get_event()
    {
        if (!free_.empty()) { hipEvent_t e = free_.back(); free_.pop_back(); return e; }
        hipEvent_t e = nullptr;
        (void)hipEventCreate(&e);
        return e;
    }
    std::vector<Pending> pending_;
    std::vector<hipEvent_t> free_;
};

}  // namespace rama

struct rama_ctx {
    hipStream_t stream = nullptr;
    int device = 0;
    rama::Pool pool;                 // the ctx's own cache (caller's allocator or hipMalloc)
    rama::Pool arena;                // carves up the static scratch array of this device (rama_solve_static)
    rama::Pool *active = &pool;      // where Buf takes its memory from: `pool`, or `arena` during a call that must not allocate
    rama::Profiler prof;
    std::vector<rama_round_stats> rounds;   // per-round record of the last rama_solve
    static constexpr int kStageEvents = 4 * 64;
    hipEvent_t stage_ev[kStageEvents] = {};  // stage clock of rama_solve: four marks per round, created once
    std::string err;
    void *pinned = nullptr;  // small pinned host block for scalar read-backs
    static constexpr size_t kPinnedBytes = 4096;
    // Scalars the host waits for (counts that size the next launch) travel through a mailbox in pinned host
    // memory: the producing kernel stores the values, fences, and stores the running message number last; the
    // host polls that number for a bounded time instead of going through a stream synchronisation (~9 us
    // instead of ~17 us per round trip measured), and falls back to the synchronisation when the kernels in
    // front of the message take longer.
    static constexpr size_t kMailWords = 64;          // 8-byte words of one message, word 0 is the number
    uint64_t mail_seq = 0;
    uint32_t *ticket = nullptr;  // device word, zero at rest: "last workgroup to finish" election of the fused scans
    // Flags and counters that must start at zero (a dozen per round, a few words each) are handed out from one
    // page of device words that is zero beyond zero_used; it is cleared again -- one launch -- when half of it
    // is used up, at the start of a stage, where no word handed out before is still needed.
    static constexpr size_t kZeroPageWords = size_t(1) << 14;
    uint32_t *zero_page = nullptr;
    size_t zero_used = 0;
    int cycle_search = 0;                      // see rama_set_cycle_search
    size_t sort_split_min = size_t(1) << 21;   // arrays at least this long may take the split sort ...
    int sort_split_gain = 2;                   // ... when it replaces at least this many passes
};

namespace rama {

using Ctx = rama_ctx;

// brackets the launches made during its lifetime with the profiler's events (no-op when off)
struct ProfScope {
    Ctx &ctx;
    bool active;
    ProfScope(Ctx &c, const char *name, double bytes) : ctx(c), active(c.prof.wants(name))
    {
        if (active) ctx.prof.begin(ctx.stream, name, bytes);
    }
    ~ProfScope()
    {
        if (active) ctx.prof.end(ctx.stream);
    }
};

inline hipError_t sync_stream(Ctx &ctx)
{
    hipError_t e = hipStreamSynchronize(ctx.stream);
    if (e == hipSuccess && ctx.prof.on) ctx.prof.collect();
    return e;
}

inline rama_status fail(Ctx &ctx, rama_status st, const std::string &msg)
{
    ctx.err = msg;
    return st;
}

#define RAMA_TRY(expr)                                   \
    do {                                                 \
        rama_status _st = (expr);                        \
        if (_st != RAMA_OK) return _st;                  \
    } while (0)

#define HIP_TRY(ctx, call)                                                                       \
    do {                                                                                         \
        hipError_t _e = (call);                                                                  \
        if (_e != hipSuccess) {                                                                  \
            (void)hipGetLastError();                                                             \
            return ::rama::fail((ctx), _e == hipErrorOutOfMemory ? RAMA_ERR_OOM : RAMA_ERR_HIP,  \
                                std::string(#call) + ": " + hipGetErrorString(_e));              \
        }                                                                                        \
    } while (0)

// launch check: the launch itself can fail (bad configuration); kernel faults surface at the next sync
#define LAUNCH_TRY(ctx, what) HIP_TRY(ctx, hipGetLastError())

// RAII device array from the ctx pool
template <typename T>
class Buf {
public:
    Buf() = default;
    Buf(const Buf &) = delete;
    Buf &operator=(const Buf &) = delete;
    Buf(Buf &&o) noexcept { steal(o); }
    Buf &operator=(Buf &&o) noexcept
    {
        if (this != &o) { reset(); steal(o); }
        return *this;
    }
    ~Buf() { reset(); }
    rama_status alloc(Ctx &ctx, size_t count)
    {
        reset();
        void *p = nullptr;
        hipError_t e = ctx.active->alloc(count * sizeof(T), &p);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, RAMA_ERR_OOM, std::string(ctx.active->is_arena() ? "static scratch exhausted: " : "") +
                                               "device allocation of " + std::to_string(count * sizeof(T)) + " bytes failed");
        }
        ctx_ = ctx.active; ptr_ = (T *)p; count_ = count;
        return RAMA_OK;
    }
    // memory that somebody else owns (the ctx's page of zeroed words): never released
    void borrow(T *p, size_t count)
    {
        reset();
        ptr_ = p; count_ = count;
    }
    void reset()
    {
        if (ptr_ && ctx_) ctx_->release(ptr_);
        ptr_ = nullptr; count_ = 0; ctx_ = nullptr;
    }
    T *get() const { return ptr_; }
    operator T *() const { return ptr_; }
    size_t size() const { return count_; }
    void swap(Buf &o) { std::swap(ctx_, o.ctx_); std::swap(ptr_, o.ptr_); std::swap(count_, o.count_); }

private:
    void steal(Buf &o) { ctx_ = o.ctx_; ptr_ = o.ptr_; count_ = o.count_; o.ptr_ = nullptr; o.count_ = 0; o.ctx_ = nullptr; }
    Pool *ctx_ = nullptr;   // the pool the block came from
    T *ptr_ = nullptr;
    size_t count_ = 0;
};

inline unsigned grid_for(size_t n, int per_block = kBlock) { return (unsigned)((n + per_block - 1) / per_block); }

// number of bits needed to write values in [0, n)
inline int bits_for(uint64_t n)
{
    int b = 1;
    while (b < 64 && (uint64_t(1) << b) < n) ++b;
    return b;
}

// the mailbox as kernels see it (pinned host memory is mapped at the same address on the device)
inline uint64_t *mailbox(Ctx &ctx) { return (uint64_t *)((char *)ctx.pinned + 2048); }

// waits until message `seq` is in the mailbox: bounded polling, then the stream synchronisation.  (The
// per-kernel timers are collected at the synchronisation that ends every call of the library.)
inline rama_status wait_mail(Ctx &ctx, uint64_t seq)
{
    volatile uint64_t *m = mailbox(ctx);
    {
        // polls as long as it takes the kernels in front of the message; the clock is only there to end the
        // wait if the message never comes (a failed launch, a fault): the synchronisation below then reports it
        const auto t0 = std::chrono::steady_clock::now();
        for (;;) {
            for (int spin = 0; spin < 4096; ++spin)
                if (m[0] == seq) return RAMA_OK;
            if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) break;
        }
    }
    HIP_TRY(ctx, sync_stream(ctx));
    if (m[0] != seq) return fail(ctx, RAMA_ERR_HIP, "a kernel did not deliver its message to the host");
    return RAMA_OK;
}

// copy `bytes` from device to host and wait
inline rama_status read_back_sync(Ctx &ctx, void *host, const void *dev, size_t bytes)
{
    if (bytes <= Ctx::kPinnedBytes) {
        HIP_TRY(ctx, hipMemcpyAsync(ctx.pinned, dev, bytes, hipMemcpyDeviceToHost, ctx.stream));
        HIP_TRY(ctx, sync_stream(ctx));
        memcpy(host, ctx.pinned, bytes);
    } else {
        HIP_TRY(ctx, hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, ctx.stream));
        HIP_TRY(ctx, sync_stream(ctx));
    }
    return RAMA_OK;
}

// A canonical graph in device memory: i<j, sorted by (i,j), no duplicates.
struct Graph {
    int32_t n = 0;
    int64_t m = 0;
    Buf<int32_t> i, j;
    Buf<float> c;
    // optional, left by the kernel that wrote c: per tile of 2048 edges the number of positive (low half) and
    // negative (high half) costs; valid only while c is what that kernel wrote
    Buf<uint64_t> sign_sums;
};

constexpr int kMaxCycleLen = RAMA_MAX_CYCLE_LEN;
constexpr int kCycleLists = kMaxCycleLen - 2;   // list k holds the (k+3)-cycles

struct CycleLists {
    int64_t n[kCycleLists] = {};
    Buf<int32_t> v[kCycleLists];  // [L*n[L-3]]
    int64_t n_attractive = 0, n_repulsive = 0;   // sign split of the searched graph
};

// ---- stage entry points on canonical device graphs (defined in the stage files) ----

// a0: any edge list -> canonical graph
rama_status canonicalise(Ctx &ctx, int32_t n, int64_t m, const int32_t *i, const int32_t *j, const float *c, Graph &out);

// a1: conflicted cycles of lengths 3..max_len; shortest_only keeps, per repulsive edge, only the
// cycles of its smallest length.  With count_only the lists stay empty.
rama_status find_cycles(Ctx &ctx, const Graph &g, int max_len, bool shortest_only, bool count_only, CycleLists &out);

// a2+a3: triangulate, k iterations of message passing; `out` = augmented graph with reduced costs
struct DualInfo {
    int64_t n_triangles = 0;
};
// triangles of a graph with their costs c_t, handed from one dual round on a graph to the next
struct DualState {
    size_t T = 0;
    Buf<int32_t> tri_nodes;   // [3T] sorted node triples u<v<w
    Buf<float> ct;            // [3T]
};
// cycles[k] / n_cycles[k]: device list and number of the (k+3)-cycles, k < lists.  The triangles of
// `prev` (optional) stay in the relaxation with their costs; `next` (optional) receives the
// triangle set and costs after the last iteration.
rama_status dual_update(Ctx &ctx, const Graph &g, int lists, const int32_t *const *cycles, const int64_t *n_cycles,
                        bool validate_cycles, int k_iters, Graph &out, double *lower_bound, double *lb_trace,
                        DualInfo *info, const DualState *prev = nullptr, DualState *next = nullptr,
                        Graph *donor = nullptr);

// a4..a6: one primal update.  fmap[n] -> [0,n_new); n_matched = |S|.  If |S|==0 nothing else is produced.
rama_status contract_once(Ctx &ctx, const Graph &g, float tau, int rounds_cap, float forest_ratio, Buf<int32_t> &fmap,
                          int32_t &n_new, Graph &out, int64_t &n_matched, bool *used_forest = nullptr);

// diagonal of K^T A K for a mapping F on canonical graph g: diag[a] = sum of edges with F(i)=F(j)=a
rama_status contraction_diagonal(Ctx &ctx, const Graph &g, const int32_t *fmap, int32_t n_new, float *diag);

// sum of min(0,c) over the edges, in double
rama_status negative_cost_sum(Ctx &ctx, const float *c, int64_t m, double *out);

}  // namespace rama
