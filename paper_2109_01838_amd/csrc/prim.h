// Device-wide primitives for gfx950, written for 64-wide wavefronts:
//   exclusive scan (reduce-then-scan, functor input), stable LSD radix sort (wave-level
//   match-any ranking), row boundaries of a sorted key array, deterministic sum reductions.
// Everything is integer-exact or uses a fixed reduction tree, so results do not depend on
// scheduling.
#pragma once

#include <list>

#include "common.h"
#include <type_traits>

namespace rama {

template <typename T>
rama_status fill(Ctx &ctx, T *p, T v, size_t n);   // defined with the reductions below

// `count` elements that are zero: from the ctx's page of zeroed words when they are few (no launch), else a block
// of their own plus a fill.  Page words are for use inside one stage (see zero_page_recycle).
template <typename T>
rama_status zeroed(Ctx &ctx, size_t count, Buf<T> &b)
{
    const size_t words = (count * sizeof(T) + 15) / 16 * 4;
    if (ctx.zero_page && words <= 1024 && ctx.zero_used + words <= rama_ctx::kZeroPageWords) {
        b.borrow((T *)(ctx.zero_page + ctx.zero_used), count);
        ctx.zero_used += words;
        return RAMA_OK;
    }
    RAMA_TRY(b.alloc(ctx, count > 0 ? count : 1));
    return fill<T>(ctx, b.get(), (T)0, count > 0 ? count : 1);
}
// At the start of a stage (nothing handed out from the page is needed any more): clear the page once half of it is used.
inline rama_status zero_page_recycle(Ctx &ctx)
{
    if (!ctx.zero_page || ctx.zero_used * 2 <= rama_ctx::kZeroPageWords) return RAMA_OK;
    RAMA_TRY(fill<uint32_t>(ctx, ctx.zero_page, 0u, rama_ctx::kZeroPageWords));
    ctx.zero_used = 0;
    return RAMA_OK;
}

// ------------------------------------------------------------------------------------------
// wave / block helpers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & 63); }

// Consecutive workgroups of a launch go to the eight XCDs in turn, each with an L2 of its own.  A kernel whose
// neighbouring workgroups gather from the same stretch of an array then fetches that stretch into all eight L2s.
// Launched with xcd_grid(nb) workgroups and numbering its work by xcd_block(), a kernel gives every XCD one
// contiguous eighth of the work instead; numbers beyond nb - 1 come up for the padding and must leave at once.
// (The assignment of workgroups to XCDs only decides how well this works, not what is computed.)
inline uint32_t xcd_grid(uint32_t nb) { return ((nb + 7u) / 8u) * 8u; }
__device__ __forceinline__ uint32_t xcd_block()
{
    if (gridDim.x & 7u) return blockIdx.x;     // not launched with xcd_grid: plain numbering (every number still comes up once)
    return (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
}

template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v)
{
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        T t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    return v;
}

// 32-bit integers: the same scan on the data-parallel-primitive path of the vector ALU instead of
// the LDS crossbar -- shifts by 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of rows 0 and
// 2 is broadcast into rows 1 and 3, then lane 31 into rows 2 and 3.  Lanes without a source add 0.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
    return v;
}
__device__ __forceinline__ int32_t wave_inclusive_scan(int32_t v) { return (int32_t)wave_inclusive_scan((uint32_t)v); }

// value of lane 63, the same in every lane
template <typename T>
__device__ __forceinline__ T wave_last(T v) { return __shfl(v, 63, 64); }
__device__ __forceinline__ uint32_t wave_last(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, 63); }

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// inclusive scan over the 256 threads of a block; *total gets the block sum
template <typename T>
__device__ __forceinline__ T block_inclusive_scan(T v, T *total)
{
    __shared__ T wave_tot[4];
    const int w = threadIdx.x >> 6;
    T inc = wave_inclusive_scan(v);
    if (lane_id() == 63) wave_tot[w] = inc;
    __syncthreads();
    T pre = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        T x = wave_tot[k];
        if (k < w) pre += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return inc + pre;
}

// sum over the block in a fixed order (lane tree, then waves 0..3)
template <typename T>
__device__ __forceinline__ T block_sum(T v)
{
    __shared__ T wave_tot[4];
    T s = wave_sum(v);
    if (lane_id() == 0) wave_tot[threadIdx.x >> 6] = s;
    __syncthreads();
    T tot = ((wave_tot[0] + wave_tot[1]) + wave_tot[2]) + wave_tot[3];
    __syncthreads();
    return tot;
}

// ------------------------------------------------------------------------------------------
// scalars for the host: the mailbox
// ------------------------------------------------------------------------------------------
// closes message `seq`: everything this workgroup stored into mail[1..] before is visible to the host first
__device__ __forceinline__ void mail_send(uint64_t *mail, uint64_t seq)
{
    __threadfence_system();
    __syncthreads();
    if (threadIdx.x == 0) {
        *(volatile uint64_t *)mail = seq;
        __threadfence_system();
    }
}

// `words` 4-byte words from device memory into the mailbox
static __global__ __launch_bounds__(kBlock) void k_publish(const uint32_t *src, unsigned words, uint64_t *mail, uint64_t seq)
{
    uint32_t *dst = (uint32_t *)(mail + 1);
    for (unsigned k = threadIdx.x; k < words; k += kBlock) dst[k] = src[k];
    mail_send(mail, seq);
}

// copy `bytes` (a multiple of 4, at most what a message holds) from device memory to the host and wait
inline rama_status read_back(Ctx &ctx, void *host, const void *dev, size_t bytes)
{
    if (bytes % 4 != 0 || bytes > (Ctx::kMailWords - 1) * 8) return read_back_sync(ctx, host, dev, bytes);
    const uint64_t seq = ++ctx.mail_seq;
    k_publish<<<1, kBlock, 0, ctx.stream>>>((const uint32_t *)dev, (unsigned)(bytes / 4), mailbox(ctx), seq);
    LAUNCH_TRY(ctx, "publish");
    RAMA_TRY(wait_mail(ctx, seq));
    memcpy(host, (const void *)(mailbox(ctx) + 1), bytes);
    return RAMA_OK;
}

// ------------------------------------------------------------------------------------------
// exclusive scan of f(0..n-1) into out[0..n] (out[n] = total)
// ------------------------------------------------------------------------------------------
// A workgroup owns a tile of 2048 consecutive items, each of its four waves 512 of them, taken
// 64 at a time: lane l of the wave reads item 64*q + l in step q, so every access is one
// contiguous 256-byte (or 512-byte) piece per wave.
constexpr int kScanItems = 8;
constexpr int kScanTile = kBlock * kScanItems;
constexpr int kScanWaveItems = 64 * kScanItems;

template <typename T>
struct PtrInput {
    static constexpr int bytes = (int)sizeof(T);   // bytes read per item
    static constexpr const char *tag = "PtrInput";
    const T *p;
    __device__ __forceinline__ T operator()(size_t k) const { return p[k]; }
};

// "<kernel><<functor tag>>", built once per (kernel, functor) pair
template <typename F>
inline const char *kernel_name(const char *kernel)
{
    static std::list<std::pair<std::string, std::string>> names;   // list: stable addresses
    for (auto &p : names) if (p.first == kernel) return p.second.c_str();
    names.emplace_back(std::string(kernel), std::string(kernel) + "<" + F::tag + ">");
    return names.back().second.c_str();
}

// exclusive scan of up to kScanMidMax tile sums by one workgroup, chunk after chunk; out[nb] = total
constexpr unsigned kScanMidMax = 1u << 13;
constexpr unsigned kScanFusedMax = 256;   // up to this many tiles (2^19 items) the reduce launch scans its own tile sums
template <typename TO, bool COHERENT>
__device__ __forceinline__ TO scan_tile_sums(const TO *in, TO *out, unsigned nb)
{
    TO carry = 0;
    for (unsigned c0 = 0; c0 < nb; c0 += kScanTile) {
        unsigned base = c0 + threadIdx.x * kScanItems;
        TO v[kScanItems];
        TO s = 0;
#pragma unroll
        for (int q = 0; q < kScanItems; ++q) {
            // sums written by other workgroups of the same launch are read past the local cache
            v[q] = (base + q < nb) ? (COHERENT ? __hip_atomic_load(in + base + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                               : in[base + q])
                                   : (TO)0;
            s += v[q];
        }
        TO tot;
        TO run = block_inclusive_scan(s, &tot) - s + carry;
#pragma unroll
        for (int q = 0; q < kScanItems; ++q) {
            if (base + q < nb) out[base + q] = run;
            run += v[q];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) out[nb] = carry;
    return carry;
}

// Tile sums.  With a ticket word the launch also scans them: every workgroup publishes its sum and draws
// a ticket; the one that draws the last ticket sees all sums, scans them into offs[0..nb] (offs[nb] = total),
// puts the ticket word back to zero and -- if a mailbox is given -- sends the total and the caller's
// `extra` words behind it (written by earlier launches) to the host.  One launch instead of two, and the
// total reaches the host without a copy.
template <typename TO, typename F>
__global__ __launch_bounds__(kBlock) void k_scan_reduce(F f, TO *block_sums, size_t n, TO *offs, uint32_t *ticket,
                                                        uint64_t *mail, uint64_t seq, int extra)
{
    const size_t base = (size_t)blockIdx.x * kScanTile + threadIdx.x;
    TO s = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const size_t k = base + (size_t)q * kBlock;
        if (k < n) s += (TO)f(k);
    }
    TO tot = block_sum(s);
    if (!ticket) {
        if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
        return;
    }
    __shared__ bool last;
    if (threadIdx.x == 0) {
        __hip_atomic_store(block_sums + blockIdx.x, tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        last = atomicAdd(ticket, 1u) == gridDim.x - 1;
    }
    __syncthreads();
    if (!last) return;
    __threadfence();
    const TO total = scan_tile_sums<TO, true>(block_sums, offs, gridDim.x);
    if (threadIdx.x == 0) *ticket = 0u;
    if (mail) {
        if (threadIdx.x == 0) {
            mail[1] = (uint64_t)total;
            for (int e = 0; e < extra; ++e) mail[2 + e] = (uint64_t)offs[gridDim.x + 1 + e];
        }
        mail_send(mail, seq);
    }
}

// the scan of the tile sums as a launch of its own (long arrays: the election above would make every
// workgroup of the reduce launch wait for its sum to be visible, which costs more than a launch)
template <typename TO>
__global__ __launch_bounds__(kBlock) void k_scan_mid(const TO *in, TO *out, unsigned nb, uint64_t *mail, uint64_t seq, int extra)
{
    const TO total = scan_tile_sums<TO, false>(in, out, nb);
    if (mail) {
        if (threadIdx.x == 0) {
            mail[1] = (uint64_t)total;
            for (int e = 0; e < extra; ++e) mail[2 + e] = (uint64_t)out[nb + 1 + e];
        }
        mail_send(mail, seq);
    }
}

template <typename TO, typename F>
__global__ __launch_bounds__(kBlock) void k_scan_apply(F f, TO *out, const TO *block_offsets, size_t n)
{
    __shared__ TO wave_tot[4];
    const int w = threadIdx.x >> 6;
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)w * kScanWaveItems + lane_id();
    TO v[kScanItems];
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const size_t k = base + (size_t)q * 64;
        v[q] = (k < n) ? (TO)f(k) : (TO)0;
    }
    TO carry = 0;   // sum of the wave's items before step q
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const TO inc = wave_inclusive_scan(v[q]);
        v[q] = inc - v[q] + carry;
        carry += wave_last(inc);
    }
    if (lane_id() == 0) wave_tot[w] = carry;
    __syncthreads();
    TO pre = block_offsets ? block_offsets[blockIdx.x] : (TO)0;
#pragma unroll
    for (int k = 0; k < 3; ++k)
        if (k < w) pre += wave_tot[k];
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const size_t k = base + (size_t)q * 64;
        if (k < n) out[k] = v[q] + pre;
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kBlock - 1) out[n] = pre + carry;
}

template <typename TO>
__global__ void k_store_zero(TO *p) { *p = 0; }

template <typename TO, typename F>
rama_status exclusive_scan(Ctx &ctx, F f, TO *out, size_t n)
{
    if (n == 0) {
        {
            ProfScope ps_(ctx, "k_store_zero", (double)(0));
            k_store_zero<TO><<<1, 1, 0, ctx.stream>>>(out);
        }
        LAUNCH_TRY(ctx, "scan0");
        return RAMA_OK;
    }
    unsigned nb = grid_for(n, kScanTile);
    if (nb == 1) {
        {
            ProfScope ps_(ctx, kernel_name<F>("k_scan_apply"), (double)(n * (F::bytes + sizeof(TO))));
            k_scan_apply<TO, F><<<1, kBlock, 0, ctx.stream>>>(f, out, (const TO *)nullptr, n);
        }
        LAUNCH_TRY(ctx, "scan1");
        return RAMA_OK;
    }
    Buf<TO> sums, offs;
    RAMA_TRY(sums.alloc(ctx, nb));
    RAMA_TRY(offs.alloc(ctx, (size_t)nb + 1));
    const bool fused = nb <= kScanFusedMax;   // the last workgroup of the reduce launch scans the tile sums
    {
        ProfScope ps_(ctx, kernel_name<F>("k_scan_reduce"), (double)(n * F::bytes));
        k_scan_reduce<TO, F><<<nb, kBlock, 0, ctx.stream>>>(f, sums.get(), n, offs.get(), fused ? ctx.ticket : nullptr,
                                                           (uint64_t *)nullptr, 0, 0);
    }
    LAUNCH_TRY(ctx, "scan_reduce");
    if (!fused && nb <= kScanMidMax) {
        ProfScope ps_(ctx, "k_scan_mid", (double)((size_t)nb * 2 * sizeof(TO)));
        k_scan_mid<TO><<<1, kBlock, 0, ctx.stream>>>(sums.get(), offs.get(), nb, (uint64_t *)nullptr, 0, 0);
        LAUNCH_TRY(ctx, "scan_mid");
    } else if (!fused) {
        RAMA_TRY((exclusive_scan<TO, PtrInput<TO>>(ctx, PtrInput<TO>{sums.get()}, offs.get(), nb)));
    }
    {
        ProfScope ps_(ctx, kernel_name<F>("k_scan_apply"), (double)(n * (F::bytes + sizeof(TO))));
        k_scan_apply<TO, F><<<nb, kBlock, 0, ctx.stream>>>(f, out, offs.get(), n);
    }
    LAUNCH_TRY(ctx, "scan_apply");
    return RAMA_OK;
}

// ------------------------------------------------------------------------------------------
// Scan with a consumer instead of an output array.  scan_totals runs the reduce step and the scan of
// the tile sums and reads the total back (the caller sizes its outputs with it); scan_emit then
// recomputes f and hands every item k its value and exclusive prefix: emit(k, f(k), prefix).  The
// array of prefixes is never stored and the consumer does not re-read what the scan already had in
// registers.  `extra` words behind the total belong to the caller (e.g. a maximum a producer kernel
// left there) and come back with the same read.
// ------------------------------------------------------------------------------------------
template <typename TO>
struct ScanPlan {
    Buf<TO> offs;   // [nb] tile offsets, [nb] total, then the caller's extra words
    Buf<TO> sums;
    unsigned nb = 0;
    size_t n = 0;
    int extra = 0;
    TO total = 0;
    TO extra_value[2] = {0, 0};
    TO *extra_ptr() { return offs.get() + nb + 1; }
};

template <typename TO>
rama_status scan_plan_alloc(Ctx &ctx, size_t n, int extra, ScanPlan<TO> &plan)
{
    plan.n = n;
    plan.nb = grid_for(n, kScanTile);
    plan.extra = extra;
    RAMA_TRY(plan.offs.alloc(ctx, (size_t)plan.nb + 1 + 2));
    RAMA_TRY(plan.sums.alloc(ctx, plan.nb > 0 ? plan.nb : 1));
    // the total is always written by the scan of the tile sums; only the caller's words start at zero
    if (extra > 0) return fill<TO>(ctx, plan.extra_ptr(), (TO)0, (size_t)extra);
    return RAMA_OK;
}

// `presums`: the tile sums exist already (the kernel that produced f's input left them, tile by tile of
// kScanTile items, in plan.sums or in an array of its own), so the counting launch is skipped
template <typename TO, typename F>
rama_status scan_totals(Ctx &ctx, F f, ScanPlan<TO> &plan, const TO *presums = nullptr)
{
    plan.total = 0;
    const unsigned nb = plan.nb;
    const bool presummed = presums != nullptr;
    const TO *sums = presummed ? presums : plan.sums.get();
    TO back[3] = {0, 0, 0};
    if (plan.n > 0 && nb <= kScanMidMax) {
        // short arrays, one launch: tile sums, their scan by the last workgroup, total and extra words into the
        // mailbox; longer arrays: the scan of the tile sums is a launch of its own
        const uint64_t seq = ++ctx.mail_seq;
        const bool fused = nb <= kScanFusedMax && !presummed;
        if (!presummed) {
            ProfScope ps_(ctx, kernel_name<F>("k_scan_reduce"), (double)(plan.n * F::bytes));
            k_scan_reduce<TO, F><<<nb, kBlock, 0, ctx.stream>>>(f, plan.sums.get(), plan.n, plan.offs.get(),
                                                               fused ? ctx.ticket : nullptr, mailbox(ctx), seq, plan.extra);
        }
        LAUNCH_TRY(ctx, "scan_reduce");
        if (!fused) {
            ProfScope ps_(ctx, "k_scan_mid", (double)((size_t)nb * 2 * sizeof(TO)));
            k_scan_mid<TO><<<1, kBlock, 0, ctx.stream>>>(sums, plan.offs.get(), nb, mailbox(ctx), seq, plan.extra);
            LAUNCH_TRY(ctx, "scan_mid");
        }
        RAMA_TRY(wait_mail(ctx, seq));
        const volatile uint64_t *m = mailbox(ctx);
        for (int k = 0; k < 1 + plan.extra; ++k) back[k] = (TO)m[1 + k];
    } else if (plan.n > 0) {
        if (!presummed) {
            ProfScope ps_(ctx, kernel_name<F>("k_scan_reduce"), (double)(plan.n * F::bytes));
            k_scan_reduce<TO, F><<<nb, kBlock, 0, ctx.stream>>>(f, plan.sums.get(), plan.n, (TO *)nullptr, (uint32_t *)nullptr,
                                                               (uint64_t *)nullptr, 0, 0);
        }
        LAUNCH_TRY(ctx, "scan_reduce");
        // the nested scan writes nb+1 words (offsets and total), nothing beyond: the caller's extra words,
        // which sit one further on, stay as they are
        RAMA_TRY((exclusive_scan<TO, PtrInput<TO>>(ctx, PtrInput<TO>{sums}, plan.offs.get(), nb)));
        RAMA_TRY(read_back(ctx, back, plan.offs.get() + nb, (size_t)(1 + plan.extra) * sizeof(TO)));
    } else if (plan.extra > 0) {
        RAMA_TRY(read_back(ctx, back + 1, plan.extra_ptr(), (size_t)plan.extra * sizeof(TO)));
    }
    plan.total = back[0];
    plan.extra_value[0] = back[1];
    plan.extra_value[1] = back[2];
    plan.sums.reset();
    return RAMA_OK;
}

// A consumer that works with whole waves (shuffles, ballots) declares `static constexpr bool whole_wave = true`:
// it is then also called for the places behind the end of the array, with value 0.
template <typename E, typename = void>
struct EmitWholeWave { static constexpr bool value = false; };
template <typename E>
struct EmitWholeWave<E, std::void_t<decltype(E::whole_wave)>> { static constexpr bool value = E::whole_wave; };

template <typename TO, typename F, typename E>
__global__ __launch_bounds__(kBlock) void k_scan_emit(F f, E emit, const TO *block_offsets, size_t n)
{
    __shared__ TO wave_tot[4];
    const int w = threadIdx.x >> 6;
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)w * kScanWaveItems + lane_id();
    TO x[kScanItems], v[kScanItems];
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const size_t k = base + (size_t)q * 64;
        x[q] = (k < n) ? (TO)f(k) : (TO)0;
    }
    TO carry = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const TO inc = wave_inclusive_scan(x[q]);
        v[q] = inc - x[q] + carry;
        carry += wave_last(inc);
    }
    if (lane_id() == 0) wave_tot[w] = carry;
    __syncthreads();
    TO pre = block_offsets[blockIdx.x];
#pragma unroll
    for (int k = 0; k < 3; ++k)
        if (k < w) pre += wave_tot[k];
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const size_t k = base + (size_t)q * 64;
        if (EmitWholeWave<E>::value || k < n) emit(k, x[q], v[q] + pre);
    }
}

// `bytes`: what the consumer moves per launch beyond reading f's input (for the timers)
template <typename TO, typename F, typename E>
rama_status scan_emit(Ctx &ctx, F f, E emit, const ScanPlan<TO> &plan, double bytes)
{
    if (plan.n == 0) return RAMA_OK;
    {
        ProfScope ps_(ctx, kernel_name<E>("k_scan_emit"), (double)(plan.n * F::bytes) + bytes);
        k_scan_emit<TO, F, E><<<plan.nb, kBlock, 0, ctx.stream>>>(f, emit, plan.offs.get(), plan.n);
    }
    LAUNCH_TRY(ctx, "scan_emit");
    return RAMA_OK;
}

// ------------------------------------------------------------------------------------------
// row boundaries: keys[0..m) ascending with values in [0,n); ptr[v] = first position whose key
// is >= v, for v in [0,n]  (ptr[n] = m).  One launch, and every row is written exactly once:
//  - keys at least an eighth as many as rows: one thread per position fills the gap of rows before it when
//    the key changes there; a gap of more than kRowGapInline rows goes to a list in LDS that the whole
//    workgroup then fills side by side, so no thread ever loops over a long stretch alone;
//  - fewer keys than that (the empty stretches of a sparse key set are the rule): one thread per row,
//    binary search.
// ------------------------------------------------------------------------------------------
constexpr int kRowGapInline = 32;

// four positions per thread, read as one 16-byte vector (keys are 4 bytes wide)
template <typename K, typename P>
__global__ __launch_bounds__(kBlock) void k_row_bounds_fill(const K *keys, size_t m, int64_t n, P *ptr)
{
    static_assert(sizeof(K) == 4, "32-bit keys");
    __shared__ uint32_t s_count;
    __shared__ int64_t s_from[kBlock * 4], s_to[kBlock * 4];
    __shared__ P s_pos[kBlock * 4];
    if (threadIdx.x == 0) s_count = 0u;
    __syncthreads();
    const size_t e0 = ((size_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (e0 <= m) {
        K k[4];
        if (e0 + 4 <= m) {
            const uint4 v = *reinterpret_cast<const uint4 *>(keys + e0);   // e0 is a multiple of 4, the array 16-byte aligned
            k[0] = (K)v.x; k[1] = (K)v.y; k[2] = (K)v.z; k[3] = (K)v.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) k[q] = e0 + q < m ? keys[e0 + q] : (K)0;
        }
        int64_t prev = (e0 == 0) ? -1 : (int64_t)keys[e0 - 1];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const size_t e = e0 + q;
            if (e > m) break;
            const int64_t cur = (e == m) ? n : (int64_t)k[q];
            if (cur != prev) {
                if (cur - prev <= kRowGapInline) {
                    for (int64_t v = prev + 1; v <= cur; ++v) ptr[v] = (P)e;
                } else {      // at most one entry per position: the list cannot overflow
                    const uint32_t slot = atomicAdd(&s_count, 1u);
                    s_from[slot] = prev + 1; s_to[slot] = cur; s_pos[slot] = (P)e;
                }
            }
            prev = cur;
        }
    }
    __syncthreads();
    const uint32_t n_long = s_count;
    for (uint32_t g = 0; g < n_long; ++g) {
        const int64_t to = s_to[g];
        const P e = s_pos[g];
        for (int64_t v = s_from[g] + threadIdx.x; v <= to; v += kBlock) ptr[v] = e;
    }
}

// four rows per thread; a row's search starts where the row before it ended
template <typename K, typename P>
__global__ __launch_bounds__(kBlock) void k_row_bounds_search(const K *keys, size_t m, int64_t n, P *ptr)
{
    const int64_t v0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (v0 > n) return;
    size_t from = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t v = v0 + q;
        if (v > n) break;
        size_t lo = from, hi = m;
        while (lo < hi) {
            size_t mid = lo + ((hi - lo) >> 1);
            if ((int64_t)keys[mid] < v) lo = mid + 1; else hi = mid;
        }
        ptr[v] = (P)lo;
        from = lo;
    }
}

// ------------------------------------------------------------------------------------------
// stable LSD radix sort, up to kRadixBits bits per pass, 6144 / 5120 keys per workgroup.
// Ranking inside a wave uses ballot-based match-any, so equal digits keep their order
// without any atomics in the scatter pass.
// ------------------------------------------------------------------------------------------
// keys per thread: larger tiles give longer contiguous runs per digit on the way out; 24 (64-bit
// keys) and 20 (32-bit keys) measured best, beyond that the LDS footprint costs more than it gains
template <typename K>
struct SortTile {
    static constexpr int items = sizeof(K) == 8 ? 24 : 20;
    static constexpr int size = kBlock * items;
};
#ifndef RAMA_RADIX_BITS
#define RAMA_RADIX_BITS 8
#endif

constexpr int kRadixBits = RAMA_RADIX_BITS;        // widest digit of a pass
constexpr int kRadix = 1 << kRadixBits;
constexpr int kDigitsPerThread = kRadix / kBlock;   // digits owned by one thread in the prefix step
static_assert(kRadix >= kBlock && kRadix % kBlock == 0, "radix must be a multiple of the block size");

// 16 bytes per lane and load: a plain copy with 4-byte accesses tops out near 3.8 TB/s on this
// chip, one with 16-byte accesses reaches 6 TB/s.  Only the histogram uses them: the scatter
// kernel gained nothing from 16-byte loads/stores, and a persistent variant that prefetches the
// next tile into registers was slower (its registers leave room for one workgroup per CU) -- it
// is bound by the latency of its load -> rank -> stage -> store chain at two tiles per CU.
// Chained passes (one histogram kernel for all digits, then per pass a single kernel whose tiles
// take tickets and read their predecessors' published digit counts instead of a scanned
// histogram) were also measured: the scatter kernels ran 25-50 % slower while they waited on the
// agent-scope status words, the all-digit histogram is bound by its LDS atomics, and the whole
// solve took 11 % longer than with histogram + scan + scatter per pass.
// Where one pass over 9.8e7 (64-bit key, value) pairs spends its time (one 8-bit pass, measured with
// keys built for the purpose): the scatter kernel takes 0.78 ms on uniformly random digits, 0.57 ms
// when every key has the same digit (the output is then one sequential stream), and 0.47 ms for a
// 4-bit digit with sequential output -- so roughly 0.37 ms is moving the 24 bytes per key (6.3 TB/s),
// 0.2 ms the ballot ranking (about 26 us per digit bit) and 0.2 ms the cost of writing 256 separate
// pieces of ~24 keys per tile.  Computing all rows' ballots before touching the counters, or
// skipping the ballots for rows with a single digit, changed nothing measurable.
template <typename K>
struct alignas(16) KeyVec {
    K k[16 / sizeof(K)];
};

// The [digit][tile] tables of a pass: a workgroup stores (and later fetches) one word in each of up to 256 rows.
// Workgroups take their tiles by xcd_block(): with tile = workgroup number, a cache line of a row collected the
// words of sixteen workgroups on eight XCDs, two words per L2, and went to memory in pieces (26 MB written for a
// 3.2 MB table); the runs the scatter kernel writes for neighbouring tiles meet in one L2 as well.
template <typename K>
__global__ __launch_bounds__(kBlock) void k_rs_hist(const K *keys, uint32_t *hist, size_t n, int shift, int bits,
                                                    uint32_t nb)
{
    constexpr int kPer = 16 / (int)sizeof(K);                 // keys per vector
    constexpr int kVecs = SortTile<K>::items / kPer;          // vectors per thread
    static_assert(SortTile<K>::items % kPer == 0, "tile must be a whole number of vectors per thread");
    __shared__ uint32_t h[kRadix];
    for (int k = threadIdx.x; k < kRadix; k += kBlock) h[k] = 0;
    __syncthreads();
    const uint32_t mask = (1u << bits) - 1u;
    const uint32_t tile_id = xcd_block();
    if (tile_id >= nb) return;      // the whole workgroup (padding of the grid)
    const size_t tile = (size_t)tile_id * SortTile<K>::size;
    if (tile + SortTile<K>::size <= n) {                      // full tile: vector loads (tile starts are 16-byte aligned)
        const KeyVec<K> *src = reinterpret_cast<const KeyVec<K> *>(keys + tile);
#pragma unroll
        for (int r = 0; r < kVecs; ++r) {
            KeyVec<K> v = src[(size_t)r * kBlock + threadIdx.x];
#pragma unroll
            for (int q = 0; q < kPer; ++q) {
                // The top digits of nearly sorted keys (edge lists keyed by their first endpoint, the edges of
                // triangles listed triangle by triangle) take one, two or three values across a wave more often
                // than not, and atomics on one LDS word run one after the other: up to four times the lanes that
                // share the digit of the first lane left add their count once, as long as they are eight or more
                // (spread digits pay for one look only: on a neighbour graph's keys four looks per key made this
                // kernel 68 % slower); what is left then adds lane by lane.
                const uint32_t d = (uint32_t)(v.k[q] >> shift) & mask;
                uint64_t left = ~0ull;
#pragma unroll
                for (int round = 0; round < 4; ++round) {
                    const int first = __ffsll((long long)left) - 1;
                    const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)d, first);
                    const uint64_t same = __ballot(d == d0) & left;
                    if (__popcll(same) < 8) break;                                     // uniform: digits are spread, no point
                    if (lane_id() == first) atomicAdd(&h[d0], (uint32_t)__popcll(same));
                    left &= ~same;
                    if (left == 0ull) break;                                           // uniform
                }
                if (left & (1ull << lane_id())) atomicAdd(&h[d], 1u);
            }
        }
    } else {
        for (size_t idx = tile + threadIdx.x; idx < n; idx += kBlock)
            atomicAdd(&h[(uint32_t)(keys[idx] >> shift) & mask], 1u);
    }
    __syncthreads();
    for (uint32_t d = threadIdx.x; d <= mask; d += kBlock) hist[(size_t)d * nb + tile_id] = h[d];
}

// Offsets of a pass from its [digit][tile] histogram: workgroup d scans row d (keys with digit d in
// earlier tiles) and stores the row's total behind the table; the scatter kernel adds the keys of
// smaller digits itself, from the 256 totals.  One launch instead of the three of a general scan.
static __global__ __launch_bounds__(kBlock) void k_rs_rowscan(const uint32_t *hist, uint32_t *offs, uint32_t nb, uint32_t *totals)
{
    const uint32_t *in = hist + (size_t)blockIdx.x * nb;
    uint32_t *out = offs + (size_t)blockIdx.x * nb;
    uint32_t carry = 0;
    for (uint32_t c0 = 0; c0 < nb; c0 += kScanTile) {
        const uint32_t base = c0 + threadIdx.x * kScanItems;
        uint32_t v[kScanItems], s = 0;
#pragma unroll
        for (int q = 0; q < kScanItems; ++q) {
            v[q] = (base + q < nb) ? in[base + q] : 0u;
            s += v[q];
        }
        uint32_t tot;
        uint32_t run = block_inclusive_scan(s, &tot) - s + carry;
#pragma unroll
        for (int q = 0; q < kScanItems; ++q) {
            if (base + q < nb) out[base + q] = run;
            run += v[q];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

__device__ __forceinline__ uint64_t match_digit(uint32_t d, int bits, uint64_t valid)
{
    uint64_t m = valid;
    for (int b = 0; b < bits; ++b) {
        bool bit = (d >> b) & 1u;
        uint64_t bal = __ballot(bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

// One pass of the sort for one tile: (1) every wave ranks its items x 64 keys by digit with ballots,
// (2) per-digit prefix over the four waves and over the digits gives each key its place in the
// tile's digit-sorted order, (3) keys (and values) are staged in LDS in that order, (4) the tile
// is written out linearly -- neighbouring lanes hold neighbouring keys of the same digit, so the
// global stores fall into contiguous runs instead of 64 scattered lines per instruction.
// With LOCAL_SCAN (few tiles) `offs` is the raw [digit][tile] histogram and every workgroup derives
// its own global offsets from it, which saves the scan launch of the pass.
constexpr uint32_t kSortLocalScanTiles = 32;
template <typename K, typename V, bool HAS_V, bool LOCAL_SCAN>
__global__ __launch_bounds__(kBlock) void k_rs_scatter(const K *kin, const V *vin, K *kout, V *vout,
                                                       const uint32_t *offs, size_t n, int shift, int bits,
                                                       uint32_t nb)
{
    constexpr int kSortItems = SortTile<K>::items;
    constexpr int kSortTile = SortTile<K>::size;
    __shared__ uint32_t whist[4][kRadix];
    __shared__ uint32_t gdelta[kRadix];
    __shared__ K skey[kSortTile];
    __shared__ uint32_t sval[HAS_V ? kSortTile : 1];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t mask = (1u << bits) - 1u;
    const uint32_t tile_id = xcd_block();
    if (tile_id >= nb) return;      // the whole workgroup (padding of the grid)
    for (int k = tid; k < 4 * kRadix; k += kBlock) (&whist[0][0])[k] = 0;
    __syncthreads();
    const size_t tile_base = (size_t)tile_id * kSortTile;
    const size_t wave_base = tile_base + (size_t)w * (64 * kSortItems);
    const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    K key[kSortItems];
    uint32_t val[kSortItems];
    uint32_t rank[kSortItems];
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        size_t idx = wave_base + (size_t)r * 64 + lane;
        bool valid = idx < n;
        key[r] = valid ? kin[idx] : (K)0;
        if (HAS_V) val[r] = valid ? (vin ? (uint32_t)vin[idx] : (uint32_t)idx) : 0u;   // no array of values: a key's value is its place
    }
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        size_t idx = wave_base + (size_t)r * 64 + lane;
        bool valid = idx < n;
        uint32_t d = (uint32_t)(key[r] >> shift) & mask;
        uint64_t m = match_digit(d, bits, __ballot(valid));
        uint32_t before = whist[w][d];
        rank[r] = before + (uint32_t)__popcll(m & lt);
        __builtin_amdgcn_wave_barrier();
        if (valid && lane == (__ffsll((long long)m) - 1)) whist[w][d] = before + (uint32_t)__popcll(m);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    {   // this thread owns the digits [tid*kDigitsPerThread, +kDigitsPerThread)
        uint32_t c[kDigitsPerThread][4], tot = 0, all;
#pragma unroll
        for (int q = 0; q < kDigitsPerThread; ++q)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                c[q][k] = whist[k][tid * kDigitsPerThread + q];
                tot += c[q][k];
            }
        uint32_t run = block_inclusive_scan(tot, &all) - tot;
        uint32_t goff[kDigitsPerThread];
        if (LOCAL_SCAN) {
            // keys of smaller digits (all tiles) + keys of the same digit in earlier tiles
            uint32_t rows = 0, before[kDigitsPerThread], rowsum[kDigitsPerThread];
#pragma unroll
            for (int q = 0; q < kDigitsPerThread; ++q) {
                const uint32_t d = (uint32_t)(tid * kDigitsPerThread + q);
                before[q] = 0; rowsum[q] = 0;
                if (d <= mask)
                    for (uint32_t b = 0; b < nb; ++b) {
                        uint32_t h = offs[(size_t)d * nb + b];
                        if (b < tile_id) before[q] += h;
                        rowsum[q] += h;
                    }
                rows += rowsum[q];
            }
            uint32_t dummy;
            uint32_t dig = block_inclusive_scan(rows, &dummy) - rows;
#pragma unroll
            for (int q = 0; q < kDigitsPerThread; ++q) { goff[q] = dig + before[q]; dig += rowsum[q]; }
        } else {
            // offs: per digit the keys in earlier tiles, and behind the table the digits' totals
            const uint32_t *totals = offs + (size_t)kRadix * nb;
            uint32_t rows = 0, rowsum[kDigitsPerThread];
#pragma unroll
            for (int q = 0; q < kDigitsPerThread; ++q) {
                const uint32_t d = (uint32_t)(tid * kDigitsPerThread + q);
                rowsum[q] = d <= mask ? totals[d] : 0u;
                rows += rowsum[q];
            }
            uint32_t dummy;
            uint32_t dig = block_inclusive_scan(rows, &dummy) - rows;
#pragma unroll
            for (int q = 0; q < kDigitsPerThread; ++q) {
                const uint32_t d = (uint32_t)(tid * kDigitsPerThread + q);
                goff[q] = dig + (d <= mask ? offs[(size_t)d * nb + tile_id] : 0u);
                dig += rowsum[q];
            }
        }
#pragma unroll
        for (int q = 0; q < kDigitsPerThread; ++q) {
            const uint32_t d = (uint32_t)(tid * kDigitsPerThread + q);
            gdelta[d] = goff[q] - run;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                whist[k][d] = run;
                run += c[q][k];
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        size_t idx = wave_base + (size_t)r * 64 + lane;
        if (idx < n) {
            uint32_t d = (uint32_t)(key[r] >> shift) & mask;
            uint32_t lpos = whist[w][d] + rank[r];
            skey[lpos] = key[r];
            if (HAS_V) sval[lpos] = val[r];
        }
    }
    __syncthreads();
    const uint32_t cnt = (uint32_t)((n - tile_base) < (size_t)kSortTile ? (n - tile_base) : (size_t)kSortTile);
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        uint32_t idx = (uint32_t)r * kBlock + tid;
        if (idx < cnt) {
            K k = skey[idx];
            uint32_t pos = gdelta[(uint32_t)(k >> shift) & mask] + idx;
            kout[pos] = k;
            if (HAS_V) vout[pos] = (V)sval[idx];
        }
    }
}

template <typename K, bool HAS_V>
inline const char *rs_scatter_name()
{
    if (HAS_V) return sizeof(K) == 8 ? "k_rs_scatter<u64,u32>" : "k_rs_scatter<u32,u32>";
    return sizeof(K) == 8 ? "k_rs_scatter<u64>" : "k_rs_scatter<u32>";
}

// ---- split sort: the top bits by LSD passes, the rest inside LDS ----------------------------------
// After stable passes over the top bits the array consists of segments of equal top bits, each of
// which only has to be sorted by its low bits -- and a segment that fits into LDS is sorted there in
// one read and one write of the data, however many digits its low bits have.  Workgroup b takes the
// segments that START inside window [b*W, (b+1)*W): bounds[b] is the first segment start at or
// behind b*W, so a workgroup holds fewer than W + (longest segment) elements.  `oversize` is raised
// when that exceeds what a workgroup can hold; the caller then sorts the classical way.
template <typename K>
__device__ __forceinline__ size_t first_segment_start_from(const K *keys, size_t n, int low_bits, size_t x)
{
    if (x == 0) return 0;
    if (x >= n) return n;
    const K p = keys[x] >> low_bits;
    if ((keys[x - 1] >> low_bits) != p) return x;
    // end of the segment that contains x: gallop, then bisect.  keys[lo] has top bits p, keys[hi] has not (or hi == n)
    size_t lo = x, hi, step = 1;
    for (;;) {
        hi = lo + step;
        if (hi >= n) { hi = n; break; }
        if ((keys[hi] >> low_bits) != p) break;
        lo = hi;
        step <<= 1;
    }
    while (hi - lo > 1) {
        const size_t mid = lo + (hi - lo) / 2;
        if ((keys[mid] >> low_bits) == p) lo = mid; else hi = mid;
    }
    return hi;
}

template <typename K>
__global__ __launch_bounds__(kBlock) void k_seg_bounds(const K *keys, size_t n, int low_bits, uint32_t window, uint32_t cap,
                                                       int local_key_bits, uint32_t nbk, uint32_t *bounds, uint32_t *oversize)
{
    const uint32_t b = blockIdx.x * kBlock + threadIdx.x;
    if (b > nbk) return;
    if (b == nbk) { bounds[b] = (uint32_t)n; return; }
    const size_t f0 = first_segment_start_from(keys, n, low_bits, (size_t)b * window);
    const size_t f1 = first_segment_start_from(keys, n, low_bits, (size_t)(b + 1) * window);
    bounds[b] = (uint32_t)f0;
    if (f1 - f0 > cap) *oversize = 1u;
    if (f1 > f0) {      // the workgroup's keys relative to its first segment must fit the local key type
        const uint64_t top_span = (uint64_t)((keys[f1 - 1] >> low_bits) - (keys[f0] >> low_bits));
        if (low_bits + (top_span ? 64 - __clzll((long long)top_span) : 0) > local_key_bits) *oversize = 1u;
    }
}

// Sorts the elements [bounds[b], bounds[b+1]) by their low bits (and by the few top bits in which
// the segments of one workgroup differ: the keys are taken relative to the first segment's top
// bits, so those cost digits only where a workgroup spans many sparse segments).  Waves hold
// consecutive chunks, the passes are those of k_rs_scatter with LDS as the destination; between
// passes the keys return to registers in the new order.
// LK is the type of the keys while they are being sorted: 32 bits whenever the low bits (plus the
// few top bits in which a workgroup's segments differ) fit, which halves the LDS a key takes.
// Measured on 9.8e7 (64-bit key, value) pairs with 26 low bits: what counts is the number of waves a
// CU holds (LDS is the limit) and a workgroup of at most eight waves; 16 keys x 8 waves (two
// workgroups per CU) takes 1.45 ms -- 0.55 ms for reading and writing the data and 0.22 ms per 7-bit
// pass, which is the ballot ranking -- against 2.3 ms for 32 keys x 4 waves or 64-bit local keys.
constexpr int kLocalSortWaves = 8;
template <typename LK>
struct LocalSort {
    static constexpr int items = sizeof(LK) == 8 ? 8 : 16;
    static constexpr int threads = kLocalSortWaves * 64;
    static constexpr int cap = threads * items;
};
template <typename K, typename V, bool HAS_V, typename LK>
__global__ __launch_bounds__(kLocalSortWaves * 64) void k_rs_local(const K *kin, const V *vin, K *kout, V *vout,
                                                                   const uint32_t *bounds, int low_bits, uint32_t n_all,
                                                                   uint32_t *head_sums)
{
    constexpr int NW = kLocalSortWaves;
    constexpr int kItems = LocalSort<LK>::items;
    constexpr int kThreads = LocalSort<LK>::threads;
    constexpr int kCap = LocalSort<LK>::cap;
    static_assert(kRadix == 256 && kThreads >= kRadix, "one digit per thread of the first four waves");
    __shared__ uint32_t whist[NW][kRadix];
    __shared__ uint32_t wave_tot[4];
    __shared__ LK skey[kCap];
    __shared__ uint32_t sval[HAS_V ? kCap : 1];
    // without a bounds array the (single) workgroup takes the whole array of n_all keys
    const uint32_t beg = bounds ? bounds[blockIdx.x] : 0u, end = bounds ? bounds[blockIdx.x + 1] : n_all;
    const uint32_t cnt = end - beg;
    if (cnt == 0 || cnt > (uint32_t)kCap) return;      // the caller has ruled the second case out
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const K base = (kin[beg] >> low_bits) << low_bits;
    const uint64_t top_span = (uint64_t)((kin[end - 1] >> low_bits) - (kin[beg] >> low_bits));
    const int sort_bits = low_bits + (top_span ? 64 - __clzll((long long)top_span) : 0);
    const int passes = (sort_bits + kRadixBits - 1) / kRadixBits;
    const int rows = (int)((cnt + kThreads - 1) / kThreads);       // rows of 64 keys per wave
    const uint32_t wave_base = (uint32_t)w * (uint32_t)rows * 64u;
    const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    LK key[kItems];
    uint32_t val[kItems];
    uint32_t rank[kItems];
#pragma unroll
    for (int r = 0; r < kItems; ++r) {
        const uint32_t idx = wave_base + (uint32_t)r * 64u + lane;
        const bool valid = r < rows && idx < cnt;
        key[r] = valid ? (LK)(kin[beg + idx] - base) : (LK)0;
        if (HAS_V) val[r] = valid ? (uint32_t)vin[beg + idx] : 0u;
    }
    int shift = 0, remaining = sort_bits;
    for (int p = 0; p < passes; ++p) {
        const int bits = (remaining + (passes - p) - 1) / (passes - p);
        const uint32_t mask = (1u << bits) - 1u;
        for (int k = tid; k < NW * kRadix; k += kThreads) (&whist[0][0])[k] = 0;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kItems; ++r) {
            if (r < rows) {
                const uint32_t idx = wave_base + (uint32_t)r * 64u + lane;
                const bool valid = idx < cnt;
                const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
                const uint64_t m = match_digit(d, bits, __ballot(valid));
                const uint32_t before = whist[w][d];
                rank[r] = before + (uint32_t)__popcll(m & lt);
                __builtin_amdgcn_wave_barrier();
                if (valid && lane == (__ffsll((long long)m) - 1)) whist[w][d] = before + (uint32_t)__popcll(m);
                __builtin_amdgcn_wave_barrier();
            }
        }
        __syncthreads();
        {   // thread d < 256 owns digit d: places of the waves' keys with this digit in the sorted order
            uint32_t c[NW], tot = 0;
            if (tid < kRadix) {
#pragma unroll
                for (int k = 0; k < NW; ++k) { c[k] = whist[k][tid]; tot += c[k]; }
            }
            const uint32_t inc = wave_inclusive_scan(tot);
            if (tid < kRadix && lane == 63) wave_tot[w] = inc;
            __syncthreads();
            if (tid < kRadix) {
                uint32_t run = inc - tot;
#pragma unroll
                for (int k = 0; k < 3; ++k)
                    if (k < w) run += wave_tot[k];
#pragma unroll
                for (int k = 0; k < NW; ++k) { whist[k][tid] = run; run += c[k]; }
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kItems; ++r) {
            if (r < rows) {
                const uint32_t idx = wave_base + (uint32_t)r * 64u + lane;
                if (idx < cnt) {
                    const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
                    const uint32_t lpos = whist[w][d] + rank[r];
                    skey[lpos] = key[r];
                    if (HAS_V) sval[lpos] = val[r];
                }
            }
        }
        __syncthreads();
        if (p + 1 < passes) {
#pragma unroll
            for (int r = 0; r < kItems; ++r) {
                if (r < rows) {
                    const uint32_t idx = wave_base + (uint32_t)r * 64u + lane;
                    if (idx < cnt) {
                        key[r] = skey[idx];
                        if (HAS_V) val[r] = sval[idx];
                    }
                }
            }
        }
        shift += bits;
        remaining -= bits;
    }
    if (!head_sums) {   // uniform
        for (uint32_t idx = tid; idx < cnt; idx += kThreads) {
            kout[beg + idx] = (K)((K)skey[idx] + base);
            if (HAS_V) vout[beg + idx] = (V)sval[idx];
        }
        return;
    }
    // The sorted keys are at hand: count the heads of runs of equal keys per tile of kScanTile places, for a scan
    // over the heads that follows the sort (it then needs no counting pass).  A workgroup's first key starts a
    // new segment of top bits, so it is a head; its places span at most kHeadTiles tiles.
    constexpr int kHeadTiles = kCap / kScanTile + 1;
    __shared__ uint32_t s_heads[kHeadTiles];
    if (tid < kHeadTiles) s_heads[tid] = 0;
    __syncthreads();
    const uint32_t tile0 = beg / (uint32_t)kScanTile;
    for (uint32_t idx0 = 0; idx0 < cnt; idx0 += kThreads) {
        const uint32_t idx = idx0 + tid;
        const bool valid = idx < cnt;
        bool head = false;
        if (valid) {
            const LK k = skey[idx];
            kout[beg + idx] = (K)((K)k + base);
            if (HAS_V) vout[beg + idx] = (V)sval[idx];
            head = idx == 0 || k != skey[idx - 1];
        }
        // the wave's 64 places lie in one tile or in two
        const uint32_t first = beg + idx0 + (uint32_t)w * 64u;
        const uint32_t t_lo = first / (uint32_t)kScanTile, t_hi = (first + 63u) / (uint32_t)kScanTile;
        const uint64_t heads = __ballot(head);
        if (t_lo == t_hi) {
            if (lane == 0 && heads) atomicAdd(&s_heads[t_lo - tile0], (uint32_t)__popcll(heads));
        } else {
            const uint32_t n_lo = t_hi * (uint32_t)kScanTile - first;     // places of the wave that lie in the lower tile
            const uint64_t low = (~0ull) >> (64u - n_lo);
            if (lane == 0) {
                if (heads & low) atomicAdd(&s_heads[t_lo - tile0], (uint32_t)__popcll(heads & low));
                if (heads & ~low) atomicAdd(&s_heads[t_hi - tile0], (uint32_t)__popcll(heads & ~low));
            }
        }
    }
    __syncthreads();
    if (tid < kHeadTiles && s_heads[tid]) atomicAdd(&head_sums[tile0 + tid], s_heads[tid]);
}

template <typename K, bool HAS_V, typename LK>
inline const char *rs_local_name()
{
    if (sizeof(LK) == 8) {      // 64-bit keys inside LDS: the low bits did not fit 32
        if (HAS_V) return sizeof(K) == 8 ? "k_rs_local<u64,u32,wide>" : "k_rs_local<u32,u32,wide>";
        return sizeof(K) == 8 ? "k_rs_local<u64,wide>" : "k_rs_local<u32,wide>";
    }
    if (HAS_V) return sizeof(K) == 8 ? "k_rs_local<u64,u32>" : "k_rs_local<u32,u32>";
    return sizeof(K) == 8 ? "k_rs_local<u64>" : "k_rs_local<u32>";
}

// stable LSD passes over the key bits [shift, shift + total_bits); a/b swap with every pass
template <typename K, typename V, bool HAS_V>
rama_status radix_passes(Ctx &ctx, K *&ka, V *&va, K *&kb, V *&vb, size_t n, int shift, int total_bits, uint32_t *hist,
                         uint32_t *offs, bool *result_in_b, bool *iota, K *&kc, V *&vc)
{
    const uint32_t nb = grid_for(n, SortTile<K>::size);
    const int passes = (total_bits + kRadixBits - 1) / kRadixBits;
    int remaining = total_bits;
    for (int p = 0; p < passes; ++p) {
        int bits = (remaining + (passes - p) - 1) / (passes - p);
        {
            ProfScope ps_(ctx, (sizeof(K) == 8 ? "k_rs_hist<u64>" : "k_rs_hist<u32>"), (double)(n * sizeof(K)));
            k_rs_hist<K><<<xcd_grid(nb), kBlock, 0, ctx.stream>>>(ka, hist, n, shift, bits, nb);
        }
        LAUNCH_TRY(ctx, "rs_hist");
        const V *vin = (HAS_V && *iota) ? (const V *)nullptr : va;   // the first pass of a sort whose values are the places 0..n-1
        *iota = false;
        if (nb <= kSortLocalScanTiles) {
            ProfScope ps_(ctx, rs_scatter_name<K, HAS_V>(), (double)(n * (2 * sizeof(K) + (HAS_V ? 8 : 0))));
            k_rs_scatter<K, V, HAS_V, true><<<xcd_grid(nb), kBlock, 0, ctx.stream>>>(ka, vin, kb, vb, hist, n, shift, bits, nb);
        } else {
            {
                ProfScope ps_(ctx, "k_rs_rowscan", (double)(((size_t)nb << bits) * 8));
                k_rs_rowscan<<<1u << bits, kBlock, 0, ctx.stream>>>(hist, offs, nb, offs + (size_t)kRadix * nb);
            }
            LAUNCH_TRY(ctx, "rs_rowscan");
            ProfScope ps_(ctx, rs_scatter_name<K, HAS_V>(), (double)(n * (2 * sizeof(K) + (HAS_V ? 8 : 0))));
            k_rs_scatter<K, V, HAS_V, false><<<xcd_grid(nb), kBlock, 0, ctx.stream>>>(ka, vin, kb, vb, offs, n, shift, bits, nb);
        }
        LAUNCH_TRY(ctx, "rs_scatter");
        std::swap(ka, kb);
        std::swap(va, vb);
        if (kc) {   // the input must stay as it is: from now on the passes alternate between the two other buffers
            kb = kc; vb = vc;
            kc = nullptr; vc = nullptr;
        }
        *result_in_b = !*result_in_b;
        shift += bits;
        remaining -= bits;
    }
    return RAMA_OK;
}

// zeroed counters for the heads per scan tile of an array of n sorted keys (k_rs_local fills them)
inline rama_status head_sums_alloc(Ctx &ctx, size_t n, Buf<uint32_t> *head_sums)
{
    if (!head_sums) return RAMA_OK;
    const size_t tiles = (n + kScanTile - 1) / kScanTile + 1;
    return zeroed<uint32_t>(ctx, tiles, *head_sums);
}

// bounds + in-LDS sort of an array already sorted by its bits above low_bits; *done stays false
// when some workgroup could not hold its segments (nothing has been written then)
template <typename K, typename V, bool HAS_V, typename LK>
rama_status split_sort_tail(Ctx &ctx, K *ka, V *va, K *kb, V *vb, size_t n, int low_bits, bool *done, Buf<uint32_t> *head_sums)
{
    using LS = LocalSort<LK>;
    *done = false;
    const uint32_t window = LS::cap / 2;
    const uint32_t nbk = grid_for(n, (int)window);
    Buf<uint32_t> bounds, over_flag;
    RAMA_TRY(bounds.alloc(ctx, (size_t)nbk + 1));
    RAMA_TRY(zeroed<uint32_t>(ctx, 1, over_flag));
    uint32_t *oversize = over_flag.get();
    {
        ProfScope ps_(ctx, "k_seg_bounds", (double)((size_t)nbk * (4 + 32 * sizeof(K))));
        k_seg_bounds<K><<<grid_for((size_t)nbk + 1), kBlock, 0, ctx.stream>>>(ka, n, low_bits, window, (uint32_t)LS::cap,
                                                                             8 * (int)sizeof(LK), nbk, bounds.get(), oversize);
    }
    LAUNCH_TRY(ctx, "seg_bounds");
    uint32_t over = 0;
    RAMA_TRY(read_back(ctx, &over, oversize, 4));
    if (over) return RAMA_OK;
    RAMA_TRY(head_sums_alloc(ctx, n, head_sums));
    {
        ProfScope ps_(ctx, rs_local_name<K, HAS_V, LK>(), (double)(n * (2 * sizeof(K) + (HAS_V ? 8 : 0))));
        k_rs_local<K, V, HAS_V, LK><<<nbk, LS::threads, 0, ctx.stream>>>(ka, va, kb, vb, bounds.get(), low_bits, (uint32_t)n,
                                                                      head_sums ? head_sums->get() : nullptr);
    }
    LAUNCH_TRY(ctx, "rs_local");
    *done = true;
    return RAMA_OK;
}

// Sorts keys (and 32-bit values) by the low `total_bits` bits of the key.  a/b are two buffers
// of n elements each; input in a; on return *result_in_b says where the sorted data is.
// Long arrays are split when that replaces at least two passes: passes over the top bits until
// the segments of equal top bits are at most two fifths of a workgroup's capacity on average, then one
// in-LDS sort of the rest.  Should the keys be so uneven that some workgroup cannot hold its
// segments, the array (by then stably sorted by the top bits, which does no harm) is sorted by
// passes over all bits instead.
// `iota`: the values are the places 0..n-1 and va holds nothing yet -- the first pass makes them up instead of
// reading them (an array one workgroup sorts alone gets them from a fill first).
static __global__ __launch_bounds__(kBlock) void k_iota(size_t n, uint32_t *p)
{
    size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (k < n) p[k] = (uint32_t)k;
}
template <typename K, typename V, bool HAS_V>
rama_status radix_sort_impl(Ctx &ctx, K *ka, V *va, K *kb, V *vb, size_t n, int total_bits, bool *result_in_b, bool iota = false,
                            Buf<uint32_t> *head_sums = nullptr, uint64_t key_limit = 0, K *kc = nullptr, V *vc = nullptr,
                            K **res_k = nullptr, V **res_v = nullptr)
{
    // kc, vc (optional): a third pair of buffers; the input a is then only read, and the sorted data ends up in b or
    // in c: *res_k, *res_v say where
    // key_limit (optional): all keys are below it (and it needs total_bits bits); 0 = nothing known
    if (key_limit && (total_bits >= 64 || key_limit > (uint64_t(1) << total_bits))) key_limit = 0;
    // head_sums (optional): comes back allocated and filled -- per tile of kScanTile places the number of keys that
    // differ from their left neighbour -- when the sort ends in the in-LDS kernel, and empty otherwise
    if (head_sums) head_sums->reset();
    *result_in_b = false;
    if (n <= 1 || total_bits <= 0) return RAMA_OK;
    if (n >= (size_t(1) << 32)) return fail(ctx, RAMA_ERR_CAPACITY, "radix sort: more than 2^32 keys");
    // an array that one workgroup can hold is sorted inside LDS by a single launch
    if (total_bits < 8 * (int)sizeof(K) && ctx.sort_split_min < (size_t)INT64_MAX) {
        const bool narrow = total_bits <= 32 && n <= (size_t)LocalSort<uint32_t>::cap;
        const bool wide = !narrow && n <= (size_t)LocalSort<uint64_t>::cap;
        if ((narrow || wide) && HAS_V && iota) {
            ProfScope ps_(ctx, "k_iota", (double)(n * 4));
            k_iota<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, (uint32_t *)va);
            LAUNCH_TRY(ctx, "iota");
            iota = false;
        }
        if (narrow || wide) {
            RAMA_TRY(head_sums_alloc(ctx, n, head_sums));
            uint32_t *hs = head_sums ? head_sums->get() : nullptr;
            if (narrow) {
                ProfScope ps_(ctx, rs_local_name<K, HAS_V, uint32_t>(), (double)(n * (2 * sizeof(K) + (HAS_V ? 8 : 0))));
                k_rs_local<K, V, HAS_V, uint32_t><<<1, LocalSort<uint32_t>::threads, 0, ctx.stream>>>(ka, va, kb, vb, (const uint32_t *)nullptr,
                                                                                                  total_bits, (uint32_t)n, hs);
            } else {
                ProfScope ps_(ctx, rs_local_name<K, HAS_V, uint64_t>(), (double)(n * (2 * sizeof(K) + (HAS_V ? 8 : 0))));
                k_rs_local<K, V, HAS_V, uint64_t><<<1, LocalSort<uint64_t>::threads, 0, ctx.stream>>>(ka, va, kb, vb, (const uint32_t *)nullptr,
                                                                                                  total_bits, (uint32_t)n, hs);
            }
            LAUNCH_TRY(ctx, "rs_local");
            *result_in_b = true;
            if (res_k) { *res_k = kb; *res_v = vb; }
            return RAMA_OK;
        }
    }
    const uint32_t nb = grid_for(n, SortTile<K>::size);
    Buf<uint32_t> hist, offs;
    RAMA_TRY(hist.alloc(ctx, (size_t)kRadix * nb));
    RAMA_TRY(offs.alloc(ctx, (size_t)kRadix * nb + kRadix));
    const int all_passes = (total_bits + kRadixBits - 1) / kRadixBits;
    if (n >= ctx.sort_split_min) {
        // top bits: whole passes, enough of them for segments that a workgroup can hold.  A workgroup takes the
        // segments that start in half a capacity of places, so what it gets stays below the capacity as long as no
        // segment is longer than half the capacity.  Without knowledge of the keys the segments are assumed to be a
        // quarter of the capacity on average at most (the keys seldom fill the whole range of their bits: fewer,
        // longer segments).  With a bound on the keys (`key_limit`) the number of segments is known and two fifths of
        // the capacity are allowed (the incidence sort of the 320^3 grid, 1.9e8 keys below 1.3e8: two top-bit passes
        // and one in-LDS sort instead of four passes, -0.6 ms).  A few spare low bits leave room for the top bits in
        // which a workgroup's segments differ.
        auto plan = [&](int cap, int *top_bits) {
            const uint64_t seg = key_limit ? (uint64_t)cap * 2 / 5 : (uint64_t)cap / 4;
            int t = kRadixBits;
            for (; t < total_bits; t += kRadixBits) {
                const uint64_t nseg = key_limit ? ((key_limit - 1) >> (total_bits - t)) + 1 : (uint64_t(1) << t);
                if (((uint64_t)n + nseg - 1) / nseg <= seg) break;
            }
            *top_bits = t;
            return t < total_bits && all_passes - t / kRadixBits >= ctx.sort_split_gain;
        };
        int top_bits = 0;
        bool narrow = plan(LocalSort<uint32_t>::cap, &top_bits) && total_bits - top_bits + 6 <= 32;
        const bool split = narrow || plan(LocalSort<uint64_t>::cap, &top_bits);
        if (split) {
            const int low_bits = total_bits - top_bits;
            RAMA_TRY((radix_passes<K, V, HAS_V>(ctx, ka, va, kb, vb, n, low_bits, top_bits, hist.get(), offs.get(), result_in_b, &iota, kc, vc)));
            bool done = false;
            if (narrow) RAMA_TRY((split_sort_tail<K, V, HAS_V, uint32_t>(ctx, ka, va, kb, vb, n, low_bits, &done, head_sums)));
            else RAMA_TRY((split_sort_tail<K, V, HAS_V, uint64_t>(ctx, ka, va, kb, vb, n, low_bits, &done, head_sums)));
            if (done) {
                *result_in_b = !*result_in_b;
                if (res_k) { *res_k = kb; *res_v = vb; }
                return RAMA_OK;
            }
        }
    }
    RAMA_TRY((radix_passes<K, V, HAS_V>(ctx, ka, va, kb, vb, n, 0, total_bits, hist.get(), offs.get(), result_in_b, &iota, kc, vc)));
    if (res_k) { *res_k = ka; *res_v = va; }
    return RAMA_OK;
}

// Convenience wrappers working on Buf pairs: after the call `k`/`v` hold the sorted data.
// `iota`: v comes in unset and stands for the values 0..n-1
template <typename K, typename V>
rama_status radix_sort_pairs(Ctx &ctx, Buf<K> &k, Buf<V> &v, size_t n, int total_bits, bool iota = false,
                             Buf<uint32_t> *head_sums = nullptr, uint64_t key_limit = 0)
{
    static_assert(sizeof(V) == 4, "32-bit payload");
    if (head_sums) head_sums->reset();
    if (n <= 1 || total_bits <= 0) {
        if (iota && n >= 1) {
            k_iota<<<grid_for(n), kBlock, 0, ctx.stream>>>(n, (uint32_t *)v.get());
            LAUNCH_TRY(ctx, "iota");
        }
        return RAMA_OK;
    }
    Buf<K> k2;
    Buf<V> v2;
    RAMA_TRY(k2.alloc(ctx, n));
    RAMA_TRY(v2.alloc(ctx, n));
    bool in_b = false;
    RAMA_TRY((radix_sort_impl<K, V, true>(ctx, k.get(), v.get(), k2.get(), v2.get(), n, total_bits, &in_b, iota, head_sums, key_limit)));
    if (in_b) { k.swap(k2); v.swap(v2); }
    return RAMA_OK;
}

// The same sort for pairs that must stay where they are (kin, vin are only read): k, v are allocated here and hold
// the sorted pairs on return.
template <typename K, typename V>
rama_status radix_sort_pairs_from(Ctx &ctx, const K *kin, const V *vin, Buf<K> &k, Buf<V> &v, size_t n, int total_bits,
                                  uint64_t key_limit = 0)
{
    static_assert(sizeof(V) == 4, "32-bit payload");
    RAMA_TRY(k.alloc(ctx, n > 0 ? n : 1));
    RAMA_TRY(v.alloc(ctx, n > 0 ? n : 1));
    if (n <= 1 || total_bits <= 0) {
        if (n > 0) {
            HIP_TRY(ctx, hipMemcpyAsync(k.get(), kin, n * sizeof(K), hipMemcpyDeviceToDevice, ctx.stream));
            HIP_TRY(ctx, hipMemcpyAsync(v.get(), vin, n * sizeof(V), hipMemcpyDeviceToDevice, ctx.stream));
        }
        return RAMA_OK;
    }
    Buf<K> k2;
    Buf<V> v2;
    RAMA_TRY(k2.alloc(ctx, n));
    RAMA_TRY(v2.alloc(ctx, n));
    bool in_b = false;
    K *rk = nullptr;
    V *rv = nullptr;
    RAMA_TRY((radix_sort_impl<K, V, true>(ctx, const_cast<K *>(kin), const_cast<V *>(vin), k.get(), v.get(), n, total_bits, &in_b, false,
                                          nullptr, key_limit, k2.get(), v2.get(), &rk, &rv)));
    if (rk == k2.get()) { k.swap(k2); v.swap(v2); }
    return RAMA_OK;
}

template <typename K>
rama_status radix_sort_keys(Ctx &ctx, Buf<K> &k, size_t n, int total_bits, Buf<uint32_t> *head_sums = nullptr, uint64_t key_limit = 0)
{
    if (head_sums) head_sums->reset();
    if (n <= 1) return RAMA_OK;
    Buf<K> k2;
    RAMA_TRY(k2.alloc(ctx, n));
    bool in_b = false;
    RAMA_TRY((radix_sort_impl<K, uint32_t, false>(ctx, k.get(), (uint32_t *)nullptr, k2.get(), (uint32_t *)nullptr, n,
                                                  total_bits, &in_b, false, head_sums, key_limit)));
    if (in_b) k.swap(k2);
    return RAMA_OK;
}

// ------------------------------------------------------------------------------------------
// deterministic sum of f(0..n-1) in double: per-block partials, then one block adds them in order
// ------------------------------------------------------------------------------------------
constexpr int kSumItems = 32;

template <typename F>
__global__ __launch_bounds__(kBlock) void k_sum_partial(F f, double *partial, size_t n)
{
    size_t base = (size_t)blockIdx.x * (kBlock * kSumItems) + threadIdx.x;
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < kSumItems; ++q) {
        size_t idx = base + (size_t)q * kBlock;
        if (idx < n) s += f(idx);
    }
    double tot = block_sum(s);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

static __global__ __launch_bounds__(kBlock) void k_sum_final(const double *partial, size_t nb, double *out, int accumulate)
{
    // thread t adds partial[t], partial[t+256], ... in order; then the fixed block tree
    double s = 0.0;
    for (size_t k = threadIdx.x; k < nb; k += kBlock) s += partial[k];
    double tot = block_sum(s);
    if (threadIdx.x == 0) *out = accumulate ? (*out + tot) : tot;
}

template <typename F>
rama_status device_sum(Ctx &ctx, F f, size_t n, double *out_dev, bool accumulate)
{
    unsigned nb = grid_for(n, kBlock * kSumItems);
    if (nb == 0) nb = 1;
    Buf<double> partial;
    RAMA_TRY(partial.alloc(ctx, nb));
    {
        ProfScope ps_(ctx, kernel_name<F>("k_sum_partial"), (double)(n * F::bytes));
        k_sum_partial<F><<<nb, kBlock, 0, ctx.stream>>>(f, partial.get(), n);
    }
    LAUNCH_TRY(ctx, "sum_partial");
    {
        ProfScope ps_(ctx, "k_sum_final", (double)(nb * 8));
        k_sum_final<<<1, kBlock, 0, ctx.stream>>>(partial.get(), nb, out_dev, accumulate ? 1 : 0);
    }
    LAUNCH_TRY(ctx, "sum_final");
    return RAMA_OK;
}

// ------------------------------------------------------------------------------------------
// small fill / iota kernels
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void k_fill(T *p, T v, size_t n)
{
    size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (k < n) p[k] = v;
}
// 16 bytes per thread; p must be 16-byte aligned
template <typename T>
__global__ __launch_bounds__(kBlock) void k_fill_wide(T *p, T v, size_t n)
{
    constexpr int kPer = 16 / (int)sizeof(T);
    struct alignas(16) Vec { T x[kPer]; };
    size_t k = ((size_t)blockIdx.x * kBlock + threadIdx.x) * kPer;
    if (k + kPer <= n) {
        Vec w;
#pragma unroll
        for (int q = 0; q < kPer; ++q) w.x[q] = v;
        *reinterpret_cast<Vec *>(p + k) = w;
    } else {
        for (; k < n; ++k) p[k] = v;
    }
}
// up to four arrays of 32-bit words filled by one launch (arrays that one step sets up together);
// every array is 16-byte aligned (pool blocks are) and is written 16 bytes per thread
struct FillJobs {
    uint32_t *p[4];
    uint32_t v[4];
    size_t end[4];   // running totals of the arrays' lengths in 16-byte pieces
    size_t words[4];
};
static __global__ __launch_bounds__(kBlock) void k_fill_multi(FillJobs jobs)
{
    const size_t k = (size_t)blockIdx.x * kBlock + threadIdx.x;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const size_t first = a ? jobs.end[a - 1] : 0;
        if (k >= first && k < jobs.end[a]) {
            const size_t w = (k - first) * 4;
            uint32_t *p = jobs.p[a] + w;
            const uint32_t v = jobs.v[a];
            if (w + 4 <= jobs.words[a]) *reinterpret_cast<uint4 *>(p) = make_uint4(v, v, v, v);
            else for (size_t q = w; q < jobs.words[a]; ++q) jobs.p[a][q] = v;
        }
    }
}
class MultiFill {
public:
    template <typename T>
    void add(T *p, uint32_t pattern, size_t count)   // `count` elements of T, every 32-bit word of which becomes `pattern`
    {
        static_assert(sizeof(T) % 4 == 0, "whole words");
        if (count == 0 || n_ >= 4) { overflow_ |= (count != 0); return; }
        jobs_.p[n_] = reinterpret_cast<uint32_t *>(p);
        jobs_.v[n_] = pattern;
        jobs_.words[n_] = count * (sizeof(T) / 4);
        total_ += (jobs_.words[n_] + 3) / 4;
        jobs_.end[n_] = total_;
        bytes_ += (double)(count * sizeof(T));
        ++n_;
    }
    rama_status run(Ctx &ctx)
    {
        if (overflow_) return fail(ctx, RAMA_ERR_INVALID_ARG, "more than four arrays in one fill");
        if (n_ == 0) return RAMA_OK;
        for (int a = n_; a < 4; ++a) { jobs_.p[a] = nullptr; jobs_.v[a] = 0; jobs_.end[a] = total_; jobs_.words[a] = 0; }
        {
            ProfScope ps_(ctx, "k_fill", bytes_);
            k_fill_multi<<<grid_for(total_), kBlock, 0, ctx.stream>>>(jobs_);
        }
        LAUNCH_TRY(ctx, "fill_multi");
        return RAMA_OK;
    }

private:
    FillJobs jobs_{};
    int n_ = 0;
    size_t total_ = 0;
    double bytes_ = 0.0;
    bool overflow_ = false;
};

template <typename T>
rama_status fill(Ctx &ctx, T *p, T v, size_t n)
{
    if (n == 0) return RAMA_OK;
    constexpr int kPer = 16 / (int)sizeof(T);
    const bool wide = sizeof(T) < 16 && n >= 1024 && (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
    {
        ProfScope ps_(ctx, "k_fill", (double)(n * sizeof(T)));
        if (wide) k_fill_wide<T><<<grid_for((n + kPer - 1) / kPer), kBlock, 0, ctx.stream>>>(p, v, n);
        else k_fill<T><<<grid_for(n), kBlock, 0, ctx.stream>>>(p, v, n);
    }
    LAUNCH_TRY(ctx, "fill");
    return RAMA_OK;
}

template <typename K, typename P>
rama_status row_bounds(Ctx &ctx, const K *keys, size_t m, int64_t n, P *ptr)
{
    if (m >= (size_t)n / 8) {
        ProfScope ps_(ctx, "k_row_bounds_fill", (double)(m * sizeof(K) + ((size_t)n + 1) * sizeof(P)));
        k_row_bounds_fill<K, P><<<grid_for(m / 4 + 1), kBlock, 0, ctx.stream>>>(keys, m, n, ptr);
    } else {
        ProfScope ps_(ctx, "k_row_bounds_search", (double)(m * sizeof(K) + ((size_t)n + 1) * sizeof(P)));
        k_row_bounds_search<K, P><<<grid_for((size_t)n / 4 + 1), kBlock, 0, ctx.stream>>>(keys, m, n, ptr);
    }
    LAUNCH_TRY(ctx, "row_bounds");
    return RAMA_OK;
}

// Edge keys.  An undirected edge (lo,hi), lo<hi, sorts as the pair (lo, hi-lo): same order as
// (lo,hi), but the second field only needs bits(max hi-lo) bits -- on grid-like graphs that saves
// a radix pass.  key = lo << dbits | (hi-lo).
__device__ __forceinline__ uint64_t edge_key(uint32_t lo, uint32_t hi, int dbits) { return ((uint64_t)lo << dbits) | (hi - lo); }

// maximum over the workgroup folded into *out (which only ever grows, so a stale read can only
// cause a redundant atomic)
__device__ __forceinline__ void block_max_into(uint32_t v, uint32_t *out)
{
    __shared__ uint32_t wmax[4];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, off, 64));
    if (lane_id() == 0) wmax[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        v = max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));
        if (v > *(volatile uint32_t *)out) atomicMax(out, v);
    }
}

// Sums runs of equal keys in order of appearance (one thread per run, sequential adds) and writes run number p
// -- endpoint pair and cost -- at place p.  The tiling is that of the scan over the run heads (HeadFlag), whose
// tile offsets come in through `block_offsets`.  A workgroup keeps its 2048 values and head marks in LDS:
// the heads are found from the keys in registers (the left neighbour's key by a shuffle), and a run is
// added up from LDS instead of by a chain of dependent fetches of keys and values; only a run that
// crosses the end of the tile goes on in memory.
static // `sign_sums` (optional, zero on entry): per tile of kScanTile *outputs* the number of positive costs (low half)
// and of negative costs (high half) -- the tile sums of the scan that splits the new graph by sign, which then
// needs no counting pass.  A workgroup's outputs are contiguous and at most a tile long: two atomic adds.
__global__ __launch_bounds__(kBlock) void k_reduce_runs(size_t m, const uint64_t *key, const uint32_t *val, int dbits,
                                                        const uint32_t *block_offsets, int32_t *io, int32_t *jo, float *co,
                                                        unsigned long long *sign_sums)
{
    __shared__ float s_val[kScanTile];
    __shared__ uint8_t s_head[kScanTile];
    __shared__ uint32_t wave_tot[4];
    const int w = threadIdx.x >> 6, lane = lane_id();
    const size_t tile0 = (size_t)blockIdx.x * kScanTile;
    const int local0 = w * kScanWaveItems + lane;
    uint64_t k[kScanItems];
    uint32_t x[kScanItems], v[kScanItems];
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const int local = local0 + q * 64;
        const size_t e = tile0 + (size_t)local;
        k[q] = e < m ? key[e] : 0ull;
        uint64_t left = __shfl_up(k[q], 1, 64);
        if (lane == 0 && e > 0 && e < m) left = key[e - 1];
        x[q] = (e < m && (e == 0 || k[q] != left)) ? 1u : 0u;
        s_val[local] = e < m ? __uint_as_float(val[e]) : 0.0f;
        s_head[local] = (uint8_t)(e < m ? x[q] : 1u);   // what lies behind the array ends every run
    }
    uint32_t carry = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        const uint32_t inc = wave_inclusive_scan(x[q]);
        v[q] = inc - x[q] + carry;
        carry += wave_last(inc);
    }
    if (lane == 0) wave_tot[w] = carry;
    __syncthreads();
    const uint32_t pre0 = block_offsets[blockIdx.x];
    uint32_t pre = pre0;
#pragma unroll
    for (int j = 0; j < 3; ++j)
        if (j < w) pre += wave_tot[j];
    const uint32_t tile_a = pre0 / (uint32_t)kScanTile;
    unsigned long long sa = 0ull, sb = 0ull;   // sign counts of the outputs in tile_a and in the tile behind it
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        if (!x[q]) continue;
        int pos = local0 + q * 64;
        float acc = s_val[pos];
        for (++pos; pos < kScanTile && !s_head[pos]; ++pos) acc = acc + s_val[pos];
        if (pos == kScanTile)
            for (size_t f = tile0 + kScanTile; f < m && key[f] == k[q]; ++f) acc = acc + __uint_as_float(val[f]);
        const uint32_t p = v[q] + pre;
        const uint32_t lo = (uint32_t)(k[q] >> dbits);
        io[p] = (int32_t)lo;
        jo[p] = (int32_t)(lo + (uint32_t)(k[q] & ((1ull << dbits) - 1ull)));
        co[p] = acc;
        const unsigned long long sgn = acc > 0.0f ? 1ull : (acc < 0.0f ? (1ull << 32) : 0ull);
        if (p / (uint32_t)kScanTile == tile_a) sa += sgn;
        else sb += sgn;
    }
    if (sign_sums) {   // uniform
        sa = block_sum(sa);
        sb = block_sum(sb);
        if (threadIdx.x == 0) {
            if (sa) atomicAdd(&sign_sums[tile_a], sa);
            if (sb) atomicAdd(&sign_sums[tile_a + 1], sb);
        }
    }
}

// `plan`: the scan over HeadFlag{key} (scan_totals has run); uniq = its total.  `sign_sums` (optional): an array of
// ceil(uniq / kScanTile) words that gets the sign counts of the output costs per tile.
inline rama_status reduce_runs(Ctx &ctx, const ScanPlan<uint32_t> &plan, const uint64_t *key, const uint32_t *val, int dbits,
                               int32_t *io, int32_t *jo, float *co, Buf<uint64_t> *sign_sums = nullptr)
{
    if (plan.n == 0) return RAMA_OK;
    unsigned long long *ss = nullptr;
    if (sign_sums) {
        const size_t tiles = ((size_t)plan.total + kScanTile - 1) / kScanTile;
        RAMA_TRY(sign_sums->alloc(ctx, tiles > 0 ? tiles : 1));
        RAMA_TRY(fill<uint64_t>(ctx, sign_sums->get(), 0ull, tiles > 0 ? tiles : 1));
        ss = (unsigned long long *)sign_sums->get();
    }
    {
        ProfScope ps_(ctx, "k_reduce_runs", (double)(plan.n * 12 + (size_t)plan.total * 12));
        k_reduce_runs<<<plan.nb, kBlock, 0, ctx.stream>>>(plan.n, key, val, dbits, plan.offs.get(), io, jo, co, ss);
    }
    LAUNCH_TRY(ctx, "reduce_runs");
    return RAMA_OK;
}

// position of the canonical edge (u,v), u<v, in rows given by rowptr over i (upper CSR) or -1
__device__ __forceinline__ int32_t find_edge_in_row(const int32_t *rowptr, const int32_t *j, int32_t u, int32_t v)
{
    int32_t lo = rowptr[u], hi = rowptr[u + 1];
    if (hi - lo <= 8) {
        // a short row: eight entries with two 16-byte loads (one wait instead of a chain of probes);
        // what lies behind the row's end is read but not looked at (device arrays end with slack)
        int32_t row[8];
        __builtin_memcpy(row, j + lo, sizeof(row));
        int32_t pos = -1;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (lo + k < hi && row[k] == v) pos = lo + k;
        return pos;
    }
    const int32_t end = hi;
    while (lo < hi) {
        int32_t mid = lo + ((hi - lo) >> 1);
        if (j[mid] < v) lo = mid + 1; else hi = mid;
    }
    return (lo < end && j[lo] == v) ? lo : -1;
}

}  // namespace rama
