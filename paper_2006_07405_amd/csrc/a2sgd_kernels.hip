// HIP kernels of the A2SGD step for gfx950 (CDNA4, 64-wide wavefronts).
//
// The whole path is bandwidth-bound streaming: a reduction pass over g and e (Algorithm 1 line 3) and one
// fused elementwise pass (lines 4, 6, 7).  Every global access of the two big passes is a 128-bit load or
// store, consecutive lanes touching consecutive 16-byte groups, so a wavefront moves 1 KiB per instruction.
// No matrix cores: there is no contraction anywhere in the method.
#include <type_traits>

#include "a2sgd_device.h"

namespace a2sgd {

// grid = (B, P).  Block b of worker p takes the tiles b, b + B, b + 2B, ... of that worker's vector; a tile is
// kBlock * kReduceUnroll consecutive float4 groups.  Whatever does not fill a tile is taken one float4 group
// per thread, and the last n % 4 elements one per thread, both with exact bounds: a padded lane would
// otherwise count as "v >= 0".
template <bool HAS_E, bool NT>
__global__ __launch_bounds__(kBlock) void k_local_partials(const PtrTable tab, const uint64_t n, const uint32_t B,
                                                           Partials out)
{
    const uint32_t p = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
    const float *__restrict__ g = tab.g[p];
    const float *__restrict__ e = HAS_E ? tab.e[p] : nullptr;
    const vf4 *__restrict__ g4 = reinterpret_cast<const vf4 *>(g);
    const vf4 *__restrict__ e4 = reinterpret_cast<const vf4 *>(e);

    const uint64_t nvec = n >> 2;
    constexpr uint64_t kTile = static_cast<uint64_t>(kBlock) * kReduceUnroll;
    const uint64_t ntile = nvec / kTile;

    LaneAcc acc;
    for (uint64_t t = b; t < ntile; t += B) {
        const uint64_t base = t * kTile + tid;
        vf4 gv[kReduceUnroll], ev[kReduceUnroll];
#pragma unroll
        for (int u = 0; u < kReduceUnroll; ++u)
            gv[u] = ld4<NT>(g4 + base + u * kBlock);
        if (HAS_E) {
#pragma unroll
            for (int u = 0; u < kReduceUnroll; ++u)
                ev[u] = ld4<NT>(e4 + base + u * kBlock);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep every load of the tile ahead of the first use
#pragma unroll
        for (int u = 0; u < kReduceUnroll; ++u)
            acc.add4(HAS_E ? gv[u] + ev[u] : gv[u]);
        acc.flush();
    }
    // float4 groups past the last full tile
    for (uint64_t i = ntile * kTile + static_cast<uint64_t>(b) * kBlock + tid; i < nvec;
         i += static_cast<uint64_t>(B) * kBlock) {
        vf4 v = ld4<NT>(g4 + i);
        if (HAS_E)
            v += ld4<NT>(e4 + i);
        acc.add4(v);
        acc.flush();
    }
    // last n % 4 elements
    if (b == 0 && tid < (n & 3)) {
        const uint64_t i = (nvec << 2) + tid;
        acc.add(HAS_E ? g[i] + e[i] : g[i]);
        acc.flush();
    }

    // block reduction: shuffle tree inside each wavefront (the counts are wavefront totals already), then the 4
    // wavefront results in index order
    Sums mine;
    mine.s_pos = wave_sum(acc.s_pos);
    mine.s_neg = wave_sum(acc.s_neg);
    mine.n_pos = acc.c_pos;
    mine.n_neg = acc.c_neg;
    mine.n_zero = acc.c_zero;
    const Sums total = block_sum_of_waves(mine);
    if (tid == 0)
        store_record(out, static_cast<size_t>(p) * B + b, total);
}

// Second level, one block per worker: the B block partials in a fixed order (strided per thread, shuffle
// tree, wavefronts in index order), then the two local means rounded to the fp32 that a worker would send
// (Sec. 4.3: two means, 64 bits).  An empty group has mean 0.
__global__ __launch_bounds__(kBlock) void k_local_finalize(const uint64_t n, const uint32_t B, const Partials in,
                                                           WsHeader *__restrict__ hdr)
{
    const uint32_t p = blockIdx.x, tid = threadIdx.x;
    const size_t row = static_cast<size_t>(p) * B;
    Sums mine;
    for (uint32_t j = tid; j < B; j += kBlock)
        add_record(mine, in, row + j);
    const Sums t = block_sum(mine);
    if (tid == 0) {
        a2sgd_worker_stats_t r;
        r.mu_pos = t.n_pos ? static_cast<float>(t.s_pos / static_cast<double>(t.n_pos)) : 0.0f;
        r.mu_neg = t.n_neg ? static_cast<float>(t.s_neg / static_cast<double>(t.n_neg)) : 0.0f;
        r.n_pos = t.n_pos;
        r.n_neg = t.n_neg;
        r.n_zero = t.n_zero;
        r.n_nan = n - t.n_pos - t.n_neg;
        hdr->workers[p] = r;
    }
}

// Algorithm 1 line 5 on one GPU: the 2P fp32 scalars to 2, summed p = 0..P-1 in fp64, divided by P.
__global__ void k_global_average(const uint32_t P, WsHeader *__restrict__ hdr)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double sp = 0.0, sn = 0.0;
        for (uint32_t p = 0; p < P; ++p) {
            sp += static_cast<double>(hdr->workers[p].mu_pos);
            sn += static_cast<double>(hdr->workers[p].mu_neg);
        }
        hdr->gmu_pos = static_cast<float>(sp / static_cast<double>(P));
        hdr->gmu_neg = static_cast<float>(sn / static_cast<double>(P));
        uint32_t any_nan = 0;
        for (uint32_t p = 0; p < P; ++p)
            any_nan |= hdr->workers[p].n_nan != 0 ? 1u : 0u;
        hdr->any_nan = any_nan;
    }
    // the same local means again, packed and pre-negated the way the apply pass consumes them
    for (uint32_t p = threadIdx.x; p < P && blockIdx.x == 0; p += blockDim.x) {
        hdr->neg_mu_pos[p] = -hdr->workers[p].mu_pos;
        hdr->mu_neg[p] = hdr->workers[p].mu_neg;
    }
}

// Algorithm 1 line 5 when the caller does the averaging (workers on several GPUs): the local pairs out, the global
// pair in.  The import also fills what k_global_average fills besides the global means.
__global__ void k_export_local_means(const uint32_t P, const WsHeader *__restrict__ hdr, float *__restrict__ out)
{
    for (uint32_t p = threadIdx.x; p < P && blockIdx.x == 0; p += blockDim.x) {
        out[2 * p] = hdr->workers[p].mu_pos;
        out[2 * p + 1] = hdr->workers[p].mu_neg;
    }
}

__global__ void k_import_global_means(const uint32_t P, WsHeader *__restrict__ hdr, const float *__restrict__ gmu)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        hdr->gmu_pos = gmu[0];
        hdr->gmu_neg = gmu[1];
        uint32_t any_nan = 0;
        for (uint32_t p = 0; p < P; ++p)
            any_nan |= hdr->workers[p].n_nan != 0 ? 1u : 0u;
        hdr->any_nan = any_nan;
    }
    for (uint32_t p = threadIdx.x; p < P && blockIdx.x == 0; p += blockDim.x) {
        hdr->neg_mu_pos[p] = -hdr->workers[p].mu_pos;
        hdr->mu_neg[p] = hdr->workers[p].mu_neg;
    }
}

// ---------------------------------------------------------------------------------------------------------
// Fused apply pass (Algorithm 1 lines 4, 6, 7; Eq. 2 for the encoding; Eq. 1 for the average over workers)
// ---------------------------------------------------------------------------------------------------------

// Body of the apply pass for one workgroup.  Thread t owns the float4 groups base + it * BLOCK (it < ITEMS) of
// every worker and of w.  The g and e loads of UP workers x ITEMS groups are all issued before the first use:
// the pass runs fastest with few wavefronts per compute unit, each with many loads in flight.  FULL = every
// group of the workgroup is in range (all workgroups but the last).  neg_mu_pos[p] = -mu_pos of worker p and
// mu_neg[p] are read where the caller keeps them (the workspace header, or LDS in the single-launch step).
template <int MODE, bool HAS_E, bool NT, int UP, int ITEMS, int BLOCK, bool FULL>
__device__ __forceinline__ void apply_body(const PtrTable &tab, float *__restrict__ w, const uint64_t nvec,
                                           const uint64_t base, const uint32_t P, const float eta_over_P,
                                           const float *neg_mu_pos, const float *mu_neg, const float gmu_pos,
                                           const float neg_gmu_neg)
{
    vf4 *w4 = reinterpret_cast<vf4 *>(w);
    vf4 wv[ITEMS], acc[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        acc[it] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
        if (FULL || base + it * BLOCK < nvec)
            wv[it] = ld4<NT>(w4 + base + it * BLOCK);
    }
    // One group of up to UP workers starting at p0.  With PARTIAL the group may be short: worker p0 + u takes part
    // only if it exists, a test that is uniform over the grid.
    auto group = [&](auto partial, const uint32_t p0) {
        constexpr bool PARTIAL = decltype(partial)::value;
        vf4 v[UP * ITEMS], ev[UP * ITEMS];
        float nmp[UP], mn[UP];
#pragma unroll
        for (int u = 0; u < UP; ++u)
            if (!PARTIAL || p0 + u < P) {
                nmp[u] = neg_mu_pos[p0 + u];
                mn[u] = mu_neg[p0 + u];
            }
#pragma unroll
        for (int u = 0; u < UP; ++u)
            if (!PARTIAL || p0 + u < P) {
                const vf4 *gp = reinterpret_cast<const vf4 *>(tab.g[p0 + u]);
#pragma unroll
                for (int it = 0; it < ITEMS; ++it)
                    if (FULL || base + it * BLOCK < nvec)
                        v[u * ITEMS + it] = ld4<NT>(gp + base + it * BLOCK);
            }
        if (HAS_E) {
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P) {
                    const vf4 *ep = reinterpret_cast<const vf4 *>(tab.e[p0 + u]);
#pragma unroll
                    for (int it = 0; it < ITEMS; ++it)
                        if (FULL || base + it * BLOCK < nvec)
                            ev[u * ITEMS + it] = ld4<NT>(ep + base + it * BLOCK);
                }
        }
        __builtin_amdgcn_sched_barrier(0);  // keep every load of the group ahead of the first use
#pragma unroll
        for (int u = 0; u < UP; ++u)
            if (!PARTIAL || p0 + u < P) {
                vf4 *ep = reinterpret_cast<vf4 *>(tab.e[p0 + u]);
#pragma unroll
                for (int it = 0; it < ITEMS; ++it) {
                    if (FULL || base + it * BLOCK < nvec) {
                        const vf4 vv = HAS_E ? v[u * ITEMS + it] + ev[u * ITEMS + it] : v[u * ITEMS + it];
                        const vf4 err = apply4<MODE>(vv, acc[it], nmp[u], mn[u], gmu_pos, neg_gmu_neg);
                        if (HAS_E)
                            st4<NT>(ep + base + it * BLOCK, err);
                    }
                }
            }
    };
    uint32_t p0 = 0;
    for (; p0 + UP <= P; p0 += UP)
        group(std::false_type{}, p0);
    if (UP > 1 && p0 < P)  // the workers past the last full group, in one short group
        group(std::true_type{}, p0);
#pragma unroll
    for (int it = 0; it < ITEMS; ++it)
        if (FULL || base + it * BLOCK < nvec) {
            const vf4 wn = wv[it] - eta_over_P * acc[it];
            st4<NT>(w4 + base + it * BLOCK, wn);
        }
}

// grid = ceil(ceil(n/4) / (BLOCK * ITEMS * SEQ)) workgroups, each launched once; a workgroup runs the body SEQ
// times on consecutive spans of BLOCK * ITEMS float4 groups.  The kernel uses no LDS itself: the launcher
// requests dynamic LDS only to cap how many workgroups share a compute unit.  The last workgroup's first
// n % 4 threads also take the scalar tail.
template <int MODE, bool HAS_E, bool NT, int UP, int ITEMS, int SEQ, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_apply(const PtrTable tab, float *__restrict__ w, const uint64_t n,
                                                 const uint32_t P, const float eta_over_P,
                                                 const WsHeader *__restrict__ hdr)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t lz = opaque_zero();
    const float *neg_mu_pos = hdr->neg_mu_pos + lz, *mu_neg = hdr->mu_neg + lz;
    const float gmu_pos = (&hdr->gmu_pos)[lz];  // vector loads, issued ahead of the big ones
    const float neg_gmu_neg = -(&hdr->gmu_neg)[lz];
    const uint64_t nvec = n >> 2;
    constexpr uint64_t kSpan = static_cast<uint64_t>(BLOCK) * ITEMS;
#pragma unroll
    for (int sq = 0; sq < SEQ; ++sq) {
        const uint64_t first = (static_cast<uint64_t>(blockIdx.x) * SEQ + sq) * kSpan;
        if (first + kSpan <= nvec)
            apply_body<MODE, HAS_E, NT, UP, ITEMS, BLOCK, true>(tab, w, nvec, first + tid, P, eta_over_P, neg_mu_pos,
                                                                mu_neg, gmu_pos, neg_gmu_neg);
        else if (first < nvec)
            apply_body<MODE, HAS_E, NT, UP, ITEMS, BLOCK, false>(tab, w, nvec, first + tid, P, eta_over_P, neg_mu_pos,
                                                                 mu_neg, gmu_pos, neg_gmu_neg);
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t k = (nvec << 2) + tid;
        float acc = 0.0f;
        for (uint32_t p = 0; p < P; ++p) {
            float v = tab.g[p][k];
            if (HAS_E)
                v += tab.e[p][k];
            acc += apply1<MODE>(v, hdr->neg_mu_pos[p], hdr->mu_neg[p], gmu_pos, neg_gmu_neg);
            if (HAS_E)
                tab.e[p][k] = v;
        }
        w[k] -= eta_over_P * acc;
    }
}

// ---------------------------------------------------------------------------------------------------------
// Single-launch step for models whose g, e and w fit the on-chip caches (Algorithm 1 lines 3-7 in one kernel)
// ---------------------------------------------------------------------------------------------------------

// Grid-wide barrier for the single-launch step.  The cells live in device memory that the loader zeroes, so
// neither the caller nor the plan has to allocate or initialise anything; the host hands each cell to at most one
// live plan.  It is a sense-reversing barrier: the last workgroup to arrive clears the arrival count and advances
// the generation, which leaves the cell ready for the next launch.  It is only used with grids that are resident
// all at once (no more workgroups of kFusedBlock threads than the device has compute units, checked at launch), so
// every arrival is certain; the wait is bounded all the same, and a wait that runs out marks the cell as failed:
// later launches on it exit at once and report through the workspace header instead of computing on a cell whose
// count can no longer be trusted, until the host, having seen the report, resets the cell.
struct GridBarrier {
    uint32_t arrive, generation, failed, pad;
};
static __device__ GridBarrier g_barriers[kBarrierSlots + 1];  // the last cell belongs to the self-test
constexpr uint32_t kBarrierSpinLimit = 1u << 21;  // polls of about a microsecond each

// Device-scope relaxed atomic accessors.  They go to the memory side of the chip, past the XCD's own L2, which
// is what lets workgroups on different XCDs exchange a few words without flushing or invalidating that cache.
template <class T>
__device__ __forceinline__ void store_device(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T>
__device__ __forceinline__ T load_device(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Waits until every vector-memory operation of this wavefront, stores included, has been acknowledged
// (s_waitcnt with vmcnt = 0 and the other counters left at their maxima, gfx9 encoding).
__device__ __forceinline__ void wait_vector_memory()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

// Called by every thread of every workgroup.  Returns false if the wait ran out (or the cell is marked failed).
// Only thread 0 talks to the cell.  Everything that crosses this barrier (the partial records) is written with
// store_device and read with load_device, so no cache-wide fence is needed: a device-scope fence on this chip
// writes back or invalidates the XCD's whole L2, which costs tens of microseconds when every workgroup does
// it.  What is needed is order: every wavefront waits for its record stores to be acknowledged before its
// workgroup arrives, and the records are read only after the generation was seen to move.
__device__ __forceinline__ bool grid_barrier(GridBarrier *bar, const uint32_t G, const uint32_t spin_limit)
{
    __shared__ uint32_t s_ok;
    wait_vector_memory();
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t ok = 1;
        const uint32_t gen = load_device(&bar->generation);
        const uint32_t old = __hip_atomic_fetch_add(&bar->arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == G - 1) {
            store_device(&bar->arrive, 0u);
            wait_vector_memory();  // the reset has landed before anyone is released
            __hip_atomic_fetch_add(&bar->generation, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            uint32_t polls = 0;
            while (load_device(&bar->generation) == gen) {
                if (++polls > spin_limit) {
                    store_device(&bar->failed, 1u);
                    ok = 0;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        }
        s_ok = ok;
    }
    __syncthreads();
    return s_ok != 0;
}

// Self-test of the barrier on the spare cell: every workgroup goes through one barrier that expects `expected`
// arrivals and reports whether it got through.  With expected = gridDim.x it must; with expected = gridDim.x + 1
// and a small spin limit nobody is ever last, every wait runs out, and every workgroup still exits.
__global__ __launch_bounds__(kBlock) void k_barrier_selftest(const uint32_t expected, const uint32_t spin_limit,
                                                             uint32_t *__restrict__ passed)
{
    const bool ok = grid_barrier(&g_barriers[kBarrierSlots], expected, spin_limit);
    if (threadIdx.x == 0)
        passed[blockIdx.x] = ok ? 1u : 0u;
}

// Puts a cell back into its initial state; cell_failed_out (may be null) receives its failed flag first.
__global__ void k_barrier_reset(const uint32_t cell, uint32_t *__restrict__ cell_failed_out)
{
    GridBarrier *bar = &g_barriers[cell];
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        if (cell_failed_out != nullptr)
            *cell_failed_out = load_device(&bar->failed);
        store_device(&bar->arrive, 0u);
        store_device(&bar->generation, 0u);
        store_device(&bar->failed, 0u);
    }
}

constexpr int kFusedUnroll = 4;  // float4 groups per thread per loop trip in the reduction phase
// kFusedBlock threads per workgroup (a2sgd_internal.h): large workgroups keep the number of partial records,
// which every workgroup reads back from the memory side after the barrier, small.

// grid = G workgroups, few enough to be resident all at once.  Workgroup b owns one contiguous slice of the
// float4 groups of every worker and of w in BOTH phases, so what it read for the sums is what it re-reads for
// the update, from the L2 of its own XCD.  Phase 1 writes one partial record per (worker, workgroup); after the
// grid-wide barrier every workgroup combines the G records of each worker in the same fixed order, so all of
// them hold bit-identical means without a second barrier; phase 3 is the apply pass on the slice.  Workgroup 0
// also writes the header that a2sgd_read_stats reads.  The last n % 4 elements belong to the last workgroup.
// The second launch bound asks for 4 wavefronts per SIMD, i.e. two workgroups per compute unit (at most 128 vector
// registers, which is why the workers are taken in groups of 4 at most here): the single-launch steps of two plans
// then fit the device together whatever their grids.
template <int MODE, bool HAS_E, int UP>
__global__ __launch_bounds__(kFusedBlock, 4) void k_fused_step(const PtrTable tab, float *__restrict__ w, const uint64_t n,
                                                       const uint32_t P, const float eta_over_P, const Partials part,
                                                       WsHeader *__restrict__ hdr, const uint32_t slot,
                                                       const uint32_t token)
{
    GridBarrier *bar = &g_barriers[slot];
    __shared__ uint32_t s_cell_failed;
    if (threadIdx.x == 0)
        s_cell_failed = __hip_atomic_load(&bar->failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_cell_failed != 0) {  // the same for every thread of the workgroup
        if (threadIdx.x == 0)
            hdr->failed_token = token;
        return;
    }
    __shared__ double sh_pos[kMaxWorkers][kFusedBlock / 64], sh_neg[kMaxWorkers][kFusedBlock / 64];
    __shared__ uint64_t sh_cp[kMaxWorkers][kFusedBlock / 64], sh_cn[kMaxWorkers][kFusedBlock / 64],
        sh_cz[kMaxWorkers][kFusedBlock / 64];
    __shared__ float s_neg_mu_pos[kMaxWorkers], s_mu_neg[kMaxWorkers], s_gmu[2];

    const uint32_t G = gridDim.x, b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint64_t nvec = n >> 2;
    const uint64_t q = nvec / G, r = nvec % G;
    const uint64_t lo = b * q + (b < r ? b : r), hi = lo + q + (b < r ? 1 : 0);
    const bool owns_tail = (b == G - 1) && tid < (n & 3);
    const uint64_t tail = (nvec << 2) + tid;

    // ---- phase 1: sums and counts of this slice, per worker
    for (uint32_t p = 0; p < P; ++p) {
        const float *__restrict__ g = tab.g[p];
        const float *__restrict__ e = HAS_E ? tab.e[p] : nullptr;
        const vf4 *g4 = reinterpret_cast<const vf4 *>(g), *e4 = reinterpret_cast<const vf4 *>(e);
        LaneAcc acc;
        for (uint64_t i0 = lo + tid; i0 < hi; i0 += static_cast<uint64_t>(kFusedBlock) * kFusedUnroll) {
            vf4 gv[kFusedUnroll], ev[kFusedUnroll];
#pragma unroll
            for (int u = 0; u < kFusedUnroll; ++u)
                if (i0 + u * kFusedBlock < hi) {
                    gv[u] = g4[i0 + u * kFusedBlock];
                    if (HAS_E)
                        ev[u] = e4[i0 + u * kFusedBlock];
                }
#pragma unroll
            for (int u = 0; u < kFusedUnroll; ++u)
                if (i0 + u * kFusedBlock < hi)
                    acc.add4(HAS_E ? gv[u] + ev[u] : gv[u]);
            acc.flush();
        }
        if (owns_tail) {
            acc.add(HAS_E ? g[tail] + e[tail] : g[tail]);
            acc.flush();
        }
        const double wp = wave_sum(acc.s_pos), wn = wave_sum(acc.s_neg);
        // the counts are wavefront totals held by the lanes that were active; lane 0 is active whenever any is
        if (lane == 0) {
            sh_pos[p][wave] = wp;
            sh_neg[p][wave] = wn;
            sh_cp[p][wave] = acc.c_pos;
            sh_cn[p][wave] = acc.c_neg;
            sh_cz[p][wave] = acc.c_zero;
        }
    }
    __syncthreads();
    if (tid < P) {
        double sp = 0.0, sn = 0.0;
        uint64_t cp = 0, cn = 0, cz = 0;
#pragma unroll
        for (int k = 0; k < kFusedBlock / 64; ++k) {
            sp += sh_pos[tid][k];
            sn += sh_neg[tid][k];
            cp += sh_cp[tid][k];
            cn += sh_cn[tid][k];
            cz += sh_cz[tid][k];
        }
        const size_t slot = static_cast<size_t>(tid) * G + b;
        store_device(part.s_pos + slot, sp);
        store_device(part.s_neg + slot, sn);
        store_device(part.n_pos + slot, cp);
        store_device(part.n_neg + slot, cn);
        store_device(part.n_zero + slot, cz);
    }
    if (!grid_barrier(bar, G, kBarrierSpinLimit)) {  // uniform per workgroup
        if (tid == 0)
            hdr->failed_token = token;
        return;
    }

    // ---- phase 2: every workgroup combines the G records of each worker, all in the same order: one wavefront
    // per worker (wavefront k takes workers k, k + 8, ...), records strided over its lanes, then the shuffle tree
    for (uint32_t p = wave; p < P; p += kFusedBlock / 64) {
        const size_t row = static_cast<size_t>(p) * G;
        double sp = 0.0, sn = 0.0;
        uint64_t cp = 0, cn = 0, cz = 0;
        for (uint32_t j = lane; j < G; j += 64) {
            sp += load_device(part.s_pos + row + j);
            sn += load_device(part.s_neg + row + j);
            cp += load_device(part.n_pos + row + j);
            cn += load_device(part.n_neg + row + j);
            cz += load_device(part.n_zero + row + j);
        }
        const double tp = wave_sum(sp), tn = wave_sum(sn);
        const uint64_t np = wave_sum(cp), nn = wave_sum(cn), nz = wave_sum(cz);
        if (lane == 0) {
            a2sgd_worker_stats_t st;
            st.mu_pos = np ? static_cast<float>(tp / static_cast<double>(np)) : 0.0f;
            st.mu_neg = nn ? static_cast<float>(tn / static_cast<double>(nn)) : 0.0f;
            st.n_pos = np;
            st.n_neg = nn;
            st.n_zero = nz;
            st.n_nan = n - np - nn;
            s_neg_mu_pos[p] = -st.mu_pos;
            s_mu_neg[p] = st.mu_neg;
            if (b == 0) {
                hdr->workers[p] = st;
                hdr->neg_mu_pos[p] = -st.mu_pos;
                hdr->mu_neg[p] = st.mu_neg;
            }
        }
    }
    __syncthreads();
    if (tid == 0) {  // Algorithm 1 line 5
        double sp = 0.0, sn = 0.0;
        for (uint32_t p = 0; p < P; ++p) {
            sp -= static_cast<double>(s_neg_mu_pos[p]);
            sn += static_cast<double>(s_mu_neg[p]);
        }
        s_gmu[0] = static_cast<float>(sp / static_cast<double>(P));
        s_gmu[1] = static_cast<float>(sn / static_cast<double>(P));
        if (b == 0) {
            hdr->gmu_pos = s_gmu[0];
            hdr->gmu_neg = s_gmu[1];
        }
    }
    __syncthreads();
    const float gmu_pos = s_gmu[0], neg_gmu_neg = -s_gmu[1];

    // ---- phase 3: error write-back and weight update on the same slice (bounds: hi instead of nvec)
    static_assert(UP <= 4, "groups of 8 workers would need more than 128 vector registers");
    for (uint64_t i = lo + tid; i < hi; i += 2 * kFusedBlock)
        apply_body<MODE, HAS_E, false, UP, 2, kFusedBlock, false>(tab, w, hi, i, P, eta_over_P, s_neg_mu_pos, s_mu_neg,
                                                             gmu_pos, neg_gmu_neg);
    if (owns_tail) {
        float acc = 0.0f;
        for (uint32_t p = 0; p < P; ++p) {
            float v = tab.g[p][tail];
            if (HAS_E)
                v += tab.e[p][tail];
            acc += apply1<MODE>(v, s_neg_mu_pos[p], s_mu_neg[p], gmu_pos, neg_gmu_neg);
            if (HAS_E)
                tab.e[p][tail] = v;
        }
        w[tail] -= eta_over_P * acc;
    }
}

// The single-launch step on a plan with tensors (one pair of means per worker and tensor): Algorithm 1 lines 3-7 in
// one kernel for models that stay in the caches, such as the paper's own FNN-3, ResNet-20 and VGG-16 (Table 1) with a
// per-layer hook.  The unit of work is an item of at most kFusedItemElems elements inside one tensor; workgroup b owns
// a contiguous run of items in all phases, so what it read for the sums it re-reads for the update from its own
// XCD's L2.  Phase 1: one partial record per (worker, item).  Barrier.  Phase 2: the tensors are dealt out to the
// wavefronts of the whole grid; a wavefront combines, worker by worker, the records of its tensor's items in a fixed
// order, rounds the two local means, and averages them over the workers (line 5); means and global means go to the
// tables of the three-pass form, the statistics to where a2sgd_read_segment_stats reads them.  Barrier.  Phase 3:
// the apply body on every item with the means of its tensor; an item starts and ends anywhere, so the elements
// before its first and after its last 16-byte boundary go one per thread.  Everything that crosses a barrier is
// written and read with device-scope accesses, as in k_fused_step.
template <int MODE, bool HAS_E, int UP>
__global__ __launch_bounds__(kFusedBlock, 4) void k_seg_fused_step(const PtrTable tab, float *__restrict__ w, const uint32_t P,
                                                                const float eta_over_P, const SegView sv,
                                                                const FusedSegView fv, const uint32_t slot,
                                                                const uint32_t token)
{
    GridBarrier *bar = &g_barriers[slot];
    WsHeader *hdr = sv.hdr;
    __shared__ uint32_t s_stop;
    if (threadIdx.x == 0) {
        const uint32_t cell_failed = __hip_atomic_load(&bar->failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cell_failed != 0)
            hdr->failed_token = token;
        s_stop = cell_failed;
    }
    __syncthreads();
    // both tests give the same answer in every workgroup of the grid, so either all go on to the barrier or none
    if (s_stop != 0 || !seg_tables_ok(sv))
        return;
    __shared__ double sh_pos[kMaxWorkers][kFusedBlock / 64], sh_neg[kMaxWorkers][kFusedBlock / 64];
    __shared__ uint64_t sh_cp[kMaxWorkers][kFusedBlock / 64], sh_cn[kMaxWorkers][kFusedBlock / 64],
        sh_cz[kMaxWorkers][kFusedBlock / 64];
    __shared__ float s_neg_mu_pos[kMaxWorkers], s_mu_neg[kMaxWorkers], s_gmu[2];

    const uint32_t G = gridDim.x, b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t q = fv.num_items / G, r = fv.num_items % G;
    const uint32_t it_lo = b * q + (b < r ? b : r), it_hi = it_lo + q + (b < r ? 1 : 0);

    // ---- phase 1
    for (uint32_t it = it_lo; it < it_hi; ++it) {
        const SegItem item = fv.item[it];
        const uint64_t lo = item.start, hi = item.start + item.count;
        uint64_t a = (lo + 3) & ~static_cast<uint64_t>(3);
        if (a > hi)
            a = hi;
        const uint64_t z = a + ((hi - a) & ~static_cast<uint64_t>(3));
        const uint64_t v_lo = a >> 2, v_hi = z >> 2;
        for (uint32_t p = 0; p < P; ++p) {
            const float *__restrict__ g = tab.g[p];
            const float *__restrict__ e = HAS_E ? tab.e[p] : nullptr;
            const vf4 *g4 = reinterpret_cast<const vf4 *>(g), *e4 = reinterpret_cast<const vf4 *>(e);
            LaneAcc acc;
            if (tid < a - lo) {
                acc.add(HAS_E ? g[lo + tid] + e[lo + tid] : g[lo + tid]);
                acc.flush();
            }
            for (uint64_t i = v_lo + tid; i < v_hi; i += kFusedBlock) {
                acc.add4(HAS_E ? g4[i] + e4[i] : g4[i]);
                acc.flush();
            }
            if (tid < hi - z) {
                acc.add(HAS_E ? g[z + tid] + e[z + tid] : g[z + tid]);
                acc.flush();
            }
            const double wp = wave_sum(acc.s_pos), wn = wave_sum(acc.s_neg);
            if (lane == 0) {
                sh_pos[p][wave] = wp;
                sh_neg[p][wave] = wn;
                sh_cp[p][wave] = acc.c_pos;
                sh_cn[p][wave] = acc.c_neg;
                sh_cz[p][wave] = acc.c_zero;
            }
        }
        __syncthreads();
        if (tid < P) {
            double sp = 0.0, sn = 0.0;
            uint64_t cp = 0, cn = 0, cz = 0;
#pragma unroll
            for (int k = 0; k < kFusedBlock / 64; ++k) {
                sp += sh_pos[tid][k];
                sn += sh_neg[tid][k];
                cp += sh_cp[tid][k];
                cn += sh_cn[tid][k];
                cz += sh_cz[tid][k];
            }
            const size_t rec = static_cast<size_t>(tid) * fv.num_items + it;
            store_device(fv.r_spos + rec, sp);
            store_device(fv.r_sneg + rec, sn);
            store_device(fv.r_npos + rec, cp);
            store_device(fv.r_nneg + rec, cn);
            store_device(fv.r_nzero + rec, cz);
        }
        __syncthreads();  // the LDS slots are free again for the next item
    }
    if (!grid_barrier(bar, G, kBarrierSpinLimit)) {
        if (tid == 0)
            hdr->failed_token = token;
        return;
    }

    // ---- phase 2: one wavefront per tensor
    for (uint32_t s = b * (kFusedBlock / 64) + wave; s < sv.S; s += G * (kFusedBlock / 64)) {
        const uint32_t lo = fv.item_lo[s], hi = fv.item_lo[s + 1];
        const uint64_t len = sv.seg_end[s] - sv.seg_start[s];
        double gp = 0.0, gn = 0.0;  // sums of the workers' means, lane 0
        for (uint32_t p = 0; p < P; ++p) {
            const size_t row = static_cast<size_t>(p) * fv.num_items;
            double sp = 0.0, sn = 0.0;
            uint64_t cp = 0, cn = 0, cz = 0;
            for (uint32_t j = lo + lane; j < hi; j += 64) {
                sp += load_device(fv.r_spos + row + j);
                sn += load_device(fv.r_sneg + row + j);
                cp += load_device(fv.r_npos + row + j);
                cn += load_device(fv.r_nneg + row + j);
                cz += load_device(fv.r_nzero + row + j);
            }
            sp = wave_sum(sp);
            sn = wave_sum(sn);
            cp = wave_sum(cp);
            cn = wave_sum(cn);
            cz = wave_sum(cz);
            if (lane == 0) {
                a2sgd_worker_stats_t st;
                st.mu_pos = cp ? static_cast<float>(sp / static_cast<double>(cp)) : 0.0f;
                st.mu_neg = cn ? static_cast<float>(sn / static_cast<double>(cn)) : 0.0f;
                st.n_pos = cp;
                st.n_neg = cn;
                st.n_zero = cz;
                st.n_nan = len - cp - cn;
                sv.stats[static_cast<size_t>(p) * sv.S + s] = st;
                store_device(sv.neg_mu_pos + static_cast<size_t>(s) * P + p, -st.mu_pos);
                store_device(sv.mu_neg + static_cast<size_t>(s) * P + p, st.mu_neg);
                gp += static_cast<double>(st.mu_pos);
                gn += static_cast<double>(st.mu_neg);
            }
        }
        if (lane == 0) {  // Algorithm 1 line 5 for this tensor
            store_device(sv.gmu + 2 * s, static_cast<float>(gp / static_cast<double>(P)));
            store_device(sv.gmu + 2 * s + 1, -static_cast<float>(gn / static_cast<double>(P)));
        }
    }
    if (!grid_barrier(bar, G, kBarrierSpinLimit)) {
        if (tid == 0)
            hdr->failed_token = token;
        return;
    }

    // ---- phase 3
    for (uint32_t it = it_lo; it < it_hi; ++it) {
        const SegItem item = fv.item[it];
        const uint32_t s = item.seg;
        if (tid < P) {
            s_neg_mu_pos[tid] = load_device(sv.neg_mu_pos + static_cast<size_t>(s) * P + tid);
            s_mu_neg[tid] = load_device(sv.mu_neg + static_cast<size_t>(s) * P + tid);
        }
        if (tid < 2)
            s_gmu[tid] = load_device(sv.gmu + 2 * s + tid);
        __syncthreads();
        const float gmu_pos = s_gmu[0], neg_gmu_neg = s_gmu[1];
        const uint64_t lo = item.start, hi = item.start + item.count;
        uint64_t a = (lo + 3) & ~static_cast<uint64_t>(3);
        if (a > hi)
            a = hi;
        const uint64_t z = a + ((hi - a) & ~static_cast<uint64_t>(3));
        auto scalar = [&](const uint64_t k) {  // lines 4, 6, 7 on one element outside the float4 groups
            float acc = 0.0f;
            for (uint32_t p = 0; p < P; ++p) {
                float v = tab.g[p][k];
                if (HAS_E)
                    v += tab.e[p][k];
                acc += apply1<MODE>(v, s_neg_mu_pos[p], s_mu_neg[p], gmu_pos, neg_gmu_neg);
                if (HAS_E)
                    tab.e[p][k] = v;
            }
            w[k] -= eta_over_P * acc;
        };
        if (tid < a - lo)
            scalar(lo + tid);
        // an item has at most kFusedItemElems / 4 float4 groups: two per thread
        static_assert(kFusedItemElems == 2 * 4 * kFusedBlock, "apply_body covers an item with ITEMS = 2");
        static_assert(UP <= 4, "groups of 8 workers would need more than 128 vector registers");
        if ((a >> 2) + tid < (z >> 2))
            apply_body<MODE, HAS_E, false, UP, 2, kFusedBlock, false>(tab, w, z >> 2, (a >> 2) + tid, P, eta_over_P,
                                                                     s_neg_mu_pos, s_mu_neg, gmu_pos, neg_gmu_neg);
        if (tid < hi - z)
            scalar(z + tid);
        __syncthreads();  // the means in LDS may be replaced
    }
}

// Eq. 1 / Algorithm 1 lines 9-10: w <- w - eta * mean_p g^p.  Same shape as the apply pass: single-wavefront
// workgroups launched once each, thread t owning ITEMS float4 groups of w and of every worker, the loads of UP
// workers issued together, residency capped by the launcher's dynamic-LDS request.
template <bool NT, int UP, int ITEMS, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_dense_step(const PtrTable tab, float *__restrict__ w, const uint64_t n,
                                                      const uint32_t P, const float eta_over_P)
{
    const uint32_t tid = threadIdx.x;
    const uint64_t nvec = n >> 2;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * (BLOCK * ITEMS) + tid;
    vf4 *w4 = reinterpret_cast<vf4 *>(w);
    vf4 wv[ITEMS], acc[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        acc[it] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
        if (base + it * BLOCK < nvec)
            wv[it] = ld4<NT>(w4 + base + it * BLOCK);
    }
    auto group = [&](auto partial, const uint32_t p0) {  // up to UP workers; PARTIAL: the last, short group
        constexpr bool PARTIAL = decltype(partial)::value;
        vf4 v[UP * ITEMS];
#pragma unroll
        for (int u = 0; u < UP; ++u)
            if (!PARTIAL || p0 + u < P)
#pragma unroll
                for (int it = 0; it < ITEMS; ++it)
                    if (base + it * BLOCK < nvec)
                        v[u * ITEMS + it] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.g[p0 + u]) + base + it * BLOCK);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < UP; ++u)
            if (!PARTIAL || p0 + u < P)
#pragma unroll
                for (int it = 0; it < ITEMS; ++it)
                    if (base + it * BLOCK < nvec)
                        acc[it] += v[u * ITEMS + it];
    };
    uint32_t p0 = 0;
    for (; p0 + UP <= P; p0 += UP)
        group(std::false_type{}, p0);
    if (UP > 1 && p0 < P)
        group(std::true_type{}, p0);
#pragma unroll
    for (int it = 0; it < ITEMS; ++it)
        if (base + it * BLOCK < nvec) {
            const vf4 wn = wv[it] - eta_over_P * acc[it];
            st4<NT>(w4 + base + it * BLOCK, wn);
        }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t k = (nvec << 2) + tid;
        float a = 0.0f;
        for (uint32_t p = 0; p < P; ++p)
            a += tab.g[p][k];
        w[k] -= eta_over_P * a;
    }
}

// ---------------------------------------------------------------------------------------------------------
// One weight vector per worker (Algorithm 1 line 7 as printed), the replica form of the final synchronisation
// (lines 9-10), and the replica-drift diagnostic
// ---------------------------------------------------------------------------------------------------------

// Same shape as k_apply with one float4 group per thread; per worker it also loads and stores that worker's
// own weights, w^p <- w^p - eta * u^p, and nothing is summed over the workers.
template <int MODE, bool HAS_E, bool NT, int UP, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_apply_replicas(const PtrTable tab, const ReplicaTable wt, const uint64_t n,
                                                          const uint32_t P, const float eta,
                                                          const WsHeader *__restrict__ hdr)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t lz = opaque_zero();
    const float *neg_mu_pos = hdr->neg_mu_pos + lz, *mu_neg = hdr->mu_neg + lz;
    const float gmu_pos = (&hdr->gmu_pos)[lz];
    const float neg_gmu_neg = -(&hdr->gmu_neg)[lz];
    const uint64_t nvec = n >> 2;
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * BLOCK + tid;
    if (i < nvec) {
        auto group = [&](auto partial, const uint32_t p0) {  // up to UP workers; PARTIAL: the last, short group
            constexpr bool PARTIAL = decltype(partial)::value;
            vf4 v[UP], ev[UP], wv[UP];
            float nmp[UP], mn[UP];
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P) {
                    nmp[u] = neg_mu_pos[p0 + u];
                    mn[u] = mu_neg[p0 + u];
                }
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P)
                    v[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.g[p0 + u]) + i);
            if (HAS_E) {
#pragma unroll
                for (int u = 0; u < UP; ++u)
                    if (!PARTIAL || p0 + u < P)
                        ev[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.e[p0 + u]) + i);
            }
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P)
                    wv[u] = ld4<NT>(reinterpret_cast<const vf4 *>(wt.w[p0 + u]) + i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P) {
                    const vf4 vv = HAS_E ? v[u] + ev[u] : v[u];
                    vf4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
                    const vf4 err = apply4<MODE>(vv, upd, nmp[u], mn[u], gmu_pos, neg_gmu_neg);
                    if (HAS_E)
                        st4<NT>(reinterpret_cast<vf4 *>(tab.e[p0 + u]) + i, err);
                    const vf4 wn = wv[u] - eta * upd;
                    st4<NT>(reinterpret_cast<vf4 *>(wt.w[p0 + u]) + i, wn);
                }
        };
        uint32_t p0 = 0;
        for (; p0 + UP <= P; p0 += UP)
            group(std::false_type{}, p0);
        if (UP > 1 && p0 < P)
            group(std::true_type{}, p0);
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t k = (nvec << 2) + tid;
        for (uint32_t p = 0; p < P; ++p) {
            float v = tab.g[p][k];
            if (HAS_E)
                v += tab.e[p][k];
            const float u = apply1<MODE>(v, neg_mu_pos[p], mu_neg[p], gmu_pos, neg_gmu_neg);
            if (HAS_E)
                tab.e[p][k] = v;
            wt.w[p][k] -= eta * u;
        }
    }
}

// The same pass with one worker per workgroup: grid = (workgroups of 64 * ITEMS float4 groups, P).  Nothing is summed
// over the workers here, so a workgroup needs only its own worker's three buffers (g^p, e^p, w^p), and the
// workgroups that run at one time are on the same worker or two: with many workers the grouped form above loses to
// address translation what this one does not (as the shared-weight apply pass does from 8 workers on).  Single
// wavefronts launched once, ITEMS groups of each buffer per thread, all loads ahead of the first store.
template <int MODE, bool HAS_E, bool NT, int ITEMS>
__global__ __launch_bounds__(64) void k_apply_replicas_per_worker(const PtrTable tab, const ReplicaTable wt,
                                                                  const uint64_t n, const float eta,
                                                                  const WsHeader *__restrict__ hdr)
{
    const uint32_t p = blockIdx.y, tid = threadIdx.x;
    const uint32_t lz = opaque_zero();
    const float nmp = hdr->neg_mu_pos[p + lz], mn = hdr->mu_neg[p + lz];
    const float gmu_pos = (&hdr->gmu_pos)[lz];
    const float neg_gmu_neg = -(&hdr->gmu_neg)[lz];
    const vf4 *__restrict__ g4 = reinterpret_cast<const vf4 *>(tab.g[p]);
    vf4 *e4 = HAS_E ? reinterpret_cast<vf4 *>(tab.e[p]) : nullptr;
    vf4 *w4 = reinterpret_cast<vf4 *>(wt.w[p]);
    const uint64_t nvec = n >> 2;
    constexpr uint64_t kPer = 64ull * ITEMS;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * kPer + tid;
    if ((static_cast<uint64_t>(blockIdx.x) + 1) * kPer <= nvec) {
        vf4 v[ITEMS], ev[ITEMS], wv[ITEMS];
#pragma unroll
        for (int u = 0; u < ITEMS; ++u)
            v[u] = ld4<NT>(g4 + base + u * 64);
        if (HAS_E) {
#pragma unroll
            for (int u = 0; u < ITEMS; ++u)
                ev[u] = ld4<NT>(e4 + base + u * 64);
        }
#pragma unroll
        for (int u = 0; u < ITEMS; ++u)
            wv[u] = ld4<NT>(w4 + base + u * 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const vf4 vv = HAS_E ? v[u] + ev[u] : v[u];
            vf4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
            const vf4 err = apply4<MODE>(vv, upd, nmp, mn, gmu_pos, neg_gmu_neg);
            if (HAS_E)
                st4<NT>(e4 + base + u * 64, err);
            const vf4 wn = wv[u] - eta * upd;
            st4<NT>(w4 + base + u * 64, wn);
        }
    } else {
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const uint64_t i = base + static_cast<uint64_t>(u) * 64;
            if (i < nvec) {
                vf4 vv = ld4<NT>(g4 + i);
                if (HAS_E)
                    vv += ld4<NT>(e4 + i);
                const vf4 wv = ld4<NT>(w4 + i);
                vf4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
                const vf4 err = apply4<MODE>(vv, upd, nmp, mn, gmu_pos, neg_gmu_neg);
                if (HAS_E)
                    st4<NT>(e4 + i, err);
                const vf4 wn = wv - eta * upd;
                st4<NT>(w4 + i, wn);
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t k = (nvec << 2) + tid;
        float v = tab.g[p][k];
        if (HAS_E)
            v += tab.e[p][k];
        const float u = apply1<MODE>(v, nmp, mn, gmu_pos, neg_gmu_neg);
        if (HAS_E)
            tab.e[p][k] = v;
        wt.w[p][k] -= eta * u;
    }
}

// Algorithm 1 lines 9-10 on replicas: the dense average of the gradients, applied to every w^p.
template <bool NT, int UP, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_dense_step_replicas(const PtrTable tab, const ReplicaTable wt,
                                                               const uint64_t n, const uint32_t P,
                                                               const float eta_over_P)
{
    const uint32_t tid = threadIdx.x;
    const uint64_t nvec = n >> 2;
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * BLOCK + tid;
    if (i < nvec) {
        vf4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        vf4 step;
        auto sum_group = [&](auto partial, const uint32_t p0) {  // up to UP workers; PARTIAL: the last, short group
            constexpr bool PARTIAL = decltype(partial)::value;
            vf4 v[UP];
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P)
                    v[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.g[p0 + u]) + i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P)
                    acc += v[u];
        };
        auto update_group = [&](auto partial, const uint32_t p0) {
            constexpr bool PARTIAL = decltype(partial)::value;
            vf4 wv[UP];
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P)
                    wv[u] = ld4<NT>(reinterpret_cast<const vf4 *>(wt.w[p0 + u]) + i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P) {
                    const vf4 wn = wv[u] - step;
                    st4<NT>(reinterpret_cast<vf4 *>(wt.w[p0 + u]) + i, wn);
                }
        };
        uint32_t p0 = 0;
        for (; p0 + UP <= P; p0 += UP)
            sum_group(std::false_type{}, p0);
        if (UP > 1 && p0 < P)
            sum_group(std::true_type{}, p0);
        step = eta_over_P * acc;
        for (p0 = 0; p0 + UP <= P; p0 += UP)
            update_group(std::false_type{}, p0);
        if (UP > 1 && p0 < P)
            update_group(std::true_type{}, p0);
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t k = (nvec << 2) + tid;
        float a = 0.0f;
        for (uint32_t p = 0; p < P; ++p)
            a += tab.g[p][k];
        for (uint32_t p = 0; p < P; ++p)
            wt.w[p][k] -= eta_over_P * a;
    }
}

// Replica drift, first level.  grid = (kDriftBlocks, P): block (b, p) strides over the elements and, for each,
// forms the mean over all replicas in fp64 (p ascending) and worker p's deviation from it; the P blocks with
// the same b read the same data, which the L2 serves.  Per block: max |deviation| and the fp64 sum of squares.
__global__ __launch_bounds__(kBlock) void k_replica_drift(const ReplicaTable wt, const uint64_t n, const uint32_t P,
                                                          double *__restrict__ max_part, double *__restrict__ sq_part)
{
    const uint32_t p = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
    double mx = 0.0, sq = 0.0;
    for (uint64_t i = static_cast<uint64_t>(b) * kBlock + tid; i < n; i += static_cast<uint64_t>(gridDim.x) * kBlock) {
        double s = 0.0;
        for (uint32_t q = 0; q < P; ++q)
            s += static_cast<double>(wt.w[q][i]);
        const double d = static_cast<double>(wt.w[p][i]) - s / static_cast<double>(P);
        const double a = fabs(d);
        mx = (a > mx || a != a) ? a : mx;
        sq += d * d;
    }
    __shared__ double sh_mx[kBlock / 64], sh_sq[kBlock / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double o = __shfl_down(mx, off);
        mx = (o > mx || o != o) ? o : mx;
    }
    sq = wave_sum(sq);
    if ((tid & 63) == 0) {
        sh_mx[tid >> 6] = mx;
        sh_sq[tid >> 6] = sq;
    }
    __syncthreads();
    if (tid == 0) {
        double m = 0.0, t = 0.0;
#pragma unroll
        for (int k = 0; k < kBlock / 64; ++k) {
            m = (sh_mx[k] > m || sh_mx[k] != sh_mx[k]) ? sh_mx[k] : m;
            t += sh_sq[k];
        }
        max_part[static_cast<size_t>(p) * gridDim.x + b] = m;
        sq_part[static_cast<size_t>(p) * gridDim.x + b] = t;
    }
}

// Second level: one thread per worker walks that worker's records in index order.
__global__ void k_replica_drift_finalize(const uint64_t n, const uint32_t P, const uint32_t B,
                                         const double *__restrict__ max_part, const double *__restrict__ sq_part,
                                         double *__restrict__ result)
{
    const uint32_t p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < P) {
        double m = 0.0, t = 0.0;
        for (uint32_t j = 0; j < B; ++j) {
            const double x = max_part[static_cast<size_t>(p) * B + j];
            m = (x > m || x != x) ? x : m;
            t += sq_part[static_cast<size_t>(p) * B + j];
        }
        result[p] = m;
        result[P + p] = sqrt(t / static_cast<double>(n));
    }
}

// ---------------------------------------------------------------------------------------------------------
// Lazy error state: the buffer keeps the folded vector v of the last step, the header keeps that step's local
// means, and e = v - enc(v) (Eq. 2, Algorithm 1 line 4) is formed when the buffer is next read
// ---------------------------------------------------------------------------------------------------------

// Reduction pass on the lazy state: each element is e = pending error of the stored value, v = fl32(g + e); v is
// written back in place of the stored value and enters the sums and counts.  tab.e holds the state buffers.
// 8 bytes read and 4 written per element-worker.  Because it stores, it has the shape of the apply pass and not of
// k_local_partials: grid = (blocks, P) of single-wavefront workgroups launched once, each with kLazyItems float4
// groups per thread, all loads issued before the first store (a loop would wait for its own older stores before
// it could use newer loads, since both are counted together).  Every workgroup writes one record; the records
// of a worker are combined in index order by k_fold_partials and k_local_finalize.
// With SIGNS the pass also leaves pos(v) of Eq. 2 as one bit per element for the apply pass: thread `tid` of
// workgroup b collects 32 bits, bit 31 - (4 * u + c) for component c of its float4 group u (0 where the group lies
// past the end), and writes them as two 16-bit halves, sign[b][h][p][tid] (h = 0: groups 0-3), so that a
// workgroup of the apply pass, which covers half of the groups, reads 128 contiguous bytes per worker, and all
// workers' bytes next to each other.
template <bool NT, bool SIGNS>
__global__ __launch_bounds__(64) void k_lazy_partials(const PtrTable tab, const uint64_t n, const uint32_t blocks,
                                                      const WsHeader *__restrict__ hdr, Partials out,
                                                      uint16_t *__restrict__ sign)
{
    static_assert(4 * kLazyItems == 32, "one thread's sign bits fill two 16-bit halves");
    const uint32_t p = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
    const uint32_t lz = opaque_zero();
    // the means of the step that stored the values
    const float nmp = hdr->neg_mu_pos[p + lz], mn = hdr->mu_neg[p + lz];
    const float *__restrict__ g = tab.g[p];
    float *s = tab.e[p];
    const vf4 *__restrict__ g4 = reinterpret_cast<const vf4 *>(g);
    vf4 *s4 = reinterpret_cast<vf4 *>(s);
    const uint64_t nvec = n >> 2;
    constexpr uint64_t kPer = 64ull * kLazyItems;
    const uint64_t base = static_cast<uint64_t>(b) * kPer + tid;

    LaneAcc acc;
    uint32_t bits = 0;
    if ((static_cast<uint64_t>(b) + 1) * kPer <= nvec) {
        vf4 gv[kLazyItems], sv[kLazyItems];
#pragma unroll
        for (int u = 0; u < kLazyItems; ++u)
            gv[u] = ld4<NT>(g4 + base + u * 64);
#pragma unroll
        for (int u = 0; u < kLazyItems; ++u)
            sv[u] = ld4<NT>(s4 + base + u * 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kLazyItems; ++u) {
            const vf4 v = gv[u] + pending_error4(sv[u], nmp, mn);
            st4<NT>(s4 + base + u * 64, v);
            acc.add4(v);
            if (SIGNS)
                bits = push_signs(bits, v);
        }
    } else {
#pragma unroll
        for (int u = 0; u < kLazyItems; ++u) {
            const uint64_t i = base + static_cast<uint64_t>(u) * 64;
            if (i < nvec) {
                const vf4 v = ld4<NT>(g4 + i) + pending_error4(ld4<NT>(s4 + i), nmp, mn);
                st4<NT>(s4 + i, v);
                acc.add4(v);
                if (SIGNS)
                    bits = push_signs(bits, v);
            } else {
                bits <<= 4;
            }
        }
    }
    if (SIGNS) {
        sign_row(sign, gridDim.y, b, 0, p)[tid] = static_cast<uint16_t>(bits >> 16);
        sign_row(sign, gridDim.y, b, 1, p)[tid] = static_cast<uint16_t>(bits & 0xffffu);
    }
    if (b == 0 && tid < (n & 3)) {
        const uint64_t i = (nvec << 2) + tid;
        const float v = g[i] + pending_error(s[i], nmp, mn);
        s[i] = v;
        acc.add(v);
    }
    acc.flush();

    const double wp = wave_sum(acc.s_pos), wn = wave_sum(acc.s_neg);
    if (tid == 0) {
        const size_t slot = static_cast<size_t>(p) * blocks + b;
        out.s_pos[slot] = wp;
        out.s_neg[slot] = wn;
        out.n_pos[slot] = acc.c_pos;
        out.n_neg[slot] = acc.c_neg;
        out.n_zero[slot] = acc.c_zero;
    }
}

// First half of the apply pass in its two-kernel form (retained-error mode, many workers).  In that mode the update
// of parameter i depends only on how many workers have i in the positive group, so the pass over g and e need not
// touch w at all: workgroup (x, p) rewrites 1024 elements of worker p's error (Algorithm 1 line 4, Eq. 2) and leaves
// pos(v) in the sign words, in k_lazy_partials' layout (one half of a row per workgroup); k_apply_signs then updates
// w from the sign words alone.  A workgroup has 3 buffers open instead of 2P + 1, and all workgroups that run at one
// time are on the same worker or two: what the single kernel loses to address translation as P grows is not lost
// here.  Single wavefronts launched once, ITEMS float4 groups of g and of e per thread, all loads ahead of the first
// store.  The last n % 4 elements are left to k_apply_signs.
template <bool NT, int ITEMS>
__global__ __launch_bounds__(64) void k_error_signs(const PtrTable tab, const uint64_t n,
                                                    const WsHeader *__restrict__ hdr, uint16_t *__restrict__ sign)
{
    static_assert(ITEMS == kLazyItems || 2 * ITEMS == kLazyItems, "a workgroup fills both halves of a sign row or one");
    constexpr uint32_t kParts = kLazyItems / ITEMS;
    const uint32_t p = blockIdx.y, tid = threadIdx.x;
    const uint32_t b = blockIdx.x / kParts, h = blockIdx.x % kParts;  // sign row, and which half of it
    const uint32_t lz = opaque_zero();
    const float nmp = hdr->neg_mu_pos[p + lz], mn = hdr->mu_neg[p + lz];
    const vf4 *__restrict__ g4 = reinterpret_cast<const vf4 *>(tab.g[p]);
    vf4 *e4 = reinterpret_cast<vf4 *>(tab.e[p]);
    const uint64_t nvec = n >> 2;
    constexpr uint64_t kPer = 64ull * ITEMS;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * kPer + tid;
    uint32_t bits = 0;
    if ((static_cast<uint64_t>(blockIdx.x) + 1) * kPer <= nvec) {
        vf4 gv[ITEMS], ev[ITEMS];
#pragma unroll
        for (int u = 0; u < ITEMS; ++u)
            gv[u] = ld4<NT>(g4 + base + u * 64);
#pragma unroll
        for (int u = 0; u < ITEMS; ++u)
            ev[u] = ld4<NT>(e4 + base + u * 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const vf4 v = gv[u] + ev[u];
            bits = push_signs(bits, v);
            const vf4 err = pending_error4(v, nmp, mn);  // v - enc(v)
            st4<NT>(e4 + base + u * 64, err);
        }
    } else {
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const uint64_t i = base + static_cast<uint64_t>(u) * 64;
            if (i < nvec) {
                const vf4 v = ld4<NT>(g4 + i) + ld4<NT>(e4 + i);
                bits = push_signs(bits, v);
                const vf4 err = pending_error4(v, nmp, mn);
                st4<NT>(e4 + i, err);
            } else {
                bits <<= 4;
            }
        }
    }
    if (kParts == 1) {
        sign_row(sign, gridDim.y, b, 0, p)[tid] = static_cast<uint16_t>(bits >> 16);
        sign_row(sign, gridDim.y, b, 1, p)[tid] = static_cast<uint16_t>(bits & 0xffffu);
    } else {
        sign_row(sign, gridDim.y, b, h, p)[tid] = static_cast<uint16_t>(bits);  // 4 groups of 4 bits
    }
}

// Between the one-shot reduction and k_local_finalize: workgroup (j, p) adds the records
// [j * kFoldSpan, (j + 1) * kFoldSpan) of worker p in a fixed order (strided per thread, shuffle tree, wavefronts
// in index order) into record j of the folded table.
__global__ __launch_bounds__(kBlock) void k_fold_partials(const uint32_t rows, const Partials in, const uint32_t folded,
                                                          Partials out)
{
    const uint32_t p = blockIdx.y, j = blockIdx.x, tid = threadIdx.x;
    const size_t row = static_cast<size_t>(p) * rows;
    const uint32_t lo = j * kFoldSpan, hi = rows - lo < kFoldSpan ? rows : lo + kFoldSpan;
    Sums mine;
    for (uint32_t k = lo + tid; k < hi; k += kBlock)
        add_record(mine, in, row + k);
    const Sums total = block_sum(mine);
    if (tid == 0)
        store_record(out, static_cast<size_t>(p) * folded + j, total);
}

// Apply pass on the lazy state: the buffers already hold v, so all that is left of Algorithm 1 lines 6-7 is to
// read each worker's v for its sign group (and, in literal mode, its error) and update w.  Shape of k_apply:
// single-wavefront workgroups launched once, one float4 group per thread, UP workers' loads issued together.
template <int MODE, bool NT, int UP, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_lazy_apply(const PtrTable tab, float *__restrict__ w, const uint64_t n,
                                                      const uint32_t P, const float eta_over_P,
                                                      const WsHeader *__restrict__ hdr)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t lz = opaque_zero();
    const float *neg_mu_pos = hdr->neg_mu_pos + lz, *mu_neg = hdr->mu_neg + lz;
    const float gmu_pos = (&hdr->gmu_pos)[lz];
    const float neg_gmu_neg = -(&hdr->gmu_neg)[lz];
    const uint64_t nvec = n >> 2;
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * BLOCK + tid;
    if (i < nvec) {
        vf4 *w4 = reinterpret_cast<vf4 *>(w) + i;
        const vf4 wv = ld4<NT>(w4);
        vf4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        auto group = [&](auto partial, const uint32_t p0) {  // up to UP workers; PARTIAL: the last, short group
            constexpr bool PARTIAL = decltype(partial)::value;
            vf4 v[UP];
            float nmp[UP], mn[UP];
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P) {
                    nmp[u] = neg_mu_pos[p0 + u];
                    mn[u] = mu_neg[p0 + u];
                }
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P)
                    v[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.e[p0 + u]) + i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (!PARTIAL || p0 + u < P)
                    (void)apply4<MODE>(v[u], acc, nmp[u], mn[u], gmu_pos, neg_gmu_neg);
        };
        uint32_t p0 = 0;
        for (; p0 + UP <= P; p0 += UP)
            group(std::false_type{}, p0);
        if (UP > 1 && p0 < P)
            group(std::true_type{}, p0);
        const vf4 wn = wv - eta_over_P * acc;
        st4<NT>(w4, wn);
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t k = (nvec << 2) + tid;
        float a = 0.0f;
        for (uint32_t p = 0; p < P; ++p) {
            float v = tab.e[p][k];
            a += apply1<MODE>(v, neg_mu_pos[p], mu_neg[p], gmu_pos, neg_gmu_neg);
        }
        w[k] -= eta_over_P * a;
    }
}

constexpr int kErrorItems = 4;  // float4 groups per array per thread in k_error_signs: half a sign row per workgroup
constexpr uint32_t kLazySignLds = 8 * 1024;  // its dynamic-LDS request when streaming (20 workgroups per CU)

// Weight update in retained-error mode from the sign words: there the update of an element is
// (k * gmu_pos - (P - k) * gmu_neg) / P with k = the number of workers whose v is >= 0 (Algorithm 1 line 6 summed
// over the workers as in Eq. 1), so the pass reads one bit per element-worker instead of v.  A workgroup is one
// wavefront; it covers one half (4) of the float4 groups that each thread of one workgroup of the pass that wrote
// the sign words owned, so a thread finds its 16 bits in that thread's half-word of every worker.
// LAZY: the apply pass of the lazy state; tab.e holds v.  A NaN has no sign: if the reduction counted any, the pass
// reads v as k_lazy_apply does (a branch that is uniform over the grid), and the scalar tail reads v too.
// !LAZY: second half of the two-kernel apply pass; tab.e holds the new errors that k_error_signs wrote, which are
// NaN exactly where v was, so with NaNs about the pass reads them next to the sign bits; the last n % 4 elements,
// which k_error_signs left alone, get the whole of lines 4, 6 and 7 here.
template <bool NT, int UP, bool LAZY>
__global__ __launch_bounds__(64) void k_apply_signs(const PtrTable tab, const uint16_t *__restrict__ sign,
                                                    float *__restrict__ w, const uint64_t n, const uint32_t P,
                                                    const float eta_over_P, const WsHeader *__restrict__ hdr)
{
    constexpr int ITEMS = 4;
    constexpr uint32_t kParts = kLazyItems / ITEMS;
    static_assert(kParts == 2, "two 16-bit halves per thread of the reduction pass");
    const uint32_t lane = threadIdx.x;
    const uint32_t lz = opaque_zero();
    const float gmu_pos = (&hdr->gmu_pos)[lz], gmu_neg = (&hdr->gmu_neg)[lz];
    const uint32_t any_nan = (&hdr->any_nan)[lz];
    const uint64_t nvec = n >> 2;
    const uint64_t b = blockIdx.x / kParts;            // workgroup of the reduction pass
    const uint32_t u0 = (blockIdx.x % kParts) * ITEMS;  // first of its float4 groups handled here
    const uint64_t first = b * (64ull * kLazyItems) + u0 * 64ull + lane;
    vf4 *w4 = reinterpret_cast<vf4 *>(w);
    vf4 wv[ITEMS];
#pragma unroll
    for (int t = 0; t < ITEMS; ++t)
        if (first + t * 64 < nvec)
            wv[t] = ld4<NT>(w4 + first + t * 64);
    vf4 acc[ITEMS];
    if (any_nan == 0) {
        const uint16_t *half = sign + static_cast<uint64_t>(blockIdx.x) * P * 64 + lane;  // sign[b][h][.][lane]
        uint32_t k[ITEMS][4];
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            k[t][0] = k[t][1] = k[t][2] = k[t][3] = 0;
        uint32_t p0 = 0;
        for (; p0 + UP <= P; p0 += UP) {
            uint32_t d[UP];
#pragma unroll
            for (int q = 0; q < UP; ++q)
                d[q] = half[(p0 + q) * 64];
#pragma unroll
            for (int q = 0; q < UP; ++q)
#pragma unroll
                for (int t = 0; t < ITEMS; ++t)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        k[t][c] += (d[q] >> (15u - (4u * t + c))) & 1u;
        }
        for (; p0 < P; ++p0) {
            const uint32_t d = half[p0 * 64];
#pragma unroll
            for (int t = 0; t < ITEMS; ++t)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    k[t][c] += (d >> (15u - (4u * t + c))) & 1u;
        }
        const float gsum = gmu_pos + gmu_neg, base = static_cast<float>(P) * gmu_neg;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            acc[t] = vf4{static_cast<float>(k[t][0]) * gsum - base, static_cast<float>(k[t][1]) * gsum - base,
                         static_cast<float>(k[t][2]) * gsum - base, static_cast<float>(k[t][3]) * gsum - base};
    } else if (LAZY) {
        const float neg_gmu_neg = -gmu_neg;
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            acc[t] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
        for (uint32_t p = 0; p < P; ++p) {
            const vf4 *v4 = reinterpret_cast<const vf4 *>(tab.e[p]);
            const float nmp = hdr->neg_mu_pos[p], mn = hdr->mu_neg[p];
#pragma unroll
            for (int t = 0; t < ITEMS; ++t)
                if (first + t * 64 < nvec)
                    (void)apply4<A2SGD_MODE_RETAINED_ERROR>(ld4<NT>(v4 + first + t * 64), acc[t], nmp, mn, gmu_pos,
                                                            neg_gmu_neg);
        }
    } else {
        const uint16_t *half = sign + static_cast<uint64_t>(blockIdx.x) * P * 64 + lane;  // sign[b][h][.][lane]
#pragma unroll
        for (int t = 0; t < ITEMS; ++t)
            acc[t] = vf4{0.0f, 0.0f, 0.0f, 0.0f};
        for (uint32_t p = 0; p < P; ++p) {
            const vf4 *e4 = reinterpret_cast<const vf4 *>(tab.e[p]);
            const uint32_t d = half[p * 64];
#pragma unroll
            for (int t = 0; t < ITEMS; ++t)
                if (first + t * 64 < nvec) {
                    const vf4 err = ld4<NT>(e4 + first + t * 64);
                    const float x[4] = {err.x, err.y, err.z, err.w};
                    float u[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        u[c] = ((d >> (15u - (4u * t + c))) & 1u) ? gmu_pos : -gmu_neg;
                        u[c] = (x[c] != x[c]) ? x[c] : u[c];  // the error is NaN exactly where v was
                    }
                    acc[t] += vf4{u[0], u[1], u[2], u[3]};
                }
        }
    }
#pragma unroll
    for (int t = 0; t < ITEMS; ++t)
        if (first + t * 64 < nvec) {
            const vf4 wn = wv[t] - eta_over_P * acc[t];
            st4<NT>(w4 + first + t * 64, wn);
        }
    if (blockIdx.x == gridDim.x - 1 && lane < (n & 3)) {  // the scalar tail reads v itself
        const uint64_t i = (nvec << 2) + lane;
        float a = 0.0f;
        for (uint32_t p = 0; p < P; ++p) {
            float v = LAZY ? tab.e[p][i] : tab.g[p][i] + tab.e[p][i];
            a += apply1<A2SGD_MODE_RETAINED_ERROR>(v, hdr->neg_mu_pos[p], hdr->mu_neg[p], gmu_pos, -gmu_neg);
            if (!LAZY)
                tab.e[p][i] = v;  // apply1 has turned v into the new error
        }
        w[i] -= eta_over_P * a;
    }
}

// s <- pending error of s, in place, for every worker: grid = (workgroups, P) of single wavefronts launched once,
// kMaterializeItems float4 groups per thread, all loads ahead of the first store (the shape of the other passes
// that store).
constexpr int kMaterializeItems = 4;
template <bool NT>
__global__ __launch_bounds__(64) void k_lazy_materialize(const PtrTable tab, const uint64_t n,
                                                         const WsHeader *__restrict__ hdr)
{
    const uint32_t p = blockIdx.y, tid = threadIdx.x;
    const uint32_t lz = opaque_zero();
    const float nmp = hdr->neg_mu_pos[p + lz], mn = hdr->mu_neg[p + lz];
    float *s = tab.e[p];
    vf4 *s4 = reinterpret_cast<vf4 *>(s);
    const uint64_t nvec = n >> 2;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * (64 * kMaterializeItems) + tid;
    if ((static_cast<uint64_t>(blockIdx.x) + 1) * (64 * kMaterializeItems) <= nvec) {
        vf4 v[kMaterializeItems];
#pragma unroll
        for (int u = 0; u < kMaterializeItems; ++u)
            v[u] = ld4<NT>(s4 + base + u * 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kMaterializeItems; ++u) {
            const vf4 e = pending_error4(v[u], nmp, mn);
            st4<NT>(s4 + base + u * 64, e);
        }
    } else {
        for (int u = 0; u < kMaterializeItems; ++u) {
            const uint64_t i = base + static_cast<uint64_t>(u) * 64;
            if (i < nvec) {
                const vf4 e = pending_error4(ld4<NT>(s4 + i), nmp, mn);
                st4<NT>(s4 + i, e);
            }
        }
    }
    if (blockIdx.x == 0 && tid < (n & 3)) {
        const uint64_t i = (nvec << 2) + tid;
        s[i] = pending_error(s[i], nmp, mn);
    }
}

// Clears the carried means: from here on the buffers are read as true errors.
__global__ void k_lazy_reset(WsHeader *__restrict__ hdr)
{
    for (uint32_t p = threadIdx.x; p < kMaxWorkers; p += blockDim.x) {
        hdr->neg_mu_pos[p] = 0.0f;
        hdr->mu_neg[p] = 0.0f;
    }
}

// Test aid: pos(v) of Eq. 2 as one bit per element.  grid = (ceil(n / kBlock), P); a wavefront covers 64
// consecutive elements, so its ballot is exactly one output word.
template <bool HAS_E>
__global__ __launch_bounds__(kBlock) void k_export_mask(const PtrTable tab, const uint64_t n, const uint64_t words,
                                                        uint64_t *__restrict__ mask)
{
    const uint32_t p = blockIdx.y;
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    bool bit = false;
    if (i < n) {
        float v = tab.g[p][i];
        if (HAS_E)
            v += tab.e[p][i];
        bit = v >= 0.0f;
    }
    const uint64_t word = __ballot(bit);
    if ((threadIdx.x & 63) == 0 && (i >> 6) < words)
        mask[static_cast<uint64_t>(p) * words + (i >> 6)] = word;
}

// ---------------------------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------------------------

hipError_t launch_local_partials(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, void *ws, hipStream_t s)
{
    const dim3 grid(pl.B, pl.P), block(kBlock);
    const Partials out = partials_of(ws, pl.P, pl.B);
    if (has_e) {
        if (pl.streaming)
            k_local_partials<true, true><<<grid, block, 0, s>>>(tab, pl.n, pl.B, out);
        else
            k_local_partials<true, false><<<grid, block, 0, s>>>(tab, pl.n, pl.B, out);
    } else {
        if (pl.streaming)
            k_local_partials<false, true><<<grid, block, 0, s>>>(tab, pl.n, pl.B, out);
        else
            k_local_partials<false, false><<<grid, block, 0, s>>>(tab, pl.n, pl.B, out);
    }
    return hipGetLastError();
}

hipError_t launch_local_finalize(const a2sgd_plan_t &pl, void *ws, hipStream_t s)
{
    k_local_finalize<<<dim3(pl.P), dim3(kBlock), 0, s>>>(pl.n, pl.B, partials_of(ws, pl.P, pl.B),
                                                        static_cast<WsHeader *>(ws));
    return hipGetLastError();
}

hipError_t launch_export_local_means(const a2sgd_plan_t &pl, const void *ws, float *out, hipStream_t s)
{
    k_export_local_means<<<dim3(1), dim3(64), 0, s>>>(pl.P, static_cast<const WsHeader *>(ws), out);
    return hipGetLastError();
}

hipError_t launch_import_global_means(const a2sgd_plan_t &pl, void *ws, const float *gmu, hipStream_t s)
{
    k_import_global_means<<<dim3(1), dim3(64), 0, s>>>(pl.P, static_cast<WsHeader *>(ws), gmu);
    return hipGetLastError();
}

hipError_t launch_global_average(const a2sgd_plan_t &pl, void *ws, hipStream_t s)
{
    k_global_average<<<dim3(1), dim3(64), 0, s>>>(pl.P, static_cast<WsHeader *>(ws));
    return hipGetLastError();
}

// One instantiation of the apply kernel.  lds_bytes of dynamic LDS are requested only to limit the workgroups
// per compute unit (160 KiB of LDS per CU); 0 = no limit.
template <int MODE, bool HAS_E, bool NT, int UP, int ITEMS, int SEQ, int BLOCK>
hipError_t launch_apply_geom(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop, const WsHeader *hdr,
                             uint32_t lds_bytes, hipStream_t s)
{
    auto kern = k_apply<MODE, HAS_E, NT, UP, ITEMS, SEQ, BLOCK>;  // lds_bytes <= 48 KiB: no attribute to raise
    const uint64_t nvec = (pl.n + 3) >> 2;  // the scalar tail rides in the last workgroup even when n < 4
    const uint64_t per = static_cast<uint64_t>(BLOCK) * ITEMS * SEQ;
    const dim3 grid(static_cast<uint32_t>((nvec + per - 1) / per)), block(BLOCK);
    kern<<<grid, block, lds_bytes, s>>>(tab, w, pl.n, pl.P, eop, hdr);
    return hipGetLastError();
}

template <int MODE, bool HAS_E, bool NT>
static hipError_t launch_apply_shape(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop,
                                     const WsHeader *hdr, hipStream_t s)
{
    const ApplyGeom &ge = pl.apply;
    // single-wavefront workgroups; one float4 group per thread and worker (two at P = 1)
    if (ge.up == 8)
        return launch_apply_geom<MODE, HAS_E, NT, 8, 1, 1, 64>(pl, tab, w, eop, hdr, ge.lds_bytes, s);
    if (ge.up == 4)
        return launch_apply_geom<MODE, HAS_E, NT, 4, 1, 1, 64>(pl, tab, w, eop, hdr, ge.lds_bytes, s);
    if (ge.up == 2)
        return launch_apply_geom<MODE, HAS_E, NT, 2, 1, 1, 64>(pl, tab, w, eop, hdr, ge.lds_bytes, s);
    if (ge.up == 1)
        return launch_apply_geom<MODE, HAS_E, NT, 1, 2, 1, 64>(pl, tab, w, eop, hdr, ge.lds_bytes, s);
    return hipErrorInvalidValue;
}

// The apply pass as two kernels (k_error_signs, then k_apply_signs on the sign words it left): streaming plans in
// retained-error mode with many workers.  The sign words live where the lazy calls keep theirs.
static hipError_t launch_apply_two_kernels(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop, void *ws,
                                           hipStream_t s)
{
    const WsHeader *hdr = static_cast<const WsHeader *>(ws);
    uint16_t *sign = reinterpret_cast<uint16_t *>(static_cast<char *>(ws) + pl.lazy_sign_offset);
    // 4 float4 groups of g and of e per thread and 8 workgroups per compute unit (64 KiB of loads in flight per CU):
    // measured at 16 workers against 8 groups per thread with 6 workgroups per CU, 4.26 ms against 4.65 ms
    k_error_signs<true, kErrorItems><<<dim3(pl.lazy_blocks * (kLazyItems / kErrorItems), pl.P), dim3(64), 18 * 1024, s>>>(
        tab, pl.n, hdr, sign);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    const dim3 grid(pl.lazy_blocks * 2), block(64);
    if (pl.P >= 16)  // the sign words of 16, 8 or 4 workers are loaded together
        k_apply_signs<true, 16, false><<<grid, block, kLazySignLds, s>>>(tab, sign, w, pl.n, pl.P, eop, hdr);
    else if (pl.P >= 8)
        k_apply_signs<true, 8, false><<<grid, block, kLazySignLds, s>>>(tab, sign, w, pl.n, pl.P, eop, hdr);
    else
        k_apply_signs<true, 4, false><<<grid, block, kLazySignLds, s>>>(tab, sign, w, pl.n, pl.P, eop, hdr);
    return hipGetLastError();
}

hipError_t launch_apply(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                        bool one_kernel, hipStream_t s)
{
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    const WsHeader *hdr = static_cast<const WsHeader *>(ws);
    const bool lit = pl.mode == A2SGD_MODE_ALG1_LITERAL;
    if (pl.apply.two_kernels && !one_kernel && !lit && has_e)
        return launch_apply_two_kernels(pl, tab, w, eop, ws, s);
#define A2SGD_APPLY_CASE(L, E, N)                                                                              \
    if (lit == L && has_e == E && pl.streaming == N)                                                           \
        return launch_apply_shape<L ? A2SGD_MODE_ALG1_LITERAL : A2SGD_MODE_RETAINED_ERROR, E, N>(pl, tab, w, eop, \
                                                                                                 hdr, s);
    A2SGD_APPLY_CASE(false, true, true)
    A2SGD_APPLY_CASE(false, true, false)
    A2SGD_APPLY_CASE(false, false, true)
    A2SGD_APPLY_CASE(false, false, false)
    A2SGD_APPLY_CASE(true, true, true)
    A2SGD_APPLY_CASE(true, true, false)
    A2SGD_APPLY_CASE(true, false, true)
    A2SGD_APPLY_CASE(true, false, false)
#undef A2SGD_APPLY_CASE
    return hipErrorInvalidValue;
}

template <int MODE, bool HAS_E>
static hipError_t launch_fused_inst(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop, void *ws,
                                    uint32_t token, hipStream_t s)
{
    const dim3 grid(pl.fused_grid), block(kFusedBlock);
    const Partials part = partials_of(ws, pl.P, pl.fused_grid);
    WsHeader *hdr = static_cast<WsHeader *>(ws);
    switch (pl.apply.up) {
    case 8:
    case 4: k_fused_step<MODE, HAS_E, 4><<<grid, block, 0, s>>>(tab, w, pl.n, pl.P, eop, part, hdr, static_cast<uint32_t>(pl.barrier_cell), token); break;
    case 2: k_fused_step<MODE, HAS_E, 2><<<grid, block, 0, s>>>(tab, w, pl.n, pl.P, eop, part, hdr, static_cast<uint32_t>(pl.barrier_cell), token); break;
    default: k_fused_step<MODE, HAS_E, 1><<<grid, block, 0, s>>>(tab, w, pl.n, pl.P, eop, part, hdr, static_cast<uint32_t>(pl.barrier_cell), token); break;
    }
    return hipGetLastError();
}

hipError_t launch_fused_step(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                             uint32_t token, hipStream_t s)
{
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    if (pl.mode == A2SGD_MODE_ALG1_LITERAL)
        return has_e ? launch_fused_inst<A2SGD_MODE_ALG1_LITERAL, true>(pl, tab, w, eop, ws, token, s)
                     : launch_fused_inst<A2SGD_MODE_ALG1_LITERAL, false>(pl, tab, w, eop, ws, token, s);
    return has_e ? launch_fused_inst<A2SGD_MODE_RETAINED_ERROR, true>(pl, tab, w, eop, ws, token, s)
                 : launch_fused_inst<A2SGD_MODE_RETAINED_ERROR, false>(pl, tab, w, eop, ws, token, s);
}

FusedSegView fused_seg_view(const a2sgd_plan_t &pl, void *ws)
{
    char *b = static_cast<char *>(ws);
    const SegPlan &sp = pl.seg;
    const size_t stride = 8ull * pl.P * sp.fitem.size();
    FusedSegView v;
    v.num_items = static_cast<uint32_t>(sp.fitem.size());
    v.item = reinterpret_cast<const SegItem *>(b + sp.off_fitem);
    v.item_lo = reinterpret_cast<const uint32_t *>(b + sp.off_fitem_lo);
    v.r_spos = reinterpret_cast<double *>(b + sp.off_frecords);
    v.r_sneg = reinterpret_cast<double *>(b + sp.off_frecords + stride);
    v.r_npos = reinterpret_cast<uint64_t *>(b + sp.off_frecords + 2 * stride);
    v.r_nneg = reinterpret_cast<uint64_t *>(b + sp.off_frecords + 3 * stride);
    v.r_nzero = reinterpret_cast<uint64_t *>(b + sp.off_frecords + 4 * stride);
    return v;
}

template <int MODE, bool HAS_E>
static hipError_t launch_seg_fused_inst(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop, void *ws,
                                        uint32_t token, hipStream_t s)
{
    const dim3 grid(pl.fused_grid), block(kFusedBlock);
    const SegView sv = seg_view(pl, ws);
    const FusedSegView fv = fused_seg_view(pl, ws);
    const uint32_t cell = static_cast<uint32_t>(pl.barrier_cell);
    switch (pl.apply.up) {
    case 8:
    case 4: k_seg_fused_step<MODE, HAS_E, 4><<<grid, block, 0, s>>>(tab, w, pl.P, eop, sv, fv, cell, token); break;
    case 2: k_seg_fused_step<MODE, HAS_E, 2><<<grid, block, 0, s>>>(tab, w, pl.P, eop, sv, fv, cell, token); break;
    default: k_seg_fused_step<MODE, HAS_E, 1><<<grid, block, 0, s>>>(tab, w, pl.P, eop, sv, fv, cell, token); break;
    }
    return hipGetLastError();
}

hipError_t launch_seg_fused_step(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                                 uint32_t token, hipStream_t s)
{
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    if (pl.mode == A2SGD_MODE_ALG1_LITERAL)
        return has_e ? launch_seg_fused_inst<A2SGD_MODE_ALG1_LITERAL, true>(pl, tab, w, eop, ws, token, s)
                     : launch_seg_fused_inst<A2SGD_MODE_ALG1_LITERAL, false>(pl, tab, w, eop, ws, token, s);
    return has_e ? launch_seg_fused_inst<A2SGD_MODE_RETAINED_ERROR, true>(pl, tab, w, eop, ws, token, s)
                 : launch_seg_fused_inst<A2SGD_MODE_RETAINED_ERROR, false>(pl, tab, w, eop, ws, token, s);
}

template <int MODE, bool HAS_E, bool NT>
static hipError_t launch_apply_replicas_shape(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt,
                                              float eta, const WsHeader *hdr, hipStream_t s)
{
    constexpr int kThreads = 64;
    const uint64_t nvec = (pl.n + 3) >> 2;
    if (NT && pl.P >= kPerWorkerReplicas) {
        // one worker per workgroup, 2 float4 groups of g, e and w^p per thread, 8 workgroups per CU (measured, whole
        // replica step in ms at configs 4 / 2: grouped form 10.42 / 0.914; this form with 2 groups per thread and 10, 8,
        // 6, 4 workgroups per CU 9.64 / 0.890, 9.36 / 0.877, 9.53 / 0.905, 10.62 / 1.019; with 4 groups per thread
        // 9.73 / 0.934, 9.52 / 0.915, 9.43 / 0.884, 9.74 / 0.926; at config 5, 4 workers, the grouped form wins,
        // 25.5 against 26.3)
        constexpr int kItems = 2;
        const uint64_t per = 64ull * kItems;
        const dim3 per_worker(static_cast<uint32_t>((nvec + per - 1) / per), pl.P);
        k_apply_replicas_per_worker<MODE, HAS_E, NT, kItems><<<per_worker, dim3(64), 18 * 1024, s>>>(tab, wt, pl.n, eta, hdr);
        return hipGetLastError();
    }
    const dim3 grid(static_cast<uint32_t>((nvec + kThreads - 1) / kThreads)), block(kThreads);
    // 3 loads per worker instead of 2: groups of 4 workers at most, and then 6 workgroups per CU whatever P is
    // (the shared pass has groups of 8 for P >= 8 and caps residency lower)
    const uint32_t lds = pl.apply.lds_bytes > 25 * 1024 ? 25 * 1024 : pl.apply.lds_bytes;
    if (pl.apply.up >= 4)
        k_apply_replicas<MODE, HAS_E, NT, 4, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eta, hdr);
    else if (pl.apply.up == 2)
        k_apply_replicas<MODE, HAS_E, NT, 2, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eta, hdr);
    else
        k_apply_replicas<MODE, HAS_E, NT, 1, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eta, hdr);
    return hipGetLastError();
}

hipError_t launch_apply_replicas(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt, bool has_e,
                                 float eta, void *ws, hipStream_t s)
{
    const WsHeader *hdr = static_cast<const WsHeader *>(ws);
    const bool lit = pl.mode == A2SGD_MODE_ALG1_LITERAL;
#define A2SGD_REPL_CASE(L, E, N)                                                                               \
    if (lit == L && has_e == E && pl.streaming == N)                                                           \
        return launch_apply_replicas_shape<L ? A2SGD_MODE_ALG1_LITERAL : A2SGD_MODE_RETAINED_ERROR, E, N>(      \
            pl, tab, wt, eta, hdr, s);
    A2SGD_REPL_CASE(false, true, true)
    A2SGD_REPL_CASE(false, true, false)
    A2SGD_REPL_CASE(false, false, true)
    A2SGD_REPL_CASE(false, false, false)
    A2SGD_REPL_CASE(true, true, true)
    A2SGD_REPL_CASE(true, true, false)
    A2SGD_REPL_CASE(true, false, true)
    A2SGD_REPL_CASE(true, false, false)
#undef A2SGD_REPL_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_dense_step_replicas(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt, float eta,
                                      hipStream_t s)
{
    constexpr int kThreads = 64;
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    const uint64_t nvec = (pl.n + 3) >> 2;
    const dim3 grid(static_cast<uint32_t>((nvec + kThreads - 1) / kThreads)), block(kThreads);
    const uint32_t lds = pl.apply.lds_bytes;
    if (pl.streaming) {
        if (pl.apply.up >= 4)
            k_dense_step_replicas<true, 4, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eop);
        else
            k_dense_step_replicas<true, 1, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eop);
    } else {
        if (pl.apply.up >= 4)
            k_dense_step_replicas<false, 4, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eop);
        else
            k_dense_step_replicas<false, 1, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eop);
    }
    return hipGetLastError();
}

size_t drift_result_offset(const a2sgd_plan_t &pl)
{
    return kHeaderBytes + 2ull * 8ull * pl.P * kDriftBlocks;
}

hipError_t launch_replica_drift(const a2sgd_plan_t &pl, const ReplicaTable &wt, void *ws, hipStream_t s)
{
    char *base = static_cast<char *>(ws) + kHeaderBytes;
    double *max_part = reinterpret_cast<double *>(base);
    double *sq_part = max_part + static_cast<size_t>(pl.P) * kDriftBlocks;
    double *result = reinterpret_cast<double *>(static_cast<char *>(ws) + drift_result_offset(pl));
    k_replica_drift<<<dim3(kDriftBlocks, pl.P), dim3(kBlock), 0, s>>>(wt, pl.n, pl.P, max_part, sq_part);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    k_replica_drift_finalize<<<dim3(1), dim3(64), 0, s>>>(pl.n, pl.P, kDriftBlocks, max_part, sq_part, result);
    return hipGetLastError();
}

hipError_t launch_lazy_reset(const a2sgd_plan_t &, void *ws, hipStream_t s)
{
    k_lazy_reset<<<dim3(1), dim3(64), 0, s>>>(static_cast<WsHeader *>(ws));
    return hipGetLastError();
}

// The lazy state's reduction: one-shot pass, fold of its records, local means.  The dynamic LDS request only limits
// the workgroups per compute unit (6 of them keep about 96 KiB of loads in flight per CU).
hipError_t launch_lazy_partials(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s)
{
    const dim3 grid(pl.lazy_blocks, pl.P), block(64);
    const Partials rec = partials_at(ws, pl.lazy_offset, pl.P, pl.lazy_blocks);
    const size_t folded_offset = pl.lazy_offset + 5ull * 8ull * pl.P * pl.lazy_blocks;
    const Partials folded = partials_at(ws, folded_offset, pl.P, pl.lazy_folded);
    WsHeader *hdr = static_cast<WsHeader *>(ws);
    uint16_t *sign = reinterpret_cast<uint16_t *>(static_cast<char *>(ws) + pl.lazy_sign_offset);
    const bool signs = pl.mode == A2SGD_MODE_RETAINED_ERROR;  // the literal mode's apply pass needs v itself
    if (pl.streaming) {
        if (signs)
            k_lazy_partials<true, true><<<grid, block, 25 * 1024, s>>>(tab, pl.n, pl.lazy_blocks, hdr, rec, sign);
        else
            k_lazy_partials<true, false><<<grid, block, 25 * 1024, s>>>(tab, pl.n, pl.lazy_blocks, hdr, rec, sign);
    } else {
        if (signs)
            k_lazy_partials<false, true><<<grid, block, 0, s>>>(tab, pl.n, pl.lazy_blocks, hdr, rec, sign);
        else
            k_lazy_partials<false, false><<<grid, block, 0, s>>>(tab, pl.n, pl.lazy_blocks, hdr, rec, sign);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    k_fold_partials<<<dim3(pl.lazy_folded, pl.P), dim3(kBlock), 0, s>>>(pl.lazy_blocks, rec, pl.lazy_folded, folded);
    if ((err = hipGetLastError()) != hipSuccess)
        return err;
    k_local_finalize<<<dim3(pl.P), dim3(kBlock), 0, s>>>(pl.n, pl.lazy_folded, folded, hdr);
    return hipGetLastError();
}

template <int MODE, bool NT>
static hipError_t launch_lazy_apply_shape(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop,
                                          const WsHeader *hdr, hipStream_t s)
{
    constexpr int kThreads = 64;
    const uint64_t nvec = (pl.n + 3) >> 2;
    const dim3 grid(static_cast<uint32_t>((nvec + kThreads - 1) / kThreads)), block(kThreads);
    // up + 1 loads in flight per thread, about half of what the eager apply pass has: about twice as many
    // workgroups per CU (same 160 KiB of LDS, a smaller request)
    const uint32_t lds = pl.apply.lds_bytes ? pl.apply.lds_bytes / 2 + 3 * 1024 : 0;
    switch (pl.apply.up) {
    case 8: k_lazy_apply<MODE, NT, 8, kThreads><<<grid, block, lds, s>>>(tab, w, pl.n, pl.P, eop, hdr); break;
    case 4: k_lazy_apply<MODE, NT, 4, kThreads><<<grid, block, lds, s>>>(tab, w, pl.n, pl.P, eop, hdr); break;
    case 2: k_lazy_apply<MODE, NT, 2, kThreads><<<grid, block, lds, s>>>(tab, w, pl.n, pl.P, eop, hdr); break;
    default: k_lazy_apply<MODE, NT, 1, kThreads><<<grid, block, lds, s>>>(tab, w, pl.n, pl.P, eop, hdr); break;
    }
    return hipGetLastError();
}

hipError_t launch_lazy_apply(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eta, void *ws, hipStream_t s)
{
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    const WsHeader *hdr = static_cast<const WsHeader *>(ws);
    if (pl.mode == A2SGD_MODE_ALG1_LITERAL)
        return pl.streaming ? launch_lazy_apply_shape<A2SGD_MODE_ALG1_LITERAL, true>(pl, tab, w, eop, hdr, s)
                            : launch_lazy_apply_shape<A2SGD_MODE_ALG1_LITERAL, false>(pl, tab, w, eop, hdr, s);
    // retained-error mode: from the sign bits that the reduction pass left, two workgroups per workgroup of that
    // pass (one per half of its float4 groups)
    const uint16_t *sign = reinterpret_cast<const uint16_t *>(static_cast<const char *>(ws) + pl.lazy_sign_offset);
    const dim3 grid(pl.lazy_blocks * 2), block(64);
    if (pl.streaming) {
        if (pl.P >= 4)
            k_apply_signs<true, 4, true><<<grid, block, kLazySignLds, s>>>(tab, sign, w, pl.n, pl.P, eop, hdr);
        else
            k_apply_signs<true, 1, true><<<grid, block, kLazySignLds, s>>>(tab, sign, w, pl.n, pl.P, eop, hdr);
    } else {
        if (pl.P >= 4)
            k_apply_signs<false, 4, true><<<grid, block, 0, s>>>(tab, sign, w, pl.n, pl.P, eop, hdr);
        else
            k_apply_signs<false, 1, true><<<grid, block, 0, s>>>(tab, sign, w, pl.n, pl.P, eop, hdr);
    }
    return hipGetLastError();
}

hipError_t launch_lazy_materialize(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s)
{
    const uint64_t nvec = pl.n >> 2, per = 64ull * kMaterializeItems;
    const dim3 grid(static_cast<uint32_t>(nvec ? (nvec + per - 1) / per : 1), pl.P), block(64);
    const WsHeader *hdr = static_cast<const WsHeader *>(ws);
    if (pl.streaming)
        k_lazy_materialize<true><<<grid, block, 12 * 1024, s>>>(tab, pl.n, hdr);  // 13 workgroups per CU
    else
        k_lazy_materialize<false><<<grid, block, 0, s>>>(tab, pl.n, hdr);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    return launch_lazy_reset(pl, ws, s);
}

hipError_t launch_barrier_selftest(uint32_t grid, uint32_t expected, uint32_t spin_limit, uint32_t *passed,
                                   uint32_t *cell_failed, hipStream_t s)
{
    k_barrier_selftest<<<dim3(grid), dim3(kBlock), 0, s>>>(expected, spin_limit, passed);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    k_barrier_reset<<<dim3(1), dim3(64), 0, s>>>(kBarrierSlots, cell_failed);
    return hipGetLastError();
}

hipError_t launch_barrier_reset(uint32_t cell, hipStream_t s)
{
    if (cell >= kBarrierSlots)
        return hipErrorInvalidValue;
    k_barrier_reset<<<dim3(1), dim3(64), 0, s>>>(cell, nullptr);
    return hipGetLastError();
}

hipError_t launch_export_mask(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, uint64_t *mask, hipStream_t s)
{
    const uint64_t words = (pl.n + 63) / 64;
    const dim3 grid(static_cast<uint32_t>((pl.n + kBlock - 1) / kBlock), pl.P), block(kBlock);
    if (has_e)
        k_export_mask<true><<<grid, block, 0, s>>>(tab, pl.n, words, mask);
    else
        k_export_mask<false><<<grid, block, 0, s>>>(tab, pl.n, words, mask);
    return hipGetLastError();
}

template <bool NT, int UP>
static hipError_t launch_dense_inst(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop, hipStream_t s)
{
    constexpr int kItems = 2, kThreads = 64;
    const uint64_t nvec = (pl.n + 3) >> 2, per = static_cast<uint64_t>(kThreads) * kItems;
    const dim3 grid(static_cast<uint32_t>((nvec + per - 1) / per)), block(kThreads);
    k_dense_step<NT, UP, kItems, kThreads><<<grid, block, pl.apply.dense_lds_bytes, s>>>(tab, w, pl.n, pl.P, eop);
    return hipGetLastError();
}

hipError_t launch_dense_step(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eta, hipStream_t s)
{
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    const int up = pl.apply.up;
    if (pl.streaming)
        return up == 8   ? launch_dense_inst<true, 8>(pl, tab, w, eop, s)
               : up == 4 ? launch_dense_inst<true, 4>(pl, tab, w, eop, s)
               : up == 2 ? launch_dense_inst<true, 2>(pl, tab, w, eop, s)
                         : launch_dense_inst<true, 1>(pl, tab, w, eop, s);
    return up == 8   ? launch_dense_inst<false, 8>(pl, tab, w, eop, s)
           : up == 4 ? launch_dense_inst<false, 4>(pl, tab, w, eop, s)
           : up == 2 ? launch_dense_inst<false, 2>(pl, tab, w, eop, s)
                     : launch_dense_inst<false, 1>(pl, tab, w, eop, s);
}

}  // namespace a2sgd
