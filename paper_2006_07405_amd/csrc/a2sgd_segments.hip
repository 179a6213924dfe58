// Per-tensor means: the A2SGD step with one pair of local means per worker AND per tensor (segment) of the flat
// gradient instead of one pair per worker.  The paper states its operator for "a gradient vector v" (Sec. 3.1,
// Eq. 2) and applies it to the whole model; this is the same operator and the same Algorithm 1 lines 3-7 applied
// tensor by tensor, the way a per-layer hook would.  Segments are contiguous, in packing order, and cover [0, n).
//
// The plan splits every segment into work items of at most kSegItemElems elements that never cross a segment
// boundary.  Reduction: one partial record per (worker, item); second level per (worker, segment) over that
// segment's items in index order; then the per-segment global means.  The apply pass is the one-shot
// single-wavefront shape of k_apply; a workgroup reads its segment from a table with one entry per workgroup, and the few
// workgroups that straddle a boundary fall back to a per-element path.
#include "a2sgd_device.h"

namespace a2sgd {

SegView seg_view(const a2sgd_plan_t &pl, void *ws)
{
    char *b = static_cast<char *>(ws);
    const SegPlan &sp = pl.seg;
    SegView v;
    v.S = sp.S;
    v.num_items = static_cast<uint32_t>(sp.item.size());
    v.hdr = reinterpret_cast<WsHeader *>(b);
    v.tag = sp.tag;
    v.seg_start = reinterpret_cast<const uint64_t *>(b + sp.off_seg_start);
    v.seg_end = reinterpret_cast<const uint64_t *>(b + sp.off_seg_end);
    v.item = reinterpret_cast<const SegItem *>(b + sp.off_item);
    v.item_lo = reinterpret_cast<const uint32_t *>(b + sp.off_item_lo);
    v.coarse = reinterpret_cast<const uint32_t *>(b + sp.off_coarse);
    v.sched_lo = reinterpret_cast<const uint32_t *>(b + sp.off_sched_lo);
    v.sched_item = reinterpret_cast<const uint32_t *>(b + sp.off_sched_item);
    v.stats = reinterpret_cast<a2sgd_worker_stats_t *>(b + sp.off_stats);
    v.neg_mu_pos = reinterpret_cast<float *>(b + sp.off_nmp);
    v.mu_neg = reinterpret_cast<float *>(b + sp.off_mn);
    v.gmu = reinterpret_cast<float *>(b + sp.off_gmu);
    v.rec = partials_at(ws, sp.off_records, pl.P, v.num_items);
    return v;
}

__global__ void k_seg_mark(WsHeader *__restrict__ hdr, const uint64_t tag)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        hdr->seg_tag = tag;
        hdr->seg_fault = 0u;
    }
}

// ---------------------------------------------------------------------------------------------------------
// Reduction, first level (Algorithm 1 line 3 per tensor).  grid = (B, P); block b of worker p takes the items
// that the plan's schedule gives it (about equal work per block).  An item starts and ends anywhere: elements up to the first 16-byte boundary and after the
// last one are taken one per thread, the float4 groups in between kSegUnroll per thread per trip.
// ---------------------------------------------------------------------------------------------------------
constexpr int kSegUnroll = 4;
// Dynamic LDS request of the lazy state's reduction: 6 workgroups per CU, as in the whole-model form (measured at
// configs 5 / 4 / 2, lazy step in ms: 8 per CU 13.75 / 4.58 / 0.447, 6 per CU 13.47 / 4.46 / 0.457, 5 per CU 13.63 /
// 4.52 / 0.492, 4 per CU 14.77 / 5.02 / 0.573).
constexpr uint32_t kSegLazyLds = 25 * 1024;

template <bool HAS_E, bool NT>
__global__ __launch_bounds__(kBlock) void k_seg_partials(const PtrTable tab, const SegView sv)
{
    const uint32_t p = blockIdx.y, tid = threadIdx.x;
    const float *__restrict__ g = tab.g[p];
    const float *__restrict__ e = HAS_E ? tab.e[p] : nullptr;
    const vf4 *g4 = reinterpret_cast<const vf4 *>(g);
    const vf4 *e4 = reinterpret_cast<const vf4 *>(e);
    if (!seg_tables_ok(sv))
        return;
    const uint32_t k_end = sv.sched_lo[blockIdx.x + 1];
    for (uint32_t k = sv.sched_lo[blockIdx.x]; k < k_end; ++k) {
        const uint32_t it = sv.sched_item[k];
        const SegItem item = sv.item[it];
        const uint64_t lo = item.start, hi = item.start + item.count;
        uint64_t a = (lo + 3) & ~static_cast<uint64_t>(3);  // first element on a 16-byte boundary
        if (a > hi)
            a = hi;
        const uint64_t z = a + ((hi - a) & ~static_cast<uint64_t>(3));  // end of the float4 groups
        auto scalar = [&](const uint64_t i) {  // one element outside the float4 groups
            return HAS_E ? g[i] + e[i] : g[i];
        };
        LaneAcc acc;
        if (tid < a - lo) {  // head, at most 3 elements
            acc.add(scalar(lo + tid));
            acc.flush();
        }
        const uint64_t v_lo = a >> 2, v_hi = z >> 2;
        for (uint64_t i0 = v_lo + tid; i0 < v_hi; i0 += static_cast<uint64_t>(kBlock) * kSegUnroll) {
            vf4 gv[kSegUnroll], ev[kSegUnroll];
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u)
                if (i0 + u * kBlock < v_hi) {
                    gv[u] = ld4<NT>(g4 + i0 + u * kBlock);
                    if (HAS_E)
                        ev[u] = ld4<NT>(e4 + i0 + u * kBlock);
                }
#pragma unroll
            for (int u = 0; u < kSegUnroll; ++u)
                if (i0 + u * kBlock < v_hi) {
                    acc.add4(HAS_E ? gv[u] + ev[u] : gv[u]);
                }
            acc.flush();
        }
        if (tid < hi - z) {  // tail, at most 3 elements
            acc.add(scalar(z + tid));
            acc.flush();
        }
        // block reduction of this item (the counts are wavefront totals, valid in lane 0: indices grow with the lane)
        Sums mine;
        mine.s_pos = wave_sum(acc.s_pos);
        mine.s_neg = wave_sum(acc.s_neg);
        mine.n_pos = acc.c_pos;
        mine.n_neg = acc.c_neg;
        mine.n_zero = acc.c_zero;
        const Sums total = block_sum_of_waves(mine);
        if (tid == 0)
            store_record(sv.rec, static_cast<size_t>(p) * sv.num_items + it, total);
        __syncthreads();  // the LDS slots are free again for the next item
    }
}

// Second level: grid = (S, P), one wavefront per (segment, worker): that segment's records in a fixed order, then
// the two local means rounded to fp32 (Sec. 3.1; empty group: 0).
__global__ __launch_bounds__(64) void k_seg_finalize(const SegView sv)
{
    const uint32_t s = blockIdx.x, p = blockIdx.y, lane = threadIdx.x;
    if (!seg_tables_ok(sv))
        return;
    if (s == 0 && p == 0 && lane == 0)
        sv.hdr->any_nan = 0u;  // k_seg_global, next on the stream, raises it if any worker counted a NaN in any tensor
    const uint32_t lo = sv.item_lo[s], hi = sv.item_lo[s + 1];
    const size_t row = static_cast<size_t>(p) * sv.num_items;
    Sums t;
    for (uint32_t j = lo + lane; j < hi; j += 64)
        add_record(t, sv.rec, row + j);
    t.s_pos = wave_sum(t.s_pos);
    t.s_neg = wave_sum(t.s_neg);
    t.n_pos = wave_sum(t.n_pos);
    t.n_neg = wave_sum(t.n_neg);
    t.n_zero = wave_sum(t.n_zero);
    if (lane == 0) {
        const uint64_t len = sv.seg_end[s] - sv.seg_start[s];
        a2sgd_worker_stats_t r;
        r.mu_pos = t.n_pos ? static_cast<float>(t.s_pos / static_cast<double>(t.n_pos)) : 0.0f;
        r.mu_neg = t.n_neg ? static_cast<float>(t.s_neg / static_cast<double>(t.n_neg)) : 0.0f;
        r.n_pos = t.n_pos;
        r.n_neg = t.n_neg;
        r.n_zero = t.n_zero;
        r.n_nan = len - t.n_pos - t.n_neg;
        sv.stats[static_cast<size_t>(p) * sv.S + s] = r;
    }
}

// Second level with pooled means: grid = P, one block per worker: all of its records in a fixed order (strided per
// thread, shuffle tree, wavefronts in index order), one pair of means over all tensors together, and that result
// into every tensor's row so that the following passes need not know the difference.
__global__ __launch_bounds__(kBlock) void k_seg_finalize_pooled(const SegView sv, const uint64_t covered)
{
    const uint32_t p = blockIdx.x, tid = threadIdx.x;
    const size_t row = static_cast<size_t>(p) * sv.num_items;
    if (p == 0 && tid == 0)
        sv.hdr->any_nan = 0u;  // as in k_seg_finalize
    Sums mine;
    for (uint32_t j = tid; j < sv.num_items; j += kBlock)
        add_record(mine, sv.rec, row + j);
    __shared__ a2sgd_worker_stats_t sh_result;
    const Sums t = block_sum(mine);
    if (tid == 0) {
        a2sgd_worker_stats_t r;
        r.mu_pos = t.n_pos ? static_cast<float>(t.s_pos / static_cast<double>(t.n_pos)) : 0.0f;
        r.mu_neg = t.n_neg ? static_cast<float>(t.s_neg / static_cast<double>(t.n_neg)) : 0.0f;
        r.n_pos = t.n_pos;
        r.n_neg = t.n_neg;
        r.n_zero = t.n_zero;
        r.n_nan = covered - t.n_pos - t.n_neg;
        sh_result = r;
    }
    __syncthreads();
    for (uint32_t s = tid; s < sv.S; s += kBlock)
        sv.stats[static_cast<size_t>(p) * sv.S + s] = sh_result;
}

// Algorithm 1 line 5 per segment, and the tables the apply pass reads: one thread per segment.
__global__ __launch_bounds__(64) void k_seg_global(const uint32_t P, const SegView sv)
{
    const uint32_t s = blockIdx.x * 64 + threadIdx.x;
    if (s >= sv.S)
        return;
    double sp = 0.0, sn = 0.0;
    bool any_nan = false;
    for (uint32_t p = 0; p < P; ++p) {
        const a2sgd_worker_stats_t &r = sv.stats[static_cast<size_t>(p) * sv.S + s];
        any_nan |= r.n_nan != 0;
        sp += static_cast<double>(r.mu_pos);
        sn += static_cast<double>(r.mu_neg);
        sv.neg_mu_pos[static_cast<size_t>(s) * P + p] = -r.mu_pos;
        sv.mu_neg[static_cast<size_t>(s) * P + p] = r.mu_neg;
    }
    sv.gmu[2 * s] = static_cast<float>(sp / static_cast<double>(P));
    sv.gmu[2 * s + 1] = -static_cast<float>(sn / static_cast<double>(P));
    if (any_nan)
        atomicOr(&sv.hdr->any_nan, 1u);  // an integer flag: a NaN has no sign bit for the two-kernel apply pass
}

// ---------------------------------------------------------------------------------------------------------
// Apply pass (Algorithm 1 lines 4, 6, 7 per tensor)
// ---------------------------------------------------------------------------------------------------------

// Segment of element idx, scanning forward from a segment known to start at or before it.
__device__ __forceinline__ uint32_t seg_of(const SegView &sv, uint32_t s, uint64_t idx)
{
    while (sv.seg_end[s] <= idx)
        ++s;
    return s;
}

// Per-element path for the workgroups that straddle a segment boundary and for the last n % 4 elements.
template <int MODE, bool HAS_E>
__device__ __forceinline__ void seg_apply_element(const PtrTable &tab, float *w, const uint64_t idx, const uint32_t s,
                                                  const uint32_t P, const float eta_over_P, const SegView &sv)
{
    const float gmu_pos = sv.gmu[2 * s], neg_gmu_neg = sv.gmu[2 * s + 1];
    float acc = 0.0f;
    for (uint32_t p = 0; p < P; ++p) {
        float v = tab.g[p][idx];
        if (HAS_E)
            v += tab.e[p][idx];
        acc += apply1<MODE>(v, sv.neg_mu_pos[static_cast<size_t>(s) * P + p], sv.mu_neg[static_cast<size_t>(s) * P + p],
                            gmu_pos, neg_gmu_neg);
        if (HAS_E)
            tab.e[p][idx] = v;
    }
    w[idx] -= eta_over_P * acc;
}

// grid = ceil(ceil(n/4) / BLOCK) single-wavefront workgroups, thread t owning float4 group t.  The big loads of
// the first UP workers are issued first; the segment lookup and, behind it, the loads of that segment's end and
// means follow and overlap with them.
template <int MODE, bool HAS_E, bool NT, int UP, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_seg_apply(const PtrTable tab, float *__restrict__ w, const uint64_t n,
                                                     const uint32_t P, const float eta_over_P, const SegView sv)
{
    const uint32_t tid = threadIdx.x;
    const uint64_t nvec = n >> 2;
    const uint64_t first = static_cast<uint64_t>(blockIdx.x) * BLOCK;  // first float4 group of the workgroup
    const uint64_t i = first + tid;
    const bool live = i < nvec;
    vf4 *w4 = reinterpret_cast<vf4 *>(w) + i;
    vf4 wv, v[UP], ev[UP];
    if (live) {  // these loads need no table
        wv = ld4<NT>(w4);
#pragma unroll
        for (int u = 0; u < UP; ++u)
            if (static_cast<uint32_t>(u) < P)
                v[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.g[u]) + i);
        if (HAS_E) {
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (static_cast<uint32_t>(u) < P)
                    ev[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.e[u]) + i);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // the table has exactly one entry per workgroup, the segment of its first element; the entry's address does not
    // depend on what the tables hold, so it is read together with the tag that says whether they may be trusted
    static_assert(BLOCK * 4 == (1 << kSegCoarseShift), "one lookup entry per apply workgroup");
    const uint32_t entry = sv.coarse[blockIdx.x];
    if (!seg_tables_ok(sv))
        return;
    if (first < nvec) {
        const uint32_t s0 = entry & ~kSegInsideBit;  // the first segment that ends after the workgroup's first element
        if (entry & kSegInsideBit) {
            // the whole workgroup lies in segment s0
            if (live) {
                const uint32_t lz = opaque_zero();
                const float *nmp = sv.neg_mu_pos + static_cast<size_t>(s0) * P + lz;
                const float *mn = sv.mu_neg + static_cast<size_t>(s0) * P + lz;
                const float gmu_pos = sv.gmu[2 * s0 + lz], neg_gmu_neg = sv.gmu[2 * s0 + 1 + lz];
                vf4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int u = 0; u < UP; ++u)
                    if (static_cast<uint32_t>(u) < P) {
                        const vf4 vv = HAS_E ? v[u] + ev[u] : v[u];
                        const vf4 err = apply4<MODE>(vv, acc, nmp[u], mn[u], gmu_pos, neg_gmu_neg);
                        if (HAS_E)
                            st4<NT>(reinterpret_cast<vf4 *>(tab.e[u]) + i, err);
                    }
                for (uint32_t p0 = UP; p0 < P; p0 += UP) {  // further groups of UP workers
                    vf4 v2[UP], e2[UP];
#pragma unroll
                    for (int u = 0; u < UP; ++u)
                        if (p0 + u < P) {
                            v2[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.g[p0 + u]) + i);
                            if (HAS_E)
                                e2[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.e[p0 + u]) + i);
                        }
#pragma unroll
                    for (int u = 0; u < UP; ++u)
                        if (p0 + u < P) {
                            const vf4 vv = HAS_E ? v2[u] + e2[u] : v2[u];
                            const vf4 err = apply4<MODE>(vv, acc, nmp[p0 + u], mn[p0 + u], gmu_pos, neg_gmu_neg);
                            if (HAS_E)
                                st4<NT>(reinterpret_cast<vf4 *>(tab.e[p0 + u]) + i, err);
                        }
                }
                const vf4 wn = wv - eta_over_P * acc;
                st4<NT>(w4, wn);
            }
        } else if (live) {
            // A boundary inside the workgroup: each of the lane's four elements has its own segment, or none (padding
            // between tensors).  A float4 group that lies wholly inside segments still goes as one float4 per
            // worker and array, only the means are gathered per element; a group with padding in it goes element by
            // element, and padding is not touched.  (What was loaded above is reloaded, from the cache, to keep
            // this rare path simple.)
            uint32_t sc[4];
            bool in[4];
            uint32_t sx = s0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                sx = seg_of(sv, sx, (i << 2) + c);
                sc[c] = sx;
                in[c] = sv.seg_start[sx] <= (i << 2) + c;
            }
            if (in[0] && in[1] && in[2] && in[3]) {
                vf4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
                for (uint32_t p = 0; p < P; ++p) {
                    vf4 vv = ld4<NT>(reinterpret_cast<const vf4 *>(tab.g[p]) + i);
                    if (HAS_E)
                        vv += ld4<NT>(reinterpret_cast<const vf4 *>(tab.e[p]) + i);
                    float x[4] = {vv.x, vv.y, vv.z, vv.w}, a[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const size_t k = static_cast<size_t>(sc[c]) * P + p;
                        a[c] += apply1<MODE>(x[c], sv.neg_mu_pos[k], sv.mu_neg[k], sv.gmu[2 * sc[c]],
                                             sv.gmu[2 * sc[c] + 1]);
                    }
                    acc = vf4{a[0], a[1], a[2], a[3]};
                    if (HAS_E) {
                        const vf4 err = vf4{x[0], x[1], x[2], x[3]};
                        st4<NT>(reinterpret_cast<vf4 *>(tab.e[p]) + i, err);
                    }
                }
                const vf4 wn = wv - eta_over_P * acc;
                st4<NT>(w4, wn);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (in[c])
                        seg_apply_element<MODE, HAS_E>(tab, w, (i << 2) + c, sc[c], P, eta_over_P, sv);
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t idx = (nvec << 2) + tid;
        const uint32_t s = seg_of(sv, sv.coarse[idx >> kSegCoarseShift] & ~kSegInsideBit, idx);
        if (sv.seg_start[s] <= idx)
            seg_apply_element<MODE, HAS_E>(tab, w, idx, s, P, eta_over_P, sv);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Apply pass as two kernels (retained-error mode, many workers, streaming sizes): as in the whole-model form the
// update of a parameter depends only on how many workers have it in the positive group, now with the global means
// of the parameter's tensor.  k_seg_error_signs rewrites one worker's errors per workgroup and leaves pos(v) in
// the sign words; k_seg_apply_signs updates w from them.  A workgroup covers 1024 elements, i.e. four entries of
// the lookup table; a chunk that lies wholly inside one tensor takes that tensor's means for all its elements, the
// others look every element up (padding is neither written nor given a sign bit).
// ---------------------------------------------------------------------------------------------------------
constexpr int kSegSignItems = 4;  // float4 groups per array per thread: half a sign row per workgroup

// The segment of each of a float4 group's four elements (or S where the element is padding), scanning from s0.
__device__ __forceinline__ void seg_of4(const SegView &sv, uint32_t s0, const uint64_t first, uint32_t sc[4])
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        s0 = seg_of(sv, s0, first + c);
        sc[c] = sv.seg_start[s0] <= first + c ? s0 : sv.S;
    }
}

template <bool NT>
__global__ __launch_bounds__(64) void k_seg_error_signs(const PtrTable tab, const uint64_t n, const uint64_t chunks,
                                                        const SegView sv, uint16_t *__restrict__ sign)
{
    const uint32_t p = blockIdx.y, P = gridDim.y, lane = threadIdx.x;
    const vf4 *__restrict__ g4 = reinterpret_cast<const vf4 *>(tab.g[p]);
    float *e = tab.e[p];
    vf4 *e4 = reinterpret_cast<vf4 *>(e);
    const uint64_t nvec = n >> 2;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * (64 * kSegSignItems) + lane;
    vf4 gv[kSegSignItems], ev[kSegSignItems];
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u)
        if (base + u * 64 < nvec) {
            gv[u] = ld4<NT>(g4 + base + u * 64);
            ev[u] = ld4<NT>(e4 + base + u * 64);
        }
    __builtin_amdgcn_sched_barrier(0);
    static_assert(64 * 4 == (1 << kSegCoarseShift), "one lookup entry per 64 float4 groups");
    uint32_t entry[kSegSignItems];
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u) {
        const uint64_t c = static_cast<uint64_t>(blockIdx.x) * kSegSignItems + u;
        entry[u] = c < chunks ? sv.coarse[c] : 0u;
    }
    if (!seg_tables_ok(sv))
        return;
    // the means of every chunk's first tensor, all asked for at once (behind the entries, ahead of the arithmetic):
    // fetched chunk by chunk, each would cost the workgroup a memory latency with nothing else in flight
    float nmp[kSegSignItems], mn[kSegSignItems];
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u) {
        const uint32_t t = min(entry[u] & ~kSegInsideBit, sv.S - 1);  // S where no tensor follows: not used then
        nmp[u] = sv.neg_mu_pos[static_cast<size_t>(t) * P + p];
        mn[u] = sv.mu_neg[static_cast<size_t>(t) * P + p];
    }
    uint32_t bits = 0;
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u) {
        const uint64_t i = base + u * 64;
        if (i >= nvec) {
            bits <<= 4;
            continue;
        }
        const vf4 v = gv[u] + ev[u];
        const uint32_t s0 = entry[u] & ~kSegInsideBit;
        if (entry[u] & kSegInsideBit) {
            bits = push_signs(bits, v);
            const vf4 err = pending_error4(v, nmp[u], mn[u]);  // v - enc(v) with this tensor's means
            st4<NT>(e4 + i, err);
        } else {
            uint32_t sc[4];
            seg_of4(sv, s0, i << 2, sc);
            const float x[4] = {v.x, v.y, v.z, v.w};
            float err[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool in = sc[c] != sv.S;
                bits = bits * 2u + (in && x[c] >= 0.0f ? 1u : 0u);
                err[c] = in ? pending_error(x[c], sv.neg_mu_pos[static_cast<size_t>(sc[c]) * P + p],
                                            sv.mu_neg[static_cast<size_t>(sc[c]) * P + p])
                            : 0.0f;
            }
            if (sc[0] != sv.S && sc[1] != sv.S && sc[2] != sv.S && sc[3] != sv.S) {
                const vf4 out = vf4{err[0], err[1], err[2], err[3]};
                st4<NT>(e4 + i, out);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (sc[c] != sv.S)
                        e[(i << 2) + c] = err[c];
            }
        }
    }
    sign_row(sign, P, blockIdx.x / 2, blockIdx.x % 2, p)[lane] = static_cast<uint16_t>(bits);
}

// LAZY: the sign words are those of the lazy state's reduction and tab.g = tab.e = the state buffers, which hold v.
template <bool NT, int UP, bool LAZY>
__global__ __launch_bounds__(64) void k_seg_apply_signs(const PtrTable tab, const uint16_t *__restrict__ sign,
                                                        float *__restrict__ w, const uint64_t n, const uint64_t chunks,
                                                        const uint32_t P, const float eta_over_P, const SegView sv)
{
    const uint32_t lane = threadIdx.x;
    const uint64_t nvec = n >> 2;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * (64 * kSegSignItems) + lane;
    vf4 *w4 = reinterpret_cast<vf4 *>(w);
    vf4 wv[kSegSignItems];
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u)
        if (base + u * 64 < nvec)
            wv[u] = ld4<NT>(w4 + base + u * 64);
    // k[u][c]: how many workers have component c of group u in the positive group
    const uint16_t *half = sign + static_cast<uint64_t>(blockIdx.x) * P * 64 + lane;
    uint32_t k[kSegSignItems][4];
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u)
        k[u][0] = k[u][1] = k[u][2] = k[u][3] = 0;
    uint32_t p0 = 0;
    for (; p0 + UP <= P; p0 += UP) {
        uint32_t d[UP];
#pragma unroll
        for (int q = 0; q < UP; ++q)
            d[q] = half[(p0 + q) * 64];
#pragma unroll
        for (int q = 0; q < UP; ++q)
#pragma unroll
            for (int u = 0; u < kSegSignItems; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    k[u][c] += (d[q] >> (15u - (4u * u + c))) & 1u;
    }
    for (; p0 < P; ++p0) {
        const uint32_t d = half[p0 * 64];
#pragma unroll
        for (int u = 0; u < kSegSignItems; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                k[u][c] += (d >> (15u - (4u * u + c))) & 1u;
    }
    uint32_t entry[kSegSignItems];
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u) {
        const uint64_t c = static_cast<uint64_t>(blockIdx.x) * kSegSignItems + u;
        entry[u] = c < chunks ? sv.coarse[c] : 0u;
    }
    if (!seg_tables_ok(sv))
        return;
    const bool any_nan = sv.hdr->any_nan != 0;  // the same for the whole grid
    const float fP = static_cast<float>(P);
    float gp0[kSegSignItems], ngn0[kSegSignItems];  // global means of every chunk's first tensor, asked for at once
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u) {
        const uint32_t t = min(entry[u] & ~kSegInsideBit, sv.S - 1);
        gp0[u] = sv.gmu[2 * t];
        ngn0[u] = sv.gmu[2 * t + 1];
    }
#pragma unroll
    for (int u = 0; u < kSegSignItems; ++u) {
        const uint64_t i = base + u * 64;
        if (i >= nvec)
            continue;
        // acc: the sum over the workers of +gmu_pos or -gmu_neg of the element's tensor (the table keeps -gmu_neg)
        const uint32_t s0 = entry[u] & ~kSegInsideBit;
        uint32_t sc[4] = {s0, s0, s0, s0};
        float acc[4];
        if (entry[u] & kSegInsideBit) {  // one tensor for the whole chunk
#pragma unroll
            for (int c = 0; c < 4; ++c)
                acc[c] = static_cast<float>(k[u][c]) * (gp0[u] - ngn0[u]) + fP * ngn0[u];
        } else {
            seg_of4(sv, s0, i << 2, sc);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t t = sc[c] != sv.S ? sc[c] : 0u;
                const float gp = sv.gmu[2 * t], ngn = sv.gmu[2 * t + 1];
                acc[c] = static_cast<float>(k[u][c]) * (gp - ngn) + fP * ngn;
            }
        }
        if (any_nan) {
            // a NaN has no sign bit, but it left a NaN in that worker's new error: that element's update is NaN
            for (uint32_t p = 0; p < P; ++p) {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (sc[c] != sv.S) {
                        const float x = tab.e[p][(i << 2) + c];
                        acc[c] = (x != x) ? x : acc[c];
                    }
            }
        }
        const float x[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
        if (sc[0] != sv.S && sc[1] != sv.S && sc[2] != sv.S && sc[3] != sv.S) {
            const vf4 wn = vf4{x[0] - eta_over_P * acc[0], x[1] - eta_over_P * acc[1], x[2] - eta_over_P * acc[2],
                               x[3] - eta_over_P * acc[3]};
            st4<NT>(w4 + i, wn);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (sc[c] != sv.S)
                    w[(i << 2) + c] = x[c] - eta_over_P * acc[c];
        }
    }
    // the last n % 4 elements, which k_seg_error_signs left alone, get the whole of lines 4, 6 and 7 here (on the
    // lazy state: lines 6 and 7 from the stored v, which has no sign bit in the words)
    if (blockIdx.x == gridDim.x - 1 && lane < (n & 3)) {
        const uint64_t idx = (nvec << 2) + lane;
        const uint32_t s = seg_of(sv, sv.coarse[idx >> kSegCoarseShift] & ~kSegInsideBit, idx);
        if (sv.seg_start[s] <= idx)
            seg_apply_element<A2SGD_MODE_RETAINED_ERROR, !LAZY>(tab, w, idx, s, P, eta_over_P, sv);
    }
}

// One weight vector per worker on a plan with tensors (Algorithm 1 line 7 as each worker runs it, per tensor):
// w^p <- w^p - eta * u^p with the means of the element's tensor.  Same lookup as k_seg_apply; workers in groups of
// UP whose g, e and w^p loads are issued together.
template <int MODE, bool HAS_E>
__device__ __forceinline__ void seg_apply_element_replicas(const PtrTable &tab, const ReplicaTable &wt, const uint64_t idx,
                                                           const uint32_t s, const uint32_t P, const float eta,
                                                           const SegView &sv)
{
    const float gmu_pos = sv.gmu[2 * s], neg_gmu_neg = sv.gmu[2 * s + 1];
    for (uint32_t p = 0; p < P; ++p) {
        float v = tab.g[p][idx];
        if (HAS_E)
            v += tab.e[p][idx];
        const float u = apply1<MODE>(v, sv.neg_mu_pos[static_cast<size_t>(s) * P + p],
                                     sv.mu_neg[static_cast<size_t>(s) * P + p], gmu_pos, neg_gmu_neg);
        if (HAS_E)
            tab.e[p][idx] = v;
        wt.w[p][idx] -= eta * u;
    }
}

template <int MODE, bool HAS_E, bool NT, int UP, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_seg_apply_replicas(const PtrTable tab, const ReplicaTable wt, const uint64_t n,
                                                              const uint32_t P, const float eta, const SegView sv)
{
    const uint32_t tid = threadIdx.x;
    const uint64_t nvec = n >> 2;
    const uint64_t first = static_cast<uint64_t>(blockIdx.x) * BLOCK;
    const uint64_t i = first + tid;
    static_assert(BLOCK * 4 == (1 << kSegCoarseShift), "one lookup entry per apply workgroup");
    const uint32_t entry = sv.coarse[blockIdx.x];
    if (!seg_tables_ok(sv))
        return;
    if (i < nvec) {
        const uint32_t s0 = entry & ~kSegInsideBit;
        if (entry & kSegInsideBit) {
            const float *nmp = sv.neg_mu_pos + static_cast<size_t>(s0) * P;
            const float *mn = sv.mu_neg + static_cast<size_t>(s0) * P;
            const float gmu_pos = sv.gmu[2 * s0], neg_gmu_neg = sv.gmu[2 * s0 + 1];
            for (uint32_t p0 = 0; p0 < P; p0 += UP) {
                vf4 v[UP], ev[UP], wv[UP];
#pragma unroll
                for (int u = 0; u < UP; ++u)
                    if (p0 + u < P) {
                        v[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.g[p0 + u]) + i);
                        if (HAS_E)
                            ev[u] = ld4<NT>(reinterpret_cast<const vf4 *>(tab.e[p0 + u]) + i);
                        wv[u] = ld4<NT>(reinterpret_cast<const vf4 *>(wt.w[p0 + u]) + i);
                    }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < UP; ++u)
                    if (p0 + u < P) {
                        const vf4 vv = HAS_E ? v[u] + ev[u] : v[u];
                        vf4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
                        const vf4 err = apply4<MODE>(vv, upd, nmp[p0 + u], mn[p0 + u], gmu_pos, neg_gmu_neg);
                        if (HAS_E)
                            st4<NT>(reinterpret_cast<vf4 *>(tab.e[p0 + u]) + i, err);
                        const vf4 wn = wv[u] - eta * upd;
                        st4<NT>(reinterpret_cast<vf4 *>(wt.w[p0 + u]) + i, wn);
                    }
            }
        } else {
            // a boundary or padding inside the workgroup: element by element, padding is not touched
            uint32_t sx = s0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                sx = seg_of(sv, sx, (i << 2) + c);
                if (sv.seg_start[sx] <= (i << 2) + c)
                    seg_apply_element_replicas<MODE, HAS_E>(tab, wt, (i << 2) + c, sx, P, eta, sv);
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t idx = (nvec << 2) + tid;
        const uint32_t s = seg_of(sv, sv.coarse[idx >> kSegCoarseShift] & ~kSegInsideBit, idx);
        if (sv.seg_start[s] <= idx)
            seg_apply_element_replicas<MODE, HAS_E>(tab, wt, idx, s, P, eta, sv);
    }
}

// The same pass with one worker per workgroup, for many workers at streaming sizes (as k_apply_replicas_per_worker
// on whole-model plans: a workgroup has three buffers open instead of 3P).  grid = (workgroups of 512 elements, P);
// a workgroup covers two entries of the lookup table and asks for the means of both chunks' first tensors at once.
constexpr int kSegReplItems = 2;
template <int MODE, bool HAS_E, bool NT>
__global__ __launch_bounds__(64) void k_seg_apply_replicas_per_worker(const PtrTable tab, const ReplicaTable wt,
                                                                      const uint64_t n, const uint64_t chunks,
                                                                      const float eta, const SegView sv)
{
    const uint32_t p = blockIdx.y, P = gridDim.y, lane = threadIdx.x;
    const vf4 *__restrict__ g4 = reinterpret_cast<const vf4 *>(tab.g[p]);
    float *e = HAS_E ? tab.e[p] : nullptr;
    vf4 *e4 = reinterpret_cast<vf4 *>(e);
    float *w = wt.w[p];
    vf4 *w4 = reinterpret_cast<vf4 *>(w);
    const uint64_t nvec = n >> 2;
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * (64 * kSegReplItems) + lane;
    vf4 gv[kSegReplItems], ev[kSegReplItems], wv[kSegReplItems];
#pragma unroll
    for (int u = 0; u < kSegReplItems; ++u)
        if (base + u * 64 < nvec) {
            gv[u] = ld4<NT>(g4 + base + u * 64);
            if (HAS_E)
                ev[u] = ld4<NT>(e4 + base + u * 64);
            wv[u] = ld4<NT>(w4 + base + u * 64);
        }
    __builtin_amdgcn_sched_barrier(0);
    uint32_t entry[kSegReplItems];
#pragma unroll
    for (int u = 0; u < kSegReplItems; ++u) {
        const uint64_t c = static_cast<uint64_t>(blockIdx.x) * kSegReplItems + u;
        entry[u] = c < chunks ? sv.coarse[c] : 0u;
    }
    if (!seg_tables_ok(sv))
        return;
    float nmp[kSegReplItems], mn[kSegReplItems], gp[kSegReplItems], ngn[kSegReplItems];
#pragma unroll
    for (int u = 0; u < kSegReplItems; ++u) {
        const uint32_t t = min(entry[u] & ~kSegInsideBit, sv.S - 1);  // S where no tensor follows: not used then
        nmp[u] = sv.neg_mu_pos[static_cast<size_t>(t) * P + p];
        mn[u] = sv.mu_neg[static_cast<size_t>(t) * P + p];
        gp[u] = sv.gmu[2 * t];
        ngn[u] = sv.gmu[2 * t + 1];
    }
#pragma unroll
    for (int u = 0; u < kSegReplItems; ++u) {
        const uint64_t i = base + u * 64;
        if (i >= nvec)
            continue;
        const vf4 vv = HAS_E ? gv[u] + ev[u] : gv[u];
        if (entry[u] & kSegInsideBit) {  // one tensor for the whole chunk
            vf4 upd = {0.0f, 0.0f, 0.0f, 0.0f};
            const vf4 err = apply4<MODE>(vv, upd, nmp[u], mn[u], gp[u], ngn[u]);
            if (HAS_E)
                st4<NT>(e4 + i, err);
            const vf4 wn = wv[u] - eta * upd;
            st4<NT>(w4 + i, wn);
        } else {
            uint32_t sc[4];
            seg_of4(sv, entry[u] & ~kSegInsideBit, i << 2, sc);
            float x[4] = {vv.x, vv.y, vv.z, vv.w};
            const float wo[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
            float wn[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t t = sc[c] != sv.S ? sc[c] : 0u;
                const float upd = apply1<MODE>(x[c], sv.neg_mu_pos[static_cast<size_t>(t) * P + p],
                                               sv.mu_neg[static_cast<size_t>(t) * P + p], sv.gmu[2 * t], sv.gmu[2 * t + 1]);
                wn[c] = wo[c] - eta * upd;
            }
            if (sc[0] != sv.S && sc[1] != sv.S && sc[2] != sv.S && sc[3] != sv.S) {
                if (HAS_E) {
                    const vf4 err = vf4{x[0], x[1], x[2], x[3]};
                    st4<NT>(e4 + i, err);
                }
                const vf4 out = vf4{wn[0], wn[1], wn[2], wn[3]};
                st4<NT>(w4 + i, out);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (sc[c] != sv.S) {  // padding is not touched
                        if (HAS_E)
                            e[(i << 2) + c] = x[c];
                        w[(i << 2) + c] = wn[c];
                    }
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1 && lane < (n & 3)) {
        const uint64_t idx = (nvec << 2) + lane;
        const uint32_t t = seg_of(sv, sv.coarse[idx >> kSegCoarseShift] & ~kSegInsideBit, idx);
        if (sv.seg_start[t] <= idx) {
            float v = tab.g[p][idx];
            if (HAS_E)
                v += e[idx];
            const float upd = apply1<MODE>(v, sv.neg_mu_pos[static_cast<size_t>(t) * P + p],
                                           sv.mu_neg[static_cast<size_t>(t) * P + p], sv.gmu[2 * t], sv.gmu[2 * t + 1]);
            if (HAS_E)
                e[idx] = v;
            w[idx] -= eta * upd;
        }
    }
}

// Lazy state on a plan with tensors, back to true errors: s <- pending error of s with the carried means of the
// element's tensor.  grid = (workgroups of 64 float4 groups, P).
template <bool NT>
__global__ __launch_bounds__(64) void k_seg_materialize(const PtrTable tab, const uint64_t n, const SegView sv)
{
    const uint32_t p = blockIdx.y, P = gridDim.y, tid = threadIdx.x;
    const uint64_t nvec = n >> 2;
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 64 + tid;
    const uint32_t entry = sv.coarse[blockIdx.x];
    if (!seg_tables_ok(sv))
        return;
    float *s = tab.e[p];
    if (i < nvec) {
        const uint32_t s0 = entry & ~kSegInsideBit;
        vf4 *s4 = reinterpret_cast<vf4 *>(s) + i;
        if (entry & kSegInsideBit) {
            const vf4 err = pending_error4(ld4<NT>(s4), sv.neg_mu_pos[static_cast<size_t>(s0) * P + p],
                                           sv.mu_neg[static_cast<size_t>(s0) * P + p]);
            st4<NT>(s4, err);
        } else {
            uint32_t sx = s0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint64_t idx = (i << 2) + c;
                sx = seg_of(sv, sx, idx);
                if (sv.seg_start[sx] <= idx)
                    s[idx] = pending_error(s[idx], sv.neg_mu_pos[static_cast<size_t>(sx) * P + p],
                                           sv.mu_neg[static_cast<size_t>(sx) * P + p]);
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1 && tid < (n & 3)) {
        const uint64_t idx = (nvec << 2) + tid;
        const uint32_t sx = seg_of(sv, sv.coarse[idx >> kSegCoarseShift] & ~kSegInsideBit, idx);
        if (sv.seg_start[sx] <= idx)
            s[idx] = pending_error(s[idx], sv.neg_mu_pos[static_cast<size_t>(sx) * P + p],
                                   sv.mu_neg[static_cast<size_t>(sx) * P + p]);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Lazy error state on a plan with tensors: the reduction (Algorithm 1 line 3 per tensor on v = fl32(g + the pending
// error of the stored value, formed with the carried means of the element's tensor); v is written back in place of
// the stored value).  Because it stores, it has the one-shot shape of the whole-model form: grid = (blocks of
// kSegLazyElems elements by position, P), single wavefronts, all loads ahead of the first store.  A block that lies
// wholly inside one tensor takes that tensor's carried means for all its elements and leaves one record in the
// table of block records.  Any other block walks the tensors it touches: per tensor the elements inside it are
// folded, summed and counted (the others enter as NaN, which is counted nowhere), and the record goes straight into
// that tensor's first or last slot of the folded table.  Padding is neither written nor given a sign bit.
// With SIGNS the pass leaves pos(v) in the sign words, in the layout of k_seg_error_signs (both halves of a row).
// ---------------------------------------------------------------------------------------------------------
template <bool NT, bool SIGNS>
__global__ __launch_bounds__(64) void k_seg_lazy_partials(const PtrTable tab, const uint64_t n, const uint64_t chunks,
                                                          const SegView lv, const uint32_t blocks, const Partials rec,
                                                          const uint32_t sign_rows, uint16_t *__restrict__ sign)
{
    static_assert(4 * kSegLazyItems == 32, "one thread's sign bits fill two 16-bit halves");
    const uint32_t p = blockIdx.y, P = gridDim.y, b = blockIdx.x, lane = threadIdx.x;
    const float *__restrict__ g = tab.g[p];
    float *st = tab.e[p];
    const vf4 *__restrict__ g4 = reinterpret_cast<const vf4 *>(g);
    vf4 *s4 = reinterpret_cast<vf4 *>(st);
    const uint64_t nvec = n >> 2;
    constexpr uint64_t kPer = 64ull * kSegLazyItems;
    const uint64_t base = static_cast<uint64_t>(b) * kPer + lane;
    const bool full = (static_cast<uint64_t>(b) + 1) * kPer <= nvec;  // all float4 groups of the block exist
    vf4 gv[kSegLazyItems], sx[kSegLazyItems];
    if (full) {
#pragma unroll
        for (int u = 0; u < kSegLazyItems; ++u)
            gv[u] = ld4<NT>(g4 + base + u * 64);
#pragma unroll
        for (int u = 0; u < kSegLazyItems; ++u)
            sx[u] = ld4<NT>(s4 + base + u * 64);
    } else {
#pragma unroll
        for (int u = 0; u < kSegLazyItems; ++u) {
            const bool there = base + u * 64 < nvec;
            gv[u] = there ? ld4<NT>(g4 + base + u * 64) : vf4{0.0f, 0.0f, 0.0f, 0.0f};
            sx[u] = there ? ld4<NT>(s4 + base + u * 64) : vf4{0.0f, 0.0f, 0.0f, 0.0f};
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    static_assert(64 * 4 == (1 << kSegCoarseShift), "one lookup entry per 64 float4 groups");
    uint32_t entry[kSegLazyItems];
#pragma unroll
    for (int u = 0; u < kSegLazyItems; ++u) {
        const uint64_t c = static_cast<uint64_t>(b) * kSegLazyItems + u;
        entry[u] = c < chunks ? lv.coarse[c] : 0u;
    }
    if (!seg_tables_ok(lv))
        return;
    bool whole = full && (entry[0] & kSegInsideBit) != 0;  // the same for every thread of the block
#pragma unroll
    for (int u = 1; u < kSegLazyItems; ++u)
        whole = whole && entry[u] == entry[0];

    if (whole) {
        const uint32_t t = entry[0] & ~kSegInsideBit;
        const float nmp = lv.neg_mu_pos[static_cast<size_t>(t) * P + p], mn = lv.mu_neg[static_cast<size_t>(t) * P + p];
        LaneAcc acc;
        uint32_t bits = 0;
#pragma unroll
        for (int u = 0; u < kSegLazyItems; ++u) {
            const vf4 v = gv[u] + pending_error4(sx[u], nmp, mn);
            st4<NT>(s4 + base + u * 64, v);
            acc.add4(v);
            if (SIGNS)
                bits = push_signs(bits, v);
        }
        if (SIGNS) {
            sign_row(sign, P, b, 0, p)[lane] = static_cast<uint16_t>(bits >> 16);
            sign_row(sign, P, b, 1, p)[lane] = static_cast<uint16_t>(bits & 0xffffu);
        }
        acc.flush();
        Sums total;
        total.s_pos = wave_sum(acc.s_pos);
        total.s_neg = wave_sum(acc.s_neg);
        total.n_pos = acc.c_pos;
        total.n_neg = acc.c_neg;
        total.n_zero = acc.c_zero;
        if (lane == 0)
            store_record(rec, static_cast<size_t>(p) * blocks + b, total);
        return;
    }

    // A block with a tensor boundary, padding or the end of the buffers in it.
    const uint64_t blo = static_cast<uint64_t>(b) * kSegLazyElems, bhi = blo + kSegLazyElems;
    // the last n % 4 elements, outside every float4 group, belong to the block at their position: one per lane
    const uint64_t tail_idx = (nvec << 2) + lane;
    const bool tail_block = (n & 3) != 0 && (nvec << 2) >= blo && (nvec << 2) < bhi;  // uniform
    const bool tail_lane = tail_block && lane < (n & 3);
    const float tail_g = tail_lane ? g[tail_idx] : 0.0f, tail_s = tail_lane ? st[tail_idx] : 0.0f;
    float tail_v = 0.0f;
    bool tail_in = false;
    float out[kSegLazyItems][4];
    uint32_t inside = 0;  // bit 4 * u + c: the element belongs to a tensor and out[u][c] holds its v
#pragma unroll
    for (int u = 0; u < kSegLazyItems; ++u)
        out[u][0] = out[u][1] = out[u][2] = out[u][3] = 0.0f;
    const float nan = __builtin_nanf("");
    for (uint32_t t = entry[0] & ~kSegInsideBit; t < lv.S; ++t) {  // entry[0]: the first tensor that ends after blo
        const uint64_t ts = lv.seg_start[t], te = lv.seg_end[t];
        if (ts >= bhi)
            break;
        const float nmp = lv.neg_mu_pos[static_cast<size_t>(t) * P + p], mn = lv.mu_neg[static_cast<size_t>(t) * P + p];
        LaneAcc acc;
#pragma unroll
        for (int u = 0; u < kSegLazyItems; ++u) {
            const uint64_t clo = blo + u * 256ull;
            if (ts >= clo + 256 || te <= clo)  // this chunk has nothing of tensor t (uniform)
                continue;
            const uint64_t e0 = (base + u * 64) << 2;
            const bool there = base + u * 64 < nvec;
            const float x[4] = {gv[u].x, gv[u].y, gv[u].z, gv[u].w}, y[4] = {sx[u].x, sx[u].y, sx[u].z, sx[u].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool in = there && e0 + c >= ts && e0 + c < te;
                const float v = in ? x[c] + pending_error(y[c], nmp, mn) : nan;
                acc.add(v);
                out[u][c] = in ? v : out[u][c];
                inside |= in ? 1u << (4 * u + c) : 0u;
            }
        }
        if (tail_block) {
            const bool in = tail_lane && tail_idx >= ts && tail_idx < te;
            const float v = in ? tail_g + pending_error(tail_s, nmp, mn) : nan;
            acc.add(v);
            tail_v = in ? v : tail_v;
            tail_in = tail_in || in;
        }
        acc.flush();
        Sums total;
        total.s_pos = wave_sum(acc.s_pos);
        total.s_neg = wave_sum(acc.s_neg);
        total.n_pos = acc.c_pos;
        total.n_neg = acc.c_neg;
        total.n_zero = acc.c_zero;
        if (lane == 0) {
            // the block holds the tensor's first element (its first slot) or, failing that, its last one
            const uint32_t k = ts >= blo ? lv.item_lo[t] : lv.item_lo[t + 1] - 1;
            store_record(lv.rec, static_cast<size_t>(p) * lv.num_items + k, total);
        }
    }
    uint32_t bits = 0;
#pragma unroll
    for (int u = 0; u < kSegLazyItems; ++u) {
        const uint32_t m = (inside >> (4 * u)) & 15u;
        const uint64_t i = base + u * 64;
        if (m == 15u) {
            const vf4 v = vf4{out[u][0], out[u][1], out[u][2], out[u][3]};
            st4<NT>(s4 + i, v);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (m >> c & 1u)
                    st[(i << 2) + c] = out[u][c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c)
            bits = bits * 2u + ((m >> c & 1u) != 0 && out[u][c] >= 0.0f ? 1u : 0u);
    }
    if (tail_in)
        st[tail_idx] = tail_v;
    if (SIGNS && b < sign_rows) {
        sign_row(sign, P, b, 0, p)[lane] = static_cast<uint16_t>(bits >> 16);
        sign_row(sign, P, b, 1, p)[lane] = static_cast<uint16_t>(bits & 0xffffu);
    }
}

// Between that pass and the second level: workgroup (j, p) adds the block records [lo, hi) of fold entry j in a
// fixed order (strided per thread, shuffle tree, wavefronts in index order) into its slot of the folded table; an
// empty range clears the slot.
__global__ __launch_bounds__(kBlock) void k_seg_lazy_fold(const SegFold *__restrict__ fold, const uint32_t blocks,
                                                          const Partials in, const SegView lv)
{
    const uint32_t p = blockIdx.y, tid = threadIdx.x;
    if (!seg_tables_ok(lv))
        return;
    const SegFold f = fold[blockIdx.x];
    const size_t row = static_cast<size_t>(p) * blocks;
    Sums mine;
    for (uint32_t k = f.lo + tid; k < f.hi; k += kBlock)
        add_record(mine, in, row + k);
    const Sums total = block_sum(mine);
    if (tid == 0)
        store_record(lv.rec, static_cast<size_t>(p) * lv.num_items + f.slot, total);
}

// Clears the carried means of every tensor and worker: from here on the state buffers are read as true errors.
__global__ __launch_bounds__(256) void k_seg_lazy_reset(const uint64_t entries, const SegView sv)
{
    const uint64_t k = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (k < entries) {
        sv.neg_mu_pos[k] = 0.0f;
        sv.mu_neg[k] = 0.0f;
    }
}

// ---------------------------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------------------------

hipError_t launch_seg_partials(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, void *ws, hipStream_t s)
{
    const SegView sv = seg_view(pl, ws);
    const dim3 grid(pl.seg.blocks, pl.P), block(kBlock);
    if (has_e) {
        if (pl.streaming)
            k_seg_partials<true, true><<<grid, block, 0, s>>>(tab, sv);
        else
            k_seg_partials<true, false><<<grid, block, 0, s>>>(tab, sv);
    } else {
        if (pl.streaming)
            k_seg_partials<false, true><<<grid, block, 0, s>>>(tab, sv);
        else
            k_seg_partials<false, false><<<grid, block, 0, s>>>(tab, sv);
    }
    return hipGetLastError();
}

// The tables as the lazy state's second level sees them: a tensor's records are its slots of the folded table.
static SegView seg_lazy_view(const a2sgd_plan_t &pl, void *ws)
{
    char *b = static_cast<char *>(ws);
    const SegPlan &sp = pl.seg;
    SegView v = seg_view(pl, ws);
    v.num_items = sp.lz_slot_lo[sp.S];
    v.item = nullptr;  // the lazy passes go by position, not by item
    v.item_lo = reinterpret_cast<const uint32_t *>(b + sp.off_lz_slot_lo);
    v.rec = partials_at(ws, sp.off_lz_folded, pl.P, v.num_items);
    return v;
}

hipError_t launch_seg_lazy_partials(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s)
{
    const SegPlan &sp = pl.seg;
    const SegView lv = seg_lazy_view(pl, ws);
    const Partials rec = partials_at(ws, sp.off_lz_records, pl.P, sp.lz_blocks);
    const SegFold *fold = reinterpret_cast<const SegFold *>(static_cast<char *>(ws) + sp.off_lz_fold);
    uint16_t *sign = reinterpret_cast<uint16_t *>(static_cast<char *>(ws) + sp.off_sign);
    const uint64_t chunks = (pl.n + (1ull << kSegCoarseShift) - 1) >> kSegCoarseShift;
    const bool signs = pl.mode == A2SGD_MODE_RETAINED_ERROR;  // the literal mode's apply pass needs v itself
    const dim3 grid(sp.lz_blocks, pl.P), block(64);
    const uint32_t lds = kSegLazyLds;
    if (pl.streaming) {
        if (signs)
            k_seg_lazy_partials<true, true><<<grid, block, lds, s>>>(tab, pl.n, chunks, lv, sp.lz_blocks, rec, pl.lazy_blocks, sign);
        else
            k_seg_lazy_partials<true, false><<<grid, block, lds, s>>>(tab, pl.n, chunks, lv, sp.lz_blocks, rec, pl.lazy_blocks, sign);
    } else {
        if (signs)
            k_seg_lazy_partials<false, true><<<grid, block, 0, s>>>(tab, pl.n, chunks, lv, sp.lz_blocks, rec, pl.lazy_blocks, sign);
        else
            k_seg_lazy_partials<false, false><<<grid, block, 0, s>>>(tab, pl.n, chunks, lv, sp.lz_blocks, rec, pl.lazy_blocks, sign);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    if (!sp.lz_fold.empty()) {  // empty if no tensor has a block to itself and every first and last slot is in use
        k_seg_lazy_fold<<<dim3(static_cast<uint32_t>(sp.lz_fold.size()), pl.P), dim3(kBlock), 0, s>>>(fold, sp.lz_blocks, rec, lv);
        if ((err = hipGetLastError()) != hipSuccess)
            return err;
    }
    if (sp.pooled)
        k_seg_finalize_pooled<<<dim3(pl.P), dim3(kBlock), 0, s>>>(lv, sp.covered);
    else
        k_seg_finalize<<<dim3(lv.S, pl.P), dim3(64), 0, s>>>(lv);
    return hipGetLastError();
}

hipError_t launch_seg_lazy_apply_signs(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eta, void *ws,
                                       hipStream_t s)
{
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    const SegView sv = seg_view(pl, ws);
    const uint16_t *sign = reinterpret_cast<const uint16_t *>(static_cast<char *>(ws) + pl.seg.off_sign);
    const uint64_t chunks = (pl.n + (1ull << kSegCoarseShift) - 1) >> kSegCoarseShift;
    const dim3 grid(pl.lazy_blocks * 2), block(64);  // workgroups of 1024 elements: two per row of sign words
    const uint32_t lds = pl.streaming ? 8 * 1024 : 0;
#define A2SGD_SEG_LAZY_SIGNS(NT, UP) \
    k_seg_apply_signs<NT, UP, true><<<grid, block, lds, s>>>(tab, sign, w, pl.n, chunks, pl.P, eop, sv)
    if (pl.streaming) {
        if (pl.P >= 16)
            A2SGD_SEG_LAZY_SIGNS(true, 16);
        else if (pl.P >= 8)
            A2SGD_SEG_LAZY_SIGNS(true, 8);
        else
            A2SGD_SEG_LAZY_SIGNS(true, 4);
    } else {
        if (pl.P >= 8)
            A2SGD_SEG_LAZY_SIGNS(false, 8);
        else
            A2SGD_SEG_LAZY_SIGNS(false, 4);
    }
#undef A2SGD_SEG_LAZY_SIGNS
    return hipGetLastError();
}

hipError_t launch_seg_mark(const a2sgd_plan_t &pl, void *ws, hipStream_t s)
{
    k_seg_mark<<<dim3(1), dim3(64), 0, s>>>(static_cast<WsHeader *>(ws), pl.seg.tag);
    return hipGetLastError();
}

hipError_t launch_seg_finalize(const a2sgd_plan_t &pl, void *ws, hipStream_t s)
{
    const SegView sv = seg_view(pl, ws);
    if (pl.seg.pooled)
        k_seg_finalize_pooled<<<dim3(pl.P), dim3(kBlock), 0, s>>>(sv, pl.seg.covered);
    else
        k_seg_finalize<<<dim3(sv.S, pl.P), dim3(64), 0, s>>>(sv);
    return hipGetLastError();
}

hipError_t launch_seg_global(const a2sgd_plan_t &pl, void *ws, hipStream_t s)
{
    const SegView sv = seg_view(pl, ws);
    k_seg_global<<<dim3((sv.S + 63) / 64), dim3(64), 0, s>>>(pl.P, sv);
    return hipGetLastError();
}

template <int MODE, bool HAS_E, bool NT>
static hipError_t launch_seg_apply_shape(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop,
                                         const SegView &sv, hipStream_t s)
{
    constexpr int kThreads = 64;
    const uint64_t nvec = (pl.n + 3) >> 2;
    const dim3 grid(static_cast<uint32_t>((nvec + kThreads - 1) / kThreads)), block(kThreads);
    // The segment lookup sits between a workgroup's big loads and its arithmetic and makes it live longer, so more
    // workgroups per CU are wanted than in k_apply for the same bytes in flight (measured best: 11 instead of 6 at
    // P = 4, 11 instead of 4 at P = 8, 8 instead of 3 at P = 16).
    uint32_t lds = 0;
    if (pl.streaming)
        lds = pl.P >= 16 ? 20 * 1024 : pl.P >= 4 ? 14 * 1024 : 10 * 1024;
    if (pl.apply.up == 8)
        k_seg_apply<MODE, HAS_E, NT, 8, kThreads><<<grid, block, lds, s>>>(tab, w, pl.n, pl.P, eop, sv);
    else
        k_seg_apply<MODE, HAS_E, NT, 4, kThreads><<<grid, block, lds, s>>>(tab, w, pl.n, pl.P, eop, sv);
    return hipGetLastError();
}

static hipError_t launch_seg_apply_two_kernels(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eop,
                                               const SegView &sv, void *ws, hipStream_t s)
{
    uint16_t *sign = reinterpret_cast<uint16_t *>(static_cast<char *>(ws) + pl.seg.off_sign);
    const uint64_t chunks = (pl.n + (1ull << kSegCoarseShift) - 1) >> kSegCoarseShift;
    const uint32_t halves = pl.lazy_blocks * 2;  // workgroups of 1024 elements: two per row of sign words
    // The lookup (table entries, then the means they point to) leaves a workgroup with nothing in flight for a while,
    // so more of them share a compute unit than in the whole-model form: 13 per CU at 16 workers and more, 16 below
    // (measured at configs 4 and 2: 4.18 ms against 5.06 ms and 0.417 ms against 0.510 ms with the whole-model
    // form's 8 per CU).
    const uint32_t lds = pl.P >= 16 ? 12 * 1024 : 10 * 1024;
    k_seg_error_signs<true><<<dim3(halves, pl.P), dim3(64), lds, s>>>(tab, pl.n, chunks, sv, sign);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    if (pl.P >= 16)
        k_seg_apply_signs<true, 16, false><<<dim3(halves), dim3(64), 8 * 1024, s>>>(tab, sign, w, pl.n, chunks, pl.P, eop, sv);
    else
        k_seg_apply_signs<true, 8, false><<<dim3(halves), dim3(64), 8 * 1024, s>>>(tab, sign, w, pl.n, chunks, pl.P, eop, sv);
    return hipGetLastError();
}

hipError_t launch_seg_apply(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                            hipStream_t s)
{
    const float eop = static_cast<float>(static_cast<double>(eta) / static_cast<double>(pl.P));
    const SegView sv = seg_view(pl, ws);
    const bool lit = pl.mode == A2SGD_MODE_ALG1_LITERAL;
    if (pl.apply.two_kernels && !lit && has_e)
        return launch_seg_apply_two_kernels(pl, tab, w, eop, sv, ws, s);
#define A2SGD_SEG_CASE(L, E, N)                                                                                  \
    if (lit == L && has_e == E && pl.streaming == N)                                                             \
        return launch_seg_apply_shape<L ? A2SGD_MODE_ALG1_LITERAL : A2SGD_MODE_RETAINED_ERROR, E, N>(pl, tab, w, eop, \
                                                                                                     sv, s);
    A2SGD_SEG_CASE(false, true, true)
    A2SGD_SEG_CASE(false, true, false)
    A2SGD_SEG_CASE(false, false, true)
    A2SGD_SEG_CASE(false, false, false)
    A2SGD_SEG_CASE(true, true, true)
    A2SGD_SEG_CASE(true, true, false)
    A2SGD_SEG_CASE(true, false, true)
    A2SGD_SEG_CASE(true, false, false)
#undef A2SGD_SEG_CASE
    return hipErrorInvalidValue;
}

template <int MODE, bool HAS_E, bool NT>
static hipError_t launch_seg_apply_replicas_shape(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt,
                                                  float eta, const SegView &sv, hipStream_t s)
{
    constexpr int kThreads = 64;
    const uint64_t nvec = (pl.n + 3) >> 2;
    if (NT && pl.P >= kPerWorkerReplicas) {
        // one worker per workgroup, 13 workgroups per CU (measured, whole replica step in ms at configs 4 / 2 with
        // per-tensor means: grouped form 10.73 / 0.953; this form with 26, 20, 16, 13, 10, 8 workgroups per CU 10.72 /
        // 0.913, 9.91 / 0.911, 10.04 / 0.901, 9.34 / 0.875, 9.55 / 0.913, 9.88 / 0.952)
        const uint64_t chunks = (pl.n + (1ull << kSegCoarseShift) - 1) >> kSegCoarseShift;
        const uint64_t per = 64ull * kSegReplItems;
        const dim3 per_worker(static_cast<uint32_t>((nvec + per - 1) / per), pl.P);
        k_seg_apply_replicas_per_worker<MODE, HAS_E, NT><<<per_worker, dim3(64), 12 * 1024, s>>>(tab, wt, pl.n, chunks, eta, sv);
        return hipGetLastError();
    }
    const dim3 grid(static_cast<uint32_t>((nvec + kThreads - 1) / kThreads)), block(kThreads);
    const uint32_t lds = pl.streaming ? 14 * 1024 : 0;  // 11 workgroups per CU, as the shared-weight pass at P = 4
    if (pl.P >= 4)
        k_seg_apply_replicas<MODE, HAS_E, NT, 4, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eta, sv);
    else
        k_seg_apply_replicas<MODE, HAS_E, NT, 2, kThreads><<<grid, block, lds, s>>>(tab, wt, pl.n, pl.P, eta, sv);
    return hipGetLastError();
}

hipError_t launch_seg_apply_replicas(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt, bool has_e,
                                     float eta, void *ws, hipStream_t s)
{
    const SegView sv = seg_view(pl, ws);
    const bool lit = pl.mode == A2SGD_MODE_ALG1_LITERAL;
#define A2SGD_SEG_REPL_CASE(L, E, N)                                                                                  \
    if (lit == L && has_e == E && pl.streaming == N)                                                                  \
        return launch_seg_apply_replicas_shape<L ? A2SGD_MODE_ALG1_LITERAL : A2SGD_MODE_RETAINED_ERROR, E, N>(pl, tab, wt, \
                                                                                                              eta, sv, s);
    A2SGD_SEG_REPL_CASE(false, true, true)
    A2SGD_SEG_REPL_CASE(false, true, false)
    A2SGD_SEG_REPL_CASE(false, false, true)
    A2SGD_SEG_REPL_CASE(false, false, false)
    A2SGD_SEG_REPL_CASE(true, true, true)
    A2SGD_SEG_REPL_CASE(true, true, false)
    A2SGD_SEG_REPL_CASE(true, false, true)
    A2SGD_SEG_REPL_CASE(true, false, false)
#undef A2SGD_SEG_REPL_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_seg_lazy_reset(const a2sgd_plan_t &pl, void *ws, hipStream_t s)
{
    const SegView sv = seg_view(pl, ws);
    const uint64_t entries = static_cast<uint64_t>(sv.S) * pl.P;
    k_seg_lazy_reset<<<dim3(static_cast<uint32_t>((entries + 255) / 256)), dim3(256), 0, s>>>(entries, sv);
    return hipGetLastError();
}

hipError_t launch_seg_materialize(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s)
{
    const SegView sv = seg_view(pl, ws);
    const uint64_t nvec = (pl.n + 3) >> 2;
    const dim3 grid(static_cast<uint32_t>((nvec + 63) / 64), pl.P), block(64);
    if (pl.streaming)
        k_seg_materialize<true><<<grid, block, 12 * 1024, s>>>(tab, pl.n, sv);
    else
        k_seg_materialize<false><<<grid, block, 0, s>>>(tab, pl.n, sv);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return err;
    return launch_seg_lazy_reset(pl, ws, s);
}

}  // namespace a2sgd
