// Host side of the C ABI declared in include/a2sgd.h: plan construction, argument validation, and the
// sequencing of the kernels of one step.  No device memory is allocated here.
#include <stddef.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "a2sgd_internal.h"

using namespace a2sgd;

// Scratch memory for a2sgd_step_static, whose callers cannot allocate: the workspace of the three eager passes
// (header and block partial records) in a fixed array that every GPU the library runs on holds until the process
// ends.  In host code the array's name is only a handle for the runtime, not a device address.
constexpr size_t kStaticScratchBytes = A2SGD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// One workgroup of the apply-type passes covers as little as 64 float4 groups and a grid holds fewer than 2^31
// workgroups: n up to 2^38 (1 TiB per buffer) keeps every grid below 2^30.
constexpr uint64_t kMaxN = 1ull << 38;
// Compute units of one MI355X, for the geometry that a plan fixes on the host.  Both big passes run fastest with
// few wavefronts per compute unit, each with many 128-bit loads in flight (about 60 KiB in flight per CU); more
// wavefronts only widen the span of addresses that is open at once and HBM efficiency drops.  The reduction keeps
// 2 workgroups of 256 threads per CU.
constexpr uint32_t kComputeUnits = 256;
constexpr uint32_t kReduceBlocksPerCU = 2;
// The single-launch step asks for at most this many workgroups of kFusedBlock threads; a2sgd_step launches it only
// on a device that has at least as many compute units as the plan's grid has workgroups.  Its kernels are built for
// two workgroups per compute unit (launch bounds), so one grid is resident as a whole even next to a second one:
// that is what its grid-wide barrier relies on.
constexpr uint32_t kFusedGridMax = 256;

// The apply pass runs single-wavefront workgroups and caps how many share a CU through its dynamic-LDS request
// (160 KiB per CU; the request sits in the middle of the range that yields the wanted count).  A wavefront has
// items * (2 * up + 1) float4 loads per lane in flight, so fewer wavefronts are wanted when up is larger: the
// product stays at 50 to 70 KiB in flight per CU.
uint32_t apply_lds_bytes(uint32_t P)
{
    if (P >= 16)
        return 48 * 1024;  // 3 per CU
    if (P >= 8)
        return 36 * 1024;  // 4 per CU
    if (P >= 4)
        return 25 * 1024;  // 6 per CU
    return 16 * 1024;      // 10 per CU
}
// The dense step has items * (up + 1) loads per lane in flight (items = 2), about half of what the apply pass has,
// and takes its workers in groups of at most 8 one after the other, so from 8 workers on it wants more workgroups
// per CU than the apply pass (measured: config 4, 16 workers, 1.97 ms with 3 per CU, 1.82 with 6, 1.75 with 10,
// 1.69 with 13, 1.71 with 16 and more; config 2, 8 workers, 0.169 ms with 4 per CU, 0.160 with 6, 0.161 with 8
// to 11, 0.164 with 13 and more; config 5, 4 workers, best with 6).
uint32_t dense_lds_bytes(uint32_t P)
{
    if (P >= 16)
        return 12 * 1024;  // 13 per CU
    if (P >= 4)
        return 25 * 1024;  // 6 per CU
    return P >= 2 ? 16 * 1024 : 12 * 1024;  // 10 and 13 per CU
}
// Above this many bytes of g + e + w the step cannot live in the 256 MiB last-level cache between its two
// passes, and every load and store is issued as non-temporal.
constexpr uint64_t kStreamingBytes = 192ull << 20;

constexpr uint32_t kMaxSegments = 1u << 20;
constexpr uint32_t kTwoKernelWorkers = 8;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Static tables of a per-tensor plan: segment ends, work items of at most kSegItemElems elements that stay
// inside one segment, the items of each segment, a coarse element -> segment lookup; and where all of that, the
// per-segment results and the partial records live in the workspace.
void build_segments(a2sgd_plan_t &pl, uint32_t S, const uint64_t *len, const uint64_t *start, bool pooled)
{
    SegPlan &sp = pl.seg;
    sp.S = S;
    sp.pooled = pooled;
    sp.seg_start.resize(S + 1);
    sp.seg_end.resize(S + 1);
    sp.item_lo.resize(S + 1);
    uint64_t packed = 0;
    sp.covered = 0;
    for (uint32_t s = 0; s < S; ++s) {
        const uint64_t off = start ? start[s] : packed;
        sp.item_lo[s] = static_cast<uint32_t>(sp.item.size());
        for (uint64_t lo = off; lo < off + len[s]; lo += kSegItemElems) {
            const uint64_t left = off + len[s] - lo;
            sp.item.push_back(SegItem{lo, static_cast<uint32_t>(left < kSegItemElems ? left : kSegItemElems), s});
        }
        sp.seg_start[s] = off;
        sp.seg_end[s] = off + len[s];
        packed = off + len[s];
        sp.covered += len[s];
    }
    sp.seg_start[S] = sp.seg_end[S] = ~0ull;  // sentinel: ends the forward scans, contains no element
    sp.item_lo[S] = static_cast<uint32_t>(sp.item.size());
    const uint64_t chunks = (pl.n + (1ull << kSegCoarseShift) - 1) >> kSegCoarseShift;
    sp.coarse.resize(chunks);
    uint32_t s = 0;
    const uint64_t vec_end = pl.n & ~3ull;  // the apply pass takes the last n % 4 elements one by one
    for (uint64_t c = 0; c < chunks; ++c) {
        const uint64_t idx = c << kSegCoarseShift;
        while (sp.seg_end[s] <= idx)
            ++s;
        // top bit: the chunk's float4 groups all lie inside segment s (the apply pass then needs no bounds)
        uint64_t last = idx + (1ull << kSegCoarseShift);
        last = (last < vec_end ? last : vec_end) - 1;
        const bool inside = vec_end > idx && sp.seg_start[s] <= idx && sp.seg_end[s] > last;
        sp.coarse[c] = s | (inside ? kSegInsideBit : 0u);
    }
    // Which workgroup of the reduction takes which items: the items differ in size (a tensor's last item, small
    // tensors), so they are dealt out largest first, each to the workgroup with the least work so far; a workgroup
    // then walks its items in address order.  The result does not depend on the deal: every item has its own record.
    const uint32_t num_items = static_cast<uint32_t>(sp.item.size());
    sp.blocks = pl.B < num_items ? pl.B : num_items;
    {
        std::vector<uint32_t> order(num_items);
        for (uint32_t i = 0; i < num_items; ++i)
            order[i] = i;
        std::stable_sort(order.begin(), order.end(),
                         [&](uint32_t a, uint32_t b) { return sp.item[a].count > sp.item[b].count; });
        std::vector<std::vector<uint32_t>> mine(sp.blocks);
        // (load, workgroup) min-heap
        std::vector<std::pair<uint64_t, uint32_t>> heap(sp.blocks);
        for (uint32_t b = 0; b < sp.blocks; ++b)
            heap[b] = {0, b};
        auto later = [](const std::pair<uint64_t, uint32_t> &x, const std::pair<uint64_t, uint32_t> &y) { return x > y; };
        std::make_heap(heap.begin(), heap.end(), later);
        for (uint32_t i : order) {
            std::pop_heap(heap.begin(), heap.end(), later);
            auto &least = heap.back();
            mine[least.second].push_back(i);
            least.first += sp.item[i].count + 256;  // a fixed cost per item for its block reduction and record
            std::push_heap(heap.begin(), heap.end(), later);
        }
        sp.sched_lo.assign(sp.blocks + 1, 0);
        sp.sched_item.clear();
        sp.sched_item.reserve(num_items);
        for (uint32_t b = 0; b < sp.blocks; ++b) {
            std::sort(mine[b].begin(), mine[b].end());
            sp.sched_lo[b] = static_cast<uint32_t>(sp.sched_item.size());
            sp.sched_item.insert(sp.sched_item.end(), mine[b].begin(), mine[b].end());
        }
        sp.sched_lo[sp.blocks] = static_cast<uint32_t>(sp.sched_item.size());
    }
    // Items of the single-launch step: only for models that stay in the caches, with one pair of means per tensor.
    if (!pl.streaming && !pooled) {
        sp.fitem_lo.resize(S + 1);
        for (uint32_t k = 0; k < S; ++k) {
            sp.fitem_lo[k] = static_cast<uint32_t>(sp.fitem.size());
            for (uint64_t lo = sp.seg_start[k]; lo < sp.seg_end[k]; lo += kFusedItemElems) {
                const uint64_t left = sp.seg_end[k] - lo;
                sp.fitem.push_back(SegItem{lo, static_cast<uint32_t>(left < kFusedItemElems ? left : kFusedItemElems), k});
            }
        }
        sp.fitem_lo[S] = static_cast<uint32_t>(sp.fitem.size());
    }
    // The lazy state's reduction: which blocks lie wholly inside one tensor (the kernel decides the same way, from
    // the same lookup entries), and from that every tensor's slots in the folded table and the folds that fill them.
    {
        const uint64_t elems = kSegLazyElems, per = elems / 4, nvec = pl.n >> 2;
        sp.lz_blocks = static_cast<uint32_t>((pl.n + elems - 1) / elems);
        auto whole = [&](uint64_t b) {
            if ((b + 1) * per > nvec)
                return false;
            const uint32_t first = sp.coarse[b * kSegLazyItems];
            for (int u = 1; u < kSegLazyItems; ++u)
                if (sp.coarse[b * kSegLazyItems + u] != first)
                    return false;
            return (first & kSegInsideBit) != 0;
        };
        sp.lz_slot_lo.resize(S + 1);
        uint32_t slot = 0;
        for (uint32_t k = 0; k < S; ++k) {
            sp.lz_slot_lo[k] = slot;
            const uint64_t f = sp.seg_start[k] / elems, l = (sp.seg_end[k] - 1) / elems;
            const bool f_whole = whole(f), l_whole = whole(l);
            if (f_whole)  // the tensor starts on a block of its own: nothing is left in its first slot
                sp.lz_fold.push_back(SegFold{slot, 0, 0});
            ++slot;
            const uint64_t lo = f + (f_whole ? 0 : 1), hi = l + (l_whole ? 1 : 0);
            for (uint64_t x = lo; x < hi; x += kSegFoldSpan)
                sp.lz_fold.push_back(SegFold{slot++, static_cast<uint32_t>(x),
                                             static_cast<uint32_t>(x + kSegFoldSpan < hi ? x + kSegFoldSpan : hi)});
            if (l == f || l_whole)  // no shared last block
                sp.lz_fold.push_back(SegFold{slot, 0, 0});
            ++slot;
        }
        sp.lz_slot_lo[S] = slot;
    }
    size_t o = pl.workspace_bytes;  // after the header and the whole-model partials region
    o = align_up(o, 256);
    sp.off_seg_start = o;
    o = align_up(o + 8ull * (S + 1), 256);
    sp.off_seg_end = o;
    o = align_up(o + 8ull * (S + 1), 256);
    sp.off_item = o;
    o = align_up(o + sizeof(SegItem) * sp.item.size(), 256);
    sp.off_item_lo = o;
    o = align_up(o + 4ull * (S + 1), 256);
    sp.off_coarse = o;
    o = align_up(o + 4ull * chunks, 256);
    sp.off_sched_lo = o;
    o = align_up(o + 4ull * (sp.blocks + 1), 256);
    sp.off_sched_item = o;
    o = align_up(o + 4ull * num_items, 256);
    sp.off_stats = o;
    o = align_up(o + sizeof(a2sgd_worker_stats_t) * pl.P * S, 256);
    sp.off_nmp = o;
    o = align_up(o + 4ull * S * pl.P, 256);
    sp.off_mn = o;
    o = align_up(o + 4ull * S * pl.P, 256);
    sp.off_gmu = o;
    o = align_up(o + 8ull * S, 256);
    sp.off_records = o;
    o = align_up(o + 5ull * 8ull * pl.P * sp.item.size(), 256);
    sp.off_lz_slot_lo = o;
    o = align_up(o + 4ull * (S + 1), 256);
    sp.off_lz_fold = o;
    o = align_up(o + sizeof(SegFold) * sp.lz_fold.size(), 256);
    sp.off_lz_records = o;
    o = align_up(o + 5ull * 8ull * pl.P * sp.lz_blocks, 256);
    sp.off_lz_folded = o;
    o = align_up(o + 5ull * 8ull * pl.P * sp.lz_slot_lo[S], 256);
    if (!sp.fitem.empty()) {
        sp.off_fitem = o;
        o = align_up(o + sizeof(SegItem) * sp.fitem.size(), 256);
        sp.off_fitem_lo = o;
        o = align_up(o + 4ull * (S + 1), 256);
        sp.off_frecords = o;
        o = align_up(o + 5ull * 8ull * pl.P * sp.fitem.size(), 256);
    }
    if (pl.mode == A2SGD_MODE_RETAINED_ERROR) {  // one sign bit per element and worker, for the lazy state and the
        sp.off_sign = o;                         // two-kernel apply pass: the last thing in the workspace
        o += 4ull * pl.P * (64ull * pl.lazy_blocks);
    }
    sp.end = o;
}

inline bool segmented(const a2sgd_plan_t *plan) { return plan->seg.S > 0; }

// Checksum of a per-tensor plan's tables and of the sizes that fix where they lie in the workspace (FNV-1a over
// 64-bit words).  a2sgd_workspace_init leaves it in the workspace; the kernels that index through the tables
// compare it first.  Never 0, which is what fresh device memory most often holds.
uint64_t tag_words(uint64_t h, const void *data, size_t bytes)
{
    const unsigned char *p = static_cast<const unsigned char *>(data);
    for (size_t i = 0; i < bytes; i += 8) {
        uint64_t word = 0;
        for (size_t k = 0; k < 8 && i + k < bytes; ++k)
            word |= static_cast<uint64_t>(p[i + k]) << (8 * k);
        h = (h ^ word) * 0x100000001b3ull;
    }
    return h;
}

uint64_t tables_tag(const a2sgd_plan_t &pl)
{
    const SegPlan &sp = pl.seg;
    const uint64_t sizes[] = {pl.n, pl.P, sp.S, sp.item.size(), sp.blocks, sp.pooled ? 1u : 0u, sp.end};
    uint64_t h = 0xcbf29ce484222325ull;
    h = tag_words(h, sizes, sizeof(sizes));
    h = tag_words(h, sp.seg_start.data(), 8 * sp.seg_start.size());
    h = tag_words(h, sp.seg_end.data(), 8 * sp.seg_end.size());
    h = tag_words(h, sp.item.data(), sizeof(SegItem) * sp.item.size());
    h = tag_words(h, sp.item_lo.data(), 4 * sp.item_lo.size());
    h = tag_words(h, sp.coarse.data(), 4 * sp.coarse.size());
    h = tag_words(h, sp.sched_lo.data(), 4 * sp.sched_lo.size());
    h = tag_words(h, sp.sched_item.data(), 4 * sp.sched_item.size());
    h = tag_words(h, sp.fitem.data(), sizeof(SegItem) * sp.fitem.size());
    h = tag_words(h, sp.fitem_lo.data(), 4 * sp.fitem_lo.size());
    h = tag_words(h, sp.lz_slot_lo.data(), 4 * sp.lz_slot_lo.size());
    h = tag_words(h, sp.lz_fold.data(), sizeof(SegFold) * sp.lz_fold.size());
    return h != 0 ? h : 1;
}

// The grid-barrier cells of the single-launch step: kBarrierSlots of them in device memory (every GPU has its own
// copy of the array; the hand-out is per process, which is the stricter rule).  A plan that can use the single
// launch takes a free cell when it is made and gives it back when it is destroyed, so no two live plans ever
// share one; a plan that finds none runs the three passes, which give the same results.
class CellPool {
public:
    int take()
    {
        std::lock_guard<std::mutex> lock(mutex_);
        for (uint32_t c = 0; c < kBarrierSlots; ++c)
            if (!(busy_ >> c & 1ull)) {
                busy_ |= 1ull << c;
                return static_cast<int>(c);
            }
        return -1;
    }
    void give(int c)
    {
        std::lock_guard<std::mutex> lock(mutex_);
        if (c >= 0 && c < static_cast<int>(kBarrierSlots))
            busy_ &= ~(1ull << c);
    }

private:
    static_assert(kBarrierSlots == 64, "one bit per cell");
    std::mutex mutex_;
    uint64_t busy_ = 0;
};
CellPool g_cells;
std::atomic<uint32_t> g_next_token{1};

// Compute units of the current device, asked once per device; 0 if it cannot be told.
uint32_t current_device_compute_units()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<uint32_t> cached[kMaxDevices];
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices)
        return 0;
    uint32_t cu = cached[device].load(std::memory_order_relaxed);
    if (cu == 0) {
        int value = 0;
        if (hipDeviceGetAttribute(&value, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || value <= 0)
            return 0;
        cu = static_cast<uint32_t>(value);
        cached[device].store(cu, std::memory_order_relaxed);
    }
    return cu;
}

// The device address of `scratch` on the current device: asked for once per device, with that device current, and
// kept; every later use of the array's memory in host code goes through this address, never through the name.
a2sgd_status_t static_scratch(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static void *address[kMaxDevices];  // zero-initialised: not asked yet
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices)
        return A2SGD_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mutex);
    if (address[device] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr)
            return A2SGD_ERR_DEVICE;
        address[device] = ptr;
    }
    *out = address[device];
    return A2SGD_OK;
}

// A plan made for one device refuses to launch while another one is current.
a2sgd_status_t check_device(const a2sgd_plan_t *plan)
{
    if (plan->device < 0)
        return A2SGD_OK;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device != plan->device)
        return A2SGD_ERR_DEVICE;
    return A2SGD_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

uint32_t choose_blocks_per_worker(uint64_t n, uint32_t P)
{
    const uint64_t tile = static_cast<uint64_t>(kBlock) * kReduceUnroll * 4;  // elements per tile
    uint64_t tiles = (n + tile - 1) / tile;
    // rounded down: one workgroup more than the chip holds at once would run after all the others
    uint64_t want = static_cast<uint64_t>(kComputeUnits) * kReduceBlocksPerCU / P;
    uint64_t B = tiles < want ? tiles : want;
    if (B < 1)
        B = 1;
    if (B > kMaxBlocksPerWorker)
        B = kMaxBlocksPerWorker;
    return static_cast<uint32_t>(B);
}

// Checks the P pointers of one table; `required` = a NULL table or entry is an error.
a2sgd_status_t check_table(const float *const *tab, uint32_t P, bool required, bool *present)
{
    *present = false;
    if (tab == nullptr)
        return required ? A2SGD_ERR_INVALID_ARG : A2SGD_OK;
    for (uint32_t p = 0; p < P; ++p) {
        if (tab[p] == nullptr)
            return A2SGD_ERR_INVALID_ARG;
        if (!aligned16(tab[p]))
            return A2SGD_ERR_ALIGNMENT;
    }
    *present = true;
    return A2SGD_OK;
}

a2sgd_status_t check_buffer(const void *p)
{
    if (p == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    return aligned16(p) ? A2SGD_OK : A2SGD_ERR_ALIGNMENT;
}

void fill_replicas(ReplicaTable &t, uint32_t P, float *const *w)
{
    for (uint32_t p = 0; p < kMaxWorkers; ++p)
        t.w[p] = p < P ? w[p] : nullptr;
}

void fill_table(PtrTable &t, uint32_t P, const float *const *g, const float *const *e)
{
    for (uint32_t p = 0; p < kMaxWorkers; ++p) {
        t.g[p] = (g && p < P) ? g[p] : nullptr;
        t.e[p] = (e && p < P) ? const_cast<float *>(e[p]) : nullptr;
    }
}

// Address ranges of one call, for the aliasing rule: a buffer that the call writes must not overlap any other
// buffer of the call; buffers that are only read may coincide (two workers may share one g).
struct Ranges {
    struct R {
        uintptr_t lo, hi;
        bool written;
    };
    R r[3 * kMaxWorkers + 2];
    size_t count = 0;
    void add(const void *p, uint64_t bytes, bool written)
    {
        if (p != nullptr && bytes != 0 && count < sizeof(r) / sizeof(r[0]))
            r[count++] = R{reinterpret_cast<uintptr_t>(p), reinterpret_cast<uintptr_t>(p) + bytes, written};
    }
    void add_table(const float *const *tab, uint32_t P, uint64_t n, bool written)
    {
        for (uint32_t p = 0; tab != nullptr && p < P; ++p)
            add(tab[p], 4 * n, written);
    }
    // In order of start address, an earlier range overlaps the current one exactly if it ends after the
    // current one starts; so it is enough to carry the furthest end seen so far, of all ranges and of the
    // written ones.
    bool disjoint()
    {
        std::sort(r, r + count, [](const R &a, const R &b) { return a.lo < b.lo; });
        uintptr_t end_any = 0, end_written = 0;
        for (size_t i = 0; i < count; ++i) {
            if (r[i].lo < (r[i].written ? end_any : end_written))
                return false;
            end_any = r[i].hi > end_any ? r[i].hi : end_any;
            if (r[i].written)
                end_written = r[i].hi > end_written ? r[i].hi : end_written;
        }
        return true;
    }
};

// What the kernels of a plan with tensors leave in the workspace header about the tables: the tag of the tables
// that a2sgd_workspace_init uploaded, and whether a kernel has refused to use them since.
struct SegState {
    uint64_t tag;
    uint32_t fault;
    uint32_t reserved;
};
static_assert(offsetof(WsHeader, seg_fault) == offsetof(WsHeader, seg_tag) + 8, "SegState mirrors the header's tail");

inline a2sgd_status_t dev(hipError_t err) { return err == hipSuccess ? A2SGD_OK : A2SGD_ERR_DEVICE; }

// Validation shared by the calls that take g and e.  In retained-error mode e is required.
a2sgd_status_t check_g_e(const a2sgd_plan_t *plan, const float *const *g, const float *const *e, bool *has_e)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_g = false;
    a2sgd_status_t st = check_table(g, plan->P, true, &has_g);
    if (st != A2SGD_OK)
        return st;
    return check_table(e, plan->P, plan->mode == A2SGD_MODE_RETAINED_ERROR, has_e);
}

// Called with the failed_token field of a workspace header that was read after the stream was synchronised.  True
// if the plan's last single-launch step gave up at its grid barrier: its outputs are invalid.  Its grid has drained,
// so the cell is put back into its initial state for whoever owns it next, and this plan runs the three passes from
// now on.
bool single_launch_gave_up(const a2sgd_plan_t *plan, uint32_t failed_token, hipStream_t s)
{
    if (plan->last_token == 0 || failed_token != plan->last_token)
        return false;
    plan->fused_grid = 0;
    plan->last_token = 0;
    (void)launch_barrier_reset(static_cast<uint32_t>(plan->barrier_cell), s);
    return true;
}

// True if a2sgd_step may take the single launch now: the plan has a grid and a cell for it, and the current device
// holds the whole grid at once.
bool single_launch_now(const a2sgd_plan_t *plan)
{
    return plan->fused_grid != 0 && plan->barrier_cell >= 0 && plan->fused_grid <= current_device_compute_units();
}

// The aliasing rule for a call that reads g, updates e (if given) and w (one vector, or one per worker) in place
// and uses the workspace.
a2sgd_status_t check_step_ranges(const a2sgd_plan_t *plan, const float *const *g, const float *const *e, const float *w,
                                 const float *const *w_replicas, const void *workspace)
{
    Ranges rg;
    rg.add_table(g, plan->P, plan->n, false);
    rg.add_table(e, plan->P, plan->n, true);
    rg.add(w, 4 * plan->n, true);
    rg.add_table(w_replicas, plan->P, plan->n, true);
    rg.add(workspace, plan->workspace_bytes, true);
    return rg.disjoint() ? A2SGD_OK : A2SGD_ERR_INVALID_ARG;
}

}  // namespace

extern "C" {

a2sgd_status_t a2sgd_plan(const a2sgd_config_t *cfg, a2sgd_plan_t **out_plan)
{
    if (cfg == nullptr || out_plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    if (cfg->n == 0 || cfg->n > kMaxN)
        return A2SGD_ERR_INVALID_ARG;
    if (cfg->num_workers == 0 || cfg->num_workers > kMaxWorkers)
        return A2SGD_ERR_INVALID_ARG;
    if (cfg->mode != A2SGD_MODE_RETAINED_ERROR && cfg->mode != A2SGD_MODE_ALG1_LITERAL)
        return A2SGD_ERR_INVALID_ARG;
    if (cfg->blocks_per_worker > kMaxBlocksPerWorker || cfg->num_segments > kMaxSegments)
        return A2SGD_ERR_INVALID_ARG;
    if (cfg->num_segments == 0 && (cfg->pooled_means != 0 || cfg->seg_offset != nullptr))
        return A2SGD_ERR_INVALID_ARG;
    if (cfg->pooled_means > 1 || cfg->device < -1)
        return A2SGD_ERR_INVALID_ARG;
    if (cfg->num_segments >= 1) {
        if (cfg->seg_length == nullptr)
            return A2SGD_ERR_INVALID_ARG;
        uint64_t end = 0;  // end of the previous tensor
        for (uint32_t s = 0; s < cfg->num_segments; ++s) {
            const uint64_t off = cfg->seg_offset ? cfg->seg_offset[s] : end;
            if (off < end || off >= cfg->n || cfg->seg_length[s] == 0 || cfg->seg_length[s] > cfg->n - off)
                return A2SGD_ERR_INVALID_ARG;
            end = off + cfg->seg_length[s];
        }
        if (cfg->seg_offset == nullptr && end != cfg->n)
            return A2SGD_ERR_INVALID_ARG;
    }
    a2sgd_plan_t *pl = new (std::nothrow) a2sgd_plan_t;
    if (pl == nullptr)
        return A2SGD_ERR_NOMEM;
    pl->n = cfg->n;
    pl->P = cfg->num_workers;
    pl->mode = cfg->mode;
    pl->B = cfg->blocks_per_worker ? cfg->blocks_per_worker : choose_blocks_per_worker(pl->n, pl->P);
    pl->streaming = (2ull * pl->P + 1) * 4ull * pl->n > kStreamingBytes;
    pl->apply.up = pl->P >= 8 ? 8 : pl->P >= 4 ? 4 : pl->P >= 2 ? 2 : 1;
    pl->apply.lds_bytes = pl->streaming ? apply_lds_bytes(pl->P) : 0;
    pl->apply.dense_lds_bytes = pl->streaming ? dense_lds_bytes(pl->P) : 0;
    // From kTwoKernelWorkers workers on, a workgroup of the one-kernel apply pass has so many buffers open (2P + 1)
    // that address translation costs it more than the sign words cost the two-kernel form (nP/4 extra bytes).
    pl->apply.two_kernels = pl->streaming && pl->mode == A2SGD_MODE_RETAINED_ERROR && pl->P >= kTwoKernelWorkers;
    pl->device = cfg->device;
    // Single-launch step while everything fits the caches: one workgroup of kFusedBlock threads per 2048 elements,
    // at most kFusedGridMax of them.  It needs a grid-barrier cell of its own; without one the plan runs the three
    // passes.
    pl->barrier_cell = -1;
    pl->last_token = 0;
    pl->fused_grid = 0;
    const bool may_fuse = !pl->streaming && !(cfg->num_segments >= 1 && cfg->pooled_means != 0);
    if (may_fuse && (pl->barrier_cell = g_cells.take()) >= 0) {
        const uint64_t want = (pl->n + 4 * kFusedBlock - 1) / (4 * kFusedBlock);
        pl->fused_grid = static_cast<uint32_t>(want < kFusedGridMax ? want : kFusedGridMax);  // tensors: set below
    }
    // the records have room for the single launch's grid whether or not this plan got a cell, so that the size of
    // the workspace does not depend on how many other plans are alive
    const uint64_t fused_rows = pl->streaming ? 0 : std::min<uint64_t>((pl->n + 4 * kFusedBlock - 1) / (4 * kFusedBlock), kFusedGridMax);
    const uint32_t rows = pl->B > fused_rows ? pl->B : static_cast<uint32_t>(fused_rows);
    const size_t partials = 5ull * 8ull * pl->P * rows;
    const size_t drift = 2ull * 8ull * pl->P * (kDriftBlocks + 1);  // the drift diagnostic reuses the same region
    pl->workspace_bytes = kHeaderBytes + (partials > drift ? partials : drift);
    pl->eager_bytes = pl->workspace_bytes;
    pl->lazy_folded = 0;
    pl->lazy_offset = pl->lazy_sign_offset = 0;
    {
        const uint64_t per = 64ull * kLazyItems, nvec = pl->n >> 2;
        pl->lazy_blocks = static_cast<uint32_t>(nvec ? (nvec + per - 1) / per : 1);
    }
    if (cfg->num_segments == 0) {
        // one record per workgroup of the lazy state's one-shot reduction pass, and their folded table
        pl->lazy_folded = (pl->lazy_blocks + kFoldSpan - 1) / kFoldSpan;
        pl->lazy_offset = (pl->workspace_bytes + 255) & ~static_cast<size_t>(255);
        pl->lazy_sign_offset = pl->lazy_offset + 5ull * 8ull * pl->P * (static_cast<size_t>(pl->lazy_blocks) + pl->lazy_folded);
        pl->lazy_sign_offset = (pl->lazy_sign_offset + 255) & ~static_cast<size_t>(255);
        pl->workspace_bytes = pl->lazy_sign_offset + 4ull * pl->P * (64ull * pl->lazy_blocks);
    }
    if (cfg->num_segments >= 1) {
        try {
            build_segments(*pl, cfg->num_segments, cfg->seg_length, cfg->seg_offset, cfg->pooled_means != 0);
            pl->seg.tag = tables_tag(*pl);
        } catch (const std::bad_alloc &) {
            g_cells.give(pl->barrier_cell);
            delete pl;
            return A2SGD_ERR_NOMEM;
        }
        pl->workspace_bytes = pl->seg.end;
        // Single launch on tensors: one workgroup per item of at most kFusedItemElems elements, up to kFusedGridMax.
        // Beyond four items per workgroup (about 4 M elements) the three passes are faster (measured on the
        // 14.7 M-parameter VGG-16 of Table 1 at P = 1: 103 us against 90 us), and the cell goes back.
        if (pl->fused_grid != 0) {
            const size_t items = pl->seg.fitem.size();
            pl->fused_grid = static_cast<uint32_t>(items < kFusedGridMax ? items : kFusedGridMax);
            if (items > 4 * kFusedGridMax) {
                pl->fused_grid = 0;
                g_cells.give(pl->barrier_cell);
                pl->barrier_cell = -1;
            }
        }
    }
    *out_plan = pl;
    return A2SGD_OK;
}

a2sgd_status_t a2sgd_plan_destroy(a2sgd_plan_t *plan)
{
    if (plan != nullptr)
        g_cells.give(plan->barrier_cell);
    delete plan;
    return A2SGD_OK;
}

size_t a2sgd_workspace_bytes(const a2sgd_plan_t *plan) { return plan ? plan->workspace_bytes : 0; }

a2sgd_status_t a2sgd_workspace_check(const a2sgd_plan_t *plan, const void *workspace, size_t bytes)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    a2sgd_status_t st = check_buffer(workspace);
    if (st != A2SGD_OK)
        return st;
    return bytes >= plan->workspace_bytes ? A2SGD_OK : A2SGD_ERR_WORKSPACE_TOO_SMALL;
}

uint32_t a2sgd_plan_blocks_per_worker(const a2sgd_plan_t *plan) { return plan ? plan->B : 0; }

int32_t a2sgd_plan_single_launch_cell(const a2sgd_plan_t *plan)
{
    return plan != nullptr && plan->fused_grid != 0 ? plan->barrier_cell : -1;
}

a2sgd_status_t a2sgd_local_averages(const a2sgd_plan_t *plan, const float *const *g, const float *const *e,
                                    void *workspace, a2sgd_stream_t stream)
{
    bool has_e = false;
    a2sgd_status_t st = check_g_e(plan, g, e, &has_e);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    Ranges rg;
    rg.add_table(g, plan->P, plan->n, false);
    rg.add_table(has_e ? e : nullptr, plan->P, plan->n, false);
    rg.add(workspace, plan->workspace_bytes, true);
    if (!rg.disjoint())
        return A2SGD_ERR_INVALID_ARG;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    fill_table(tab, plan->P, g, has_e ? e : nullptr);
    plan->last_token = 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (segmented(plan)) {
        if ((st = dev(launch_seg_partials(*plan, tab, has_e, workspace, s))) != A2SGD_OK)
            return st;
        return dev(launch_seg_finalize(*plan, workspace, s));
    }
    if ((st = dev(launch_local_partials(*plan, tab, has_e, workspace, s))) != A2SGD_OK)
        return st;
    return dev(launch_local_finalize(*plan, workspace, s));
}

a2sgd_status_t a2sgd_global_average(const a2sgd_plan_t *plan, void *workspace, a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    a2sgd_status_t st = check_buffer(workspace);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    if (segmented(plan))
        return dev(launch_seg_global(*plan, workspace, static_cast<hipStream_t>(stream)));
    return dev(launch_global_average(*plan, workspace, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_export_local_means(const a2sgd_plan_t *plan, const void *workspace, float *out,
                                        a2sgd_stream_t stream)
{
    if (plan == nullptr || segmented(plan) || workspace == nullptr || out == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(out) & 3u) != 0)
        return A2SGD_ERR_ALIGNMENT;
    if (check_device(plan) != A2SGD_OK)
        return A2SGD_ERR_DEVICE;
    return dev(launch_export_local_means(*plan, workspace, out, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_import_global_means(const a2sgd_plan_t *plan, void *workspace, const float *gmu,
                                         a2sgd_stream_t stream)
{
    if (plan == nullptr || segmented(plan) || workspace == nullptr || gmu == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(gmu) & 3u) != 0)
        return A2SGD_ERR_ALIGNMENT;
    if (check_device(plan) != A2SGD_OK)
        return A2SGD_ERR_DEVICE;
    plan->last_token = 0;
    return dev(launch_import_global_means(*plan, workspace, gmu, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_apply_and_update_error(const a2sgd_plan_t *plan, const float *const *g, float *const *e,
                                            float *w, float eta, void *workspace, a2sgd_stream_t stream)
{
    bool has_e = false;
    a2sgd_status_t st = check_g_e(plan, g, e, &has_e);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_buffer(w)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, has_e ? e : nullptr, w, nullptr, workspace)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    fill_table(tab, plan->P, g, has_e ? e : nullptr);
    if (segmented(plan))
        return dev(launch_seg_apply(*plan, tab, has_e, w, eta, workspace, static_cast<hipStream_t>(stream)));
    return dev(launch_apply(*plan, tab, has_e, w, eta, workspace, false, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_step(const a2sgd_plan_t *plan, const float *const *g, float *const *e, float *w, float eta,
                          void *workspace, a2sgd_stream_t stream)
{
    // validate everything first so that a failed step has enqueued nothing
    bool has_e = false;
    a2sgd_status_t st = check_g_e(plan, g, e, &has_e);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_buffer(w)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, has_e ? e : nullptr, w, nullptr, workspace)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    if (single_launch_now(plan)) {
        PtrTable tab;
        fill_table(tab, plan->P, g, has_e ? e : nullptr);
        uint32_t token = g_next_token.fetch_add(1);
        if (token == 0)
            token = g_next_token.fetch_add(1);
        plan->last_token = token;
        if (segmented(plan))
            return dev(launch_seg_fused_step(*plan, tab, has_e, w, eta, workspace, token, static_cast<hipStream_t>(stream)));
        return dev(launch_fused_step(*plan, tab, has_e, w, eta, workspace, token, static_cast<hipStream_t>(stream)));
    }
    if ((st = a2sgd_local_averages(plan, g, e, workspace, stream)) != A2SGD_OK)
        return st;
    if ((st = a2sgd_global_average(plan, workspace, stream)) != A2SGD_OK)
        return st;
    return a2sgd_apply_and_update_error(plan, g, e, w, eta, workspace, stream);
}

a2sgd_status_t a2sgd_step_static(const a2sgd_plan_t *plan, const float *const *g, float *const *e, float *w, float eta,
                                 a2sgd_stream_t stream)
{
    bool has_e = false;
    a2sgd_status_t st = check_g_e(plan, g, e, &has_e);
    if (st != A2SGD_OK)
        return st;
    if (segmented(plan))
        return A2SGD_ERR_INVALID_ARG;
    if ((st = check_buffer(w)) != A2SGD_OK)
        return st;
    // the built-in array lies in the library's own device memory: no buffer of the caller can overlap it
    if ((st = check_step_ranges(plan, g, has_e ? e : nullptr, w, nullptr, nullptr)) != A2SGD_OK)
        return st;
    // the three passes touch the header and P * B partial records, nothing else
    if (kHeaderBytes + 5ull * 8ull * plan->P * plan->B > kStaticScratchBytes)
        return A2SGD_ERR_SCRATCH_LIMIT;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    void *ws = nullptr;
    if ((st = static_scratch(&ws)) != A2SGD_OK)
        return st;
    PtrTable tab;
    fill_table(tab, plan->P, g, has_e ? e : nullptr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((st = dev(launch_local_partials(*plan, tab, has_e, ws, s))) != A2SGD_OK)
        return st;
    if ((st = dev(launch_local_finalize(*plan, ws, s))) != A2SGD_OK)
        return st;
    if ((st = dev(launch_global_average(*plan, ws, s))) != A2SGD_OK)
        return st;
    return dev(launch_apply(*plan, tab, has_e, w, eta, ws, true, s));  // the array has no room for sign words
}

a2sgd_status_t a2sgd_read_stats(const a2sgd_plan_t *plan, const void *workspace, a2sgd_stream_t stream,
                                a2sgd_worker_stats_t *out_workers, a2sgd_global_stats_t *out_global)
{
    if (plan == nullptr || workspace == nullptr || (segmented(plan) && !plan->seg.pooled))
        return A2SGD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (segmented(plan)) {
        // pooled means: every tensor's row of the tables holds the same pair; read tensor 0's
        const SegPlan &sp = plan->seg;
        const char *b = static_cast<const char *>(workspace);
        float gmu[2] = {0.0f, 0.0f};
        SegState state = {};
        if (hipMemcpyAsync(&state, b + offsetof(WsHeader, seg_tag), sizeof(state), hipMemcpyDeviceToHost, s) != hipSuccess)
            return A2SGD_ERR_DEVICE;
        for (uint32_t p = 0; out_workers && p < plan->P; ++p)
            if (hipMemcpyAsync(out_workers + p, b + sp.off_stats + sizeof(a2sgd_worker_stats_t) * p * sp.S,
                               sizeof(a2sgd_worker_stats_t), hipMemcpyDeviceToHost, s) != hipSuccess)
                return A2SGD_ERR_DEVICE;
        if (out_global && hipMemcpyAsync(gmu, b + sp.off_gmu, sizeof(gmu), hipMemcpyDeviceToHost, s) != hipSuccess)
            return A2SGD_ERR_DEVICE;
        if (hipStreamSynchronize(s) != hipSuccess)
            return A2SGD_ERR_DEVICE;
        if (state.tag != sp.tag || state.fault != 0)
            return A2SGD_ERR_WORKSPACE_STATE;
        if (out_global) {
            out_global->gmu_pos = gmu[0];
            out_global->gmu_neg = -gmu[1];  // the table keeps the negated value for the apply pass
        }
        return A2SGD_OK;
    }
    WsHeader hdr;
    if (hipMemcpyAsync(&hdr, workspace, sizeof(WsHeader), hipMemcpyDeviceToHost, s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    if (single_launch_gave_up(plan, hdr.failed_token, s))
        return A2SGD_ERR_DEVICE;
    if (out_workers)
        for (uint32_t p = 0; p < plan->P; ++p)
            out_workers[p] = hdr.workers[p];
    if (out_global) {
        out_global->gmu_pos = hdr.gmu_pos;
        out_global->gmu_neg = hdr.gmu_neg;
    }
    return A2SGD_OK;
}

a2sgd_status_t a2sgd_export_mask(const a2sgd_plan_t *plan, const float *const *g, const float *const *e,
                                 uint64_t *mask, a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_g = false, has_e = false;
    a2sgd_status_t st = check_table(g, plan->P, true, &has_g);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_table(e, plan->P, false, &has_e)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(mask)) != A2SGD_OK)
        return st;
    Ranges rg;
    rg.add_table(g, plan->P, plan->n, false);
    rg.add_table(has_e ? e : nullptr, plan->P, plan->n, false);
    rg.add(mask, 8ull * plan->P * ((plan->n + 63) / 64), true);
    if (!rg.disjoint())
        return A2SGD_ERR_INVALID_ARG;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    fill_table(tab, plan->P, g, has_e ? e : nullptr);
    return dev(launch_export_mask(*plan, tab, has_e, mask, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_dense_step(const a2sgd_plan_t *plan, const float *const *g, float *w, float eta,
                                a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_g = false;
    a2sgd_status_t st = check_table(g, plan->P, true, &has_g);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_buffer(w)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, nullptr, w, nullptr, nullptr)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    fill_table(tab, plan->P, g, nullptr);
    return dev(launch_dense_step(*plan, tab, w, eta, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_apply_and_update_error_replicas(const a2sgd_plan_t *plan, const float *const *g, float *const *e,
                                                     float *const *w, float eta, void *workspace,
                                                     a2sgd_stream_t stream)
{
    bool has_e = false, has_w = false;
    a2sgd_status_t st = check_g_e(plan, g, e, &has_e);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_table(w, plan->P, true, &has_w)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, has_e ? e : nullptr, nullptr, w, workspace)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    ReplicaTable wt;
    fill_table(tab, plan->P, g, has_e ? e : nullptr);
    if (segmented(plan)) {
        fill_replicas(wt, plan->P, w);
        return dev(launch_seg_apply_replicas(*plan, tab, wt, has_e, eta, workspace, static_cast<hipStream_t>(stream)));
    }
    if (plan->P == 1)  // one worker: its own replica is the shared vector, and that pass is the tuned one
        return dev(launch_apply(*plan, tab, has_e, w[0], eta, workspace, false, static_cast<hipStream_t>(stream)));
    fill_replicas(wt, plan->P, w);
    return dev(launch_apply_replicas(*plan, tab, wt, has_e, eta, workspace, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_step_replicas(const a2sgd_plan_t *plan, const float *const *g, float *const *e, float *const *w,
                                   float eta, void *workspace, a2sgd_stream_t stream)
{
    bool has_e = false, has_w = false;
    a2sgd_status_t st = check_g_e(plan, g, e, &has_e);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_table(w, plan->P, true, &has_w)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, has_e ? e : nullptr, nullptr, w, workspace)) != A2SGD_OK)
        return st;
    if ((st = a2sgd_local_averages(plan, g, e, workspace, stream)) != A2SGD_OK)
        return st;
    if ((st = a2sgd_global_average(plan, workspace, stream)) != A2SGD_OK)
        return st;
    return a2sgd_apply_and_update_error_replicas(plan, g, e, w, eta, workspace, stream);
}

a2sgd_status_t a2sgd_dense_step_replicas(const a2sgd_plan_t *plan, const float *const *g, float *const *w, float eta,
                                         a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_g = false, has_w = false;
    a2sgd_status_t st = check_table(g, plan->P, true, &has_g);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_table(w, plan->P, true, &has_w)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, nullptr, nullptr, w, nullptr)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    ReplicaTable wt;
    fill_table(tab, plan->P, g, nullptr);
    fill_replicas(wt, plan->P, w);
    return dev(launch_dense_step_replicas(*plan, tab, wt, eta, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_replica_drift(const a2sgd_plan_t *plan, const float *const *w, void *workspace,
                                   a2sgd_stream_t stream, double *out_max_abs, double *out_rms)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_w = false;
    a2sgd_status_t st = check_table(w, plan->P, true, &has_w);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    ReplicaTable wt;
    fill_replicas(wt, plan->P, const_cast<float *const *>(w));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((st = dev(launch_replica_drift(*plan, wt, workspace, s))) != A2SGD_OK)
        return st;
    double res[2 * kMaxWorkers];
    if (hipMemcpyAsync(res, static_cast<const char *>(workspace) + drift_result_offset(*plan),
                       2 * sizeof(double) * plan->P, hipMemcpyDeviceToHost, s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    for (uint32_t p = 0; p < plan->P; ++p) {
        if (out_max_abs)
            out_max_abs[p] = res[p];
        if (out_rms)
            out_rms[p] = res[plan->P + p];
    }
    return A2SGD_OK;
}

a2sgd_status_t a2sgd_lazy_reset(const a2sgd_plan_t *plan, void *workspace, a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    a2sgd_status_t st = check_buffer(workspace);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    if (segmented(plan))
        return dev(launch_seg_lazy_reset(*plan, workspace, static_cast<hipStream_t>(stream)));
    return dev(launch_lazy_reset(*plan, workspace, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_lazy_local_averages(const a2sgd_plan_t *plan, const float *const *g, float *const *s,
                                         void *workspace, a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_g = false, has_s = false;
    a2sgd_status_t st = check_table(g, plan->P, true, &has_g);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_table(s, plan->P, true, &has_s)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, s, nullptr, nullptr, workspace)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    fill_table(tab, plan->P, g, s);
    plan->last_token = 0;
    if (segmented(plan))
        return dev(launch_seg_lazy_partials(*plan, tab, workspace, static_cast<hipStream_t>(stream)));
    return dev(launch_lazy_partials(*plan, tab, workspace, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_lazy_apply(const a2sgd_plan_t *plan, const float *const *s, float *w, float eta, void *workspace,
                                a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_s = false;
    a2sgd_status_t st = check_table(s, plan->P, true, &has_s);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_buffer(w)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    Ranges rg;
    rg.add_table(s, plan->P, plan->n, false);
    rg.add(w, 4 * plan->n, true);
    rg.add(workspace, plan->workspace_bytes, true);
    if (!rg.disjoint())
        return A2SGD_ERR_INVALID_ARG;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    if (segmented(plan) && plan->mode == A2SGD_MODE_ALG1_LITERAL) {
        // the per-tensor apply pass with the stored v in the place of the gradient and no error buffer: it reads v,
        // forms the update from its sign group and its error and writes w only
        fill_table(tab, plan->P, s, nullptr);
        return dev(launch_seg_apply(*plan, tab, false, w, eta, workspace, static_cast<hipStream_t>(stream)));
    }
    if (segmented(plan)) {  // retained-error mode: from the sign bits that the reduction pass left
        fill_table(tab, plan->P, s, s);
        return dev(launch_seg_lazy_apply_signs(*plan, tab, w, eta, workspace, static_cast<hipStream_t>(stream)));
    }
    fill_table(tab, plan->P, s, s);  // the pass reads the state buffers only
    return dev(launch_lazy_apply(*plan, tab, w, eta, workspace, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_lazy_step(const a2sgd_plan_t *plan, const float *const *g, float *const *s, float *w, float eta,
                               void *workspace, a2sgd_stream_t stream)
{
    // validate everything first so that a failed step has enqueued nothing
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_g = false, has_s = false;
    a2sgd_status_t st = check_table(g, plan->P, true, &has_g);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_table(s, plan->P, true, &has_s)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(w)) != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_step_ranges(plan, g, s, w, nullptr, workspace)) != A2SGD_OK)
        return st;
    if ((st = a2sgd_lazy_local_averages(plan, g, s, workspace, stream)) != A2SGD_OK)
        return st;
    if ((st = a2sgd_global_average(plan, workspace, stream)) != A2SGD_OK)
        return st;
    return a2sgd_lazy_apply(plan, s, w, eta, workspace, stream);
}

a2sgd_status_t a2sgd_lazy_materialize(const a2sgd_plan_t *plan, float *const *s, void *workspace,
                                      a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    bool has_s = false;
    a2sgd_status_t st = check_table(s, plan->P, true, &has_s);
    if (st != A2SGD_OK)
        return st;
    if ((st = check_buffer(workspace)) != A2SGD_OK)
        return st;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    PtrTable tab;
    fill_table(tab, plan->P, s, s);
    if (segmented(plan))
        return dev(launch_seg_materialize(*plan, tab, workspace, static_cast<hipStream_t>(stream)));
    return dev(launch_lazy_materialize(*plan, tab, workspace, static_cast<hipStream_t>(stream)));
}

a2sgd_status_t a2sgd_selftest_barrier(void *buffer, a2sgd_stream_t stream)
{
    a2sgd_status_t st = check_buffer(buffer);
    if (st != A2SGD_OK)
        return st;
    constexpr uint32_t kGrid = 128;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t *passed = static_cast<uint32_t *>(buffer);
    uint32_t *cell_failed = passed + kGrid;
    uint32_t host[kGrid + 1];
    for (int round = 0; round < 2; ++round) {
        const bool starve = round == 1;  // second round: one arrival too few, tiny spin limit
        if (launch_barrier_selftest(kGrid, starve ? kGrid + 1 : kGrid, starve ? 64u : (1u << 21), passed, cell_failed,
                                    s) != hipSuccess)
            return A2SGD_ERR_DEVICE;
        if (hipMemcpyAsync(host, buffer, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return A2SGD_ERR_DEVICE;
        for (uint32_t b = 0; b < kGrid; ++b)
            if (host[b] != (starve ? 0u : 1u))
                return A2SGD_ERR_DEVICE;
        if (host[kGrid] != (starve ? 1u : 0u))
            return A2SGD_ERR_DEVICE;
    }
    return A2SGD_OK;
}

a2sgd_status_t a2sgd_workspace_init(const a2sgd_plan_t *plan, void *workspace, a2sgd_stream_t stream)
{
    if (plan == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    a2sgd_status_t st = check_buffer(workspace);
    if (st != A2SGD_OK)
        return st;
    if (!segmented(plan))
        return A2SGD_OK;
    if ((st = check_device(plan)) != A2SGD_OK)
        return st;
    const SegPlan &sp = plan->seg;
    char *b = static_cast<char *>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const struct {
        size_t off;
        const void *src;
        size_t bytes;
    } parts[] = {{sp.off_seg_start, sp.seg_start.data(), 8ull * sp.seg_start.size()},
                 {sp.off_seg_end, sp.seg_end.data(), 8ull * sp.seg_end.size()},
                 {sp.off_item, sp.item.data(), sizeof(SegItem) * sp.item.size()},
                 {sp.off_item_lo, sp.item_lo.data(), 4ull * sp.item_lo.size()},
                 {sp.off_coarse, sp.coarse.data(), 4ull * sp.coarse.size()},
                 {sp.off_sched_lo, sp.sched_lo.data(), 4ull * sp.sched_lo.size()},
                 {sp.off_sched_item, sp.sched_item.data(), 4ull * sp.sched_item.size()},
                 {sp.off_lz_slot_lo, sp.lz_slot_lo.data(), 4ull * sp.lz_slot_lo.size()},
                 {sp.off_lz_fold, sp.lz_fold.data(), sizeof(SegFold) * sp.lz_fold.size()}};
    for (const auto &part : parts)
        if (hipMemcpyAsync(b + part.off, part.src, part.bytes, hipMemcpyHostToDevice, s) != hipSuccess)
            return A2SGD_ERR_DEVICE;
    if (!sp.fitem.empty() &&
        (hipMemcpyAsync(b + sp.off_fitem, sp.fitem.data(), sizeof(SegItem) * sp.fitem.size(), hipMemcpyHostToDevice, s) != hipSuccess ||
         hipMemcpyAsync(b + sp.off_fitem_lo, sp.fitem_lo.data(), 4ull * sp.fitem_lo.size(), hipMemcpyHostToDevice, s) != hipSuccess))
        return A2SGD_ERR_DEVICE;
    // last, in stream order: the tag that tells the kernels whose tables these are
    if ((st = dev(launch_seg_mark(*plan, workspace, s))) != A2SGD_OK)
        return st;
    // the copies read the plan's own host vectors: wait for them, so that the plan may be destroyed at any time
    return hipStreamSynchronize(s) == hipSuccess ? A2SGD_OK : A2SGD_ERR_DEVICE;
}

a2sgd_status_t a2sgd_read_segment_stats(const a2sgd_plan_t *plan, const void *workspace, a2sgd_stream_t stream,
                                        a2sgd_worker_stats_t *out_workers, a2sgd_global_stats_t *out_global)
{
    if (plan == nullptr || workspace == nullptr || !segmented(plan))
        return A2SGD_ERR_INVALID_ARG;
    const SegPlan &sp = plan->seg;
    const char *b = static_cast<const char *>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    std::vector<float> gmu;
    try {
        gmu.resize(2ull * sp.S);
    } catch (const std::bad_alloc &) {
        return A2SGD_ERR_NOMEM;
    }
    SegState state = {};
    uint32_t failed_token = 0;
    if (hipMemcpyAsync(&state, b + offsetof(WsHeader, seg_tag), sizeof(state), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipMemcpyAsync(&failed_token, b + offsetof(WsHeader, failed_token), 4, hipMemcpyDeviceToHost, s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    if (out_workers && hipMemcpyAsync(out_workers, b + sp.off_stats, sizeof(a2sgd_worker_stats_t) * plan->P * sp.S,
                                      hipMemcpyDeviceToHost, s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    if (out_global &&
        hipMemcpyAsync(gmu.data(), b + sp.off_gmu, 8ull * sp.S, hipMemcpyDeviceToHost, s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    if (state.tag != sp.tag || state.fault != 0)
        return A2SGD_ERR_WORKSPACE_STATE;
    if (single_launch_gave_up(plan, failed_token, s))
        return A2SGD_ERR_DEVICE;
    if (out_global)
        for (uint32_t k = 0; k < sp.S; ++k) {
            out_global[k].gmu_pos = gmu[2 * k];
            out_global[k].gmu_neg = -gmu[2 * k + 1];  // the table keeps the negated value for the apply pass
        }
    return A2SGD_OK;
}

a2sgd_status_t a2sgd_device_info(a2sgd_device_info_t *out)
{
    if (out == nullptr)
        return A2SGD_ERR_INVALID_ARG;
    int device = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&device) != hipSuccess || hipGetDeviceProperties(&prop, device) != hipSuccess)
        return A2SGD_ERR_DEVICE;
    out->compute_units = static_cast<uint32_t>(prop.multiProcessorCount);
    out->memory_clock_khz = static_cast<uint32_t>(prop.memoryClockRate);
    out->memory_bus_bits = static_cast<uint32_t>(prop.memoryBusWidth);
    out->reserved = 0;
    out->total_memory_bytes = prop.totalGlobalMem;
    out->l2_bytes = static_cast<uint64_t>(prop.l2CacheSize);
    return A2SGD_OK;
}

const char *a2sgd_status_string(a2sgd_status_t status)
{
    switch (status) {
    case A2SGD_OK: return "ok";
    case A2SGD_ERR_INVALID_ARG: return "invalid argument";
    case A2SGD_ERR_ALIGNMENT: return "device pointer not 16-byte aligned";
    case A2SGD_ERR_DEVICE: return "HIP call or kernel launch failed";
    case A2SGD_ERR_NOMEM: return "out of host memory";
    case A2SGD_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than a2sgd_workspace_bytes";
    case A2SGD_ERR_WORKSPACE_STATE: return "workspace not initialised for this plan (a2sgd_workspace_init)";
    case A2SGD_ERR_SCRATCH_LIMIT: return "plan needs more scratch than the library's built-in array holds";
    }
    return "unknown status";
}

}  // extern "C"
