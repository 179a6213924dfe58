// Shared between the host API (a2sgd_api.cpp) and the kernels (a2sgd_kernels.hip): workspace layout, the
// plan, and the launchers' signatures.  Nothing outside this library includes it.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "a2sgd.h"

namespace a2sgd {

constexpr uint32_t kMaxWorkers = A2SGD_MAX_WORKERS;
constexpr int kBlock = 256;           // threads per workgroup: 4 wavefronts of 64
constexpr int kReduceUnroll = 4;      // float4 loads per array per thread per tile in the reduction
constexpr uint32_t kMaxBlocksPerWorker = 65536;
constexpr int kFusedBlock = 512;       // threads per workgroup of the single-launch step
constexpr uint32_t kBarrierSlots = 64;  // grid-barrier cells of the single-launch step: a live plan owns at most one
constexpr int kLazyItems = 8;           // float4 groups per array per thread in the lazy state's reduction pass
constexpr uint32_t kPerWorkerReplicas = 8;  // from this many workers on the replica apply pass takes one worker per workgroup
constexpr uint32_t kFoldSpan = 4096;    // records that one workgroup of k_fold_partials adds up

// Device workspace, in this order:
//   WsHeader                                   (kHeaderBytes, padded)
//   double   s_pos [P][B]   block partial sums of v over v >= 0
//   double   s_neg [P][B]   block partial sums of |v| over v < 0
//   uint64_t n_pos [P][B], n_neg [P][B], n_zero [P][B]
//   whole-model plans only, at plan.lazy_offset: the same five arrays as [P][lazy_blocks] (one record per
//   workgroup of the lazy state's reduction pass), then as [P][lazy_folded]; at plan.lazy_sign_offset:
//   uint16_t sign [lazy_blocks][2][P][64], one bit per element: pos(v) of Eq. 2
struct WsHeader {
    float gmu_pos, gmu_neg;  // Algorithm 1 line 5
    uint32_t failed_token;   // set to the launch's token by a single-launch step that could not complete
    uint32_t any_nan;        // nonzero if any worker counted a NaN in the last reduction (set with the global means)
    a2sgd_worker_stats_t workers[kMaxWorkers];  // Algorithm 1 line 3, per worker
    float neg_mu_pos[kMaxWorkers];  // -mu_pos and mu_neg of every worker again, packed for the apply pass
    float mu_neg[kMaxWorkers];
    // Plans with tensors: a2sgd_workspace_init leaves the tag of the tables it uploaded here.  A kernel that is about
    // to index through those tables compares it with its plan's tag first and, on a mismatch (workspace never
    // initialised, or initialised for another plan), sets seg_fault and exits without touching the tables.
    uint64_t seg_tag;
    uint32_t seg_fault;
    uint32_t reserved;
};
constexpr size_t kHeaderBytes = 4096;
static_assert(sizeof(WsHeader) <= kHeaderBytes, "header must fit its slot");
static_assert(sizeof(a2sgd_worker_stats_t) == 40, "stats record layout is part of the ABI");

struct Partials {
    double *s_pos, *s_neg;
    uint64_t *n_pos, *n_neg, *n_zero;
};

inline Partials partials_at(void *workspace, size_t offset, uint32_t P, uint32_t B)
{
    char *base = static_cast<char *>(workspace) + offset;
    const size_t stride = static_cast<size_t>(P) * B * 8;
    Partials q;
    q.s_pos = reinterpret_cast<double *>(base);
    q.s_neg = reinterpret_cast<double *>(base + stride);
    q.n_pos = reinterpret_cast<uint64_t *>(base + 2 * stride);
    q.n_neg = reinterpret_cast<uint64_t *>(base + 3 * stride);
    q.n_zero = reinterpret_cast<uint64_t *>(base + 4 * stride);
    return q;
}

inline Partials partials_of(void *workspace, uint32_t P, uint32_t B)
{
    return partials_at(workspace, kHeaderBytes, P, B);
}

// Kernel argument block: the P device pointers of each kind, passed by value (1 KiB of kernarg).
struct PtrTable {
    const float *g[kMaxWorkers];
    float *e[kMaxWorkers];
};
// The P weight replicas, for the per-replica entry points only.
struct ReplicaTable {
    float *w[kMaxWorkers];
};
constexpr uint32_t kDriftBlocks = 256;  // workgroups per worker of the replica-drift reduction

}  // namespace a2sgd

namespace a2sgd {
// Shape of the apply pass: the loads of `up` workers are issued together; lds_bytes of dynamic LDS per
// workgroup (0 = none) set how many workgroups fit a compute unit.
struct ApplyGeom {
    int up;
    uint32_t lds_bytes;
    uint32_t dense_lds_bytes;  // the same for the dense step
    bool two_kernels;          // retained-error mode: error write-back and weight update as two kernels (many workers)
};
}  // namespace a2sgd

namespace a2sgd {

// ---- per-tensor means: static tables the plan builds on the host and a2sgd_workspace_init uploads --------------
constexpr uint32_t kSegItemElems = 65536;  // a work item of the segmented reduction covers at most this many elements
constexpr uint32_t kSegInsideBit = 1u << 31;  // in a lookup entry: the whole chunk lies inside that segment
constexpr uint32_t kSegCoarseShift = 8;    // the lookup table has one entry per 2^8 elements: one per apply workgroup

struct SegItem {  // one work item: a run of elements inside one segment
    uint64_t start;
    uint32_t count;
    uint32_t seg;
};

// Device views of the segmented part of the workspace (all offsets are fixed by the plan).
struct SegView {
    uint32_t S;
    uint32_t num_items;
    WsHeader *hdr;  // holds the tag of the tables that a2sgd_workspace_init uploaded
    uint64_t tag;   // the tag of this plan's tables
    const uint64_t *seg_start;  // [S + 1] first element of every segment; entry S is a sentinel (2^64 - 1)
    const uint64_t *seg_end;    // [S + 1] exclusive end of every segment; entry S is a sentinel (2^64 - 1)
    const SegItem *item;       // [num_items], ascending start
    const uint32_t *item_lo;   // [S + 1]: items of segment s are item_lo[s] .. item_lo[s + 1] - 1
    const uint32_t *coarse;    // [ceil(n / 2^8)]: the first segment that ends after element k * 2^8 (S if none),
                               // with kSegInsideBit set if the chunk's float4 groups all lie inside it
    const uint32_t *sched_lo;  // [blocks + 1]: workgroup b of the reduction takes sched_item[sched_lo[b] .. sched_lo[b + 1])
    const uint32_t *sched_item;  // [num_items]
    a2sgd_worker_stats_t *stats;  // [P][S]
    float *neg_mu_pos, *mu_neg;   // [S][P], packed for the apply pass
    float *gmu;                   // [S][2]: gmu_pos, -gmu_neg
    Partials rec;                 // [P][num_items] partial records of the reduction
};

// The single-launch step on a plan with tensors works on finer items (at most kFusedItemElems elements inside one
// tensor, so that a small model still spreads over many workgroups): one partial record per (worker, item).
constexpr uint32_t kFusedItemElems = 4096;  // 2 float4 groups per thread of a kFusedBlock workgroup
struct FusedSegView {
    uint32_t num_items;
    const SegItem *item;      // [num_items], ascending start
    const uint32_t *item_lo;  // [S + 1]: items of segment s
    double *r_spos, *r_sneg;  // [P][num_items]
    uint64_t *r_npos, *r_nneg, *r_nzero;
};

// The lazy error state on a plan with tensors.  Its reduction is a one-shot pass over blocks of kSegLazyElems elements
// by position, whatever the tensors: a block that lies wholly inside one tensor leaves one record in a table with a
// row per block; any other block (a tensor boundary, padding, the end of the buffers) leaves one record per tensor it
// touches, straight into that tensor's slots of the folded table.  Tensor s owns the folded records
// lz_slot_lo[s] .. lz_slot_lo[s + 1] - 1: the first is its part of a shared first block, the last its part of a
// shared last block, and between them its whole blocks added up kSegFoldSpan at a time by the entries of `lz_fold`
// (an entry with hi == lo clears a first or last slot that no block writes).
constexpr int kSegLazyItems = 8;  // float4 groups per array per thread, as in the whole-model form: a full sign row
constexpr uint32_t kSegLazyElems = 256u * kSegLazyItems;
constexpr uint32_t kSegFoldSpan = 1024;
struct SegFold {
    uint32_t slot, lo, hi;  // folded record `slot` = the block records [lo, hi) added in index order
};

struct SegPlan {
    uint32_t S = 0;  // 0 = the plan has no segments: whole-model means over [0, n)
    bool pooled = false;  // one pair of means per worker over all segments together
    uint64_t covered = 0;  // elements inside segments
    std::vector<uint64_t> seg_start, seg_end;
    std::vector<SegItem> item;
    std::vector<uint32_t> item_lo, coarse;
    uint32_t blocks = 0;  // workgroups per worker of the reduction
    std::vector<uint32_t> sched_lo, sched_item;
    std::vector<SegItem> fitem;       // items of the single-launch step; empty if the plan cannot take it
    std::vector<uint32_t> fitem_lo;
    size_t off_fitem = 0, off_fitem_lo = 0, off_frecords = 0;
    size_t off_sign = 0;  // sign words of the two-kernel apply pass and of the lazy state (retained-error mode)
    uint32_t lz_blocks = 0;              // blocks of kSegLazyElems elements by position: ceil(n / kSegLazyElems)
    std::vector<uint32_t> lz_slot_lo;    // [S + 1]
    std::vector<SegFold> lz_fold;
    size_t off_lz_slot_lo = 0, off_lz_fold = 0, off_lz_records = 0, off_lz_folded = 0;
    uint64_t tag = 0;  // checksum of the tables above and of the sizes that fix their layout; never 0
    // byte offsets into the workspace
    size_t off_seg_start = 0, off_seg_end = 0, off_item = 0, off_item_lo = 0, off_coarse = 0, off_sched_lo = 0, off_sched_item = 0,
           off_stats = 0, off_nmp = 0, off_mn = 0, off_gmu = 0, off_records = 0, end = 0;
};

}  // namespace a2sgd

struct a2sgd_plan {
    uint64_t n;
    uint32_t P;
    int32_t mode;
    uint32_t B;           // blocks per worker in the first-level reduction
    bool streaming;       // footprint exceeds the on-chip caches: use non-temporal loads and stores
    a2sgd::ApplyGeom apply;
    int32_t device;       // HIP device the calls must find current, or -1: whichever is current
    // The three fields below change after the plan is made (a single-launch step notes its token; a step that gave
    // up at its barrier switches the plan to the three passes), which is why a plan is not safe to share between
    // host threads without the caller's own lock.
    mutable uint32_t fused_grid;  // workgroups of the single-launch step; 0 = a2sgd_step runs the three passes
    int32_t barrier_cell;         // the grid-barrier cell this plan owns until it is destroyed; -1 = none
    mutable uint32_t last_token;  // token of the last single-launch step enqueued with this plan; 0 = none
    a2sgd::SegPlan seg;
    uint32_t lazy_blocks;  // blocks of 2048 elements: workgroups per worker of the lazy state's reduction pass (one
                           // record each) and rows of sign words
    uint32_t lazy_folded;  // records per worker after k_fold_partials
    size_t lazy_offset;    // byte offset of those records in the workspace; 0 = the plan has no lazy state
    size_t lazy_sign_offset;  // byte offset of the sign words
    size_t eager_bytes;       // header + partial records: all that the three eager passes of a whole-model plan touch
    size_t workspace_bytes;
};

namespace a2sgd {

// Launchers: enqueue on `stream`, return the launch status.  Arguments were validated by the caller.
hipError_t launch_local_partials(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, void *ws, hipStream_t s);
hipError_t launch_local_finalize(const a2sgd_plan_t &pl, void *ws, hipStream_t s);
hipError_t launch_global_average(const a2sgd_plan_t &pl, void *ws, hipStream_t s);
hipError_t launch_export_local_means(const a2sgd_plan_t &pl, const void *ws, float *out, hipStream_t s);
hipError_t launch_import_global_means(const a2sgd_plan_t &pl, void *ws, const float *gmu, hipStream_t s);
// one_kernel: never the two-kernel form (whose sign words need the whole workspace)
hipError_t launch_apply(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                        bool one_kernel, hipStream_t s);
hipError_t launch_fused_step(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                             uint32_t token, hipStream_t s);
hipError_t launch_apply_replicas(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt, bool has_e,
                                 float eta, void *ws, hipStream_t s);
hipError_t launch_dense_step_replicas(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt, float eta,
                                      hipStream_t s);
// Writes 2 * P doubles (max_abs[P], then rms[P]) at ws + drift_result_offset(pl).
hipError_t launch_replica_drift(const a2sgd_plan_t &pl, const ReplicaTable &wt, void *ws, hipStream_t s);
size_t drift_result_offset(const a2sgd_plan_t &pl);
hipError_t launch_lazy_reset(const a2sgd_plan_t &pl, void *ws, hipStream_t s);
hipError_t launch_lazy_partials(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s);
hipError_t launch_lazy_apply(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eta, void *ws, hipStream_t s);
hipError_t launch_lazy_materialize(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s);
// Runs one barrier on the spare cell with `grid` workgroups expecting `expected` arrivals; passed[grid] and
// *cell_failed (device memory) receive the outcome; the spare cell is cleared afterwards.
hipError_t launch_barrier_selftest(uint32_t grid, uint32_t expected, uint32_t spin_limit, uint32_t *passed,
                                   uint32_t *cell_failed, hipStream_t s);
// Puts a grid-barrier cell back into its initial state.  Only for a cell whose grid has drained.
hipError_t launch_barrier_reset(uint32_t cell, hipStream_t s);
// Writes the tag of the uploaded tables into the workspace header and clears its fault flag.
hipError_t launch_seg_mark(const a2sgd_plan_t &pl, void *ws, hipStream_t s);
// Per-tensor means (a2sgd_segments.hip).
SegView seg_view(const a2sgd_plan_t &pl, void *ws);
hipError_t launch_seg_partials(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, void *ws, hipStream_t s);
hipError_t launch_seg_finalize(const a2sgd_plan_t &pl, void *ws, hipStream_t s);
hipError_t launch_seg_global(const a2sgd_plan_t &pl, void *ws, hipStream_t s);
hipError_t launch_seg_apply(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                            hipStream_t s);
// Single-launch step on a plan with tensors (a2sgd_kernels.hip, next to the grid barrier it uses).
FusedSegView fused_seg_view(const a2sgd_plan_t &pl, void *ws);
hipError_t launch_seg_fused_step(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, float *w, float eta, void *ws,
                                 uint32_t token, hipStream_t s);
// Replica calls and the lazy state on plans with tensors.
hipError_t launch_seg_apply_replicas(const a2sgd_plan_t &pl, const PtrTable &tab, const ReplicaTable &wt, bool has_e,
                                     float eta, void *ws, hipStream_t s);
// the whole reduction on the lazy state: first level, fold, second level (means and statistics per tensor)
hipError_t launch_seg_lazy_partials(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s);
// retained-error mode: w from the sign words that launch_seg_lazy_partials left (tab.g = tab.e = the state buffers)
hipError_t launch_seg_lazy_apply_signs(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eta, void *ws,
                                       hipStream_t s);
hipError_t launch_seg_lazy_reset(const a2sgd_plan_t &pl, void *ws, hipStream_t s);
hipError_t launch_seg_materialize(const a2sgd_plan_t &pl, const PtrTable &tab, void *ws, hipStream_t s);
hipError_t launch_export_mask(const a2sgd_plan_t &pl, const PtrTable &tab, bool has_e, uint64_t *mask, hipStream_t s);
hipError_t launch_dense_step(const a2sgd_plan_t &pl, const PtrTable &tab, float *w, float eta, hipStream_t s);

}  // namespace a2sgd
