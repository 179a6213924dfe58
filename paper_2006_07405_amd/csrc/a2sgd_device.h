// Device-side helpers shared by the kernel files: 128-bit streaming loads and stores, the per-lane accumulator of
// the reduction, and the per-element arithmetic of the apply pass.  Included by .hip files only.
#pragma once

#include "a2sgd_internal.h"

namespace a2sgd {

typedef float vf4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ vf4 ld4(const vf4 *p)
{
    if (NT)
        return __builtin_nontemporal_load(p);
    return *p;
}

// Streaming store: non-temporal and written through at device scope (sc1), so the line does not linger in the
// XCD's write-back L2.  Measured on the apply pass's mix of 9 read and 5 write streams: 4.5 % faster than the
// non-temporal hint alone, 14 % faster than plain stores.  The instruction is spelled out because the compiler
// offers no builtin for the scope bit on a 128-bit store (and its non-temporal metadata has been seen to get
// lost on the way through the optimiser).  The s_nop belongs to the store: on this chip a vector instruction
// must not overwrite the data registers of a store wider than 64 bits within 2 wait states of it, a hazard the
// compiler pads by itself for its own stores but cannot see inside an asm statement.
template <bool NT>
__device__ __forceinline__ void st4(vf4 *p, vf4 v)
{
    if (NT)
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else
        *p = v;
}

// ---------------------------------------------------------------------------------------------------------
// First-level reduction (Algorithm 1 line 3; group definitions of Sec. 3.1)
// ---------------------------------------------------------------------------------------------------------

// Running sums and counts of one lane.  Sums in fp64 so that the fp32 means come out the same as an exactly
// summed reference; counts are taken per wavefront with a ballot and a scalar popcount, which keeps them off
// the vector ALU.  A NaN fails both comparisons: it is counted nowhere and added to neither sum.
struct LaneAcc {
    double s_pos = 0.0, s_neg = 0.0;
    // Counts of the whole wavefront, identical in every active lane.  The block reduction reads them from
    // lane 0, which is active whenever any lane of its wavefront is (indices grow with the lane number).
    // 32 bits hold one tile's worth (at most 64 * 16 per call of flush); the totals are 64-bit.
    uint32_t t_pos = 0, t_neg = 0, t_zero = 0;
    uint64_t c_pos = 0, c_neg = 0, c_zero = 0;

    __device__ __forceinline__ void add(float v)
    {
        const bool ge = v >= 0.0f;
        const bool lt = v < 0.0f;
        s_pos += static_cast<double>(ge ? v : 0.0f);
        s_neg -= static_cast<double>(lt ? v : 0.0f);
        t_pos += __popcll(__ballot(ge));
        t_neg += __popcll(__ballot(lt));
        t_zero += __popcll(__ballot(v == 0.0f));
    }
    __device__ __forceinline__ void flush()
    {
        c_pos += t_pos;
        c_neg += t_neg;
        c_zero += t_zero;
        t_pos = t_neg = t_zero = 0;
    }
    __device__ __forceinline__ void add4(vf4 v)
    {
        add(v.x);
        add(v.y);
        add(v.z);
        add(v.w);
    }
};

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x += __shfl_down(x, off);
    return x;  // valid in lane 0; the tree shape is fixed, so the result is reproducible
}

__device__ __forceinline__ uint64_t wave_sum(uint64_t x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x += __shfl_down(static_cast<unsigned long long>(x), off);
    return x;
}

// One record of the reduction: the sums of the two groups, their sizes, and the zeros among the first.
struct Sums {
    double s_pos = 0.0, s_neg = 0.0;
    uint64_t n_pos = 0, n_neg = 0, n_zero = 0;
};

__device__ __forceinline__ void add_record(Sums &a, const Partials &t, const size_t slot)
{
    a.s_pos += t.s_pos[slot];
    a.s_neg += t.s_neg[slot];
    a.n_pos += t.n_pos[slot];
    a.n_neg += t.n_neg[slot];
    a.n_zero += t.n_zero[slot];
}

__device__ __forceinline__ void store_record(const Partials &t, const size_t slot, const Sums &r)
{
    t.s_pos[slot] = r.s_pos;
    t.s_neg[slot] = r.s_neg;
    t.n_pos[slot] = r.n_pos;
    t.n_neg[slot] = r.n_neg;
    t.n_zero[slot] = r.n_zero;
}

// Adds one record per wavefront (valid in lane 0 of each) over a workgroup of kBlock threads, wavefronts in index
// order; the total is valid in thread 0.  Every thread of the workgroup calls it; before a second call the
// workgroup needs a __syncthreads() of its own, since the staging slots are reused.
__device__ __forceinline__ Sums block_sum_of_waves(const Sums &wave_total)
{
    __shared__ double sh_pos[kBlock / 64], sh_neg[kBlock / 64];
    __shared__ uint64_t sh_cp[kBlock / 64], sh_cn[kBlock / 64], sh_cz[kBlock / 64];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        sh_pos[wave] = wave_total.s_pos;
        sh_neg[wave] = wave_total.s_neg;
        sh_cp[wave] = wave_total.n_pos;
        sh_cn[wave] = wave_total.n_neg;
        sh_cz[wave] = wave_total.n_zero;
    }
    __syncthreads();
    Sums total;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 0; k < kBlock / 64; ++k) {
            total.s_pos += sh_pos[k];
            total.s_neg += sh_neg[k];
            total.n_pos += sh_cp[k];
            total.n_neg += sh_cn[k];
            total.n_zero += sh_cz[k];
        }
    }
    return total;
}

// The same for one record per thread: shuffle tree inside each wavefront first.  The order is fixed, so the result
// is reproducible.
__device__ __forceinline__ Sums block_sum(Sums mine)
{
    mine.s_pos = wave_sum(mine.s_pos);
    mine.s_neg = wave_sum(mine.s_neg);
    mine.n_pos = wave_sum(mine.n_pos);
    mine.n_neg = wave_sum(mine.n_neg);
    mine.n_zero = wave_sum(mine.n_zero);
    return block_sum_of_waves(mine);
}

// One element of one worker: rewrites v into the new error and returns that worker's contribution u to the
// update.  Written as selects on register values so that it compiles to v_cndmask, not to branches.  A NaN
// fails v >= 0, so v + mu_neg keeps it NaN in e; the extra select keeps it NaN in u as well.
template <int MODE>
__device__ __forceinline__ float apply1(float &v, float neg_mu_pos, float mu_neg, float gmu_pos, float neg_gmu_neg)
{
    const bool ge = v >= 0.0f;
    const float err = v + (ge ? neg_mu_pos : mu_neg);  // v - enc(v): Eq. 2, Algorithm 1 line 4
    float glob = ge ? gmu_pos : neg_gmu_neg;           // global-mean vector at this position: line 6
    glob = (v != v) ? v : glob;
    v = err;
    return MODE == A2SGD_MODE_ALG1_LITERAL ? err + glob : glob;
}

// Four elements of one worker.  Returns the new error as a fresh value (storing a value that was updated in
// place in a register array has been seen to lose its non-temporal hint on the way through the optimiser).
template <int MODE>
__device__ __forceinline__ vf4 apply4(vf4 v, vf4 &acc, float neg_mu_pos, float mu_neg, float gmu_pos,
                                      float neg_gmu_neg)
{
    float x = v.x, y = v.y, z = v.z, t = v.w;
    acc.x += apply1<MODE>(x, neg_mu_pos, mu_neg, gmu_pos, neg_gmu_neg);
    acc.y += apply1<MODE>(y, neg_mu_pos, mu_neg, gmu_pos, neg_gmu_neg);
    acc.z += apply1<MODE>(z, neg_mu_pos, mu_neg, gmu_pos, neg_gmu_neg);
    acc.w += apply1<MODE>(t, neg_mu_pos, mu_neg, gmu_pos, neg_gmu_neg);
    return vf4{x, y, z, t};
}

// The pending error of one stored element of the lazy state: s - enc(s) with the carried means (Eq. 2, Algorithm 1
// line 4).  A NaN stays a NaN.
__device__ __forceinline__ float pending_error(float s, float neg_mu_pos, float mu_neg)
{
    return s + (s >= 0.0f ? neg_mu_pos : mu_neg);
}

__device__ __forceinline__ vf4 pending_error4(vf4 s, float neg_mu_pos, float mu_neg)
{
    return vf4{pending_error(s.x, neg_mu_pos, mu_neg), pending_error(s.y, neg_mu_pos, mu_neg),
               pending_error(s.z, neg_mu_pos, mu_neg), pending_error(s.w, neg_mu_pos, mu_neg)};
}

// The kernels of plans with tensors index through tables that a2sgd_workspace_init uploads.  Before its first such access every
// workgroup compares the tag in the workspace header with the tag of its plan's tables; on a mismatch (the
// workspace was never initialised, or for another plan) it raises the header's fault flag and the caller returns
// without reading a table entry or writing any output.  The answer is the same for every thread of the grid.
__device__ __forceinline__ bool seg_tables_ok(const SegView &sv)
{
    if (sv.hdr->seg_tag == sv.tag)
        return true;
    if (threadIdx.x == 0)
        sv.hdr->seg_fault = 1u;  // every writer stores the same value
    return false;
}

// Where the sign words of worker p for half h of the 2048-element block b start: uint16_t sign[blocks][2][P][64].
// A workgroup of the pass that reads them covers one (b, h) and finds every worker's 128 bytes side by side.
__device__ __forceinline__ uint16_t *sign_row(uint16_t *sign, const uint32_t P, const uint64_t b, const uint32_t h,
                                              const uint32_t p)
{
    return sign + ((b * 2 + h) * P + p) * 64;
}

// Shifts pos(v) of the four components into the low end of `bits`, x first.
__device__ __forceinline__ uint32_t push_signs(uint32_t bits, vf4 v)
{
    bits = bits * 2u + (v.x >= 0.0f ? 1u : 0u);
    bits = bits * 2u + (v.y >= 0.0f ? 1u : 0u);
    bits = bits * 2u + (v.z >= 0.0f ? 1u : 0u);
    bits = bits * 2u + (v.w >= 0.0f ? 1u : 0u);
    return bits;
}

// A zero the compiler cannot see through, in a vector register.  Added to an index it turns a load with a
// wavefront-uniform address into an ordinary vector load.  The apply pass wants that for the handful of means
// it reads from the workspace: vector loads return in issue order and are counted apart from the scalar loads
// of the kernel arguments, so when they are issued first they cost a freshly launched workgroup no wait of
// their own, whereas a scalar load would be waited for together with the kernel-argument pointers before the
// first big load could be issued.
__device__ __forceinline__ uint32_t opaque_zero()
{
    uint32_t z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

}  // namespace a2sgd
