// Benchmark infrastructure, not part of the A2SGD path: plain streaming kernels that show what this device's HBM
// gives to the access mixes the step's two passes have, so that bench.py can report the step's bandwidth next to a
// measured ceiling and not only next to the published peak.  "Plain" means: 128-bit non-temporal loads and stores
// through the compiler's own builtins, every wavefront the grid has resident at once, no residency cap, no
// write-through stores; a kernel of the step that beats the matching line here does so through those measures.
//
//   kind 0  read      1 read stream                      (the reduction pass reads 2P streams and writes nothing)
//   kind 1  copy      1 read stream, 1 write stream
//   kind 2  add       2 read streams, 1 write stream
//   kind 3  mix       R read streams of which the first W are updated in place: the apply pass's mix, R = 2P + 1,
//                     W = P + 1 (e^p and w are read and written, g^p only read)
//   kind 4  fill      1 write stream, nothing read        (what the writes of a pass cost on their own)
//
// C ABI (built into libhbm_streams.so, loaded by bench.py with ctypes):
//   int hbm_stream_run(int kind, float *const *buf, int reads, int writes, uint64_t n, void *stream)
//     buf: HOST array of `reads` DEVICE pointers to n floats each, 16-byte aligned; buffers 0..writes-1 are written.
//     kind 0: reads = 1, writes = 0 (buf[1] must point to at least 4 bytes: receives a value that is never set in
//     practice, which keeps the loads alive); kind 1: reads = 2 (buf[1] <- buf[0]); kind 2: reads = 3
//     (buf[0] <- buf[1] + buf[2]); kind 3: reads = 2P + 1 and writes = P + 1 for P = 1, 2, 4, 8 or 16; kind 4:
//     reads = 0, writes = 1 (buf[0] <- a constant).
//     Enqueues one kernel on `stream` and returns 0, or a nonzero code if the arguments are wrong or the launch failed.
//   uint64_t hbm_stream_bytes(int kind, int reads, int writes, uint64_t n): bytes that launch moves.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float vf4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kMaxStreams = 33;
struct StreamTable {
    float *p[kMaxStreams];
};

// Persistent grid: workgroup b takes tiles b, b + G, ... of 256 * 8 float4 groups, all 8 loads of a thread issued
// before the first use.
__global__ __launch_bounds__(256) void k_read(const vf4 *__restrict__ a, const uint64_t nvec, float *__restrict__ sink)
{
    vf4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    constexpr uint64_t kTile = 256 * 8;
    for (uint64_t t = blockIdx.x; t * kTile < nvec; t += gridDim.x) {
        vf4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint64_t i = t * kTile + u * 256 + threadIdx.x;
            v[u] = i < nvec ? __builtin_nontemporal_load(a + i) : vf4{0.0f, 0.0f, 0.0f, 0.0f};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc += v[u];
    }
    if (acc.x + acc.y + acc.z + acc.w == 1.2345678e30f)  // never true for the benchmark's data
        sink[0] = acc.x;
}

// One-shot grid of 256-thread workgroups, one float4 group per thread and stream (of the plain shapes tried on this
// device the fastest copy).
__global__ __launch_bounds__(256) void k_copy(const vf4 *__restrict__ a, vf4 *__restrict__ b, const uint64_t nvec)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < nvec)
        __builtin_nontemporal_store(__builtin_nontemporal_load(a + i), b + i);
}

__global__ __launch_bounds__(256) void k_fill(vf4 *__restrict__ a, const uint64_t nvec, const float value)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < nvec)
        __builtin_nontemporal_store(vf4{value, value, value, value}, a + i);
}

__global__ __launch_bounds__(256) void k_add(vf4 *__restrict__ c, const vf4 *__restrict__ a, const vf4 *__restrict__ b,
                                             const uint64_t nvec)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < nvec) {
        const vf4 x = __builtin_nontemporal_load(a + i), y = __builtin_nontemporal_load(b + i);
        __builtin_nontemporal_store(x + y, c + i);
    }
}

// One float4 group per thread and stream: all R loads first, then stream j < W <- stream j + stream W + j % (R - W).
template <int R, int W>
__global__ __launch_bounds__(64) void k_mix(const StreamTable tab, const uint64_t nvec)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 64 + threadIdx.x;
    if (i >= nvec)
        return;
    vf4 v[R];
#pragma unroll
    for (int k = 0; k < R; ++k)
        v[k] = __builtin_nontemporal_load(reinterpret_cast<const vf4 *>(tab.p[k]) + i);
#pragma unroll
    for (int j = 0; j < W; ++j)
        __builtin_nontemporal_store(v[j] + v[W + j % (R - W)], reinterpret_cast<vf4 *>(tab.p[j]) + i);
}

template <int R, int W>
void launch_mix(const StreamTable &tab, uint64_t nvec, hipStream_t s)
{
    k_mix<R, W><<<dim3(static_cast<uint32_t>((nvec + 63) / 64)), dim3(64), 0, s>>>(tab, nvec);
}

}  // namespace

extern "C" {

uint64_t hbm_stream_bytes(int kind, int reads, int writes, uint64_t n)
{
    switch (kind) {
    case 0: return 4 * n;
    case 1: return 8 * n;
    case 2: return 12 * n;
    case 3: return 4 * n * static_cast<uint64_t>(reads + writes);
    case 4: return 4 * n;
    }
    return 0;
}

int hbm_stream_run(int kind, float *const *buf, int reads, int writes, uint64_t n, void *stream)
{
    if (buf == nullptr || n == 0 || (n & 3) != 0 || n > (1ull << 38))
        return 1;
    const int need = kind == 0 ? 2 : kind == 1 ? 2 : kind == 2 ? 3 : kind == 4 ? 1 : reads;
    if (kind < 0 || kind > 4)
        return 1;
    if (kind == 3 && ((reads != 3 && reads != 5 && reads != 9 && reads != 17 && reads != 33) || writes != (reads + 1) / 2))
        return 1;
    for (int k = 0; k < need; ++k)
        if (buf[k] == nullptr || (reinterpret_cast<uintptr_t>(buf[k]) & 15u) != 0)
            return 2;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t nvec = n >> 2;
    if (kind == 0) {
        int device = 0, cus = 0;
        if (hipGetDevice(&device) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
            return 3;
        k_read<<<dim3(2 * cus), dim3(256), 0, s>>>(reinterpret_cast<const vf4 *>(buf[0]), nvec, buf[1]);
    } else if (kind == 1) {
        k_copy<<<dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0, s>>>(
            reinterpret_cast<const vf4 *>(buf[0]), reinterpret_cast<vf4 *>(buf[1]), nvec);
    } else if (kind == 2) {
        k_add<<<dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0, s>>>(
            reinterpret_cast<vf4 *>(buf[0]), reinterpret_cast<const vf4 *>(buf[1]),
            reinterpret_cast<const vf4 *>(buf[2]), nvec);
    } else if (kind == 4) {
        k_fill<<<dim3(static_cast<uint32_t>((nvec + 255) / 256)), dim3(256), 0, s>>>(reinterpret_cast<vf4 *>(buf[0]), nvec,
                                                                                       1.0e-3f);
    } else {
        StreamTable tab;
        for (int k = 0; k < kMaxStreams; ++k)
            tab.p[k] = k < reads ? buf[k] : nullptr;
        switch (reads) {  // writes == (reads + 1) / 2 was checked above
        case 3: launch_mix<3, 2>(tab, nvec, s); break;
        case 5: launch_mix<5, 3>(tab, nvec, s); break;
        case 9: launch_mix<9, 5>(tab, nvec, s); break;
        case 17: launch_mix<17, 9>(tab, nvec, s); break;
        default: launch_mix<33, 17>(tab, nvec, s); break;
        }
    }
    return hipGetLastError() == hipSuccess ? 0 : 3;
}

}  // extern "C"
