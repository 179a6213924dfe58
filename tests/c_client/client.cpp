// A caller of the C ABI that uses nothing but the HIP runtime and include/a2sgd.h: reads P gradients, P errors and
// the weights (fp32, raw) from a file, runs one whole-model step on the GPU and writes the per-worker statistics,
// the global means, the new errors and the new weights to another file.  Built by build(); run by a GPU test, which
// writes the input with numpy and checks the output against the CPU oracle.
//
//   client <in> <out> <n> <P> <mode> <eta> <calls: 0 = a2sgd_step, 1 = the three calls, 2 = a2sgd_step_static>
// After a2sgd_step_static there are no statistics to read (it has no workspace): that part of the output is zeros.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#include "a2sgd.h"

#define CHECK_HIP(x)                                                                     \
    do {                                                                                 \
        hipError_t err_ = (x);                                                           \
        if (err_ != hipSuccess) {                                                        \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(err_));               \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define CHECK_A2SGD(x)                                                                   \
    do {                                                                                 \
        a2sgd_status_t st_ = (x);                                                        \
        if (st_ != A2SGD_OK) {                                                           \
            std::fprintf(stderr, "%s: %s\n", #x, a2sgd_status_string(st_));              \
            return 3;                                                                    \
        }                                                                                \
    } while (0)

int main(int argc, char **argv)
{
    if (argc != 8) {
        std::fprintf(stderr, "usage: client <in> <out> <n> <P> <mode> <eta> <calls>\n");
        return 1;
    }
    const uint64_t n = std::strtoull(argv[3], nullptr, 10);
    const uint32_t P = static_cast<uint32_t>(std::atoi(argv[4]));
    const int mode = std::atoi(argv[5]);
    const float eta = static_cast<float>(std::atof(argv[6]));
    const int calls = std::atoi(argv[7]);

    std::vector<float> host(n * (2ull * P + 1));
    std::FILE *in = std::fopen(argv[1], "rb");
    if (in == nullptr || std::fread(host.data(), sizeof(float), host.size(), in) != host.size())
        return 1;
    std::fclose(in);

    a2sgd_config_t cfg = {};
    cfg.n = n;
    cfg.num_workers = P;
    cfg.mode = mode;
    cfg.device = 0;  // this program runs on HIP device 0
    a2sgd_plan_t *plan = nullptr;
    CHECK_A2SGD(a2sgd_plan(&cfg, &plan));

    std::vector<float *> g(P), e(P);
    float *w = nullptr;
    void *workspace = nullptr;
    for (uint32_t p = 0; p < P; ++p) {
        CHECK_HIP(hipMalloc(reinterpret_cast<void **>(&g[p]), n * sizeof(float)));
        CHECK_HIP(hipMalloc(reinterpret_cast<void **>(&e[p]), n * sizeof(float)));
        CHECK_HIP(hipMemcpy(g[p], host.data() + p * n, n * sizeof(float), hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(e[p], host.data() + (P + p) * n, n * sizeof(float), hipMemcpyHostToDevice));
    }
    CHECK_HIP(hipMalloc(reinterpret_cast<void **>(&w), n * sizeof(float)));
    CHECK_HIP(hipMemcpy(w, host.data() + 2ull * P * n, n * sizeof(float), hipMemcpyHostToDevice));
    const size_t workspace_bytes = a2sgd_workspace_bytes(plan);
    CHECK_HIP(hipMalloc(&workspace, workspace_bytes));
    CHECK_A2SGD(a2sgd_workspace_check(plan, workspace, workspace_bytes));
    if (a2sgd_workspace_check(plan, workspace, workspace_bytes - 1) != A2SGD_ERR_WORKSPACE_TOO_SMALL) {
        std::fprintf(stderr, "a2sgd_workspace_check accepted a workspace one byte short\n");
        return 4;
    }

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    std::vector<a2sgd_worker_stats_t> stats(P);
    a2sgd_global_stats_t global = {};
    if (calls == 2) {
        CHECK_A2SGD(a2sgd_step_static(plan, g.data(), e.data(), w, eta, stream));
        CHECK_HIP(hipStreamSynchronize(stream));
    } else if (calls == 1) {
        CHECK_A2SGD(a2sgd_local_averages(plan, g.data(), e.data(), workspace, stream));
        CHECK_A2SGD(a2sgd_global_average(plan, workspace, stream));
        CHECK_A2SGD(a2sgd_apply_and_update_error(plan, g.data(), e.data(), w, eta, workspace, stream));
    } else {
        CHECK_A2SGD(a2sgd_step(plan, g.data(), e.data(), w, eta, workspace, stream));
    }
    if (calls != 2)
        CHECK_A2SGD(a2sgd_read_stats(plan, workspace, stream, stats.data(), &global));  // waits for the stream

    std::FILE *out = std::fopen(argv[2], "wb");
    if (out == nullptr)
        return 1;
    std::fwrite(stats.data(), sizeof(a2sgd_worker_stats_t), P, out);
    std::fwrite(&global, sizeof(global), 1, out);
    for (uint32_t p = 0; p < P; ++p) {
        CHECK_HIP(hipMemcpy(host.data(), e[p], n * sizeof(float), hipMemcpyDeviceToHost));
        std::fwrite(host.data(), sizeof(float), n, out);
    }
    CHECK_HIP(hipMemcpy(host.data(), w, n * sizeof(float), hipMemcpyDeviceToHost));
    std::fwrite(host.data(), sizeof(float), n, out);
    std::fclose(out);

    for (uint32_t p = 0; p < P; ++p) {
        CHECK_HIP(hipFree(g[p]));
        CHECK_HIP(hipFree(e[p]));
    }
    CHECK_HIP(hipFree(w));
    CHECK_HIP(hipFree(workspace));
    CHECK_HIP(hipStreamDestroy(stream));
    CHECK_A2SGD(a2sgd_plan_destroy(plan));
    return 0;
}
