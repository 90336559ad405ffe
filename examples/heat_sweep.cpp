// libstencil from plain C++ through its C ABI: 1000 steps of the heat equation on a 1024 x 1024
// matrix with wrap-around borders, the workgroup-size sweep of Section 5 of the paper, and a run
// at the size the sweep found.  No Python, no PyTorch: device memory comes from the HIP runtime.
//
//   hipcc -O2 examples/heat_sweep.cpp -Iinclude -Lpaper_1511_02490_amd/_lib -lstencil \
//         -Wl,-rpath,$PWD/paper_1511_02490_amd/_lib -o heat_sweep && ./heat_sweep [training pairs]
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <vector>

#include "libstencil.h"

#define HIP_OK(call)                                                                    \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess) {                                                         \
            std::fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));             \
            return 1;                                                                   \
        }                                                                               \
    } while (0)
#define STENCIL_OK_OR_DIE(call)                                                         \
    do {                                                                                \
        if ((call) < 0) {                                                               \
            std::fprintf(stderr, "%s: %s\n", #call, stencil_last_error());              \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

int main(int argc, char **argv) {
    const int rows = 1024, cols = 1024, steps = 1000;
    std::vector<float> host((size_t)rows * cols, 1.0f);
    for (int r = 400; r < 432; ++r)
        for (int c = 600; c < 632; ++c) host[(size_t)r * cols + c] = 1000.0f;   // a hot square
    double before = 0.0;
    for (float v : host) before += v;

    float *in = nullptr, *out = nullptr;
    const size_t bytes = host.size() * sizeof(float);
    HIP_OK(hipMalloc((void **)&in, bytes));
    HIP_OK(hipMalloc((void **)&out, bytes));
    HIP_OK(hipMemcpy(in, host.data(), bytes, hipMemcpyHostToDevice));

    stencil_t *st = nullptr;
    STENCIL_OK_OR_DIE(stencil_create(&st, rows, cols, STENCIL_F32, 1, 1, 1, 1, STENCIL_WRAP));
    const float alpha = 0.2f;
    STENCIL_OK_OR_DIE(stencil_set_kernel(st, STENCIL_HEAT, nullptr, 0, &alpha, 1));
    STENCIL_OK_OR_DIE(stencil_set_mapping(st, STENCIL_STAGING_DIRECT, 2, 4));

    // Before anything is swept the library chooses by itself (wg 0x0): with training pairs recorded
    // on this device (argv[1], e.g. paper_1511_02490_amd/tuning_data/mi355x_local_2_4.txt) it asks
    // a decision tree over the scenario's features, otherwise it takes its built-in default.
    stencil_predictor_t *pred = nullptr;
    if (argc > 1) {
        STENCIL_OK_OR_DIE(stencil_predictor_load(&pred, argv[1], STENCIL_CLASSIFIER_TREE));
        STENCIL_OK_OR_DIE(stencil_attach_predictor(st, pred, STENCIL_FALLBACK_NEAREST));
    }
    int guess_r = 0, guess_c = 0;
    STENCIL_OK_OR_DIE(stencil_default_wg(st, &guess_r, &guess_c));
    STENCIL_OK_OR_DIE(stencil_run(st, in, out, 10, 0, 0, nullptr));
    std::printf("%s size before any sweep: %dx%d\n", pred ? "predicted" : "default", guess_r, guess_c);

    // every power-of-two workgroup size up to the kernel's limit, 30 samples of 10 steps each
    const int w_max = stencil_max_wg_size(st);
    const int n = stencil_enumerate_wg(STENCIL_ENUM_POW2, w_max, nullptr, nullptr, 0);
    std::vector<int> wr(n), wc(n), status(n);
    std::vector<double> mean(n);
    STENCIL_OK_OR_DIE(stencil_enumerate_wg(STENCIL_ENUM_POW2, w_max, wr.data(), wc.data(), n));
    int best = -1;
    double speedup = 0.0;
    STENCIL_OK_OR_DIE(stencil_sweep_wg(st, in, out, 10, wr.data(), wc.data(), n, 4, 4, 30, mean.data(), nullptr, nullptr,
                                       nullptr, status.data(), &best, &speedup, nullptr));
    if (best < 0) {
        std::fprintf(stderr, "no legal workgroup size\n");
        return 1;
    }
    std::printf("%d sizes swept; best %dx%d: %.2f us per step, %.2fx over 4x4\n", n, wr[best], wc[best],
                mean[best] / 10 * 1e3, speedup);

    // wg 0x0: the size the sweep just found
    STENCIL_OK_OR_DIE(stencil_run(st, in, out, steps, 0, 0, nullptr));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(host.data(), out, bytes, hipMemcpyDeviceToHost));
    double after = 0.0;
    float peak = 0.0f;
    for (float v : host) {
        after += v;
        peak = std::fmax(peak, v);
    }
    // periodic borders conserve the total; diffusion has flattened the square
    std::printf("total %.1f -> %.1f, hottest cell 1000 -> %.2f after %d steps\n", before, after, peak, steps);
    stencil_destroy(st);
    stencil_predictor_destroy(pred);
    HIP_OK(hipFree(in));
    HIP_OK(hipFree(out));
    return (std::fabs(after - before) <= 1e-4 * before && peak < 500.0f) ? 0 : 2;
}
