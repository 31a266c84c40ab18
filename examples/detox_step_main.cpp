// A caller of libdetox that uses nothing but the C ABI of include/detox.h and the HIP runtime:
// it fills an n x d matrix in device memory, runs one parameter-server step (filter -> B block
// means -> aggregator) and prints winner[] and the d-vector, one value per line, as the bit
// patterns of the results.
//
//   detox_step_main <n> <r> <d> <B> <aggregator 0..4> <f> <m> <seed>
//
// Row g*r+k of the matrix is the vector of node group g, x[c] = ((a*c + b) mod 31) - 15 with
// (a, b) drawn per group from a 31-bit linear congruential generator seeded with <seed>; member
// k = 1 of every third group is replaced by the constant 9 (one outvoted Byzantine node) when
// r >= 3.  Small integers: every sum below is exact, so the output is checked bit for bit.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/detox.h"

#define HIP_OK(call)                                                                            \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            std::fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));              \
            return 2;                                                                           \
        }                                                                                       \
    } while (0)

int main(int argc, char **argv)
{
    if (argc != 9) {
        std::fprintf(stderr, "usage: %s n r d B aggregator f m seed\n", argv[0]);
        return 1;
    }
    const int64_t n = std::atoll(argv[1]);
    const int r = std::atoi(argv[2]);
    const int64_t d = std::atoll(argv[3]), B = std::atoll(argv[4]);
    const int agg = std::atoi(argv[5]), f = std::atoi(argv[6]), m = std::atoi(argv[7]);
    uint32_t state = (uint32_t)std::atoll(argv[8]);
    if (n <= 0 || r <= 0 || d <= 0 || n % r != 0) return 1;
    const int64_t groups = n / r;

    std::vector<float> G((size_t)(n * d));
    for (int64_t g = 0; g < groups; ++g) {
        state = (1103515245u * state + 12345u) & 0x7fffffffu;
        const uint32_t a = state % 29u + 1u;
        state = (1103515245u * state + 12345u) & 0x7fffffffu;
        const uint32_t b = state % 31u;
        for (int k = 0; k < r; ++k)
            for (int64_t c = 0; c < d; ++c) {
                float x = (float)(int)((a * (uint64_t)c + b) % 31u) - 15.0f;
                if (r >= 3 && g % 3 == 0 && k == 1) x = 9.0f;
                G[(size_t)((g * r + k) * d + c)] = x;
            }
    }

    float *dG = nullptr, *dOut = nullptr, *dZhat = nullptr;
    int32_t *dWinner = nullptr, *dSelected = nullptr;
    void *ws = nullptr;
    const size_t ws_bytes = detox_workspace_bytes(DETOX_OP_STEP, n, d, B);
    HIP_OK(hipMalloc(&dG, G.size() * sizeof(float)));
    HIP_OK(hipMalloc(&dOut, (size_t)d * sizeof(float)));
    HIP_OK(hipMalloc(&dZhat, (size_t)(B * d) * sizeof(float)));
    HIP_OK(hipMalloc(&dWinner, (size_t)groups * sizeof(int32_t)));
    HIP_OK(hipMalloc(&dSelected, (size_t)(B > 0 ? B : 1) * sizeof(int32_t)));
    HIP_OK(hipMalloc(&ws, ws_bytes ? ws_bytes : 256));
    HIP_OK(hipMemcpy(dG, G.data(), G.size() * sizeof(float), hipMemcpyHostToDevice));

    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    const int rc = detox_step(dG, n, d, d, r, /*q=*/0, nullptr, B, nullptr, agg, f, m, 50, 1e-8, dWinner,
                              dZhat, d, dSelected, dOut, ws, ws_bytes, stream);
    if (rc != DETOX_OK) {
        std::fprintf(stderr, "detox_step: %s (hip error %d)\n", detox_strerror(rc), detox_last_hip_error());
        return 3;
    }
    HIP_OK(hipStreamSynchronize(stream));

    std::vector<int32_t> winner((size_t)groups);
    std::vector<float> out((size_t)d);
    HIP_OK(hipMemcpy(winner.data(), dWinner, winner.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(out.data(), dOut, out.size() * sizeof(float), hipMemcpyDeviceToHost));
    for (int64_t g = 0; g < groups; ++g) std::printf("w %d\n", winner[(size_t)g]);
    for (int64_t c = 0; c < d; ++c) {
        uint32_t bits;
        std::memcpy(&bits, &out[(size_t)c], 4);
        std::printf("x %08x\n", bits);
    }
    HIP_OK(hipStreamDestroy(stream));
    HIP_OK(hipFree(dG)); HIP_OK(hipFree(dOut)); HIP_OK(hipFree(dZhat));
    HIP_OK(hipFree(dWinner)); HIP_OK(hipFree(dSelected)); HIP_OK(hipFree(ws));
    return 0;
}
