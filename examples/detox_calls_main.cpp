// A second caller that uses nothing but the C ABI of include/detox.h and the HIP runtime: it
// runs the stages of the parameter-server step as SEPARATE calls (the six named entry points and
// their companions) and prints every result as bit patterns, one value per line behind a tag:
//
//   detox_majority_filter   -> "w"  winner[], votes Z kept in device memory
//   detox_block_mean        -> "z"  the B block means
//   detox_filter_block_mean -> "zf" the same in one pass (must equal "z")
//   robust_coord_median     -> "med"   over the block means
//   robust_trimmed_mean     -> "trim"  over the block means, B/4 dropped at each end
//   robust_geomedian        -> "gm"    over the block means, 20 iterations
//   robust_pairwise_sqdist  -> "dist"  over the votes (64-bit patterns)
//   robust_multikrum        -> "mksel" / "mk"   over the votes, f = 1, m = votes - 3
//   robust_bulyan           -> "bulsel" / "bul" over the votes, f = 1
//   robust_coord_median_many-> "medmany" over all n rows
//   detox_step_robust_blocks-> "rbw" / "rbsel" / "rb": Multi-Krum(f = 1) inside 2 vote groups, mean across
//   detox_sign_majority     -> "sw" / "sp" / "sn" on the bit-packed signs of the same matrix
//
//   detox_calls_main <n> <r> <d> <B> <seed>
//
// The matrix is the one detox_step_main builds: row g*r+k is the vector of node group g,
// x[c] = ((a*c + b) mod 31) - 15 with (a, b) drawn per group from a 31-bit linear congruential
// generator; member k = 1 of every third group is replaced by the constant 9 when r >= 3.
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
#define DETOX_OK_OR_DIE(call)                                                                   \
    do {                                                                                        \
        const int rc_ = (call);                                                                 \
        if (rc_ != DETOX_OK) {                                                                  \
            std::fprintf(stderr, "%s: %s (hip error %d)\n", #call, detox_strerror(rc_),         \
                         detox_last_hip_error());                                               \
            return 3;                                                                           \
        }                                                                                       \
    } while (0)

template <class T>
static int dev_alloc(T **p, size_t count)
{
    return hipMalloc(reinterpret_cast<void **>(p), (count ? count : 1) * sizeof(T)) == hipSuccess ? 0 : 1;
}

static void print_floats(const char *tag, const float *dev, size_t count)
{
    std::vector<float> h(count);
    (void)hipMemcpy(h.data(), dev, count * sizeof(float), hipMemcpyDeviceToHost);
    for (size_t i = 0; i < count; ++i) {
        uint32_t bits;
        std::memcpy(&bits, &h[i], 4);
        std::printf("%s %08x\n", tag, bits);
    }
}

static void print_ints(const char *tag, const int32_t *dev, size_t count)
{
    std::vector<int32_t> h(count);
    (void)hipMemcpy(h.data(), dev, count * sizeof(int32_t), hipMemcpyDeviceToHost);
    for (size_t i = 0; i < count; ++i) std::printf("%s %d\n", tag, h[i]);
}

int main(int argc, char **argv)
{
    if (argc != 6) {
        std::fprintf(stderr, "usage: %s n r d B seed\n", argv[0]);
        return 1;
    }
    const int64_t n = std::atoll(argv[1]);
    const int r = std::atoi(argv[2]);
    const int64_t d = std::atoll(argv[3]), B = std::atoll(argv[4]);
    uint32_t state = (uint32_t)std::atoll(argv[5]);
    if (n <= 0 || r <= 0 || d <= 0 || n % r != 0 || B < 1 || B > n / r) return 1;
    const int64_t V = n / r, words = (d + 31) / 32;

    std::vector<float> G((size_t)(n * d));
    std::vector<uint32_t> S((size_t)(n * words), 0u);
    for (int64_t g = 0; g < V; ++g) {
        state = (1103515245u * state + 12345u) & 0x7fffffffu;
        const uint32_t a = state % 29u + 1u;
        state = (1103515245u * state + 12345u) & 0x7fffffffu;
        const uint32_t b = state % 31u;
        for (int k = 0; k < r; ++k)
            for (int64_t c = 0; c < d; ++c) {
                float x = (float)(int)((a * (uint64_t)c + b) % 31u) - 15.0f;
                if (r >= 3 && g % 3 == 0 && k == 1) x = 9.0f;
                G[(size_t)((g * r + k) * d + c)] = x;
                if (x >= 0.0f) S[(size_t)((g * r + k) * words + c / 32)] |= 1u << (c % 32);
            }
    }

    float *dG, *dZ, *dZhat, *dZf, *dOut, *dBlocks;
    uint32_t *dS, *dPos, *dNeg;
    int32_t *dWinner, *dSel;
    double *dD;
    if (dev_alloc(&dG, G.size()) || dev_alloc(&dZ, (size_t)(V * d)) || dev_alloc(&dZhat, (size_t)(B * d)) ||
        dev_alloc(&dZf, (size_t)(B * d)) || dev_alloc(&dOut, (size_t)d) || dev_alloc(&dBlocks, (size_t)(2 * d)) ||
        dev_alloc(&dS, S.size()) || dev_alloc(&dPos, (size_t)words) || dev_alloc(&dNeg, (size_t)words) ||
        dev_alloc(&dWinner, (size_t)V) || dev_alloc(&dSel, (size_t)V) || dev_alloc(&dD, (size_t)(V * V))) {
        std::fprintf(stderr, "hipMalloc failed\n");
        return 2;
    }
    // one workspace for every call: the largest any of them asks for
    size_t ws_bytes = 256;
    const size_t asks[] = {detox_workspace_bytes(DETOX_OP_FILTER, V, d, 0),
                           detox_workspace_bytes(DETOX_OP_PAIRWISE_SQDIST, V, d, 0),
                           detox_workspace_bytes(DETOX_OP_MULTIKRUM, V, d, 0),
                           detox_workspace_bytes(DETOX_OP_BULYAN, V, d, 0),
                           detox_workspace_bytes(DETOX_OP_GEOMEDIAN, B, d, 0),
                           detox_workspace_bytes(DETOX_OP_COORD_MEDIAN_MANY, n, d, 0),
                           detox_workspace_bytes(DETOX_OP_STEP_ROBUST_BLOCKS, V, d, 2),
                           detox_workspace_bytes(DETOX_OP_FILTER, V, words, 0)};
    for (size_t a : asks) ws_bytes = a > ws_bytes ? a : ws_bytes;
    void *ws = nullptr;
    HIP_OK(hipMalloc(&ws, ws_bytes));
    HIP_OK(hipMemcpy(dG, G.data(), G.size() * sizeof(float), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dS, S.data(), S.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    // the three stages of the step, one call each
    DETOX_OK_OR_DIE(detox_majority_filter(dG, n, d, d, r, nullptr, dWinner, dZ, d, ws, ws_bytes, stream));
    DETOX_OK_OR_DIE(detox_block_mean(dG, d, d, dWinner, V, B, nullptr, dZhat, d, stream));
    HIP_OK(hipStreamSynchronize(stream));
    print_ints("w", dWinner, (size_t)V);
    print_floats("z", dZhat, (size_t)(B * d));
    DETOX_OK_OR_DIE(detox_filter_block_mean(dG, n, d, d, r, nullptr, B, nullptr, dSel, dZf, d, ws, ws_bytes, stream));
    HIP_OK(hipStreamSynchronize(stream));
    print_floats("zf", dZf, (size_t)(B * d));

    DETOX_OK_OR_DIE(robust_coord_median(dZhat, B, d, d, dOut, stream));
    HIP_OK(hipStreamSynchronize(stream));
    print_floats("med", dOut, (size_t)d);
    DETOX_OK_OR_DIE(robust_trimmed_mean(dZhat, B, d, d, (int)(B / 4), dOut, stream));
    HIP_OK(hipStreamSynchronize(stream));
    print_floats("trim", dOut, (size_t)d);
    DETOX_OK_OR_DIE(robust_geomedian(dZhat, B, d, d, 20, 1e-8, dOut, ws, ws_bytes, stream));
    HIP_OK(hipStreamSynchronize(stream));
    print_floats("gm", dOut, (size_t)d);

    // the aggregators on the votes themselves
    DETOX_OK_OR_DIE(robust_pairwise_sqdist(dZ, V, d, d, dD, ws, ws_bytes, stream));
    HIP_OK(hipStreamSynchronize(stream));
    {
        std::vector<double> h((size_t)(V * V));
        HIP_OK(hipMemcpy(h.data(), dD, h.size() * sizeof(double), hipMemcpyDeviceToHost));
        for (double x : h) {
            uint64_t bits;
            std::memcpy(&bits, &x, 8);
            std::printf("dist %016llx\n", (unsigned long long)bits);
        }
    }
    if (V >= 5) {
        const int m = (int)V - 3;
        DETOX_OK_OR_DIE(robust_multikrum(dZ, V, d, d, 1, m, dOut, dSel, nullptr, ws, ws_bytes, stream));
        HIP_OK(hipStreamSynchronize(stream));
        print_ints("mksel", dSel, (size_t)m);
        print_floats("mk", dOut, (size_t)d);
    }
    if (V >= 7) {
        DETOX_OK_OR_DIE(robust_bulyan(dZ, V, d, d, 1, dOut, dSel, ws, ws_bytes, stream));
        HIP_OK(hipStreamSynchronize(stream));
        print_ints("bulsel", dSel, (size_t)(V - 2));
        print_floats("bul", dOut, (size_t)d);
    }
    DETOX_OK_OR_DIE(robust_coord_median_many(dG, n, d, d, dOut, ws, ws_bytes, stream));
    HIP_OK(hipStreamSynchronize(stream));
    print_floats("medmany", dOut, (size_t)d);

    // the deployed hierarchy: Multi-Krum(f = 1, m = size - 1) inside 2 vote groups, mean across
    if (V >= 10) {
        HIP_OK(hipMemset(dSel, 0xff, (size_t)V * sizeof(int32_t)));
        DETOX_OK_OR_DIE(detox_step_robust_blocks(dG, n, d, d, r, nullptr, 2, nullptr, DETOX_AGG_MULTIKRUM, 1, -1,
                                                 dWinner, dBlocks, d, dSel, dOut, ws, ws_bytes, stream));
        HIP_OK(hipStreamSynchronize(stream));
        print_ints("rbw", dWinner, (size_t)V);
        print_ints("rbsel", dSel, (size_t)V);
        print_floats("rb", dOut, (size_t)d);
    }

    // signSGD pairing on the packed signs
    if (B <= 255 && (V + B - 1) / B <= 255) {
        DETOX_OK_OR_DIE(detox_sign_majority(dS, n, d, words, r, nullptr, B, nullptr, dWinner, dPos, dNeg, ws, ws_bytes, stream));
        HIP_OK(hipStreamSynchronize(stream));
        print_ints("sw", dWinner, (size_t)V);
        print_ints("sp", reinterpret_cast<const int32_t *>(dPos), (size_t)words);
        print_ints("sn", reinterpret_cast<const int32_t *>(dNeg), (size_t)words);
    }
    HIP_OK(hipStreamDestroy(stream));
    return 0;
}
