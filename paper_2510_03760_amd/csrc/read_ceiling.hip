// Read-only streaming ceiling of the device: a trivial kernel that reads 8 GiB once and
// keeps nothing (XOR of all words, compared with a value it cannot have).  It gives the
// rate the check kernel's loads could reach if nothing else cost anything, so that an
// achieved bandwidth can be quoted against what the machine delivers as well as against
// the vendor's peak.  Stand-alone program, not part of libevo.so:
//     read_ceiling [GiB]            prints one JSON line
// Each thread issues U independent 16-byte loads per iteration; consecutive lanes read
// consecutive vectors.  "nt" marks the loads non-temporal, as the check kernel does for
// data it reads once.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int U, bool NT>
__global__ void __launch_bounds__(256) read_all(const u32x4 *__restrict__ p, size_t nvec, uint32_t *out) {
    const size_t stride = (size_t)gridDim.x * 256 * U;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i + 256 * (U - 1) < nvec; i += stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = NT ? __builtin_nontemporal_load(&p[i + u * 256]) : p[i + u * 256];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;   // the buffer holds 0x01 bytes
}

#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::fprintf(stderr, "%s: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

template <typename K>
static int timed(K kern, int grid, const u32x4 *d, size_t nvec, uint32_t *out, double *gbps) {
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, 0, d, nvec, out);
    CK(hipEventRecord(a));
    const int reps = 10;
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, 0, d, nvec, out);
    CK(hipEventRecord(b));
    CK(hipEventSynchronize(b));
    CK(hipGetLastError());
    float ms = 0.0f;
    CK(hipEventElapsedTime(&ms, a, b));
    *gbps = (double)nvec * 16.0 / (ms / reps) / 1e6;
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
    return 0;
}

int main(int argc, char **argv) {
    const size_t gib = argc > 1 ? (size_t)std::atoi(argv[1]) : 8;
    if (gib < 1 || gib > 64) {
        std::fprintf(stderr, "usage: read_ceiling [GiB, 1..64]\n");
        return 2;
    }
    const size_t bytes = gib << 30, nvec = bytes / 16;
    u32x4 *d = nullptr;
    uint32_t *out = nullptr;
    CK(hipMalloc(&d, bytes));
    CK(hipMemset(d, 1, bytes));
    CK(hipMalloc(&out, 4));
    CK(hipMemset(out, 0, 4));
    double best_nt = 0.0, best_plain = 0.0, g = 0.0;
    const int grids[] = {1024, 2048, 4096, 16384};
    for (int grid : grids) {
        if (timed(read_all<4, true>, grid, d, nvec, out, &g)) return 1;
        if (g > best_nt) best_nt = g;
        if (timed(read_all<8, true>, grid, d, nvec, out, &g)) return 1;
        if (g > best_nt) best_nt = g;
        if (timed(read_all<8, false>, grid, d, nvec, out, &g)) return 1;
        if (g > best_plain) best_plain = g;
    }
    std::printf("{\"read_ceiling_gib\": %zu, \"nontemporal_GBps\": %.0f, \"plain_GBps\": %.0f}\n", gib,
                best_nt, best_plain);
    CK(hipFree(d));
    CK(hipFree(out));
    return 0;
}
