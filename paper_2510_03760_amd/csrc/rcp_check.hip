// Stand-alone device check of evo_rcp.h: recip_shortcut(x) == 1.0f / x, bit for bit, for
// every binary32 x in [2^-126, 2^126).  Prints the number of mismatches; exit status 0
// iff there is none.  Built by paper_2510_03760_amd/build.py next to the library.
#include <cstdint>
#include <cstdio>

#include "evo_rcp.h"

__global__ void compare_all(unsigned long long *n_bad, uint32_t lo, uint32_t hi) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    unsigned long long bad = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x + lo; i <= hi; i += stride) {
        const float a = __builtin_bit_cast(float, (uint32_t)i);
        const float exact = 1.0f / a;
        const float fast = evo::recip_shortcut(a);
        if (__builtin_bit_cast(uint32_t, exact) != __builtin_bit_cast(uint32_t, fast)) ++bad;
    }
    if (bad) atomicAdd(n_bad, bad);
}

int main() {
    unsigned long long *d_bad = nullptr, bad = 0;
    if (hipMalloc(reinterpret_cast<void **>(&d_bad), sizeof bad) != hipSuccess) return 2;
    if (hipMemcpy(d_bad, &bad, sizeof bad, hipMemcpyHostToDevice) != hipSuccess) return 2;
    const uint32_t lo = 0x00800000u;                                               // 2^-126
    const uint32_t hi = __builtin_bit_cast(uint32_t, evo::kRecipShortcutBelow) - 1u;  // below 2^126
    hipLaunchKernelGGL(compare_all, dim3(4096), dim3(256), 0, 0, d_bad, lo, hi);
    if (hipDeviceSynchronize() != hipSuccess) return 2;
    if (hipMemcpy(&bad, d_bad, sizeof bad, hipMemcpyDeviceToHost) != hipSuccess) return 2;
    std::printf("inputs 0x%08x..0x%08x: %llu mismatches\n", lo, hi, bad);
    return bad == 0 ? 0 : 1;
}
