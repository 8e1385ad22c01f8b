// Launcher of the walking form of the H and dV kernels (tile_walk.h).  A translation unit of its own: it is
// compiled with MFMA results in ordinary vector registers, which lets the register allocator park values in the
// accumulation registers instead of in scratch memory (the kernel keeps 256 registers of X fragments and
// accumulators per lane; a spill to scratch would also be a vector-memory operation the ring does not count).
#include "tile_walk.h"

namespace tfla {

hipError_t launch_tile_walk(const TileArgs& a, int mode, int BH, hipStream_t s) {
    if (!tile_walk_supported(a.d1, a.d2, a.L) || (mode != MODE_H && mode != MODE_DV)) return hipErrorInvalidValue;
    dim3 grid((unsigned)((long)(a.L / 256) * BH * a.Nc));
#ifndef TFLA_WALK_NW
#define TFLA_WALK_NW 8
#endif
    constexpr int NW = TFLA_WALK_NW;
    if (mode == MODE_H) {
        if (a.d1 == 256) hipLaunchKernelGGL((walk_kernel_bf16<256, MODE_H, NW>), grid, dim3(NW * 64), 0, s, a);
        else hipLaunchKernelGGL((walk_kernel_bf16<128, MODE_H, NW>), grid, dim3(NW * 64), 0, s, a);
    } else {
        if (a.d1 == 256) hipLaunchKernelGGL((walk_kernel_bf16<256, MODE_DV, NW>), grid, dim3(NW * 64), 0, s, a);
        else hipLaunchKernelGGL((walk_kernel_bf16<128, MODE_DV, NW>), grid, dim3(NW * 64), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace tfla

#ifdef TFLA_WALK_TL
extern "C" __attribute__((visibility("default"))) int tfla_debug_walk_timeline(unsigned long long* host, size_t n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(tfla::walk_tl), n * sizeof(unsigned long long));
}
#endif
