// Compiled once per TFLA_TILE_MODE (0 = H, 1 = dV, 2 = dQ, 3 = dK): instantiates the tiled
// kernel family of that mode.  The mode is given on the compiler command line.
#ifndef TFLA_TILE_MODE
#error "compile with -DTFLA_TILE_MODE=<0..3>"
#endif
#include "tile.hip"

#if defined(TFLA_TIMELINE)
#define TFLA_CAT2(a, b) a##b
#define TFLA_CAT(a, b) TFLA_CAT2(a, b)
extern "C" __attribute__((visibility("default"))) int TFLA_CAT(tfla_debug_timeline_mode, TFLA_TILE_MODE)(unsigned long long* host, size_t n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(tfla::tfla_timeline), n * sizeof(unsigned long long));
}
#endif
