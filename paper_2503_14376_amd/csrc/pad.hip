// Sequence lengths that are not a multiple of the chunk size (App. B.2 defines N_c = ceil(T / L))
// and head dimensions between the kernels' own (64, 128, 256, 512):
// the kernels work on whole chunks and on those widths, so the library copies the inputs into
// buffers of N_c L steps per (batch, head) and the next supported width inside the caller's
// workspace, zero-filling the steps past T and the columns past the head dimension, runs the
// kernels there, and copies the first T steps and the true columns of the results back.  Zero
// columns of q and k add nothing to any q . k, zero columns of v give zero columns of the output.  A zero k, v (and upstream
// gradient) row contributes nothing to any state, output or gradient, and the gate kernels give
// the padded steps a forget gate of one and an input gate of zero, so the result is exactly
// that of the shorter sequence.
#include "tfla_device.h"
#include "tfla_internal.h"

namespace tfla {

namespace {

// rows of 16-byte words; (BH, T, rw) -> (BH, Tp, rwp), zero outside the source
__global__ void __launch_bounds__(256) pad_rows_kernel(const uint4* in, uint4* out, long total, int T, int Tp, int rw, int rwp) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long bh = i / ((long)Tp * rwp);
        const long rem = i - bh * (long)Tp * rwp;
        const int t = (int)(rem / rwp), w = (int)(rem - (long)t * rwp);
        out[i] = (t < T && w < rw) ? in[((long)bh * T + t) * rw + w] : make_uint4(0u, 0u, 0u, 0u);
    }
}
// (BH, Tp, rwp) -> (BH, T, rw)
__global__ void __launch_bounds__(256) unpad_rows_kernel(const uint4* in, uint4* out, long total, int T, int Tp, int rw, int rwp) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long bh = i / ((long)T * rw);
        const long rem = i - bh * (long)T * rw;
        const int t = (int)(rem / rw), w = (int)(rem - (long)t * rw);
        out[i] = in[(bh * (long)Tp + t) * rwp + w];
    }
}
__global__ void __launch_bounds__(256) pad_scalar_kernel(const float* in, float* out, long total, int T, int Tp, float fill) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long bh = i / Tp;
        const int t = (int)(i - bh * Tp);
        out[i] = t < T ? in[bh * T + t] : fill;
    }
}
__global__ void __launch_bounds__(256) unpad_scalar_kernel(const float* in, float* out, long total, int T, int Tp) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const long bh = i / T;
        out[i] = in[bh * Tp + (i - bh * T)];
    }
}

inline unsigned grid_for(long total) {
    const long g = (total + 255) / 256;
    return (unsigned)(g < 1 ? 1 : (g > 65536 ? 65536 : g));
}

}  // namespace

hipError_t launch_pad_rows(const void* in, void* out, long BH, int T, int Tp, int row_bytes, int row_bytes_p, hipStream_t s) {
    const int rw = row_bytes / 16, rwp = row_bytes_p / 16;
    const long total = BH * (long)Tp * rwp;
    hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_for(total)), dim3(256), 0, s, reinterpret_cast<const uint4*>(in),
                       reinterpret_cast<uint4*>(out), total, T, Tp, rw, rwp);
    return hipGetLastError();
}
hipError_t launch_unpad_rows(const void* in, void* out, long BH, int T, int Tp, int row_bytes, int row_bytes_p, hipStream_t s) {
    const int rw = row_bytes / 16, rwp = row_bytes_p / 16;
    const long total = BH * (long)T * rw;
    hipLaunchKernelGGL(unpad_rows_kernel, dim3(grid_for(total)), dim3(256), 0, s, reinterpret_cast<const uint4*>(in),
                       reinterpret_cast<uint4*>(out), total, T, Tp, rw, rwp);
    return hipGetLastError();
}
hipError_t launch_pad_scalar(const float* in, float* out, long BH, int T, int Tp, float fill, hipStream_t s) {
    const long total = BH * (long)Tp;
    hipLaunchKernelGGL(pad_scalar_kernel, dim3(grid_for(total)), dim3(256), 0, s, in, out, total, T, Tp, fill);
    return hipGetLastError();
}
hipError_t launch_unpad_scalar(const float* in, float* out, long BH, int T, int Tp, hipStream_t s) {
    const long total = BH * (long)T;
    hipLaunchKernelGGL(unpad_scalar_kernel, dim3(grid_for(total)), dim3(256), 0, s, in, out, total, T, Tp);
    return hipGetLastError();
}

}  // namespace tfla
