// Inter-chunk recurrent kernel (paper Sec. 3 "recurrent kernel"; App. B.2 inter-chunk
// recurrence; App. B.3 recurrence of delta C).  Sequential over chunks, parallel over
// (batch*head) and over BM x BN tiles of the d1 x d2 state.
//
//   state <- gbar_k * state + (rs (.) X_k)^T Y_k
//
// Forward:  X = K, Y = V, rs = a-bar, state = C;  backward: X = Q, Y = delta H,
// rs = b-bar * qscale / h_denom, state = delta C, chunks visited last to first.  The state
// before each update is written (in the element type of X/Y) to slot k in one or both of the
// layouts the tiled kernels read: stT[k] = state^T (d2 x d1) and stN[k] = state (d1 x d2).
#include "tfla_device.h"
#include "tfla_internal.h"
#include "recurrent_fast.h"

namespace tfla {

// Generic kernel (any element type, operands staged transposed through registers); bf16 uses
// recurrent_kernel_bf16 (recurrent_fast.h), this one serves fp32.

template <typename DT, int MI, int NI, int BK>
__global__ void __launch_bounds__(256) recurrent_kernel(RecArgs a) {
    using E = Elem<DT>;
    constexpr int BM = 64 * MI, BN = 64 * NI, NT = 256;
    constexpr int LS = BK + E::PAD;
    constexpr int D = 4;   // pieces (BK rows of X and Y) in flight from global memory
    __shared__ __attribute__((aligned(16))) DT ldsX[2][BM * LS];
    __shared__ __attribute__((aligned(16))) DT ldsY[2][BN * LS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    // XCD-aware decomposition: all state tiles of one (batch, head) share K/V and sit on one XCD
    const unsigned nwg = gridDim.x * gridDim.y * gridDim.z;
    unsigned wg = xcd_remap(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), nwg);
    const int bx = wg % gridDim.x; wg /= gridDim.x;
    const int by = wg % gridDim.y; const int bh = wg / gridDim.y;
    const int n0 = bx * BN, m0 = by * BM;
    const DT* X = reinterpret_cast<const DT*>(a.X) + (long)bh * a.T * a.d1 + m0;
    const DT* Y = reinterpret_cast<const DT*>(a.Y) + (long)bh * a.T * a.d2 + n0;
    const float* rs = a.rs + (long)bh * a.T;
    const bool with_n = (a.nst != nullptr) && bx == 0;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 32 * MI + 32 * mi + acc_row(v, g);
                const int n = n0 + wn * 32 * NI + 32 * ni + l32;
                acc[mi][ni][v] = a.S0 ? a.S0[((long)bh * a.d1 + m) * a.d2 + n] : 0.0f;
            }
        }
    float nacc = 0.0f;
    if (with_n && tid < BM && a.n0) nacc = a.n0[(long)bh * a.d1 + m0 + tid];

    // The sequence is consumed as P pieces of BK rows; piece i belongs to chunk step i / PPC.
    const int PPC = a.L / BK, P = a.Nc * PPC;
    auto piece_row = [&](int i) -> long {
        const int stepc = i / PPC;
        const int kc = a.reverse ? a.Nc - 1 - stepc : stepc;
        return (long)kc * a.L + (long)(i % PPC) * BK;
    };
    using PX = TrPrefetch<DT, BK, BM, NT, false>;
    using PY = TrPrefetch<DT, BK, BN, NT, false>;
    PX px[D];
    PY py[D];
    float prs[D][PX::N][8];
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < P) {
            const long tr = piece_row(d);
            px[d].load(X + tr * a.d1, a.d1, tid);
            py[d].load(Y + tr * a.d2, a.d2, tid);
            px[d].load_scales(prs[d], rs + tr, tid);
        }
    px[0].store_scaled(ldsX[0], LS, prs[0], tid);
    py[0].template store<false>(ldsY[0], LS, nullptr, tid);
    if (D < P) {
        const long tr = piece_row(D);
        px[0].load(X + tr * a.d1, a.d1, tid);
        py[0].load(Y + tr * a.d2, a.d2, tid);
        px[0].load_scales(prs[0], rs + tr, tid);
    }
    __syncthreads();

    for (int i0 = 0; i0 < P; i0 += D) {
#pragma unroll
        for (int dd = 0; dd < D; ++dd) {
            const int i = i0 + dd;
            if (i < P) {
                const int r = (dd + 1) % D;   // ring slot that holds piece i+1
                // ---- stage piece i+1 into the other LDS buffer, refill its ring slot
                if (i + 1 < P) {
                    px[r].store_scaled(ldsX[(i + 1) & 1], LS, prs[r], tid);
                    py[r].template store<false>(ldsY[(i + 1) & 1], LS, nullptr, tid);
                    if (i + 1 + D < P) {
                        const long tr = piece_row(i + 1 + D);
                        px[r].load(X + tr * a.d1, a.d1, tid);
                        py[r].load(Y + tr * a.d2, a.d2, tid);
                        px[r].load_scales(prs[r], rs + tr, tid);
                    }
                }
                // ---- chunk boundary: emit the state before this chunk's update, then decay
                if (i % PPC == 0) {
                    const int stepc = i / PPC;
                    const int kc = a.reverse ? a.Nc - 1 - stepc : stepc;
                    const long slot = (long)bh * a.Nc + kc;
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) {
                            const int n = n0 + wn * 32 * NI + 32 * ni + l32;
                            if (a.stN) {
                                DT* dst = reinterpret_cast<DT*>(a.stN) + slot * a.d1 * a.d2;
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const int m = m0 + wm * 32 * MI + 32 * mi + acc_row(v, g);
                                    dst[(long)m * a.d2 + n] = E::from_f32(acc[mi][ni][v]);
                                }
                            }
                            if (a.stT) {
                                // registers 4j..4j+3 hold four consecutive m: one packed store each
                                DT* dst = reinterpret_cast<DT*>(a.stT) + slot * a.d1 * a.d2;
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const int m = m0 + wm * 32 * MI + 32 * mi + acc_row(4 * j, g);
                                    store4(dst + (long)n * a.d1 + m, acc[mi][ni][4 * j], acc[mi][ni][4 * j + 1],
                                           acc[mi][ni][4 * j + 2], acc[mi][ni][4 * j + 3]);
                                }
                            }
                        }
                    if (with_n && tid < BM) a.nst[slot * a.d1 + m0 + tid] = nacc;
                    const float gb = a.gbar[(long)bh * a.Nc + kc];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[mi][ni][v] *= gb;
                    nacc *= gb;
                }
                // ---- multiply piece i
                const DT* xb = ldsX[i & 1];
                const DT* yb = ldsY[i & 1];
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    typename E::frag af[MI], bf[NI];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        af[mi] = E::load(xb + (wm * 32 * MI + 32 * mi + l32) * LS + 16 * ks + 8 * g);
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
                        bf[ni] = E::load(yb + (wn * 32 * NI + 32 * ni + l32) * LS + 16 * ks + 8 * g);
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = E::mma(af[mi], bf[ni], acc[mi][ni]);
                }
                if (with_n && tid < BM) {
                    // n += column sums of the staged (a-bar (.) K) piece, from the same rounded values
                    float sacc = 0.0f;
#pragma unroll
                    for (int c = 0; c < BK; c += 8) {
                        const typename E::frag f = E::load(xb + tid * LS + c);
#pragma unroll
                        for (int e = 0; e < 8; ++e) sacc += E::frag_elem(f, e);
                    }
                    nacc += sacc;
                }
                __syncthreads();
            }
        }
    }
    // ---- final state
    if (a.Sfinal || a.Sfinal2) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * 32 * MI + 32 * mi + acc_row(v, g);
                    const int n = n0 + wn * 32 * NI + 32 * ni + l32;
                    {
                    const long o = ((long)bh * a.d1 + m) * a.d2 + n;
                    if (a.Sfinal) a.Sfinal[o] = acc[mi][ni][v];
                    if (a.Sfinal2) a.Sfinal2[o] = acc[mi][ni][v];
                }
                }
    }
    if (with_n && tid < BM && a.nfinal) a.nfinal[(long)bh * a.d1 + m0 + tid] = nacc;
}

template <typename DT, int MI, int NI>
static hipError_t launch_rec_t(const RecArgs& a, int BH, hipStream_t s) {
    constexpr int BK = sizeof(DT) == 2 ? 64 : 32;
    dim3 grid(a.d2 / (64 * NI), a.d1 / (64 * MI), BH);
    hipLaunchKernelGGL((recurrent_kernel<DT, MI, NI, BK>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

template <int WN>
static hipError_t launch_rec_bf16(const RecArgs& a, int BH, hipStream_t s) {
    dim3 grid(a.d2 / (WN * 32), a.d1 / 64, BH);
    // pieces of 128 rows (half as many workgroup barriers) whenever the chunk size allows
    if (a.L % 128 == 0) hipLaunchKernelGGL((recurrent_kernel_bf16<WN, 128>), grid, dim3(WN * 128), 0, s, a);
    else hipLaunchKernelGGL((recurrent_kernel_bf16<WN, 64>), grid, dim3(WN * 128), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_recurrent(const RecArgs& a, int BH, int dtype, hipStream_t s) {
    if (dtype == 1) {
        // the bf16 kernel writes the chunk states as (d2, d1) only
        if (a.stN) return hipErrorInvalidValue;
        return a.d2 % 128 == 0 ? launch_rec_bf16<4>(a, BH, s) : launch_rec_bf16<2>(a, BH, s);
    }
    // fp32: 128x128 state tiles when that still fills the chip, 64x64 tiles otherwise
    const bool big_ok = (a.d1 % 128 == 0) && (a.d2 % 128 == 0);
    const long wg_big = (long)BH * (a.d1 / 128) * (a.d2 / 128);
    const bool big = big_ok && wg_big >= 192;
    return big ? launch_rec_t<float, 2, 2>(a, BH, s) : launch_rec_t<float, 1, 1>(a, BH, s);
}

}  // namespace tfla

#ifdef TFLA_TIMELINE
extern "C" __attribute__((visibility("default"))) int tfla_debug_rec_timeline(unsigned long long* host, size_t n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(tfla::tfla_rec_timeline), n * sizeof(unsigned long long));
}
#endif
