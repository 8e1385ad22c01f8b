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

namespace tfla {

template <typename DT, int MI, int NI, int BK>
__global__ void __launch_bounds__(256) recurrent_kernel(RecArgs a) {
    using E = Elem<DT>;
    constexpr int BM = 64 * MI, BN = 64 * NI, NT = 256;
    constexpr int LS = BK + E::PAD;
    __shared__ __attribute__((aligned(16))) DT ldsX[BM * LS];
    __shared__ __attribute__((aligned(16))) DT ldsY[BN * LS];
    __shared__ float ldsRs[BK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM, bh = blockIdx.z;
    const DT* X = reinterpret_cast<const DT*>(a.X) + (long)bh * a.T * a.d1 + m0;
    const DT* Y = reinterpret_cast<const DT*>(a.Y) + (long)bh * a.T * a.d2 + n0;
    const float* rs = a.rs + (long)bh * a.T;
    const bool with_n = (a.nst != nullptr) && blockIdx.x == 0;

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

    for (int step = 0; step < a.Nc; ++step) {
        const int kc = a.reverse ? a.Nc - 1 - step : step;
        // ---- emit the state before this chunk's update
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
                    DT* dst = reinterpret_cast<DT*>(a.stT) + slot * a.d1 * a.d2;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int m = m0 + wm * 32 * MI + 32 * mi + acc_row(v, g);
                        dst[(long)n * a.d1 + m] = E::from_f32(acc[mi][ni][v]);
                    }
                }
            }
        if (with_n && tid < BM) a.nst[slot * a.d1 + m0 + tid] = nacc;

        // ---- decay
        const float gb = a.gbar[(long)bh * a.Nc + kc];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mi][ni][v] *= gb;
        nacc *= gb;

        // ---- accumulate the chunk, BK rows at a time
        for (int r0 = 0; r0 < a.L; r0 += BK) {
            const long trow = (long)kc * a.L + r0;
            __syncthreads();
            if (tid < BK) ldsRs[tid] = rs[trow + tid];
            __syncthreads();
            stage_transposed<BK, BM, NT, false, true>(ldsX, LS, X + trow * a.d1, a.d1, ldsRs, tid);
            stage_transposed<BK, BN, NT, false, false>(ldsY, LS, Y + trow * a.d2, a.d2, nullptr, tid);
            __syncthreads();
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                typename E::frag af[MI], bf[NI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    af[mi] = E::load(ldsX + (wm * 32 * MI + 32 * mi + l32) * LS + 16 * ks + 8 * g);
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    bf[ni] = E::load(ldsY + (wn * 32 * NI + 32 * ni + l32) * LS + 16 * ks + 8 * g);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = E::mma(af[mi], bf[ni], acc[mi][ni]);
            }
            if (with_n && tid < BM) {
                // n += sum over the staged rows of (a-bar (.) K), from the same rounded values
                float sacc = 0.0f;
#pragma unroll
                for (int c = 0; c < BK; c += 8) {
                    const typename E::frag f = E::load(ldsX + tid * LS + c);
#pragma unroll
                    for (int e = 0; e < 8; ++e) sacc += E::frag_elem(f, e);
                }
                nacc += sacc;
            }
        }
    }
    // ---- final state
    if (a.Sfinal) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + wm * 32 * MI + 32 * mi + acc_row(v, g);
                    const int n = n0 + wn * 32 * NI + 32 * ni + l32;
                    a.Sfinal[((long)bh * a.d1 + m) * a.d2 + n] = acc[mi][ni][v];
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

hipError_t launch_recurrent(const RecArgs& a, int BH, int dtype, hipStream_t s) {
    // 128x128 state tiles when that still fills the chip, 64x64 tiles otherwise
    const bool big_ok = (a.d1 % 128 == 0) && (a.d2 % 128 == 0);
    const long wg_big = (long)BH * (a.d1 / 128) * (a.d2 / 128);
    const bool big = big_ok && wg_big >= 192;
    if (dtype == 1) return big ? launch_rec_t<bf16_t, 2, 2>(a, BH, s) : launch_rec_t<bf16_t, 1, 1>(a, BH, s);
    return big ? launch_rec_t<float, 2, 2>(a, BH, s) : launch_rec_t<float, 1, 1>(a, BH, s);
}

}  // namespace tfla
