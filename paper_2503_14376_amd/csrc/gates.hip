// Gate kernels: chunkwise log gates and max states (forward and backward preparation) and
// the final gate-gradient reduction.  All scalar-per-step work of the method lives here;
// it is VALU + wavefront-scan work on (B*NH*T) floats.
#include "tfla_device.h"
#include "tfla_internal.h"

namespace tfla {

static constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float log_sigmoid(float x) { return fminf(x, 0.0f) - log1pf(expf(-fabsf(x))); }
// gate soft-cap c tanh(x / c) (App. E, soft-capping equation); c = 0 leaves x as it is
__device__ __forceinline__ float soft_cap(float x, float c) { return c > 0.0f ? c * tanhf(x / c) : x; }
__device__ __forceinline__ float soft_cap_grad(float x, float c) {
    if (!(c > 0.0f)) return 1.0f;
    const float t = tanhf(x / c);
    return 1.0f - t * t;
}
__device__ __forceinline__ float sigmoid_neg(float x) {  // sigma(-x), no overflow
    const float e = expf(-fabsf(x));
    return x >= 0.0f ? e / (1.0f + e) : 1.0f / (1.0f + e);
}

// The pre-pass is written over an arithmetic type AT.  float serves the bf16 kernels.  The fp32 kernels get the
// pre-pass in double (AT = double) and its two exponents as a (rounded, remainder) pair of floats each: the row and the
// column term of a weight both have the size of the chunk's cumulative log forget gate and nearly cancel, so a single
// float per term limits a weight to the fp32 spacing at that size (2.4e-4 at |sum f-bar| = 2560), while the sum of two
// such pairs is exact to fp32 again.
template <typename AT> __device__ __forceinline__ AT log_sigmoid_t(AT x);
template <> __device__ __forceinline__ float log_sigmoid_t<float>(float x) { return log_sigmoid(x); }
template <> __device__ __forceinline__ double log_sigmoid_t<double>(double x) { return fmin(x, 0.0) - log1p(exp(-fabs(x))); }
template <typename AT> __device__ __forceinline__ AT soft_cap_t(AT x, float c);
template <> __device__ __forceinline__ float soft_cap_t<float>(float x, float c) { return soft_cap(x, c); }
template <> __device__ __forceinline__ double soft_cap_t<double>(double x, float c) { return c > 0.0f ? (double)c * tanh(x / (double)c) : x; }
template <typename AT> __device__ __forceinline__ AT max_t(AT x, AT y);
template <> __device__ __forceinline__ float max_t<float>(float x, float y) { return fmaxf(x, y); }
template <> __device__ __forceinline__ double max_t<double>(double x, double y) { return fmax(x, y); }
template <typename AT> __device__ __forceinline__ AT exp_t(AT x);
template <> __device__ __forceinline__ float exp_t<float>(float x) { return expf(x); }
template <> __device__ __forceinline__ double exp_t<double>(double x) { return exp(x); }

template <typename AT> __device__ __forceinline__ AT wave_excl_scan_add(AT v, int lane) {
    AT x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const AT y = __shfl_up(x, o, 64); if (lane >= o) x += y; }
    const AT p = __shfl_up(x, 1, 64);
    return lane == 0 ? (AT)0 : p;
}
template <typename AT> __device__ __forceinline__ AT wave_excl_rscan_add(AT v, int lane) {
    AT x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const AT y = __shfl_down(x, o, 64); if (lane + o < 64) x += y; }
    const AT p = __shfl_down(x, 1, 64);
    return lane == 63 ? (AT)0 : p;
}
template <typename AT> __device__ __forceinline__ AT wave_excl_scan_max(AT v, int lane) {
    AT x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const AT y = __shfl_up(x, o, 64); if (lane >= o) x = max_t<AT>(x, y); }
    const AT p = __shfl_up(x, 1, 64);
    return lane == 0 ? (AT)-INFINITY : p;
}
template <typename AT> __device__ __forceinline__ AT wave_sum_t(AT x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
template <typename AT> __device__ __forceinline__ AT wave_max_t(AT x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = max_t<AT>(x, __shfl_xor(x, o, 64));
    return x;
}

// The gate pre-pass runs as two kernels, each with one wavefront per chunk (four chunks per
// workgroup), so that it fills the chip also when batch * heads is small.
//
// Kernel 1, for chunk k: b = cumsum(f-bar), a = reverse cumsum shifted by one + i-bar (the stable
// form of App. B.2), the running maximum of (i-bar_j - b_j), and the chunk summaries g_k = sum
// f-bar and max_j a_j.
// Kernel 2: every workgroup first runs the scalar recurrence m_k = max(g_k + m_{k-1}, max_j a_kj)
// over all chunks of its (batch, head) -- as a scan: the maps m -> max(m + g, c) compose to
// (g1 + g2, max(c1 + g2, c2)) -- and then forms the per-step quantities the matrix kernels
// consume for its own chunks.
//
// The intra-chunk row maximum is separable: max_{j<=i}(b_i - b_j + i-bar_j) = b_i +
// cummax_j(i-bar_j - b_j), so the combined max state m_i = b_i + max(m_{k-1}, cummax_i) is known
// before any matrix product and no online rescaling is needed in the tiled kernel.
static constexpr int GATE_WAVES = 4;

// EC > 0: the lane's E <= EC steps keep their log gates in registers (one evaluation of the logarithms per
// step instead of one per pass); EC = 0: any E, the log gates are evaluated again in every pass.
// tmp and csum hold values of type AT.
template <int EC, typename AT>
__global__ void __launch_bounds__(GATE_WAVES * 64) gates_chunk_kernel(GateArgs a) {
    const int bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kc = blockIdx.x * GATE_WAVES + wave;
    if (kc >= a.Nc) return;
    const int E = a.L / 64;
    const bool is_exp = a.variant == 0;
    const long row = (long)bh * a.T;
    AT* tb = reinterpret_cast<AT*>(a.tmp) + (long)bh * 3 * a.T;
    AT* tc = tb + a.T;
    AT* ta = tc + a.T;
    AT* csum = reinterpret_cast<AT*>(a.csum);
    const AT log2e = (AT)1.4426950408889634;
    const long t0 = (long)kc * a.L + (long)lane * E;
    // log gates of step t; the padding steps of a sequence that does not fill its last chunk keep the
    // state as it is (log forget gate 0) and add nothing (log input gate far below every other)
    auto fbar_at = [&](long t) { return t < a.Tvalid ? log_sigmoid_t<AT>(soft_cap_t<AT>((AT)a.f_pre[row + t], a.softcap)) : (AT)0; };
    auto ibar_at = [&](long t) {
        if (t >= a.Tvalid) return (AT)-1.0e30f;
        const AT ip = soft_cap_t<AT>((AT)a.i_pre[row + t], a.softcap);
        return is_exp ? ip : log_sigmoid_t<AT>(ip);
    };
    constexpr int NC = EC > 0 ? EC : 1;
    AT fbv[NC], ibv[NC];
    if constexpr (EC > 0) {
#pragma unroll
        for (int e = 0; e < EC; ++e) {
            fbv[e] = (AT)0; ibv[e] = (AT)0;
            if (e < E) { fbv[e] = fbar_at(t0 + e); ibv[e] = ibar_at(t0 + e); }
        }
    }
    auto fbar = [&](int e) { if constexpr (EC > 0) return fbv[e]; else return fbar_at(t0 + e); };
    auto ibar = [&](int e) { if constexpr (EC > 0) return ibv[e]; else return ibar_at(t0 + e); };
    const int EB = EC > 0 ? EC : E;                 // loop bound (compile-time when the gates are cached)
    AT fsum = (AT)0;
#pragma unroll
    for (int e = 0; e < EB; ++e)
        if (e < E) fsum += fbar(e);
    const AT off = wave_excl_scan_add<AT>(fsum, lane);
    const AT roff = wave_excl_rscan_add<AT>(fsum, lane);
    // forward pass: b, u = i-bar - b, running max of u
    AT b = off, cmx = (AT)-INFINITY;
#pragma unroll
    for (int e = 0; e < EB; ++e)
        if (e < E) {
            b += fbar(e);
            cmx = max_t<AT>(cmx, ibar(e) - b);
        }
    const AT cmoff = wave_excl_scan_max<AT>(cmx, lane);
    b = off; cmx = cmoff;
#pragma unroll
    for (int e = 0; e < EB; ++e)
        if (e < E) {
            b += fbar(e);
            const AT u = ibar(e) - b;
            cmx = max_t<AT>(cmx, u);
            tb[t0 + e] = b;
            tc[t0 + e] = cmx;
            const AT ul = u * log2e;
            const float uh = (float)ul;
            a.ucol[row + t0 + e] = uh;
            if (a.ucol_lo) a.ucol_lo[row + t0 + e] = (float)(ul - (AT)uh);
        }
    // reverse pass: a_j = sum_{s>j} f-bar_s + i-bar_j
    AT run = roff, amax = (AT)-INFINITY;
#pragma unroll
    for (int e = EB - 1; e >= 0; --e)
        if (e < E) {
            const AT av = run + ibar(e);
            ta[t0 + e] = av;
            amax = max_t<AT>(amax, av);
            run += fbar(e);
        }
    amax = wave_max_t<AT>(amax);
    const AT gsum = wave_sum_t<AT>(fsum);
    if (lane == 0) {
        csum[((long)bh * 2 + 0) * a.Nc + kc] = gsum;
        csum[((long)bh * 2 + 1) * a.Nc + kc] = amax;
    }
}

template <typename AT>
__global__ void __launch_bounds__(GATE_WAVES * 64) gates_step_kernel(GateArgs a) {
    extern __shared__ double cm_raw[];   // [Nc + 1] values of type AT: m before chunk k
    AT* cm = reinterpret_cast<AT*>(cm_raw);
    const int bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool is_exp = a.variant == 0;
    const AT* cg = reinterpret_cast<const AT*>(a.csum) + ((long)bh * 2 + 0) * a.Nc;
    const AT* camax = reinterpret_cast<const AT*>(a.csum) + ((long)bh * 2 + 1) * a.Nc;
    if (wave == 0) {
        // lane l composes the maps of its segment of chunks, a wavefront scan composes the segments,
        // then every lane walks its segment again from its incoming m
        const int seg = (a.Nc + 63) / 64;
        const int k0 = lane * seg, k1 = min(a.Nc, k0 + seg);
        AT G = (AT)0, C = (AT)-INFINITY;
        for (int k = k0; k < k1; ++k) { C = max_t<AT>(C + cg[k], camax[k]); G += cg[k]; }
        // inclusive scan of the composed maps over the lanes
        AT Gs = G, Cs = C;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const AT Gp = __shfl_up(Gs, o, 64), Cp = __shfl_up(Cs, o, 64);
            if (lane >= o) { Cs = max_t<AT>(Cp + Gs, Cs); Gs = Gp + Gs; }
        }
        // exclusive: the map of all chunks before this lane's segment, applied to m0
        const AT Ge = __shfl_up(Gs, 1, 64), Ce = __shfl_up(Cs, 1, 64);
        const AT m_init = (is_exp && a.m0) ? (AT)a.m0[bh] : (AT)0;
        AT m = lane == 0 ? m_init : max_t<AT>(m_init + Ge, Ce);
        if (!is_exp) m = (AT)0;
        for (int k = k0; k < k1; ++k) {
            cm[k] = m;
            const AT mn = is_exp ? max_t<AT>(cg[k] + m, camax[k]) : (AT)0;
            if (blockIdx.x == 0) a.gbar[(long)bh * a.Nc + k] = (float)exp_t<AT>(cg[k] + m - mn);
            m = mn;
        }
        if (k1 == a.Nc && k0 < k1) {
            cm[a.Nc] = m;
            if (blockIdx.x == 0 && a.mfinal) a.mfinal[bh] = (float)m;
        }
    }
    __syncthreads();
    const int kc = blockIdx.x * GATE_WAVES + wave;
    if (kc >= a.Nc) return;
    const int E = a.L / 64;
    const long row = (long)bh * a.T;
    const AT* tb = reinterpret_cast<const AT*>(a.tmp) + (long)bh * 3 * a.T;
    const AT* tc = tb + a.T;
    const AT* ta = tc + a.T;
    const AT log2e = (AT)1.4426950408889634;
    const AT lq = (AT)log2f(a.qscale);
    const long t0 = (long)kc * a.L + (long)lane * E;
    const AT mprev = cm[kc], mk = cm[kc + 1];
    for (int e = 0; e < E; ++e) {
        const AT b = tb[t0 + e], cmx = tc[t0 + e], av = ta[t0 + e];
        AT wr, sh, mo;
        if (is_exp) {
            const AT M = max_t<AT>(mprev, cmx);
            wr = -M * log2e + lq;
            sh = exp_t<AT>(mprev - M) * (AT)a.qscale;
            mo = b + M;
        } else {
            wr = b * log2e + lq;
            sh = exp_t<AT>(b) * (AT)a.qscale;
            mo = (AT)0;
        }
        const float wh = (float)wr;
        a.wrow[row + t0 + e] = wh;
        if (a.wrow_lo) a.wrow_lo[row + t0 + e] = (float)(wr - (AT)wh);
        a.sH[row + t0 + e] = (float)sh;
        a.aK[row + t0 + e] = (float)exp_t<AT>(av - mk);
        a.mout[row + t0 + e] = (float)mo;
    }
}

template <typename AT> static hipError_t launch_gates_t(const GateArgs& a, int BH, hipStream_t s) {
    const dim3 grid((a.Nc + GATE_WAVES - 1) / GATE_WAVES, BH);
    // the log gates of a lane's steps stay in registers for every chunk size the library accepts (L <= 2048)
    if (a.L / 64 <= 8) hipLaunchKernelGGL((gates_chunk_kernel<8, AT>), grid, dim3(GATE_WAVES * 64), 0, s, a);
    else if (a.L / 64 <= 16) hipLaunchKernelGGL((gates_chunk_kernel<16, AT>), grid, dim3(GATE_WAVES * 64), 0, s, a);
    else if (a.L / 64 <= 32) hipLaunchKernelGGL((gates_chunk_kernel<32, AT>), grid, dim3(GATE_WAVES * 64), 0, s, a);
    else hipLaunchKernelGGL((gates_chunk_kernel<0, AT>), grid, dim3(GATE_WAVES * 64), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gates_step_kernel<AT>, grid, dim3(GATE_WAVES * 64), sizeof(AT) * (size_t)(a.Nc + 1), s, a);
    return hipGetLastError();
}

// a.precise: the fp32 kernels' pre-pass (double arithmetic, two-float exponents; tmp and csum then hold doubles)
hipError_t launch_gates(const GateArgs& a, int BH, hipStream_t s) {
    return a.precise ? launch_gates_t<double>(a, BH, s) : launch_gates_t<float>(a, BH, s);
}

// Backward preparation: fold delta H~ = delta H / h_denom (App. B.3) into the weights.
__global__ void gate_bwd_prep_kernel(GateBwdPrepArgs a) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n) return;
    float den = 1.0f;
    if (a.variant == 0) den = fmaxf(fabsf(a.n_out[i]), expf(-a.m_out[i])) + a.eps;
    if (a.wrowB_lo) {
        // fp32 kernels: the difference to double accuracy, as a (rounded, remainder) pair
        const double w = (double)a.wrow[i] + (double)a.wrow_lo[i] - log2((double)den);
        const float wh = (float)w;
        a.wrowB[i] = wh;
        a.wrowB_lo[i] = (float)(w - (double)wh);
    } else {
        a.wrowB[i] = a.wrow[i] - log2f(den);
    }
    a.sQ[i] = a.sH[i] / den;
}
hipError_t launch_gate_bwd_prep(const GateBwdPrepArgs& a, hipStream_t s) {
    const int nt = 256;
    hipLaunchKernelGGL(gate_bwd_prep_kernel, dim3((unsigned)((a.n + nt - 1) / nt)), dim3(nt), 0, s, a);
    return hipGetLastError();
}

// Gate gradients.  q_t . dq_t and k_t . dk_t are the row and column sums of the gradient
// w.r.t. the log weights (each log weight is linear in the f-bar_s it spans and in i-bar_j), so
//   d i-bar_j = k_j . dk_j ,   d f-bar_s = sum_{t>=s} (q_t . dq_t - k_t . dk_t) + <C_T, dC_T>.
// This regroups the cumulative-gate gradients of App. B.3 (delta g, delta a, delta b and the
// row/column sums of the intra-chunk gate-matrix gradient) into one reverse cumulative sum.
// Two kernels over blocks of GG_BLOCK steps: block sums first, then every block adds the sums of
// the blocks after it and scans its own steps (in fp64: the terms cancel heavily).
static constexpr int GG_BLOCK = 1024;

__device__ __forceinline__ void gate_grad_terms(const GateGradArgs& a, long idx, float& r, float& c) {
    r = 0.0f; c = 0.0f;
    for (int nb = 0; nb < a.nbQ; ++nb) r += a.partQ[(long)nb * a.BHT + idx];
    for (int nb = 0; nb < a.nbK; ++nb) c += a.partK[(long)nb * a.BHT + idx];
}

__global__ void __launch_bounds__(256) gate_grads_sum_kernel(GateGradArgs a) {
    __shared__ double wt[4];
    const int bh = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    const long row = (long)bh * a.T;
    double tot = 0.0;
    for (int e = 0; e < GG_BLOCK / 256; ++e) {
        const int t = blk * GG_BLOCK + e * 256 + tid;
        if (t < a.T) {
            float r, c;
            gate_grad_terms(a, row + t, r, c);
            tot += (double)r - (double)c;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) tot += __shfl_xor(tot, o, 64);
    if ((tid & 63) == 0) wt[tid >> 6] = tot;
    __syncthreads();
    if (tid == 0) a.bsum[(long)bh * gridDim.x + blk] = wt[0] + wt[1] + wt[2] + wt[3];
}

__global__ void __launch_bounds__(256) gate_grads_kernel(GateGradArgs a) {
    __shared__ double wt[4];
    __shared__ double after;
    const int bh = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nblk = gridDim.x;
    const long row = (long)bh * a.T;
    // sum of the blocks after this one
    double later = 0.0;
    for (int b2 = blk + 1 + tid; b2 < nblk; b2 += 256) later += a.bsum[(long)bh * nblk + b2];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) later += __shfl_xor(later, o, 64);
    if (lane == 0) wt[wave] = later;
    __syncthreads();
    if (tid == 0) after = wt[0] + wt[1] + wt[2] + wt[3] + (a.cdot ? (double)a.cdot[bh] : 0.0);
    __syncthreads();
    // thread tid owns GG_BLOCK / 256 consecutive steps
    constexpr int SEG = GG_BLOCK / 256;
    const int t0 = blk * GG_BLOCK + tid * SEG;
    float r[SEG], c[SEG];
    double tot = 0.0;
#pragma unroll
    for (int e = 0; e < SEG; ++e) {
        r[e] = 0.0f; c[e] = 0.0f;
        if (t0 + e < a.T) gate_grad_terms(a, row + t0 + e, r[e], c[e]);
        tot += (double)r[e] - (double)c[e];
    }
    double x = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const double y = __shfl_down(x, o, 64); if (lane + o < 64) x += y; }
    double excl = __shfl_down(x, 1, 64);
    if (lane == 63) excl = 0.0;
    __syncthreads();
    if (lane == 0) wt[wave] = x;
    __syncthreads();
    for (int w = wave + 1; w < 4; ++w) excl += wt[w];
    double run = excl + after;
#pragma unroll
    for (int e = SEG - 1; e >= 0; --e) {
        const int t = t0 + e;
        if (t < a.T) {
            run += (double)r[e] - (double)c[e];
            const float fp = a.f_pre[row + t], ip = a.i_pre[row + t];
            a.d_f[row + t] = (float)run * sigmoid_neg(soft_cap(fp, a.softcap)) * soft_cap_grad(fp, a.softcap);
            a.d_i[row + t] = (a.variant == 0 ? c[e] : c[e] * sigmoid_neg(soft_cap(ip, a.softcap))) * soft_cap_grad(ip, a.softcap);
        }
    }
}
// The same with anchors.  The value of the reverse cumulative sum at a chunk boundary is known exactly:
// the log forget gate of the first step of chunk k + 1 scales the boundary state C_{k+1} in every later
// use, so d f-bar there is <C_{k+1}, dC_{k+1}>, which needs no summation over time.  Every block of G chunks
// then scans its own steps only, from the anchor at its end, and the rounding noise of the terms no longer
// accumulates over the whole sequence (it grows with sqrt(T) in the unanchored scan).  One workgroup per
// block (at most 2048 steps); a thread owns up to eight consecutive steps.
__global__ void __launch_bounds__(256) gate_grads_anchored_kernel(GateGradArgs a) {
    __shared__ double wt[4];
    const int bh = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long row = (long)bh * a.T;
    const int kc0 = blk * a.G, kc1 = min(kc0 + a.G, a.Nc);      // chunks [kc0, kc1)
    const long tb = (long)kc0 * a.L;                            // first step of the block
    const int len = (kc1 - kc0) * a.L;                          // steps in this block
    const int SEG = (a.G * a.L + 255) / 256;           // <= 8: G * L <= 2048
    const int l0 = tid * SEG;                          // first of this thread's steps within the block
    float r[8], c[8];
    double tot = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        r[e] = 0.0f; c[e] = 0.0f;
        if (e < SEG && l0 + e < len) gate_grad_terms(a, row + tb + l0 + e, r[e], c[e]);
        tot += (double)r[e] - (double)c[e];
    }
    double x = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const double y = __shfl_down(x, o, 64); if (lane + o < 64) x += y; }
    double excl = __shfl_down(x, 1, 64);
    if (lane == 63) excl = 0.0;
    if (lane == 0) wt[wave] = x;
    __syncthreads();
    for (int w = wave + 1; w < 4; ++w) excl += wt[w];
    // the anchor at the end of the block: <C_T, dC_T> (or nothing) at the end of the sequence, else <C, dC> at the
    // boundary after the block, which the reversed recurrent launch left as npart partial sums
    __shared__ double wa[4];
    double anc = 0.0;
    if (kc1 == a.Nc) {
        anc = a.cdot ? (double)a.cdot[bh] : 0.0;
    } else {
        const int nslot = (a.Nc + a.G - 1) / a.G;
        const float* pp = a.anchor + ((long)bh * nslot + kc1 / a.G) * a.npart;
        double ps = 0.0;
        for (int q = tid; q < a.npart; q += 256) ps += (double)pp[q];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o, 64);
        if (lane == 0) wa[wave] = ps;
        __syncthreads();
        anc = (wa[0] + wa[1]) + (wa[2] + wa[3]);
    }
    double run = excl + anc;
#pragma unroll
    for (int e = 7; e >= 0; --e) {
        if (e < SEG && l0 + e < len) {
            const long t = tb + l0 + e;
            run += (double)r[e] - (double)c[e];
            const float fp = a.f_pre[row + t], ip = a.i_pre[row + t];
            a.d_f[row + t] = (float)run * sigmoid_neg(soft_cap(fp, a.softcap)) * soft_cap_grad(fp, a.softcap);
            a.d_i[row + t] = (a.variant == 0 ? c[e] : c[e] * sigmoid_neg(soft_cap(ip, a.softcap))) * soft_cap_grad(ip, a.softcap);
        }
    }
}

hipError_t launch_gate_grads(const GateGradArgs& a, int BH, hipStream_t s) {
    if (a.anchor) {
        if (a.G < 1 || (long)a.G * a.L > 2048) return hipErrorInvalidValue;
        hipLaunchKernelGGL(gate_grads_anchored_kernel, dim3((a.Nc + a.G - 1) / a.G, BH), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    const dim3 grid((a.T + GG_BLOCK - 1) / GG_BLOCK, BH);
    hipLaunchKernelGGL(gate_grads_sum_kernel, grid, dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gate_grads_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

__global__ void fill_zero_kernel(float* p, long n) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}
hipError_t launch_fill_zero(float* p, long n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

// up to four arrays in one launch: element i of the concatenation belongs to the first array whose end lies beyond i
__global__ void __launch_bounds__(256) fill_zero4_kernel(FillList f) {
    long i = (long)blockIdx.x * 256 + threadIdx.x;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (i < f.n[q]) { f.p[q][i] = 0.0f; return; }
        i -= f.n[q];
    }
}
hipError_t launch_fill_zero4(const FillList& f, hipStream_t s) {
    long total = 0;
    for (int q = 0; q < 4; ++q) {
        if (f.n[q] < 0 || (f.n[q] > 0 && !f.p[q])) return hipErrorInvalidValue;
        total += f.n[q];
    }
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, f);
    return hipGetLastError();
}

// out[bh] = <A[bh], B[bh]> over `per` floats
__global__ void __launch_bounds__(1024) state_dot_kernel(const float* A, const float* Bm, float* out, long per) {
    __shared__ double wt[16];
    const int bh = blockIdx.x, tid = threadIdx.x;
    double acc = 0.0;
    for (long i = tid; i < per; i += 1024) acc += (double)A[bh * per + i] * (double)Bm[bh * per + i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((tid & 63) == 0) wt[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        double t = 0.0;
        for (int w = 0; w < 16; ++w) t += wt[w];
        out[bh] = (float)t;
    }
}
hipError_t launch_state_dot(const float* A, const float* Bm, float* out, long per, int BH, hipStream_t s) {
    hipLaunchKernelGGL(state_dot_kernel, dim3(BH), dim3(1024), 0, s, A, Bm, out, per);
    return hipGetLastError();
}

}  // namespace tfla
