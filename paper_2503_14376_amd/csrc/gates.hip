// Gate kernels: chunkwise log gates and max states (forward and backward preparation) and
// the final gate-gradient reduction.  All scalar-per-step work of the method lives here;
// it is VALU + wavefront-scan work on (B*NH*T) floats.
#include "tfla_device.h"
#include "tfla_internal.h"

namespace tfla {

static constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float log_sigmoid(float x) { return fminf(x, 0.0f) - log1pf(expf(-fabsf(x))); }
__device__ __forceinline__ float sigmoid_neg(float x) {  // sigma(-x), no overflow
    const float e = expf(-fabsf(x));
    return x >= 0.0f ? e / (1.0f + e) : 1.0f / (1.0f + e);
}

__device__ __forceinline__ float wave_excl_scan_add(float v, int lane) {
    float x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const float y = __shfl_up(x, o, 64); if (lane >= o) x += y; }
    const float p = __shfl_up(x, 1, 64);
    return lane == 0 ? 0.0f : p;
}
__device__ __forceinline__ float wave_excl_rscan_add(float v, int lane) {
    float x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const float y = __shfl_down(x, o, 64); if (lane + o < 64) x += y; }
    const float p = __shfl_down(x, 1, 64);
    return lane == 63 ? 0.0f : p;
}
__device__ __forceinline__ float wave_excl_scan_max(float v, int lane) {
    float x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const float y = __shfl_up(x, o, 64); if (lane >= o) x = fmaxf(x, y); }
    const float p = __shfl_up(x, 1, 64);
    return lane == 0 ? -INFINITY : p;
}

// One workgroup per (batch, head).  Phase 1: every wave takes chunks round-robin and forms,
// for chunk k: b = cumsum(f-bar), a = reverse cumsum shifted by one + i-bar (the stable form of
// App. B.2), the running maximum of (i-bar_j - b_j), g_k = sum f-bar and max_j a_j.
// Phase 2: one thread runs the scalar recurrence m_k = max(g_k + m_{k-1}, max_j a_kj).
// Phase 3: the per-step quantities the matrix kernels consume.
//
// The intra-chunk row maximum is separable: max_{j<=i}(b_i - b_j + i-bar_j) = b_i +
// cummax_j(i-bar_j - b_j), so the combined max state m_i = b_i + max(m_{k-1}, cummax_i) is known
// before any matrix product and no online rescaling is needed in the tiled kernel.
__global__ void __launch_bounds__(1024) gates_kernel(GateArgs a) {
    extern __shared__ float sm[];
    float* cg = sm;                 // [Nc]
    float* camax = sm + a.Nc;       // [Nc]
    float* cm = sm + 2 * a.Nc;      // [Nc + 1]
    const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int E = a.L / 64;
    const bool is_exp = a.variant == 0;
    const long row = (long)bh * a.T;
    float* tb = a.tmp + (long)bh * 3 * a.T;
    float* tc = tb + a.T;
    float* ta = tc + a.T;

    for (int kc = wave; kc < a.Nc; kc += nw) {
        const long t0 = (long)kc * a.L + (long)lane * E;
        float fsum = 0.0f;
        for (int e = 0; e < E; ++e) fsum += log_sigmoid(a.f_pre[row + t0 + e]);
        const float off = wave_excl_scan_add(fsum, lane);
        const float roff = wave_excl_rscan_add(fsum, lane);
        // forward pass: b, u = i-bar - b, running max of u
        float b = off, cmx = -INFINITY;
        for (int e = 0; e < E; ++e) {
            const float fb = log_sigmoid(a.f_pre[row + t0 + e]);
            const float ip = a.i_pre[row + t0 + e];
            const float ib = is_exp ? ip : log_sigmoid(ip);
            b += fb;
            const float u = ib - b;
            cmx = fmaxf(cmx, u);
            tb[t0 + e] = b;
            tc[t0 + e] = cmx;
            a.ucol[row + t0 + e] = u * LOG2E;
        }
        const float cmoff = wave_excl_scan_max(cmx, lane);
        for (int e = 0; e < E; ++e) tc[t0 + e] = fmaxf(tc[t0 + e], cmoff);
        // reverse pass: a_j = sum_{s>j} f-bar_s + i-bar_j
        float run = roff, amax = -INFINITY;
        for (int e = E - 1; e >= 0; --e) {
            const float ip = a.i_pre[row + t0 + e];
            const float ib = is_exp ? ip : log_sigmoid(ip);
            const float av = run + ib;
            ta[t0 + e] = av;
            amax = fmaxf(amax, av);
            run += log_sigmoid(a.f_pre[row + t0 + e]);
        }
        amax = wave_max(amax);
        const float g = wave_sum(fsum);
        if (lane == 0) { cg[kc] = g; camax[kc] = amax; }
    }
    __syncthreads();
    if (tid == 0) {
        float m = (is_exp && a.m0) ? a.m0[bh] : 0.0f;
        cm[0] = m;
        for (int kc = 0; kc < a.Nc; ++kc) {
            const float mn = is_exp ? fmaxf(cg[kc] + m, camax[kc]) : 0.0f;
            a.gbar[(long)bh * a.Nc + kc] = expf(cg[kc] + m - mn);
            m = mn;
            cm[kc + 1] = m;
        }
        if (a.mfinal) a.mfinal[bh] = m;
    }
    __syncthreads();
    const float lq = log2f(a.qscale);
    for (int kc = wave; kc < a.Nc; kc += nw) {
        const long t0 = (long)kc * a.L + (long)lane * E;
        const float mprev = cm[kc], mk = cm[kc + 1];
        for (int e = 0; e < E; ++e) {
            const float b = tb[t0 + e], cmx = tc[t0 + e], av = ta[t0 + e];
            float wr, sh, mo;
            if (is_exp) {
                const float M = fmaxf(mprev, cmx);
                wr = -M * LOG2E + lq;
                sh = expf(mprev - M) * a.qscale;
                mo = b + M;
            } else {
                wr = b * LOG2E + lq;
                sh = expf(b) * a.qscale;
                mo = 0.0f;
            }
            a.wrow[row + t0 + e] = wr;
            a.sH[row + t0 + e] = sh;
            a.aK[row + t0 + e] = expf(av - mk);
            a.mout[row + t0 + e] = mo;
        }
    }
}

hipError_t launch_gates(const GateArgs& a, int BH, hipStream_t s) {
    const size_t sh = sizeof(float) * (size_t)(3 * a.Nc + 1);
    const int nt = a.Nc >= 16 ? 1024 : (a.Nc >= 4 ? 256 : 64);
    hipLaunchKernelGGL(gates_kernel, dim3(BH), dim3(nt), sh, s, a);
    return hipGetLastError();
}

// Backward preparation: fold delta H~ = delta H / h_denom (App. B.3) into the weights.
__global__ void gate_bwd_prep_kernel(GateBwdPrepArgs a) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n) return;
    float den = 1.0f;
    if (a.variant == 0) den = fmaxf(fabsf(a.n_out[i]), expf(-a.m_out[i])) + a.eps;
    a.wrowB[i] = a.wrow[i] - log2f(den);
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
__global__ void __launch_bounds__(1024) gate_grads_kernel(GateGradArgs a) {
    __shared__ double wt[16];
    const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = (a.T + 1023) / 1024;
    const long row = (long)bh * a.T;
    const int t0 = tid * seg;
    double tot = 0.0;
    for (int e = 0; e < seg; ++e) {
        const int t = t0 + e;
        if (t < a.T) {
            float r = 0.0f, c = 0.0f;
            for (int nb = 0; nb < a.nbQ; ++nb) r += a.partQ[(long)nb * a.BHT + row + t];
            for (int nb = 0; nb < a.nbK; ++nb) c += a.partK[(long)nb * a.BHT + row + t];
            tot += (double)r - (double)c;
        }
    }
    double x = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const double y = __shfl_down(x, o, 64); if (lane + o < 64) x += y; }
    double excl = __shfl_down(x, 1, 64);
    if (lane == 63) excl = 0.0;
    if (lane == 0) wt[wave] = x;
    __syncthreads();
    for (int w = wave + 1; w < 16; ++w) excl += wt[w];
    double run = excl + (a.cdot ? (double)a.cdot[bh] : 0.0);
    for (int e = seg - 1; e >= 0; --e) {
        const int t = t0 + e;
        if (t < a.T) {
            float r = 0.0f, c = 0.0f;
            for (int nb = 0; nb < a.nbQ; ++nb) r += a.partQ[(long)nb * a.BHT + row + t];
            for (int nb = 0; nb < a.nbK; ++nb) c += a.partK[(long)nb * a.BHT + row + t];
            run += (double)r - (double)c;
            a.d_f[row + t] = (float)run * sigmoid_neg(a.f_pre[row + t]);
            a.d_i[row + t] = a.variant == 0 ? c : c * sigmoid_neg(a.i_pre[row + t]);
        }
    }
}
hipError_t launch_gate_grads(const GateGradArgs& a, int BH, hipStream_t s) {
    hipLaunchKernelGGL(gate_grads_kernel, dim3(BH), dim3(1024), 0, s, a);
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
