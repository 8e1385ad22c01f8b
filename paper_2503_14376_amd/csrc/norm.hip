// What surrounds the cell in an mLSTM layer (paper Sec. 2.1, hidden-state output equation
// h = sigma(o~) (.) NORM(h~); RMS norm as written out in Sec. 4.1, LayerNorm as its alternative),
// its exact backward, and the gains of the transfer-behaviour experiment (Sec. 4.1, gain
// equation; App. D.2).  All of it is row-wise work over d_hv values per (batch, head, step):
// one wavefront per row, a row kept in registers between its one load and its one store.
#include "tfla_device.h"
#include "tfla_internal.h"

namespace tfla {

namespace {

constexpr int NORM_RPB = 128;   // rows per workgroup of the backward kernel (32 per wavefront)

// eight consecutive elements of a row as floats
template <typename DT> struct Row8;
template <> struct Row8<bf16_t> {
    static __device__ __forceinline__ void load(const void* base, long idx, float (&x)[8]) {
        // every row is read once per launch: non-temporal, so that the stream does not displace other data from the caches
        const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const bf16_t*>(base) + idx));
#pragma unroll
        for (int e = 0; e < 4; ++e) { x[2 * e] = bf16_lo_to_f32(w[e]); x[2 * e + 1] = bf16_hi_to_f32(w[e]); }
    }
    static __device__ __forceinline__ void store(void* base, long idx, const float (&x)[8]) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(x[2 * e], x[2 * e + 1]);
        *reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(base) + idx) = w;
    }
    // for results that the next kernels do not read
    static __device__ __forceinline__ void store_stream(void* base, long idx, const float (&x)[8]) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(x[2 * e], x[2 * e + 1]);
        __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(base) + idx));
    }
};
template <> struct Row8<float> {
    static __device__ __forceinline__ void load(const void* base, long idx, float (&x)[8]) {
        const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + idx);
        const float4 a = p[0], b = p[1];
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
    static __device__ __forceinline__ void store(void* base, long idx, const float (&x)[8]) {
        float4* p = reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + idx);
        p[0] = make_float4(x[0], x[1], x[2], x[3]);
        p[1] = make_float4(x[4], x[5], x[6], x[7]);
    }
    static __device__ __forceinline__ void store_stream(void* base, long idx, const float (&x)[8]) { store(base, idx, x); }
};

__device__ __forceinline__ void load8f(const float* p, float (&x)[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

__device__ __forceinline__ float sigmoidf_(float x) {
    const float e = expf(-fabsf(x));
    return x >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
}

// A row of d values spread over a wavefront: lane l holds the 8-element groups l, l + 64, ...
// (J groups at most).  center() turns x into x - mean (LayerNorm; mean is 0 for the RMS norm)
// and returns 1 / sqrt(mean((x - mean)^2) + eps).
template <typename DT, int J> struct RowRegs {
    float x[J][8];
    __device__ __forceinline__ void load(const void* base, long row, int d, int lane) {
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int c = (lane + 64 * j) * 8;
            if (c < d) Row8<DT>::load(base, row * d + c, x[j]);
            else {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[j][e] = 0.0f;
            }
        }
    }
    __device__ __forceinline__ float center(int d, int lane, int kind, float eps) {
        if (kind == 1) {
            float s = 0.0f;
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) s += x[j][e];
            const float mu = wave_sum(s) / (float)d;
#pragma unroll
            for (int j = 0; j < J; ++j)
                if ((lane + 64 * j) * 8 < d) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[j][e] -= mu;
                }
        }
        float ss = 0.0f;
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += x[j][e] * x[j][e];
        return 1.0f / sqrtf(wave_sum(ss) / (float)d + eps);
    }
};

template <typename DT, int J>
__global__ void __launch_bounds__(256) norm_gate_fwd_kernel(NormArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long row = (long)blockIdx.x * 4 + wave;
    if (row >= a.rows) return;
    const int d = a.d;
    const int head = (int)((row / a.T) % a.NH);
    RowRegs<DT, J> r;
    r.load(a.h, row, d, lane);
    const float rstd = r.center(d, lane, a.kind, a.eps);
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int c = (lane + 64 * j) * 8;
        if (c >= d) continue;
        float g[8], be[8], o[8], y[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { g[e] = 1.0f; be[e] = 0.0f; o[e] = 0.0f; }
        if (a.gamma) load8f(a.gamma + (long)head * d + c, g);
        if (a.beta && a.kind == 1) load8f(a.beta + (long)head * d + c, be);
        if (a.o_pre) Row8<DT>::load(a.o_pre, row * d + c, o);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float n = r.x[j][e] * rstd * g[e] + be[e];
            y[e] = a.o_pre ? n * sigmoidf_(o[e]) : n;
        }
        Row8<DT>::store_stream(a.y, row * d + c, y);
    }
}

// Backward of h = sigma(o~) (.) (gamma (.) x^ + beta), x^ = (h~ - mean) * rstd:
//   d o~ = dy (.) n (.) o (1 - o),  dn = dy (.) o,  dx^ = dn (.) gamma,
//   d h~ = rstd (dx^ - mean(dx^) [LayerNorm only] - x^ mean(dx^ (.) x^)),
//   d gamma = sum over rows of dn (.) x^,  d beta = sum over rows of dn.
// A workgroup takes NORM_RPB consecutive steps of one (batch, head) and leaves its partial
// parameter sums in `part` (reduced in a fixed order by norm_param_grad_kernel).
template <typename DT, int J>
__global__ void __launch_bounds__(256) norm_gate_bwd_kernel(NormBwdArgs a) {
    __shared__ float red[4][2][J * 512];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bh = blockIdx.y, blk = blockIdx.x, d = a.d;
    const int head = bh % a.NH;
    float ag[J][8], ab[J][8], g[J][8], be[J][8];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int c = (lane + 64 * j) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) { ag[j][e] = 0.0f; ab[j][e] = 0.0f; g[j][e] = 1.0f; be[j][e] = 0.0f; }
        if (c < d) {
            if (a.gamma) load8f(a.gamma + (long)head * d + c, g[j]);
            if (a.beta && a.kind == 1) load8f(a.beta + (long)head * d + c, be[j]);
        }
    }
    const int t_end = min(a.T, (blk + 1) * NORM_RPB);
    for (int t = blk * NORM_RPB + wave; t < t_end; t += 4) {
        const long row = (long)bh * a.T + t;
        RowRegs<DT, J> r;
        r.load(a.h, row, d, lane);
        const float rstd = r.center(d, lane, a.kind, a.eps);
        float dx[J][8];
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int c = (lane + 64 * j) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) dx[j][e] = 0.0f;
            if (c >= d) continue;
            float dy[8], o[8], dop[8];
            Row8<DT>::load(a.dy, row * d + c, dy);
            if (a.o_pre) Row8<DT>::load(a.o_pre, row * d + c, o);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float xh = r.x[j][e] * rstd;
                r.x[j][e] = xh;
                float dn = dy[e];
                if (a.o_pre) {
                    const float og = sigmoidf_(o[e]);
                    dop[e] = dy[e] * (xh * g[j][e] + be[j][e]) * og * (1.0f - og);
                    dn = dy[e] * og;
                }
                ag[j][e] += dn * xh;
                ab[j][e] += dn;
                dx[j][e] = dn * g[j][e];
                s1 += dx[j][e];
                s2 += dx[j][e] * xh;
            }
            if (a.o_pre && a.do_pre) Row8<DT>::store_stream(a.do_pre, row * d + c, dop);
        }
        s1 = a.kind == 1 ? wave_sum(s1) / (float)d : 0.0f;
        s2 = wave_sum(s2) / (float)d;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int c = (lane + 64 * j) * 8;
            if (c >= d) continue;
            float dh[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) dh[e] = rstd * (dx[j][e] - s1 - r.x[j][e] * s2);
            Row8<DT>::store(a.dh, row * d + c, dh);
        }
    }
    if (!a.part) return;
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int c = (lane + 64 * j) * 8;
        if (c >= d) continue;
#pragma unroll
        for (int e = 0; e < 8; ++e) { red[wave][0][c + e] = ag[j][e]; red[wave][1][c + e] = ab[j][e]; }
    }
    __syncthreads();
    float* out = a.part + ((long)bh * gridDim.x + blk) * 2 * d;
    for (int i = threadIdx.x; i < 2 * d; i += 256) {
        const int w = i / d, c = i - w * d;
        out[i] = (red[0][w][c] + red[1][w][c]) + (red[2][w][c] + red[3][w][c]);
    }
}


// ---- rows of 64, 128 or 256 values: LPR = d / 8 lanes per row, 64 / LPR rows of one wavefront side by side ----
// (one row per wavefront would leave three quarters or more of the lanes idle)
template <int LPR> __device__ __forceinline__ float row_sum(float x) {
#pragma unroll
    for (int m = 1; m < LPR; m <<= 1) x += __shfl_xor(x, m, 64);
    return x;
}
// x (this lane's eight values of its row) -> x - mean for LayerNorm; returns 1 / sqrt(mean((x - mean)^2) + eps)
template <int LPR> __device__ __forceinline__ float center_packed(float (&x)[8], int kind, float eps) {
    constexpr float invd = 1.0f / (float)(LPR * 8);
    if (kind == 1) {
        float sm = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sm += x[e];
        const float mu = row_sum<LPR>(sm) * invd;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] -= mu;
    }
    float ss = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
    return 1.0f / sqrtf(row_sum<LPR>(ss) * invd + eps);
}

template <typename DT, int LPR>
__global__ void __launch_bounds__(256) norm_gate_fwd_packed_kernel(NormArgs a) {
    constexpr int R = 64 / LPR, d = LPR * 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane / LPR, c = (lane % LPR) * 8;
    const long row = ((long)blockIdx.x * 4 + wave) * R + sub;
    const bool live = row < a.rows;
    const long rr = live ? row : a.rows - 1;            // (lanes past the end repeat the last row and store nothing)
    const int head = (int)((rr / a.T) % a.NH);
    float x[8], g[8], be[8], o[8], y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { g[e] = 1.0f; be[e] = 0.0f; o[e] = 0.0f; }
    Row8<DT>::load(a.h, rr * d + c, x);
    if (a.gamma) load8f(a.gamma + (long)head * d + c, g);
    if (a.beta && a.kind == 1) load8f(a.beta + (long)head * d + c, be);
    if (a.o_pre) Row8<DT>::load(a.o_pre, rr * d + c, o);
    const float rstd = center_packed<LPR>(x, a.kind, a.eps);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float n = x[e] * rstd * g[e] + be[e];
        y[e] = a.o_pre ? n * sigmoidf_(o[e]) : n;
    }
    if (live) Row8<DT>::store_stream(a.y, row * d + c, y);
}

template <typename DT, int LPR>
__global__ void __launch_bounds__(256) norm_gate_bwd_packed_kernel(NormBwdArgs a) {
    constexpr int R = 64 / LPR, d = LPR * 8;
    __shared__ float red[4][2][d];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane / LPR, c = (lane % LPR) * 8;
    const int bh = blockIdx.y, blk = blockIdx.x;
    const int head = bh % a.NH;
    float ag[8], ab[8], g[8], be[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { ag[e] = 0.0f; ab[e] = 0.0f; g[e] = 1.0f; be[e] = 0.0f; }
    if (a.gamma) load8f(a.gamma + (long)head * d + c, g);
    if (a.beta && a.kind == 1) load8f(a.beta + (long)head * d + c, be);
    const int t_end = min(a.T, (blk + 1) * NORM_RPB);
    for (int t0 = blk * NORM_RPB + wave * R; t0 < t_end; t0 += 4 * R) {
        const int t = t0 + sub;
        const bool live = t < t_end;
        const long row = (long)bh * a.T + (live ? t : t_end - 1);
        float x[8], dy[8], o[8], dop[8], dx[8];
        Row8<DT>::load(a.h, row * d + c, x);
        Row8<DT>::load(a.dy, row * d + c, dy);
        if (a.o_pre) Row8<DT>::load(a.o_pre, row * d + c, o);
        const float rstd = center_packed<LPR>(x, a.kind, a.eps);
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float xh = x[e] * rstd;
            x[e] = xh;
            float dn = dy[e];
            if (a.o_pre) {
                const float og = sigmoidf_(o[e]);
                dop[e] = dy[e] * (xh * g[e] + be[e]) * og * (1.0f - og);
                dn = dy[e] * og;
            }
            if (live) { ag[e] += dn * xh; ab[e] += dn; }
            dx[e] = dn * g[e];
            s1 += dx[e];
            s2 += dx[e] * xh;
        }
        constexpr float invd = 1.0f / (float)d;
        s1 = a.kind == 1 ? row_sum<LPR>(s1) * invd : 0.0f;
        s2 = row_sum<LPR>(s2) * invd;
        if (live) {
            if (a.o_pre && a.do_pre) Row8<DT>::store_stream(a.do_pre, row * d + c, dop);
            float dh[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) dh[e] = rstd * (dx[e] - s1 - x[e] * s2);
            Row8<DT>::store(a.dh, row * d + c, dh);
        }
    }
    if (!a.part) return;
    // the wavefront's R side-by-side rows add up first (lanes LPR apart hold the same columns), then the four wavefronts
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
        for (int m = LPR; m < 64; m <<= 1) { ag[e] += __shfl_xor(ag[e], m, 64); ab[e] += __shfl_xor(ab[e], m, 64); }
    }
    if (sub == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { red[wave][0][c + e] = ag[e]; red[wave][1][c + e] = ab[e]; }
    }
    __syncthreads();
    float* out = a.part + ((long)bh * gridDim.x + blk) * 2 * d;
    for (int i = threadIdx.x; i < 2 * d; i += 256) {
        const int w = i / d, cc = i - w * d;
        out[i] = (red[0][w][cc] + red[1][w][cc]) + (red[2][w][cc] + red[3][w][cc]);
    }
}

// d gamma[h][c] = sum over batch elements and row blocks of the partial sums (fixed order, fp64).
// A workgroup takes 64 columns of one head; its sixteen wavefronts split the (batch, row block) list (the list is
// a chain of dependent loads per wavefront, and there are only d / 64 x NH workgroups).
constexpr int NPG_WAVES = 16;
__global__ void __launch_bounds__(NPG_WAVES * 64) norm_param_grad_kernel(NormParamGradArgs a) {
    __shared__ double red[NPG_WAVES][2][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane, head = blockIdx.y;
    double sg = 0.0, sb = 0.0;
    if (c < a.d) {
        const int n = a.B * a.nblk;
        for (int i = wave; i < n; i += NPG_WAVES) {
            const int b = i / a.nblk, blk = i - b * a.nblk;
            const float* p = a.part + (((long)b * a.NH + head) * a.nblk + blk) * 2 * a.d;
            sg += (double)p[c];
            sb += (double)p[a.d + c];
        }
    }
    red[wave][0][lane] = sg; red[wave][1][lane] = sb;
    __syncthreads();
    if (wave == 0 && c < a.d) {
        sg = 0.0; sb = 0.0;
#pragma unroll
        for (int w = 0; w < NPG_WAVES; ++w) { sg += red[w][0][lane]; sb += red[w][1][lane]; }
        if (a.dgamma) a.dgamma[(long)head * a.d + c] = (float)sg;
        if (a.dbeta) a.dbeta[(long)head * a.d + c] = (float)sb;
    }
}

// Gains of one (batch, head): time averages of max|h~_t| / max|v_t| and max|NORM(h~_t)| / max|v_t|
// (unit scale, no shift).
template <typename DT, int J>
__global__ void __launch_bounds__(256) transfer_gain_kernel(GainArgs a) {
    __shared__ float red[4][2];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, bh = blockIdx.x, d = a.d;
    float sb = 0.0f, sa = 0.0f;
    for (int t = wave; t < a.T; t += 4) {
        const long row = (long)bh * a.T + t;
        RowRegs<DT, J> r, v;
        r.load(a.h, row, d, lane);
        v.load(a.v, row, d, lane);
        float mh = 0.0f, mv = 0.0f, mc = 0.0f;
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) { mh = fmaxf(mh, fabsf(r.x[j][e])); mv = fmaxf(mv, fabsf(v.x[j][e])); }
        const float rstd = r.center(d, lane, a.kind, a.eps);
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) mc = fmaxf(mc, fabsf(r.x[j][e]));
        mh = wave_max(mh); mv = wave_max(mv); mc = wave_max(mc);
        sb += mh / mv;
        sa += mc * rstd / mv;
    }
    if (lane == 0) { red[wave][0] = sb; red[wave][1] = sa; }
    __syncthreads();
    if (threadIdx.x == 0) {
        a.g_before[bh] = ((red[0][0] + red[1][0]) + (red[2][0] + red[3][0])) / (float)a.T;
        a.g_after[bh] = ((red[0][1] + red[1][1]) + (red[2][1] + red[3][1])) / (float)a.T;
    }
}

template <typename DT, int LPR> hipError_t norm_fwd_packed(const NormArgs& a, hipStream_t s) {
    const long rpb = 4 * (64 / LPR);      // rows per workgroup
    hipLaunchKernelGGL((norm_gate_fwd_packed_kernel<DT, LPR>), dim3((unsigned)((a.rows + rpb - 1) / rpb)), dim3(256), 0, s, a);
    return hipGetLastError();
}
template <typename DT> hipError_t norm_fwd_dt(const NormArgs& a, hipStream_t s) {
    if (a.d == 64) return norm_fwd_packed<DT, 8>(a, s);
    if (a.d == 128) return norm_fwd_packed<DT, 16>(a, s);
    if (a.d == 256) return norm_fwd_packed<DT, 32>(a, s);
    const dim3 grid((unsigned)((a.rows + 3) / 4));
    if (a.d <= 512) hipLaunchKernelGGL((norm_gate_fwd_kernel<DT, 1>), grid, dim3(256), 0, s, a);
    else if (a.d <= 1024) hipLaunchKernelGGL((norm_gate_fwd_kernel<DT, 2>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((norm_gate_fwd_kernel<DT, 4>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}
template <typename DT> hipError_t norm_bwd_dt(const NormBwdArgs& a, int BH, hipStream_t s) {
    const dim3 grid((a.T + NORM_RPB - 1) / NORM_RPB, BH);
    if (a.d == 64 || a.d == 128 || a.d == 256) {
        if (a.d == 64) hipLaunchKernelGGL((norm_gate_bwd_packed_kernel<DT, 8>), grid, dim3(256), 0, s, a);
        else if (a.d == 128) hipLaunchKernelGGL((norm_gate_bwd_packed_kernel<DT, 16>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((norm_gate_bwd_packed_kernel<DT, 32>), grid, dim3(256), 0, s, a);
        return hipGetLastError();
    }
    if (a.d <= 512) hipLaunchKernelGGL((norm_gate_bwd_kernel<DT, 1>), grid, dim3(256), 0, s, a);
    else if (a.d <= 1024) hipLaunchKernelGGL((norm_gate_bwd_kernel<DT, 2>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((norm_gate_bwd_kernel<DT, 4>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}
template <typename DT> hipError_t gain_dt(const GainArgs& a, int BH, hipStream_t s) {
    if (a.d <= 512) hipLaunchKernelGGL((transfer_gain_kernel<DT, 1>), dim3(BH), dim3(256), 0, s, a);
    else if (a.d <= 1024) hipLaunchKernelGGL((transfer_gain_kernel<DT, 2>), dim3(BH), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((transfer_gain_kernel<DT, 4>), dim3(BH), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace

int norm_row_blocks(int T) { return (T + NORM_RPB - 1) / NORM_RPB; }

hipError_t launch_norm_gate_fwd(const NormArgs& a, hipStream_t s) {
    return a.dtype == 1 ? norm_fwd_dt<bf16_t>(a, s) : norm_fwd_dt<float>(a, s);
}
hipError_t launch_norm_gate_bwd(const NormBwdArgs& a, int BH, hipStream_t s) {
    return a.dtype == 1 ? norm_bwd_dt<bf16_t>(a, BH, s) : norm_bwd_dt<float>(a, BH, s);
}
hipError_t launch_norm_param_grad(const NormParamGradArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(norm_param_grad_kernel, dim3((a.d + 63) / 64, a.NH), dim3(NPG_WAVES * 64), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_transfer_gain(const GainArgs& a, int BH, hipStream_t s) {
    return a.dtype == 1 ? gain_dt<bf16_t>(a, BH, s) : gain_dt<float>(a, BH, s);
}

}  // namespace tfla
