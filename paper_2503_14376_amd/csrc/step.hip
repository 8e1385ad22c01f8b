// Single-step recurrent kernel (paper Sec. 2.1 for mLSTMexp, Sec. 4.1 for mLSTMsig): the form
// used for generation, where the state (C, n, m) is read and written once per step.  The
// step is bound by the traffic of the matrix memory C (App. F, memory operation counts of the
// recurrent formulation): 2 d_qk d_hv floats per head.
//
// One workgroup owns all d_qk rows of a 64-column slab of C for one (batch, head): thread
// (ty, tx) walks rows ty, ty + 16, ... and holds columns 4 tx .. 4 tx + 3, so every row
// segment moves as one coalesced 256-byte access, C is updated in registers between its load
// and its store, and the numerator C'^T q~ needs only one reduction over the 16 row groups.
// The normaliser n' q~ and the max state are recomputed by every slab (d_qk values).
#include "tfla_device.h"
#include "tfla_internal.h"

namespace tfla {

template <typename DT>
__global__ void __launch_bounds__(256) step_kernel(StepArgs a) {
    using E = Elem<DT>;
    __shared__ float sk[1024], sq[1024];
    __shared__ float snum[16][64];
    __shared__ float sred[4];
    const int bh = blockIdx.y, nb = blockIdx.x, tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int dqk = a.dqk, dhv = a.dhv;
    const bool is_exp = a.variant == 0;
    const DT* q = reinterpret_cast<const DT*>(a.q) + (long)bh * dqk;
    const DT* k = reinterpret_cast<const DT*>(a.k) + (long)bh * dqk;
    const DT* v = reinterpret_cast<const DT*>(a.v) + (long)bh * dhv + nb * 64;
    float ip = a.i_pre[bh], fp = a.f_pre[bh];
    if (a.softcap > 0.0f) { ip = a.softcap * tanhf(ip / a.softcap); fp = a.softcap * tanhf(fp / a.softcap); }
    const float qscale = 1.0f / sqrtf((float)dqk);
    // gates (Sec. 2.1: m_t = max(log sigma(f~) + m_{t-1}, i~), stabilised f', i'; Sec. 4.1: sigmoids)
    float fg, ig, m_new = 0.0f;
    if (is_exp) {
        const float fbar = fminf(fp, 0.0f) - log1pf(expf(-fabsf(fp)));
        const float m_old = a.m ? a.m[bh] : 0.0f;
        m_new = fmaxf(fbar + m_old, ip);
        fg = expf(fbar + m_old - m_new);
        ig = expf(ip - m_new);
    } else {
        fg = 1.0f / (1.0f + expf(-fp));
        ig = 1.0f / (1.0f + expf(-ip));
    }
    for (int i = tid; i < dqk; i += 256) {
        sk[i] = E::to_f32(k[i]);
        sq[i] = E::to_f32(q[i]) * qscale;
    }
    __syncthreads();
    // normaliser: n' = f' n + i' k, dot = n'^T q~ (every slab recomputes it; slab 0 stores n')
    float dot = 0.0f;
    if (is_exp) {
        for (int i = tid; i < dqk; i += 256) {
            const float nn = fg * (a.n ? a.n[(long)bh * dqk + i] : 0.0f) + ig * sk[i];
            if (nb == 0 && a.n_out) a.n_out[(long)bh * dqk + i] = nn;
            dot += nn * sq[i];
        }
        dot = wave_sum(dot);
        if ((tid & 63) == 0) sred[tid >> 6] = dot;
    }
    // matrix memory: C' = f' C + i' k v^T, numerator C'^T q~
    const float4 vv = {E::to_f32(v[4 * tx]), E::to_f32(v[4 * tx + 1]), E::to_f32(v[4 * tx + 2]), E::to_f32(v[4 * tx + 3])};
    const float* Cin = a.C + ((long)bh * dqk) * dhv + nb * 64 + 4 * tx;
    float* Cout = a.C_out + ((long)bh * dqk) * dhv + nb * 64 + 4 * tx;
    float4 num = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int m = ty; m < dqk; m += 16) {
        const float4 c = *reinterpret_cast<const float4*>(Cin + (long)m * dhv);
        const float ik = ig * sk[m], qm = sq[m];
        float4 o;
        o.x = fg * c.x + ik * vv.x; o.y = fg * c.y + ik * vv.y; o.z = fg * c.z + ik * vv.z; o.w = fg * c.w + ik * vv.w;
        *reinterpret_cast<float4*>(Cout + (long)m * dhv) = o;
        num.x += o.x * qm; num.y += o.y * qm; num.z += o.z * qm; num.w += o.w * qm;
    }
    *reinterpret_cast<float4*>(&snum[ty][4 * tx]) = num;
    __syncthreads();
    if (tid < 64) {
        float s = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) s += snum[r][tid];
        float den = 1.0f;
        if (is_exp) {
            const float d = sred[0] + sred[1] + sred[2] + sred[3];
            den = fmaxf(fabsf(d), expf(-m_new)) + a.eps;
        }
        reinterpret_cast<DT*>(a.h)[(long)bh * dhv + nb * 64 + tid] = E::from_f32(s / den);
    }
    if (is_exp && nb == 0 && tid == 0 && a.m_out) a.m_out[bh] = m_new;
}

hipError_t launch_step(const StepArgs& a, int BH, hipStream_t s) {
    const dim3 grid(a.dhv / 64, BH);
    if (a.dtype == 1) hipLaunchKernelGGL(step_kernel<bf16_t>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(step_kernel<float>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace tfla
