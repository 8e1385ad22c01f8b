/*
 * TEST INFRASTRUCTURE ONLY -- fp64 CPU oracle for the mLSTM forward pass.
 *
 * Plain step-by-step evaluation of the recurrent mLSTM formulation
 * (paper Sec. 2.1, the state-update equations for m_t, C_t, n_t and the
 * hidden state h~_t) and of the sigmoid-input-gate variant mLSTMsig
 * (paper Sec. 4.1).  One (batch, head) slice at a time, one time step at a
 * time, every quantity in double precision.  No chunking, no tiling, no
 * reordering: this is the definition the GPU kernels are checked against.
 *
 * Readings of the paper taken here:
 *  - the kernel output is h~_t (the NORM layer and the output gate of
 *    Sec. 2.1 are left out, as in Sec. 2.2);
 *  - q is scaled by 1/sqrt(d_qk) here (it is part of the h~_t equation),
 *    callers pass the raw q;
 *  - eps is added to the denominator max{|n^T q|, exp(-m_t)}; eps = 0 is the
 *    paper's formula;
 *  - states are kept in the stabilised coordinates of the recurrence
 *    (true C = C * exp(m)).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg use this
 * file.  It shares no code with the HIP path.
 *
 * Parallelism: OpenMP over (batch, head) slices only.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double log_sigmoid(double x) {
    /* log(1/(1+exp(-x))) without overflow for either sign of x */
    return (x < 0.0 ? x : 0.0) - log1p(exp(-fabs(x)));
}

static double sigmoid(double x) {
    if (x >= 0.0) return 1.0 / (1.0 + exp(-x));
    double e = exp(x);
    return e / (1.0 + e);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * q,k: (BH, T, dqk); v: (BH, T, dhv); i_pre,f_pre: (BH, T);
 * C0: (BH, dqk, dhv) or NULL; n0: (BH, dqk) or NULL; m0: (BH) or NULL.
 * variant: 0 = exponential input gate, 1 = sigmoid input gate.
 * Outputs: H (BH,T,dhv); Cn (BH,dqk,dhv), nn (BH,dqk), mn (BH) final state;
 * n_out (BH,T) = n_t^T q~_t (signed), m_out (BH,T) = m_t.  Any output may be
 * NULL.  For the sigmoid variant nn, mn, n_out, m_out are written as zero.
 * Returns 0, or -1 if memory could not be obtained.
 */
int oracle_mlstm_recurrent_fwd(const double* q, const double* k, const double* v,
                               const double* i_pre, const double* f_pre,
                               const double* C0, const double* n0, const double* m0,
                               long BH, long T, long dqk, long dhv, int variant, double eps,
                               double* H, double* Cn, double* nn, double* mn,
                               double* n_out, double* m_out) {
    int fail = 0;
    const double qscale = 1.0 / sqrt((double)dqk);
#pragma omp parallel for schedule(dynamic, 1)
    for (long s = 0; s < BH; ++s) {
        double* C = (double*)malloc(sizeof(double) * (size_t)(dqk * dhv));
        double* n = (double*)malloc(sizeof(double) * (size_t)dqk);
        double* num = (double*)malloc(sizeof(double) * (size_t)dhv);
        if (!C || !n || !num) {
#pragma omp atomic write
            fail = 1;
            free(C); free(n); free(num);
            continue;
        }
        if (C0) memcpy(C, C0 + s * dqk * dhv, sizeof(double) * (size_t)(dqk * dhv));
        else memset(C, 0, sizeof(double) * (size_t)(dqk * dhv));
        if (n0) memcpy(n, n0 + s * dqk, sizeof(double) * (size_t)dqk);
        else memset(n, 0, sizeof(double) * (size_t)dqk);
        double m = (m0 && variant == 0) ? m0[s] : 0.0;

        for (long t = 0; t < T; ++t) {
            const double* qt = q + (s * T + t) * dqk;
            const double* kt = k + (s * T + t) * dqk;
            const double* vt = v + (s * T + t) * dhv;
            const double it = i_pre[s * T + t];
            const double ft = f_pre[s * T + t];
            double fgate, igate;
            if (variant == 0) {
                /* m_t = max{log sigma(f~_t) + m_{t-1}, i~_t};
                   f_t = exp(log sigma(f~_t) + m_{t-1} - m_t); i_t = exp(i~_t - m_t) */
                const double lf = log_sigmoid(ft);
                const double m_new = fmax(lf + m, it);
                fgate = exp(lf + m - m_new);
                igate = exp(it - m_new);
                m = m_new;
            } else {
                /* C_t = sigma(f~_t) C_{t-1} + sigma(i~_t) k_t v_t^T */
                fgate = sigmoid(ft);
                igate = sigmoid(it);
            }
            /* C_t = f_t C_{t-1} + i_t k_t v_t^T ; n_t = f_t n_{t-1} + i_t k_t ;
               numerator C_t^T (q_t / sqrt(d_qk)) ; normaliser n_t^T (q_t / sqrt(d_qk)) */
            for (long e = 0; e < dhv; ++e) num[e] = 0.0;
            double qn = 0.0;
            for (long d = 0; d < dqk; ++d) {
                double* Cd = C + d * dhv;
                const double ik = igate * kt[d];
                const double qd = qt[d] * qscale;
                for (long e = 0; e < dhv; ++e) {
                    const double c = fgate * Cd[e] + ik * vt[e];
                    Cd[e] = c;
                    num[e] += c * qd;
                }
                n[d] = fgate * n[d] + ik;
                qn += n[d] * qd;
            }
            double den = 1.0;
            if (variant == 0) den = fmax(fabs(qn), exp(-m)) + eps;
            if (H) {
                double* Ht = H + (s * T + t) * dhv;
                for (long e = 0; e < dhv; ++e) Ht[e] = num[e] / den;
            }
            if (n_out) n_out[s * T + t] = (variant == 0) ? qn : 0.0;
            if (m_out) m_out[s * T + t] = (variant == 0) ? m : 0.0;
        }
        if (Cn) memcpy(Cn + s * dqk * dhv, C, sizeof(double) * (size_t)(dqk * dhv));
        if (nn) {
            if (variant == 0) memcpy(nn + s * dqk, n, sizeof(double) * (size_t)dqk);
            else memset(nn + s * dqk, 0, sizeof(double) * (size_t)dqk);
        }
        if (mn) mn[s] = (variant == 0) ? m : 0.0;
        free(C); free(n); free(num);
    }
    return fail ? -1 : 0;
}
