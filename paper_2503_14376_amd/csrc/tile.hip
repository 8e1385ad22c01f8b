// Intra-chunk tiled kernel (paper Sec. 3; App. C.3 Alg. 1 for H; App. C.4 for the three
// gradient kernels, with the parallel / loop dimensions of the paper's parallelisation table).
//
// One template covers the four kernels.  For a block of output rows r of one chunk:
//
//   out[r, :] = sum_{c causal} exp2(wrow[r] + wcol[c]) * (X_r . Y_c) * Z_c  +  srow[r] * (X_r St)
//
//   H   : X=Q  Y=K  Z=V   St=C_{k-1}^T        c <= r      (Alg. 1, both parts in one accumulator)
//   dV  : X=K  Y=Q  Z=dH  St=dC_k^T           c >= r
//   dQ  : X=dH Y=V  Z=K   St=C_{k-1}          c <= r
//   dK  : X=V  Y=dH Z=Q   St=dC_k             c >= r
//
// Differences from Alg. 1: the max state of every row is known from the gates alone (see the
// gate kernel), so the weights are final when they are formed -- no running maximum, no
// rescaling of the accumulator, and the inter-chunk product shares the accumulator and the
// register-resident X fragments with the intra-chunk loop for mLSTMexp as well.
//
// Work split: grid = (d2 / BD2, L / (32*NW), B*NH*Nc).  A wavefront owns 32 output rows and
// all BD2 columns of its workgroup; X_r stays in registers for the whole kernel; Y tiles
// (natural) and Z tiles (transposed, k-permuted) go through LDS and are shared by the
// waves.  The product (X_r . Y_c) is formed transposed (rows = c) so that its MFMA result is
// already laid out as the A operand of the second product.
#include "tfla_device.h"
#include "tfla_internal.h"
#include "tile_fast.h"

namespace tfla {

// Generic kernel (any element type; operands staged through registers).  bf16 uses
// tile_kernel_bf16 (tile_fast.h); this one serves fp32.
// SPLIT as in tile_kernel_bf16: 1 / 2 = the first / second D1-wide half of a contraction over 2 D1 columns (rows of
// X, Y and the state are 2 D1 apart); the first half stores its raw accumulators, the second adds them to its own.
template <typename DT, int D1, int BD2, int BC, int NW, int MODE, int SPLIT = 0>
__global__ void __launch_bounds__(NW * 64) tile_kernel(TileArgs a) {
    using E = Elem<DT>;
    using frag = typename E::frag;
    constexpr bool UPPER = (MODE & 1) != 0;
    constexpr int NT = NW * 64, BR = NW * 32;
    constexpr int KS1 = D1 / 16, NB = BD2 / 32, NK = D1 / BC;
    constexpr int YS = D1 + E::PAD, ZS = BC + E::PAD;
    constexpr int ld1 = SPLIT ? 2 * D1 : D1;    // row stride of the operands with D1 columns
    // two stages of (Y tile, Z tile, column weights): one is multiplied while the other is filled
    __shared__ __attribute__((aligned(16))) DT ldsY[2][BC * YS];
    __shared__ __attribute__((aligned(16))) DT ldsZ[2][BD2 * ZS];
    __shared__ float ldsW[2][BC];
    __shared__ float ldsWl[2][BC];     // rounding remainders of the column exponents (zeros when there are none)
    __shared__ float ldsR[NW * 32];
    __shared__ float ldsN[(MODE == MODE_H) ? D1 : 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    // XCD-aware decomposition of the workgroup id: the workgroups of one chunk (all d2 blocks
    // and row blocks, which share K/V/state tiles) are neighbours on one XCD.
    // one-dimensional launch (the number of workgroups can exceed what the y and z grid dimensions hold):
    // linear id -> (column block, row block, chunk, batch*head), column blocks fastest
    const unsigned nwg = gridDim.x, gx = (unsigned)a.d2 / BD2, gy = (unsigned)a.L / (32 * NW);
    unsigned wg = xcd_remap(blockIdx.x, nwg);
    const int nb2 = wg % gx; wg /= gx;
    // later row blocks of a lower-triangular kernel (earlier ones of an upper one) have more
    // column tiles: start them first
    const int rbi = wg % gy; wg /= gy;
    const int rb = UPPER ? rbi : (int)gy - 1 - rbi;
    const int kc = wg % a.Nc, bh = wg / a.Nc;
    const long tbase = (long)bh * a.T + (long)kc * a.L;   // first step of the chunk
    const int r0 = rb * BR;                               // chunk-local first row of the workgroup
    const int wr0 = r0 + wave * 32;                       // ... of the wavefront
    const int d2 = a.d2;

    const DT* X = reinterpret_cast<const DT*>(a.X);
    const DT* Y = reinterpret_cast<const DT*>(a.Y) + tbase * ld1;
    const DT* Z = reinterpret_cast<const DT*>(a.Z) + tbase * d2 + (long)nb2 * BD2;
    const DT* St = reinterpret_cast<const DT*>(a.St) + (((long)bh * a.Nc + kc) * d2 + (long)nb2 * BD2) * ld1;
    const float* wcol = a.wcol + tbase;
    const float* wcol_lo = a.wcol_lo ? a.wcol_lo + tbase : nullptr;

    // X fragments of the wavefront's 32 rows (lane: row l32, k-group g)
    frag xf[KS1];
    {
        const DT* xr = X + (tbase + wr0 + l32) * ld1 + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks) xf[ks] = E::load(xr + 16 * ks);
    }
    if (MODE == MODE_H) {
        if (a.variant == 0)
            for (int i = tid; i < D1; i += NT) ldsN[i] = a.nstate[((long)bh * a.Nc + kc) * ld1 + i];
    }

    f32x16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.0f;

    const int ct_lo = UPPER ? r0 / BC : 0;
    const int ct_hi = UPPER ? a.L / BC : (r0 + BR) / BC;

    RowsPrefetch<DT, BD2, BC, NT> ps;          // state chunk  [BD2][BC]
    RowsPrefetch<DT, BC, D1, NT> py;           // Y tile       [BC][D1]
    TrPrefetch<DT, BC, BD2, NT, true> pz;      // Z tile       [BC][BD2] -> [BD2][BC]
    float pw = 0.0f, pwl = 0.0f;
    int buf = 0;

    // ---------------- inter-chunk part: acc = X_r St, BC columns of d1 per stage
    ps.load(St, ld1, tid);
    ps.store(ldsZ[0], ZS, tid);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NK; ++j) {
        if (j + 1 < NK) {
            ps.load(St + (j + 1) * BC, ld1, tid);
        } else {
            py.load(Y + (long)ct_lo * BC * ld1, ld1, tid);
            pz.load(Z + (long)ct_lo * BC * d2, d2, tid);
            if (tid < BC) { pw = wcol[ct_lo * BC + tid]; pwl = wcol_lo ? wcol_lo[ct_lo * BC + tid] : 0.0f; }
        }
        const DT* zb = ldsZ[buf];
#pragma unroll
        for (int ks = 0; ks < BC / 16; ++ks)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = E::mma(xf[j * (BC / 16) + ks], E::load(zb + (nb * 32 + l32) * ZS + 16 * ks + 8 * g), acc[nb]);
        if (j + 1 < NK) {
            ps.store(ldsZ[buf ^ 1], ZS, tid);
        } else {
            py.store(ldsY[buf ^ 1], YS, tid);
            pz.template store<false>(ldsZ[buf ^ 1], ZS, nullptr, tid);
            if (tid < BC) { ldsW[buf ^ 1][tid] = pw; ldsWl[buf ^ 1][tid] = pwl; }
        }
        __syncthreads();
        buf ^= 1;
    }
    {
        float sr[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) sr[v] = a.srow[tbase + wr0 + acc_row(v, g)];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][v] *= sr[v];
    }

    // mLSTMexp normaliser, inter-chunk part: srow_i * (q_i . n_{k-1}), one value per row
    float nrm = 0.0f;
    if (MODE == MODE_H) {
        if (a.variant == 0) {
            float dot = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) dot += E::frag_elem(xf[ks], e) * ldsN[16 * ks + 8 * g + e];
            dot += __shfl_xor(dot, 32, 64);
            nrm = dot * a.srow[tbase + wr0 + l32];
        }
    }

    // ---------------- intra-chunk part
    const float wr = a.wrow[tbase + wr0 + l32];
    const float wrl = a.wrow_lo ? a.wrow_lo[tbase + wr0 + l32] : 0.0f;
    float rowsum = 0.0f;
    for (int ct = ct_lo; ct < ct_hi; ++ct) {
        const int c0 = ct * BC;
        const bool more = ct + 1 < ct_hi;
        if (more) {
            py.load(Y + (long)(c0 + BC) * ld1, ld1, tid);
            pz.load(Z + (long)(c0 + BC) * d2, d2, tid);
            if (tid < BC) { pw = wcol[c0 + BC + tid]; pwl = wcol_lo ? wcol_lo[c0 + BC + tid] : 0.0f; }
        }
        const DT* yb = ldsY[buf];
        const DT* zb = ldsZ[buf];
        const float* wb = ldsW[buf];
        const float* wbl = ldsWl[buf];
#pragma unroll
        for (int st = 0; st < BC / 32; ++st) {
            const int cs = c0 + 32 * st;
            if (UPPER ? (cs + 31 < wr0) : (cs > wr0 + 31)) continue;      // fully masked for this wave
            const bool diag = UPPER ? (cs < wr0 + 31) : (cs + 31 > wr0);
            f32x16 s;
#pragma unroll
            for (int v = 0; v < 16; ++v) s[v] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks)
                s = E::mma(E::load(yb + (32 * st + l32) * YS + 16 * ks + 8 * g), xf[ks], s);
            float p[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int cl = acc_row(v, g);
                // (rounded parts first: they nearly cancel, and their sum is exact in fp32)
                float w = fast_exp2((wr + wb[32 * st + cl]) + (wrl + wbl[32 * st + cl]));
                if (diag) {
                    const bool keep = UPPER ? (cs + cl >= wr0 + l32) : (cs + cl <= wr0 + l32);
                    w = keep ? w : 0.0f;
                }
                p[v] = s[v] * w;
                rowsum += p[v];
            }
            const frag p0 = E::pack(p), p1 = E::pack(p + 8);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const DT* zrow = zb + (nb * 32 + l32) * ZS + 32 * st + 8 * g;
                acc[nb] = E::mma(p0, E::load(zrow), acc[nb]);
                acc[nb] = E::mma(p1, E::load(zrow + 16), acc[nb]);
            }
        }
        if (more) {
            py.store(ldsY[buf ^ 1], YS, tid);
            pz.template store<false>(ldsZ[buf ^ 1], ZS, nullptr, tid);
            if (tid < BC) { ldsW[buf ^ 1][tid] = pw; ldsWl[buf ^ 1][tid] = pwl; }
        }
        __syncthreads();
        buf ^= 1;
    }

    // ---------------- epilogue
    float inv[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) inv[v] = 1.0f;
    if (MODE == MODE_H) {
        if (a.variant == 0) {
            rowsum += __shfl_xor(rowsum, 32, 64);
            nrm += rowsum;
        }
    }
    if constexpr (SPLIT == 1) {
        // first half: raw accumulators (and this half's share of the normaliser) for the second launch
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const long t = tbase + wr0 + acc_row(v, g);
                a.acc_out[t * d2 + (long)nb2 * BD2 + nb * 32 + l32] = acc[nb][v];
            }
        if (MODE == MODE_H && a.variant == 0 && g == 0 && nb2 == 0) a.nrm_out[tbase + wr0 + l32] = nrm;
        return;
    }
    if constexpr (SPLIT == 2) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const long t = tbase + wr0 + acc_row(v, g);
                acc[nb][v] += a.acc_in[t * d2 + (long)nb2 * BD2 + nb * 32 + l32];
            }
        if (MODE == MODE_H && a.variant == 0) nrm += a.nrm_in[tbase + wr0 + l32];
    }
    if (MODE == MODE_H) {
        if (a.variant == 0) {
            const long t = tbase + wr0 + l32;
            const float den = fmaxf(fabsf(nrm), expf(-a.mout[t])) + a.eps;
            if (g == 0) {
                ldsR[wave * 32 + l32] = 1.0f / den;
                if (a.nout && nb2 == 0) a.nout[t] = nrm;
                if (a.wrowB_out && nb2 == 0) {
                    if (a.wrowB_lo_out) {
                        const double w = (double)wr + (double)wrl - log2((double)den);
                        const float wh = (float)w;
                        a.wrowB_out[t] = wh;
                        a.wrowB_lo_out[t] = (float)(w - (double)wh);
                    } else {
                        a.wrowB_out[t] = a.wrow[t] - log2f(den);
                    }
                    a.sQ_out[t] = a.srow[t] / den;
                }
            }
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) inv[v] = ldsR[wave * 32 + acc_row(v, g)];
        }
    }
    DT* Out = reinterpret_cast<DT*>(a.Out);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            // straight into the caller's tensor: its own row count and row length, true steps and columns only
            const int ts = kc * a.L + wr0 + acc_row(v, g), col = nb2 * BD2 + nb * 32 + l32;
            if (ts < a.out_T && col < a.out_cols)
                Out[((long)bh * a.out_T + ts) * a.out_ld + col] = E::from_f32(acc[nb][v] * inv[v]);
        }
    if (MODE == MODE_DQ || MODE == MODE_DK) {
        const DT* W = reinterpret_cast<const DT*>(a.dotwith);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const long t = tbase + wr0 + acc_row(v, g);
            float d = 0.0f;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                d += acc[nb][v] * E::to_f32(W[t * d2 + (long)nb2 * BD2 + nb * 32 + l32]);
            d = half_sum(d);
            if (l32 == 0) a.dotpart[(long)nb2 * (long)(nwg / (gx * gy * (unsigned)a.Nc)) * a.T + t] = d;
        }
    }
}

// ------------------------------------------------------------------------------------------
template <typename DT, int D1, int BD2, int NW, int MODE, int SPLIT = 0>
static hipError_t launch_tile_t(const TileArgs& a0, int BH, hipStream_t s) {
    TileArgs a = a0;
    dim3 grid((unsigned)((long)(a.d2 / BD2) * (a.L / (32 * NW)) * BH * a.Nc));
    if constexpr (sizeof(DT) == 2) {
        // what the kernel's decomposition of the linear workgroup id divides by
        auto log2_or_neg = [](int v) { return (v > 0 && (v & (v - 1)) == 0) ? __builtin_ctz((unsigned)v) : -1; };
        a.dec_bh = BH;
        a.dec_bpx = BH % 8 == 0 ? BH / 8 : 1;
        a.sh_gx = log2_or_neg(a.d2 / BD2); a.sh_gy = log2_or_neg(a.L / (32 * NW));
        a.sh_bpx = log2_or_neg(a.dec_bpx); a.sh_nc = log2_or_neg(a.Nc);
        // two workgroups per CU when the accumulator is narrow enough for 256 registers per lane
        constexpr int OCC = (BD2 <= 128 && D1 <= 256) ? 2 : 1;
        // dQ / dK share the weighted matrix E through memory only where the contraction that forms it is wide
        constexpr int NOE = ((MODE == MODE_DQ || MODE == MODE_DK) && D1 <= TFLA_NOE_MAX_D1) ? 1 : 0;
        // a padded problem stores its true part straight into the caller's tensor (the first half of a split
        // contraction stores no output at all)
        const bool padded = a.out_T != a.T || a.out_ld != a.d2;
        if constexpr (MODE == MODE_H && SPLIT == 0 && BD2 <= 128) {
            // the layer output next to h~: whole rows in one workgroup, nothing padded (the entry point has checked)
            if (a.fz_y) {
                if (padded || a.d2 != BD2) return hipErrorInvalidValue;
                hipLaunchKernelGGL((tile_kernel_bf16<D1, BD2, NW, MODE, OCC, 0, 0, 0, 1>), grid, dim3(64 * NW), 0, s, a);
                return hipGetLastError();
            }
        }
        if (a.fz_y) return hipErrorInvalidValue;
        if (SPLIT != 1 && padded)
            hipLaunchKernelGGL((tile_kernel_bf16<D1, BD2, NW, MODE, OCC, SPLIT, NOE, SPLIT != 1>), grid, dim3(64 * NW), 0, s, a);
        else
            hipLaunchKernelGGL((tile_kernel_bf16<D1, BD2, NW, MODE, OCC, SPLIT, NOE, 0>), grid, dim3(64 * NW), 0, s, a);
    } else {
        constexpr int BC = 32;   // two LDS stages must fit in 160 KB
        hipLaunchKernelGGL((tile_kernel<DT, D1, BD2, BC, NW, MODE, SPLIT>), grid, dim3(64 * NW), 0, s, a);
    }
    return hipGetLastError();
}

template <typename DT, int D1, int MODE, int SPLIT = 0>
static hipError_t launch_tile_d1(const TileArgs& a, int BH, int bd2, hipStream_t s) {
    if (a.L % 128 == 0) {
        if constexpr (sizeof(DT) == 2 && D1 > 256 && SPLIT == 0 && (MODE == MODE_DQ || MODE == MODE_DK)) {   // see tile_bd2()
            if (bd2 == 256) return launch_tile_t<DT, D1, 256, 4, MODE>(a, BH, s);
        }
        if (bd2 == 128) return launch_tile_t<DT, D1, 128, 4, MODE, SPLIT>(a, BH, s);
        if (bd2 == 64) return launch_tile_t<DT, D1, 64, 4, MODE, SPLIT>(a, BH, s);
        return hipErrorInvalidValue;    // the caller sized its buffers for a block width that is not built
    }
    if (bd2 == 128) return launch_tile_t<DT, D1, 128, 2, MODE, SPLIT>(a, BH, s);
    if (bd2 == 64) return launch_tile_t<DT, D1, 64, 2, MODE, SPLIT>(a, BH, s);
    return hipErrorInvalidValue;
}

template <typename DT, int MODE>
static hipError_t launch_tile_m(const TileArgs& a, int BH, int bd2, hipStream_t s) {
    switch (a.d1) {
        case 64: return launch_tile_d1<DT, 64, MODE>(a, BH, bd2, s);
        case 128: return launch_tile_d1<DT, 128, MODE>(a, BH, bd2, s);
        case 256: return launch_tile_d1<DT, 256, MODE>(a, BH, bd2, s);
        case 512:
            if (sizeof(DT) == 2) return launch_tile_d1<DT, (sizeof(DT) == 2 ? 512 : 64), MODE>(a, BH, bd2, s);
            break;
        default: break;
    }
    return hipErrorInvalidValue;
}

// one 512-wide half (SPLIT = 1, 2) of a bf16 contraction over 1024 columns
template <int MODE, int SPLIT>
static hipError_t launch_tile_half(const TileArgs& a, int BH, int bd2, hipStream_t s) {
    return launch_tile_d1<bf16_t, 512, MODE, SPLIT>(a, BH, bd2, s);
}

template <int MODE>
hipError_t launch_tile_mode(const TileArgs& a0, int BH, int dtype, hipStream_t s) {
    TileArgs a = a0;
    a.acc_in = nullptr; a.nrm_in = nullptr; a.acc_out = nullptr; a.nrm_out = nullptr;
    // Chunk order of each kernel of the sequence gates -> recurrence (first to last) -> H and reversed recurrence
    // (last to first) -> dV -> dQ -> dK, chosen by measurement (eight of the sixteen combinations on one box):
    // what matters is that H walks the chunks first to last, like the recurrence before it -- starting with the
    // states that were stored last (with non-temporal stores) costs 2 % of the step; among the gradient kernels
    // the differences are a few tenths of a percent, dK walking against dQ being the best.
#ifndef TFLA_KC_ORDER
#define TFLA_KC_ORDER 0x8   // bit m = 1: mode m walks the chunks last to first.  H, dV, dQ first to last, dK last to first
#endif
    a.kc_desc = ((TFLA_KC_ORDER) >> MODE) & 1;
    const int bd2 = tile_bd2(a.d1, a.d2, dtype, MODE, a.L);
    const bool nrm = MODE == MODE_H && a.variant == 0;
    if (dtype != 1) {
        if (a.d1 <= 256) return launch_tile_m<float, MODE>(a, BH, bd2, s);
        // fp32, d1 = 512: a wavefront's rows of X fill the register file at 256 fp32 columns, so the contraction runs
        // as two 256-wide launches that meet in fp32, exactly like the 1024-wide bf16 case below
        if (a.d1 != 512 || !a.part_acc || (nrm && !a.part_nrm)) return hipErrorInvalidValue;
        TileArgs h = a;
        h.d1 = 256;
        h.acc_out = a.part_acc; h.nrm_out = a.part_nrm;
        hipError_t e = launch_tile_d1<float, 256, MODE, 1>(h, BH, bd2, s);
        if (e != hipSuccess) return e;
        h.acc_out = nullptr; h.nrm_out = nullptr;
        h.acc_in = a.part_acc; h.nrm_in = a.part_nrm;
        h.X = reinterpret_cast<const float*>(a.X) + 256;
        h.Y = reinterpret_cast<const float*>(a.Y) + 256;
        h.St = reinterpret_cast<const float*>(a.St) + 256;
        if (a.nstate) h.nstate = a.nstate + 256;
        return launch_tile_d1<float, 256, MODE, 2>(h, BH, bd2, s);
    }
    if (a.d1 <= 512) return launch_tile_m<bf16_t, MODE>(a, BH, bd2, s);
    // d1 = 1024: the kernels hold a workgroup's X rows in registers, which ends at 512 columns.  Every term of
    // the result is linear in the products over d1 (the weights depend on the gates only), so the contraction
    // runs as two launches over 512 columns each: the first leaves its unnormalised accumulators (and its share
    // of the normaliser) in fp32, the second adds them to its own before the epilogue.  dQ writes one matrix E
    // per half (its products run over the halves of d_hv); dK reads the matching one in each of its launches.
    constexpr bool STT = (MODE == MODE_DQ || MODE == MODE_DK);
    if (a.d1 != 1024 || !a.part_acc || (nrm && !a.part_nrm) || (STT && a.E && !a.E2)) return hipErrorInvalidValue;
    TileArgs h = a;
    h.d1 = 512;
    h.acc_out = a.part_acc; h.nrm_out = a.part_nrm;
    hipError_t e = launch_tile_half<MODE, 1>(h, BH, bd2, s);
    if (e != hipSuccess) return e;
    h.acc_out = nullptr; h.nrm_out = nullptr;
    h.acc_in = a.part_acc; h.nrm_in = a.part_nrm;
    h.X = reinterpret_cast<const bf16_t*>(a.X) + 512;
    if (MODE != MODE_DK) h.Y = reinterpret_cast<const bf16_t*>(a.Y) + 512;
    h.St = reinterpret_cast<const bf16_t*>(a.St) + (STT ? (long)512 * a.d2 : 512);
    // (n_{k-1} is stored as bf16 rows: 512 columns are 1024 bytes)
    if (a.nstate) h.nstate = reinterpret_cast<const float*>(reinterpret_cast<const char*>(a.nstate) + 1024);
    if (STT) h.E = a.E2;
    return launch_tile_half<MODE, 2>(h, BH, bd2, s);
}

// One translation unit per (mode, element type) keeps compile times parallel: tile_inst.hip
// is compiled once for every TFLA_TILE_MODE.
template hipError_t launch_tile_mode<TFLA_TILE_MODE>(const TileArgs&, int, int, hipStream_t);

}  // namespace tfla
