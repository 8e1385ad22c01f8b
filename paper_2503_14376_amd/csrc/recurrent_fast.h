// bf16 fast path of the inter-chunk recurrent kernel (see recurrent.hip for what is computed).
//
//   state <- gbar_k * state + (rs (.) X_k)^T Y_k        (contraction over the rows of a chunk)
//
// Both operands are contracted over their row index, so both stay in their natural row-major
// layout in LDS and are read through the transposing LDS read.  X and Y pieces (64 rows) and
// the 64 row scales of a piece all arrive by asynchronous global->LDS loads in a ring of NS
// stages that runs across chunk boundaries, so the sequential dependence between chunks never
// drains the pipeline and no operand is staged through registers.  The row scale is applied
// to the A fragments in registers (fp32 multiply, rounded back to bf16) right before the MFMA.
#pragma once
#include "lds_tiles.h"
#include "tfla_internal.h"

namespace tfla {

#ifdef TFLA_TIMELINE
static __device__ unsigned long long tfla_rec_timeline[8192];
#define TFLA_RTL(slot) if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && (slot) < 8192) tfla_rec_timeline[(slot)] = __builtin_amdgcn_s_memtime()
#else
#define TFLA_RTL(slot)
#endif

template <int WM, int WN, int MI, int NI>
__global__ void __launch_bounds__(WM * WN * 64) recurrent_kernel_bf16(RecArgs a) {
    using E = Elem<bf16_t>;
    using frag = E::frag;
    constexpr int NWV = WM * WN, NT = NWV * 64, BM = WM * 32 * MI, BN = WN * 32 * NI, BK = 64;
    constexpr int XB = BK * BM * 2, YB = BK * BN * 2, STAGE = XB + YB;
    constexpr int NS = 4;
    using DX = DmaTile<BK, BM, NT, SWZ_T>;
    using DY = DmaTile<BK, BN, NT, SWZ_T>;
    constexpr int CPP = DX::N + DY::N + 2;          // loads per wave and piece (X, Y, row scales, gbar)
    constexpr int STEADY = (NS - 2) * CPP;          // loads younger than piece i's while waiting for it

    __shared__ __attribute__((aligned(1024))) char smem[NS * STAGE];
    __shared__ __attribute__((aligned(256))) float ldsRs[NS][NWV][BK];   // each wave keeps its own copy
    // gbar of the piece's chunk (64 copies): fetched with the piece so that no plain load, whose
    // compiler-placed wait would drain the ring, is needed at a chunk boundary
    __shared__ __attribute__((aligned(256))) float ldsG[NS][NWV][64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    const unsigned nwg = gridDim.x * gridDim.y * gridDim.z;
    unsigned wg = xcd_remap(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), nwg);
    // readfirstlane: tell the compiler these are wave-uniform, so that everything derived from them
    // (addresses of per-chunk scalars in particular) is fetched with scalar loads
    const int bx = __builtin_amdgcn_readfirstlane((int)(wg % gridDim.x)); wg /= gridDim.x;
    const int by = __builtin_amdgcn_readfirstlane((int)(wg % gridDim.y));
    const int bh = __builtin_amdgcn_readfirstlane((int)(wg / gridDim.y));
    const int n0 = bx * BN, m0 = by * BM;
    const bf16_t* X = reinterpret_cast<const bf16_t*>(a.X) + (long)bh * a.T * a.d1 + m0;
    const bf16_t* Y = reinterpret_cast<const bf16_t*>(a.Y) + (long)bh * a.T * a.d2 + n0;
    const float* rs = a.rs + (long)bh * a.T;
    // the normaliser vector is kept by the waves wn == 0 of the workgroups bx == 0: lane (l32, g = 0)
    // of such a wave owns element m0 + (wm * MI + mi) * 32 + l32
    const bool with_n = (a.nst != nullptr) && bx == 0 && wn == 0;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * MI + mi) * 32 + acc_row(v, g);
                const int n = n0 + (wn * NI + ni) * 32 + l32;
                acc[mi][ni][v] = a.S0 ? a.S0[((long)bh * a.d1 + m) * a.d2 + n] : 0.0f;
            }
    float nacc[MI], npart[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        nacc[mi] = (with_n && a.n0) ? a.n0[(long)bh * a.d1 + m0 + (wm * MI + mi) * 32 + l32] : 0.0f;
        npart[mi] = 0.0f;
    }

    const int PPC = a.L / BK, P = a.Nc * PPC;
    auto chunk_of = [&](int i) -> int {
        const int stepc = i / PPC;
        return a.reverse ? a.Nc - 1 - stepc : stepc;
    };

    DX dx; dx.init(a.d1, tid);
    DY dy; dy.init(a.d2, tid);
    const uint32_t smem_a = lds_addr(smem), rs_a = lds_addr(ldsRs), g_a = lds_addr(ldsG);
    auto load_piece = [&](int p, int slot) {
        const long tr = (long)chunk_of(p) * a.L + (long)(p % PPC) * BK;
        dx.issue(X + tr * a.d1, smem_a + (uint32_t)slot * STAGE, tid);
        dy.issue(Y + tr * a.d2, smem_a + (uint32_t)slot * STAGE + XB, tid);
        dma4(rs + tr, (uint32_t)lane * 4u, rs_a + (uint32_t)((slot * NWV + wave) * BK * 4));
        dma4(a.gbar + (long)bh * a.Nc + chunk_of(p), 0u, g_a + (uint32_t)((slot * NWV + wave) * 64 * 4));
    };

    TFragReader<BM> ra; ra.init(lane, 8);
    TFragReader<BN> rb; rb.init(lane, 8);
    uint32_t aoff[MI], boff[NI];      // LDS byte offsets of this wave's A / B column blocks
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) aoff[mi] = ra.block_offset(wm * MI + mi);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) boff[ni] = rb.block_offset(wn * NI + ni);

    // plain loads above (initial state) must not be counted against the ring
    wait_vmcnt<0>();
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < P) load_piece(p, p);

    for (int i0 = 0; i0 < P; i0 += NS) {
#pragma unroll
        for (int dd = 0; dd < NS; ++dd) {
            const int i = i0 + dd;
            if (i < P) {
                TFLA_RTL(4 * i);
                if (i + NS - 2 < P) wait_vmcnt<STEADY>(); else wait_vmcnt<0>();
                TFLA_RTL(4 * i + 1);
                barrier_nofence();
                TFLA_RTL(4 * i + 2);
                if (i + NS - 1 < P) load_piece(i + NS - 1, (dd + NS - 1) % NS);
                // ---- chunk boundary: emit the state before this chunk's update, then decay
                if (i % PPC == 0) {
                    const int kc = chunk_of(i);
                    const long slot = (long)bh * a.Nc + kc;
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) {
                            const int n = n0 + (wn * NI + ni) * 32 + l32;
                            if (a.stN) {
                                bf16_t* dst = reinterpret_cast<bf16_t*>(a.stN) + slot * a.d1 * a.d2;
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const int m = m0 + (wm * MI + mi) * 32 + acc_row(v, g);
                                    dst[(long)m * a.d2 + n] = E::from_f32(acc[mi][ni][v]);
                                }
                            }
                            if (a.stT) {
                                bf16_t* dst = reinterpret_cast<bf16_t*>(a.stT) + slot * a.d1 * a.d2;
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const int m = m0 + (wm * MI + mi) * 32 + acc_row(4 * j, g);
                                    store4(dst + (long)n * a.d1 + m, acc[mi][ni][4 * j], acc[mi][ni][4 * j + 1],
                                           acc[mi][ni][4 * j + 2], acc[mi][ni][4 * j + 3]);
                                }
                            }
                        }
                    const float gb = ldsG[dd][wave][lane];
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[mi][ni][v] *= gb;
                }
                TFLA_RTL(4 * i + 3);
                // ---- multiply piece i
                const char* xt = smem + dd * STAGE;
                const char* yt = xt + XB;
                const float* rsp = &ldsRs[dd][wave][0];
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    frag af[MI], bfr[NI];
                    const f32x4 s0 = *reinterpret_cast<const f32x4*>(rsp + 16 * ks + 8 * g);
                    const f32x4 s1 = *reinterpret_cast<const f32x4*>(rsp + 16 * ks + 8 * g + 4);
                    const float sc[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) {
                        const bf16x8 raw = TFragReader<BM>::load_at(xt, aoff[mi], 16 * ks, 16 * ks + 4);
                        const u32x4 w = __builtin_bit_cast(u32x4, raw);
                        u32x4 o;
                        float part = 0.0f;
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            const float lo = bf16_lo_to_f32(w[d]) * sc[2 * d], hi = bf16_hi_to_f32(w[d]) * sc[2 * d + 1];
                            part += lo + hi;
                            o[d] = pack_bf16x2(lo, hi);
                        }
                        npart[mi] += part;
                        af[mi].v = __builtin_bit_cast(bf16x8, o);
                    }
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) bfr[ni].v = TFragReader<BN>::load_at(yt, boff[ni], 16 * ks, 16 * ks + 4);
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = E::mma(af[mi], bfr[ni], acc[mi][ni]);
                }
                // ---- the normaliser vector closes a chunk with its last piece
                if ((i + 1) % PPC == 0) {
                    const int kc = chunk_of(i);
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) {
                        const float t = npart[mi] + __shfl_xor(npart[mi], 32, 64);
                        npart[mi] = 0.0f;
                        if (with_n && g == 0)
                            a.nst[((long)bh * a.Nc + kc) * a.d1 + m0 + (wm * MI + mi) * 32 + l32] = nacc[mi];
                        nacc[mi] = ldsG[dd][wave][lane] * nacc[mi] + t;
                    }
                }
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
                    const int m = m0 + (wm * MI + mi) * 32 + acc_row(v, g);
                    const int n = n0 + (wn * NI + ni) * 32 + l32;
                    {
                    const long o = ((long)bh * a.d1 + m) * a.d2 + n;
                    if (a.Sfinal) a.Sfinal[o] = acc[mi][ni][v];
                    if (a.Sfinal2) a.Sfinal2[o] = acc[mi][ni][v];
                }
                }
    }
    if (with_n && g == 0 && a.nfinal) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) a.nfinal[(long)bh * a.d1 + m0 + (wm * MI + mi) * 32 + l32] = nacc[mi];
    }
}

}  // namespace tfla
