// bf16 fast path of the inter-chunk recurrent kernel (see recurrent.hip for what is computed).
//
//   state <- gbar_k * state + (rs (.) X_k)^T Y_k        (contraction over the rows of a chunk)
//
// A workgroup owns a 64 x (32 WN) tile of the state for the whole sequence and consumes the
// sequence in pieces of 64 rows.  Its 2 WN wavefronts have two roles that run side by side
// between the workgroup barriers (one barrier per piece):
//   * WN consumer wavefronts: wavefront c keeps the columns [32 c, 32 c + 32) of the tile in
//     MFMA accumulators, multiplies piece i into them, requests the Y part of piece
//     i + NS - 1 between its matrix instructions, and at chunk boundaries writes the state out
//     and applies the decay;
//   * WN producer wavefronts: they request the X part (and the scalars) of piece i + NS - 1
//     and rescale the X part of piece i + 1.
// Both operands are contracted over their row index, so both stay in their natural row-major
// layout in LDS and are read through the transposing LDS read.  X and Y pieces, the 64 row
// scales and gbar of the piece's chunk all arrive by asynchronous global->LDS loads in a ring
// of NS stages that runs across chunk boundaries, so the sequential dependence between chunks
// never drains the pipeline.
//
// The row scale is applied once per workgroup, not once per MFMA operand: every producer
// rescales, in place in LDS, exactly the 16-byte chunks of the X piece that it fetched itself
// (so its own load counter orders the two), and the barrier that hands the piece over
// publishes the scaled values to the consumers.
//
// Vector-memory operations of one wavefront retire in issue order on gfx9 (loads and stores
// share one counter), which is what lets the waits below name "operations younger than the
// piece I need" as a number.
#pragma once
#include "lds_tiles.h"
#include "tfla_internal.h"

namespace tfla {

#ifdef TFLA_TIMELINE
// development aid: phase timestamps of the first consumer and the first producer of workgroup 0,
// kept in LDS during the run (a global store would disturb the load counters being studied)
static __device__ unsigned long long tfla_rec_timeline[8192];
#define TFLA_RTL_DECL __shared__ unsigned long long tl_lds[2][128];
#ifndef TFLA_TL_BY
#define TFLA_TL_BY 0
#endif
#define TFLA_RTL(slot) if ((tid & 255) == 0 && blockIdx.x == 0 && blockIdx.y == TFLA_TL_BY && blockIdx.z == 0 && (slot) >= 0 && (slot) < 128) tl_lds[tid >> 8][(slot)] = __builtin_amdgcn_s_memtime()
#define TFLA_RTL_FLUSH __syncthreads(); if (blockIdx.x == 0 && blockIdx.y == TFLA_TL_BY && blockIdx.z == 0) for (int q_ = tid; q_ < 256; q_ += blockDim.x) tfla_rec_timeline[(q_ >> 7) * 4096 + (q_ & 127)] = tl_lds[q_ >> 7][q_ & 127];
#else
#define TFLA_RTL_DECL
#define TFLA_RTL(slot)
#define TFLA_RTL_FLUSH
#endif

template <int WN, int BK>
__global__ void __launch_bounds__(WN * 128) recurrent_kernel_bf16(RecArgs a) {
    using E = Elem<bf16_t>;
    using frag = E::frag;
    constexpr int NTP = WN * 64, BM = 64, BN = WN * 32, MI = 2, KS = BK / 16;
    constexpr int XB = BK * BM * 2, YB = BK * BN * 2, STAGE = XB + YB;
    constexpr int NS = BK == 64 ? 6 : 3;            // ring stages (the ring is 144 KB of LDS)
    constexpr int NH = NS - 3;                      // earlier iterations whose stores are younger than the awaited piece
    using DX = DmaTile<BK, BM, NTP, SWZ_T>;         // the producers' share of a piece
    using DY = DmaTile<BK, BN, NTP, SWZ_T>;
    constexpr int NX = DX::N;                       // 16-byte chunks of the X piece per producer lane
    constexpr int CPP = DX::N + BK / 64 + 1;        // loads per producer and piece (X, row scales, gbar)
    constexpr int CPC = DY::N;                      // loads per consumer and piece (Y)
    constexpr int NST = 4;                          // state stores per consumer at a chunk boundary
    constexpr int STEADY = (NS - 2) * CPP, STEADY_C = (NS - 2) * CPC;
    static_assert(STEADY + 2 * (NH + 1) <= 63 && STEADY_C + (NH + 1) * NST <= 63, "wait counts must fit the 6-bit counter");
    static_assert(CPC % KS == 0, "Y requests are spread evenly over the k steps");

    __shared__ __attribute__((aligned(1024))) char smem[NS * STAGE];
    __shared__ __attribute__((aligned(1024))) char stage_out[WN * 2048];        // per consumer: [32 n][32 m] bf16
    __shared__ __attribute__((aligned(256))) float ldsRs[NS][BK];
    __shared__ __attribute__((aligned(256))) float ldsG[NS][64];
    __shared__ __attribute__((aligned(256))) float ldsNx[2][WN][BM];            // column sums of scaled X, per producer
    TFLA_RTL_DECL

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= WN;
    const int wc = producer ? wave - WN : wave;     // consumer: column block; producer: index among producers
    const unsigned nwg = gridDim.x * gridDim.y * gridDim.z;
    unsigned wg = xcd_remap(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), nwg);
    // readfirstlane: tell the compiler these are wave-uniform, so that everything derived from them
    // lives in scalar registers
    const int bx = __builtin_amdgcn_readfirstlane((int)(wg % gridDim.x)); wg /= gridDim.x;
    const int by = __builtin_amdgcn_readfirstlane((int)(wg % gridDim.y));
    const int bh = __builtin_amdgcn_readfirstlane((int)(wg / gridDim.y));
    const int n0 = bx * BN, m0 = by * BM;
    const int PPC = a.L / BK, P = a.Nc * PPC;
    const uint32_t smem_a = lds_addr(smem), rs_a = lds_addr(ldsRs), g_a = lds_addr(ldsG);
    // the normaliser vector n (one value per state row) is kept by the workgroups bx == 0:
    // lane l of the first producer owns row m0 + l
    const bool with_n = (a.nst != nullptr) && bx == 0;

    if (producer) {
        // =============================== producers ===========================================
        // the wavefronts that feed the ring issue ahead of the consumer on their SIMD (1.5 % on the kernel)
        __builtin_amdgcn_s_setprio(3);
        const int ptid = tid - NTP;
        const bool n_owner = with_n && wc == 0;
        float nacc = (n_owner && a.n0) ? a.n0[(long)bh * a.d1 + m0 + lane] : 0.0f;
        // make the compiler wait for this plain load here: a wait that it places later, inside the
        // loop, would also wait for every global->LDS load in flight
        asm volatile("" : "+v"(nacc));
        float nsum[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) nsum[e] = 0.0f;
        DX dx; dx.init(a.d1, ptid);
        // Pieces are requested in order.  The addresses of the next piece to request advance
        // incrementally (no multiplication or division in the loop): 64 rows per piece; when the
        // recurrence runs backwards the chunks are visited last to first, rows inside a chunk still
        // ascending, so the step at a chunk's end is 64 - 2 L rows.
        const long row0 = a.reverse ? (long)(a.Nc - 1) * a.L : 0;
        const bf16_t* xreq = reinterpret_cast<const bf16_t*>(a.X) + ((long)bh * a.T + row0) * a.d1 + m0;
        const float* rsreq = a.rs + (long)bh * a.T + row0;
        const float* greq = a.gbar + (long)bh * a.Nc + (a.reverse ? a.Nc - 1 : 0);
        const long step_rows = BK, wrap_rows = a.reverse ? (long)BK - 2L * a.L : (long)BK;
        const long gstep = a.reverse ? -1 : 1;
        int lsub = 0, lslot = 0;
        uint32_t lst = smem_a;
        auto request = [&]() {
#pragma unroll
            for (int q = 0; q < DX::N; ++q) dma16(xreq, dx.goff[q], lst + (wc + q * WN) * 1024);
            // every producer fetches the same 64 row scales and gbar to the same place: identical
            // data, and each wavefront's own counter then covers what it reads
#pragma unroll
            for (int r = 0; r < BK / 64; ++r)
                dma4(rsreq + 64 * r, (uint32_t)lane * 4u, rs_a + (uint32_t)((lslot * BK + 64 * r) * 4));
            dma4(greq, 0u, g_a + (uint32_t)(lslot * 64 * 4));
            const bool wrap = ++lsub == PPC;
            const long dr = wrap ? wrap_rows : step_rows;
            xreq += dr * a.d1; rsreq += dr;
            if (wrap) { lsub = 0; greq += gstep; }
            if (++lslot == NS) { lslot = 0; lst = smem_a; } else lst += STAGE;
        };
        // Rescale, in place, this wave's own chunks of the X piece in `slot` (piece of chunk step
        // `stp`, last piece of its chunk if `closes`), after waiting until at most `pending` younger
        // operations of this wave are outstanding.
        auto rescale = [&](int slot, int stp, bool closes, int pending, int tl = -1) {
            if (pending == STEADY) wait_vmcnt<STEADY>();
            else wait_vmcnt_dyn(pending);
            TFLA_RTL(tl);
            char* xt = smem + slot * STAGE;
#pragma unroll
            for (int j = 0; j < NX; ++j) {
                const int cidx = (wc + j * WN) * 64 + lane;            // 16-byte chunk of the tile
                const float sc = ldsRs[slot][cidx >> 3];
                u32x4 w = *reinterpret_cast<const u32x4*>(xt + cidx * 16);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const float lo = bf16_lo_to_f32(w[d]) * sc, hi = bf16_hi_to_f32(w[d]) * sc;
                    if (with_n) { nsum[2 * d] += lo; nsum[2 * d + 1] += hi; }
                    w[d] = pack_bf16x2(lo, hi);
                }
                *reinterpret_cast<u32x4*>(xt + cidx * 16) = w;
            }
            // the piece that closes a chunk also closes the chunk's column sums
            if (with_n && closes) {
                // lanes whose chunks hold the same eight columns differ in lane bits 3 and 5, and in
                // bits 2 and 4 together (the swizzle moves a chunk by four positions on odd row pairs)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float s = nsum[e];
                    s += __shfl_xor(s, 20, 64);
                    s += __shfl_xor(s, 8, 64);
                    s += __shfl_xor(s, 32, 64);
                    nsum[e] = s;
                }
                if (lane < 8) {
                    float* dst = &ldsNx[stp & 1][wc][8 * lane];
#pragma unroll
                    for (int e = 0; e < 8; ++e) dst[e] = nsum[e];
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) nsum[e] = 0.0f;
            }
        };

        int requested = 0;
#pragma unroll
        for (int p = 0; p < NS - 1; ++p)
            if (p < P) { request(); ++requested; }
        rescale(0, 0, PPC == 1, (requested - 1) * CPP);

        // Iteration i (consumers multiply piece i): request piece i + NS - 1 into the slot of piece
        // i - 1, which the consumers have left; rescale piece i + 1.  (sub, step, slot) describe
        // piece i; sth[] counts this wave's stores of the NH previous iterations.
        int sub = 0, step = 0, slot = 0, sth[NH + 1] = {};
        for (int i = 0; i < P; ++i) {
            // the rescaled chunks (plain LDS writes) must have landed before the barrier hands them over
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            barrier_nofence();
            TFLA_RTL(4 * i);
            int st0 = 0;
            // normaliser vector: piece i closes its chunk, whose column sums every producer has just
            // published; emit n before that chunk, then apply the chunk
            if (n_owner && sub == PPC - 1) {
                const int kc = a.reverse ? a.Nc - 1 - step : step;
                // n before this chunk leaves as two bf16 rows of d1: the rounded value and the rounding
                // remainder (together good to 2^-17), the form in which the parallel kernel feeds it to the
                // matrix unit next to the state
                uint16_t* np = reinterpret_cast<uint16_t*>(a.nst) + ((long)bh * a.Nc + kc) * 2 * a.d1 + m0 + lane;
                const uint32_t nhi = bf16_bits_rne(nacc);
                np[0] = (uint16_t)nhi;
                np[a.d1] = (uint16_t)bf16_bits_rne(nacc - bf16_lo_to_f32(nhi));
                float s = 0.0f;
#pragma unroll
                for (int w = 0; w < WN; ++w) s += ldsNx[step & 1][w][lane];
                nacc = ldsG[slot][lane] * nacc + s;
                st0 = 2;
            }
            if (i + NS - 1 < P) request();
            TFLA_RTL(4 * i + 1);
            int sub1 = sub + 1, step1 = step, slot1 = slot + 1;
            if (sub1 == PPC) { sub1 = 0; ++step1; }
            if (slot1 == NS) slot1 = 0;
            if (i + 1 < P) {
                // younger than the loads of piece i + 1: the requests made after it and the stores
                // issued since (this iteration's and those of the NS - 3 iterations before)
                int ahead = P - 2 - i;
                ahead = ahead > NS - 2 ? NS - 2 : ahead;
                int pending = ahead * CPP + st0;
#pragma unroll
                for (int h = 0; h < NH; ++h) pending += sth[h];
                rescale(slot1, step1, sub1 == PPC - 1, pending, 4 * i + 3);
            }
            TFLA_RTL(4 * i + 2);
            sub = sub1; step = step1; slot = slot1;
#pragma unroll
            for (int h = NH; h > 0; --h) sth[h] = sth[h - 1];
            sth[0] = st0;
        }
        if (n_owner && a.nfinal) a.nfinal[(long)bh * a.d1 + m0 + lane] = nacc;
    } else {
        // =============================== consumers ===========================================
        f32x16 acc[MI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + mi * 32 + acc_row(v, g);
                const int n = n0 + wc * 32 + l32;
                acc[mi][v] = a.S0 ? a.S0[((long)bh * a.d1 + m) * a.d2 + n] : 0.0f;
            }
        // make the compiler wait for these plain loads here rather than inside the loop, where its
        // wait would also cover the state stores in flight
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(acc[mi][v]));
        TFragReader<BM> ra; ra.init(lane, 8);
        TFragReader<BN> rb; rb.init(lane, 8);
        uint32_t boff = rb.block_offset(wc);        // LDS byte offset of this wave's B column block
        // (the compiler may fetch this from a small table in memory: make it wait for that here, because a wait
        // that it places inside the loop would also wait for every global->LDS load in flight)
        asm volatile("" : "+v"(boff));
        // the consumers fetch the Y pieces (same order and address stepping as the producers' X)
        DY dy; dy.init(a.d2, tid);
        const long row0 = a.reverse ? (long)(a.Nc - 1) * a.L : 0;
        const bf16_t* yreq = reinterpret_cast<const bf16_t*>(a.Y) + ((long)bh * a.T + row0) * a.d2 + n0;
        const long step_rows = BK, wrap_rows = a.reverse ? (long)BK - 2L * a.L : (long)BK;
        int lsub = 0, lslot = 0;
        uint32_t lst = smem_a + XB;
        auto request_part = [&](int q) { dma16(yreq, dy.goff[q], lst + (wc + q * WN) * 1024); };
        auto request_end = [&]() {
            const bool wrap = ++lsub == PPC;
            yreq += (wrap ? wrap_rows : step_rows) * a.d2;
            if (wrap) lsub = 0;
            if (++lslot == NS) { lslot = 0; lst = smem_a + XB; } else lst += STAGE;
        };
        int requested = 0;
#pragma unroll
        for (int p = 0; p < NS - 1; ++p)
            if (p < P) {
#pragma unroll
                for (int q = 0; q < CPC; ++q) request_part(q);
                request_end();
                ++requested;
            }
        wait_vmcnt_dyn((requested - 1) * CPC);      // this wave's part of piece 0 has landed
        int sub = 0, step = 0, slot = 0, sth[NH + 1] = {};
        for (int i = 0; i < P; ++i) {
            barrier_nofence();
            TFLA_RTL(4 * i);
            int st0 = 0;
            const char* xt = smem + slot * STAGE;
            const char* yt = xt + XB;
            frag af[KS][MI], bfr[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) af[ks][mi].v = ra.load(xt, mi, 16 * ks, 16 * ks + 4);
                bfr[ks].v = TFragReader<BN>::load_at(yt, boff, 16 * ks, 16 * ks + 4);
            }
            // chunk boundary: emit the state before this chunk's update, then decay
            if (sub == 0) {
                const int kc = a.reverse ? a.Nc - 1 - step : step;
                if (a.stT) {
                    st0 = NST;
                    // through a private LDS tile [16 n][64 m] per half of the wave's 32 columns (16-byte chunks
                    // XOR-swizzled by the row) so that the state leaves in whole 128-byte lines
                    char* ot = stage_out + wc * 2048;
                    char* gdst = reinterpret_cast<char*>(a.stT) +
                                 ((((long)bh * a.Nc + kc) * a.d2 + n0 + wc * 32) * a.d1 + m0) * 2;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        if ((l32 >> 4) == h) {
                            const int n = l32 & 15;
#pragma unroll
                            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    uint2 w;
                                    w.x = pack_bf16x2(acc[mi][4 * j], acc[mi][4 * j + 1]);
                                    w.y = pack_bf16x2(acc[mi][4 * j + 2], acc[mi][4 * j + 3]);
                                    *reinterpret_cast<uint2*>(ot + n * 128 + (((4 * mi + j) ^ (n & 7)) * 16) + 8 * g) = w;
                                }
                        }
                        // (compiler-level ordering of the differently typed LDS accesses; the hardware runs
                        // one wavefront's LDS operations in order)
                        asm volatile("" ::: "memory");
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const int n = q * 8 + (lane >> 3), c = lane & 7;
                            const u32x4 w = *reinterpret_cast<const u32x4*>(ot + n * 128 + ((c ^ (n & 7)) * 16));
                            // (non-temporal: measured slightly faster for the tiled kernels that follow)
                            __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(gdst + ((long)(16 * h + n) * a.d1 + 8 * c) * 2));
                        }
                        asm volatile("" ::: "memory");
                    }
                }
                // Boundaries between the blocks of the forget-gate gradient scan (the state here is the one between
                // chunks kb - 1 and kb): the forward launch leaves an fp32 copy of its accumulators, the reversed
                // launch multiplies that copy with its own and leaves the partial inner product.
                if (a.anc || a.anc_in) {
                    const int kb = a.reverse ? kc + 1 : kc;
                    if (kb % a.anc_G == 0 && kb > 0 && kb < a.Nc) {
                        const long per = (long)a.d1 * a.d2;
                        const int nslot = (a.Nc + a.anc_G - 1) / a.anc_G;
                        const int part = (by * (int)gridDim.x + bx) * WN + wc;
                        const long off = ((long)bh * nslot + kb / a.anc_G) * per + ((long)part * (MI * 4) * 64 + lane) * 4;
                        if (a.anc) {
                            st0 += MI * 4;
#pragma unroll
                            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const f32x4 w = {acc[mi][4 * j], acc[mi][4 * j + 1], acc[mi][4 * j + 2], acc[mi][4 * j + 3]};
                                    // (read again only by the reversed launch, much later: non-temporal)
                                    __builtin_nontemporal_store(w, reinterpret_cast<f32x4*>(a.anc + off + (long)(mi * 4 + j) * 256));
                                }
                        }
                        if (a.anc_in) {
                            f32x4 c[MI * 4];
#pragma unroll
                            for (int q = 0; q < MI * 4; ++q) c[q] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.anc_in + off + (long)q * 256));
                            float dot = 0.0f;
#pragma unroll
                            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                                for (int j = 0; j < 4; ++j)
#pragma unroll
                                    for (int e = 0; e < 4; ++e) dot += acc[mi][4 * j + e] * c[mi * 4 + j][e];
                            // Everything this wavefront has in flight has landed once these plain loads have (the
                            // compiler's own wait for them may or may not say so; this one does).  Operations from
                            // before this point can then never be younger than a piece that is still awaited, so the
                            // wait counts below stay valid without knowing about the loads.
                            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                            dot = wave_sum(dot);
                            if (lane == 0) a.anc_part[((long)bh * nslot + kb / a.anc_G) * (gridDim.x * gridDim.y * WN) + part] = dot;
                            st0 += 1;
                        }
                        asm volatile("" ::: "memory");
                    }
                }
                const float gb = ldsG[slot][lane];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mi][v] *= gb;
            }
            TFLA_RTL(4 * i + 1);
            // the Y part of piece i + NS - 1 (into the slot of piece i - 1, which every consumer has
            // left) is requested between the matrix instructions
            const bool req = i + NS - 1 < P;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) acc[mi] = E::mma(af[ks][mi], bfr[ks], acc[mi]);
                if (req) {
#pragma unroll
                    for (int q = ks * CPC / KS; q < (ks + 1) * CPC / KS; ++q) request_part(q);
                }
            }
            if (req) request_end();
            TFLA_RTL(4 * i + 2);
            // this wave's part of Y of piece i + 1 must have landed before the next barrier; younger
            // than it are the requests made after it and the stores of this and the NH previous
            // iterations
            if (i + 1 < P) {
                int ahead = P - 2 - i;
                ahead = ahead > NS - 2 ? NS - 2 : ahead;
                int pending = ahead * CPC + st0;
#pragma unroll
                for (int h = 0; h < NH; ++h) pending += sth[h];
                if (pending == STEADY_C) wait_vmcnt<STEADY_C>();
                else if (pending == STEADY_C + NST) wait_vmcnt<STEADY_C + NST>();
                else wait_vmcnt_dyn(pending);
            }
#pragma unroll
            for (int h = NH; h > 0; --h) sth[h] = sth[h - 1];
            sth[0] = st0;
            if (++sub == PPC) { sub = 0; ++step; }
            if (++slot == NS) slot = 0;
        }
        if (a.Sfinal || a.Sfinal2) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + mi * 32 + acc_row(v, g);
                    const int n = n0 + wc * 32 + l32;
                    const long o = ((long)bh * a.d1 + m) * a.d2 + n;
                    if (a.Sfinal) a.Sfinal[o] = acc[mi][v];
                    if (a.Sfinal2) a.Sfinal2[o] = acc[mi][v];
                }
        }
    }
    TFLA_RTL_FLUSH
}

}  // namespace tfla
