// bf16 fast path of the inter-chunk recurrent kernel (see recurrent.hip for what is computed).
//
//   state <- gbar_k * state + (rs (.) X_k)^T Y_k        (contraction over the rows of a chunk)
//
// A workgroup of WN wavefronts owns a 64 x (32 NI WN) tile of the state for the whole sequence;
// wavefront w keeps the columns [32 NI w, 32 NI (w+1)) in MFMA accumulators.  The sequence is
// consumed in pieces of 64 rows.  Both operands are contracted over their row index, so both
// stay in their natural row-major layout in LDS and are read through the transposing LDS
// read.  X and Y pieces, the 64 row scales and gbar of the piece's chunk all arrive by
// asynchronous global->LDS loads in a ring of NS stages that runs across chunk boundaries, so
// the sequential dependence between chunks never drains the pipeline.
//
// The row scale is applied once per workgroup, not once per MFMA operand: one piece ahead of
// the multiplication every wavefront rescales, in place in LDS, exactly the 16-byte chunks of
// the X piece that it fetched itself (so its own load counter orders the two), and the
// workgroup barrier that hands the piece over publishes the scaled values to the others.
//
// Vector-memory operations of one wavefront retire in issue order on gfx9 (loads and stores
// share one counter), which is what lets the waits below name "operations younger than the
// piece I need" as a number.
#pragma once
#include "lds_tiles.h"
#include "tfla_internal.h"

namespace tfla {

#ifdef TFLA_TIMELINE
static __device__ unsigned long long tfla_rec_timeline[8192];
#define TFLA_RTL(slot) if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && (slot) >= 0 && (slot) < 8192) tfla_rec_timeline[(slot)] = __builtin_amdgcn_s_memtime()
#else
#define TFLA_RTL(slot)
#endif

template <int WN, int NI>
__global__ void __launch_bounds__(WN * 64, 2) recurrent_kernel_bf16(RecArgs a) {
    using E = Elem<bf16_t>;
    using frag = E::frag;
    constexpr int NT = WN * 64, BM = 64, BN = WN * 32 * NI, BK = 64, MI = 2;
    constexpr int XB = BK * BM * 2, YB = BK * BN * 2, STAGE = XB + YB;
    constexpr int NS = 5;
    using DX = DmaTile<BK, BM, NT, SWZ_T>;
    using DY = DmaTile<BK, BN, NT, SWZ_T>;
    constexpr int NX = DX::N;                       // 16-byte chunks of the X piece per lane
    constexpr int CPP = DX::N + DY::N + 2;          // loads per wave and piece (X, Y, row scales, gbar)
    constexpr int NST = 4 * NI;                     // state stores per wave at a chunk boundary
    static_assert((NS - 2) * CPP + 3 * (NST + 1) <= 63, "wait counts must fit the 6-bit counter");

    __shared__ __attribute__((aligned(1024))) char smem[NS * STAGE];
    __shared__ __attribute__((aligned(1024))) char stage_out[WN * NI * 4096];   // per wave and block: [32 n][64 m] bf16
    __shared__ __attribute__((aligned(256))) float ldsRs[NS][BK];
    __shared__ __attribute__((aligned(256))) float ldsG[NS][64];
    __shared__ __attribute__((aligned(256))) float ldsNx[2][WN][BM];            // column sums of scaled X, per wave

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned nwg = gridDim.x * gridDim.y * gridDim.z;
    unsigned wg = xcd_remap(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), nwg);
    // readfirstlane: tell the compiler these are wave-uniform, so that everything derived from them
    // lives in scalar registers
    const int bx = __builtin_amdgcn_readfirstlane((int)(wg % gridDim.x)); wg /= gridDim.x;
    const int by = __builtin_amdgcn_readfirstlane((int)(wg % gridDim.y));
    const int bh = __builtin_amdgcn_readfirstlane((int)(wg / gridDim.y));
    const int n0 = bx * BN, m0 = by * BM;
    const bf16_t* X = reinterpret_cast<const bf16_t*>(a.X) + (long)bh * a.T * a.d1 + m0;
    const bf16_t* Y = reinterpret_cast<const bf16_t*>(a.Y) + (long)bh * a.T * a.d2 + n0;
    const float* rs = a.rs + (long)bh * a.T;
    // the normaliser vector n (one value per state row) is kept by the workgroups bx == 0:
    // lane l of wavefront 0 owns row m0 + l
    const bool with_n = (a.nst != nullptr) && bx == 0;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + mi * 32 + acc_row(v, g);
                const int n = n0 + (wave * NI + ni) * 32 + l32;
                acc[mi][ni][v] = a.S0 ? a.S0[((long)bh * a.d1 + m) * a.d2 + n] : 0.0f;
            }
    float nacc = (with_n && a.n0 && wave == 0) ? a.n0[(long)bh * a.d1 + m0 + lane] : 0.0f;
    // make the compiler wait for these plain loads here: a wait that it places later, inside the
    // loop, would also wait for every global->LDS load in flight
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(acc[mi][ni][v]));
    asm volatile("" : "+v"(nacc));
    float nsum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) nsum[e] = 0.0f;

    const int PPC = a.L / BK, P = a.Nc * PPC;

    DX dx; dx.init(a.d1, tid);
    DY dy; dy.init(a.d2, tid);
    const uint32_t smem_a = lds_addr(smem), rs_a = lds_addr(ldsRs), g_a = lds_addr(ldsG);
    // Pieces are requested in order; (lstep, lsub) = (chunk step, piece within the chunk) of the next
    // one, kept incrementally (no integer division in the loop).  Chunk step c visits chunk c, or
    // chunk Nc - 1 - c when the recurrence runs backwards.  A request is CPP loads; they can be
    // issued one at a time so that they interleave with the matrix instructions.
    int lstep = 0, lsub = 0, lslot = 0;
    long ltr = 0;
    int lkc = 0;
    auto request_begin = [&]() {
        lkc = a.reverse ? a.Nc - 1 - lstep : lstep;
        ltr = (long)lkc * a.L + (long)lsub * BK;
    };
    auto request_part = [&](int q) {      // q is a compile-time value in every caller
        const uint32_t st = smem_a + (uint32_t)lslot * STAGE;
        if (q < DX::N) dma16(X + ltr * a.d1, dx.goff[q], st + (wave + q * WN) * 1024);
        else if (q < DX::N + DY::N) dma16(Y + ltr * a.d2, dy.goff[q - DX::N], st + XB + (wave + (q - DX::N) * WN) * 1024);
        // every wavefront fetches the same 64 row scales and gbar to the same place: identical
        // data, and each wavefront's own counter then covers what it reads
        else if (q == DX::N + DY::N) dma4(rs + ltr, (uint32_t)lane * 4u, rs_a + (uint32_t)(lslot * BK * 4));
        else dma4(a.gbar + (long)bh * a.Nc + lkc, 0u, g_a + (uint32_t)(lslot * 64 * 4));
    };
    auto request_end = [&]() {
        if (++lsub == PPC) { lsub = 0; ++lstep; }
        if (++lslot == NS) lslot = 0;
    };
    const bool n_owner = with_n && wave == 0;

    TFragReader<BM> ra; ra.init(lane, 8);
    TFragReader<BN> rb; rb.init(lane, 8);
    uint32_t boff[NI];                 // LDS byte offsets of this wave's B column blocks
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) boff[ni] = rb.block_offset(wave * NI + ni);

    // Rescale, in place, this wave's own chunks of the X piece in `slot` (piece of chunk step `stp`,
    // last piece of its chunk if `closes`), after waiting until at most `pending` younger operations
    // of this wave are outstanding.
    auto rescale = [&](int slot, int stp, bool closes, int pending, int tl) {
        wait_vmcnt_dyn(pending);
        TFLA_RTL(4096 + tl);
        char* xt = smem + slot * STAGE;
#pragma unroll
        for (int j = 0; j < NX; ++j) {
            const int cidx = (wave + j * WN) * 64 + lane;          // 16-byte chunk of the tile
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
                float* dst = &ldsNx[stp & 1][wave][8 * lane];
#pragma unroll
                for (int e = 0; e < 8; ++e) dst[e] = nsum[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) nsum[e] = 0.0f;
        }
    };

    wait_vmcnt<0>();
    int requested = 0;
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < P) {
            request_begin();
#pragma unroll
            for (int q = 0; q < CPP; ++q) request_part(q);
            request_end();
            ++requested;
        }
    rescale(0, 0, PPC == 1, (requested - 1) * CPP, 4095);

    // Iteration i multiplies piece i, requests piece i + NS - 1 and rescales piece i + 1.
    // (sub, step, slot) describe piece i; st1, st2 count the stores of the two previous iterations.
    int sub = 0, step = 0, slot = 0;
    int st1 = 0, st2 = 0;
    for (int i = 0; i < P; ++i) {
        TFLA_RTL(4 * i);
        // the rescaled chunks (plain LDS writes) must have landed before the barrier hands them over
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        barrier_nofence();
        TFLA_RTL(4 * i + 1);
        int st0 = 0;
        const int kc = a.reverse ? a.Nc - 1 - step : step;
        // ---- normaliser vector: piece i closes its chunk, whose column sums every wave has just
        // published; emit n before that chunk, then apply the chunk
        if (n_owner && sub == PPC - 1) {
            a.nst[((long)bh * a.Nc + kc) * a.d1 + m0 + lane] = nacc;
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < WN; ++w) s += ldsNx[step & 1][w][lane];
            nacc = ldsG[slot][lane] * nacc + s;
            st0 += 1;
        }
        // ---- chunk boundary: emit the state before this chunk's update, then decay
        if (sub == 0) {
            const long st_slot = (long)bh * a.Nc + kc;
            if (a.stT) {
                st0 += NST;
                // through a private LDS tile [32 n][64 m] (16-byte chunks XOR-swizzled by n) so that
                // the state leaves in full 128-byte rows
                char* gdst = reinterpret_cast<char*>(a.stT) + (st_slot * a.d1 * a.d2) * 2;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    char* ot = stage_out + (wave * NI + ni) * 4096;
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            uint2 w;
                            w.x = pack_bf16x2(acc[mi][ni][4 * j], acc[mi][ni][4 * j + 1]);
                            w.y = pack_bf16x2(acc[mi][ni][4 * j + 2], acc[mi][ni][4 * j + 3]);
                            *reinterpret_cast<uint2*>(ot + l32 * 128 + (((4 * mi + j) ^ (l32 & 7)) * 16) + 8 * g) = w;
                        }
                    const int nb = n0 + (wave * NI + ni) * 32;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = q * 8 + (lane >> 3), c = lane & 7;
                        const u32x4 w = *reinterpret_cast<const u32x4*>(ot + n * 128 + ((c ^ (n & 7)) * 16));
                        *reinterpret_cast<u32x4*>(gdst + ((long)(nb + n) * a.d1 + m0 + 8 * c) * 2) = w;
                    }
                }
            }
            const float gb = ldsG[slot][lane];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mi][ni][v] *= gb;
        }
        TFLA_RTL(4 * i + 2);
        // ---- multiply piece i; the request for piece i + NS - 1 (into the slot of piece i - 1, which
        // every wave has left) is issued between the matrix instructions
        const char* xt = smem + slot * STAGE;
        const char* yt = xt + XB;
        constexpr int KS = BK / 16;
        frag af[KS][MI], bfr[KS][NI];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) af[ks][mi].v = ra.load(xt, mi, 16 * ks, 16 * ks + 4);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) bfr[ks][ni].v = TFragReader<BN>::load_at(yt, boff[ni], 16 * ks, 16 * ks + 4);
        }
        const bool req = i + NS - 1 < P;
        if (req) request_begin();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = E::mma(af[ks][mi], bfr[ks][ni], acc[mi][ni]);
            if (req) {
#pragma unroll
                for (int q = ks * CPP / KS; q < (ks + 1) * CPP / KS; ++q) request_part(q);
            }
        }
        if (req) request_end();
        TFLA_RTL(4 * i + 3);
        // ---- piece i + 1: wait for this wave's own loads of it, rescale this wave's chunks of X.
        // Younger than those loads are the requests made after it and the stores of this and the
        // two previous iterations.
        int sub1 = sub + 1, step1 = step, slot1 = slot + 1;
        if (sub1 == PPC) { sub1 = 0; ++step1; }
        if (slot1 == NS) slot1 = 0;
        if (i + 1 < P) {
            int ahead = P - 2 - i;
            ahead = ahead > NS - 2 ? NS - 2 : ahead;
            rescale(slot1, step1, sub1 == PPC - 1, ahead * CPP + st0 + st1 + st2, i);
        }
        sub = sub1; step = step1; slot = slot1;
        st2 = st1; st1 = st0;
    }
    // ---- final state
    if (a.Sfinal || a.Sfinal2) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = m0 + mi * 32 + acc_row(v, g);
                    const int n = n0 + (wave * NI + ni) * 32 + l32;
                    const long o = ((long)bh * a.d1 + m) * a.d2 + n;
                    if (a.Sfinal) a.Sfinal[o] = acc[mi][ni][v];
                    if (a.Sfinal2) a.Sfinal2[o] = acc[mi][ni][v];
                }
    }
    if (n_owner && a.nfinal) a.nfinal[(long)bh * a.d1 + m0 + lane] = nacc;
}

}  // namespace tfla
