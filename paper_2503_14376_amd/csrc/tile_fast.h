// bf16 fast path of the intra-chunk tiled kernels (see tile.hip for what is computed).
//
// Every operand tile reaches LDS through asynchronous global->LDS loads in a ring of NS
// stages; nothing is staged through registers and no VALU work is spent on data movement.
// Column tiles are BC = 32 wide.  Per stage: Y tile [32][D1] (k-contiguous fragments) and
// Z tile [32][BD2] (read through the transposing LDS read, because its contraction index is
// the row index); the inter-chunk state is streamed through the same ring in [BD2][BCS]
// slices before the column tiles.
#pragma once
#include <type_traits>

#include "lds_tiles.h"
#include "tfla_internal.h"


namespace tfla {

// Development aid, compiled only with -DTFLA_TIMELINE: wave 0 of every workgroup records the
// shader clock at phase boundaries.
#ifdef TFLA_TIMELINE
static __device__ unsigned long long tfla_timeline[1 << 18];
#define TFLA_TL(k)                                                                                         \
    if (tid == 0)                                                                                          \
    tfla_timeline[((blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z)) * 8 + (k)) & ((1 << 18) - 1)] = \
        __builtin_amdgcn_s_memtime()
#else
#define TFLA_TL(k)
#endif

// Order of the first NXS + NKS ring items of a workgroup: the slices of its own X rows ([BR][BXS], read into registers)
// and the slices of the inter-chunk state ([BD2][BCS] or transposed), interleaved so that every X slice arrives just
// before the first state slice whose products need it.  The matrix work then starts after one X slice instead of
// after all of them, and the later X slices load behind the products of the earlier state slices.
// pre_item(item, BXS, BCS) returns 2 * index + 1 for the X slice `index`, 2 * index for the state slice `index`
// (closed forms, so that they fold for every unrolled item).
__host__ __device__ constexpr int pre_item(int item, int BXS, int BCS) {
    if (BXS >= BCS) {                       // one X slice, then the BXS / BCS state slices it covers
        const int R = BXS / BCS, grp = item / (R + 1), w = item % (R + 1);
        return w == 0 ? 2 * grp + 1 : 2 * (grp * R + w - 1);
    }
    const int Q = BCS / BXS, grp = item / (Q + 1), w = item % (Q + 1);   // the Q X slices of a state slice, then it
    return w < Q ? 2 * (grp * Q + w) + 1 : 2 * grp;
}

// SPLIT: 0 = the whole contraction over D1 in this launch; 1 / 2 = the first / second 512-wide half of a
// contraction over 1024 columns (rows of the D1-wide operands are 2 D1 apart): the first half stores its raw fp32
// accumulators, the second adds them to its own before the epilogue.
// NOE: 1 = the dQ kernel does not store the weighted matrix E and the dK kernel recomputes it from dH and V
// like every other mode (narrow contractions: E, L x L per chunk, is then more bytes than the operands it replaces).
// PADOUT: 1 = the kernel runs on a zero-padded copy of the problem and stores only the true steps and columns,
// straight into the caller's tensor (TileArgs::out_T, out_ld, out_cols); 0 = whole blocks, nothing padded.
// FUSE: 1 = MODE_H also stores the layer output y = sigma(o~) (.) NORM(h~) (Sec. 2.1, hidden-state output equation) of
// its rows; the column block covers all of d2 (the launcher checks), nothing is padded.
template <int D1, int BD2, int NW, int MODE, int OCC, int SPLIT = 0, int NOE = 0, int PADOUT = 0, int FUSE = 0>
__global__ void __launch_bounds__(NW * 64, OCC) tile_kernel_bf16(TileArgs a) {
    static_assert(!FUSE || (MODE == MODE_H && SPLIT == 0 && !PADOUT), "the fused layer output belongs to the plain H kernel");
    using E = Elem<bf16_t>;
    using frag = E::frag;
    constexpr bool UPPER = (MODE & 1) != 0;
    constexpr bool STT = (MODE == MODE_DQ || MODE == MODE_DK);   // state slices are contraction-major
    constexpr bool ELITE = MODE == MODE_DK && !NOE;              // column tiles carry E instead of Y
    constexpr bool EWRITE = MODE == MODE_DQ && !NOE;
    constexpr int NT = NW * 64, BR = NW * 32, BC = 32;
    constexpr int KS1 = D1 / 16, NB = BD2 / 32;
    constexpr int YB = ELITE ? BC * BR * 2 : BC * D1 * 2, ZB = BC * BD2 * 2;         // bytes
    constexpr int XSMIN = BR * (D1 < 128 ? D1 : 128) * 2;       // room for wide X slices when the tiles are small
    constexpr int STAGE = (ELITE && YB + ZB < XSMIN) ? XSMIN : YB + ZB;
    constexpr int ESTG = EWRITE ? NW * 2048 : 0;                // per-wave staging of E tiles
    // LDS budget of one workgroup: 160 KB shared by OCC resident workgroups, minus the small arrays
    constexpr int BUDGET = (OCC >= 2 ? 80 : 160) * 1024 - 6144 - ESTG;
    constexpr int NS = STAGE * 4 <= BUDGET ? 4 : (STAGE * 3 <= BUDGET ? 3 : 2);
    static_assert(NS * STAGE <= BUDGET, "ring does not fit");
    constexpr int BCS_RAW = STAGE / (BD2 * 2);
    constexpr int BCS = BCS_RAW >= 64 ? 64 : 32;                                    // state slice width
    constexpr int NKS = D1 / BCS;
    // the workgroup's rows of X arrive in [BR][BXS] slices
    constexpr int BXS_RAW = STAGE / (BR * 2);
    constexpr int BXS = BXS_RAW >= 128 ? 128 : (BXS_RAW >= 64 ? 64 : 32);
    constexpr int NXS = D1 / BXS, NPRE = NXS + NKS;
    static_assert(BR * BXS * 2 <= STAGE && BXS <= D1 && D1 % BXS == 0, "X slice must fit a stage");
    static_assert(BD2 * BCS * 2 <= STAGE && BCS <= 64 && D1 % BCS == 0, "state slice must fit a stage");

    // after the loops the ring's memory holds the output block (and the dot operand) of each wave
    constexpr bool WTILE = MODE == MODE_DQ || MODE == MODE_DK || FUSE;   // the epilogue reads a second per-wave tile
    constexpr int EPI = (WTILE ? 2 : 1) * NW * 32 * BD2 * 2;
    constexpr int SMEM = NS * STAGE > EPI ? NS * STAGE : EPI;
    static_assert(SMEM <= BUDGET, "LDS budget");
    // The epilogue's per-wave tiles ([32][BD2] bf16: the output block on its way out and, for dQ / dK, the wave's rows
    // of the dot operand -- for the fused layer output, of the gate pre-activations) live in slots of the ring's memory.  Slots are numbered from the stage after the one that
    // holds the last ring item: the first (NS - 1) SPS of them are free while that item is being multiplied, so the dot
    // operand (slots 0 .. NW-1) is requested then and its latency hides behind the last tile; the output tiles take
    // the slots NW .. 2 NW - 1 once every wave has left the ring.
    constexpr int SLOT = 32 * BD2 * 2, SPS = STAGE / SLOT >= 1 ? STAGE / SLOT : 1;
    // (not where a slot is larger than a stage, and not in the first half of a split contraction, which has no epilogue)
    constexpr bool WPRE = WTILE && SPLIT != 1 && STAGE >= SLOT && (NS - 1) * SPS >= NW && NS * SPS >= 2 * NW;
    __shared__ __attribute__((aligned(1024))) char smem[SMEM];
    __shared__ __attribute__((aligned(1024))) char ldsE[EWRITE ? ESTG : 16];
    __shared__ __attribute__((aligned(256))) float ldsW[NS][NW][64];   // column weights of a tile, one copy per wave
    // per-row scalars of each wave's 32 rows (two copies side by side), fetched like the tiles
    __shared__ __attribute__((aligned(256))) float ldsS[NW][64];    // inter-chunk row scale
    __shared__ __attribute__((aligned(256))) float ldsWr[NW][64];   // row term of the weights
    __shared__ __attribute__((aligned(256))) float ldsM[(MODE == MODE_H) ? NW : 1][64];  // max state (mLSTMexp forward)
    __shared__ __attribute__((aligned(256))) float ldsN[(MODE == MODE_H) ? D1 : 64];     // n_{k-1}

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    TFLA_TL(0);
    // one-dimensional launch (the number of workgroups can exceed what the y and z grid dimensions hold):
    // linear id -> (column block, row block, chunk, batch*head), column blocks fastest
    const unsigned nwg = gridDim.x, gx = (unsigned)a.d2 / BD2, gy = (unsigned)a.L / (32 * NW);
    unsigned wg = xcd_remap(blockIdx.x, nwg);
    // quotient and remainder by a divisor whose log2 the launcher supplies when it has one
    auto divmod = [](unsigned n, unsigned d, int sh, unsigned& rem) {
        const unsigned q = sh >= 0 ? n >> sh : n / d;
        rem = n - q * d;
        return q;
    };
    unsigned rem;
    wg = divmod(wg, gx, a.sh_gx, rem);
    const int nb2 = __builtin_amdgcn_readfirstlane((int)rem);
    wg = divmod(wg, gy, a.sh_gy, rem);
    const int rbi = __builtin_amdgcn_readfirstlane((int)rem);
    const int rb = UPPER ? rbi : (int)gy - 1 - rbi;      // row blocks with more column tiles first
    // Order in time: every XCD walks the chunks of its own (batch, head) slices together, chunk by chunk, in
    // the direction a.kc_desc gives (the launcher's choice, by measurement).
    // bpx = slices per XCD (the XCD's contiguous range of ids then covers exactly its slices)
    const unsigned bhn = (unsigned)a.dec_bh, bpx = (unsigned)a.dec_bpx;
    wg = divmod(wg, bpx, a.sh_bpx, rem);
    const unsigned bl = rem;
    wg = divmod(wg, (unsigned)a.Nc, a.sh_nc, rem);
    const int kci = __builtin_amdgcn_readfirstlane((int)rem);
    const int kc = a.kc_desc ? a.Nc - 1 - kci : kci;
    const int bh = __builtin_amdgcn_readfirstlane((int)(wg * bpx + bl));
    const long tbase = (long)bh * a.T + (long)kc * a.L;
    const int r0 = rb * BR, wr0 = r0 + wave * 32;
    const int d2 = a.d2;
    constexpr int ld1 = SPLIT ? 2 * D1 : D1;    // row stride of the operands with D1 columns

    const bf16_t* X = reinterpret_cast<const bf16_t*>(a.X);
    const bf16_t* Y = reinterpret_cast<const bf16_t*>(a.Y) + tbase * ld1;
    const bf16_t* Z = reinterpret_cast<const bf16_t*>(a.Z) + tbase * d2 + (long)nb2 * BD2;
    const bf16_t* St = reinterpret_cast<const bf16_t*>(a.St) +
                       (STT ? ((long)bh * a.Nc + kc) * ld1 * d2 + (long)nb2 * BD2
                            : (((long)bh * a.Nc + kc) * d2 + (long)nb2 * BD2) * ld1);

    const int ct_lo = UPPER ? r0 / BC : 0;
    const int ct_hi = UPPER ? a.L / BC : (r0 + BR) / BC;
    const int NI = NPRE + (ct_hi - ct_lo);                      // items streamed through the ring

    using DS = typename std::conditional<STT, DmaTile<BCS, BD2, NT, SWZ_T>, DmaTile<BD2, BCS, NT, SWZ_K>>::type;
    DS ds;  ds.init(STT ? d2 : ld1, tid);
    using DYT = typename std::conditional<ELITE, DmaTile<BC, BR, NT, SWZ_T>, DmaTile<BC, D1, NT, SWZ_K>>::type;
    DYT dy;    dy.init(ELITE ? a.L : ld1, tid);
    DmaTile<BC, BD2, NT, SWZ_T> dz;   dz.init(d2, tid);
    // E of this chunk: (L, L), rows = query index; the dK kernel reads the columns of its own rows
    const bf16_t* Eb = reinterpret_cast<const bf16_t*>(a.E) + ((long)bh * a.Nc + kc) * a.L * a.L + (ELITE ? r0 : 0);
    constexpr int CS = DS::N;
    DmaTile<BR, BXS, NT, SWZ_K> dxs;  dxs.init(ld1, tid);
    constexpr int CX = DmaTile<BR, BXS, NT, SWZ_K>::N;
    const bf16_t* Xb = X + (tbase + r0) * ld1;
    constexpr int CT = DYT::N + DmaTile<BC, BD2, NT, SWZ_T>::N + (ELITE ? 0 : 1);
    const uint32_t smem_a = lds_addr(smem), w_a = lds_addr(ldsW);
    const float* wcol = a.wcol + tbase;

    auto issue = [&](int item) {
        const uint32_t st = smem_a + (uint32_t)(item % NS) * STAGE;
        if (item < NPRE) {
            const int pi = pre_item(item, BXS, BCS), sl = pi >> 1;
            if (pi & 1) {
                // the workgroup's own rows: no other workgroup reads them when its block covers all output columns
                if (gx == 1) dxs.template issue<true>(Xb + sl * BXS, st, tid);
                else dxs.issue(Xb + sl * BXS, st, tid);
            } else {
                // (state slices of the dQ / dK kernels carry the hint too: measured, -3 us on dQ)
                ds.template issue<STT>(St + (STT ? (long)sl * BCS * d2 : (long)sl * BCS), st, tid);
            }
        } else {
            const int ct = ct_lo + item - NPRE;
            if (ELITE) {
                // (E of this workgroup's rows: read by this workgroup only)
                dy.template issue<true>(Eb + (long)ct * BC * a.L, st, tid);
                dz.issue(Z + (long)ct * BC * d2, st + YB, tid);
            } else {
                dy.issue(Y + (long)ct * BC * ld1, st, tid);
                dz.issue(Z + (long)ct * BC * d2, st + YB, tid);
                // the tile's 32 column weights (both half-waves fetch the same 32 floats)
                dma4(wcol + ct * BC, (uint32_t)(lane & 31) * 4u, w_a + (uint32_t)(((item % NS) * NW + wave) * 256));
            }
        }
    };
    // the same, spread over `nparts` calls that are placed between matrix instructions
    auto issue_part = [&](int item, int part, int nparts) {
        const uint32_t st = smem_a + (uint32_t)(item % NS) * STAGE;
        if (item < NPRE) {
            const int pi = pre_item(item, BXS, BCS), sl = pi >> 1;
            if (pi & 1) {
                if (gx == 1) dxs.template issue_part<true>(Xb + sl * BXS, st, tid, part, nparts);
                else dxs.issue_part(Xb + sl * BXS, st, tid, part, nparts);
            } else {
                ds.template issue_part<STT>(St + (STT ? (long)sl * BCS * d2 : (long)sl * BCS), st, tid, part, nparts);
            }
        } else {
            const int ct = ct_lo + item - NPRE;
            if (ELITE) {
                dy.template issue_part<true>(Eb + (long)ct * BC * a.L, st, tid, part, nparts);
                dz.issue_part(Z + (long)ct * BC * d2, st + YB, tid, part, nparts);
            } else {
                dy.issue_part(Y + (long)ct * BC * ld1, st, tid, part, nparts);
                dz.issue_part(Z + (long)ct * BC * d2, st + YB, tid, part, nparts);
                if (part == 0)
                    dma4(wcol + ct * BC, (uint32_t)(lane & 31) * 4u, w_a + (uint32_t)(((item % NS) * NW + wave) * 256));
            }
        }
    };
    // loads of this wave issued after those of item i and still allowed in flight while waiting for i
    auto pending_after = [&](int i) {
        int p = 0;
#pragma unroll
        for (int j = 1; j <= NS - 2; ++j)
            if (i + j < NI) p += (i + j < NPRE) ? ((pre_item(i + j, BXS, BCS) & 1) ? CX : CS) : CT;
        return p;
    };

    // per-row scalars of the workgroup's rows, issued before the ring so that, loads retiring in
    // order, they have landed once the first ring item has
    {
        const uint32_t vo = (uint32_t)(lane & 31) * 4u;
        dma4(a.srow + tbase + wr0, vo, lds_addr(&ldsS[wave][0]));
        dma4(a.wrow + tbase + wr0, vo, lds_addr(&ldsWr[wave][0]));
        if (MODE == MODE_H) {
            if (a.variant == 0) {
                dma4(a.mout + tbase + wr0, vo, lds_addr(&ldsM[wave][0]));
                // n_{k-1}: two bf16 rows (rounded value, rounding remainder) of ld1 columns per chunk; the rows
                // are contiguous when this launch covers all their columns
                const char* nsrc = reinterpret_cast<const char*>(a.nstate) + ((long)bh * a.Nc + kc) * ld1 * 4;
                if constexpr (SPLIT == 0) {
                    for (int c = wave; c < D1 / 64; c += NW)
                        dma4(nsrc + 256 * c, (uint32_t)lane * 4u, lds_addr(ldsN) + 256u * c);
                } else {
                    constexpr int PR = D1 / 128;        // 256-byte loads per row
                    for (int c = wave; c < 2 * PR; c += NW) {
                        const int r = c / PR, cc = c % PR;
                        dma4(nsrc + (long)r * ld1 * 2 + 256 * cc, (uint32_t)lane * 4u,
                             lds_addr(ldsN) + (uint32_t)(r * D1 * 2 + 256 * cc));
                    }
                }
            }
        }
    }
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < NI) issue(p);
    TFLA_TL(1);

    // ---------------- the workgroup's X rows (fragments of the wavefront's 32 rows: lane = row l32, k-group g) and the
    // inter-chunk part acc = X_r St, slice by slice in the order pre_item() gives
    static_assert(BXS >= BCS ? (BXS % BCS == 0) : (BCS % BXS == 0), "slice widths nest");
    frag xf[KS1];
    KFragReader<BXS> rx;   rx.init(l32, g);
    KFragReader<BCS> rs_;  rs_.init(l32, g);
    KFragReader<D1> ry;    ry.init(l32, g);
    TFragReader<BD2> rz;   rz.init(lane, 4);
    TFragReader<BD2> rzn;  rzn.init(lane, 8);    // natural k order, for contraction-major state slices

    f32x16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.0f;

    // mLSTMexp forward: accumulator of the normaliser's inter-chunk dot q~ . n_{k-1} (see below)
    f32x16 an;
#pragma unroll
    for (int v = 0; v < 16; ++v) an[v] = 0.0f;
    const char* nrow = reinterpret_cast<const char*>(ldsN) + (l32 & 1) * (D1 * 2) + 16 * g;

#pragma unroll
    for (int i = 0; i < NPRE; ++i) {
        const int pi = pre_item(i, BXS, BCS), sl = pi >> 1;
        wait_vmcnt_dyn(pending_after(i));
        // the fragment reads of an X slice (not consumed by any instruction yet) have left LDS before its stage is refilled
        if (i == 0 || (pre_item(i > 0 ? i - 1 : 0, BXS, BCS) & 1)) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        barrier_nofence();
        const char* sb = smem + (i % NS) * STAGE;
        if (pi & 1) {
            if (i + NS - 1 < NI) issue(i + NS - 1);
#pragma unroll
            for (int ks = 0; ks < BXS / 16; ++ks) xf[sl * (BXS / 16) + ks].v = rx.load(sb, ks, wave);
            // 512-wide rows are 128 registers per lane, as many as the widest accumulator: together they fill the
            // ordinary vector registers.  Left alone, the compiler parks the rows in accumulation registers and copies
            // them back before the products of every column tile (122 copies per tile in the dQ kernel); defined in
            // accumulation registers here, they are read from there by the matrix instructions themselves.
            // (dK, whose column tiles carry E, fits the ordinary registers and gains nothing.)
            if constexpr (D1 == 512 && OCC == 1 && !ELITE) {
#pragma unroll
                for (int ks = 0; ks < BXS / 16; ++ks) asm volatile("" : "+a"(xf[sl * (BXS / 16) + ks].v));
            }
            if (MODE == MODE_H) {
                if (a.variant == 0) {
                    // this slice's share of q~ . n_{k-1}: it fills matrix-unit time that the loads leave idle here
                    // (n has landed: it was requested before the ring and this is past the first barrier)
#pragma unroll
                    for (int ks = sl * (BXS / 16); ks < (sl + 1) * (BXS / 16); ++ks) {
                        frag bn;
                        bn.v = *reinterpret_cast<const bf16x8*>(nrow + 32 * ks);
                        if (l32 >= 2) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) bn.v[e] = (bf16_t)0.0f;
                        }
                        an = E::mma(bn, xf[ks], an);
                    }
                }
            }
        } else {
            const bool req = i + NS - 1 < NI;
            constexpr int KSS = BCS / 16, NF = KSS * NB;
            if constexpr (OCC == 1) {
                // one wavefront per SIMD: nothing else hides the time the request spends in the memory
                // pipeline's queue, so it is spread between the matrix instructions; the fragments of k step
                // ks + 1 are read while the matrix instructions of k step ks run
                frag b[2][NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) b[0][nb].v = STT ? rzn.load(sb, nb, 0, 4) : rs_.load(sb, 0, nb);
#pragma unroll
                for (int ks = 0; ks < KSS; ++ks) {
                    if (ks + 1 < KSS) {
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            b[(ks + 1) & 1][nb].v = STT ? rzn.load(sb, nb, 16 * (ks + 1), 16 * (ks + 1) + 4) : rs_.load(sb, ks + 1, nb);
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) acc[nb] = E::mma(b[ks & 1][nb], xf[sl * KSS + ks], acc[nb]);
                    if (req) issue_part(i + NS - 1, ks, KSS);
                }
            } else {
                if (req) issue(i + NS - 1);
                frag b[KSS][NB];
#pragma unroll
                for (int ks = 0; ks < KSS; ++ks)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        b[ks][nb].v = STT ? rzn.load(sb, nb, 16 * ks, 16 * ks + 4) : rs_.load(sb, ks, nb);
#pragma unroll
                for (int ks = 0; ks < KSS; ++ks)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) acc[nb] = E::mma(b[ks][nb], xf[sl * KSS + ks], acc[nb]);
                // LDS reads run PF fragments ahead of the MFMAs that consume them
                constexpr int PF = NF < 4 ? NF : 4;
                constexpr int DSR = STT ? 2 : 1;            // LDS reads per fragment
#pragma unroll
                for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x100, DSR, 0);
#pragma unroll
                for (int q = 0; q < NF - PF; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, DSR, 0);
                }
#pragma unroll
                for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }

        }
    }
    TFLA_TL(2);
    // The accumulators are kept transposed (rows = columns of the output block, columns = the
    // wave's 32 output rows): every per-row quantity is then one scalar per lane.
    const float srl = ldsS[wave][l32];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] *= srl;
    float nrm = 0.0f;
    if (MODE == MODE_H) {
        if (a.variant == 0) {
            // q~ . n_{k-1} on the matrix unit: n sits in LDS as two bf16 rows (value, remainder), which enter as
            // rows 0 and 1 of an otherwise empty 32-row operand next to the X fragments in registers; the
            // two result columns of a row add up to its dot product
            // (the products were formed slice by slice while the X rows arrived, see above)
            float dot = g == 0 ? an[0] + an[1] : 0.0f;
            dot += __shfl_xor(dot, 32, 64);
            nrm = dot * srl;
        }
    }
    TFLA_TL(3);
    // ---------------- intra-chunk part, one 32-column tile per item
    const float wr = ldsWr[wave][l32];
    float rowsum = 0.0f;
    uint32_t eoff = 0;
    if constexpr (ELITE) {
        TFragReader<BR> re;  re.init(lane, 4);
        eoff = re.block_offset(wave);
    }
    for (int ct = ct_lo; ct < ct_hi; ++ct) {
        const int i = NPRE + ct - ct_lo;
        __builtin_assume(i >= NPRE);            // (column tiles only from here on: lets the item-kind tests fold)
        wait_vmcnt_dyn(pending_after(i));
        barrier_nofence();
        const bool req = i + NS - 1 < NI;
        if constexpr (WPRE) {
            if (i == NI - 1) {
                const int sl = wave, stg = (i + 1 + sl / SPS) % NS;
                DmaTile<32, BD2, 64, SWZ_K> dw;
                dw.init(d2, lane);
                const bf16_t* wsrc = reinterpret_cast<const bf16_t*>(FUSE ? a.fz_o : a.dotwith) + (tbase + wr0) * d2 + (long)nb2 * BD2;
                const uint32_t wdst = smem_a + (uint32_t)(stg * STAGE + (sl % SPS) * SLOT);
                if (FUSE && !a.fz_o) {}                  // no output gate: nothing to fetch
                else if (gx == 1) dw.template issue<true>(wsrc, wdst, lane);
                else dw.issue(wsrc, wdst, lane);
            }
        }
        const int cs = ct * BC;
        const bool masked = UPPER ? (cs + 31 < wr0) : (cs > wr0 + 31);   // fully masked for this wave
        // with one wavefront per SIMD the request is spread between the matrix instructions below
        // with 128-column blocks measured slower (the groups lose the read-ahead across their boundaries); with
        // 256-column blocks it keeps the Y fragments of a tile within the register budget
        constexpr bool SPREAD = !ELITE && BD2 == 256 && D1 == 512;
        if (req && (!SPREAD || masked)) issue(i + NS - 1);
        if (masked) continue;
        const bool diag = UPPER ? (cs < wr0 + 31) : (cs + 31 > wr0);
        const char* yb = smem + (i % NS) * STAGE;
        const char* zb = yb + YB;
        const float* wb = &ldsW[i % NS][wave][0];
        frag p0, p1;
        if constexpr (ELITE) {
            // E^T of this wave's rows: the tile is [32 query rows][BR rows of this workgroup]
            p0.v = TFragReader<BR>::load_at(yb, eoff, 0, 8);
            p1.v = TFragReader<BR>::load_at(yb, eoff, 16, 24);
        } else {
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.0f;
        if constexpr (SPREAD) {
            constexpr int G = 4, KG = KS1 / G;
#pragma unroll
            for (int gq = 0; gq < G; ++gq) {
                frag ya[KG];
#pragma unroll
                for (int ks = 0; ks < KG; ++ks) ya[ks].v = ry.load(yb, gq * KG + ks, 0);
#pragma unroll
                for (int ks = 0; ks < KG; ++ks) s = E::mma(ya[ks], xf[gq * KG + ks], s);
                constexpr int PF = KG < 4 ? KG : 4;
#pragma unroll
                for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
                for (int q = 0; q < KG - PF; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
#pragma unroll
                for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (req) issue_part(i + NS - 1, gq, G);
            }
        } else {
            frag ya[KS1];
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) ya[ks].v = ry.load(yb, ks, 0);
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) s = E::mma(ya[ks], xf[ks], s);
            // LDS reads run PF fragments ahead of the MFMAs that consume them
            constexpr int PF = KS1 < 4 ? KS1 : 4;
#pragma unroll
            for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
            for (int q = 0; q < KS1 - PF; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
#pragma unroll
            for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        float p[16];
        if (diag) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int cl = acc_row(v, g);
                const float w = fast_exp2(wr + wb[cl]);
                const bool keep = UPPER ? (cs + cl >= wr0 + l32) : (cs + cl <= wr0 + l32);
                p[v] = keep ? s[v] * w : 0.0f;
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) p[v] = s[v] * fast_exp2(wr + wb[acc_row(v, g)]);
        }
        if (MODE == MODE_H) {
#pragma unroll
            for (int v = 0; v < 16; ++v) rowsum += p[v];
        }
        p0 = E::pack(p); p1 = E::pack(p + 8);
        if constexpr (EWRITE) {
            if (nb2 == 0 && a.E) {
                // E[wr0 + r][cs + c]: through a wave-private [32 r][32 c] tile so that rows leave in
                // 64-byte segments; lane (r, g) holds c = 8 q + 4 g + {0..3} in register pair q
                char* et = ldsE + wave * 2048;
                const u32x4 w0 = __builtin_bit_cast(u32x4, p0.v), w1 = __builtin_bit_cast(u32x4, p1.v);
                const int sw = (l32 >> 1) & 3;
                *reinterpret_cast<uint2*>(et + l32 * 64 + ((0 ^ sw) * 16) + 8 * g) = uint2{w0[0], w0[1]};
                *reinterpret_cast<uint2*>(et + l32 * 64 + ((1 ^ sw) * 16) + 8 * g) = uint2{w0[2], w0[3]};
                *reinterpret_cast<uint2*>(et + l32 * 64 + ((2 ^ sw) * 16) + 8 * g) = uint2{w1[0], w1[1]};
                *reinterpret_cast<uint2*>(et + l32 * 64 + ((3 ^ sw) * 16) + 8 * g) = uint2{w1[2], w1[3]};
                char* eg = reinterpret_cast<char*>(a.E) +
                           ((((long)bh * a.Nc + kc) * a.L + wr0) * a.L + cs) * 2;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int n = q * 16 + (lane >> 2), c4 = lane & 3;
                    const u32x4 w = *reinterpret_cast<const u32x4*>(et + n * 64 + ((c4 ^ ((n >> 1) & 3)) * 16));
                    // (non-temporal like the kernel's other results: the dK kernel reads E once, from memory)
                    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(eg + ((long)n * a.L + 8 * c4) * 2));
                }
            }
        }
        }
        {
            frag z[NB][2];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                z[nb][0].v = rz.load(zb, nb, 0, 8);
                z[nb][1].v = rz.load(zb, nb, 16, 24);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                acc[nb] = E::mma(z[nb][0], p0, acc[nb]);
                acc[nb] = E::mma(z[nb][1], p1, acc[nb]);
            }
            // every Z fragment pair costs four transposing reads; keep two pairs ahead
            constexpr int PF = NB < 2 ? NB : 2;
#pragma unroll
            for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int q = 0; q < NB - PF; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            }
#pragma unroll
            for (int q = 0; q < PF; ++q) __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
    }

    TFLA_TL(4);
    // ---------------- epilogue
    const long t = tbase + wr0 + l32;       // this lane's output row
    if (MODE == MODE_H) {
        if (a.variant == 0) {
            rowsum += __shfl_xor(rowsum, 32, 64);
            nrm += rowsum;
        }
    }
    // One half of a contraction wider than D1: register quad 4j..4j+3 of block nb holds columns
    // 32 nb + 8 j + 4 g + {0..3} of row t, so the fp32 partial results move as 16-byte accesses.
    if constexpr (SPLIT == 2) {
        const float* pin = a.acc_in + t * d2 + (long)nb2 * BD2 + 4 * g;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const f32x4 w = *reinterpret_cast<const f32x4*>(pin + 32 * nb + 8 * j);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[nb][4 * j + e] += w[e];
            }
            asm volatile("" ::: "memory");      // one block's loads at a time: no register pile-up
        }
        if (MODE == MODE_H && a.variant == 0) nrm += a.nrm_in[t];
    }
    if constexpr (SPLIT == 1) {
        float* pout = a.acc_out + t * d2 + (long)nb2 * BD2 + 4 * g;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = acc[nb][4 * j + e];
                *reinterpret_cast<f32x4*>(pout + 32 * nb + 8 * j) = w;
            }
        if (MODE == MODE_H && a.variant == 0 && g == 0 && nb2 == 0) a.nrm_out[t] = nrm;
        return;
    }
    float inv = 1.0f;
    if (MODE == MODE_H) {
        if (a.variant == 0) {
            const float den = fmaxf(fabsf(nrm), expf(-ldsM[wave][l32])) + a.eps;
            inv = 1.0f / den;
            if (g == 0 && a.nout && nb2 == 0) a.nout[t] = nrm;
            if (g == 0 && a.wrowB_out && nb2 == 0) {
                a.wrowB_out[t] = wr - log2f(den);
                a.sQ_out[t] = srl / den;
            }
        }
    }
    // Register quad 4j..4j+3 of block nb holds columns 32 nb + 8 j + 4 g + {0..3} of row t.  The
    // output block goes through LDS (the ring is free now) so that it leaves in full 16-byte,
    // row-contiguous stores: per wave a [32][BD2] bf16 tile with XOR-swizzled 16-byte chunks.
    barrier_nofence();                                   // every wave is done reading the ring
    constexpr int OCPR = BD2 / 8, ORB = BD2 * 2;         // chunks and bytes per tile row
    auto slot_at = [&](int sl) { return smem + ((NI + sl / SPS) % NS) * STAGE + (sl % SPS) * SLOT; };
    char* otile = WPRE ? slot_at(NW + wave) : smem + wave * (32 * ORB);
    char* wtile = WPRE ? slot_at(wave) : smem + NW * (32 * ORB) + wave * (32 * ORB);
    if (WTILE && !WPRE) {
        DmaTile<32, BD2, 64, SWZ_K> dw;                  // this wave's rows of the dot operand (of the gate pre-activations)
        dw.init(d2, lane);
        const bf16_t* wsrc = reinterpret_cast<const bf16_t*>(FUSE ? a.fz_o : a.dotwith) + (tbase + wr0) * d2 + (long)nb2 * BD2;
        if (FUSE && !a.fz_o) {}                          // no output gate: nothing to fetch
        else if (gx == 1) dw.template issue<true>(wsrc, lds_addr(wtile), lane);
        else dw.issue(wsrc, lds_addr(wtile), lane);
    }
    // fused layer output: this lane's eight columns of the per-head scale and shift (requested here, ahead of the
    // output stores, so that the wait further down covers them together with the gate pre-activations)
    float fz_g[8], fz_b[8];
    if constexpr (FUSE) {
        const int c8 = (lane % (BD2 / 8)) * 8;
        const long hoff = (long)(bh % a.fz_NH) * d2 + c8;
#pragma unroll
        for (int e = 0; e < 8; ++e) { fz_g[e] = 1.0f; fz_b[e] = 0.0f; }
        if (a.fz_gamma) {
            const f32x4 g0 = *reinterpret_cast<const f32x4*>(a.fz_gamma + hoff), g1 = *reinterpret_cast<const f32x4*>(a.fz_gamma + hoff + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { fz_g[e] = g0[e]; fz_g[4 + e] = g1[e]; }
        }
        if (a.fz_beta && a.fz_kind == 1) {
            const f32x4 b0 = *reinterpret_cast<const f32x4*>(a.fz_beta + hoff), b1 = *reinterpret_cast<const f32x4*>(a.fz_beta + hoff + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { fz_b[e] = b0[e]; fz_b[4 + e] = b1[e]; }
        }
    }
    const int fsw = swz_mask<SWZ_K, OCPR>(l32);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint2 w;
            w.x = pack_bf16x2(acc[nb][4 * j] * inv, acc[nb][4 * j + 1] * inv);
            w.y = pack_bf16x2(acc[nb][4 * j + 2] * inv, acc[nb][4 * j + 3] * inv);
            *reinterpret_cast<uint2*>(otile + l32 * ORB + (((4 * nb + j) ^ fsw) * 16) + 8 * g) = w;
        }
    {
        constexpr int RPI = 64 / OCPR;                   // tile rows covered by one 64-lane store
        if constexpr (!PADOUT) {
            char* obase = reinterpret_cast<char*>(a.Out) + ((tbase + wr0) * d2 + (long)nb2 * BD2) * 2;
#pragma unroll
            for (int q = 0; q < 32 / RPI; ++q) {
                const int r = q * RPI + lane / OCPR, c = lane % OCPR;
                const u32x4 w = *reinterpret_cast<const u32x4*>(otile + r * ORB + ((c ^ swz_mask<SWZ_K, OCPR>(r)) * 16));
                // the result is not read again by the kernels that follow: non-temporal, so that it does not displace
                // their operands from the caches (measured: -2 % on the whole step)
                __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(obase + (long)r * d2 * 2 + c * 16));
            }
        } else {
            // straight into the caller's tensor: its own row count and row length, true steps and columns only
            const int ts0 = kc * a.L + wr0;              // first step of this wave's rows within the sequence
            char* obase = reinterpret_cast<char*>(a.Out) + (((long)bh * a.out_T + ts0) * a.out_ld + (long)nb2 * BD2) * 2;
#pragma unroll
            for (int q = 0; q < 32 / RPI; ++q) {
                const int r = q * RPI + lane / OCPR, c = lane % OCPR;
                const u32x4 w = *reinterpret_cast<const u32x4*>(otile + r * ORB + ((c ^ swz_mask<SWZ_K, OCPR>(r)) * 16));
                if (ts0 + r < a.out_T && nb2 * BD2 + c * 8 < a.out_cols)
                    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(obase + (long)r * a.out_ld * 2 + c * 16));
            }
        }
    }
    if constexpr (FUSE) {
        // y = sigma(o~) (.) (gamma (.) x^ + beta), x^ = (h~ - mean) rstd (LayerNorm) or h~ rstd (RMS norm), from the
        // rounded h~ of the tile just stored: in the row-contiguous read-back a row's BD2 columns sit in BD2 / 8
        // neighbouring lanes, eight columns each.  The gate pre-activations, the scale and the shift are older than
        // the output stores above, so the wait leaves only those stores in flight.
        constexpr int RPI = 64 / OCPR;
        wait_vmcnt<32 / RPI>();
        char* ybase = reinterpret_cast<char*>(a.fz_y) + ((tbase + wr0) * d2) * 2;
        const float invd = 1.0f / (float)BD2;
#pragma unroll
        for (int q = 0; q < 32 / RPI; ++q) {
            const int r = q * RPI + lane / OCPR, c = lane % OCPR;
            const uint32_t toff = (uint32_t)(r * ORB + ((c ^ swz_mask<SWZ_K, OCPR>(r)) * 16));
            const u32x4 hw = *reinterpret_cast<const u32x4*>(otile + toff);
            float x[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) { x[2 * e] = bf16_lo_to_f32(hw[e]); x[2 * e + 1] = bf16_hi_to_f32(hw[e]); }
            if (a.fz_kind == 1) {
                float sm = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) sm += x[e];
#pragma unroll
                for (int m = 1; m < OCPR; m <<= 1) sm += __shfl_xor(sm, m, 64);
                const float mu = sm * invd;
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] -= mu;
            }
            float ss = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
#pragma unroll
            for (int m = 1; m < OCPR; m <<= 1) ss += __shfl_xor(ss, m, 64);
            const float rstd = 1.0f / sqrtf(ss * invd + a.fz_eps);
            float y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = x[e] * rstd * fz_g[e] + fz_b[e];
            if (a.fz_o) {
                const u32x4 ow = *reinterpret_cast<const u32x4*>(wtile + toff);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float o0 = bf16_lo_to_f32(ow[e]), o1 = bf16_hi_to_f32(ow[e]);
                    const float e0 = expf(-fabsf(o0)), e1 = expf(-fabsf(o1));
                    y[2 * e] *= o0 >= 0.0f ? 1.0f / (1.0f + e0) : e0 / (1.0f + e0);
                    y[2 * e + 1] *= o1 >= 0.0f ? 1.0f / (1.0f + e1) : e1 / (1.0f + e1);
                }
            }
            u32x4 yw;
#pragma unroll
            for (int e = 0; e < 4; ++e) yw[e] = pack_bf16x2(y[2 * e], y[2 * e + 1]);
            __builtin_nontemporal_store(yw, reinterpret_cast<u32x4*>(ybase + (long)r * d2 * 2 + c * 16));
        }
    }
    if (MODE == MODE_DQ || MODE == MODE_DK) {
        // the dot operand has landed: its loads are older than the output stores above (and than the E stores of the
        // last tile), which may still be on their way.  (A padded problem issues a store only where a lane has
        // something to store, so their number is not known here.)
        if constexpr (PADOUT) wait_vmcnt<0>();
        else wait_vmcnt<32 / (64 / OCPR)>();
        float d = 0.0f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint2 w = *reinterpret_cast<const uint2*>(wtile + l32 * ORB + (((4 * nb + j) ^ fsw) * 16) + 8 * g);
                d += acc[nb][4 * j] * bf16_lo_to_f32(w.x) + acc[nb][4 * j + 1] * bf16_hi_to_f32(w.x) +
                     acc[nb][4 * j + 2] * bf16_lo_to_f32(w.y) + acc[nb][4 * j + 3] * bf16_hi_to_f32(w.y);
            }
        d += __shfl_xor(d, 32, 64);
        if (g == 0) a.dotpart[(long)nb2 * (long)bhn * a.T + t] = d;
    }
    TFLA_TL(5);
#ifdef TFLA_TIMELINE
    wait_vmcnt<0>();
    TFLA_TL(6);
#endif
}

}  // namespace tfla
