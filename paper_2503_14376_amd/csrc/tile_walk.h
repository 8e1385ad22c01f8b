// bf16 "walking" form of the intra-chunk tiled kernels for the forward outputs (H) and dV (see tile.hip for what
// is computed; the arithmetic, the fragment layouts and the order of the products are those of tile_kernel_bf16).
//
// What differs is the division of work.  One workgroup owns 256 rows of a chunk and ALL output columns: it walks
// the 128-column blocks of the output one after the other, with its rows of X held in registers for the whole
// kernel.  A wavefront owns two 32-row blocks (b and 7 - b of the eight, so that the causal triangle gives every
// wavefront the same number of column tiles): every state fragment and every column-tile fragment read from LDS
// feeds two matrix instructions instead of one, the rows of X are fetched once per chunk instead of once per
// column block, and the column tiles and state slices once per 256 rows instead of once per 128.  All operands
// stream through one ring of asynchronous global->LDS loads that keeps running across the column blocks (the
// output block leaves through a staging area of its own), so its start-up and drain are paid once per chunk.
//
// Outstanding-load bookkeeping: vector-memory operations of a wavefront retire in issue order, so "item i has
// landed" means "at most (operations issued after item i's) are outstanding".  Every wavefront counts the
// operations it issues (issued) and remembers the count at the end of each ring item (seq_end); the wait is
// computed from the two.  Counting an operation too few only makes a wait stricter; every store of the
// epilogue that is counted is one fixed-size store instruction of an unrolled loop.
#pragma once
#include <type_traits>

#include "lds_tiles.h"
#include "tfla_internal.h"

namespace tfla {

// Development aid, compiled only with -DTFLA_WALK_TL: wavefronts 0 and NW - 1 of workgroup 0 record the shader clock
// per ring item: before the wait, after the barrier, after the requests, at the end of the item's work.
#ifdef TFLA_WALK_TL
static __device__ unsigned long long walk_tl[2 * 4 * 512];
#define TFLA_WTL(k)                                                                       \
    do {                                                                                  \
        if (blockIdx.x == 0 && lane == 0 && (wave == 0 || wave == NW - 1) && tl_item < 512) \
            walk_tl[((wave == 0 ? 0 : 1) * 512 + tl_item) * 4 + (k)] = __builtin_amdgcn_s_memtime(); \
    } while (0)
#define TFLA_WTL_NEXT() (++tl_item)
#else
#define TFLA_WTL(k)
#define TFLA_WTL_NEXT()
#endif

#ifdef TFLA_WALK_NOSGB
#define TFLA_SGB(a, b, c)
#else
#define TFLA_SGB(a, b, c) __builtin_amdgcn_sched_group_barrier(a, b, c)
#endif

// NW = 4: four wavefronts with two row blocks each (b and 7 - b); NW = 8: eight wavefronts with one row block each,
// the two wavefronts of a SIMD (w and w + 4) holding blocks b and 7 - b.
template <int D1, int MODE, int NW>
__global__ void __launch_bounds__(NW * 64, 1) walk_kernel_bf16(TileArgs a) {
    using E = Elem<bf16_t>;
    using frag = E::frag;
    static_assert(MODE == MODE_H || MODE == MODE_DV, "walking kernel: H and dV");
    static_assert(D1 == 128 || D1 == 256, "contraction widths 128 and 256");
    constexpr bool UPPER = MODE == MODE_DV;
    static_assert(NW == 4 || NW == 8, "four or eight wavefronts");
    constexpr int MB = 8 / NW;                                   // row blocks per wavefront
    constexpr int NT = NW * 64, BR = 256, BC = 32, BD2 = 128, NB = BD2 / 32, KS1 = D1 / 16;
    constexpr int YB = BC * D1 * 2, ZB = BC * BD2 * 2;
    constexpr int STAGE = YB + ZB < 16384 ? 16384 : YB + ZB;
    constexpr int BXS = 32, NXS = D1 / BXS;                      // X rows arrive as [256][32] slices (16 KB)
    constexpr int BCS = 64, NKS = D1 / BCS, KSS = BCS / 16;      // state slices [128][64] (16 KB)
    constexpr int EW = NW == 4 ? BD2 : BD2 / 2;                  // width of a wavefront's output staging tile
    constexpr int EPI = NW * 32 * EW * 2;                        // output staging, [32][EW] per wavefront
    constexpr int NS_RAW = (160 * 1024 - EPI - 6144) / STAGE;
    constexpr int NS = NS_RAW > 6 ? 6 : NS_RAW;
    static_assert(NS >= 3 && BR * BXS * 2 <= STAGE && BD2 * BCS * 2 <= STAGE, "ring stage sizes");

    __shared__ __attribute__((aligned(1024))) char smem[NS * STAGE];
    __shared__ __attribute__((aligned(1024))) char epi[EPI];
    __shared__ __attribute__((aligned(256))) float ldsW[NS][64];      // column weights of the tile in each stage
    __shared__ __attribute__((aligned(256))) float ldsS[8][32];       // per-row scalars of the 8 row blocks
    __shared__ __attribute__((aligned(256))) float ldsWr[8][32];
    __shared__ __attribute__((aligned(256))) float ldsM[8][32];
    __shared__ __attribute__((aligned(256))) float ldsN[(MODE == MODE_H) ? D1 : 64];

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // linear id -> (row block of 256, chunk, batch*head); chunks of an XCD's slices are walked together
    const unsigned nwg = gridDim.x, gy = (unsigned)a.L / BR;
    unsigned wg = xcd_remap(blockIdx.x, nwg);
    const int rbi = __builtin_amdgcn_readfirstlane((int)(wg % gy)); wg /= gy;
    const int rb = UPPER ? rbi : (int)gy - 1 - rbi;
    const unsigned bhn = nwg / (gy * (unsigned)a.Nc);
    const unsigned bpx = (bhn % 8u == 0u) ? bhn / 8u : 1u;
    const unsigned bl = wg % bpx; wg /= bpx;
    const int kci = __builtin_amdgcn_readfirstlane((int)(wg % a.Nc));
    const int kc = a.kc_desc ? a.Nc - 1 - kci : kci;
    const int bh = __builtin_amdgcn_readfirstlane((int)((wg / a.Nc) * bpx + bl));
    const long tbase = (long)bh * a.T + (long)kc * a.L;
    const int r0 = rb * BR;
    const int d2 = a.d2, NCB = d2 / BD2;
    // the wavefront's row blocks and their first rows (two blocks: index 0 = block `wave`, index 1 = block 7 - wave)
    const int blk[2] = {MB == 2 ? wave : (wave < 4 ? wave : 11 - wave), 7 - wave};
    const int wr0[2] = {r0 + 32 * blk[0], r0 + 32 * blk[1]};

    const bf16_t* Xb = reinterpret_cast<const bf16_t*>(a.X) + (tbase + r0) * D1;
    const bf16_t* Y = reinterpret_cast<const bf16_t*>(a.Y) + tbase * D1;
    const bf16_t* Z = reinterpret_cast<const bf16_t*>(a.Z) + tbase * d2;
    const bf16_t* St = reinterpret_cast<const bf16_t*>(a.St) + ((long)bh * a.Nc + kc) * d2 * D1;
    const float* wcol = a.wcol + tbase;
    const bool with_n = MODE == MODE_H && a.variant == 0;

    const int ct_lo = UPPER ? r0 / BC : 0;
    const int ct_hi = UPPER ? a.L / BC : (r0 + BR) / BC;
    const int NTL = ct_hi - ct_lo, PER = NKS + NTL;
    const int NI = NXS + NCB * PER;                               // items streamed through the ring

    DmaTile<BR, BXS, NT, SWZ_K> dxs;   dxs.init(D1, tid);
    DmaTile<BD2, BCS, NT, SWZ_K> ds;   ds.init(D1, tid);
    DmaTile<BC, D1, NT, SWZ_K> dy;     dy.init(D1, tid);
    DmaTile<BC, BD2, NT, SWZ_T> dz;    dz.init(d2, tid);
    const uint32_t smem_a = lds_addr(smem), w_a = lds_addr(ldsW);

    // ---- ring bookkeeping (all wave-uniform)
    int issued = 0;                        // vector-memory operations this wavefront has issued so far
    int seq_end[NS];                       // `issued` right after the last load of the item in each stage
#pragma unroll
    for (int s = 0; s < NS; ++s) seq_end[s] = 0;
    int iss_item = 0, iss_stage = 0, iss_cb = 0, iss_q = 0;      // the next item to request
    int cons_stage = 0;                                           // stage of the item consumed next
#ifdef TFLA_WALK_TL
    int tl_item = 0;
#endif
    // (macros rather than lambdas: the counters must stay in scalar registers, and a by-reference capture next to
    // the volatile asm of the loads leaves them in scratch memory, whose accesses are vector-memory operations)
    // Requesting the next ring item is split into a preparation (which item, where from, where to), MAXP parts of
    // one load instruction each that the work loops place between their matrix instructions (all wavefronts
    // asking for their loads at once right behind the barrier would queue up in the one texture-address unit
    // while the matrix unit idles), and the bookkeeping at the end.
    constexpr int NXL = decltype(dxs)::N, NSL = decltype(ds)::N, NYL = decltype(dy)::N, NZL = decltype(dz)::N;
    constexpr int MAXP = NYL + NZL + 1;
    static_assert(NXL <= MAXP && NSL <= MAXP, "parts per item");
    int ip_kind = 0;                       // 0: nothing left to request, 1: X slice, 2: state slice, 3: column tile
    uint32_t ip_st = 0, ip_w = 0;
    const bf16_t* ip_g0 = nullptr;
    const bf16_t* ip_g1 = nullptr;
    const float* ip_g2 = nullptr;
#define TFLA_WALK_ISSUE_PREP()                                                                                     \
    do {                                                                                                           \
        ip_kind = 0;                                                                                               \
        if (iss_item < NI) {                                                                                       \
            ip_st = smem_a + (uint32_t)iss_stage * STAGE;                                                          \
            if (iss_item < NXS) {                                                                                  \
                ip_kind = 1; ip_g0 = Xb + iss_item * BXS;                                                          \
            } else if (iss_q < NKS) {                                                                              \
                ip_kind = 2; ip_g0 = St + (long)iss_cb * BD2 * D1 + (long)iss_q * BCS;                             \
            } else {                                                                                               \
                const int ct_ = ct_lo + iss_q - NKS;                                                               \
                ip_kind = 3; ip_g0 = Y + (long)ct_ * BC * D1; ip_g1 = Z + (long)ct_ * BC * d2 + (long)iss_cb * BD2; \
                ip_g2 = wcol + ct_ * BC; ip_w = w_a + (uint32_t)(iss_stage * 256);                                 \
            }                                                                                                      \
        }                                                                                                          \
    } while (0)
    // part J (compile-time): the J-th load instruction of this wavefront for the prepared item, if it has one.
    // Column tiles: the Y loads, the Z loads, then the tile's 32 column weights (both half-waves fetch the same 32
    // floats; every wavefront fetches them to the same place, so its own counter covers what it reads).
#define TFLA_WALK_ISSUE_PART(J)                                                                                    \
    do {                                                                                                           \
        if (ip_kind == 1) dxs.issue_one(ip_g0, ip_st, tid, (J));                                                   \
        else if (ip_kind == 2) ds.issue_one(ip_g0, ip_st, tid, (J));                                               \
        else if (ip_kind == 3) {                                                                                   \
            if ((J) < NYL) dy.issue_one(ip_g0, ip_st, tid, (J));                                                   \
            else if ((J) < NYL + NZL) dz.issue_one(ip_g1, ip_st + YB, tid, (J) - NYL);                             \
            else if ((J) == NYL + NZL) dma4_free(ip_g2, (uint32_t)(lane & 31) * 4u, ip_w);                              \
        }                                                                                                          \
    } while (0)
#define TFLA_WALK_ISSUE_FINISH()                                                                                   \
    do {                                                                                                           \
        if (ip_kind != 0) {                                                                                        \
            issued += ip_kind == 1 ? NXL : (ip_kind == 2 ? NSL : NYL + NZL + 1);                                   \
            if (ip_kind != 1) { if (++iss_q == PER) { iss_q = 0; ++iss_cb; } }                                     \
            _Pragma("unroll") for (int s_ = 0; s_ < NS; ++s_) seq_end[s_] = (s_ == iss_stage) ? issued : seq_end[s_]; \
            ++iss_item;                                                                                            \
            if (++iss_stage == NS) iss_stage = 0;                                                                  \
        }                                                                                                          \
    } while (0)
    // the whole request at once
#define TFLA_WALK_ISSUE_NEXT()                                                                                     \
    do {                                                                                                           \
        TFLA_WALK_ISSUE_PREP();                                                                                    \
        _Pragma("unroll") for (int j_ = 0; j_ < MAXP; ++j_) TFLA_WALK_ISSUE_PART(j_);                              \
        TFLA_WALK_ISSUE_FINISH();                                                                                  \
    } while (0)
    // wait until this wavefront's loads of the item in the stage consumed next have landed
#define TFLA_WALK_WAIT_ITEM()                                                                                      \
    do {                                                                                                           \
        int e_ = 0;                                                                                                \
        _Pragma("unroll") for (int s_ = 0; s_ < NS; ++s_) e_ = (s_ == cons_stage) ? seq_end[s_] : e_;              \
        const int pend_ = issued - e_;                                                                             \
        wait_vmcnt_dyn(pend_ > 63 ? 63 : pend_);                                                                   \
    } while (0)
#define TFLA_WALK_ADVANCE() do { if (++cons_stage == NS) cons_stage = 0; } while (0)

    // ---- per-row scalars of the 256 rows: wavefront p fetches those of row blocks 2p and 2p + 1 (64 rows)
    if (wave < 4) {
        const uint32_t vo = (uint32_t)lane * 4u;
        const long rr = tbase + r0 + 64 * wave;
        dma4(a.srow + rr, vo, lds_addr(&ldsS[2 * wave][0]));
        dma4(a.wrow + rr, vo, lds_addr(&ldsWr[2 * wave][0]));
        issued += 2;
        if (with_n) {
            dma4(a.mout + rr, vo, lds_addr(&ldsM[2 * wave][0]));
            issued += 1;
            // n_{k-1}: two bf16 rows (rounded value, rounding remainder) of D1 columns, contiguous
            const char* nsrc = reinterpret_cast<const char*>(a.nstate) + ((long)bh * a.Nc + kc) * D1 * 4;
            for (int c = wave; c < D1 / 64; c += 4) {
                dma4(nsrc + 256 * c, (uint32_t)lane * 4u, lds_addr(ldsN) + 256u * c);
                issued += 1;
            }
        }
    }
#pragma unroll
    for (int p = 0; p < NS - 1; ++p) TFLA_WALK_ISSUE_NEXT();

    // ---------------- X fragments of the wavefront's MB x 32 rows (lane: row l32, k-group g)
    frag xf[MB][KS1];
    {
        KFragReader<BXS> rx;  rx.init(l32, g);
#pragma unroll
        for (int i = 0; i < NXS; ++i) {
            TFLA_WTL(0);
            TFLA_WALK_WAIT_ITEM();
            // the fragment reads of the previous slice have left LDS before its stage is refilled
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            barrier_nofence();
            TFLA_WTL(1);
            TFLA_WALK_ISSUE_NEXT();
            TFLA_WTL(2);
            const char* sb = smem + cons_stage * STAGE;
#pragma unroll
            for (int ks = 0; ks < BXS / 16; ++ks)
#pragma unroll
                for (int b = 0; b < MB; ++b) xf[b][i * (BXS / 16) + ks].v = rx.load(sb, ks, blk[b]);
            TFLA_WTL(3); TFLA_WTL_NEXT();
            TFLA_WALK_ADVANCE();
        }
    }

    KFragReader<BCS> rs_;  rs_.init(l32, g);
    KFragReader<D1> ry;    ry.init(l32, g);
    TFragReader<BD2> rz;   rz.init(lane, 4);

    float srl[MB], wrl[MB], inv[MB], nrm[MB], rowsum[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b) { srl[b] = 0.0f; wrl[b] = 0.0f; inv[b] = 1.0f; nrm[b] = 0.0f; rowsum[b] = 0.0f; }
    bool first_cb = true;

    for (int cb = 0; cb < NCB; ++cb) {
        f32x16 acc[MB][NB];
#pragma unroll
        for (int b = 0; b < MB; ++b)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][nb][v] = 0.0f;

        // ---------------- inter-chunk part: acc = X_r St (a wavefront's row blocks share every state fragment)
#pragma unroll
        for (int i = 0; i < NKS; ++i) {
            TFLA_WTL(0);
            TFLA_WALK_WAIT_ITEM();
            if (i == 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            barrier_nofence();
            TFLA_WTL(1);
            TFLA_WALK_ISSUE_PREP();
            TFLA_WTL(2);
            const char* sb = smem + cons_stage * STAGE;
            // the fragments of k step ks + 1 are read while the matrix instructions of k step ks run
            frag bf[2][NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) bf[0][nb].v = rs_.load(sb, 0, nb);
#pragma unroll
            for (int ks = 0; ks < KSS; ++ks) {
                if (ks + 1 < KSS) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) bf[(ks + 1) & 1][nb].v = rs_.load(sb, ks + 1, nb);
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int b = 0; b < MB; ++b) acc[b][nb] = E::mma(bf[ks & 1][nb], xf[b][i * KSS + ks], acc[b][nb]);
                // the next item's requests go out between the matrix instructions
#pragma unroll
                for (int j = ks * MAXP / KSS; j < (ks + 1) * MAXP / KSS; ++j) TFLA_WALK_ISSUE_PART(j);
            }
            TFLA_WALK_ISSUE_FINISH();
            TFLA_WTL(3); TFLA_WTL_NEXT();
            TFLA_WALK_ADVANCE();
        }
        // The accumulators are kept transposed (rows = columns of the output block, columns = the wave's 32
        // output rows): every per-row quantity is one scalar per lane.  (The per-row scalars landed with the
        // first ring item; the barriers since then have published them.)
        if (first_cb) {
#pragma unroll
            for (int b = 0; b < MB; ++b) { srl[b] = ldsS[blk[b]][l32]; wrl[b] = ldsWr[blk[b]][l32]; }
        }
#pragma unroll
        for (int b = 0; b < MB; ++b)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[b][nb][v] *= srl[b];
        if (MODE == MODE_H) {
            if (with_n && first_cb) {
                // q~ . n_{k-1} on the matrix unit: n sits in LDS as two bf16 rows (value, remainder), which enter as
                // rows 0 and 1 of an otherwise empty 32-row operand next to the X fragments in registers; the two
                // result columns of a row add up to its dot product
                const char* nrow = reinterpret_cast<const char*>(ldsN) + (l32 & 1) * (D1 * 2) + 16 * g;
#pragma unroll
                for (int b = 0; b < MB; ++b) {
                    f32x16 an;
#pragma unroll
                    for (int v = 0; v < 16; ++v) an[v] = 0.0f;
#pragma unroll
                    for (int ks = 0; ks < KS1; ++ks) {
                        frag bn;
                        bn.v = *reinterpret_cast<const bf16x8*>(nrow + 32 * ks);
                        if (l32 >= 2) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) bn.v[e] = (bf16_t)0.0f;
                        }
                        an = E::mma(bn, xf[b][ks], an);
                    }
                    float dot = g == 0 ? an[0] + an[1] : 0.0f;
                    dot += __shfl_xor(dot, 32, 64);
                    nrm[b] = dot * srl[b];
                }
            }
        }

        // ---------------- intra-chunk part, one 32-column tile per item
        for (int ct = ct_lo; ct < ct_hi; ++ct) {
            TFLA_WTL(0);
            TFLA_WALK_WAIT_ITEM();
            barrier_nofence();
            TFLA_WTL(1);
            TFLA_WALK_ISSUE_PREP();
            TFLA_WTL(2);
            const int cs = ct * BC;
            const char* yb = smem + cons_stage * STAGE;
            const char* zb = yb + YB;
            const float* wb = &ldsW[cons_stage][0];
            TFLA_WALK_ADVANCE();
            // which of the wavefront's row blocks see this tile (with two blocks, the one with more tiles is
            // index 1 for the lower triangle, index 0 for the upper one)
            const bool act0 = UPPER ? (cs >= wr0[0]) : (cs <= wr0[0]);
            const bool act1 = MB == 2 && (UPPER ? (cs >= wr0[1]) : (cs <= wr0[1]));
            if (!act0 && !act1) {
#pragma unroll
                for (int j = 0; j < MAXP; ++j) TFLA_WALK_ISSUE_PART(j);
                TFLA_WALK_ISSUE_FINISH();
                TFLA_WTL(3); TFLA_WTL_NEXT();
                continue;
            }

            auto weigh = [&](const f32x16& s, int b, frag& p0, frag& p1) {
                float p[16];
                if (cs == wr0[b]) {         // the tile on the block's diagonal
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int cl = acc_row(v, g);
                        const float w = fast_exp2(wrl[b] + wb[cl]);
                        const bool keep = UPPER ? (cl >= l32) : (cl <= l32);
                        p[v] = keep ? s[v] * w : 0.0f;
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) p[v] = s[v] * fast_exp2(wrl[b] + wb[acc_row(v, g)]);
                }
                if (MODE == MODE_H) {
                    if (first_cb) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) rowsum[b] += p[v];
                    }
                }
                p0 = E::pack(p); p1 = E::pack(p + 8);
            };
            // one row block alone (b1 = its index)
            auto single = [&](auto bsel) {
                constexpr int B1 = decltype(bsel)::value;
                f32x16 s;
#pragma unroll
                for (int v = 0; v < 16; ++v) s[v] = 0.0f;
                // Y fragments in groups of four, the next group read while this one is multiplied; the next item's
                // requests go out between the groups
                constexpr int KG = MB == 1 ? 2 : 4, G = KS1 / KG;
                frag ya[2][KG];
#pragma unroll
                for (int k = 0; k < KG; ++k) ya[0][k].v = ry.load(yb, k, 0);
#pragma unroll
                for (int gq = 0; gq < G; ++gq) {
                    if (gq + 1 < G) {
#pragma unroll
                        for (int k = 0; k < KG; ++k) ya[(gq + 1) & 1][k].v = ry.load(yb, (gq + 1) * KG + k, 0);
                    }
#pragma unroll
                    for (int k = 0; k < KG; ++k) s = E::mma(ya[gq & 1][k], xf[B1][gq * KG + k], s);
#pragma unroll
                    for (int j = 0; j < MAXP; ++j)
                        if (j * G / MAXP == gq) TFLA_WALK_ISSUE_PART(j);
                }
                frag p0, p1;
                weigh(s, B1, p0, p1);
                frag z[NB][2];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    z[nb][0].v = rz.load(zb, nb, 0, 8);
                    z[nb][1].v = rz.load(zb, nb, 16, 24);
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    acc[B1][nb] = E::mma(z[nb][0], p0, acc[B1][nb]);
                    acc[B1][nb] = E::mma(z[nb][1], p1, acc[B1][nb]);
                }
                // every Z fragment pair costs four transposing reads; keep two pairs ahead
                constexpr int PZ = NB < 2 ? NB : 2;
#pragma unroll
                for (int q = 0; q < PZ; ++q) TFLA_SGB(0x100, 4, 0);
#pragma unroll
                for (int q = 0; q < NB - PZ; ++q) {
                    TFLA_SGB(0x008, 2, 0);
                    TFLA_SGB(0x100, 4, 0);
                }
#pragma unroll
                for (int q = 0; q < PZ; ++q) TFLA_SGB(0x008, 2, 0);
            };

            if constexpr (MB == 2) {
                if (act0 && act1) {
                    f32x16 s0, s1;
#pragma unroll
                    for (int v = 0; v < 16; ++v) { s0[v] = 0.0f; s1[v] = 0.0f; }
                    constexpr int KG = 4, G = KS1 / KG;      // Y fragments in groups of four: the register budget
                    frag ya[2][KG];
#pragma unroll
                    for (int k = 0; k < KG; ++k) ya[0][k].v = ry.load(yb, k, 0);
#pragma unroll
                    for (int gq = 0; gq < G; ++gq) {
                        if (gq + 1 < G) {
#pragma unroll
                            for (int k = 0; k < KG; ++k) ya[(gq + 1) & 1][k].v = ry.load(yb, (gq + 1) * KG + k, 0);
                        }
#pragma unroll
                        for (int k = 0; k < KG; ++k) {
                            s0 = E::mma(ya[gq & 1][k], xf[0][gq * KG + k], s0);
                            s1 = E::mma(ya[gq & 1][k], xf[MB - 1][gq * KG + k], s1);
                        }
#pragma unroll
                        for (int j = 0; j < MAXP; ++j)
                            if (j * G / MAXP == gq) TFLA_WALK_ISSUE_PART(j);
                    }
                    frag pa0, pa1, pb0, pb1;
                    weigh(s0, 0, pa0, pa1);
                    weigh(s1, 1, pb0, pb1);
                    frag z[NB][2];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        z[nb][0].v = rz.load(zb, nb, 0, 8);
                        z[nb][1].v = rz.load(zb, nb, 16, 24);
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        acc[0][nb] = E::mma(z[nb][0], pa0, acc[0][nb]);
                        acc[MB - 1][nb] = E::mma(z[nb][0], pb0, acc[MB - 1][nb]);
                        acc[0][nb] = E::mma(z[nb][1], pa1, acc[0][nb]);
                        acc[MB - 1][nb] = E::mma(z[nb][1], pb1, acc[MB - 1][nb]);
                    }
                } else {
                    single(std::integral_constant<int, UPPER ? 0 : MB - 1>{});   // the only block that can be alone
                }
            } else {
                single(std::integral_constant<int, 0>{});
            }
            TFLA_WALK_ISSUE_FINISH();
            TFLA_WTL(3); TFLA_WTL_NEXT();
        }

        // ---------------- epilogue of this column block
        if (MODE == MODE_H) {
            if (with_n && first_cb) {
#pragma unroll
                for (int b = 0; b < MB; ++b) {
                    float rsum = rowsum[b];
                    rsum += __shfl_xor(rsum, 32, 64);
                    nrm[b] += rsum;
                    const float den = fmaxf(fabsf(nrm[b]), expf(-ldsM[blk[b]][l32])) + a.eps;
                    inv[b] = 1.0f / den;
                    // (not counted in `issued`: an operation counted too few only makes a later wait stricter)
                    if (g == 0 && a.nout) a.nout[tbase + wr0[b] + l32] = nrm[b];
                }
            }
        }
        // Register quad 4j..4j+3 of block nb holds columns 32 nb + 8 j + 4 g + {0..3} of the lane's row.  The
        // output block goes through a private LDS tile [32][EW] (XOR-swizzled 16-byte chunks), EW columns at a
        // time, so that it leaves in full 16-byte, row-contiguous stores.
        {
            constexpr int OCPR = EW / 8, ORB = EW * 2, RPI = 64 / OCPR, NBH = EW / 32;
            char* otile = epi + wave * (32 * ORB);
            const int fsw = swz_mask<SWZ_K, OCPR>(l32);
#pragma unroll
            for (int b = 0; b < MB; ++b) {
#pragma unroll
                for (int h = 0; h < BD2 / EW; ++h) {
#pragma unroll
                    for (int nh = 0; nh < NBH; ++nh)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int nb = h * NBH + nh;
                            uint2 w;
                            w.x = pack_bf16x2(acc[b][nb][4 * j] * inv[b], acc[b][nb][4 * j + 1] * inv[b]);
                            w.y = pack_bf16x2(acc[b][nb][4 * j + 2] * inv[b], acc[b][nb][4 * j + 3] * inv[b]);
                            *reinterpret_cast<uint2*>(otile + l32 * ORB + (((4 * nh + j) ^ fsw) * 16) + 8 * g) = w;
                        }
                    char* obase = reinterpret_cast<char*>(a.Out) + ((tbase + wr0[b]) * d2 + (long)cb * BD2 + h * EW) * 2;
#pragma unroll
                    for (int q = 0; q < 32 / RPI; ++q) {
                        const int r = q * RPI + lane / OCPR, c = lane % OCPR;
                        const u32x4 w = *reinterpret_cast<const u32x4*>(otile + r * ORB + ((c ^ swz_mask<SWZ_K, OCPR>(r)) * 16));
                        *reinterpret_cast<u32x4*>(obase + (long)r * d2 * 2 + c * 16) = w;
                    }
                    issued += 32 / RPI;
                    // the tile is reused for the next part: order the passes for the compiler (the hardware runs
                    // one wavefront's LDS operations in order)
                    asm volatile("" ::: "memory");
                }
            }
        }
        first_cb = false;
    }
}

#undef TFLA_WALK_ISSUE_NEXT
#undef TFLA_WALK_ISSUE_PREP
#undef TFLA_WALK_ISSUE_PART
#undef TFLA_WALK_ISSUE_FINISH
#undef TFLA_WALK_WAIT_ITEM
#undef TFLA_WALK_ADVANCE

}  // namespace tfla
