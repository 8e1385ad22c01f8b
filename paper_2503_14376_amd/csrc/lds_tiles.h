// bf16 tiles in LDS for gfx950: filled asynchronously by global->LDS loads (no registers, no
// VALU work), read either as k-contiguous MFMA fragments (ds_read_b128) or, when the
// contraction index is the tile's row index, through the transposing LDS read
// (ds_read_b64_tr_b16).  Tiles are stored unpadded in their natural row-major layout; bank
// conflicts are avoided by XOR-swizzling the 16-byte chunks of each row.
//
// global->LDS load (global_load_lds_dwordx4): every lane supplies its own 16-byte global
// address; the 64 results land at consecutive 16-byte slots from a wave-uniform LDS address.
//
// transposing read (ds_read_b64_tr_b16), per group of 16 lanes: source lane j supplies the
// address of four consecutive 16-bit elements; result lane i receives, for e = 0..3, element
// (i & 3) of source lane 4e + (i >> 2).  With source lane j pointing at row k0 + (j >> 2),
// columns n0 + 4 (j & 3) .. +3 of a row-major tile, result lane i holds rows k0..k0+3 of
// column n0 + i: four consecutive contraction indices for the lane's own column, which is
// what an MFMA operand needs.
#pragma once
#include "tfla_device.h"

namespace tfla {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

enum { SWZ_K = 0, SWZ_T = 1 };   // tile read by k-contiguous fragments / by transposing reads

// XOR mask (in 16-byte chunks) applied to the chunk index of row r; CPR = chunks per row.
template <int KIND, int CPR> __device__ __forceinline__ int swz_mask(int r) {
    if (KIND == SWZ_K) {
        if (CPR >= 16) return r & 15;
        if (CPR == 8) return (r >> 1) & 7;
        return (r >> 2) & 3;
    }
    if (CPR >= 16) return 4 * (r & 3);
    return 4 * ((r >> 1) & 1);
}

// 32-bit LDS address of a __shared__ object
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// One global->LDS load of 64 x 16 bytes: lane l copies 16 bytes from gbase + voff(l) to LDS
// address lds_uniform + 16 * l.  Issued through inline assembly so that the compiler's
// wait-count insertion does not serialise later LDS reads of *other* pipeline stages behind
// it; the kernels order these loads themselves with wait_vmcnt + barrier.
__device__ __forceinline__ void dma16(const void* gbase_uniform, uint32_t voff, uint32_t lds_uniform) {
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_uniform);
    const uint64_t gb = (uint64_t)(uintptr_t)gbase_uniform;
    // readfirstlane returns a signed int: go through uint32_t so the low half is not sign-extended
    const uint32_t glo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gb);
    const uint32_t ghi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gb >> 32));
    const uint64_t gu = (uint64_t)glo | ((uint64_t)ghi << 32);
    // s_nop 4: the hardware needs 5 wait states between a write of an SGPR (the base address, M0) and
    // a vector-memory instruction that reads it; the compiler's hazard recogniser cannot see inside
    // the asm, so the distance is guaranteed here
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(la), "v"(voff), "s"(gu) : "memory", "m0");
}

// The same load without the "memory" clobber: the compiler may move ordinary LDS reads and MFMAs
// across it (it stays ordered with the kernels' barriers and waits, which are volatile asm too).
// For loads that are issued between matrix instructions into a stage nobody reads in that phase.
__device__ __forceinline__ void dma16_free(const void* gbase_uniform, uint32_t voff, uint32_t lds_uniform) {
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_uniform);
    const uint64_t gb = (uint64_t)(uintptr_t)gbase_uniform;
    const uint32_t glo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gb);
    const uint32_t ghi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gb >> 32));
    const uint64_t gu = (uint64_t)glo | ((uint64_t)ghi << 32);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(la), "v"(voff), "s"(gu) : "m0");
}

// The two loads above with the non-temporal hint: for operands that exactly one workgroup of the launch reads,
// so that they do not displace what several workgroups share from the caches.
__device__ __forceinline__ void dma16_nt(const void* gbase_uniform, uint32_t voff, uint32_t lds_uniform) {
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_uniform);
    const uint64_t gb = (uint64_t)(uintptr_t)gbase_uniform;
    const uint32_t glo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gb);
    const uint32_t ghi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gb >> 32));
    const uint64_t gu = (uint64_t)glo | ((uint64_t)ghi << 32);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :: "s"(la), "v"(voff), "s"(gu) : "memory", "m0");
}
__device__ __forceinline__ void dma16_free_nt(const void* gbase_uniform, uint32_t voff, uint32_t lds_uniform) {
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_uniform);
    const uint64_t gb = (uint64_t)(uintptr_t)gbase_uniform;
    const uint32_t glo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gb);
    const uint32_t ghi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gb >> 32));
    const uint64_t gu = (uint64_t)glo | ((uint64_t)ghi << 32);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :: "s"(la), "v"(voff), "s"(gu) : "m0");
}

// Same for 64 x 4 bytes: lane l copies one dword to LDS address lds_uniform + 4 * l.
__device__ __forceinline__ void dma4(const void* gbase_uniform, uint32_t voff, uint32_t lds_uniform) {
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_uniform);
    const uint64_t gb = (uint64_t)(uintptr_t)gbase_uniform;
    const uint32_t glo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gb);
    const uint32_t ghi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gb >> 32));
    const uint64_t gu = (uint64_t)glo | ((uint64_t)ghi << 32);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(la), "v"(voff), "s"(gu) : "memory", "m0");
}

// workgroup barrier without the fence a __syncthreads() carries (that fence would wait for
// every outstanding global->LDS load, i.e. drain the pipeline)
__device__ __forceinline__ void barrier_nofence() { asm volatile("s_barrier" ::: "memory"); }

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// wait until at most n (wave-uniform, 0..63) vector-memory operations of this wave are pending
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
    switch (n) {
#define TFLA_W(k) case k: wait_vmcnt<k>(); break;
        TFLA_W(0) TFLA_W(1) TFLA_W(2) TFLA_W(3) TFLA_W(4) TFLA_W(5) TFLA_W(6) TFLA_W(7) TFLA_W(8) TFLA_W(9)
        TFLA_W(10) TFLA_W(11) TFLA_W(12) TFLA_W(13) TFLA_W(14) TFLA_W(15) TFLA_W(16) TFLA_W(17) TFLA_W(18)
        TFLA_W(19) TFLA_W(20) TFLA_W(21) TFLA_W(22) TFLA_W(23) TFLA_W(24) TFLA_W(25) TFLA_W(26) TFLA_W(27)
        TFLA_W(28) TFLA_W(29) TFLA_W(30) TFLA_W(31) TFLA_W(32) TFLA_W(33) TFLA_W(34) TFLA_W(35) TFLA_W(36)
        TFLA_W(37) TFLA_W(38) TFLA_W(39) TFLA_W(40) TFLA_W(41) TFLA_W(42) TFLA_W(43) TFLA_W(44) TFLA_W(45)
        TFLA_W(46) TFLA_W(47) TFLA_W(48) TFLA_W(49) TFLA_W(50) TFLA_W(51) TFLA_W(52) TFLA_W(53) TFLA_W(54)
        TFLA_W(55) TFLA_W(56) TFLA_W(57) TFLA_W(58) TFLA_W(59) TFLA_W(60) TFLA_W(61) TFLA_W(62) TFLA_W(63)
#undef TFLA_W
        default: wait_vmcnt<0>(); break;
    }
}

// Asynchronous fill of a [ROWS][COLS] bf16 tile.  init() precomputes the per-lane byte offsets
// into the global tile (they depend only on the global row stride), issue() launches this
// wave's share of the loads: N instructions of 64 x 16 bytes.
template <int ROWS, int COLS, int NT, int KIND> struct DmaTile {
    static constexpr int CPR = COLS / 8, TOTAL = ROWS * CPR, NWV = NT / 64, N = TOTAL / (64 * NWV);
    static_assert(TOTAL % (64 * NWV) == 0 && N >= 1, "tile must split into whole wave loads");
    uint32_t goff[N];
    __device__ __forceinline__ void init(long gstride_elems, int tid) {
        const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int q = (wave + j * NWV) * 64 + lane;
            const int r = q / CPR, pc = q % CPR;
            const int c = pc ^ swz_mask<KIND, CPR>(r);
            goff[j] = (uint32_t)((r * gstride_elems + c * 8) * 2);
        }
    }
    // gtile: wave-uniform address of the tile's first element; lds: LDS address of the tile
    // ONCE: with the non-temporal hint (a tile that no other workgroup reads)
    template <bool ONCE = false>
    __device__ __forceinline__ void issue(const bf16_t* gtile, uint32_t lds, int tid) const {
        const int wave = tid >> 6;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            if constexpr (ONCE) dma16_nt(gtile, goff[j], lds + (wave + j * NWV) * 1024);
            else dma16(gtile, goff[j], lds + (wave + j * NWV) * 1024);
        }
    }
    // the loads j = part, part + nparts, ... only (part, nparts compile-time in the callers)
    template <bool ONCE = false>
    __device__ __forceinline__ void issue_part(const bf16_t* gtile, uint32_t lds, int tid, int part, int nparts) const {
        const int wave = tid >> 6;
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j % nparts == part) {
                if constexpr (ONCE) dma16_free_nt(gtile, goff[j], lds + (wave + j * NWV) * 1024);
                else dma16_free(gtile, goff[j], lds + (wave + j * NWV) * 1024);
            }
    }
};

// Per-lane byte offsets for k-contiguous fragment reads from a SWZ_K tile with COLS columns:
// fragment (step ks, lane group g) of row (32 * blk + l32).
template <int COLS> struct KFragReader {
    static constexpr int CPR = COLS / 8, XM = CPR >= 16 ? 16 : CPR, NJ = XM / 2, RB = COLS * 2;
    uint32_t off[NJ];
    __device__ __forceinline__ void init(int l32, int g) {
        const int x = swz_mask<SWZ_K, CPR>(l32) ^ g;
#pragma unroll
        for (int j = 0; j < NJ; ++j) off[j] = (uint32_t)(l32 * RB + (((2 * j) ^ x) * 16));
    }
    // KS and BLK are compile-time in all callers (unrolled loops), so the address is off[] + constant
    __device__ __forceinline__ bf16x8 load(const char* tile, int ks, int blk) const {
        return *reinterpret_cast<const bf16x8*>(tile + off[ks % NJ] + (ks / NJ) * (XM * 16) + blk * 32 * RB);
    }
};

// Per-lane byte offsets for transposing fragment reads from a SWZ_T tile [k rows][COLS n]:
// the fragment of column block nb whose eight k values are rows
//   rowconst + ROWG * g + (lane & 15) / 4 + {0..3}  and the same + 8 * HSTEP ... (see load()).
template <int COLS> struct TFragReader {
    static constexpr int CPR = COLS / 8, NB = COLS / 32, NJ = NB < 4 ? NB : 4, RB = COLS * 2;
    uint32_t off[NJ];
    // rowg: row offset contributed by the lane group g (4 for operands chained to an MFMA
    // result, 8 for the natural k order)
    __device__ __forceinline__ void init(int lane, int rowg) {
        const int i = lane & 15, m = lane >> 4, g = lane >> 5;
        const int row = rowg * g + (i >> 2);
        const int f = swz_mask<SWZ_T, CPR>(i >> 2);
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            off[j] = (uint32_t)(row * RB + (((4 * j) ^ f) + 2 * (m & 1) + ((i & 3) >> 1)) * 16 + (i & 1) * 8);
    }
    // byte offset of column block nb for this lane; for callers whose nb is not a compile-time value
    // (indexing off[] with a run-time value would push the array out of registers)
    __device__ __forceinline__ uint32_t block_offset(int nb) const {
        uint32_t o = off[0];
#pragma unroll
        for (int j = 1; j < NJ; ++j) o = (nb % NJ == j) ? off[j] : o;
        return o + (uint32_t)(nb / NJ) * 256u;
    }
    // the same fragment read from a precomputed block_offset()
    static __device__ __forceinline__ bf16x8 load_at(const char* tile, uint32_t boff, int rowA, int rowB) {
        const char* p = tile + boff;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4*)(p + rowA * RB));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4*)(p + rowB * RB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    // rows rowA.. and rowB.. (multiples of 4, before the lane part) give elements 0..3 and 4..7
    __device__ __forceinline__ bf16x8 load(const char* tile, int nb, int rowA, int rowB) const {
        const char* p = tile + off[nb % NJ] + (nb / NJ) * 256;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4*)(p + rowA * RB));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4*)(p + rowB * RB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
};

}  // namespace tfla
