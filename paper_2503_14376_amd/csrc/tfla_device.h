// Device-side building blocks for the gfx950 mLSTM kernels: MFMA fragments, LDS staging
// (natural and transposed), small wavefront reductions.
//
// Fragment convention used by every kernel here.  A "fragment" is 8 consecutive elements
// along the contraction index k that one lane feeds to the matrix core: lane l (0..63) of a
// 32x32 MFMA owns row/column (l & 31) of its operand and the k-group (l >> 5).  For bf16
// one fragment is the 8xbf16 operand of v_mfma_f32_32x32x16_bf16 (k = 16*step + 8*group + e);
// for fp32 the same 8 elements are fed one at a time to eight v_mfma_f32_32x32x2_f32.
// Both operands of a product use the same (step, group, e) -> k mapping, so the result does
// not depend on which k each slot really is.  The 32x32 fp32 result keeps, in register v of
// lane l, element (row 8*(v/4) + 4*(l>>5) + (v&3), column l & 31).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tfla {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int acc_row(int v, int grp) { return 8 * (v >> 2) + 4 * grp + (v & 3); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ uint32_t bf16_bits_rne(float x) {
    // round-to-nearest-even conversion, as bits in the low half
    bf16_t b = (bf16_t)x;
    return (uint32_t)__builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ float bf16_lo_to_f32(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

template <typename DT> struct Elem;

template <> struct Elem<bf16_t> {
    static constexpr int PAD = 8;  // elements of padding per LDS row (16 bytes)
    struct frag { bf16x8 v; };
    static __device__ __forceinline__ frag load(const bf16_t* p) {
        frag f; f.v = *reinterpret_cast<const bf16x8*>(p); return f;
    }
    static __device__ __forceinline__ f32x16 mma(const frag& a, const frag& b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, c, 0, 0, 0);
    }
    static __device__ __forceinline__ frag pack(const float* p) {
        frag f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f.v[e] = (bf16_t)p[e];
        return f;
    }
    static __device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
    static __device__ __forceinline__ bf16_t from_f32(float x) { return (bf16_t)x; }
    static __device__ __forceinline__ float frag_elem(const frag& f, int e) { return (float)f.v[e]; }
};

template <> struct Elem<float> {
    static constexpr int PAD = 4;
    struct frag { float v[8]; };
    static __device__ __forceinline__ frag load(const float* p) {
        frag f;
        f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { f.v[e] = a[e]; f.v[4 + e] = b[e]; }
        return f;
    }
    static __device__ __forceinline__ f32x16 mma(const frag& a, const frag& b, f32x16 c) {
#pragma unroll
        for (int e = 0; e < 8; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[e], b.v[e], c, 0, 0, 0);
        return c;
    }
    static __device__ __forceinline__ frag pack(const float* p) {
        frag f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f.v[e] = p[e];
        return f;
    }
    static __device__ __forceinline__ float to_f32(float x) { return x; }
    static __device__ __forceinline__ float from_f32(float x) { return x; }
    static __device__ __forceinline__ float frag_elem(const frag& f, int e) { return f.v[e]; }
};

// ---------------------------------------------------------------------------------------
// Natural staging: copy a [ROWS][COLS] tile (row stride gstride elements in global memory)
// into LDS with row stride lstride, 16 bytes per thread and step.
// ---------------------------------------------------------------------------------------
template <typename DT, int ROWS, int COLS, int NT>
__device__ __forceinline__ void stage_rows(DT* lds, int lstride, const DT* g, long gstride, int tid) {
    constexpr int EPC = 16 / (int)sizeof(DT);   // elements per 16-byte chunk
    constexpr int CPR = COLS / EPC;             // chunks per row
    constexpr int TOTAL = ROWS * CPR;
#pragma unroll
    for (int c = tid; c < TOTAL; c += NT) {
        const int r = c / CPR, cc = c % CPR;
        const u32x4 w = *reinterpret_cast<const u32x4*>(g + (long)r * gstride + cc * EPC);
        *reinterpret_cast<u32x4*>(lds + r * lstride + cc * EPC) = w;
    }
}

// Source row of slot (8*u + e) of a transposed tile.  With PERM the eight rows of a group
// are those that registers 8c..8c+7 of a 32x32 MFMA result hold for lane group g, so that a
// result tile can be fed back as an operand against this tile without leaving registers.
template <bool PERM> __device__ __forceinline__ int tr_src_row(int u, int e) {
    if (!PERM) return 8 * u + e;
    const int st = u >> 2, c = (u >> 1) & 1, g = u & 1;
    return 32 * st + 16 * c + 4 * g + (e & 3) + 8 * (e >> 2);
}

// ---------------------------------------------------------------------------------------
// Transposed staging: global tile [ROWS][COLS] (ROWS = contraction index, contiguous COLS)
// -> LDS [COLS][ROWS (+pad)], i.e. contraction index contiguous per LDS row.  Optional
// per-source-row scale (fp32 multiply, rounded back to the element type).
// ---------------------------------------------------------------------------------------
template <int ROWS, int COLS, int NT, bool PERM, bool SCALE>
__device__ __forceinline__ void stage_transposed(bf16_t* lds, int lstride, const bf16_t* g, long gstride,
                                                 const float* rowscale, int tid) {
    constexpr int UNITS = (ROWS / 8) * (COLS / 2);
#pragma unroll
    for (int idx = tid; idx < UNITS; idx += NT) {
        const int cp = idx % (COLS / 2), u = idx / (COLS / 2);
        uint32_t w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            w[e] = *reinterpret_cast<const uint32_t*>(g + (long)tr_src_row<PERM>(u, e) * gstride + 2 * cp);
        if (SCALE) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float s = rowscale[tr_src_row<PERM>(u, e)];
                const uint32_t lo = bf16_bits_rne(bf16_lo_to_f32(w[e]) * s);
                const uint32_t hi = bf16_bits_rne(bf16_hi_to_f32(w[e]) * s);
                w[e] = lo | (hi << 16);
            }
        }
        u32x4 lo, hi;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            lo[d] = (w[2 * d] & 0xffffu) | (w[2 * d + 1] << 16);
            hi[d] = (w[2 * d] >> 16) | (w[2 * d + 1] & 0xffff0000u);
        }
        *reinterpret_cast<u32x4*>(lds + (2 * cp) * lstride + 8 * u) = lo;
        *reinterpret_cast<u32x4*>(lds + (2 * cp + 1) * lstride + 8 * u) = hi;
    }
}

template <int ROWS, int COLS, int NT, bool PERM, bool SCALE>
__device__ __forceinline__ void stage_transposed(float* lds, int lstride, const float* g, long gstride,
                                                 const float* rowscale, int tid) {
    constexpr int UNITS = (ROWS / 8) * COLS;
#pragma unroll
    for (int idx = tid; idx < UNITS; idx += NT) {
        const int col = idx % COLS, u = idx / COLS;
        float w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            w[e] = g[(long)tr_src_row<PERM>(u, e) * gstride + col];
            if (SCALE) w[e] *= rowscale[tr_src_row<PERM>(u, e)];
        }
        f32x4 a = {w[0], w[1], w[2], w[3]}, b = {w[4], w[5], w[6], w[7]};
        *reinterpret_cast<f32x4*>(lds + col * lstride + 8 * u) = a;
        *reinterpret_cast<f32x4*>(lds + col * lstride + 8 * u + 4) = b;
    }
}

// ---------------------------------------------------------------------------------------
// Wavefront helpers (64 lanes)
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
// sum over the 32 lanes that share (lane >> 5)
__device__ __forceinline__ float half_sum(float x) {
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

}  // namespace tfla
