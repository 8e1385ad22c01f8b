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

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// two fp32 values -> one dword of two bf16 (round to nearest even), a single v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    bf16x2 v = {(bf16_t)lo, (bf16_t)hi};
    return __builtin_bit_cast(uint32_t, v);
}

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
// Split (prefetching) forms of the two stagers: load() issues the global loads into
// registers, store() writes them to LDS later, so the loads of the next tile are in flight
// while the current tile is being multiplied.
// ---------------------------------------------------------------------------------------
template <typename DT, int ROWS, int COLS, int NT> struct RowsPrefetch {
    static constexpr int EPC = 16 / (int)sizeof(DT), CPR = COLS / EPC, TOTAL = ROWS * CPR;
    static constexpr int N = (TOTAL + NT - 1) / NT;
    u32x4 r[N];
    __device__ __forceinline__ void load(const DT* g, long gstride, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = tid + i * NT;
            if (TOTAL % NT == 0 || c < TOTAL)
                r[i] = *reinterpret_cast<const u32x4*>(g + (long)(c / CPR) * gstride + (c % CPR) * EPC);
        }
    }
    __device__ __forceinline__ void store(DT* lds, int lstride, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = tid + i * NT;
            if (TOTAL % NT == 0 || c < TOTAL)
                *reinterpret_cast<u32x4*>(lds + (c / CPR) * lstride + (c % CPR) * EPC) = r[i];
        }
    }
};

template <typename DT, int ROWS, int COLS, int NT, bool PERM> struct TrPrefetch;

template <int ROWS, int COLS, int NT, bool PERM> struct TrPrefetch<bf16_t, ROWS, COLS, NT, PERM> {
    static constexpr int UNITS = (ROWS / 8) * (COLS / 2), N = (UNITS + NT - 1) / NT;
    uint32_t w[N][8];
    __device__ __forceinline__ void load(const bf16_t* g, long gstride, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int cp = idx % (COLS / 2), u = idx / (COLS / 2);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    w[i][e] = *reinterpret_cast<const uint32_t*>(g + (long)tr_src_row<PERM>(u, e) * gstride + 2 * cp);
            }
        }
    }
    // per-unit row scales held in registers (rs[i][e] = scale of source row 8u+e; PERM = false)
    __device__ __forceinline__ void load_scales(float (&rs)[N][8], const float* g, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int u = idx / (COLS / 2);
                const f32x4 a = *reinterpret_cast<const f32x4*>(g + 8 * u), b = *reinterpret_cast<const f32x4*>(g + 8 * u + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) { rs[i][e] = a[e]; rs[i][4 + e] = b[e]; }
            }
        }
    }
    __device__ __forceinline__ void store_scaled(bf16_t* lds, int lstride, const float (&rs)[N][8], int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int cp = idx % (COLS / 2), u = idx / (COLS / 2);
                uint32_t x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    x[e] = bf16_bits_rne(bf16_lo_to_f32(w[i][e]) * rs[i][e]) | (bf16_bits_rne(bf16_hi_to_f32(w[i][e]) * rs[i][e]) << 16);
                u32x4 lo, hi;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    lo[d] = (x[2 * d] & 0xffffu) | (x[2 * d + 1] << 16);
                    hi[d] = (x[2 * d] >> 16) | (x[2 * d + 1] & 0xffff0000u);
                }
                *reinterpret_cast<u32x4*>(lds + (2 * cp) * lstride + 8 * u) = lo;
                *reinterpret_cast<u32x4*>(lds + (2 * cp + 1) * lstride + 8 * u) = hi;
            }
        }
    }
    // rowscale (LDS or global, indexed by source row) may be null
    template <bool SCALE>
    __device__ __forceinline__ void store(bf16_t* lds, int lstride, const float* rowscale, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int cp = idx % (COLS / 2), u = idx / (COLS / 2);
                uint32_t x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    x[e] = w[i][e];
                    if (SCALE) {
                        const float s = rowscale[tr_src_row<PERM>(u, e)];
                        x[e] = bf16_bits_rne(bf16_lo_to_f32(x[e]) * s) | (bf16_bits_rne(bf16_hi_to_f32(x[e]) * s) << 16);
                    }
                }
                u32x4 lo, hi;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    lo[d] = (x[2 * d] & 0xffffu) | (x[2 * d + 1] << 16);
                    hi[d] = (x[2 * d] >> 16) | (x[2 * d + 1] & 0xffff0000u);
                }
                *reinterpret_cast<u32x4*>(lds + (2 * cp) * lstride + 8 * u) = lo;
                *reinterpret_cast<u32x4*>(lds + (2 * cp + 1) * lstride + 8 * u) = hi;
            }
        }
    }
};

template <int ROWS, int COLS, int NT, bool PERM> struct TrPrefetch<float, ROWS, COLS, NT, PERM> {
    static constexpr int UNITS = (ROWS / 8) * COLS, N = (UNITS + NT - 1) / NT;
    float w[N][8];
    __device__ __forceinline__ void load(const float* g, long gstride, int tid) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int col = idx % COLS, u = idx / COLS;
#pragma unroll
                for (int e = 0; e < 8; ++e) w[i][e] = g[(long)tr_src_row<PERM>(u, e) * gstride + col];
            }
        }
    }
    __device__ __forceinline__ void load_scales(float (&rs)[N][8], const float* g, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int u = idx / COLS;
                const f32x4 a = *reinterpret_cast<const f32x4*>(g + 8 * u), b = *reinterpret_cast<const f32x4*>(g + 8 * u + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) { rs[i][e] = a[e]; rs[i][4 + e] = b[e]; }
            }
        }
    }
    __device__ __forceinline__ void store_scaled(float* lds, int lstride, const float (&rs)[N][8], int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int col = idx % COLS, u = idx / COLS;
                f32x4 a = {w[i][0] * rs[i][0], w[i][1] * rs[i][1], w[i][2] * rs[i][2], w[i][3] * rs[i][3]};
                f32x4 b = {w[i][4] * rs[i][4], w[i][5] * rs[i][5], w[i][6] * rs[i][6], w[i][7] * rs[i][7]};
                *reinterpret_cast<f32x4*>(lds + col * lstride + 8 * u) = a;
                *reinterpret_cast<f32x4*>(lds + col * lstride + 8 * u + 4) = b;
            }
        }
    }
    template <bool SCALE>
    __device__ __forceinline__ void store(float* lds, int lstride, const float* rowscale, int tid) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int idx = tid + i * NT;
            if (UNITS % NT == 0 || idx < UNITS) {
                const int col = idx % COLS, u = idx / COLS;
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = SCALE ? w[i][e] * rowscale[tr_src_row<PERM>(u, e)] : w[i][e];
                f32x4 a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
                *reinterpret_cast<f32x4*>(lds + col * lstride + 8 * u) = a;
                *reinterpret_cast<f32x4*>(lds + col * lstride + 8 * u + 4) = b;
            }
        }
    }
};

// four consecutive elements as one store (8 bytes of bf16, 16 bytes of fp32)
__device__ __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
    uint2 w;
    w.x = bf16_bits_rne(a) | (bf16_bits_rne(b) << 16);
    w.y = bf16_bits_rne(c) | (bf16_bits_rne(d) << 16);
    *reinterpret_cast<uint2*>(p) = w;
}
__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d) {
    f32x4 w = {a, b, c, d};
    *reinterpret_cast<f32x4*>(p) = w;
}

// Workgroups are handed to the 8 XCDs round-robin by their linear id.  This remaps the
// hardware id so that each XCD (and its L2) works on a contiguous range of logical ids.
__device__ __forceinline__ unsigned xcd_remap(unsigned hw, unsigned total) {
    if (total % 8u != 0u) return hw;
    return (hw % 8u) * (total / 8u) + hw / 8u;
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
