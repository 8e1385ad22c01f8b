// Host-side declarations shared by the translation units of libtfla_mlstm: argument blocks
// of the kernel families and their launchers.  Nothing here is exported.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace tfla {

// ---- chunkwise gates (App. B.2 "Chunkwise Gates", App. B.2 inter-chunk max state) ----------
struct GateArgs {
    const float* i_pre;   // (BH, T)
    const float* f_pre;   // (BH, T)
    const float* m0;      // (BH) or NULL
    int T, L, Nc, variant;
    int Tvalid;           // steps t >= Tvalid of every (batch, head) are padding: forget gate 1, input gate 0
    float qscale;         // 1/sqrt(dqk)
    float softcap;        // c of the gate soft-cap c tanh(x / c) on both pre-activations; 0 = none
    // outputs, all (BH, T) unless noted
    float* wrow;          // log2-domain row term of the intra-chunk weight (includes log2 qscale)
    float* ucol;          // log2-domain column term (i-bar_j - b_j) * log2(e)
    float* sH;            // inter-chunk row scale b-bar_i * qscale
    float* aK;            // a-bar_j = exp(a_j - m_k)
    float* gbar;          // (BH, Nc) g-bar_k
    float* mout;          // combined max state m_t of every step
    float* mfinal;        // (BH) m after the last chunk, or NULL
    float* tmp;           // (BH, 3, T) scratch (values of the pre-pass's arithmetic type: doubles when `precise`)
    // fp32 kernels: pre-pass in double, and the rounding remainders of the two exponents (wrow + wrow_lo and
    // ucol + ucol_lo are the exponents to double accuracy); csum then holds doubles as well.  NULL / 0 otherwise.
    float* wrow_lo; float* ucol_lo; int precise;
    float* csum;          // (BH, 2, Nc) scratch: per-chunk sum of f-bar and max of a
};
hipError_t launch_gates(const GateArgs& a, int BH, hipStream_t s);

struct GateBwdPrepArgs {
    const float* wrow; const float* sH; const float* n_out; const float* m_out;
    float* wrowB; float* sQ;
    long n; int variant; float eps;
    const float* wrow_lo; float* wrowB_lo;   // fp32 kernels: remainders of wrow / wrowB, or NULL
};
hipError_t launch_gate_bwd_prep(const GateBwdPrepArgs& a, hipStream_t s);

struct GateGradArgs {
    const float* partQ; int nbQ;   // (nbQ, BH*T) partial q.dq
    const float* partK; int nbK;   // (nbK, BH*T) partial k.dk
    const float* cdot;             // (BH) <C_T, dC_T> or NULL
    const float* i_pre; const float* f_pre;
    float* d_i; float* d_f;
    double* bsum;                  // (BH, ceil(T / 1024)) scratch: block sums
    int T, variant; long BHT;
    float softcap;                 // as in GateArgs: the gradients are taken through the cap
    // optional anchors of the reverse cumulative sum, one per block of G chunks (G * L <= 2048): its exact value
    // just after the last step of the block, <C, dC> at that boundary, as npart partial sums per boundary
    // (RecArgs::anc_part: (BH, nslot, npart)); NULL = one scan over the whole sequence
    const float* anchor; int L, Nc, G, npart;
};
hipError_t launch_gate_grads(const GateGradArgs& a, int BH, hipStream_t s);

hipError_t launch_fill_zero(float* p, long n, hipStream_t s);
struct FillList { float* p[4]; long n[4]; };     // n[q] = 0: slot unused
hipError_t launch_fill_zero4(const FillList& f, hipStream_t s);
// (BH, T, row) <-> (BH, Tp, row_p) copies for sequence lengths that are not a multiple of the chunk and head
// dimensions between the supported ones (pad.hip); row bytes multiples of 16, pointers 16-byte aligned
hipError_t launch_pad_rows(const void* in, void* out, long BH, int T, int Tp, int row_bytes, int row_bytes_p, hipStream_t s);
hipError_t launch_unpad_rows(const void* in, void* out, long BH, int T, int Tp, int row_bytes, int row_bytes_p, hipStream_t s);
hipError_t launch_pad_scalar(const float* in, float* out, long BH, int T, int Tp, float fill, hipStream_t s);
hipError_t launch_unpad_scalar(const float* in, float* out, long BH, int T, int Tp, hipStream_t s);
hipError_t launch_state_dot(const float* A, const float* Bm, float* out, long per, int BH, hipStream_t s);
// Chunks per block of the anchored forget-gate gradient scan: four (a block has at most 2048 steps); two for heads
// wider than 512, where a row's dot products run over so many terms that the noise of a few chunks already shows
// (behind a norm layer the forget-gate gradient is what survives of an almost complete cancellation).
inline int anchor_chunks(int L, int dwide) {
    if (dwide > 512) return 2;
    return 4 * L <= 2048 ? 4 : (2048 / L > 0 ? 2048 / L : 1);
}

// ---- single recurrent step (Sec. 2.1, Sec. 4.1) ------------------------------------------------
struct StepArgs {
    const void* q; const void* k; const void* v;   // (BH, dqk), (BH, dqk), (BH, dhv)
    const float* i_pre; const float* f_pre;        // (BH)
    const float* C; const float* n; const float* m;   // state before the step; n, m may be NULL (zero)
    float* C_out; float* n_out; float* m_out;      // state after the step; n_out, m_out may be NULL
    void* h;                                       // (BH, dhv)
    int dqk, dhv, variant, dtype;
    float eps;
    float softcap;                                 // gate soft-cap, 0 = none
};
hipError_t launch_step(const StepArgs& a, int BH, hipStream_t s);

// ---- NORM + output gate around the cell (Sec. 2.1 output equation; Sec. 4.1 RMS norm), transfer gains ----
struct NormArgs {
    const void* h;        // (rows, d) cell output h~, element type per dtype
    const void* o_pre;    // (rows, d) output gate pre-activations, or NULL (gate = 1)
    const float* gamma;   // (NH, d) or NULL (1)
    const float* beta;    // (NH, d) or NULL (0); LayerNorm only
    void* y;              // (rows, d)
    long rows;            // B * NH * T, row = (b * NH + head) * T + t
    int NH, T, d, kind, dtype;   // kind 0 = RMS norm, 1 = LayerNorm
    float eps;
};
hipError_t launch_norm_gate_fwd(const NormArgs& a, hipStream_t s);
struct NormBwdArgs {
    const void* h; const void* o_pre; const float* gamma; const float* beta;
    const void* dy;       // (rows, d)
    void* dh;             // (rows, d)
    void* do_pre;         // (rows, d) or NULL
    float* part;          // (BH, row blocks, 2, d) partial sums for d gamma / d beta, or NULL
    int NH, T, d, kind, dtype;
    float eps;
};
hipError_t launch_norm_gate_bwd(const NormBwdArgs& a, int BH, hipStream_t s);
int norm_row_blocks(int T);
struct NormParamGradArgs {
    const float* part; float* dgamma; float* dbeta;   // outputs (NH, d), either may be NULL
    int B, NH, nblk, d;
};
hipError_t launch_norm_param_grad(const NormParamGradArgs& a, hipStream_t s);
struct GainArgs {
    const void* h; const void* v;   // (BH, T, d)
    float* g_before; float* g_after;   // (BH)
    int T, d, kind, dtype;
    float eps;
};
hipError_t launch_transfer_gain(const GainArgs& a, int BH, hipStream_t s);

// ---- inter-chunk recurrence (App. B.2 "Inter-chunk Recurrent Contribution"; App. B.3) -------
// state <- gbar[k] * state + (rs (.) X_k)^T Y_k, chunk by chunk; the state *before* each
// update is written to slot k.
struct RecArgs {
    const void* X;        // (BH, T, d1)
    const void* Y;        // (BH, T, d2)
    const float* rs;      // (BH, T)
    const float* gbar;    // (BH, Nc)
    const float* S0;      // (BH, d1, d2) fp32 or NULL (zero)
    void* stT;            // (BH, Nc, d2, d1) element type DT, or NULL
    void* stN;            // (BH, Nc, d1, d2) element type DT, or NULL
    float* Sfinal;        // (BH, d1, d2) fp32 or NULL
    float* Sfinal2;       // second copy of the final state, or NULL
    const float* n0;      // (BH, d1) or NULL; normaliser vector, forward mLSTMexp only
    float* nst;           // (BH, Nc, d1) or NULL (NULL = no normaliser vector); the bf16 kernel stores the same
                          // bytes as (BH, Nc, 2, d1) bf16: n rounded to bf16, and the rounding remainder
    float* nfinal;        // (BH, d1) or NULL
    int T, L, Nc, d1, d2, reverse;
    // bf16 kernel only, for the anchors of the forget-gate gradient scan (the boundaries between its blocks of anc_G
    // chunks; slot s = the boundary between chunks s * anc_G - 1 and s * anc_G, slot 0 unused):
    //   anc      (forward launch) receives fp32 copies of the state at those boundaries, (BH, nslot, d1 * d2) in the
    //            order of the kernel's accumulator registers;
    //   anc_in   (reversed launch) = what the forward launch left in anc: every wavefront multiplies its part of it
    //            with its fp32 accumulators (the same element order) and leaves the partial inner product in
    //   anc_part (BH, nslot, npart), npart = (d1 / 64) * (d2 / 32) = rec_anchor_parts().
    // NULL = none.
    float* anc; const float* anc_in; float* anc_part; int anc_G;
};
hipError_t launch_recurrent(const RecArgs& a, int BH, int dtype, hipStream_t s);
// dQ and dK weight the same matrix dH V^T.  Where the contraction that forms it (over d_hv) is wider than this, the dQ
// kernel stores its weighted tiles E (L x L per chunk) and the dK kernel reads them; up to this width both kernels
// form the matrix themselves, because E is then more bytes than the operands it replaces (measured at
// d_hv = 64 / 128 / 256: -19 % / -8 % / -1 % per step without E; at 512: +3 %).
#ifndef TFLA_NOE_MAX_D1
#define TFLA_NOE_MAX_D1 256
#endif
inline bool tile_shares_E(int dhv) { return dhv > TFLA_NOE_MAX_D1; }

inline int rec_anchor_parts(int d1, int d2) { return (d1 / 64) * (d2 / 32); }

// ---- intra-chunk tiled kernels (Sec. 3, App. C.3 Alg. 1, App. C.4) ---------------------------
// out[r,:] = sum_c exp2(wrow[r] + wcol[c]) * (X_r . Y_c) * Z_c  (causal within the chunk)
//            + srow[r] * (X_r St)
enum { MODE_H = 0, MODE_DV = 1, MODE_DQ = 2, MODE_DK = 3 };
struct TileArgs {
    const void* X; const void* Y;   // (BH, T, d1)
    const void* Z; void* Out;       // Z: (BH, T, d2); Out: (BH, out_T, out_ld), see below
    const float* wrow; const float* wcol; const float* srow;   // (BH, T)
    const void* St;                 // (BH, Nc, d2, d1)
    int T, L, Nc, d1, d2;
    int kc_desc;                    // bf16 kernels: walk the chunks last to first (set by the launcher)
    // MODE_H, mLSTMexp: normaliser
    int variant; float eps;
    const float* nstate;            // (BH, Nc, d1); bf16 kernels: (BH, Nc, 2, d1) bf16 as RecArgs::nst
    const float* mout;              // (BH, T)
    float* nout;                    // (BH, T) or NULL
    // MODE_H, mLSTMexp: the backward pass's row weights with 1 / h_denom folded in (what gate_bwd_prep_kernel
    // computes from n_out and m_out), written here while the denominator is at hand; (BH, T) each, or NULL
    float* wrowB_out; float* sQ_out;
    // MODE_DQ / MODE_DK: partial row dots  sum_n out[r,n] * dotwith[r,n]
    const void* dotwith;            // (BH, T, d2)
    float* dotpart;                 // (d2/BD2, BH*T)
    // bf16 MODE_DQ writes, bf16 MODE_DK reads: the weighted matrix E of every chunk, (BH, Nc, L, L)
    void* E;
    // Contraction widths above 512 (bf16): every term of the result is linear in the products over d1, so the
    // launcher runs the kernel once per 512-wide half and the halves meet in fp32.  The caller provides the
    // buffers; the remaining fields are filled in by the launcher.
    float* part_acc;                // (BH, T, d2) unnormalised result of the first half
    float* part_nrm;                // (BH, T) its share of the normaliser (MODE_H, mLSTMexp)
    void* E2;                       // the second half's E (MODE_DQ writes, MODE_DK reads)
    const float* acc_in; const float* nrm_in;   // add these to the accumulators / normaliser before the epilogue
    float* acc_out; float* nrm_out;             // store the raw accumulators / normaliser instead of the output
    // The output goes straight into the caller's tensor also when the kernels run on a zero-padded copy of the
    // problem: only steps t < out_T and columns < out_cols are stored, rows are out_ld elements apart
    // (out_T = T, out_ld = out_cols = d2 when nothing is padded).  out_cols is a multiple of 8.
    int out_T, out_ld, out_cols;
    // fp32 kernels: rounding remainders of the row and column exponents (the weight is exp2 of the sum of all four),
    // and where MODE_H leaves the remainder that belongs to wrowB_out; NULL = none
    const float* wrow_lo; const float* wcol_lo; float* wrowB_lo_out;
    // bf16 kernels, filled in by the launcher: what the decomposition of the linear workgroup id divides by --
    // batch*head count, slices per XCD, and for each divisor its log2 when it is a power of two, else -1
    // (a division by a run-time value costs the start of every workgroup some forty instructions)
    int dec_bh, dec_bpx, sh_gx, sh_gy, sh_bpx, sh_nc;
    // bf16 MODE_H, fused layer output (Sec. 2.1, hidden-state output equation: y = sigma(o~) (.) NORM(h~)), where one
    // workgroup holds whole rows of h~ (d2 equal to the width of its column block, nothing padded): fz_y != NULL makes
    // the kernel store y (BH, T, d2) next to h~.  fz_o: (BH, T, d2) gate pre-activations or NULL (gate = 1);
    // fz_gamma / fz_beta: (fz_NH, d2) or NULL; fz_kind 0 = RMS norm, 1 = LayerNorm (as NormArgs).
    const void* fz_o; const float* fz_gamma; const float* fz_beta; void* fz_y;
    int fz_kind, fz_NH; float fz_eps;
};
// what the layer's forward entry point hands down to the H kernel when the fusion applies
struct LayerFuse {
    const void* o_pre; const float* gamma; const float* beta; void* y;
    int kind, NH; float eps;
};
template <int MODE> hipError_t launch_tile_mode(const TileArgs& a, int BH, int dtype, hipStream_t s);
// d2 block of a tiled kernel (mode MODE_*) with contraction width d1.  128 columns keep a bf16
// wavefront within 256 registers, so that two workgroups share a CU when d1 <= 256.  The bf16 dQ and
// dK kernels take a 256-wide block when d1 = 512 (one workgroup per CU anyway): half as many
// workgroups fetch the same X rows and column tiles, and dQ computes S once per 256 columns.
// (The 256-wide instantiations exist for the four-wavefront workgroups only, i.e. for chunk sizes that are
// multiples of 128.)
// tile_width_override (set through tfla_tile_width, a measurement aid for tile-size sweeps): 0 = the choice
// described above; 64 / 128 force that width wherever it divides d2; 256 changes nothing (it is already taken
// wherever it is built).  The workspace layout depends on the width, so it must not change between the
// workspace query, the forward call and the backward call of one step.
extern int tile_width_override;
inline int tile_bd2(int d1, int d2, int dtype, int mode, int L) {
    const int ov = tile_width_override;
    if (dtype == 1 && (ov == 64 || ov == 128) && d2 % ov == 0) return ov;
    if (dtype == 1 && (mode == MODE_DK || mode == MODE_DQ) && d1 == 512 && d2 % 256 == 0 && L % 128 == 0) return 256;
    // (contractions over 1024 columns run as 512-wide halves with 128- or 64-wide blocks)
    if (d2 % 128 == 0) return 128;
    return 64;
}
// the fused layer output needs whole rows of h~ in one workgroup of the H kernel
inline bool layer_fusion_applies(int dqk, int dhv, int dtype, int L) {
    return dtype == 1 && (dhv == 64 || dhv == 128) && tile_bd2(dqk, dhv, dtype, MODE_H, L) == dhv;
}

}  // namespace tfla
