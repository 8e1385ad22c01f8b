// C ABI of libtfla_mlstm: argument validation, workspace layout and the kernel sequence of
// the forward and backward pass.  See include/tfla_mlstm.h for the contract.
#include "../../include/tfla_mlstm.h"
#include "tfla_internal.h"

#include <math.h>

#include <mutex>

using namespace tfla;

namespace tfla { int tile_width_override = 0; }

namespace {

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct Dims {
    int B, NH, T, dqk, dhv, L, variant, dtype;   // T: whole chunks (the padded length when the caller's is ragged)
    long BH, BHT;
    int Nc;
    size_t esz;
};

// the head dimension the kernels run a caller's head dimension at (zero-padded columns in between)
// a contraction wider than the tiled kernels hold in registers runs as two launches that meet in fp32
inline bool contraction_split(int d1, int dtype) { return dtype == TFLA_BF16 ? d1 > 512 : d1 > 256; }
inline int kernel_dim(int d) { return d <= 64 ? 64 : (d <= 128 ? 128 : (d <= 256 ? 256 : (d <= 512 ? 512 : 1024))); }

// core = true: the kernels' own widths only (what the kernel sequences are called with)
int check_dims(int direction, int B, int NH, int T, int dqk, int dhv, int chunk, int variant, int dtype, bool core = false) {
    if (direction != TFLA_FWD && direction != TFLA_BWD) return TFLA_ERR_ENUM;
    if (variant != TFLA_EXP && variant != TFLA_SIG) return TFLA_ERR_ENUM;
    if (dtype != TFLA_F32 && dtype != TFLA_BF16) return TFLA_ERR_ENUM;
    if (B <= 0 || NH <= 0 || T <= 0 || dqk <= 0 || dhv <= 0) return TFLA_ERR_SHAPE;
    const int dmax = dtype == TFLA_BF16 ? 1024 : 512;
    auto ok_d = [&](int d) {
        if (d > dmax || d % 8 != 0) return false;
        return !core || d == 64 || d == 128 || d == 256 || d == 512 || d == 1024;
    };
    if (!ok_d(dqk) || !ok_d(dhv)) return TFLA_ERR_SHAPE;
    if ((long)B * NH > 65535) return TFLA_ERR_SHAPE;
    if (chunk < 64 || chunk > 2048 || chunk % 64 != 0) return TFLA_ERR_CHUNK;
    const int nc = (T + chunk - 1) / chunk;
    if (nc > 4096) return TFLA_ERR_CHUNK;
    // workgroups of the largest tiled launch (one-dimensional grid): column blocks x row blocks x chunks x (batch*head)
    const long dmx = kernel_dim(dqk > dhv ? dqk : dhv);
    if ((long)B * NH * nc * (dmx / 64) * (chunk / 64) > 2147483647L) return TFLA_ERR_SHAPE;
    return TFLA_OK;
}

Dims make_dims(int B, int NH, int T, int dqk, int dhv, int chunk, int variant, int dtype) {
    Dims d;
    d.Nc = (T + chunk - 1) / chunk;
    d.B = B; d.NH = NH; d.T = d.Nc * chunk; d.dqk = dqk; d.dhv = dhv; d.L = chunk; d.variant = variant; d.dtype = dtype;
    d.BH = (long)B * NH; d.BHT = d.BH * d.T;
    d.esz = dtype == TFLA_BF16 ? 2 : 4;
    return d;
}

// Bump allocator over the caller's workspace.
struct Carver {
    char* base; size_t off;
    explicit Carver(void* p) : base(reinterpret_cast<char*>(p)), off(0) {}
    template <typename T> T* take(size_t count) {
        T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off = align_up(off + count * sizeof(T));
        return r;
    }
    void* take_bytes(size_t bytes) {
        void* r = base ? base + off : nullptr;
        off = align_up(off + bytes);
        return r;
    }
};

// The forward workspace doubles as the record the backward call can reuse (gate vectors, the
// chunk states C_{k-1} and the final state), so its layout is part of the library's contract
// with itself: carve_fwd is the only place that defines it.
// boundaries between the blocks of the anchored forget-gate gradient scan, plus the unused slot 0
inline int anchor_G(const Dims& d) { return anchor_chunks(d.L, d.dqk > d.dhv ? d.dqk : d.dhv); }
inline size_t anchor_slots(const Dims& d) { const int G = anchor_G(d); return (size_t)((d.Nc + G - 1) / G); }

struct FwdWs {
    float *wrow, *ucol, *sH, *aK, *gbar, *mout, *tmp, *csum, *nst, *Cfin, *pacc, *pnrm, *anc, *wrowB, *sQ;
    float *wrow_lo, *ucol_lo, *wrowB_lo;   // fp32 kernels: rounding remainders of the exponents (NULL for bf16)
    void* stT;
    size_t bytes;
};
FwdWs carve_fwd(const Dims& d, void* ws) {
    Carver c(ws);
    FwdWs w;
    w.wrow = c.take<float>(d.BHT); w.ucol = c.take<float>(d.BHT); w.sH = c.take<float>(d.BHT);
    // (the fp32 kernels' gate pre-pass works in double: its scratch is twice the size)
    const size_t gw = d.dtype == TFLA_BF16 ? 1 : 2;
    w.aK = c.take<float>(d.BHT); w.mout = c.take<float>(d.BHT); w.tmp = c.take<float>(gw * 3 * d.BHT);
    w.wrowB = c.take<float>(d.BHT); w.sQ = c.take<float>(d.BHT);     // the backward pass's row weights (mLSTMexp)
    w.gbar = c.take<float>(d.BH * d.Nc);
    w.csum = c.take<float>(gw * 2 * d.BH * d.Nc);
    w.wrow_lo = gw == 2 ? c.take<float>(d.BHT) : nullptr;
    w.ucol_lo = gw == 2 ? c.take<float>(d.BHT) : nullptr;
    w.wrowB_lo = gw == 2 ? c.take<float>(d.BHT) : nullptr;
    w.nst = c.take<float>(d.BH * d.Nc * d.dqk);
    w.Cfin = c.take<float>((size_t)d.BH * d.dqk * d.dhv);
    w.stT = c.take_bytes((size_t)d.BH * d.Nc * d.dqk * d.dhv * d.esz);
    // d_qk above 512: the parallel kernel contracts over d_qk in two halves that meet in fp32
    w.pacc = contraction_split(d.dqk, d.dtype) ? c.take<float>((size_t)d.BHT * d.dhv) : nullptr;
    w.pnrm = contraction_split(d.dqk, d.dtype) ? c.take<float>(d.BHT) : nullptr;
    // bf16: fp32 copies of the state at the block boundaries of the forget-gate gradient scan (see bwd_core)
    w.anc = d.dtype == TFLA_BF16 ? c.take<float>(anchor_slots(d) * (size_t)d.BH * d.dqk * d.dhv) : nullptr;
    w.bytes = c.off;
    return w;
}

struct BwdWs {
    float *wrow, *ucol, *sH, *aK, *gbar, *mout, *tmp, *csum, *wrowB, *sQ, *partQ, *partK, *cdot, *Cfinal, *anchor, *pacc, *ancC;
    float *wrow_lo, *ucol_lo, *wrowB_lo;   // fp32 kernels: rounding remainders of the exponents (NULL for bf16)
    double* bsum;
    void *cN, *dcT, *dcN, *E, *E2;
    int nbQ, nbK;
    size_t bytes;
};
BwdWs carve_bwd(const Dims& d, void* ws) {
    Carver c(ws);
    BwdWs w;
    w.wrow = c.take<float>(d.BHT); w.ucol = c.take<float>(d.BHT); w.sH = c.take<float>(d.BHT);
    const size_t gw = d.dtype == TFLA_BF16 ? 1 : 2;     // as in carve_fwd
    w.aK = c.take<float>(d.BHT); w.mout = c.take<float>(d.BHT); w.tmp = c.take<float>(gw * 3 * d.BHT);
    w.gbar = c.take<float>(d.BH * d.Nc);
    w.csum = c.take<float>(gw * 2 * d.BH * d.Nc);
    w.wrow_lo = gw == 2 ? c.take<float>(d.BHT) : nullptr;
    w.ucol_lo = gw == 2 ? c.take<float>(d.BHT) : nullptr;
    w.wrowB_lo = gw == 2 ? c.take<float>(d.BHT) : nullptr;
    w.bsum = c.take<double>(d.BH * ((d.T + 1023) / 1024));
    w.wrowB = c.take<float>(d.BHT); w.sQ = c.take<float>(d.BHT);
    w.nbQ = d.dqk / tile_bd2(d.dhv, d.dqk, d.dtype, MODE_DQ, d.L);
    w.nbK = d.dqk / tile_bd2(d.dhv, d.dqk, d.dtype, MODE_DK, d.L);
    w.partQ = c.take<float>((size_t)w.nbQ * d.BHT); w.partK = c.take<float>((size_t)w.nbK * d.BHT);
    w.cdot = c.take<float>(d.BH);
    w.Cfinal = c.take<float>((size_t)d.BH * d.dqk * d.dhv);
    const size_t st = (size_t)d.BH * d.Nc * d.dqk * d.dhv * d.esz;
    // bf16: C_{k-1} and dC_k, both as (d_hv, d_qk); fp32 additionally dC_k as (d_qk, d_hv)
    w.cN = c.take_bytes(st); w.dcT = c.take_bytes(st);
    w.dcN = d.dtype == TFLA_BF16 ? nullptr : c.take_bytes(st);
    // bf16: the weighted intra-chunk matrix shared by dQ and dK, (BH, Nc, L, L)
    w.E = (d.dtype == TFLA_BF16 && tile_shares_E(d.dhv)) ? c.take_bytes((size_t)d.BHT * d.L * d.esz) : nullptr;
    // head dimensions above 512: fp32 partial results of the gradient kernels' first half, and the second
    // half's E when the products of dQ / dK run over the halves of d_hv
    const int dwide = d.dqk > d.dhv ? d.dqk : d.dhv;
    w.pacc = contraction_split(dwide, d.dtype) ? c.take<float>((size_t)d.BHT * dwide) : nullptr;
    w.E2 = (d.dtype == TFLA_BF16 && d.dhv > 512) ? c.take_bytes((size_t)d.BHT * d.L * d.esz) : nullptr;
    // bf16: fp32 boundary copies of C (used when the states are recomputed here), and the partial inner products
    // <C, dC> of every boundary
    w.ancC = d.dtype == TFLA_BF16 ? c.take<float>(anchor_slots(d) * (size_t)d.BH * d.dqk * d.dhv) : nullptr;
    w.anchor = c.take<float>(anchor_slots(d) * (size_t)d.BH * rec_anchor_parts(d.dqk, d.dhv));
    w.bytes = c.off;
    return w;
}

#define TFLA_TRY(expr)                         \
    do {                                       \
        hipError_t e_ = (expr);                \
        if (e_ != hipSuccess) return (int)e_;  \
    } while (0)

// ---- optional per-kernel timing with HIP events on the caller's stream -------------------
enum { K_GATES = 0, K_BWD_PREP, K_REC_FWD, K_REC_BWD, K_TILE_H, K_TILE_DV, K_TILE_DQ, K_TILE_DK, K_GATE_GRADS,
       K_STATE_DOT, K_FILL, K_STEP, K_NORM_FWD, K_NORM_BWD, K_GAIN, K_PAD, K_COUNT };
const char* const kKernelNames[K_COUNT] = {"gates", "gate_bwd_prep", "recurrent_fwd", "recurrent_bwd", "tile_H",
                                           "tile_dV", "tile_dQ", "tile_dK", "gate_grads", "state_dot", "fill_zero",
                                           "recurrent_step", "norm_gate_fwd", "norm_gate_bwd", "transfer_gain", "pad_copy"};
struct Profiler {
    bool on = false;
    int cap = 0, used = 0;
    hipEvent_t* beg = nullptr;
    hipEvent_t* end = nullptr;
    int* slot = nullptr;
    double total_ms[K_COUNT] = {};
    long launches[K_COUNT] = {};
};
Profiler g_prof;

struct ProfScope {
    int idx;
    hipStream_t s;
    ProfScope(int slot, hipStream_t st) : idx(-1), s(st) {
        if (g_prof.on && g_prof.used < g_prof.cap) {
            idx = g_prof.used++;
            g_prof.slot[idx] = slot;
            (void)hipEventRecord(g_prof.beg[idx], s);
        }
    }
    ~ProfScope() {
        if (idx >= 0) (void)hipEventRecord(g_prof.end[idx], s);
    }
};
#define TFLA_LAUNCH(slot, expr)     \
    do {                            \
        ProfScope ps_((slot), s);   \
        TFLA_TRY(expr);             \
    } while (0)

void prof_collect() {
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.0f;
        if (hipEventSynchronize(g_prof.end[i]) == hipSuccess &&
            hipEventElapsedTime(&ms, g_prof.beg[i], g_prof.end[i]) == hipSuccess) {
            g_prof.total_ms[g_prof.slot[i]] += ms;
            g_prof.launches[g_prof.slot[i]] += 1;
        }
    }
    g_prof.used = 0;
}

int run_gates(const Dims& d, const float* i_pre, const float* f_pre, const float* m0, float* wrow, float* ucol,
              float* sH, float* aK, float* gbar, float* mout, float* mfinal, float* tmp, float* csum, float* wrow_lo,
              float* ucol_lo, float softcap, int Tvalid, int dqk_true, hipStream_t s) {
    GateArgs g;
    g.softcap = softcap; g.Tvalid = Tvalid;
    g.i_pre = i_pre; g.f_pre = f_pre; g.m0 = d.variant == TFLA_EXP ? m0 : nullptr;
    g.T = d.T; g.L = d.L; g.Nc = d.Nc; g.variant = d.variant;
    g.qscale = 1.0f / sqrtf((float)dqk_true);   // of the caller's head dimension, not of the padded one
    g.wrow = wrow; g.ucol = ucol; g.sH = sH; g.aK = aK; g.gbar = gbar; g.mout = mout; g.mfinal = mfinal; g.tmp = tmp; g.csum = csum;
    g.wrow_lo = wrow_lo; g.ucol_lo = ucol_lo; g.precise = d.dtype == TFLA_BF16 ? 0 : 1;
    TFLA_LAUNCH(K_GATES, launch_gates(g, (int)d.BH, s));
    return TFLA_OK;
}

// Forward pass over whole chunks: T is a multiple of chunk, steps >= Tvalid are padding.
int fwd_core(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre, const float* C0,
             const float* n0, const float* m0, int B, int NH, int T, int Tvalid, int dqk_true, int dhv_true, int dqk, int dhv,
             int chunk, int variant, int dtype, float eps, float softcap, void* H, float* Cn, float* nn, float* mn, float* n_out, float* m_out,
             void* workspace, size_t workspace_bytes, void* stream, const LayerFuse* fz = nullptr) {
    const int rc = check_dims(TFLA_FWD, B, NH, T, dqk, dhv, chunk, variant, dtype, true);
    if (rc != TFLA_OK) return rc;
    if (!q || !k || !v || !i_pre || !f_pre || !H) return TFLA_ERR_NULL;
    if (variant == TFLA_EXP) {
        const int given = (C0 != nullptr) + (n0 != nullptr) + (m0 != nullptr);
        if (given != 0 && given != 3) return TFLA_ERR_STATE;
    }
    const Dims d = make_dims(B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return TFLA_ERR_WORKSPACE;
    const FwdWs w = carve_fwd(d, workspace);
    if (workspace_bytes < w.bytes) return TFLA_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const bool is_exp = variant == TFLA_EXP;

    // 1. gates, max states
    float* mout = (is_exp && m_out) ? m_out : w.mout;
    int st = run_gates(d, i_pre, f_pre, m0, w.wrow, w.ucol, w.sH, w.aK, w.gbar, mout, is_exp ? mn : nullptr, w.tmp, w.csum, w.wrow_lo, w.ucol_lo, softcap, Tvalid, dqk_true, s);
    if (st != TFLA_OK) return st;

    // 2. recurrent kernel: C_{k-1} (transposed, element type of q/k/v) and n_{k-1} for every chunk
    RecArgs r;
    r.X = k; r.Y = v; r.rs = w.aK; r.gbar = w.gbar; r.S0 = C0;
    r.stT = w.stT; r.stN = nullptr; r.Sfinal = Cn; r.Sfinal2 = w.Cfin;
    r.n0 = is_exp ? n0 : nullptr; r.nst = is_exp ? w.nst : nullptr; r.nfinal = is_exp ? nn : nullptr;
    r.T = T; r.L = chunk; r.Nc = d.Nc; r.d1 = dqk; r.d2 = dhv; r.reverse = 0;
    r.anc = w.anc; r.anc_in = nullptr; r.anc_part = nullptr; r.anc_G = anchor_G(d);
    TFLA_LAUNCH(K_REC_FWD, launch_recurrent(r, (int)d.BH, dtype, s));

    // 3. parallel kernel
    TileArgs t{};
    t.X = q; t.Y = k; t.Z = v; t.Out = H; t.out_T = Tvalid; t.out_ld = dhv_true; t.out_cols = dhv_true;
    t.part_acc = w.pacc; t.part_nrm = w.pnrm;
    t.wrow = w.wrow; t.wcol = w.ucol; t.srow = w.sH; t.St = w.stT;
    t.T = T; t.L = chunk; t.Nc = d.Nc; t.d1 = dqk; t.d2 = dhv;
    t.variant = variant; t.eps = eps; t.nstate = w.nst; t.mout = mout; t.nout = is_exp ? n_out : nullptr;
    t.wrowB_out = is_exp ? w.wrowB : nullptr; t.sQ_out = is_exp ? w.sQ : nullptr;
    t.wrow_lo = w.wrow_lo; t.wcol_lo = w.ucol_lo; t.wrowB_lo_out = is_exp ? w.wrowB_lo : nullptr;
    t.dotwith = nullptr; t.dotpart = nullptr; t.E = nullptr;
    if (fz) {
        // the layer's output is formed by the H kernel itself (the caller has checked that its workgroups hold whole rows)
        t.fz_o = fz->o_pre; t.fz_gamma = fz->gamma; t.fz_beta = fz->beta; t.fz_y = fz->y;
        t.fz_kind = fz->kind; t.fz_NH = fz->NH; t.fz_eps = fz->eps;
    }
    TFLA_LAUNCH(K_TILE_H, launch_tile_mode<MODE_H>(t, (int)d.BH, dtype, s));

    if (!is_exp) {
        // the outputs that mLSTMsig does not have, zero-filled in one launch
        FillList fl{};
        if (nn) { fl.p[0] = nn; fl.n[0] = d.BH * dqk; }
        if (mn) { fl.p[1] = mn; fl.n[1] = d.BH; }
        if (n_out) { fl.p[2] = n_out; fl.n[2] = d.BHT; }
        if (m_out) { fl.p[3] = m_out; fl.n[3] = d.BHT; }
        if (nn || mn || n_out || m_out) TFLA_LAUNCH(K_FILL, launch_fill_zero4(fl, s));
    }
    return TFLA_OK;
}


int bwd_core(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre, const float* C0,
             const float* n0, const float* m0, const float* n_out, const float* m_out, const void* dH, const float* dCn,
             int B, int NH, int T, int Tvalid, int dqk_true, int dhv_true, int dqk, int dhv, int chunk, int variant, int dtype,
             float eps, float softcap, void* dq,
             void* dk, void* dv, float* d_i_pre, float* d_f_pre, float* dC0, const void* fwd_workspace,
             size_t fwd_workspace_bytes, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_dims(TFLA_BWD, B, NH, T, dqk, dhv, chunk, variant, dtype, true);
    if (rc != TFLA_OK) return rc;
    if (!q || !k || !v || !i_pre || !f_pre || !dH || !dq || !dk || !dv || !d_i_pre || !d_f_pre) return TFLA_ERR_NULL;
    const bool is_exp = variant == TFLA_EXP;
    if (is_exp) {
        if (!n_out || !m_out) return TFLA_ERR_NULL;
        const int given = (C0 != nullptr) + (n0 != nullptr) + (m0 != nullptr);
        if (given != 0 && given != 3) return TFLA_ERR_STATE;
    }
    const Dims d = make_dims(B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return TFLA_ERR_WORKSPACE;
    const BwdWs w = carve_bwd(d, workspace);
    if (workspace_bytes < w.bytes) return TFLA_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    // What the matching forward call left in its workspace (gate vectors, C_{k-1} for every chunk,
    // C_T) is reused when the caller hands that workspace over; otherwise it is recomputed here.
    FwdWs fw{};
    const bool reuse = fwd_workspace != nullptr;
    if (reuse) {
        if ((reinterpret_cast<uintptr_t>(fwd_workspace) & 255) != 0) return TFLA_ERR_WORKSPACE;
        fw = carve_fwd(d, const_cast<void*>(fwd_workspace));
        if (fwd_workspace_bytes < fw.bytes) return TFLA_ERR_WORKSPACE;
    }
    // the generic fp32 kernels read the states of dQ / dK as (d_qk, d_hv); the bf16 kernels read
    // (d_hv, d_qk) everywhere, so only that layout is ever written on the bf16 path
    const bool tonly = dtype == TFLA_BF16;
    const bool reuse_states = reuse && tonly;
    const float* wrow = reuse ? fw.wrow : w.wrow;
    const float* ucol = reuse ? fw.ucol : w.ucol;
    const float* sH = reuse ? fw.sH : w.sH;
    const float* aK = reuse ? fw.aK : w.aK;
    const float* gbar = reuse ? fw.gbar : w.gbar;
    const float* wrow_lo = reuse ? fw.wrow_lo : w.wrow_lo;     // fp32 kernels only, NULL otherwise
    const float* ucol_lo = reuse ? fw.ucol_lo : w.ucol_lo;

    // 1. gates as in the forward pass, then fold 1/h_denom into the backward weights
    if (!reuse) {
        int st = run_gates(d, i_pre, f_pre, m0, w.wrow, w.ucol, w.sH, w.aK, w.gbar, w.mout, nullptr, w.tmp, w.csum, w.wrow_lo, w.ucol_lo, softcap, Tvalid, dqk_true, s);
        if (st != TFLA_OK) return st;
    }
    // mLSTMsig has no denominator (the weights are the forward pass's own); for mLSTMexp the forward call has left
    // them in its workspace when it wrote n_out, otherwise they are formed here from n_out and m_out
    const float* wrowB = wrow;
    const float* wrowB_lo = wrow_lo;
    const float* sQ = sH;
    if (is_exp) {
        if (reuse) {
            wrowB = fw.wrowB; sQ = fw.sQ; wrowB_lo = fw.wrowB_lo;
        } else {
            GateBwdPrepArgs p;
            p.wrow = wrow; p.sH = sH; p.n_out = n_out; p.m_out = m_out; p.wrowB = w.wrowB; p.sQ = w.sQ;
            p.n = d.BHT; p.variant = variant; p.eps = eps;
            p.wrow_lo = wrow_lo; p.wrowB_lo = wrow_lo ? w.wrowB_lo : nullptr;
            TFLA_LAUNCH(K_BWD_PREP, launch_gate_bwd_prep(p, s));
            wrowB = w.wrowB; sQ = w.sQ; wrowB_lo = p.wrowB_lo;
        }
    }

    // 2. the chunk states C_{k-1}
    const void* cstates = reuse_states ? fw.stT : w.cN;
    const float* Cfinal = reuse_states ? fw.Cfin : w.Cfinal;
    if (!reuse_states) {
        RecArgs r;
        r.X = k; r.Y = v; r.rs = aK; r.gbar = gbar; r.S0 = C0;
        r.stT = tonly ? w.cN : nullptr; r.stN = tonly ? nullptr : w.cN;
        r.Sfinal = dCn ? w.Cfinal : nullptr; r.Sfinal2 = nullptr;
        r.n0 = nullptr; r.nst = nullptr; r.nfinal = nullptr;
        r.T = T; r.L = chunk; r.Nc = d.Nc; r.d1 = dqk; r.d2 = dhv; r.reverse = 0;
        r.anc = w.ancC; r.anc_in = nullptr; r.anc_part = nullptr; r.anc_G = anchor_G(d);
        TFLA_LAUNCH(K_REC_FWD, launch_recurrent(r, (int)d.BH, dtype, s));
    }

    // 3. backward recurrence: dC_k for every chunk, dC_0 at the end
    RecArgs rb;
    rb.X = q; rb.Y = dH; rb.rs = sQ; rb.gbar = gbar; rb.S0 = dCn;
    rb.stT = w.dcT; rb.stN = tonly ? nullptr : w.dcN; rb.Sfinal = dC0; rb.Sfinal2 = nullptr;
    rb.n0 = nullptr; rb.nst = nullptr; rb.nfinal = nullptr;
    rb.T = T; rb.L = chunk; rb.Nc = d.Nc; rb.d1 = dqk; rb.d2 = dhv; rb.reverse = 1;
    // bf16: the reversed launch also forms <C, dC> at the block boundaries of the forget-gate gradient scan, from the
    // fp32 copies of C that the forward launch left there and its own fp32 accumulators
    rb.anc = nullptr; rb.anc_in = tonly ? (reuse_states ? fw.anc : w.ancC) : nullptr; rb.anc_part = tonly ? w.anchor : nullptr;
    rb.anc_G = anchor_G(d);
    TFLA_LAUNCH(K_REC_BWD, launch_recurrent(rb, (int)d.BH, dtype, s));

    // 4. the three gradient kernels
    TileArgs t{};
    t.T = T; t.L = chunk; t.Nc = d.Nc; t.variant = variant; t.eps = eps;
    t.nstate = nullptr; t.mout = nullptr; t.nout = nullptr; t.E = w.E; t.E2 = w.E2; t.part_acc = w.pacc;
    // dV: rows = kv index j
    t.X = k; t.Y = q; t.Z = dH; t.Out = dv; t.out_T = Tvalid; t.out_ld = dhv_true; t.out_cols = dhv_true; t.wrow_lo = ucol_lo; t.wcol_lo = wrowB_lo; t.wrowB_lo_out = nullptr; t.wrow = ucol; t.wcol = wrowB; t.srow = aK; t.St = w.dcT;
    t.d1 = dqk; t.d2 = dhv; t.dotwith = nullptr; t.dotpart = nullptr;
    TFLA_LAUNCH(K_TILE_DV, launch_tile_mode<MODE_DV>(t, (int)d.BH, dtype, s));
    // dQ: rows = query index i
    t.X = dH; t.Y = v; t.Z = k; t.Out = dq; t.out_ld = dqk_true; t.out_cols = dqk_true; t.wrow_lo = wrowB_lo; t.wcol_lo = ucol_lo; t.wrow = wrowB; t.wcol = ucol; t.srow = sQ; t.St = cstates;
    t.d1 = dhv; t.d2 = dqk; t.dotwith = q; t.dotpart = w.partQ;
    TFLA_LAUNCH(K_TILE_DQ, launch_tile_mode<MODE_DQ>(t, (int)d.BH, dtype, s));
    // dK: rows = kv index j
    t.X = v; t.Y = dH; t.Z = q; t.Out = dk; t.wrow_lo = ucol_lo; t.wcol_lo = wrowB_lo; t.wrow = ucol; t.wcol = wrowB; t.srow = aK; t.St = tonly ? w.dcT : w.dcN;
    t.d1 = dhv; t.d2 = dqk; t.dotwith = k; t.dotpart = w.partK;
    TFLA_LAUNCH(K_TILE_DK, launch_tile_mode<MODE_DK>(t, (int)d.BH, dtype, s));

    // 5. gate gradients
    if (dCn) TFLA_LAUNCH(K_STATE_DOT, launch_state_dot(Cfinal, dCn, w.cdot, (long)dqk * dhv, (int)d.BH, s));
    GateGradArgs gg;
    gg.partQ = w.partQ; gg.nbQ = w.nbQ; gg.partK = w.partK; gg.nbK = w.nbK; gg.cdot = dCn ? w.cdot : nullptr;
    gg.i_pre = i_pre; gg.f_pre = f_pre; gg.d_i = d_i_pre; gg.d_f = d_f_pre; gg.T = T; gg.variant = variant;
    gg.BHT = d.BHT; gg.bsum = w.bsum; gg.softcap = softcap;
    gg.anchor = nullptr; gg.L = chunk; gg.Nc = d.Nc; gg.G = 1; gg.npart = 0;
    // bf16: the forget-gate scan is anchored with <C_k, dC_k> at the end of every block of anchor_chunks() chunks
    // (a block has at most 2048 steps), so that the rounding noise of its terms (one part in 2^9 of the boundary
    // terms per chunk, from the bf16 states) accumulates over one block instead of the whole sequence.  The anchors
    // themselves are exact to fp32: the forward recurrent launch leaves fp32 copies of the state at the block
    // boundaries and the reversed launch multiplies them with its fp32 accumulators (see RecArgs).
    if (tonly) {
        gg.G = anchor_G(d);
        gg.anchor = w.anchor; gg.npart = rec_anchor_parts(dqk, dhv);
    }
    TFLA_LAUNCH(K_GATE_GRADS, launch_gate_grads(gg, (int)d.BH, s));
    return TFLA_OK;
}


// ---- sequence lengths that do not fill the last chunk, head dimensions between the kernels' own -------
// The cores work on whole chunks and on head dimensions 64, 128, 256, 512 (bf16 also 1024).  For any other T or head
// dimension the entry points copy q, k, v (and dH) into zero-padded buffers behind the core's own workspace and
// run the core there (Tvalid = T, the 1/sqrt(dqk) of the true dqk).  The tiled kernels store the true steps and
// columns of H, dq, dk, dv straight into the caller's tensors; per-step scalars go through padded copies only when
// the sequence itself is padded, states only when a head dimension is.  `d` below always describes the padded problem.
struct PadFwd {
    void *q, *k, *v;
    float *ip, *fp, *nout, *mout, *C0, *n0, *Cn, *nn;
    size_t bytes;
};
PadFwd carve_pad_fwd(const Dims& d, void* base) {
    Carver c(base);
    PadFwd p;
    p.q = c.take_bytes((size_t)d.BHT * d.dqk * d.esz); p.k = c.take_bytes((size_t)d.BHT * d.dqk * d.esz);
    p.v = c.take_bytes((size_t)d.BHT * d.dhv * d.esz);
    p.ip = c.take<float>(d.BHT); p.fp = c.take<float>(d.BHT); p.nout = c.take<float>(d.BHT); p.mout = c.take<float>(d.BHT);
    p.C0 = c.take<float>((size_t)d.BH * d.dqk * d.dhv); p.n0 = c.take<float>((size_t)d.BH * d.dqk);
    p.Cn = c.take<float>((size_t)d.BH * d.dqk * d.dhv); p.nn = c.take<float>((size_t)d.BH * d.dqk);
    p.bytes = c.off;
    return p;
}
struct PadBwd {
    void *q, *k, *v, *dH;
    float *ip, *fp, *nout, *mout, *di, *df, *C0, *n0, *dCn, *dC0;
    size_t bytes;
};
PadBwd carve_pad_bwd(const Dims& d, void* base) {
    Carver c(base);
    PadBwd p;
    const size_t sq = (size_t)d.BHT * d.dqk * d.esz, sv = (size_t)d.BHT * d.dhv * d.esz;
    p.q = c.take_bytes(sq); p.k = c.take_bytes(sq); p.v = c.take_bytes(sv); p.dH = c.take_bytes(sv);
    p.ip = c.take<float>(d.BHT); p.fp = c.take<float>(d.BHT); p.nout = c.take<float>(d.BHT); p.mout = c.take<float>(d.BHT);
    p.di = c.take<float>(d.BHT); p.df = c.take<float>(d.BHT);
    const size_t ss = (size_t)d.BH * d.dqk * d.dhv;
    p.C0 = c.take<float>(ss); p.n0 = c.take<float>((size_t)d.BH * d.dqk); p.dCn = c.take<float>(ss); p.dC0 = c.take<float>(ss);
    p.bytes = c.off;
    return p;
}
// dp: the padded problem; padded = whether the caller's problem differs from it
size_t fwd_total_bytes(const Dims& dp, bool padded) {
    return carve_fwd(dp, nullptr).bytes + (padded ? carve_pad_fwd(dp, nullptr).bytes : 0);
}
size_t bwd_total_bytes(const Dims& dp, bool padded) {
    return carve_bwd(dp, nullptr).bytes + (padded ? carve_pad_bwd(dp, nullptr).bytes : 0);
}
inline bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }
inline bool needs_pad(int T, int dqk, int dhv, int chunk) {
    return T % chunk != 0 || dqk != kernel_dim(dqk) || dhv != kernel_dim(dhv);
}

int fwd_impl(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre, const float* C0,
             const float* n0, const float* m0, int B, int NH, int T, int dqk, int dhv, int chunk, int variant, int dtype,
             float eps, float softcap, void* H, float* Cn, float* nn, float* mn, float* n_out, float* m_out,
             void* workspace, size_t workspace_bytes, void* stream, const LayerFuse* fz = nullptr) {
    const int rc = check_dims(TFLA_FWD, B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (rc != TFLA_OK) return rc;
    if (!needs_pad(T, dqk, dhv, chunk))
        return fwd_core(q, k, v, i_pre, f_pre, C0, n0, m0, B, NH, T, T, dqk, dhv, dqk, dhv, chunk, variant, dtype, eps, softcap, H,
                        Cn, nn, mn, n_out, m_out, workspace, workspace_bytes, stream, fz);
    if (fz) return TFLA_ERR_SHAPE;      // (the fused layer output is for problems that need no padding)
    if (!q || !k || !v || !i_pre || !f_pre || !H) return TFLA_ERR_NULL;
    const bool is_exp = variant == TFLA_EXP;
    if (is_exp) {
        const int given = (C0 != nullptr) + (n0 != nullptr) + (m0 != nullptr);
        if (given != 0 && given != 3) return TFLA_ERR_STATE;
    }
    if (misaligned16(q) || misaligned16(k) || misaligned16(v) || misaligned16(H) || misaligned16(C0) || misaligned16(Cn))
        return TFLA_ERR_SHAPE;
    const int dq_p = kernel_dim(dqk), dv_p = kernel_dim(dhv);
    const Dims d = make_dims(B, NH, T, dq_p, dv_p, chunk, variant, dtype);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return TFLA_ERR_WORKSPACE;
    const size_t core_bytes = carve_fwd(d, nullptr).bytes;
    const PadFwd p = carve_pad_fwd(d, reinterpret_cast<char*>(workspace) + core_bytes);
    if (workspace_bytes < core_bytes + p.bytes) return TFLA_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const int Tp = d.T, es = (int)d.esz;
    const bool dpad = dq_p != dqk || dv_p != dhv;       // states need padding too
    TFLA_LAUNCH(K_PAD, launch_pad_rows(q, p.q, d.BH, T, Tp, dqk * es, dq_p * es, s));
    TFLA_LAUNCH(K_PAD, launch_pad_rows(k, p.k, d.BH, T, Tp, dqk * es, dq_p * es, s));
    TFLA_LAUNCH(K_PAD, launch_pad_rows(v, p.v, d.BH, T, Tp, dhv * es, dv_p * es, s));
    // per-step scalars need copies only when the sequence itself is padded
    const bool tpad = Tp != T;
    if (tpad) {
        TFLA_LAUNCH(K_PAD, launch_pad_scalar(i_pre, p.ip, d.BH, T, Tp, 0.0f, s));
        TFLA_LAUNCH(K_PAD, launch_pad_scalar(f_pre, p.fp, d.BH, T, Tp, 0.0f, s));
    }
    const float* C0c = C0; const float* n0c = n0;
    if (dpad && C0) {
        TFLA_LAUNCH(K_PAD, launch_pad_rows(C0, p.C0, d.BH, dqk, dq_p, dhv * 4, dv_p * 4, s));
        C0c = p.C0;
        if (is_exp) { TFLA_LAUNCH(K_PAD, launch_pad_scalar(n0, p.n0, d.BH, dqk, dq_p, 0.0f, s)); n0c = p.n0; }
    }
    float* Cnc = (dpad && Cn) ? p.Cn : Cn;
    float* nnc = (dpad && nn) ? p.nn : nn;
    // (the H kernel stores the true steps and columns straight into the caller's H)
    const int st = fwd_core(p.q, p.k, p.v, tpad ? p.ip : i_pre, tpad ? p.fp : f_pre, C0c, n0c, m0, B, NH, Tp, T, dqk, dhv, dq_p,
                            dv_p, chunk, variant, dtype, eps, softcap, H, Cnc, nnc, mn, (n_out && tpad) ? p.nout : n_out,
                            (m_out && tpad) ? p.mout : m_out, workspace, core_bytes, stream);
    if (st != TFLA_OK) return st;
    if (n_out && tpad) TFLA_LAUNCH(K_PAD, launch_unpad_scalar(p.nout, n_out, d.BH, T, Tp, s));
    if (m_out && tpad) TFLA_LAUNCH(K_PAD, launch_unpad_scalar(p.mout, m_out, d.BH, T, Tp, s));
    if (dpad && Cn) TFLA_LAUNCH(K_PAD, launch_unpad_rows(p.Cn, Cn, d.BH, dqk, dq_p, dhv * 4, dv_p * 4, s));
    if (dpad && nn) TFLA_LAUNCH(K_PAD, launch_unpad_scalar(p.nn, nn, d.BH, dqk, dq_p, s));
    return TFLA_OK;
}

int bwd_impl(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre, const float* C0,
             const float* n0, const float* m0, const float* n_out, const float* m_out, const void* dH, const float* dCn,
             int B, int NH, int T, int dqk, int dhv, int chunk, int variant, int dtype, float eps, float softcap, void* dq,
             void* dk, void* dv, float* d_i_pre, float* d_f_pre, float* dC0, const void* fwd_workspace,
             size_t fwd_workspace_bytes, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_dims(TFLA_BWD, B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (rc != TFLA_OK) return rc;
    if (!needs_pad(T, dqk, dhv, chunk))
        return bwd_core(q, k, v, i_pre, f_pre, C0, n0, m0, n_out, m_out, dH, dCn, B, NH, T, T, dqk, dhv, dqk, dhv, chunk, variant,
                        dtype, eps, softcap, dq, dk, dv, d_i_pre, d_f_pre, dC0, fwd_workspace, fwd_workspace_bytes,
                        workspace, workspace_bytes, stream);
    if (!q || !k || !v || !i_pre || !f_pre || !dH || !dq || !dk || !dv || !d_i_pre || !d_f_pre) return TFLA_ERR_NULL;
    const bool is_exp = variant == TFLA_EXP;
    if (is_exp) {
        if (!n_out || !m_out) return TFLA_ERR_NULL;
        const int given = (C0 != nullptr) + (n0 != nullptr) + (m0 != nullptr);
        if (given != 0 && given != 3) return TFLA_ERR_STATE;
    }
    if (misaligned16(q) || misaligned16(k) || misaligned16(v) || misaligned16(dH) || misaligned16(dq) || misaligned16(dk) ||
        misaligned16(dv) || misaligned16(C0) || misaligned16(dCn) || misaligned16(dC0))
        return TFLA_ERR_SHAPE;
    const int dq_p = kernel_dim(dqk), dv_p = kernel_dim(dhv);
    const Dims d = make_dims(B, NH, T, dq_p, dv_p, chunk, variant, dtype);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return TFLA_ERR_WORKSPACE;
    if (fwd_workspace && ((reinterpret_cast<uintptr_t>(fwd_workspace) & 255) != 0 ||
                          fwd_workspace_bytes < carve_fwd(d, nullptr).bytes))
        return TFLA_ERR_WORKSPACE;
    const size_t core_bytes = carve_bwd(d, nullptr).bytes;
    const PadBwd p = carve_pad_bwd(d, reinterpret_cast<char*>(workspace) + core_bytes);
    if (workspace_bytes < core_bytes + p.bytes) return TFLA_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const int Tp = d.T, es = (int)d.esz, eq = dqk * es, ev = dhv * es, eqp = dq_p * es, evp = dv_p * es;
    const bool dpad = dq_p != dqk || dv_p != dhv;
    const bool tpad = Tp != T;      // per-step scalars need copies only when the sequence itself is padded
    // The forward call left its padded copies of q, k, v and the gate pre-activations behind its core workspace:
    // a backward call that is handed that workspace (whole) reads them there instead of copying again.
    const void *pq = p.q, *pk = p.k, *pv = p.v;
    const float *pip = p.ip, *pfp = p.fp;
    const size_t fwd_core_bytes = carve_fwd(d, nullptr).bytes;
    if (fwd_workspace && fwd_workspace_bytes >= fwd_core_bytes + carve_pad_fwd(d, nullptr).bytes) {
        const PadFwd pf = carve_pad_fwd(d, const_cast<char*>(reinterpret_cast<const char*>(fwd_workspace)) + fwd_core_bytes);
        pq = pf.q; pk = pf.k; pv = pf.v; pip = pf.ip; pfp = pf.fp;
    } else {
        TFLA_LAUNCH(K_PAD, launch_pad_rows(q, p.q, d.BH, T, Tp, eq, eqp, s));
        TFLA_LAUNCH(K_PAD, launch_pad_rows(k, p.k, d.BH, T, Tp, eq, eqp, s));
        TFLA_LAUNCH(K_PAD, launch_pad_rows(v, p.v, d.BH, T, Tp, ev, evp, s));
        if (tpad) {
            TFLA_LAUNCH(K_PAD, launch_pad_scalar(i_pre, p.ip, d.BH, T, Tp, 0.0f, s));
            TFLA_LAUNCH(K_PAD, launch_pad_scalar(f_pre, p.fp, d.BH, T, Tp, 0.0f, s));
        }
    }
    if (!tpad) { pip = i_pre; pfp = f_pre; }
    TFLA_LAUNCH(K_PAD, launch_pad_rows(dH, p.dH, d.BH, T, Tp, ev, evp, s));
    if (is_exp && tpad) {
        // denominators of the padding steps: max{|1|, exp(0)} -- any finite non-zero value would do
        TFLA_LAUNCH(K_PAD, launch_pad_scalar(n_out, p.nout, d.BH, T, Tp, 1.0f, s));
        TFLA_LAUNCH(K_PAD, launch_pad_scalar(m_out, p.mout, d.BH, T, Tp, 0.0f, s));
    }
    const float* C0c = C0; const float* n0c = n0; const float* dCnc = dCn;
    if (dpad && C0) {
        TFLA_LAUNCH(K_PAD, launch_pad_rows(C0, p.C0, d.BH, dqk, dq_p, dhv * 4, dv_p * 4, s));
        C0c = p.C0;
        if (is_exp) { TFLA_LAUNCH(K_PAD, launch_pad_scalar(n0, p.n0, d.BH, dqk, dq_p, 0.0f, s)); n0c = p.n0; }
    }
    if (dpad && dCn) {
        TFLA_LAUNCH(K_PAD, launch_pad_rows(dCn, p.dCn, d.BH, dqk, dq_p, dhv * 4, dv_p * 4, s));
        dCnc = p.dCn;
    }
    float* dC0c = (dpad && dC0) ? p.dC0 : dC0;
    const float* noc = !is_exp ? nullptr : (tpad ? p.nout : n_out);
    const float* moc = !is_exp ? nullptr : (tpad ? p.mout : m_out);
    const int st = bwd_core(pq, pk, pv, pip, pfp, C0c, n0c, m0, noc, moc, p.dH, dCnc, B, NH, Tp, T, dqk, dhv, dq_p, dv_p,
                            chunk, variant, dtype, eps, softcap, dq, dk, dv, tpad ? p.di : d_i_pre, tpad ? p.df : d_f_pre,
                            dC0c, fwd_workspace, fwd_workspace_bytes, workspace, core_bytes, stream);
    if (st != TFLA_OK) return st;
    // (the gradient kernels stored the true steps and columns straight into the caller's dq, dk, dv)
    if (tpad) {
        TFLA_LAUNCH(K_PAD, launch_unpad_scalar(p.di, d_i_pre, d.BH, T, Tp, s));
        TFLA_LAUNCH(K_PAD, launch_unpad_scalar(p.df, d_f_pre, d.BH, T, Tp, s));
    }
    if (dpad && dC0) TFLA_LAUNCH(K_PAD, launch_unpad_rows(p.dC0, dC0, d.BH, dqk, dq_p, dhv * 4, dv_p * 4, s));
    return TFLA_OK;
}

}  // namespace

// ---- scratch memory of the allocation-free forward entry point -------------------------------------
// One array per GPU the library runs on, part of the code object: it exists from the moment the module is
// loaded on a device until the process ends.  In host code its name is only the handle that
// hipGetSymbolAddress translates; kernels and copies get the translated address.
namespace tfla {
static __device__ __align__(256) unsigned char scratch[TFLA_STATIC_SCRATCH_BYTES];
// never launched: a device-side use of the array, so that it is kept in the code object
__global__ void static_scratch_probe_kernel(unsigned* out) { *out = scratch[0]; }
}  // namespace tfla

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};      // device address of `scratch` on each device, set on first use

// address of the current device's copy of the array; nothing here allocates
int static_scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= MAX_DEVICES) return TFLA_ERR_SHAPE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(tfla::scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TFLA_OK;
}
}  // namespace

extern "C" {

int tfla_version(void) { return 1200; }

int tfla_tile_width(int width) {
    if (width != 0 && width != 64 && width != 128 && width != 256) return TFLA_ERR_ENUM;
    tfla::tile_width_override = width;
    return TFLA_OK;
}

int tfla_profile_enable(int max_launches) {
    if (g_prof.beg) {
        for (int i = 0; i < g_prof.cap; ++i) { (void)hipEventDestroy(g_prof.beg[i]); (void)hipEventDestroy(g_prof.end[i]); }
        delete[] g_prof.beg; delete[] g_prof.end; delete[] g_prof.slot;
        g_prof.beg = g_prof.end = nullptr; g_prof.slot = nullptr;
    }
    g_prof.on = false; g_prof.cap = 0; g_prof.used = 0;
    for (int k = 0; k < K_COUNT; ++k) { g_prof.total_ms[k] = 0.0; g_prof.launches[k] = 0; }
    if (max_launches <= 0) return TFLA_OK;
    g_prof.beg = new hipEvent_t[max_launches]; g_prof.end = new hipEvent_t[max_launches];
    g_prof.slot = new int[max_launches];
    for (int i = 0; i < max_launches; ++i) {
        hipError_t e = hipEventCreate(&g_prof.beg[i]);
        if (e == hipSuccess) e = hipEventCreate(&g_prof.end[i]);
        if (e != hipSuccess) return (int)e;
    }
    g_prof.cap = max_launches; g_prof.on = true;
    return TFLA_OK;
}

int tfla_profile_read(int kernel, char* name, int name_len, double* total_ms, long* launches) {
    if (kernel < 0 || kernel >= K_COUNT) return TFLA_ERR_ENUM;
    prof_collect();
    if (name && name_len > 0) {
        int i = 0;
        for (; i < name_len - 1 && kKernelNames[kernel][i]; ++i) name[i] = kKernelNames[kernel][i];
        name[i] = 0;
    }
    if (total_ms) *total_ms = g_prof.total_ms[kernel];
    if (launches) *launches = g_prof.launches[kernel];
    return TFLA_OK;
}

int tfla_profile_kernels(void) { return K_COUNT; }

const char* tfla_status_string(int status) {
    switch (status) {
        case TFLA_OK: return "ok";
        case TFLA_ERR_NULL: return "a required pointer is NULL";
        case TFLA_ERR_SHAPE: return "invalid or unsupported dimension";
        case TFLA_ERR_CHUNK: return "chunk must be a multiple of 64 in [64, 2048] with at most 4096 chunks per sequence";
        case TFLA_ERR_ENUM: return "unknown variant, dtype or direction";
        case TFLA_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
        case TFLA_ERR_STATE: return "state must be given completely (C, n, m) or not at all; n_out/m_out must not alias n/m";
        case TFLA_ERR_STATIC_LIMIT: return "the problem needs more scratch memory than the static buffer of the allocation-free entry point holds (tfla_static_scratch_bytes)";
        default: break;
    }
    if (status > 0) return hipGetErrorString((hipError_t)status);
    return "unknown status";
}

int tfla_mlstm_check(int direction, int B, int NH, int T, int dqk, int dhv, int chunk, int variant, int dtype) {
    return check_dims(direction, B, NH, T, dqk, dhv, chunk, variant, dtype);
}

size_t tfla_mlstm_workspace_bytes(int direction, int B, int NH, int T, int dqk, int dhv, int chunk, int variant,
                                  int dtype) {
    if (check_dims(direction, B, NH, T, dqk, dhv, chunk, variant, dtype) != TFLA_OK) return 0;
    const Dims d = make_dims(B, NH, T, kernel_dim(dqk), kernel_dim(dhv), chunk, variant, dtype);
    const bool padded = needs_pad(T, dqk, dhv, chunk);
    return direction == TFLA_FWD ? fwd_total_bytes(d, padded) : bwd_total_bytes(d, padded);
}

int tfla_mlstm_fwd(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                   const float* C0, const float* n0, const float* m0, int B, int NH, int T, int dqk, int dhv,
                   int chunk, int variant, int dtype, float eps, void* H, float* Cn, float* nn, float* mn,
                   float* n_out, float* m_out, void* workspace, size_t workspace_bytes, void* stream) {
    return fwd_impl(q, k, v, i_pre, f_pre, C0, n0, m0, B, NH, T, dqk, dhv, chunk, variant, dtype, eps, 0.0f, H, Cn, nn,
                    mn, n_out, m_out, workspace, workspace_bytes, stream);
}

size_t tfla_static_scratch_bytes(void) { return (size_t)TFLA_STATIC_SCRATCH_BYTES; }

int tfla_mlstm_fwd_static(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                          const float* C0, const float* n0, const float* m0, int B, int NH, int T, int dqk, int dhv,
                          int chunk, int variant, int dtype, float eps, void* H, float* Cn, float* nn, float* mn,
                          float* n_out, float* m_out, void* stream) {
    // everything that can be rejected is rejected before the first HIP call
    const int rc = check_dims(TFLA_FWD, B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (rc != TFLA_OK) return rc;
    const size_t need = tfla_mlstm_workspace_bytes(TFLA_FWD, B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (need == 0) return TFLA_ERR_SHAPE;
    if (need > (size_t)TFLA_STATIC_SCRATCH_BYTES) return TFLA_ERR_STATIC_LIMIT;
    if (!q || !k || !v || !i_pre || !f_pre || !H) return TFLA_ERR_NULL;
    void* ws = nullptr;
    const int st = static_scratch_address(&ws);
    if (st != TFLA_OK) return st;
    // the kernels write every part of the scratch memory they later read (gate vectors, chunk states), so
    // nothing has to be cleared between calls; the previous call's contents are simply overwritten
    return fwd_impl(q, k, v, i_pre, f_pre, C0, n0, m0, B, NH, T, dqk, dhv, chunk, variant, dtype, eps, 0.0f, H, Cn, nn,
                    mn, n_out, m_out, ws, (size_t)TFLA_STATIC_SCRATCH_BYTES, stream);
}

int tfla_mlstm_bwd(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                   const float* C0, const float* n0, const float* m0, const float* n_out, const float* m_out,
                   const void* dH, const float* dCn, int B, int NH, int T, int dqk, int dhv, int chunk,
                   int variant, int dtype, float eps, void* dq, void* dk, void* dv, float* d_i_pre,
                   float* d_f_pre, float* dC0, const void* fwd_workspace, size_t fwd_workspace_bytes,
                   void* workspace, size_t workspace_bytes, void* stream) {
    return bwd_impl(q, k, v, i_pre, f_pre, C0, n0, m0, n_out, m_out, dH, dCn, B, NH, T, dqk, dhv, chunk, variant, dtype,
                    eps, 0.0f, dq, dk, dv, d_i_pre, d_f_pre, dC0, fwd_workspace, fwd_workspace_bytes, workspace,
                    workspace_bytes, stream);
}

static int step_impl(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                     const float* C, const float* n, const float* m, int B, int NH, int dqk, int dhv, int variant,
                     int dtype, float eps, float softcap, void* h, float* C_out, float* n_out, float* m_out,
                     void* stream) {
    if (variant != TFLA_EXP && variant != TFLA_SIG) return TFLA_ERR_ENUM;
    if (dtype != TFLA_F32 && dtype != TFLA_BF16) return TFLA_ERR_ENUM;
    if (B <= 0 || NH <= 0 || (long)B * NH > 65535) return TFLA_ERR_SHAPE;
    if (dqk < 64 || dqk > 1024 || dqk % 64 != 0 || dhv < 64 || dhv > 1024 || dhv % 64 != 0) return TFLA_ERR_SHAPE;
    if (!q || !k || !v || !i_pre || !f_pre || !C || !C_out || !h) return TFLA_ERR_NULL;
    if (variant == TFLA_EXP) {
        if ((n != nullptr) != (m != nullptr)) return TFLA_ERR_STATE;
        if (!n_out || !m_out) return TFLA_ERR_NULL;
        if (n_out == n || m_out == m) return TFLA_ERR_STATE;    // every column slab reads n and m
    }
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    StepArgs a;
    a.q = q; a.k = k; a.v = v; a.i_pre = i_pre; a.f_pre = f_pre;
    a.C = C; a.n = variant == TFLA_EXP ? n : nullptr; a.m = variant == TFLA_EXP ? m : nullptr;
    a.C_out = C_out; a.n_out = variant == TFLA_EXP ? n_out : nullptr; a.m_out = variant == TFLA_EXP ? m_out : nullptr;
    a.h = h; a.dqk = dqk; a.dhv = dhv; a.variant = variant; a.dtype = dtype; a.eps = eps; a.softcap = softcap;
    TFLA_LAUNCH(K_STEP, launch_step(a, B * NH, s));
    if (variant == TFLA_SIG) {
        FillList fl{};
        if (n_out) { fl.p[0] = n_out; fl.n[0] = (long)B * NH * dqk; }
        if (m_out) { fl.p[1] = m_out; fl.n[1] = (long)B * NH; }
        if (n_out || m_out) TFLA_LAUNCH(K_FILL, launch_fill_zero4(fl, s));
    }
    return TFLA_OK;
}

int tfla_mlstm_step(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                    const float* C, const float* n, const float* m, int B, int NH, int dqk, int dhv, int variant,
                    int dtype, float eps, void* h, float* C_out, float* n_out, float* m_out, void* stream) {
    return step_impl(q, k, v, i_pre, f_pre, C, n, m, B, NH, dqk, dhv, variant, dtype, eps, 0.0f, h, C_out, n_out, m_out,
                     stream);
}

int tfla_mlstm_layer_step(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                          const void* o_pre, const float* gamma, const float* beta, const float* C, const float* n,
                          const float* m, int B, int NH, int dqk, int dhv, int variant, int dtype, float eps,
                          float gate_softcap, int norm_kind, float norm_eps, void* y, void* h, float* C_out,
                          float* n_out, float* m_out, void* stream) {
    if (norm_kind != TFLA_NORM_RMS && norm_kind != TFLA_NORM_LAYER) return TFLA_ERR_ENUM;
    if (!(gate_softcap >= 0.0f) || !(norm_eps >= 0.0f)) return TFLA_ERR_SHAPE;
    if (!y) return TFLA_ERR_NULL;
    const int rc = step_impl(q, k, v, i_pre, f_pre, C, n, m, B, NH, dqk, dhv, variant, dtype, eps, gate_softcap, h, C_out,
                             n_out, m_out, stream);
    if (rc != TFLA_OK) return rc;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    NormArgs a;
    a.h = h; a.o_pre = o_pre; a.gamma = gamma; a.beta = beta; a.y = y;
    a.rows = (long)B * NH; a.NH = NH; a.T = 1; a.d = dhv; a.kind = norm_kind; a.dtype = dtype; a.eps = norm_eps;
    TFLA_LAUNCH(K_NORM_FWD, launch_norm_gate_fwd(a, s));
    return TFLA_OK;
}

size_t tfla_mlstm_layer_workspace_bytes(int direction, int B, int NH, int T, int dqk, int dhv, int chunk, int variant,
                                        int dtype) {
    const size_t base = tfla_mlstm_workspace_bytes(direction, B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (base == 0 || direction == TFLA_FWD) return base;
    const Dims d = make_dims(B, NH, T, dqk, dhv, chunk, variant, dtype);
    return base + align_up((size_t)d.BH * T * dhv * d.esz) + align_up((size_t)d.BH * norm_row_blocks(T) * 2 * dhv * sizeof(float));
}

int tfla_mlstm_layer_fwd(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                         const void* o_pre, const float* gamma, const float* beta, const float* C0, const float* n0,
                         const float* m0, int B, int NH, int T, int dqk, int dhv, int chunk, int variant, int dtype,
                         float eps, float gate_softcap, int norm_kind, float norm_eps, void* Y, void* H, float* Cn,
                         float* nn, float* mn, float* n_out, float* m_out, void* workspace, size_t workspace_bytes,
                         void* stream) {
    if (norm_kind != TFLA_NORM_RMS && norm_kind != TFLA_NORM_LAYER) return TFLA_ERR_ENUM;
    if (!(gate_softcap >= 0.0f) || !(norm_eps >= 0.0f)) return TFLA_ERR_SHAPE;
    if (!Y) return TFLA_ERR_NULL;
    // Where a workgroup of the H kernel holds whole rows of h~ (bf16, d_hv of 64 or 128, nothing to pad), it forms
    // y = sigma(o~) (.) NORM(h~) itself, next to h~: one read of h~ and one launch less.  Wider heads span several
    // workgroups per row and take the separate kernel below.
    const bool fuse = check_dims(TFLA_FWD, B, NH, T, dqk, dhv, chunk, variant, dtype) == TFLA_OK &&
                      layer_fusion_applies(dqk, dhv, dtype, chunk) && !needs_pad(T, dqk, dhv, chunk) && !misaligned16(o_pre) &&
                      !misaligned16(gamma) && !misaligned16(beta) && !misaligned16(Y);
    const LayerFuse fz{o_pre, gamma, beta, Y, norm_kind, NH, norm_eps};
    const int rc = fwd_impl(q, k, v, i_pre, f_pre, C0, n0, m0, B, NH, T, dqk, dhv, chunk, variant, dtype, eps,
                            gate_softcap, H, Cn, nn, mn, n_out, m_out, workspace, workspace_bytes, stream, fuse ? &fz : nullptr);
    if (rc != TFLA_OK) return rc;
    if (fuse) return TFLA_OK;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    NormArgs a;
    a.h = H; a.o_pre = o_pre; a.gamma = gamma; a.beta = beta; a.y = Y;
    a.rows = (long)B * NH * T; a.NH = NH; a.T = T; a.d = dhv; a.kind = norm_kind; a.dtype = dtype; a.eps = norm_eps;
    TFLA_LAUNCH(K_NORM_FWD, launch_norm_gate_fwd(a, s));
    return TFLA_OK;
}

int tfla_mlstm_layer_bwd(const void* q, const void* k, const void* v, const float* i_pre, const float* f_pre,
                         const void* o_pre, const float* gamma, const float* beta, const float* C0, const float* n0,
                         const float* m0, const void* H, const float* n_out, const float* m_out, const void* dY,
                         const float* dCn, int B, int NH, int T, int dqk, int dhv, int chunk, int variant, int dtype,
                         float eps, float gate_softcap, int norm_kind, float norm_eps, void* dq, void* dk, void* dv,
                         float* d_i_pre, float* d_f_pre, void* do_pre, float* dgamma, float* dbeta, float* dC0,
                         const void* fwd_workspace, size_t fwd_workspace_bytes, void* workspace,
                         size_t workspace_bytes, void* stream) {
    const int rc = check_dims(TFLA_BWD, B, NH, T, dqk, dhv, chunk, variant, dtype);
    if (rc != TFLA_OK) return rc;
    if (norm_kind != TFLA_NORM_RMS && norm_kind != TFLA_NORM_LAYER) return TFLA_ERR_ENUM;
    if (!(gate_softcap >= 0.0f) || !(norm_eps >= 0.0f)) return TFLA_ERR_SHAPE;
    if (!q || !k || !v || !i_pre || !f_pre || !H || !dY || !dq || !dk || !dv || !d_i_pre || !d_f_pre) return TFLA_ERR_NULL;
    if (variant == TFLA_EXP) {
        if (!n_out || !m_out) return TFLA_ERR_NULL;
        const int given = (C0 != nullptr) + (n0 != nullptr) + (m0 != nullptr);
        if (given != 0 && given != 3) return TFLA_ERR_STATE;
    }
    // d: the problem the cell's kernels run (whole chunks, their own head dimensions)
    const Dims d = make_dims(B, NH, T, kernel_dim(dqk), kernel_dim(dhv), chunk, variant, dtype);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return TFLA_ERR_WORKSPACE;
    if (fwd_workspace && ((reinterpret_cast<uintptr_t>(fwd_workspace) & 255) != 0 ||
                          fwd_workspace_bytes < carve_fwd(d, nullptr).bytes))
        return TFLA_ERR_WORKSPACE;
    const size_t base = bwd_total_bytes(d, needs_pad(T, dqk, dhv, chunk));
    const int nblk = norm_row_blocks(T);
    Carver c(reinterpret_cast<char*>(workspace) + base);
    void* dHt = c.take_bytes((size_t)d.BH * T * dhv * d.esz);
    float* part = c.take<float>((size_t)d.BH * nblk * 2 * dhv);
    if (workspace_bytes < base + c.off) return TFLA_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    // NORM + output gate backward: dY -> d h~ (the cell's upstream gradient), d o~, parameter sums
    const bool want_params = dgamma != nullptr || (dbeta != nullptr && norm_kind == TFLA_NORM_LAYER);
    NormBwdArgs a;
    a.h = H; a.o_pre = o_pre; a.gamma = gamma; a.beta = beta; a.dy = dY; a.dh = dHt; a.do_pre = do_pre;
    a.part = want_params ? part : nullptr;
    a.NH = NH; a.T = T; a.d = dhv; a.kind = norm_kind; a.dtype = dtype; a.eps = norm_eps;
    TFLA_LAUNCH(K_NORM_BWD, launch_norm_gate_bwd(a, (int)d.BH, s));
    if (want_params) {
        NormParamGradArgs pg;
        pg.part = part; pg.dgamma = dgamma; pg.dbeta = norm_kind == TFLA_NORM_LAYER ? dbeta : nullptr;
        pg.B = B; pg.NH = NH; pg.nblk = nblk; pg.d = dhv;
        TFLA_LAUNCH(K_NORM_BWD, launch_norm_param_grad(pg, s));
    }
    if (dbeta && norm_kind != TFLA_NORM_LAYER) TFLA_LAUNCH(K_FILL, launch_fill_zero(dbeta, (long)NH * dhv, s));
    return bwd_impl(q, k, v, i_pre, f_pre, C0, n0, m0, n_out, m_out, dHt, dCn, B, NH, T, dqk, dhv, chunk, variant, dtype,
                    eps, gate_softcap, dq, dk, dv, d_i_pre, d_f_pre, dC0, fwd_workspace, fwd_workspace_bytes, workspace,
                    base, stream);
}

int tfla_transfer_gain(const void* h, const void* v, int B, int NH, int T, int dhv, int dtype, int norm_kind,
                       float norm_eps, float* g_before, float* g_after, void* stream) {
    if (dtype != TFLA_F32 && dtype != TFLA_BF16) return TFLA_ERR_ENUM;
    if (norm_kind != TFLA_NORM_RMS && norm_kind != TFLA_NORM_LAYER) return TFLA_ERR_ENUM;
    if (B <= 0 || NH <= 0 || T <= 0 || dhv <= 0 || dhv % 8 != 0 || dhv > 2048 || (long)B * NH > 2147483647L) return TFLA_ERR_SHAPE;
    if (!(norm_eps >= 0.0f)) return TFLA_ERR_SHAPE;
    if (!h || !v || !g_before || !g_after) return TFLA_ERR_NULL;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    GainArgs a;
    a.h = h; a.v = v; a.g_before = g_before; a.g_after = g_after; a.T = T; a.d = dhv; a.kind = norm_kind; a.dtype = dtype;
    a.eps = norm_eps;
    TFLA_LAUNCH(K_GAIN, launch_transfer_gain(a, B * NH, s));
    return TFLA_OK;
}

}  // extern "C"
