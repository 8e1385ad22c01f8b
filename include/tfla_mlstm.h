/*
 * tfla_mlstm.h -- C ABI of the MI355X (gfx950) chunkwise-parallel mLSTM kernels with
 * Tiled Flash Linear Attention.
 *
 * The library computes the hidden states h~_t of the mLSTM cell (paper Sec. 2.1; the NORM
 * layer and the output gate are not part of the kernel, as in Sec. 2.2) in the
 * chunkwise-parallel formulation (Sec. 2.2, App. B.2) with two levels of sequence
 * parallelism (Sec. 3, App. C), for the exponential-input-gate mLSTM ("mLSTMexp") and for the
 * sigmoid-input-gate variant mLSTMsig (Sec. 4.1), and the matching backward pass (App. B.3,
 * App. C.4).  The result does not depend on the chunk size.
 *
 * Conventions (all entry points)
 *  - Every tensor pointer is a DEVICE pointer to a dense row-major array owned by the
 *    caller.  The library never allocates, frees or synchronises; all work is enqueued on
 *    `stream` (a hipStream_t passed as void*; NULL = the default stream).  Outputs are
 *    overwritten, never accumulated into.
 *  - q, k: (B, NH, T, dqk); v, H, dH: (B, NH, T, dhv); element type given by `dtype`
 *    (TFLA_F32: float, TFLA_BF16: bfloat16).  Gate pre-activations i_pre, f_pre and all
 *    per-step scalars: (B, NH, T) float.  States: C (B, NH, dqk, dhv) float,
 *    n (B, NH, dqk) float, m (B, NH) float.
 *  - q is passed unscaled; the kernels apply 1/sqrt(dqk) (it is part of the h~_t equation
 *    of Sec. 2.1).
 *  - States are in the stabilised coordinates of the recurrence (true C = C * exp(m)),
 *    exactly as the recurrence of Sec. 2.1 produces them, so a returned (Cn, nn, mn) can be
 *    passed as (C0, n0, m0) of the next call (chunked continuation of a long sequence).
 *  - variant TFLA_SIG has no normaliser and no max state: n0, m0 and eps are ignored and
 *    nn, mn, n_out, m_out are filled with zeros when non-NULL.
 *  - eps is added to the denominator max{|n^T q~|, exp(-m)}; eps = 0 is the paper's formula.
 *  - Restrictions: chunk % 64 == 0, 64 <= chunk <= 2048, ceil(T / chunk) <= 4096, dqk and dhv
 *    multiples of 8, at most 1024 (at most 512 for TFLA_F32),
 *    B * NH <= 65535.
 *  - T need not be a multiple of chunk (N_c = ceil(T / chunk), Sec. 2.2), and the head dimensions need
 *    not be among the kernels' own widths 64, 128, 256, 512, 1024.  The kernels work on whole chunks and on
 *    those widths: otherwise the library copies the inputs into zero-padded buffers inside the workspace
 *    (which is correspondingly larger, see tfla_mlstm_workspace_bytes), gives the padding steps a forget
 *    gate of one and an input gate of zero, scales q by 1/sqrt of the true dqk, and copies the true part
 *    of the results back, so the result is that of the problem as given; tensor and state pointers must
 *    then be 16-byte aligned (TFLA_ERR_SHAPE).
 *  - Global state: the compute entry points keep none (their only shared data is the read-only table of
 *    kernel instantiations).  The two measurement aids at the end of this file, per-kernel timing
 *    (tfla_profile_*) and the tile-width override (tfla_tile_width), are process-wide, mutable and not
 *    thread-safe: they exist for benchmarks and tests and must not be changed while another thread is
 *    inside the library.  A program that never calls them gets the stateless library.
 *  - Return value: TFLA_OK (0) on success; a negative TFLA_ERR_* code for an invalid
 *    argument (checked before anything is launched, nothing is written); a positive value is
 *    the hipError_t of a failed launch.  No entry point throws or aborts.
 */
#ifndef TFLA_MLSTM_H
#define TFLA_MLSTM_H

#include <stddef.h>

#if defined(__GNUC__)
#define TFLA_API __attribute__((visibility("default")))
#else
#define TFLA_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

enum { TFLA_EXP = 0, TFLA_SIG = 1 };           /* variant: exponential / sigmoid input gate */
enum { TFLA_F32 = 0, TFLA_BF16 = 1 };          /* dtype of q, k, v, H, dH, dq, dk, dv        */
enum { TFLA_FWD = 0, TFLA_BWD = 1 };           /* direction for tfla_mlstm_workspace_bytes   */
enum { TFLA_NORM_RMS = 0, TFLA_NORM_LAYER = 1 }; /* norm_kind of the layer entry points      */

enum {
    TFLA_OK = 0,
    TFLA_ERR_NULL = -1,        /* a required pointer is NULL                                 */
    TFLA_ERR_SHAPE = -2,       /* a dimension is non-positive or violates the restrictions   */
    TFLA_ERR_CHUNK = -3,       /* not an allowed chunk size, or too many chunks              */
    TFLA_ERR_ENUM = -4,        /* unknown variant / dtype / direction                        */
    TFLA_ERR_WORKSPACE = -5,   /* workspace NULL, misaligned (256 B) or too small            */
    TFLA_ERR_STATE = -6,       /* C0/n0/m0 (or Cn/nn/mn) only partly given                   */
    TFLA_ERR_STATIC_LIMIT = -7 /* tfla_mlstm_fwd_static: the problem needs more scratch memory than
                                  TFLA_STATIC_SCRATCH_BYTES                                      */
};

/* size of the scratch array behind tfla_mlstm_fwd_static: 64 MiB on every GPU the library is loaded on */
#define TFLA_STATIC_SCRATCH_BYTES (64u << 20)

/*
 * Forward pass (Sec. 2.2 / App. B.2 for the mathematics, Sec. 3 / App. C for the tiling).
 *   in : q, k, v, i_pre, f_pre; optional initial state C0, n0, m0 (all three NULL = zero
 *        state with m0 = 0; for TFLA_SIG only C0 is read and n0/m0 may be NULL)
 *   out: H (required); optional final state Cn, nn, mn (each may be NULL);
 *        optional n_out, m_out (B, NH, T): the signed normaliser n_t^T q~_t and the max state
 *        m_t of every step, which tfla_mlstm_bwd needs for TFLA_EXP.
 *   workspace: device scratch of at least tfla_mlstm_workspace_bytes(TFLA_FWD, ...) bytes,
 *        256-byte aligned.  Afterwards it holds, in a layout private to the library, what the
 *        backward pass can reuse (the gate vectors, the chunk states C_{k-1} of Sec. 2.2,
 *        C_T and, where the library padded them, its padded copies of q, k, v and the gate
 *        pre-activations): a caller that keeps it untouched until the matching tfla_mlstm_bwd call may pass
 *        it there as fwd_workspace; a caller that does not may overwrite or free it.
 */
TFLA_API int tfla_mlstm_fwd(const void* q, const void* k, const void* v,
                   const float* i_pre, const float* f_pre,
                   const float* C0, const float* n0, const float* m0,
                   int B, int NH, int T, int dqk, int dhv,
                   int chunk, int variant, int dtype, float eps,
                   void* H, float* Cn, float* nn, float* mn,
                   float* n_out, float* m_out,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * The forward pass for callers that cannot allocate device memory or hand over a workspace: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as tfla_mlstm_fwd without the workspace: the scratch memory is a file-scope device array of
 * TFLA_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends; its address on
 * the current device is looked up once, on the first call on that device, which therefore must not be under
 * graph capture).  The call allocates and frees nothing and synchronises nothing.
 *  - A problem whose tfla_mlstm_workspace_bytes(TFLA_FWD, ...) exceeds TFLA_STATIC_SCRATCH_BYTES is rejected
 *    with TFLA_ERR_STATIC_LIMIT before anything is launched (tfla_static_scratch_bytes returns the limit).
 *  - Every call on a GPU uses that GPU's one array: two calls whose kernels can overlap on one GPU (different
 *    streams, or different threads) race on it; calls on one stream are ordered and safe.  The array keeps
 *    the last call's contents; the kernels overwrite what they read, so nothing needs clearing in between.
 *  - The array is not a forward workspace for tfla_mlstm_bwd: pass fwd_workspace = NULL there (recompute).
 */
TFLA_API int tfla_mlstm_fwd_static(const void* q, const void* k, const void* v,
                   const float* i_pre, const float* f_pre,
                   const float* C0, const float* n0, const float* m0,
                   int B, int NH, int T, int dqk, int dhv,
                   int chunk, int variant, int dtype, float eps,
                   void* H, float* Cn, float* nn, float* mn,
                   float* n_out, float* m_out, void* stream);
TFLA_API size_t tfla_static_scratch_bytes(void);

/*
 * Backward pass (App. B.3, App. C.4).  Computes the gradient of
 *     sum_t <dH_t, H_t>  +  <dCn, C_T>
 * with respect to q, k, v, i_pre, f_pre and C0, where -- as the paper prescribes (App. B.3,
 * "Gradients Through Normalizer States") -- the normaliser h_denom and the max states are
 * treated as constants.  For TFLA_SIG this is the exact gradient.
 *   in : q, k, v, i_pre, f_pre, C0/n0/m0 as in the forward call; n_out, m_out as written by
 *        the forward call (required for TFLA_EXP, ignored for TFLA_SIG); dH (required);
 *        dCn (B, NH, dqk, dhv) gradient w.r.t. the returned final state, or NULL for zero.
 *   out: dq, dk (B, NH, T, dqk), dv (B, NH, T, dhv) in `dtype`; d_i_pre, d_f_pre (B, NH, T)
 *        float; dC0 (B, NH, dqk, dhv) float or NULL.  No gradient is produced for n0, m0.
 *   fwd_workspace, fwd_workspace_bytes: NULL / 0, or the workspace of the forward call with
 *        exactly these inputs, dimensions, chunk, variant and dtype, unmodified since that call
 *        (read only here).  With NULL the gate vectors and the chunk states are recomputed
 *        inside this call, and nothing but n_out/m_out has to be kept from the forward call
 *        (App. B.3 leaves open whether states are stored or recomputed; both are offered).
 *        With a forward workspace the results are the same and the recomputation is skipped.
 *   workspace: at least tfla_mlstm_workspace_bytes(TFLA_BWD, ...) bytes, 256-byte aligned;
 *        must not overlap fwd_workspace.
 */
TFLA_API int tfla_mlstm_bwd(const void* q, const void* k, const void* v,
                   const float* i_pre, const float* f_pre,
                   const float* C0, const float* n0, const float* m0,
                   const float* n_out, const float* m_out,
                   const void* dH, const float* dCn,
                   int B, int NH, int T, int dqk, int dhv,
                   int chunk, int variant, int dtype, float eps,
                   void* dq, void* dk, void* dv,
                   float* d_i_pre, float* d_f_pre, float* dC0,
                   const void* fwd_workspace, size_t fwd_workspace_bytes,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * One recurrent step (Sec. 2.1 for TFLA_EXP, Sec. 4.1 for TFLA_SIG): the form used for
 * generation.  For every (batch, head): m' = max(log sigma(f~) + m, i~), C' = f' C + i' k v^T,
 * n' = f' n + i' k with the stabilised gates f' = exp(log sigma(f~) + m - m'), i' = exp(i~ - m'),
 * and h = C'^T q~ / (max{|n'^T q~|, exp(-m')} + eps), q~ = q / sqrt(dqk).  TFLA_SIG: C' =
 * sigma(f~) C + sigma(i~) k v^T, h = C'^T q~.  The state is the one tfla_mlstm_fwd returns
 * (Cn, nn, mn) and accepts (C0, n0, m0), so a prompt processed by tfla_mlstm_fwd can be
 * continued step by step.
 *   in : q, k (B, NH, dqk), v (B, NH, dhv) in `dtype`; i_pre, f_pre (B, NH) float;
 *        C (B, NH, dqk, dhv), n (B, NH, dqk), m (B, NH) float: the state before the step
 *        (n and m both NULL = zero; ignored for TFLA_SIG).
 *   out: h (B, NH, dhv) in `dtype`; C_out, n_out, m_out: the state after the step.  C_out may be
 *        the same buffer as C (updated in place); n_out and m_out must be buffers different from
 *        n and m (they are read by every workgroup of a head) and are required for TFLA_EXP;
 *        for TFLA_SIG they are zero-filled when non-NULL.
 *   dqk, dhv: multiples of 64 in [64, 1024]; B * NH <= 65535.  No workspace is needed.
 */
TFLA_API int tfla_mlstm_step(const void* q, const void* k, const void* v,
                    const float* i_pre, const float* f_pre,
                    const float* C, const float* n, const float* m,
                    int B, int NH, int dqk, int dhv,
                    int variant, int dtype, float eps,
                    void* h, float* C_out, float* n_out, float* m_out, void* stream);

/*
 * The cell inside its layer (Sec. 2.1, hidden-state output equation): soft-capped gates, the
 * cell, the multi-head NORM and the output gate,
 *     i~, f~ <- c tanh(i~ / c), c tanh(f~ / c)        (soft-capping equation of App. E; c = gate_softcap,
 *                                                      0 = no cap; the paper trains with c = 15)
 *     h~     =  cell(q, k, v, i~, f~)                  (exactly tfla_mlstm_fwd)
 *     y      =  sigma(o~) (.) NORM(h~)                 (NORM per (batch, head, step) over dhv)
 * NORM is the RMS norm as Sec. 4.1 writes it, x / sqrt(mean(x^2) + norm_eps) (.) gamma
 * (TFLA_NORM_RMS), or LayerNorm, (x - mean(x)) / sqrt(var(x) + norm_eps) (.) gamma + beta
 * (TFLA_NORM_LAYER).
 *   in : as tfla_mlstm_fwd, plus o_pre (B, NH, T, dhv) in `dtype` or NULL (gate = 1);
 *        gamma, beta (NH, dhv) float, each may be NULL (1 and 0; beta is ignored by the RMS norm).
 *   out: Y (B, NH, T, dhv) in `dtype` (required); H (required): the cell output h~, which the
 *        backward call needs; Cn, nn, mn, n_out, m_out as in tfla_mlstm_fwd.
 *   workspace: tfla_mlstm_layer_workspace_bytes(TFLA_FWD, ...) bytes; reusable by the backward
 *        call as fwd_workspace under the same conditions as for tfla_mlstm_fwd.
 * Additional errors: TFLA_ERR_ENUM for an unknown norm_kind, TFLA_ERR_SHAPE for a negative
 * gate_softcap or norm_eps.
 */
TFLA_API int tfla_mlstm_layer_fwd(const void* q, const void* k, const void* v,
                         const float* i_pre, const float* f_pre,
                         const void* o_pre, const float* gamma, const float* beta,
                         const float* C0, const float* n0, const float* m0,
                         int B, int NH, int T, int dqk, int dhv,
                         int chunk, int variant, int dtype, float eps,
                         float gate_softcap, int norm_kind, float norm_eps,
                         void* Y, void* H, float* Cn, float* nn, float* mn,
                         float* n_out, float* m_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of tfla_mlstm_layer_fwd: the exact derivative of the output gate and the NORM turns dY
 * into the cell's upstream gradient, the cell's backward is tfla_mlstm_bwd's (normaliser held
 * constant, App. B.3), and the gate gradients are taken through the soft-cap.
 *   in : the forward inputs; H, n_out, m_out as written by the forward call; dY (B, NH, T, dhv);
 *        dCn or NULL.
 *   out: dq, dk, dv, d_i_pre, d_f_pre, dC0 as in tfla_mlstm_bwd; do_pre (B, NH, T, dhv) in `dtype`
 *        (may be NULL; not written when o_pre is NULL); dgamma, dbeta (NH, dhv) float, each may be
 *        NULL (dbeta is zero-filled for the RMS norm).  The parameter gradients are summed over
 *        batch and time in a fixed order (bit-reproducible).
 *   workspace: tfla_mlstm_layer_workspace_bytes(TFLA_BWD, ...) bytes, 256-byte aligned.
 */
TFLA_API int tfla_mlstm_layer_bwd(const void* q, const void* k, const void* v,
                         const float* i_pre, const float* f_pre,
                         const void* o_pre, const float* gamma, const float* beta,
                         const float* C0, const float* n0, const float* m0,
                         const void* H, const float* n_out, const float* m_out,
                         const void* dY, const float* dCn,
                         int B, int NH, int T, int dqk, int dhv,
                         int chunk, int variant, int dtype, float eps,
                         float gate_softcap, int norm_kind, float norm_eps,
                         void* dq, void* dk, void* dv,
                         float* d_i_pre, float* d_f_pre,
                         void* do_pre, float* dgamma, float* dbeta, float* dC0,
                         const void* fwd_workspace, size_t fwd_workspace_bytes,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * One generation step of the layer: tfla_mlstm_step with soft-capped gates, followed by the NORM and
 * the output gate of tfla_mlstm_layer_fwd on the step's hidden state.
 *   in : as tfla_mlstm_step, plus o_pre (B, NH, dhv) in `dtype` or NULL, gamma, beta (NH, dhv) float or NULL.
 *   out: y (B, NH, dhv) in `dtype` (required); h: the cell output (required, also a scratch of the call);
 *        C_out, n_out, m_out as in tfla_mlstm_step.
 */
TFLA_API int tfla_mlstm_layer_step(const void* q, const void* k, const void* v,
                          const float* i_pre, const float* f_pre,
                          const void* o_pre, const float* gamma, const float* beta,
                          const float* C, const float* n, const float* m,
                          int B, int NH, int dqk, int dhv,
                          int variant, int dtype, float eps,
                          float gate_softcap, int norm_kind, float norm_eps,
                          void* y, void* h, float* C_out, float* n_out, float* m_out, void* stream);

/* Workspace bytes of the two layer entry points (host function; 0 for invalid arguments). */
TFLA_API size_t tfla_mlstm_layer_workspace_bytes(int direction, int B, int NH, int T, int dqk, int dhv,
                                        int chunk, int variant, int dtype);

/*
 * Gains of the transfer-behaviour experiment (Sec. 4.1, gain equation; App. D.2): for every
 * (batch, head) the time averages of max_i|h~_t,i| / max_i|v_t,i| (g_before) and of
 * max_i|NORM(h~_t)_i| / max_i|v_t,i| (g_after), NORM with unit scale and no shift.
 *   in : h, v (B, NH, T, dhv) in `dtype`; dhv a multiple of 8, at most 2048.
 *   out: g_before, g_after (B, NH) float.
 */
TFLA_API int tfla_transfer_gain(const void* h, const void* v, int B, int NH, int T, int dhv,
                       int dtype, int norm_kind, float norm_eps,
                       float* g_before, float* g_after, void* stream);

/*
 * Bytes of workspace the call with these arguments needs (host function, launches nothing).
 * Returns 0 if the arguments are invalid.
 */
TFLA_API size_t tfla_mlstm_workspace_bytes(int direction, int B, int NH, int T, int dqk, int dhv,
                                  int chunk, int variant, int dtype);

/* Validates the arguments of a forward / backward call without launching anything; returns
 * the status the call would return before its first launch (host function). */
TFLA_API int tfla_mlstm_check(int direction, int B, int NH, int T, int dqk, int dhv,
                     int chunk, int variant, int dtype);

/* Human-readable text for a status code (static storage). */
TFLA_API const char* tfla_status_string(int status);

/*
 * Optional per-kernel timing (host functions; not thread-safe; process-wide state).
 * tfla_profile_enable(n > 0) creates n pairs of HIP events and makes every kernel launch of
 * the two entry points record one pair on the caller's stream until n launches have been
 * recorded since the last read; tfla_profile_enable(0) switches timing off and destroys the
 * events.  tfla_profile_read synchronises on the recorded events, adds their elapsed times to
 * the per-kernel totals and returns the totals of kernel family `kernel`
 * (0 <= kernel < tfla_profile_kernels()); name receives the family's name (NUL-terminated).
 * These are the only entry points that create HIP objects; tfla_mlstm_fwd/bwd never do.
 */
TFLA_API int tfla_profile_enable(int max_launches);
TFLA_API int tfla_profile_read(int kernel, char* name, int name_len, double* total_ms, long* launches);
TFLA_API int tfla_profile_kernels(void);

/*
 * Measurement aid for tile-size sweeps (Sec. 3: the kernels' tile sizes are free parameters of the method; host
 * function, process-wide state, not thread-safe): width of the output-column block of the bf16 tiled kernels.
 * 0 (default) = chosen per kernel and shape; 64 or 128 = that width wherever it divides the tiled dimension;
 * 256 = same as 0 (256-wide blocks are already taken wherever they are built).  Results do not depend on it;
 * workspace layouts do, so set it before tfla_mlstm_workspace_bytes and keep it for the calls that use that
 * workspace.  Returns TFLA_OK or TFLA_ERR_ENUM.
 */
TFLA_API int tfla_tile_width(int width);

/* Library version, major * 1000 + minor. */
TFLA_API int tfla_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TFLA_MLSTM_H */
