/*
 * gsa.h -- C ABI of libgsa: Gated Slot Attention (GSA) on AMD MI355X (gfx950).
 *
 * The operator (paper, Section 3.2, Eq. (gsa)), per sequence and head, with
 * g_t = log alpha_t the log forget gate (one value per memory slot):
 *
 *     Kt_t = Diag(exp g_t) Kt_{t-1} + (1 - exp g_t) (x) k_t       in R^{m x d_k}
 *     Vt_t = Diag(exp g_t) Vt_{t-1} + (1 - exp g_t) (x) v_t       in R^{m x d_v}
 *     o_t  = Vt_t^T softmax(scale * Kt_t q_t)                     softmax over the m slots
 *
 * Token t reads the memories after its own write.  The paper applies no score
 * scaling; scale = 1.0f reproduces it.
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer to a dense row-major array with
 *     the last index fastest.  The caller owns every buffer, including the
 *     workspace; the library never allocates, frees or synchronises.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns at once.
 *   - q,k,v,o,dO,dq,dk,dv have element type `dtype` (fp32 or bf16); g, dg,
 *     z_saved and every memory (slot state) are fp32.  Accumulation is fp32.
 *   - g must be <= 0.  Values below -30 are treated as -30 (alpha = 9e-14,
 *     below fp32 resolution of the result).  NaN gates give NaN outputs.
 *   - Outputs must not overlap inputs, the workspace or each other: gsa_fwd*
 *     and gsa_bwd* check this on the host and return GSA_ERR_SHAPE (the decode
 *     step updates its memories in place, that is its contract; its other
 *     arguments are the caller's to keep apart).
 *   - Errors are return codes; arguments are validated on the host before any
 *     device work is enqueued, and a failed call enqueues nothing.
 *   - Supported shapes: m in {16, 32, 64, 128}; d_k and d_v
 *     multiples of 64, at most 1024; H, B >= 1; T >= 0 (T = 0 does nothing).  Anything
 *     else returns GSA_ERR_UNSUPPORTED.
 */
#ifndef GSA_H
#define GSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GSA_OK = 0,
    GSA_ERR_NULL = 1,        /* a required pointer is NULL */
    GSA_ERR_SHAPE = 2,       /* a dimension is out of range or inconsistent */
    GSA_ERR_UNSUPPORTED = 3, /* valid request this build has no kernel for */
    GSA_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small */
    GSA_ERR_HIP = 5          /* the HIP runtime reported an error at launch */
} gsa_status;

typedef enum { GSA_F32 = 0, GSA_BF16 = 1 } gsa_dtype;

/*
 * Problem shape.  Two forms:
 *   batch  : cu_seqlens == NULL; B sequences of T tokens; n_seqs is ignored.
 *   packed : cu_seqlens != NULL (device int32 [n_seqs+1], non-decreasing,
 *            cu_seqlens[0] = 0, cu_seqlens[n_seqs] = T); B must be 1; sequence
 *            s covers tokens cu_seqlens[s] .. cu_seqlens[s+1]-1 and starts from
 *            its own initial memories.  Offsets are clamped into [0,T] on the
 *            device; tokens covered by no sequence receive no output.
 * Memories are indexed by sequence: [n, H, m, d] with n = B (batch) or n_seqs.
 */
typedef struct {
    int32_t B, T, H, d_k, d_v, m;
    int32_t dtype;              /* gsa_dtype */
    float scale;
    const int32_t *cu_seqlens;  /* device pointer or NULL */
    int32_t n_seqs;
    int32_t keep_states;        /* 0: the backward recomputes the per-chunk memories (the paper's default,
                                 * Section 4 "Efficiency").  Nonzero: "GSA w/o recomp." of the throughput
                                 * and memory figures there: gsa_fwd* leaves them in the workspace and
                                 * gsa_bwd* reads them from it; see gsa_workspace_bytes. */
} gsa_problem;

const char *gsa_status_string(gsa_status s);

/* Version of this ABI (bumped when a signature changes). */
int32_t gsa_abi_version(void);

/*
 * Bytes of workspace gsa_fwd (want_bwd = 0) or gsa_bwd (want_bwd != 0) needs
 * for this problem.  The workspace holds the per-chunk memories of the
 * chunkwise evaluation (Appendix A, Eq. (gla-chunk-gate)) and small per-token
 * scratch; its contents are meaningless to the caller.  It must be 256-byte
 * aligned.  Host call, touches no device.
 * With p->keep_states set, both calls need the larger (want_bwd) size, and
 * gsa_bwd* must be given the very workspace, untouched since, that a gsa_fwd*
 * call with the same problem, the same q,k,v,g,s,K0,V0 and the same options
 * filled last: it then skips the recomputation (the gate tables and the forward
 * scan).  The library cannot check that; a workspace that went through another
 * call in between gives wrong gradients, not an error.  The memories kept are
 * (d_k + d_v) * m elements of dtype per chunk of 64 (bf16) or 32 (fp32) tokens
 * and head, i.e. for m = 64 and bf16 as many bytes as k and v together.
 */
gsa_status gsa_workspace_bytes(const gsa_problem *p, int want_bwd, size_t *bytes);

/*
 * Forward (Eq. (gsa); chunkwise evaluation after Appendix A and Algorithm 1).
 *   q,k [B,T,H,d_k]  v [B,T,H,d_v]  (dtype)      g [B,T,H,m] fp32
 *   K0,V0 [n,H,m,d_k|d_v] fp32 initial memories, or NULL for zeros
 *   o [B,T,H,d_v] (dtype)                       output
 *   z_saved [B,T,H,m] fp32 or NULL             pre-softmax slot scores
 *                                               scale*Kt_t q_t, the one tensor
 *                                               gsa_bwd needs besides the inputs
 *   KT,VT [n,H,m,d] fp32 or NULL               memories after the last token
 */
gsa_status gsa_fwd(const gsa_problem *p,
                   const void *q, const void *k, const void *v, const float *g,
                   const float *K0, const float *V0,
                   void *o, float *z_saved, float *KT, float *VT,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward of L = sum <dO_t,o_t> + <dKT,Kt_T> + <dVT,Vt_T> (Algorithm 1,
 * backward pass; the per-chunk memories are recomputed from k,v,g rather than
 * stored by the forward).
 *   inputs : q,k,v,g,K0,V0 as given to gsa_fwd; z_saved as written by it;
 *            dO [B,T,H,d_v] (dtype); dKT,dVT [n,H,m,d] fp32 or NULL (zeros)
 *   outputs: dq,dk [B,T,H,d_k], dv [B,T,H,d_v] (dtype); dg [B,T,H,m] fp32,
 *            the gradient with respect to g with the write intensity
 *            1 - exp(g) tied to it; dK0,dV0 [n,H,m,d] fp32 or NULL
 */
gsa_status gsa_bwd(const gsa_problem *p,
                   const void *q, const void *k, const void *v, const float *g,
                   const float *K0, const float *V0, const float *z_saved, const void *dO,
                   const float *dKT, const float *dVT,
                   void *dq, void *dk, void *dv, float *dg, float *dK0, float *dV0,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same two calls for the variants the paper ablates (Section 4, ablation
 * table) and the form Algorithm 1 is written in:
 *   s       [B,T,H,m] fp32 or NULL.  The write intensity as an input of its own
 *           (Algorithm 1 takes I beside the gates): the memories are updated as
 *           Kt_t = Diag(exp g_t) Kt_{t-1} + s_t (x) k_t (same for Vt).  NULL means
 *           s_t = 1 - exp(g_t), i.e. gsa_fwd/gsa_bwd.  With g = 0 and s = phi
 *           (a cumulative softmax) this is ABC, Eqs. (abc_recurrent), (abc_phi).
 *   readout how the slot scores z_t = scale*Kt_t q_t become the read weights:
 *           softmax over the slots (Eq. (gsa)), or element by element the
 *           identity, Swish z*sigmoid(z), ReLU, or ReLU squared.
 *   gate_tau 0: g is the log gate, as in gsa_fwd.  > 0: g holds gate LOGITS u and
 *           the log gate is logsigmoid(u) / gate_tau, i.e. the layer's
 *           alpha = sigmoid(W x)^(1/tau) of Section 3.3 (tau = 8 in the paper)
 *           evaluated inside the kernels; gsa_bwd_ex then returns in dg the
 *           gradient with respect to the logits.
 *   feature_map GSA_FEATURE_NONE: q, k, v enter Eq. (gsa) as given.  GSA_FEATURE_SWISH:
 *           they hold the layer's raw projections W_q x, W_k x, W_v x and the
 *           kernels apply phi(x) = x*sigmoid(x) of Section 3.3 to them as they load
 *           them (rounded once more to dtype, since they feed the matrix
 *           cores); gsa_bwd_ex then returns dq, dk, dv with respect to the raw
 *           values.
 *   gsa_bwd_ex: with s given, dg is the gradient through the decay alone and
 *           ds [B,T,H,m] fp32 (required then) receives the gradient of s; with
 *           s NULL, ds is not touched and dg is as in gsa_bwd.  The same s,
 *           readout, gate_tau and feature_map must be passed to both calls.
 * Errors as for gsa_fwd/gsa_bwd; an unknown readout or feature_map or a
 * negative or NaN gate_tau returns GSA_ERR_SHAPE.
 * gsa_decode_step_ex (below) is the decode step with the same options.
 */
typedef enum {
    GSA_READOUT_SOFTMAX = 0, GSA_READOUT_IDENTITY = 1, GSA_READOUT_SWISH = 2, GSA_READOUT_RELU = 3,
    GSA_READOUT_RELU2 = 4
} gsa_readout;
typedef enum { GSA_FEATURE_NONE = 0, GSA_FEATURE_SWISH = 1 } gsa_feature_map;

gsa_status gsa_fwd_ex(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map,
                      const void *q, const void *k, const void *v, const float *g, const float *s,
                      const float *K0, const float *V0,
                      void *o, float *z_saved, float *KT, float *VT,
                      void *workspace, size_t workspace_bytes, void *stream);

gsa_status gsa_bwd_ex(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map,
                      const void *q, const void *k, const void *v, const float *g, const float *s,
                      const float *K0, const float *V0, const float *z_saved, const void *dO,
                      const float *dKT, const float *dVT,
                      void *dq, void *dk, void *dv, float *dg, float *ds, float *dK0, float *dV0,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * gsa_fwd_ex with the layer's output epilogue fused into the kernel that writes o (Section 3.3: the layer
 * feeds RMSNorm(Swish(o)), over the concatenated heads, into its output projection):
 *   act     [B,T,H,d_v] (dtype) or NULL: Swish(o) = o*sigmoid(o), computed from o as stored (rounded to dtype)
 *   act_ssq [B,T,H,ns] fp32 or NULL, ns = ceil(d_v / gsa_act_slice_cols(dtype)): the sum of act^2 (of the
 *           stored values) over each slice of gsa_act_slice_cols(dtype) consecutive columns of a head.  The
 *           RMS norm's statistic for token t is sqrt(sum over h and slices / (H*d_v)): no pass of its own
 *           over the tensor.
 *   o       may be NULL here (inference: nothing reads the un-activated output); with both o and act NULL
 *           the call returns GSA_ERR_NULL.
 * Everything else as for gsa_fwd_ex.  The backward of the activation stays with the layer's norm backward,
 * which passes over these tensors anyway; gsa_bwd* take dO, the gradient with respect to o.
 */
gsa_status gsa_fwd_act(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map,
                       const void *q, const void *k, const void *v, const float *g, const float *s,
                       const float *K0, const float *V0,
                       void *o, void *act, float *act_ssq, float *z_saved, float *KT, float *VT,
                       void *workspace, size_t workspace_bytes, void *stream);
int32_t gsa_act_slice_cols(int32_t dtype);   /* 0 for an unknown dtype */

/*
 * One recurrent step of Eq. (gsa) (the decode form, Figure 1) for B*H
 * independent memories, which are read, updated and written back in place.
 *   q,k [B,H,d_k]  v [B,H,d_v] (dtype)   g [B,H,m] fp32
 *   K_state [B,H,m,d_k], V_state [B,H,m,d_v] fp32, in/out
 *   o [B,H,d_v] (dtype)
 * Needs no workspace.
 */
gsa_status gsa_decode_step(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m,
                           int32_t dtype, float scale,
                           const void *q, const void *k, const void *v, const float *g,
                           float *K_state, float *V_state, void *o, void *stream);

/*
 * The same step (Eq. (gsa), decode form) for callers with few memories in flight
 * (small batches, the token-by-token generation loop of Figure 4c): with B*H up
 * to 64 each memory pair is spread over m/4 workgroups, whose partial read-outs
 * (each with its own softmax maximum and sum) pass through the workspace and
 * are merged by a second kernel in a fixed order; above that the call does what
 * gsa_decode_step does.  Results agree with gsa_decode_step up to fp32 rounding
 * order and are reproducible run to run.
 *   workspace: device memory, 256-byte aligned, at least
 *   gsa_decode_workspace_bytes(...) bytes (0 when the split form is not used);
 *   contents meaningless to the caller; calls sharing a workspace must not overlap.
 * Errors as for gsa_decode_step, plus GSA_ERR_WORKSPACE.
 */
gsa_status gsa_decode_workspace_bytes(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, size_t *bytes);
gsa_status gsa_decode_step_ws(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m,
                              int32_t dtype, float scale,
                              const void *q, const void *k, const void *v, const float *g,
                              float *K_state, float *V_state, void *o,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * gsa_decode_step_ws for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * split form's partial read-outs go through an array built into the library (4 MiB of device
 * memory per GPU, held until the process ends) instead of a caller's workspace; the call
 * allocates nothing and frees nothing.  The array's address is looked up on the first call on
 * each device (make that call outside a capture).  Arguments and results as for
 * gsa_decode_step_ws on the same inputs.  A problem whose split form needs more than the array
 * holds -- B*H <= 64 and B*H * (m/4) * (d_v + 2) > 1,048,576 floats -- returns
 * GSA_ERR_WORKSPACE and enqueues nothing (above 64 memory pairs no scratch is needed and any
 * size is taken).  Every call on one GPU shares that GPU's array: calls that overlap in time on
 * one GPU (different streams, or threads) race; nothing in it needs clearing between calls.
 */
gsa_status gsa_decode_step_static(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m,
                                  int32_t dtype, float scale,
                                  const void *q, const void *k, const void *v, const float *g,
                                  float *K_state, float *V_state, void *o, void *stream);

/*
 * The decode step (Eq. (gsa), decode form) with the options of gsa_fwd_ex (Algorithm 1's
 * separate write intensity; the read-outs of Section 4's ablation table): s [B,H,m] fp32
 * or NULL, readout a gsa_readout, gate_tau and feature_map as there.  workspace may be NULL (then the call behaves like
 * gsa_decode_step) or as for gsa_decode_step_ws.
 */
gsa_status gsa_decode_step_ex(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m,
                              int32_t dtype, float scale, int32_t readout, float gate_tau, int32_t feature_map,
                              const void *q, const void *k, const void *v, const float *g, const float *s,
                              float *K_state, float *V_state, void *o,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * Per-kernel timing for roofline measurements (diagnostics; not part of the operator).
 * While enabled, every kernel the library launches is bracketed by a pair of HIP events
 * recorded on the caller's stream.  gsa_profile_read waits for the recorded events and
 * returns, for kernel slot `index` (0 .. n-1; GSA_ERR_SHAPE past the end), its name, the
 * milliseconds accumulated since the last reset and the number of launches.  The name
 * points to static storage.  Enabling costs two event records per launch; timed
 * throughput runs keep it off.
 */
gsa_status gsa_profile_enable(int on);
gsa_status gsa_profile_reset(void);
gsa_status gsa_profile_read(int32_t index, const char **name, double *ms, int64_t *launches);

/*
 * Bandwidth probe: copies `bytes` (a multiple of 16) from device memory `src` to device
 * memory `dst` (both 16-byte aligned, not overlapping) with one plain kernel
 * ("copy_probe_kernel", streaming loads and stores) on `stream`.  It reads and writes exactly `bytes` each, which makes
 * it the yardstick for hardware memory counters and for the copy rate this chip sustains.
 * Timed in slot "copy_probe_kernel" while profiling is enabled.
 */
gsa_status gsa_profile_copy(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GSA_H */
