// C ABI of libgsa (see include/gsa.h): argument validation, workspace planning, dispatch.
// All checks run on the host before anything is enqueued.
#include "../../include/gsa.h"
#include "gsa_common.h"
#include "gsa_internal.h"

namespace {

using gsa::Plan;
using gsa::Work;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool valid_m(int m, bool sequence_kernels)
{
    (void)sequence_kernels;
    return m == 16 || m == 32 || m == 64 || m == 128;
}

gsa_status make_plan(const gsa_problem *p, Plan *pl)
{
    if (!p) return GSA_ERR_NULL;
    if (p->B < 1 || p->T < 0 || p->H < 1 || p->d_k < 1 || p->d_v < 1 || p->m < 1) return GSA_ERR_SHAPE;
    if (p->dtype != GSA_F32 && p->dtype != GSA_BF16) return GSA_ERR_SHAPE;
    if (!(p->scale == p->scale)) return GSA_ERR_SHAPE;
    if (p->cu_seqlens) {
        if (p->B != 1 || p->n_seqs < 1) return GSA_ERR_SHAPE;
    }
    if (p->d_k % 64 || p->d_v % 64 || p->d_k > 1024 || p->d_v > 1024) return GSA_ERR_UNSUPPORTED;
    if (!valid_m(p->m, true)) return GSA_ERR_UNSUPPORTED;
    const int64_t tokens = (int64_t)p->B * p->T;
    if (tokens * p->H * (int64_t)(p->d_k > p->d_v ? p->d_k : p->d_v) >= ((int64_t)1 << 40)) return GSA_ERR_SHAPE;
    pl->B = p->B; pl->T = p->T; pl->H = p->H; pl->d_k = p->d_k; pl->d_v = p->d_v; pl->m = p->m;
    pl->dtype = p->dtype; pl->scale = p->scale; pl->cu_seqlens = p->cu_seqlens;
    pl->n_seqs = p->cu_seqlens ? p->n_seqs : p->B;
    pl->keep = p->keep_states != 0;
    pl->tokens = tokens;
    pl->chunk = gsa::chunk_of_dtype(p->dtype);
    const int64_t slots = p->cu_seqlens ? ((int64_t)p->T / pl->chunk + p->n_seqs)
                                        : (int64_t)p->B * ((p->T + pl->chunk - 1) / pl->chunk);
    if (slots > 0x3fffffff) return GSA_ERR_SHAPE;
    pl->chunk_slots = (int32_t)slots;
    const size_t esz = p->dtype == GSA_BF16 ? 2 : 4;
    const size_t M = p->m, dk = p->d_k, dv = p->d_v, D = dk + dv, C = pl->chunk, KM = M < 32 ? 32 : M;
    const size_t ch = (size_t)slots * p->H;                 // (chunk, head) records
    // memory snapshots: every record is [Kt | Vt] in natural orientation, [m][d_k] then [m][d_v]
    // (the apply kernel transposes the slices it needs on their way into LDS)
    pl->lay = {(long long)(M * D), 0, (long long)(M * dk)};
    const size_t tokm = (size_t)tokens * p->H * M * sizeof(float);
    size_t off = 0;
    pl->off_table = off;  off += align_up(p->cu_seqlens ? (size_t)slots * 4 * sizeof(int32_t) : 0);
    pl->off_seqtab = off; off += align_up(p->cu_seqlens ? (size_t)p->n_seqs * 4 * sizeof(int32_t) : 0);
    pl->off_segbase = off; off += align_up(p->cu_seqlens ? ((size_t)p->n_seqs + 1) * sizeof(int32_t) : 0);
    pl->off_Wf = off;     off += align_up(ch * M * C * esz);
    pl->off_dec = off;    off += align_up(ch * M * sizeof(float));
    pl->off_tA = off;     off += align_up(ch * C * C * esz);
    pl->off_tP = off;     off += align_up(ch * C * KM * esz);
    // Long sequences: the scans cut them into segments (gsa_scan.hip).  The host knows the longest a
    // sequence can be (T tokens, also in packed form) and provides for that many segments per sequence;
    // this is only done while the sequences alone do not fill the chip.
    {
        const int64_t max_nch = ((int64_t)p->T + pl->chunk - 1) / pl->chunk;
        const int64_t nseg = (max_nch + gsa::kSegChunks - 1) / gsa::kSegChunks;
        const int64_t base = (int64_t)pl->n_seqs * p->H * ((dk + dv) / 64);   // workgroups of an unsegmented scan
        const bool on = max_nch > gsa::kSegChunks + gsa::kSegChunks / 2 && base < 512 && base * nseg <= 8192;
        pl->seg_chunks = gsa::kSegChunks;
        pl->max_seg = on ? (int32_t)nseg : 1;
    }
    const size_t nsum = pl->max_seg > 1 ? (size_t)pl->n_seqs * pl->max_seg * p->H : 0;
    pl->off_sumY = off;   off += align_up(nsum * M * D * sizeof(float));
    pl->off_sumD = off;   off += align_up(nsum * (D / 64) * M * sizeof(float));
    pl->off_S = off;
    pl->total_fwd = off + align_up(ch * M * D * esz);
    off += align_up(ch * M * D * esz);
    pl->off_SF = off;     off += align_up((size_t)pl->n_seqs * p->H * M * D * esz);
    pl->off_Wr = off;     off += align_up(ch * 2 * M * C * esz);
    pl->off_E = off;      off += align_up(ch * M * D * esz);
    pl->off_tBT = off;    off += align_up(ch * C * C * esz);
    pl->off_tA2T = off;   off += align_up(ch * C * C * esz);
    pl->off_tAvT = off;   off += align_up(ch * C * C * esz);
    pl->off_tSbe = off;   off += align_up(ch * C * KM * esz);
    pl->off_dz = off;     off += align_up(tokm);
    pl->off_dgf = off;    off += align_up(tokm);
    pl->total_bwd = off;
    if (pl->keep) pl->total_fwd = pl->total_bwd;   // one workspace goes through both calls
    return GSA_OK;
}

Work make_work(const Plan &pl, void *ws)
{
    unsigned char *b = static_cast<unsigned char *>(ws);
    Work w;
    w.table = reinterpret_cast<int32_t *>(b + pl.off_table);
    w.seqtab = reinterpret_cast<int32_t *>(b + pl.off_seqtab);
    w.segbase = reinterpret_cast<int32_t *>(b + pl.off_segbase);
    w.Wf = b + pl.off_Wf;
    w.dec = reinterpret_cast<float *>(b + pl.off_dec);
    w.sumY = reinterpret_cast<float *>(b + pl.off_sumY);
    w.sumD = reinterpret_cast<float *>(b + pl.off_sumD);
    w.S = b + pl.off_S;
    w.tA = b + pl.off_tA;
    w.tP = b + pl.off_tP;
    w.SF = b + pl.off_SF;
    w.Wr = b + pl.off_Wr;
    w.E = b + pl.off_E;
    w.tBT = b + pl.off_tBT;
    w.tA2T = b + pl.off_tA2T;
    w.tAvT = b + pl.off_tAvT;
    w.tSbe = b + pl.off_tSbe;
    w.dz = reinterpret_cast<float *>(b + pl.off_dz);
    w.dgf = reinterpret_cast<float *>(b + pl.off_dgf);
    return w;
}

// An argument's bytes; n = 0 or p = NULL: absent.
struct Span {
    const void *p;
    size_t n;
};

// True when some output (the first n_out spans) shares a byte with any other span.
bool outputs_overlap(const Span *spans, int n_out, int n_all)
{
    for (int i = 0; i < n_out; ++i) {
        if (!spans[i].p || !spans[i].n) continue;
        const uintptr_t a0 = reinterpret_cast<uintptr_t>(spans[i].p), a1 = a0 + spans[i].n;
        for (int j = 0; j < n_all; ++j) {
            if (j == i || !spans[j].p || !spans[j].n) continue;
            if (j < i && j < n_out) continue;   // that pair was looked at from the other side
            const uintptr_t b0 = reinterpret_cast<uintptr_t>(spans[j].p), b1 = b0 + spans[j].n;
            if (a0 < b1 && b0 < a1) return true;
        }
    }
    return false;
}

gsa_status check_workspace(void *ws, size_t have, size_t need)
{
    if (need == 0) return GSA_OK;
    if (!ws) return GSA_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % kAlign) return GSA_ERR_WORKSPACE;
    if (have < need) return GSA_ERR_WORKSPACE;
    return GSA_OK;
}

gsa_status decode_checks(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, int32_t dtype, float scale)
{
    if (B < 0 || H < 1 || d_k < 1 || d_v < 1 || m < 1) return GSA_ERR_SHAPE;
    if (dtype != GSA_F32 && dtype != GSA_BF16) return GSA_ERR_SHAPE;
    if (!(scale == scale)) return GSA_ERR_SHAPE;
    if ((int64_t)B * H > 0x7fffffff) return GSA_ERR_SHAPE;
    if (d_k % 64 || d_v % 64 || d_k > 1024 || d_v > 1024) return GSA_ERR_UNSUPPORTED;
    if (!valid_m(m, false)) return GSA_ERR_UNSUPPORTED;
    return GSA_OK;
}

gsa_status decode_any(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, int32_t dtype, float scale,
                      const void *q, const void *k, const void *v, const float *g, float *K_state, float *V_state,
                      void *o, bool with_ws, void *workspace, size_t workspace_bytes, void *stream,
                      const float *s = nullptr, int32_t readout = GSA_READOUT_SOFTMAX, float gate_tau = 0.f,
                      int32_t feature_map = GSA_FEATURE_NONE)
{
    const gsa_status st = decode_checks(B, H, d_k, d_v, m, dtype, scale);
    if (st != GSA_OK) return st;
    if (readout < GSA_READOUT_SOFTMAX || readout > GSA_READOUT_RELU2 || !(gate_tau >= 0.f)) return GSA_ERR_SHAPE;
    if (feature_map != GSA_FEATURE_NONE && feature_map != GSA_FEATURE_SWISH) return GSA_ERR_SHAPE;
    if (B == 0) return GSA_OK;
    if (!q || !k || !v || !g || !K_state || !V_state || !o) return GSA_ERR_NULL;
    const void *ptrs[] = {q, k, v, g, K_state, V_state, o, s};
    for (const void *ptr : ptrs)
        if (!aligned16(ptr)) return GSA_ERR_SHAPE;
    float *scratch = nullptr;
    if (with_ws) {
        const size_t need = gsa::decode_scratch_floats(B * H, d_v, m) * sizeof(float);
        const gsa_status ws = check_workspace(workspace, workspace_bytes, need);
        if (ws != GSA_OK) return ws;
        if (need) scratch = static_cast<float *>(workspace);
    }
    const hipError_t e = gsa::launch_decode(B * H, d_k, d_v, m, dtype, scale, q, k, v, g, K_state, V_state, o,
                                            scratch, s, readout | (feature_map ? gsa::kFeatureMapBit : 0), gate_tau,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : GSA_ERR_HIP;
}

}  // namespace

extern "C" {

const char *gsa_status_string(gsa_status s)
{
    switch (s) {
    case GSA_OK: return "ok";
    case GSA_ERR_NULL: return "a required pointer is NULL";
    case GSA_ERR_SHAPE: return "a dimension is out of range or inconsistent, or an output overlaps another argument";
    case GSA_ERR_UNSUPPORTED: return "shape not supported by this build";
    case GSA_ERR_WORKSPACE:
        return "workspace missing, misaligned or too small (or the problem exceeds the built-in scratch)";
    case GSA_ERR_HIP: return "HIP runtime error at launch";
    }
    return "unknown status";
}

int32_t gsa_abi_version(void) { return 2; }

gsa_status gsa_workspace_bytes(const gsa_problem *p, int want_bwd, size_t *bytes)
{
    if (!bytes) return GSA_ERR_NULL;
    Plan pl;
    const gsa_status st = make_plan(p, &pl);
    if (st != GSA_OK) return st;
    *bytes = want_bwd ? pl.total_bwd : pl.total_fwd;
    return GSA_OK;
}

namespace {
gsa_status fwd_any(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map, const void *q,
                   const void *k, const void *v, const float *g, const float *s, const float *K0, const float *V0,
                   void *o, float *z_saved, float *KT, float *VT, void *workspace, size_t workspace_bytes,
                   void *stream, void *act = nullptr, float *ssq = nullptr, bool with_act = false)
{
    Plan pl;
    gsa_status st = make_plan(p, &pl);
    if (st != GSA_OK) return st;
    if (readout < GSA_READOUT_SOFTMAX || readout > GSA_READOUT_RELU2) return GSA_ERR_SHAPE;
    if (!(gate_tau >= 0.f)) return GSA_ERR_SHAPE;
    if (feature_map != GSA_FEATURE_NONE && feature_map != GSA_FEATURE_SWISH) return GSA_ERR_SHAPE;
    if (pl.tokens == 0) return GSA_OK;
    if (!q || !k || !v || !g) return GSA_ERR_NULL;
    if (with_act ? (!act && !o) : !o) return GSA_ERR_NULL;   // the epilogue form may leave o out, not both
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(o) || !aligned16(K0) ||
        !aligned16(V0) || !aligned16(z_saved) || !aligned16(KT) || !aligned16(VT) || !aligned16(s) ||
        !aligned16(act) || !aligned16(ssq))
        return GSA_ERR_SHAPE;
    st = check_workspace(workspace, workspace_bytes, pl.total_fwd);
    if (st != GSA_OK) return st;
    {
        const size_t esz = pl.dtype == GSA_BF16 ? 2 : 4, th = (size_t)pl.tokens * pl.H, M = pl.m;
        const size_t nk = th * pl.d_k * esz, nv = th * pl.d_v * esz, nm = th * M * sizeof(float);
        const size_t sk = (size_t)pl.n_seqs * pl.H * M * pl.d_k * sizeof(float);
        const size_t sv = (size_t)pl.n_seqs * pl.H * M * pl.d_v * sizeof(float);
        const int slice = gsa::apply_slice_cols(pl.dtype);
        const size_t nq = th * (size_t)((pl.d_v + slice - 1) / slice) * sizeof(float);
        const Span spans[] = {{o, nv}, {z_saved, nm}, {KT, sk}, {VT, sv}, {workspace, pl.total_fwd}, {act, nv}, {ssq, nq},
                              {q, nk}, {k, nk}, {v, nv}, {g, nm}, {s, nm}, {K0, sk}, {V0, sv}};
        if (outputs_overlap(spans, 7, (int)(sizeof(spans) / sizeof(spans[0])))) return GSA_ERR_SHAPE;
    }
    pl.act_out = act;
    pl.act_ssq = ssq;
    pl.s_in = s;
    pl.readout = readout;
    pl.gate_tau = gate_tau;
    pl.phi = feature_map;
    const Work w = make_work(pl, workspace);
    const hipError_t e = gsa::launch_fwd(pl, w, q, k, v, g, K0, V0, o, z_saved, KT, VT,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : GSA_ERR_HIP;
}

gsa_status bwd_any(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map, const void *q,
                   const void *k, const void *v, const float *g, const float *s, const float *K0, const float *V0,
                   const float *z_saved, const void *dO, const float *dKT, const float *dVT, void *dq, void *dk,
                   void *dv, float *dg, float *ds, float *dK0, float *dV0, void *workspace, size_t workspace_bytes,
                   void *stream)
{
    Plan pl;
    gsa_status st = make_plan(p, &pl);
    if (st != GSA_OK) return st;
    if (readout < GSA_READOUT_SOFTMAX || readout > GSA_READOUT_RELU2) return GSA_ERR_SHAPE;
    if (!(gate_tau >= 0.f)) return GSA_ERR_SHAPE;
    if (feature_map != GSA_FEATURE_NONE && feature_map != GSA_FEATURE_SWISH) return GSA_ERR_SHAPE;
    if (pl.tokens == 0) return GSA_OK;
    if (!q || !k || !v || !g || !z_saved || !dO || !dq || !dk || !dv || !dg) return GSA_ERR_NULL;
    if (s && !ds) return GSA_ERR_NULL;
    const void *ptrs[] = {q, k, v, g, s, K0, V0, z_saved, dO, dKT, dVT, dq, dk, dv, dg, ds, dK0, dV0};
    for (const void *ptr : ptrs)
        if (!aligned16(ptr)) return GSA_ERR_SHAPE;
    st = check_workspace(workspace, workspace_bytes, pl.total_bwd);
    if (st != GSA_OK) return st;
    {
        const size_t esz = pl.dtype == GSA_BF16 ? 2 : 4, th = (size_t)pl.tokens * pl.H, M = pl.m;
        const size_t nk = th * pl.d_k * esz, nv = th * pl.d_v * esz, nm = th * M * sizeof(float);
        const size_t sk = (size_t)pl.n_seqs * pl.H * M * pl.d_k * sizeof(float);
        const size_t sv = (size_t)pl.n_seqs * pl.H * M * pl.d_v * sizeof(float);
        const Span spans[] = {{dq, nk}, {dk, nk}, {dv, nv}, {dg, nm}, {s ? ds : nullptr, nm}, {dK0, sk}, {dV0, sv},
                              {workspace, pl.total_bwd},
                              {q, nk}, {k, nk}, {v, nv}, {g, nm}, {s, nm}, {K0, sk}, {V0, sv}, {z_saved, nm},
                              {dO, nv}, {dKT, sk}, {dVT, sv}};
        if (outputs_overlap(spans, 8, (int)(sizeof(spans) / sizeof(spans[0])))) return GSA_ERR_SHAPE;
    }
    pl.s_in = s;
    pl.ds_out = s ? ds : nullptr;
    pl.readout = readout;
    pl.gate_tau = gate_tau;
    pl.phi = feature_map;
    const Work w = make_work(pl, workspace);
    const hipError_t e = gsa::launch_bwd(pl, w, q, k, v, g, K0, V0, z_saved, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : GSA_ERR_HIP;
}
}  // namespace

gsa_status gsa_fwd(const gsa_problem *p, const void *q, const void *k, const void *v, const float *g,
                   const float *K0, const float *V0, void *o, float *z_saved, float *KT, float *VT,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    return fwd_any(p, GSA_READOUT_SOFTMAX, 0.f, GSA_FEATURE_NONE, q, k, v, g, nullptr, K0, V0, o, z_saved, KT, VT,
                   workspace, workspace_bytes, stream);
}

gsa_status gsa_fwd_ex(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map, const void *q,
                      const void *k, const void *v, const float *g, const float *s, const float *K0,
                      const float *V0, void *o, float *z_saved, float *KT, float *VT, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    return fwd_any(p, readout, gate_tau, feature_map, q, k, v, g, s, K0, V0, o, z_saved, KT, VT, workspace,
                   workspace_bytes, stream);
}

gsa_status gsa_fwd_act(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map, const void *q,
                       const void *k, const void *v, const float *g, const float *s, const float *K0,
                       const float *V0, void *o, void *act, float *act_ssq, float *z_saved, float *KT, float *VT,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    return fwd_any(p, readout, gate_tau, feature_map, q, k, v, g, s, K0, V0, o, z_saved, KT, VT, workspace,
                   workspace_bytes, stream, act, act_ssq, true);
}

int32_t gsa_act_slice_cols(int32_t dtype) { return (dtype == GSA_F32 || dtype == GSA_BF16) ? gsa::apply_slice_cols(dtype) : 0; }

gsa_status gsa_bwd(const gsa_problem *p, const void *q, const void *k, const void *v, const float *g,
                   const float *K0, const float *V0, const float *z_saved, const void *dO, const float *dKT,
                   const float *dVT, void *dq, void *dk, void *dv, float *dg, float *dK0, float *dV0,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    return bwd_any(p, GSA_READOUT_SOFTMAX, 0.f, GSA_FEATURE_NONE, q, k, v, g, nullptr, K0, V0, z_saved, dO, dKT, dVT,
                   dq, dk, dv, dg, nullptr, dK0, dV0, workspace, workspace_bytes, stream);
}

gsa_status gsa_bwd_ex(const gsa_problem *p, int32_t readout, float gate_tau, int32_t feature_map, const void *q,
                      const void *k, const void *v, const float *g, const float *s, const float *K0,
                      const float *V0, const float *z_saved, const void *dO, const float *dKT, const float *dVT,
                      void *dq, void *dk, void *dv, float *dg, float *ds, float *dK0, float *dV0, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    return bwd_any(p, readout, gate_tau, feature_map, q, k, v, g, s, K0, V0, z_saved, dO, dKT, dVT, dq, dk, dv, dg,
                   ds, dK0, dV0, workspace, workspace_bytes, stream);
}

gsa_status gsa_decode_step(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, int32_t dtype, float scale,
                           const void *q, const void *k, const void *v, const float *g, float *K_state,
                           float *V_state, void *o, void *stream)
{
    return decode_any(B, H, d_k, d_v, m, dtype, scale, q, k, v, g, K_state, V_state, o, false, nullptr, 0, stream);
}

gsa_status gsa_decode_workspace_bytes(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, size_t *bytes)
{
    if (!bytes) return GSA_ERR_NULL;
    const gsa_status st = decode_checks(B, H, d_k, d_v, m, GSA_F32, 1.0f);
    if (st != GSA_OK) return st;
    *bytes = align_up(gsa::decode_scratch_floats(B * H, d_v, m) * sizeof(float));
    return GSA_OK;
}

gsa_status gsa_decode_step_ex(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, int32_t dtype, float scale,
                              int32_t readout, float gate_tau, int32_t feature_map, const void *q, const void *k,
                              const void *v, const float *g, const float *s, float *K_state, float *V_state,
                              void *o, void *workspace, size_t workspace_bytes, void *stream)
{
    return decode_any(B, H, d_k, d_v, m, dtype, scale, q, k, v, g, K_state, V_state, o, workspace != nullptr,
                      workspace, workspace_bytes, stream, s, readout, gate_tau, feature_map);
}

gsa_status gsa_decode_step_static(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, int32_t dtype,
                                  float scale, const void *q, const void *k, const void *v, const float *g,
                                  float *K_state, float *V_state, void *o, void *stream)
{
    const gsa_status st = decode_checks(B, H, d_k, d_v, m, dtype, scale);
    if (st != GSA_OK) return st;
    if (B == 0) return GSA_OK;
    const size_t need = gsa::decode_scratch_floats(B * H, d_v, m);
    if (need > gsa::decode_static_scratch_floats()) return GSA_ERR_WORKSPACE;   // beyond the built-in scratch
    float *scratch = nullptr;
    if (need && gsa::decode_static_scratch(&scratch) != hipSuccess) return GSA_ERR_HIP;
    return decode_any(B, H, d_k, d_v, m, dtype, scale, q, k, v, g, K_state, V_state, o, need != 0, scratch,
                      need * sizeof(float), stream);
}

gsa_status gsa_decode_step_ws(int32_t B, int32_t H, int32_t d_k, int32_t d_v, int32_t m, int32_t dtype, float scale,
                              const void *q, const void *k, const void *v, const float *g, float *K_state,
                              float *V_state, void *o, void *workspace, size_t workspace_bytes, void *stream)
{
    return decode_any(B, H, d_k, d_v, m, dtype, scale, q, k, v, g, K_state, V_state, o, true, workspace,
                      workspace_bytes, stream);
}

}  // extern "C"
