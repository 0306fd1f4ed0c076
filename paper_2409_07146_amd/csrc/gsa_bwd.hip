// Backward pass of Gated Slot Attention, chunkwise (paper: Algorithm 1 backward;
// gradients derived from Eq. (gsa), not transcribed from the listing).
//
// Per sequence and head, with S = [Kt | Vt] the joint slot memory, G the chunk-local
// cumulative log gate, s = 1 - exp(g), p = softmax(z):
//
//   dp_t[i] = <Vt_t[i], dO_t>                       (same gated contraction as pass 1)
//   dz_t    = p_t * (dp_t - <p_t, dp_t>)
//   E       = gradient of the loss w.r.t. the memory at the END of a chunk, through later
//             chunks only; carried backwards by  E' = Diag(exp G_C) E + (w * exp G)^T x
//             with (w, x) = (scale*dz, q) on the key columns and (p, dO) on the value columns
//   Bm[t,r] = sum_i dz_t[i] s_r[i] exp(G_t[i]-G_r[i]),  A2[t,r] likewise with p_t   (r <= t)
//   dq = scale * ((dz*exp G) Kt_start + Bm K)        (the scale is folded into the small matrices)
//   dk = scale * Bm^T Q + (s*exp(G_C-G)) E_k          dv = A2^T dO + (s*exp(G_C-G)) E_v
//   ds_r[i] = exp(G_C-G_r)[i] <E[i], [k_r|v_r]> + sum_{t>=r} exp(G_t-G_r)[i] (scale dz_t[i] <q_t,k_r> + p_t[i] <dO_t,v_r>)
//   dGam_t = z_t dz_t + p_t dp_t - s_t ds_t          (gradient w.r.t. the cumulative log gate)
//   dg_j   = sum_{t>=j, same chunk} dGam_t + <E[i], S_end[i]> - exp(g_j) ds_j
//
// The last line replaces the sequence-long reversed cumulative sum of Algorithm 1 by a
// chunk-local one: the sum of dGam over all later chunks equals the row-wise inner product
// of the chunk-end memory with its gradient, which both scans already hold.  That keeps
// rounding errors from accumulating along the sequence (measured: summing the chunk totals
// instead costs about a third more error on dg with bf16 memories).
//
// Kernels of one backward call: gate + forward scan (gsa_scan.hip; recompute the chunk-start
// memories, since nothing but z was saved by the forward), chunk_dz (chunk-parallel: dp, dz,
// weights of the reverse scan), reverse scan (gsa_scan.hip: E), chunk_intra (chunk-parallel:
// Bm, A2, ds, dg and the small operand matrices), apply (gsa_apply.hip: dq, dk, dv).
#include "gsa_chunk.h"
#include "gsa_launch.h"

namespace gsa {

// ---------------------------------------------------------------------------------------
// dz kernel
// ---------------------------------------------------------------------------------------
template <typename T, int M> struct DzLds {
    static constexpr int C = Geo<T>::C;
    static constexpr int PAD = Atom<T>::kPad;
    static constexpr int ldg = M + 4, lda = C + PAD;
    static constexpr size_t oG = 0;
    static constexpr size_t oS = oG + sizeof(float) * C * ldg;
    static constexpr size_t oA = oS + sizeof(float) * C * ldg;
    static constexpr size_t oTot = oA;   // gate_prep's scratch, dead before As is written
    static constexpr size_t szA = sizeof(T) * C * lda > sizeof(float) * Geo<T>::NT ? sizeof(T) * C * lda
                                                                                  : sizeof(float) * Geo<T>::NT;
    static constexpr size_t oVt = oA + szA;                           // Vt [M][lda]
    static constexpr size_t oRb = oVt + sizeof(T) * M * lda;          // Rb [C/16][M] fp32
    static constexpr size_t end = oRb + sizeof(float) * (C / 16) * M;
    static constexpr int kRpr = 2;                 // row blocks per round of the reduction
    static constexpr size_t szRed = sizeof(f32x4) * kWave * (C / 16) *
                                    reduce_fragments<C / 16, C / 16 + M / 16, C / 16, kRpr>();   // from offset 0: dead before the tiles are written
    static constexpr size_t bytes = end > szRed ? end : szRed;
};

// GEN: the general form (write intensities from `sin` when it is not NULL; opts: read-out in the low
// byte).  PHI (with GEN): the feature map on v.
template <typename T, int M, bool GEN, bool PHI>
__global__ __launch_bounds__(Geo<T>::NT, (M > 64 ? 1 : 2)) void chunk_dz_kernel(ChunkMap cm, int H, int d_v, float scale,
                                                              const T *__restrict__ v, const T *__restrict__ dO,
                                                              const float *__restrict__ g, const float *__restrict__ z,
                                                              const T *__restrict__ S, StateLayout lay,
                                                              float *__restrict__ dz, float *__restrict__ dgf,
                                                              T *__restrict__ Wr, T *__restrict__ tAvT,
                                                              const float *__restrict__ sin, int opts,
                                                              float gate_tau)
{
    using L = DzLds<T, M>;
    const int readout = opts & kReadoutMask;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT;
    constexpr int MI = M / 16;
    extern __shared__ __align__(16) unsigned char smem[];
    float *Gs = reinterpret_cast<float *>(smem + L::oG);
    float *Ss = reinterpret_cast<float *>(smem + L::oS);
    float *tot = reinterpret_cast<float *>(smem + L::oTot);
    T *As = reinterpret_cast<T *>(smem + L::oA);

    ChunkInfo ci;
    int cid, h;
    chunk_order(cm, H, true, cid, h);   // the forward scan has just written the last chunks
    if (!chunk_lookup(cm, cid, ci)) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4;
    const size_t tokh = (size_t)ci.tok0 * H + h;
    const size_t ch = (size_t)cid * H + h;
    const T *Vn = S + ch * lay.stride + lay.oV;      // value memory at chunk start (tiled)
    const int rowb = 16 * w;

    float dp[MI][4];
    bool unsafe;
    // dO is hinted; v and the chunk-start value memory are read again by chunk_intra and stay cached
    gated_scores<T, M, C, GEN, L::kRpr, kHintX>(dp, unsafe, Gs, Ss, L::ldg, tot, g + tokh * M, (size_t)H * M, As, L::lda,
                               reinterpret_cast<T *>(smem + L::oVt), L::lda,
                               reinterpret_cast<float *>(smem + L::oRb), reinterpret_cast<f32x4 *>(smem), dO + tokh * d_v,
                               v + tokh * d_v, (size_t)H * d_v, d_v, Vn, ci.len, tid,
                               (GEN && sin) ? sin + tokh * M : nullptr, gate_tau,
                               PHI ? kHintY : 0);
    float zv[MI][4], p[MI][4], rmax[4], rsum[4], pdp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) rmax[j] = -INFINITY;
#pragma unroll
    for (int ni = 0; ni < MI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            zv[ni][j] = z[(tokh + (size_t)min(t, ci.len - 1) * H) * M + ni * 16 + r];   // clamped, never stored past len
            rmax[j] = fmaxf(rmax[j], zv[ni][j]);
        }
    // slope[ni][j]*(dp - pdp[j]) is dz: p and <p,dp> for the softmax, f'(z) and 0 for an element-wise read-out
    float slope[MI][4];
    if (!GEN || readout == kReadSoftmax) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { rmax[j] = row16_max(rmax[j]); rsum[j] = 0.f; pdp[j] = 0.f; }
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) { p[ni][j] = __expf(zv[ni][j] - rmax[j]); rsum[j] += p[ni][j]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) rsum[j] = 1.f / row16_sum(rsum[j]);
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) { p[ni][j] *= rsum[j]; pdp[j] += p[ni][j] * dp[ni][j]; slope[ni][j] = p[ni][j]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) pdp[j] = row16_sum(pdp[j]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) pdp[j] = 0.f;
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                p[ni][j] = readout_value(readout, zv[ni][j]);
                slope[ni][j] = readout_slope(readout, zv[ni][j]);
            }
    }
    // dz, dgf for the intra kernel; gate-weighted transposes (scale*dz*exp G, p*exp G) for the reverse scan
    T *Wk = Wr + ch * 2 * M * C, *Wv = Wk + M * C;
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) {
        const int i = ni * 16 + r;
        T wk[4], wv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            const bool live = t < ci.len;
            const float dzv = live ? slope[ni][j] * (dp[ni][j] - pdp[j]) : 0.f;
            const float eg = __expf(Gs[t * L::ldg + i]);
            wk[j] = from_f32<T>(scale * dzv * eg);
            wv[j] = from_f32<T>(live ? p[ni][j] * eg : 0.f);
            if (live) {
                const size_t off = (tokh + (size_t)t * H) * M + i;
                dz[off] = dzv;
                dgf[off] = zv[ni][j] * dzv + p[ni][j] * dp[ni][j];
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            Wk[i * C + rowb + g4 + j] = wk[j];
            Wv[i * C + rowb + g4 + j] = wv[j];
        }
    }
    // the causally masked (dO_t . v_r), transposed, for the intra kernel's ds contraction
    T *dAv = tAvT + ch * C * C;
    for (int idx = tid; idx < C * C / 8; idx += NT) {
        const int rr = idx / (C / 8), t8 = (idx - rr * (C / 8)) * 8;
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = to_f32(As[(t8 + e) * L::lda + rr]);
        store8<T>(dAv + rr * C + t8, x);
    }
}

// ---------------------------------------------------------------------------------------
// Intra-chunk gradient kernel.
// ---------------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ float frag_dot(const typename Atom<T>::Frag &a,
                                                                const typename Atom<T>::Frag &b)
{
    float d = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) d += to_f32(a[e]) * to_f32(b[e]);
    return d;
}

template <typename T, int M> struct IntraLds {
    static constexpr int C = Geo<T>::C;
    static constexpr int PAD = Atom<T>::kPad;
    static constexpr int KM = (M < 32) ? 32 : M;
    static constexpr int ldg = M + 4, lda = C + PAD;
    static constexpr size_t oG = 0;
    static constexpr size_t oS = oG + sizeof(float) * C * ldg;
    static constexpr size_t oPf = oS + sizeof(float) * C * ldg;
    static constexpr size_t oDf = oPf + sizeof(float) * C * ldg;
    static constexpr size_t oAT = oDf + sizeof(float) * C * ldg;
    static constexpr size_t oTot = oAT;   // gate_prep's and the suffix sum's scratch (ATs is dead by then)
    static constexpr size_t szAT = sizeof(T) * C * lda > sizeof(float) * Geo<T>::NT ? sizeof(T) * C * lda
                                                                                   : sizeof(float) * Geo<T>::NT;
    static constexpr int kRpr = 2;        // row blocks per round of the reduction
    static constexpr size_t szRed = sizeof(f32x4) * kWave * (C / 16) *
                                    reduce_fragments<C / 16, C / 16 + M / 16, C / 16, kRpr>();   // from offset 0: every tile is written after it
    static constexpr size_t oCarry = (oAT + szAT > szRed) ? oAT + szAT : szRed;
    static constexpr size_t bytes = oCarry + sizeof(float) * (C / 16) * M;   // per-wave partial carries
};

template <typename T> struct IntraArgs {
    const T *q, *k, *v;
    const float *g, *z, *dz, *dgf;
    const T *S, *SF, *E;
    StateLayout lay;
    const T *tAvT;
    float *dg;
    T *tB, *tBT, *tA2T, *tDZe, *tSbe;
    const float *sin;   // general form: write intensities, or NULL
    float *ds;          // general form: their gradient (with sin)
    int readout;
    float gate_tau;     // general form: > 0 when g holds gate logits
};

template <typename T, int M, bool GEN, bool PHI>
__global__ __launch_bounds__(Geo<T>::NT, (M > 64 ? 1 : 2)) void chunk_intra_kernel(ChunkMap cm, int H, int d_k, int d_v, float scale,
                                                                 IntraArgs<T> a)
{
    using L = IntraLds<T, M>;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT, NW = Geo<T>::NW;
    constexpr int MI = M / 16, CI = C / 16, KM = L::KM;
    constexpr int NB = CI + MI;
    extern __shared__ __align__(16) unsigned char smem[];
    float *Gs = reinterpret_cast<float *>(smem + L::oG);
    float *Ss = reinterpret_cast<float *>(smem + L::oS);
    float *Pf = reinterpret_cast<float *>(smem + L::oPf);    // p, later exp(g)*ds
    float *Df = reinterpret_cast<float *>(smem + L::oDf);    // dz, later dGam
    float *tot = reinterpret_cast<float *>(smem + L::oTot);
    float *carry = reinterpret_cast<float *>(smem + L::oCarry);   // [NW][M]
    T *ATs = reinterpret_cast<T *>(smem + L::oAT);           // [r][t] (q_t . k_r) for t >= r; later Bm [t][r]

    ChunkInfo ci;
    int cid, h;
    chunk_order(cm, H, false, cid, h);   // the reverse scan has just written the first chunks
    if (!chunk_lookup(cm, cid, ci)) return;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g4 = (lane >> 4) * 4, g8 = (lane >> 4) * 8;
    const size_t tokh = (size_t)ci.tok0 * H + h;
    const size_t ch = (size_t)cid * H + h;
    const T *EK = a.E + ch * a.lay.stride + a.lay.oK;        // memory gradient at chunk end
    const T *EV = a.E + ch * a.lay.stride + a.lay.oV;
    int chunk0, nch, stok0, sntok;
    seq_lookup(cm, ci.seq, chunk0, nch, stok0, sntok);
    const T *SendK, *SendV;                                  // memory at chunk end
    if (ci.idx + 1 < nch) {
        const T *rec = a.S + (ch + H) * a.lay.stride;        // = start of the next chunk
        SendK = rec + a.lay.oK;
        SendV = rec + a.lay.oV;
    } else {
        const T *rec = a.SF + ((size_t)ci.seq * H + h) * a.lay.stride;
        SendK = rec + a.lay.oK;
        SendV = rec + a.lay.oV;
    }
    const T *AvT = a.tAvT + ch * C * C;
    const int rowb = 16 * w;

    // ---- phase 1: contractions over the head dimension, operands straight from global memory
    //   A[t][r] = q_t . k_r (r <= t),  X[r][i] = <E[i], [k_r | v_r]>,  carry[i] = <E[i], S_end[i]>
    // Split over the waves in steps of 64 columns (see gated_scores): every wave covers all row
    // blocks over its share of the columns, the partial sums meet in LDS.
    f32x4 accA[CI], accX[MI];
    GatePrep<M, NT, C, GEN> gp;
    SoftmaxRows<M, C> sr;
    const bool given = GEN && a.sin != nullptr;   // write intensities are an input of their own
    {
        typedef typename Atom<T>::Frag Frag;
        f32x4 acc[NW][NB];   // [row block][k blocks (causal) | slot blocks]
#pragma unroll
        for (int rb = 0; rb < NW; ++rb)
#pragma unroll
            for (int cb = 0; cb < NB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
        float cpart[MI];     // this lane's share of the carry of slot 16*ni + lane%16
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) cpart[ni] = 0.f;
        // Token rows past the end of a ragged chunk are read as copies of its last row (finite; they
        // only feed rows that are never stored or that meet zero weights).
        uint32_t tk[CI], tv[CI], ek[MI], ev[MI];
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) {
            const uint32_t row = (uint32_t)min(ni * 16 + r, ci.len - 1) * (uint32_t)H;
            tk[ni] = row * (uint32_t)d_k + g8;
            tv[ni] = row * (uint32_t)d_v + g8;
        }
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) {
            ek[ni] = ev[ni] = (uint32_t)(ni * 16 + r) * kSnapTile + g8;   // snapshot parts are tiled
        }
        const T *qb = a.q + tokh * d_k, *kb = a.k + tokh * d_k, *vb = a.v + tokh * d_v;
        // key half: A = Q K^T, X += K E_k^T
        // (two passes over k, each in 64-column steps like the value half: together their operand
        // fragments would not fit the registers; the second read of k is served by the caches)
        // Non-temporal loads for what is read here for the last time in this call (q, v, the chunk-end
        // memories); k comes twice and the apply kernel right after reads E again, so those stay cached.
        for (int kk = 64 * w; kk < d_k; kk += 64 * NW) {
            Frag fq[2][CI], fk[2][CI];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < CI; ++ni) fq[hh][ni] = Atom<T>::load_nt(qb + tk[ni] + kk + 32 * hh);
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < CI; ++ni) fk[hh][ni] = Atom<T>::load(kb + tk[ni] + kk + 32 * hh);
            __builtin_amdgcn_sched_barrier(0);   // all loads of the step before its multiplies (see gated_scores)
            if (PHI) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                    for (int ni = 0; ni < CI; ++ni) { swish_frag<T>(fq[hh][ni]); swish_frag<T>(fk[hh][ni]); }
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int rb = 0; rb < NW; ++rb)
#pragma unroll
                    for (int cb = 0; cb <= rb; ++cb) Atom<T>::mma(acc[rb][cb], fq[hh][rb], fk[hh][cb]);
        }
        for (int kk = 64 * w; kk < d_k; kk += 64 * NW) {
            Frag fk[2][CI], fe[2][MI], fs[2][MI];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < CI; ++ni) fk[hh][ni] = Atom<T>::load(kb + tk[ni] + kk + 32 * hh);
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < MI; ++ni) fe[hh][ni] = Atom<T>::load(EK + ek[ni] + snap_col<M>(kk + 32 * hh));
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < MI; ++ni) fs[hh][ni] = Atom<T>::load_nt(SendK + ek[ni] + snap_col<M>(kk + 32 * hh));
            __builtin_amdgcn_sched_barrier(0);
            if (PHI) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                    for (int ni = 0; ni < CI; ++ni) swish_frag<T>(fk[hh][ni]);
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int rb = 0; rb < NW; ++rb)
#pragma unroll
                    for (int ni = 0; ni < MI; ++ni) Atom<T>::mma(acc[rb][CI + ni], fk[hh][rb], fe[hh][ni]);
#pragma unroll
                for (int ni = 0; ni < MI; ++ni) cpart[ni] += frag_dot<T>(fe[hh][ni], fs[hh][ni]);
            }
        }
        // value half: X += V E_v^T
        // (64 columns per wave and step here, as in gated_scores: the registers allow it in this half)
        for (int kk = 64 * w; kk < d_v; kk += 64 * NW) {
            Frag fv[2][CI], fe[2][MI], fs[2][MI];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < CI; ++ni) fv[hh][ni] = Atom<T>::load_nt(vb + tv[ni] + kk + 32 * hh);
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < MI; ++ni) fe[hh][ni] = Atom<T>::load(EV + ev[ni] + snap_col<M>(kk + 32 * hh));
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int ni = 0; ni < MI; ++ni) fs[hh][ni] = Atom<T>::load_nt(SendV + ev[ni] + snap_col<M>(kk + 32 * hh));
            __builtin_amdgcn_sched_barrier(0);
            if (PHI) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                    for (int ni = 0; ni < CI; ++ni) swish_frag<T>(fv[hh][ni]);
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int rb = 0; rb < NW; ++rb)
#pragma unroll
                    for (int ni = 0; ni < MI; ++ni) Atom<T>::mma(acc[rb][CI + ni], fv[hh][rb], fe[hh][ni]);
#pragma unroll
                for (int ni = 0; ni < MI; ++ni) cpart[ni] += frag_dot<T>(fe[hh][ni], fs[hh][ni]);
            }
        }
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) {
            float x = cpart[ni];
            x += __shfl_xor(x, 16, 64);
            x += __shfl_xor(x, 32, 64);
            if (lane < 16) carry[w * M + ni * 16 + lane] = x;   // read after the barriers of the reduction
        }
        // the loads of everything phase 2 needs from global memory land during the reduction
        gp.load(a.g + tokh * M, (size_t)H * M, ci.len, tid, given ? a.sin + tokh * M : nullptr, GEN ? a.gate_tau : 0.f);
        sr.load(a.z + tokh * M, a.dz + tokh * M, (size_t)H * M, ci.len, tid);
        f32x4 own[NB];
        reduce_row_blocks<NW, NB, CI, L::kRpr>(own, acc, reinterpret_cast<f32x4 *>(smem), lane, w);
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) accA[ni] = own[ni];
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) accX[ni] = own[CI + ni];
    }
    // gate tiles; p and dz tiles (they overwrite the reduction buffer, which every wave has left by now)
    gp.finish(Gs, Ss, L::ldg, tot, ci.len, tid);
    if (!GEN || a.readout == kReadSoftmax) sr.finish(Pf, Df, L::ldg, ci.len, tid);
    else sr.finish_elementwise(a.readout, Pf, Df, L::ldg, ci.len, tid);
    // ---- phase 2a: transposed masked A into LDS; the slot-side operand tiles of the apply kernel
#pragma unroll
    for (int ni = 0; ni < CI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j, rr = ni * 16 + r;
            ATs[rr * L::lda + t] = from_f32<T>((ni <= w && rr <= t) ? accA[ni][j] : 0.f);
        }
    __syncthreads();   // Pf, Df, ATs visible to every wave
    {
        T *dD = a.tDZe + ch * C * KM, *dS = a.tSbe + ch * C * KM;
        for (int idx = tid; idx < C * KM / 8; idx += NT) {
            const int t = idx / (KM / 8), i8 = (idx - t * (KM / 8)) * 8;
            float x[8], y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int i = i8 + e;
                x[e] = y[e] = 0.f;
                if (i < M) {
                    const float G = Gs[t * L::ldg + i];
                    x[e] = scale * Df[t * L::ldg + i] * __expf(G);
                    y[e] = Ss[t * L::ldg + i] * __expf(Gs[(C - 1) * L::ldg + i] - G);
                }
            }
            store8<T>(dD + t * KM + i8, x);
            store8<T>(dS + t * KM + i8, y);
        }
    }
    const bool unsafe = block_unsafe<M>(Gs, L::ldg, rowb, lane);
    // ---- phase 2b: write-intensity gradient ds for rows r of block w, then dGam and exp(g)*ds
    float dGam[MI][4], ads[MI][4];
    {
        f32x4 accW[MI];
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) accW[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int tstart = unsafe ? rowb + 16 : rowb;
        float gend[MI];
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) gend[ni] = Gs[(rowb + 15) * L::ldg + ni * 16 + r];
        // LDS reads are unconditional (every token of the tile exists); masking is a register select
        for (int k0 = (tstart & ~31); k0 < C; k0 += 32) {
            const typename Atom<T>::Frag aA = Atom<T>::load(ATs + (rowb + r) * L::lda + k0 + g8);
            const typename Atom<T>::Frag aAv = Atom<T>::load(AvT + (rowb + r) * C + k0 + g8);
#pragma unroll
            for (int ni = 0; ni < MI; ++ni) {
                const int i = ni * 16 + r;
                float gv[8], dv[8], pv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int t = k0 + g8 + e;
                    gv[e] = Gs[t * L::ldg + i];
                    dv[e] = Df[t * L::ldg + i];
                    pv[e] = Pf[t * L::ldg + i];
                }
                typename Atom<T>::Frag bdz, bp;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool on = k0 + g8 + e >= tstart;
                    const float f = __expf(fminf(gv[e] - gend[ni], kExpClamp));
                    bdz[e] = from_f32<T>(on ? scale * dv[e] * f : 0.f);
                    bp[e] = from_f32<T>(on ? pv[e] * f : 0.f);
                }
                Atom<T>::mma(accW[ni], aA, bdz);
                Atom<T>::mma(accW[ni], aAv, bp);
            }
        }
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) {
            const int i = ni * 16 + r;
            const float gend = Gs[(rowb + 15) * L::ldg + i], GC = Gs[(C - 1) * L::ldg + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int rr = rowb + g4 + j;
                const float Gr = Gs[rr * L::ldg + i];
                float ds = __expf(GC - Gr) * accX[ni][j] + __expf(gend - Gr) * accW[ni][j];
                if (unsafe) {
                    float sum = 0.f;
                    for (int t = rr; t < rowb + 16; ++t)
                        sum += (to_f32(ATs[rr * L::lda + t]) * scale * Df[t * L::ldg + i] +
                                to_f32(AvT[rr * C + t]) * Pf[t * L::ldg + i]) *
                               __expf(Gs[t * L::ldg + i] - Gr);
                    ds += sum;
                }
                const float sv = Ss[rr * L::ldg + i];
                const float fl = a.dgf[(tokh + (size_t)min(rr, ci.len - 1) * H) * M + i];
                const float f = (rr < ci.len) ? fl : 0.f;
                dGam[ni][j] = f - sv * ds;
                ads[ni][j] = given ? ds : (1.f - sv) * ds;   // tied: d(1 - e^g)/dg = -e^g = -(1 - s)
            }
        }
    }
    // ---- phase 2c: Bm and A2 for row block w
    f32x4 accB[CI], acc2[CI];
    {
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) { accB[ni] = f32x4{0.f, 0.f, 0.f, 0.f}; acc2[ni] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        for (int k0 = 0; k0 < KM; k0 += 32) {
            const SlotSpan<M, KM> sp(k0 + g8);
            float gref[8];
            gate_ref8(gref, Gs, L::ldg, rowb, sp.i0);
            typename Atom<T>::Frag adz, ap;
            {
                float gv[8], dv[8], pv[8];
                lds_row8(gv, Gs + (rowb + r) * L::ldg + sp.i0);
                lds_row8(dv, Df + (rowb + r) * L::ldg + sp.i0);
                lds_row8(pv, Pf + (rowb + r) * L::ldg + sp.i0);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float f = __expf(gv[e] - gref[e]);
                    adz[e] = from_f32<T>(sp.live ? dv[e] * f : 0.f);
                    ap[e] = from_f32<T>(sp.live ? pv[e] * f : 0.f);
                }
            }
#pragma unroll
            for (int ni = 0; ni < CI; ++ni) {
                if (ni > w || (unsafe && ni == w)) continue;   // wave-uniform
                const typename Atom<T>::Frag b = write_frag<T>(Gs, Ss, L::ldg, ni * 16 + r, sp.i0, sp.live, gref);
                Atom<T>::mma(accB[ni], adz, b);
                Atom<T>::mma(acc2[ni], ap, b);
            }
        }
        if (unsafe) {
            const f32x4 eb = pair_weights_exact<M, float>(Df, L::ldg, Gs, Ss, L::ldg, lane, rowb);
            const f32x4 e2 = pair_weights_exact<M, float>(Pf, L::ldg, Gs, Ss, L::ldg, lane, rowb);
#pragma unroll
            for (int ni = 0; ni < CI; ++ni)
                if (ni == w) { accB[ni] = eb; acc2[ni] = e2; }
        }
    }
    __syncthreads();   // every wave is done reading p, dz and the transposed A
    {
        T *dBT = a.tBT + ch * C * C, *dA2T = a.tA2T + ch * C * C;
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) {
            const int rr = ni * 16 + r;
            float bv[4], av[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int t = rowb + g4 + j;
                const bool keep = (ni <= w) && (rr <= t);
                bv[j] = keep ? scale * accB[ni][j] : 0.f;
                av[j] = keep ? acc2[ni][j] : 0.f;
                ATs[t * L::lda + rr] = from_f32<T>(bv[j]);     // Bm in natural orientation, staged for a row-wise copy
            }
            store4(dBT + rr * C + rowb + g4, bv[0], bv[1], bv[2], bv[3]);
            store4(dA2T + rr * C + rowb + g4, av[0], av[1], av[2], av[3]);
        }
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int rr = rowb + g4 + j, i = ni * 16 + r;
                Df[rr * L::ldg + i] = dGam[ni][j];
                Pf[rr * L::ldg + i] = ads[ni][j];
            }
    }
    __syncthreads();
    {
        T *dB = a.tB + ch * C * C;
        for (int idx = tid; idx < C * C / 8; idx += NT) {
            const int t = idx / (C / 8), c8 = (idx - t * (C / 8)) * 8;
            Raw8<T> x;
            x.load(ATs + t * L::lda + c8);
            x.store(dB + t * C + c8);
        }
    }
    __syncthreads();   // ATs is about to be reused as the suffix sum's scratch
    // ---- phase 2d: dg = (suffix sum of dGam inside the chunk) + carry - exp(g) ds
    {
        constexpr int P = NT / M, TP = C / P;
        const int i = tid % M, part = tid / M;
        float run = 0.f;
        for (int tt = TP - 1; tt >= 0; --tt) {
            const int t = part * TP + tt;
            run += Df[t * L::ldg + i];
            Df[t * L::ldg + i] = run;
        }
        tot[part * M + i] = run;
        __syncthreads();
        float off = 0.f;
#pragma unroll
        for (int u = 0; u < NW; ++u) off += carry[u * M + i];
        for (int pp = part + 1; pp < P; ++pp) off += tot[pp * M + i];
        for (int tt = 0; tt < TP; ++tt) {
            const int t = part * TP + tt;
            if (t < ci.len) {
                const size_t o = (tokh + (size_t)t * H) * M + i;
                // gate logits in g: the gradient goes on to the logit, d logsigmoid(u)/tau / du
                const float chain = (GEN && a.gate_tau > 0.f) ? log_gate_slope(a.g[o], a.gate_tau) : 1.f;
                if (given) {
                    a.dg[o] = chain * (Df[t * L::ldg + i] + off);
                    a.ds[o] = Pf[t * L::ldg + i];
                } else {
                    a.dg[o] = chain * (Df[t * L::ldg + i] + off - Pf[t * L::ldg + i]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
template <typename T, int M>
static hipError_t launch_bwd_tm(const Plan &pl, const Work &w, const void *q, const void *k, const void *v,
                                const float *g, const float *K0, const float *V0, const float *z, const void *dO,
                                const float *dKT, const float *dVT, void *dq, void *dk, void *dv, float *dg,
                                float *dK0, float *dV0, hipStream_t st)
{
    const ChunkMap cm = make_chunk_map(pl, w);
    // 1. recompute the chunk-start memories (and the memories after the last token), unless the forward
    // call left them in this workspace (Section 4, "Efficiency": the kernel without recomputation)
    if (!pl.keep) {
        GSA_HIP_TRY(launch_gates(pl, w, g, pl.s_in, pl.gate_tau, st));
        const ScanIo io = {k, v, K0, V0, nullptr, nullptr, w.SF, false, pl.phi != 0, pl.phi != 0};
        GSA_HIP_TRY(launch_scan(pl, w, io, st));
    }
    dim3 grid(pl.chunk_slots, pl.H);
    // 2. dp, dz and the weights of the reverse scan
    {
        auto kern = !pl.general() ? chunk_dz_kernel<T, M, false, false>
                    : pl.phi     ? chunk_dz_kernel<T, M, true, true>
                                 : chunk_dz_kernel<T, M, true, false>;
        const size_t lds = DzLds<T, M>::bytes;
        GSA_HIP_TRY(allow_lds(kern, lds));
        KernelTimer kt(kSlotChunkDz, st);
        hipLaunchKernelGGL(kern, grid, dim3(Geo<T>::NT), lds, st, cm, pl.H, pl.d_v, pl.scale, (const T *)v,
                           (const T *)dO, g, z, (const T *)w.S, pl.lay, w.dz, w.dgf, (T *)w.Wr, (T *)w.tAvT, pl.s_in,
                           pl.opts(), pl.gate_tau);
        GSA_HIP_TRY(hipGetLastError());
    }
    // 3. reverse scan of the memory gradient
    {
        const ScanIo io = {q, dO, dKT, dVT, dK0, dV0, nullptr, true, pl.phi != 0, false};
        GSA_HIP_TRY(launch_scan(pl, w, io, st));
    }
    // 4. everything chunk-local except the wide contractions
    {
        auto kern = !pl.general() ? chunk_intra_kernel<T, M, false, false>
                    : pl.phi     ? chunk_intra_kernel<T, M, true, true>
                                 : chunk_intra_kernel<T, M, true, false>;
        const size_t lds = IntraLds<T, M>::bytes;
        GSA_HIP_TRY(allow_lds(kern, lds));
        IntraArgs<T> a;
        a.q = (const T *)q; a.k = (const T *)k; a.v = (const T *)v;
        a.g = g; a.z = z; a.dz = w.dz; a.dgf = w.dgf;
        a.S = (const T *)w.S; a.SF = (const T *)w.SF; a.E = (const T *)w.E;
        a.lay = pl.lay;
        a.tAvT = (const T *)w.tAvT;
        a.dg = dg;
        a.tB = (T *)w.tA; a.tBT = (T *)w.tBT; a.tA2T = (T *)w.tA2T; a.tDZe = (T *)w.tP; a.tSbe = (T *)w.tSbe;
        a.sin = pl.s_in; a.ds = pl.ds_out; a.readout = pl.readout; a.gate_tau = pl.gate_tau;
        KernelTimer kt(kSlotChunkIntra, st);
        hipLaunchKernelGGL(kern, grid, dim3(Geo<T>::NT), lds, st, cm, pl.H, pl.d_k, pl.d_v, pl.scale, a);
        GSA_HIP_TRY(hipGetLastError());
    }
    // 5. dq, dk, dv (with the feature map: through its slope at the raw q, k, v)
    const bool phi = pl.phi != 0;
    const ApplyIo io[3] = {
        {w.tA, w.tP, k, w.S, pl.lay.oK, pl.lay.stride, dq, pl.d_k, phi, phi ? q : nullptr},
        {w.tBT, w.tSbe, q, w.E, pl.lay.oK, pl.lay.stride, dk, pl.d_k, phi, phi ? k : nullptr},
        {w.tA2T, w.tSbe, dO, w.E, pl.lay.oV, pl.lay.stride, dv, pl.d_v, false, phi ? v : nullptr},
    };
    return launch_apply(pl, w, io, 3, kSlotApplyBwd, st);
}

template <typename T>
static hipError_t launch_bwd_t(const Plan &pl, const Work &w, const void *q, const void *k, const void *v,
                               const float *g, const float *K0, const float *V0, const float *z, const void *dO,
                               const float *dKT, const float *dVT, void *dq, void *dk, void *dv, float *dg, float *dK0,
                               float *dV0, hipStream_t st)
{
    switch (pl.m) {
    case 16: return launch_bwd_tm<T, 16>(pl, w, q, k, v, g, K0, V0, z, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
    case 32: return launch_bwd_tm<T, 32>(pl, w, q, k, v, g, K0, V0, z, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
    case 128: return launch_bwd_tm<T, 128>(pl, w, q, k, v, g, K0, V0, z, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
    default: return launch_bwd_tm<T, 64>(pl, w, q, k, v, g, K0, V0, z, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
    }
}

hipError_t launch_bwd(const Plan &pl, const Work &w, const void *q, const void *k, const void *v, const float *g,
                      const float *K0, const float *V0, const float *z_saved, const void *dO, const float *dKT,
                      const float *dVT, void *dq, void *dk, void *dv, float *dg, float *dK0, float *dV0,
                      hipStream_t st)
{
    if (pl.tokens == 0) return hipSuccess;
    if (!pl.keep) GSA_HIP_TRY(launch_prepare(pl, w, st));
    if (pl.dtype == 0)
        return launch_bwd_t<float>(pl, w, q, k, v, g, K0, V0, z_saved, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
    return launch_bwd_t<bf16_t>(pl, w, q, k, v, g, K0, V0, z_saved, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
}

}  // namespace gsa
