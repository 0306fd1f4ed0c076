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
//   dq = scale * ((dz*exp G) Kt_start + Bm K)
//   dk = scale * Bm^T Q + (s*exp(G_C-G)) E_k          dv = A2^T dO + (s*exp(G_C-G)) E_v
//   ds_r[i] = exp(G_C-G_r)[i] <E[i], [k_r|v_r]> + sum_{t>=r} exp(G_t-G_r)[i] (scale dz_t[i] <q_t,k_r> + p_t[i] <dO_t,v_r>)
//   dGam_t = z_t dz_t + p_t dp_t - s_t ds_t          (gradient w.r.t. the cumulative log gate)
//   dg_j   = sum_{t>=j, same chunk} dGam_t + <E[i], S_end[i]> - exp(g_j) ds_j
//
// The last line replaces the sequence-long reversed cumulative sum of Algorithm 1 by a
// chunk-local one: the sum of dGam over all later chunks equals the row-wise inner product
// of the chunk-end memory with its gradient, which both scans already hold.  That keeps
// rounding errors from accumulating along the sequence.
//
// Kernels: gate + forward scan (gsa_scan.hip; recompute chunk-start memories, since nothing
// but z was saved by the forward), bwd_dz (chunk-parallel: dp, dz, weights of the reverse
// scan), reverse scan (gsa_scan.hip: E), bwd_main (chunk-parallel: everything else).
#include "gsa_chunk.h"
#include "gsa_launch.h"

namespace gsa {

// ---------------------------------------------------------------------------------------
// dz kernel
// ---------------------------------------------------------------------------------------
template <typename T, int M> struct DzLds {
    static constexpr int C = Geo<T>::C;
    static constexpr int PAD = Atom<T>::kPad;
    static constexpr int KS = (sizeof(T) == 2) ? 64 : 32;
    static constexpr int ldg = M + 4, lda = C + PAD, ldq = KS + PAD;
    static constexpr size_t oG = 0;
    static constexpr size_t oS = oG + sizeof(float) * C * ldg;
    static constexpr size_t oTot = oS + sizeof(float) * C * ldg;
    static constexpr size_t oA = oTot + sizeof(float) * Geo<T>::NT;
    static constexpr size_t oX = oA + sizeof(T) * C * lda;
    static constexpr size_t oY = oX + sizeof(T) * C * ldq;
    static constexpr size_t oSt = oY + sizeof(T) * C * ldq;
    static constexpr size_t bytes = oSt + sizeof(T) * M * ldq;
};

template <typename T, int M>
__global__ __launch_bounds__(Geo<T>::NT) void bwd_dz_kernel(ChunkMap cm, int H, int d_k, int d_v,
                                                            const T *__restrict__ v, const T *__restrict__ dO,
                                                            const float *__restrict__ g, const float *__restrict__ z,
                                                            const T *__restrict__ S, float scale,
                                                            float *__restrict__ dz, float *__restrict__ dgf,
                                                            T *__restrict__ Wr)
{
    using L = DzLds<T, M>;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT;
    constexpr int MI = M / 16;
    extern __shared__ __align__(16) unsigned char smem[];
    float *Gs = reinterpret_cast<float *>(smem + L::oG);
    float *Ss = reinterpret_cast<float *>(smem + L::oS);
    float *tot = reinterpret_cast<float *>(smem + L::oTot);
    T *As = reinterpret_cast<T *>(smem + L::oA);
    T *Xs = reinterpret_cast<T *>(smem + L::oX);
    T *Ys = reinterpret_cast<T *>(smem + L::oY);
    T *Sts = reinterpret_cast<T *>(smem + L::oSt);

    ChunkInfo ci;
    if (!chunk_lookup(cm, blockIdx.x, ci)) return;
    const int h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4;
    const int D = d_k + d_v;
    const size_t tokh = (size_t)ci.tok0 * H + h;
    const T *Sc = S + (((size_t)blockIdx.x * H + h) * M) * D;
    const int rowb = 16 * w;

    gate_prep<M, NT, C>(Gs, Ss, L::ldg, tot, g + tokh * M, (size_t)H * M, ci.len, tid);
    float dp[MI][4];
    bool unsafe;
    gated_scores<T, M, C, L::KS>(dp, unsafe, Gs, Ss, L::ldg, As, L::lda, Xs, Ys, Sts, L::ldq, dO + tokh * d_v,
                                 v + tokh * d_v, (size_t)H * d_v, d_v, Sc + d_k, (size_t)D, ci.len, tid);
    float zv[MI][4], p[MI][4], rmax[4], rsum[4], pdp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) rmax[j] = -INFINITY;
#pragma unroll
    for (int ni = 0; ni < MI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            zv[ni][j] = (t < ci.len) ? z[(tokh + (size_t)t * H) * M + ni * 16 + r] : 0.f;
            rmax[j] = fmaxf(rmax[j], zv[ni][j]);
        }
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
        for (int j = 0; j < 4; ++j) { p[ni][j] *= rsum[j]; pdp[j] += p[ni][j] * dp[ni][j]; }
#pragma unroll
    for (int j = 0; j < 4; ++j) pdp[j] = row16_sum(pdp[j]);
    // dz, dgf for the main kernel; gate-weighted transposes (scale*dz*exp G, p*exp G) for the reverse scan
    T *Wk = Wr + ((size_t)blockIdx.x * H + h) * 2 * M * C, *Wv = Wk + M * C;
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) {
        const int i = ni * 16 + r;
        T wk[4], wv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            const bool live = t < ci.len;
            const float dzv = live ? p[ni][j] * (dp[ni][j] - pdp[j]) : 0.f;
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
}

// ---------------------------------------------------------------------------------------
// Main chunk-parallel gradient kernel.
// ---------------------------------------------------------------------------------------
template <typename T, int M> struct MainLds {
    static constexpr int C = Geo<T>::C;
    static constexpr int PAD = Atom<T>::kPad;
    static constexpr int KM = (M < 32) ? 32 : M;
    static constexpr int KS = (sizeof(T) == 2) ? 64 : 32;     // contraction slice in phase 1
    static constexpr int NS = (sizeof(T) == 2) ? 128 : 32;    // output column slice in phase 3
    static constexpr int ldg = M + 4, lda = C + PAD, ldp = KM + PAD, ldq = KS + PAD, ldo = NS + PAD;
    // region F: fp32 tiles Gs, Ss, Pf, Df; reused by the phase-3 staging
    static constexpr size_t szF = 4 * sizeof(float) * C * ldg;
    static constexpr size_t oG = 0;
    static constexpr size_t oS = oG + sizeof(float) * C * ldg;
    static constexpr size_t oPf = oS + sizeof(float) * C * ldg;
    static constexpr size_t oDf = oPf + sizeof(float) * C * ldg;
    static constexpr size_t oBt = 0;                                   // [NS][lda] token-contraction operand
    static constexpr size_t oBs = oBt + sizeof(T) * NS * lda;          // [NS][ldp] slot-contraction operand
    static constexpr size_t oO = oBs + sizeof(T) * NS * ldp;           // [C][ldo]  output tile
    static constexpr size_t sz3 = oO + sizeof(T) * C * ldo;
    static constexpr size_t oTot = szF > sz3 ? szF : sz3;
    static constexpr size_t oCarry = oTot + sizeof(float) * Geo<T>::NT;
    // region T: operand tiles that live until the end
    static constexpr size_t oBm = oCarry + sizeof(float) * 128;
    static constexpr size_t oBmT = oBm + sizeof(T) * C * lda;
    static constexpr size_t oA2T = oBmT + sizeof(T) * C * lda;
    static constexpr size_t oDZe = oA2T + sizeof(T) * C * lda;
    static constexpr size_t oSbe = oDZe + sizeof(T) * C * ldp;
    // region U: phase-1 staging, then the transposed score matrices
    static constexpr size_t oU = oSbe + sizeof(T) * C * ldp;
    static constexpr size_t oX = oU;
    static constexpr size_t oY = oX + sizeof(T) * C * ldq;
    static constexpr size_t oE = oY + sizeof(T) * C * ldq;
    static constexpr size_t end1 = oE + sizeof(T) * M * ldq;
    static constexpr size_t oAT = oU;
    static constexpr size_t oAvT = oAT + sizeof(T) * C * lda;
    static constexpr size_t end2 = oAvT + sizeof(T) * C * lda;
    static constexpr size_t bytes = end1 > end2 ? end1 : end2;
};

// Stage E[M][KS] (rows of T, stride ld) into Es while accumulating the row-wise inner product
// with Send (same layout) into part[]: thread handles rows (tid + NT*it) / (KS/8).
template <typename T, int M, int KS, int NT, int ITS>
__device__ __forceinline__ void stage_E_dot(T *Es, int ldq, const T *Eg, const T *Sendg, size_t ld,
                                            float (&part)[ITS], int tid)
{
    constexpr int vpr = KS / 8;
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
        const int idx = tid + NT * it;
        if (idx < M * vpr) {
            const int i = idx / vpr, c = (idx - i * vpr) << 3;
            Raw8<T> e, s;
            e.load(Eg + (size_t)i * ld + c);
            s.load(Sendg + (size_t)i * ld + c);
            float d = 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) d += to_f32(e.get(u)) * to_f32(s.get(u));
            part[it] += d;
            e.store(Es + i * ldq + c);
        }
    }
}

// One output pass of phase 3:  out = s_tok * (A_tok B_tok) + s_slot * (A_slot B_slot), written
// to global rows.  A_tok [C][lda] contracts over the chunk's tokens with rows of `xtok`
// ([len][ncols_total], element type T); A_slot [C][ldp] contracts over slots with rows of
// `xslot` ([M][.] rows of T, row stride ldslot).
template <typename T, int M>
__device__ __forceinline__ void grad_pass(T *dst, size_t ld_dst, int dcols, const T *A_tok, const T *A_slot,
                                          const T *xtok, size_t ld_tok, const T *xslot, size_t ld_slot,
                                          float s_tok, float s_slot, T *Bt, T *Bs, T *Os, int len, int tid)
{
    using L = MainLds<T, M>;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT, NW = Geo<T>::NW;
    constexpr int CI = C / 16, NIo = L::NS / (16 * NW);
    const int lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4;
    for (int cs = 0; cs < dcols; cs += L::NS) {
        const int ncols = min(L::NS, dcols - cs);
        stage_cols<T, T>(Bt, L::lda, xtok + cs, ld_tok, C, ncols, len, tid, NT);
        stage_cols<T, T>(Bs, L::ldp, xslot + cs, ld_slot, M, ncols, M, tid, NT);
        if (M < L::KM) {
            for (int idx = tid; idx < ncols * (L::KM - M); idx += NT)
                Bs[(idx / (L::KM - M)) * L::ldp + M + idx % (L::KM - M)] = from_f32<T>(0.f);
        }
        __syncthreads();
        const int wcol = 16 * NIo * w;
        if (wcol < ncols) {
            f32x4 a1[CI][NIo], a2[CI][NIo];
            zero_acc(a1);
            zero_acc(a2);
            gemm_nt<T, CI, NIo>(a1, A_tok, L::lda, Bt + wcol * L::lda, L::lda, C, lane);
            gemm_nt<T, CI, NIo>(a2, A_slot, L::ldp, Bs + wcol * L::ldp, L::ldp, L::KM, lane);
#pragma unroll
            for (int mi = 0; mi < CI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NIo; ++ni)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        Os[(mi * 16 + g4 + j) * L::ldo + wcol + ni * 16 + r] =
                            from_f32<T>(s_tok * a1[mi][ni][j] + s_slot * a2[mi][ni][j]);
        }
        __syncthreads();
        store_tile<T>(dst + cs, ld_dst, Os, L::ldo, C, ncols, len, tid, NT);
        __syncthreads();
    }
}

template <typename T, int M>
__global__ __launch_bounds__(Geo<T>::NT) void bwd_main_kernel(
    ChunkMap cm, int H, int d_k, int d_v, float scale, const T *__restrict__ q, const T *__restrict__ k,
    const T *__restrict__ v, const T *__restrict__ dO, const float *__restrict__ g, const float *__restrict__ z,
    const float *__restrict__ dz, const float *__restrict__ dgf, const T *__restrict__ S,
    const T *__restrict__ SF, const T *__restrict__ E, T *__restrict__ dq, T *__restrict__ dk,
    T *__restrict__ dv, float *__restrict__ dg)
{
    using L = MainLds<T, M>;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT;
    constexpr int MI = M / 16, CI = C / 16;
    constexpr int ITS = (M * (L::KS / 8) + NT - 1) / NT;
    extern __shared__ __align__(16) unsigned char smem[];
    float *Gs = reinterpret_cast<float *>(smem + L::oG);
    float *Ss = reinterpret_cast<float *>(smem + L::oS);
    float *Pf = reinterpret_cast<float *>(smem + L::oPf);    // p, later exp(g)*ds
    float *Df = reinterpret_cast<float *>(smem + L::oDf);    // dz, later dGam
    float *tot = reinterpret_cast<float *>(smem + L::oTot);
    float *carry = reinterpret_cast<float *>(smem + L::oCarry);
    T *Bms = reinterpret_cast<T *>(smem + L::oBm);           // [t][r]
    T *BmTs = reinterpret_cast<T *>(smem + L::oBmT);         // [r][t]
    T *A2Ts = reinterpret_cast<T *>(smem + L::oA2T);         // [r][t]
    T *DZe = reinterpret_cast<T *>(smem + L::oDZe);          // [t][i] dz exp(G)
    T *Sbe = reinterpret_cast<T *>(smem + L::oSbe);          // [r][i] s exp(G_C - G)
    T *Xs = reinterpret_cast<T *>(smem + L::oX);
    T *Ys = reinterpret_cast<T *>(smem + L::oY);
    T *Es = reinterpret_cast<T *>(smem + L::oE);
    T *ATs = reinterpret_cast<T *>(smem + L::oAT);           // [r][t] (q_t . k_r) for t >= r
    T *AvTs = reinterpret_cast<T *>(smem + L::oAvT);         // [r][t] (dO_t . v_r) for t >= r
    T *Bt = reinterpret_cast<T *>(smem + L::oBt);
    T *Bs = reinterpret_cast<T *>(smem + L::oBs);
    T *Os = reinterpret_cast<T *>(smem + L::oO);

    ChunkInfo ci;
    if (!chunk_lookup(cm, blockIdx.x, ci)) return;
    const int h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4, g8 = (lane >> 4) * 8;
    const int D = d_k + d_v;
    const size_t tokh = (size_t)ci.tok0 * H + h;
    const T *Sc = S + (((size_t)blockIdx.x * H + h) * M) * D;           // memory at chunk start
    const T *Ec = E + (((size_t)blockIdx.x * H + h) * M) * D;           // memory gradient at chunk end
    int chunk0, nch, stok0, sntok;
    seq_lookup(cm, ci.seq, chunk0, nch, stok0, sntok);
    const T *Send = (ci.idx + 1 < nch) ? Sc + (size_t)H * M * D     // next chunk's start memory
                                           : SF + (((size_t)ci.seq * H + h) * M) * D;
    const int rowb = 16 * w;

    gate_prep<M, NT, C>(Gs, Ss, L::ldg, tot, g + tokh * M, (size_t)H * M, ci.len, tid);
    softmax_rows<M, C>(Pf, Df, L::ldg, z + tokh * M, dz + tokh * M, (size_t)H * M, ci.len, tid);

    // ---- phase 1: contractions over the head dimension
    f32x4 accA[CI], accAv[CI], accX[MI];
#pragma unroll
    for (int ni = 0; ni < CI; ++ni) { accA[ni] = f32x4{0.f, 0.f, 0.f, 0.f}; accAv[ni] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) accX[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
    float cpart[ITS];
#pragma unroll
    for (int it = 0; it < ITS; ++it) cpart[it] = 0.f;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const T *X = half ? dO + tokh * d_v : q + tokh * d_k;
        const T *Y = half ? v + tokh * d_v : k + tokh * d_k;
        const int d = half ? d_v : d_k;
        const int coff = half ? d_k : 0;
        for (int ks = 0; ks < d; ks += L::KS) {
            stage_rows<T, T>(Xs, L::ldq, X + ks, (size_t)H * d, C, L::KS, ci.len, tid, NT);
            stage_rows<T, T>(Ys, L::ldq, Y + ks, (size_t)H * d, C, L::KS, ci.len, tid, NT);
            stage_E_dot<T, M, L::KS, NT, ITS>(Es, L::ldq, Ec + coff + ks, Send + coff + ks, (size_t)D, cpart, tid);
            __syncthreads();
#pragma unroll
            for (int k0 = 0; k0 < L::KS; k0 += 32) {
                const typename Atom<T>::Frag aX = Atom<T>::load(Xs + (rowb + r) * L::ldq + k0 + g8);
                const typename Atom<T>::Frag aY = Atom<T>::load(Ys + (rowb + r) * L::ldq + k0 + g8);
#pragma unroll
                for (int ni = 0; ni < CI; ++ni) {
                    if (ni > w) continue;
                    const typename Atom<T>::Frag b = Atom<T>::load(Ys + (ni * 16 + r) * L::ldq + k0 + g8);
                    if (half) Atom<T>::mma(accAv[ni], aX, b);
                    else Atom<T>::mma(accA[ni], aX, b);
                }
#pragma unroll
                for (int ni = 0; ni < MI; ++ni)
                    Atom<T>::mma(accX[ni], aY, Atom<T>::load(Es + (ni * 16 + r) * L::ldq + k0 + g8));
            }
            __syncthreads();
        }
    }
    // carry[i] = <E[i], S_end[i]>: the sum of dGam over every later chunk of this sequence
    {
        constexpr int vpr = L::KS / 8;
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
            float x = cpart[it];
#pragma unroll
            for (int o = 1; o < vpr; o <<= 1) x += __shfl_xor(x, o, 64);
            const int idx = tid + NT * it;
            if (idx < M * vpr && (idx % vpr) == 0) carry[idx / vpr] = x;
        }
    }
    // ---- phase 2a: transposed, causally masked score matrices; gate-scaled operand tiles
#pragma unroll
    for (int ni = 0; ni < CI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j, rr = ni * 16 + r;
            const bool keep = (ni <= w) && (rr <= t);
            ATs[rr * L::lda + t] = from_f32<T>(keep ? accA[ni][j] : 0.f);
            AvTs[rr * L::lda + t] = from_f32<T>(keep ? accAv[ni][j] : 0.f);
        }
    for (int idx = tid; idx < C * L::KM; idx += NT) {
        const int t = idx / L::KM, i = idx - t * L::KM;
        float a = 0.f, b = 0.f;
        if (i < M) {
            const float G = Gs[t * L::ldg + i];
            a = Df[t * L::ldg + i] * __expf(G);
            b = Ss[t * L::ldg + i] * __expf(Gs[(C - 1) * L::ldg + i] - G);
        }
        DZe[t * L::ldp + i] = from_f32<T>(a);
        Sbe[t * L::ldp + i] = from_f32<T>(b);
    }
    __syncthreads();
    const bool unsafe = block_unsafe<M>(Gs, L::ldg, rowb, lane);
    // ---- phase 2b: Bm and A2 for row block w
    {
        f32x4 accB[CI], acc2[CI];
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) { accB[ni] = f32x4{0.f, 0.f, 0.f, 0.f}; acc2[ni] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        for (int k0 = 0; k0 < L::KM; k0 += 32) {
            typename Atom<T>::Frag adz, ap;
            {
                const int t = rowb + r;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int i = k0 + g8 + e;
                    float x = 0.f, y = 0.f;
                    if (i < M) {
                        const float gref = rowb ? Gs[(rowb - 1) * L::ldg + i] : 0.f;
                        const float f = __expf(Gs[t * L::ldg + i] - gref);
                        x = Df[t * L::ldg + i] * f;
                        y = Pf[t * L::ldg + i] * f;
                    }
                    adz[e] = from_f32<T>(x);
                    ap[e] = from_f32<T>(y);
                }
            }
#pragma unroll
            for (int ni = 0; ni < CI; ++ni) {
                if (ni > w || (unsafe && ni == w)) continue;
                const int rr = ni * 16 + r;
                typename Atom<T>::Frag b;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int i = k0 + g8 + e;
                    float val = 0.f;
                    if (i < M) {
                        const float gref = rowb ? Gs[(rowb - 1) * L::ldg + i] : 0.f;
                        val = Ss[rr * L::ldg + i] * __expf(fminf(gref - Gs[rr * L::ldg + i], kExpClamp));
                    }
                    b[e] = from_f32<T>(val);
                }
                Atom<T>::mma(accB[ni], adz, b);
                Atom<T>::mma(acc2[ni], ap, b);
            }
        }
        if (unsafe) {
            const f32x4 eb = pair_weights_exact<M>(Df, L::ldg, Gs, Ss, L::ldg, lane, rowb);
            const f32x4 e2 = pair_weights_exact<M>(Pf, L::ldg, Gs, Ss, L::ldg, lane, rowb);
#pragma unroll
            for (int ni = 0; ni < CI; ++ni)
                if (ni == w) { accB[ni] = eb; acc2[ni] = e2; }
        }
#pragma unroll
        for (int ni = 0; ni < CI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int t = rowb + g4 + j, rr = ni * 16 + r;
                const bool keep = (ni <= w) && (rr <= t);
                const T bv = from_f32<T>(keep ? accB[ni][j] : 0.f);
                Bms[t * L::lda + rr] = bv;
                BmTs[rr * L::lda + t] = bv;
                A2Ts[rr * L::lda + t] = from_f32<T>(keep ? acc2[ni][j] : 0.f);
            }
    }
    // ---- phase 2c: write-intensity gradient ds for rows r of block w, then dGam and exp(g)*ds
    float dGam[MI][4], ads[MI][4];
    {
        f32x4 accW[MI];
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) accW[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int tstart = unsafe ? rowb + 16 : rowb;
        for (int k0 = (tstart & ~31); k0 < C; k0 += 32) {
            const typename Atom<T>::Frag aA = Atom<T>::load(ATs + (rowb + r) * L::lda + k0 + g8);
            const typename Atom<T>::Frag aAv = Atom<T>::load(AvTs + (rowb + r) * L::lda + k0 + g8);
#pragma unroll
            for (int ni = 0; ni < MI; ++ni) {
                const int i = ni * 16 + r;
                const float gend = Gs[(rowb + 15) * L::ldg + i];
                typename Atom<T>::Frag bdz, bp;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int t = k0 + g8 + e;
                    float x = 0.f, y = 0.f;
                    if (t >= tstart) {
                        const float f = __expf(fminf(Gs[t * L::ldg + i] - gend, kExpClamp));
                        x = scale * Df[t * L::ldg + i] * f;
                        y = Pf[t * L::ldg + i] * f;
                    }
                    bdz[e] = from_f32<T>(x);
                    bp[e] = from_f32<T>(y);
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
                                to_f32(AvTs[rr * L::lda + t]) * Pf[t * L::ldg + i]) *
                               __expf(Gs[t * L::ldg + i] - Gr);
                    ds += sum;
                }
                const float sv = Ss[rr * L::ldg + i];
                const float f = (rr < ci.len) ? dgf[(tokh + (size_t)rr * H) * M + i] : 0.f;
                dGam[ni][j] = f - sv * ds;
                ads[ni][j] = (1.f - sv) * ds;
            }
        }
    }
    __syncthreads();   // every wave is done reading p and dz
#pragma unroll
    for (int ni = 0; ni < MI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int rr = rowb + g4 + j, i = ni * 16 + r;
            Df[rr * L::ldg + i] = dGam[ni][j];
            Pf[rr * L::ldg + i] = ads[ni][j];
        }
    __syncthreads();
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
        float off = carry[i];
        for (int pp = part + 1; pp < P; ++pp) off += tot[pp * M + i];
        for (int tt = 0; tt < TP; ++tt) {
            const int t = part * TP + tt;
            if (t < ci.len) dg[(tokh + (size_t)t * H) * M + i] = Df[t * L::ldg + i] + off - Pf[t * L::ldg + i];
        }
    }
    __syncthreads();
    // ---- phase 3: dq, dk, dv
    grad_pass<T, M>(dq + tokh * d_k, (size_t)H * d_k, d_k, Bms, DZe, k + tokh * d_k, (size_t)H * d_k, Sc, (size_t)D,
                    scale, scale, Bt, Bs, Os, ci.len, tid);
    grad_pass<T, M>(dk + tokh * d_k, (size_t)H * d_k, d_k, BmTs, Sbe, q + tokh * d_k, (size_t)H * d_k, Ec, (size_t)D,
                    scale, 1.f, Bt, Bs, Os, ci.len, tid);
    grad_pass<T, M>(dv + tokh * d_v, (size_t)H * d_v, d_v, A2Ts, Sbe, dO + tokh * d_v, (size_t)H * d_v, Ec + d_k,
                    (size_t)D, 1.f, 1.f, Bt, Bs, Os, ci.len, tid);
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
    // 1. recompute the chunk-start memories (and the memories after the last token)
    GSA_HIP_TRY(launch_gates(pl, w, g, st));
    {
        const ScanIo io = {k, v, K0, V0, nullptr, nullptr, w.SF, false};
        GSA_HIP_TRY(launch_scan(pl, w, io, st));
    }
    dim3 grid(pl.chunk_slots, pl.H);
    // 2. dp, dz and the weights of the reverse scan
    {
        auto kern = bwd_dz_kernel<T, M>;
        const size_t lds = DzLds<T, M>::bytes;
        GSA_HIP_TRY(allow_lds(kern, lds));
        KernelTimer kt(kSlotBwdDz, st);
        hipLaunchKernelGGL(kern, grid, dim3(Geo<T>::NT), lds, st, cm, pl.H, pl.d_k, pl.d_v, (const T *)v,
                           (const T *)dO, g, z, (const T *)w.S, pl.scale, w.dz, w.dgf, (T *)w.Wr);
        GSA_HIP_TRY(hipGetLastError());
    }
    // 3. reverse scan of the memory gradient
    {
        const ScanIo io = {q, dO, dKT, dVT, dK0, dV0, nullptr, true};
        GSA_HIP_TRY(launch_scan(pl, w, io, st));
    }
    // 4. everything chunk-local
    {
        auto kern = bwd_main_kernel<T, M>;
        const size_t lds = MainLds<T, M>::bytes;
        GSA_HIP_TRY(allow_lds(kern, lds));
        KernelTimer kt(kSlotBwdMain, st);
        hipLaunchKernelGGL(kern, grid, dim3(Geo<T>::NT), lds, st, cm, pl.H, pl.d_k, pl.d_v, pl.scale, (const T *)q,
                           (const T *)k, (const T *)v, (const T *)dO, g, z, w.dz, w.dgf, (const T *)w.S, (const T *)w.SF,
                           (const T *)w.E, (T *)dq,
                           (T *)dk, (T *)dv, dg);
        GSA_HIP_TRY(hipGetLastError());
    }
    return hipSuccess;
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
    default: return launch_bwd_tm<T, 64>(pl, w, q, k, v, g, K0, V0, z, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
    }
}

hipError_t launch_bwd(const Plan &pl, const Work &w, const void *q, const void *k, const void *v, const float *g,
                      const float *K0, const float *V0, const float *z_saved, const void *dO, const float *dKT,
                      const float *dVT, void *dq, void *dk, void *dv, float *dg, float *dK0, float *dV0,
                      hipStream_t st)
{
    if (pl.tokens == 0) return hipSuccess;
    GSA_HIP_TRY(launch_prepare(pl, w, st));
    if (pl.dtype == 0)
        return launch_bwd_t<float>(pl, w, q, k, v, g, K0, V0, z_saved, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
    return launch_bwd_t<bf16_t>(pl, w, q, k, v, g, K0, V0, z_saved, dO, dKT, dVT, dq, dk, dv, dg, dK0, dV0, st);
}

}  // namespace gsa
