// Forward pass of Gated Slot Attention, chunkwise (paper: Eq. (gsa), Eq. (gsa-2pass),
// Appendix A Eqs. (gla-chunk-gate)/(gla-chunk), Algorithm 1 forward).
//
// Both slot memories decay with the same gate and are written with the same
// intensity, so they are carried as ONE memory S = [Kt | Vt] of shape
// [m x (d_k+d_v)].  Kernels of one forward call:
//
//   gate_kernel +     (gsa_scan.hip) one workgroup per (sequence, head, column slice of S)
//   scan_kernel       walks the chunks in order, keeps its slice of S in matrix-core
//                     accumulators and writes the memory at the START of every chunk to the
//                     workspace (the only sequential part; column slices are independent).
//   chunk_fwd_kernel  one workgroup per (chunk, head): pass-1 scores z (inter-chunk term from
//                     the stored memory + gated intra-chunk term), softmax over the slots in
//                     registers, and the two small matrices of pass 2: p*exp(G) [C x m] and
//                     the pair weights A2 [C x C].  z and p never round-trip HBM except for
//                     the z the backward needs.
//   apply_kernel      (gsa_apply.hip) o = (p e^G) Vt_start + A2 V, the wide contraction.
//
// Gate handling inside a chunk: rows are grouped in blocks of 16 tokens.  For row block I
// the reference is the cumulative log gate just before the block, Gref_I.  exp(G_t - G_r)
// is factored as exp(G_t - Gref_I) * exp(Gref_I - G_r): the first factor is <= 1, the
// second is <= 1 for every earlier block and bounded by the decay inside one 16-token
// block on the diagonal.  If that bound exceeds e^80 (not reachable with the paper's gate
// parameterisation) the diagonal block is evaluated pairwise without factoring.
#include "gsa_chunk.h"
#include "gsa_launch.h"

namespace gsa {

// ---------------------------------------------------------------------------------------
// Packed form: build the chunk table from the device-side sequence offsets.
// ---------------------------------------------------------------------------------------
__global__ void prepare_kernel(const int32_t *__restrict__ cu, int n_seqs, int T, int kChunk, int chunk_slots,
                               int seg_chunks, int32_t *__restrict__ table, int32_t *__restrict__ seqtab,
                               int32_t *__restrict__ segbase)
{
    __shared__ int total;
    if (threadIdx.x == 0) {
        int c0 = 0, prev_end = 0, nsegs = 0;
        for (int s = 0; s < n_seqs; ++s) {
            int b = min(max(cu[s], prev_end), T);
            int e = min(max(cu[s + 1], b), T);
            const int nch = (e - b + kChunk - 1) / kChunk;
            seqtab[4 * s + 0] = c0;
            seqtab[4 * s + 1] = nch;
            seqtab[4 * s + 2] = b;
            seqtab[4 * s + 3] = e - b;
            segbase[s] = nsegs;                                    // scan segments (gsa_scan.hip); an empty
            nsegs += max(1, (nch + seg_chunks - 1) / seg_chunks);  // sequence still has one
            c0 += nch;
            prev_end = e;
        }
        segbase[n_seqs] = nsegs;
        total = c0;
    }
    __syncthreads();
    // one chunk slot per thread and pass: its sequence is the last one whose first chunk is <= the slot
    // (a sequence without tokens shares its first-chunk index with its successor, so it is never the last)
    const int used = min(total, chunk_slots);
    for (int c = threadIdx.x; c < used; c += blockDim.x) {
        int lo = 0, hi = n_seqs - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (seqtab[4 * mid + 0] <= c) lo = mid; else hi = mid - 1;
        }
        const int j = c - seqtab[4 * lo + 0];
        table[4 * c + 0] = lo;
        table[4 * c + 1] = seqtab[4 * lo + 2] + j * kChunk;
        table[4 * c + 2] = min(kChunk, seqtab[4 * lo + 3] - j * kChunk);
        table[4 * c + 3] = j;
    }
    for (int c = total + threadIdx.x; c < chunk_slots; c += blockDim.x) {
        table[4 * c + 0] = 0; table[4 * c + 1] = 0; table[4 * c + 2] = 0; table[4 * c + 3] = 0;
    }
}

hipError_t launch_prepare(const Plan &pl, const Work &w, hipStream_t st)
{
    if (!pl.cu_seqlens) return hipSuccess;
    KernelTimer kt(kSlotPrepare, st);
    hipLaunchKernelGGL(prepare_kernel, dim3(1), dim3(256), 0, st, pl.cu_seqlens, pl.n_seqs, pl.T, pl.chunk,
                       pl.chunk_slots, pl.seg_chunks, w.table, w.seqtab, w.segbase);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Chunk kernel of the forward: scores, softmax, pass-2 weights.
// ---------------------------------------------------------------------------------------
template <typename T, int M> struct ChunkFwdLds {
    static constexpr int C = Geo<T>::C;
    static constexpr int PAD = Atom<T>::kPad;
    static constexpr int KM = (M < 32) ? 32 : M;   // slots padded to the contraction depth
    static constexpr int ldg = M + 4;
    static constexpr int lda = C + PAD;            // As
    static constexpr int ldp = KM + PAD;           // Ps
    static constexpr size_t oG = 0;
    static constexpr size_t oS = oG + sizeof(float) * C * ldg;
    static constexpr size_t oA = oS + sizeof(float) * C * ldg;
    static constexpr size_t oTot = oA;             // gate_prep's scratch, dead before As is written
    static constexpr size_t szA = sizeof(T) * C * lda > sizeof(float) * Geo<T>::NT ? sizeof(T) * C * lda
                                                                                  : sizeof(float) * Geo<T>::NT;
    static constexpr size_t oP = oA + szA;
    static constexpr size_t oVt = oP + sizeof(T) * C * ldp;           // Vt [M][lda]
    static constexpr size_t oRb = oVt + sizeof(T) * M * lda;          // Rb [C/16][M] fp32
    static constexpr size_t end = oRb + sizeof(float) * (C / 16) * M;
    static constexpr int kRpr = 2;                 // row blocks per round of the reduction
    static constexpr size_t szRed = sizeof(f32x4) * kWave * (C / 16) *
                                    reduce_fragments<C / 16, C / 16 + M / 16, C / 16, kRpr>();   // from offset 0: dead before the tiles are written
    static constexpr size_t bytes = end > szRed ? end : szRed;
};

// GEN: the general form (write intensities from `sin` when it is not NULL; opts: read-out in the low
// byte).  PHI (with GEN): the feature map on q and k.
template <typename T, int M, bool GEN, bool PHI>
__global__ __launch_bounds__(Geo<T>::NT, (M > 64 ? 1 : 2)) void chunk_fwd_kernel(ChunkMap cm, int H, int d_k, float scale,
                                                               const T *__restrict__ q, const T *__restrict__ k,
                                                               const float *__restrict__ g,
                                                               const T *__restrict__ S, StateLayout lay,
                                                               float *__restrict__ z_saved, T *__restrict__ tA,
                                                               T *__restrict__ tP, const float *__restrict__ sin,
                                                               int opts, float gate_tau)
{
    using L = ChunkFwdLds<T, M>;
    const int readout = opts & kReadoutMask;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT;
    constexpr int MI = M / 16, CI = C / 16, KM = L::KM;
    extern __shared__ __align__(16) unsigned char smem[];
    float *Gs = reinterpret_cast<float *>(smem + L::oG);
    float *Ss = reinterpret_cast<float *>(smem + L::oS);
    float *tot = reinterpret_cast<float *>(smem + L::oTot);
    T *As = reinterpret_cast<T *>(smem + L::oA);      // [C][lda]  A = QK^T masked, later A2
    T *Ps = reinterpret_cast<T *>(smem + L::oP);      // [C][ldp]  softmax weights in their gated forms

    ChunkInfo ci;
    int cid, h;
    chunk_order(cm, H, true, cid, h);   // the forward scan has just written the last chunks
    if (!chunk_lookup(cm, cid, ci)) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4;
    const size_t tokh = (size_t)ci.tok0 * H + h;
    const size_t ch = (size_t)cid * H + h;
    const T *Kn = S + ch * lay.stride + lay.oK;      // key memory at chunk start (tiled)
    const int rowb = 16 * w;                          // this wave's row block

    // ---- pass 1: z = scale * (inter + gated intra), Eq. (gla-chunk) with the gate on the slot side
    float p[MI][4];
    bool unsafe;
    T *Vt = reinterpret_cast<T *>(smem + L::oVt);
    float *Rb = reinterpret_cast<float *>(smem + L::oRb);
    // q, k and the key memory are not read again by this forward call: all three hinted
    gated_scores<T, M, C, GEN, L::kRpr, kHintX | kHintY | kHintSt>(
        p, unsafe, Gs, Ss, L::ldg, tot, g + tokh * M, (size_t)H * M, As, L::lda, Vt, L::lda, Rb,
        reinterpret_cast<f32x4 *>(smem), q + tokh * d_k, k + tokh * d_k,
        (size_t)H * d_k, d_k, Kn, ci.len, tid, (GEN && sin) ? sin + tokh * M : nullptr, gate_tau,
        PHI ? (kHintX | kHintY) : 0);
    // ---- softmax over the slots, in registers
    float rmax[4], rsum[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) rmax[j] = -INFINITY;
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) {
        const int i = ni * 16 + r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            const float z = scale * p[ni][j];
            p[ni][j] = z;
            rmax[j] = fmaxf(rmax[j], z);
            if (z_saved && t < ci.len) z_saved[(tokh + (size_t)t * H) * M + i] = z;
        }
    }
    if (!GEN || readout == kReadSoftmax) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { rmax[j] = row16_max(rmax[j]); rsum[j] = 0.f; }
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) { p[ni][j] = __expf(p[ni][j] - rmax[j]); rsum[j] += p[ni][j]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) rsum[j] = 1.f / row16_sum(rsum[j]);
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) p[ni][j] *= rsum[j];
    } else {   // element-wise read-out (ablations of Section 4)
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) p[ni][j] = readout_value(readout, p[ni][j]);
    }
    if (M < KM) {   // zero the padded slot columns once
#pragma unroll
        for (int j = 0; j < 4; ++j) Ps[(rowb + g4 + j) * L::ldp + M + r] = from_f32<T>(0.f);
    }
    // ---- pass-2 pair weights A2[t][r] = sum_i p_t[i] s_r[i] exp(G_t[i] - G_r[i]), r <= t
    f32x4 exact = {0.f, 0.f, 0.f, 0.f};
    if (__syncthreads_or(unsafe)) {   // rare: some row block needs its diagonal unfactored
#pragma unroll
        for (int ni = 0; ni < MI; ++ni)
#pragma unroll
            for (int j = 0; j < 4; ++j) Ps[(rowb + g4 + j) * L::ldp + ni * 16 + r] = from_f32<T>(p[ni][j]);
        __syncthreads();
        if (unsafe) exact = pair_weights_exact<M, T>(Ps, L::ldp, Gs, Ss, L::ldg, lane, rowb);
        __syncthreads();
    }
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) {
        const int i = ni * 16 + r;
        const float gref = rowb ? Gs[(rowb - 1) * L::ldg + i] : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            Ps[t * L::ldp + i] = from_f32<T>(p[ni][j] * __expf(Gs[t * L::ldg + i] - gref));
        }
    }
    __syncthreads();
    {
        f32x4 acc2[CI];
        pair_weights<T, M, C, KM>(acc2, Ps, L::ldp, Gs, Ss, L::ldg, unsafe, lane, w);
        if (unsafe) {
#pragma unroll
            for (int ni = 0; ni < CI; ++ni)
                if (ni == w) acc2[ni] = exact;
        }
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) {
            if (ni > w) continue;   // those columns already hold zeros from the masked A
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int t = rowb + g4 + j, rr = ni * 16 + r;
                As[t * L::lda + rr] = from_f32<T>(rr <= t ? acc2[ni][j] : 0.f);
            }
        }
    }
    // inter-chunk pass-2 weights p * exp(G) (this wave's rows of Ps were read by this wave only)
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) {
        const int i = ni * 16 + r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            Ps[t * L::ldp + i] = from_f32<T>(p[ni][j] * __expf(Gs[t * L::ldg + i]));
        }
    }
    __syncthreads();
    // ---- hand the two small matrices to the apply kernel
    {
        T *dA = tA + ch * C * C, *dP = tP + ch * C * KM;
        for (int idx = tid; idx < C * C / 8; idx += NT) {
            const int t = idx / (C / 8), c8 = (idx - t * (C / 8)) * 8;
            Raw8<T> x;
            x.load(As + t * L::lda + c8);
            x.store(dA + t * C + c8);
        }
        for (int idx = tid; idx < C * KM / 8; idx += NT) {
            const int t = idx / (KM / 8), c8 = (idx - t * (KM / 8)) * 8;
            Raw8<T> x;
            x.load(Ps + t * L::ldp + c8);
            x.store(dP + t * KM + c8);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
template <typename T, int M>
static hipError_t launch_fwd_tm(const Plan &pl, const Work &w, const void *q, const void *k, const void *v,
                                const float *g, const float *K0, const float *V0, void *o, float *z_saved, float *KT,
                                float *VT, hipStream_t st)
{
    const ChunkMap cm = make_chunk_map(pl, w);
    GSA_HIP_TRY(launch_gates(pl, w, g, pl.s_in, pl.gate_tau, st));
    {
        // kept for the backward: also the memories after the last token, as the recomputation would leave them
        const ScanIo io = {k, v, K0, V0, KT, VT, pl.keep ? w.SF : nullptr, false, pl.phi != 0, pl.phi != 0};
        GSA_HIP_TRY(launch_scan(pl, w, io, st));
    }
    {
        auto kern = !pl.general() ? chunk_fwd_kernel<T, M, false, false>
                    : pl.phi     ? chunk_fwd_kernel<T, M, true, true>
                                 : chunk_fwd_kernel<T, M, true, false>;
        const size_t lds = ChunkFwdLds<T, M>::bytes;
        GSA_HIP_TRY(allow_lds(kern, lds));
        dim3 grid(pl.chunk_slots, pl.H);
        KernelTimer kt(kSlotChunkFwd, st);
        hipLaunchKernelGGL(kern, grid, dim3(Geo<T>::NT), lds, st, cm, pl.H, pl.d_k, pl.scale, (const T *)q,
                           (const T *)k, g, (const T *)w.S, pl.lay, z_saved, (T *)w.tA, (T *)w.tP, pl.s_in,
                           pl.opts(), pl.gate_tau);
        GSA_HIP_TRY(hipGetLastError());
    }
    ApplyIo io = {w.tA, w.tP, v, w.S, pl.lay.oV, pl.lay.stride, o, pl.d_v, pl.phi != 0, nullptr};
    io.act = pl.act_out;
    io.ssq = pl.act_ssq;
    return launch_apply(pl, w, &io, 1, kSlotApplyFwd, st);
}

template <typename T>
static hipError_t launch_fwd_t(const Plan &pl, const Work &w, const void *q, const void *k, const void *v,
                               const float *g, const float *K0, const float *V0, void *o, float *z_saved, float *KT,
                               float *VT, hipStream_t st)
{
    switch (pl.m) {
    case 16: return launch_fwd_tm<T, 16>(pl, w, q, k, v, g, K0, V0, o, z_saved, KT, VT, st);
    case 32: return launch_fwd_tm<T, 32>(pl, w, q, k, v, g, K0, V0, o, z_saved, KT, VT, st);
    case 128: return launch_fwd_tm<T, 128>(pl, w, q, k, v, g, K0, V0, o, z_saved, KT, VT, st);
    default: return launch_fwd_tm<T, 64>(pl, w, q, k, v, g, K0, V0, o, z_saved, KT, VT, st);
    }
}

hipError_t launch_fwd(const Plan &pl, const Work &w, const void *q, const void *k, const void *v, const float *g,
                      const float *K0, const float *V0, void *o, float *z_saved, float *KT, float *VT, hipStream_t st)
{
    if (pl.tokens == 0) return hipSuccess;
    GSA_HIP_TRY(launch_prepare(pl, w, st));
    if (pl.dtype == 0) return launch_fwd_t<float>(pl, w, q, k, v, g, K0, V0, o, z_saved, KT, VT, st);
    return launch_fwd_t<bf16_t>(pl, w, q, k, v, g, K0, V0, o, z_saved, KT, VT, st);
}

}  // namespace gsa
