// The sequential part of Gated Slot Attention: carrying the joint slot memory S = [Kt | Vt]
// (forward) and its gradient E (backward) across chunks (paper, Appendix A,
// Eq. (gla-chunk-gate); Algorithm 1, the two "for n" loops).
//
// Both recurrences have the same shape,
//     acc <- Diag(dec_n) acc + W_n X_n          W_n [m x C] gate-weighted, X_n [C x columns]
// with a snapshot of acc taken BEFORE the update of chunk n.  Forward: W = s*exp(G_C-G),
// X = [k | v], snapshots = memory at chunk start.  Reverse: W = scale*dz*exp(G) (key
// columns) or p*exp(G) (value columns), X = [q | dO], snapshots = memory gradient at chunk
// end.  Nothing in W depends on acc, so the weights are produced by chunk-parallel kernels
// (gate_kernel here, chunk_dz_kernel for the reverse scan) and the sequential loop only
// copies tiles, multiplies and stores:
//
//   * one workgroup per (sequence, head, column slice); the slice of acc lives in MFMA
//     accumulators for the whole sequence;
//   * the tiles of chunk n+1 are prefetched into registers while chunk n is multiplied;
//   * snapshots leave through an LDS tile, as one contiguous block per workgroup (the records are
//     tiled by column slice for this);
//   * workgroups that share (sequence, head) — and therefore W and dec — are mapped to
//     the same XCD so those re-reads hit its L2.
#include "gsa_chunk.h"
#include "gsa_launch.h"

namespace gsa {

// ---------------------------------------------------------------------------------------
// Gate weights of the forward scan (chunk-parallel).
// ---------------------------------------------------------------------------------------
template <typename T, int M, bool GEN>
__global__ __launch_bounds__(Geo<T>::NT) void gate_kernel(ChunkMap cm, int H, const float *__restrict__ g,
                                                          const float *__restrict__ sin, float gate_tau,
                                                          T *__restrict__ Wf, float *__restrict__ dec)
{
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT;
    constexpr int ldg = M + 1;   // odd row stride: the column reads below spread over all banks
    __shared__ float Gs[C * ldg];
    __shared__ float Ss[C * ldg];
    __shared__ float tot[NT];
    ChunkInfo ci;
    if (!chunk_lookup(cm, blockIdx.x, ci)) return;
    const int h = blockIdx.y, tid = threadIdx.x;
    const size_t ch = (size_t)blockIdx.x * H + h;
    const size_t goff = ((size_t)ci.tok0 * H + h) * M;
    gate_prep<M, NT, C, GEN>(Gs, Ss, ldg, tot, g + goff, (size_t)H * M, ci.len, tid, (GEN && sin) ? sin + goff : nullptr,
                             gate_tau);
    T *W = Wf + ch * M * C;
    for (int idx = tid; idx < M * C / 8; idx += NT) {   // eight consecutive tokens of one slot per thread
        const int i = idx / (C / 8), t8 = (idx - i * (C / 8)) * 8;
        const float gc = Gs[(C - 1) * ldg + i];
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = Ss[(t8 + e) * ldg + i] * __expf(gc - Gs[(t8 + e) * ldg + i]);
        store8<T>(W + i * C + t8, x);
    }
    if (tid < M) dec[ch * M + tid] = __expf(Gs[(C - 1) * ldg + tid]);
}

// ---------------------------------------------------------------------------------------
// The scan.
// ---------------------------------------------------------------------------------------
template <typename T> struct ScanArgs {
    const T *W;            // [chunk][H][parts][M][C]
    int w_parts;           // 1 (forward) or 2 (reverse: key part, value part)
    const float *dec;      // [chunk][H][M]
    const T *xk, *xv;      // token tensors feeding the key / value columns
    bool phi_k, phi_v;     // feature map on xk / xv on their way into LDS
    const float *initK, *initV;   // [n_seqs][H][M][d] or NULL
    T *snap;               // one record per (chunk, head)
    StateLayout lay;       // layout of every record
    float *outK, *outV;    // [n_seqs][H][M][d] or NULL: acc after the last chunk
    T *outJ;               // one record per (sequence, head), or NULL: the same, element type T
    // long sequences cut into segments (modes 1 and 2 of the kernel):
    int seg_chunks;        // chunks per segment
    int max_seg;           // segments per sequence the grid provides for
    float *sumY;           // [n_seqs][max_seg][H][M][d_k+d_v]   what a segment adds, from a zero start
    float *sumD;           // [n_seqs][max_seg][H][slices][M]    its total decay
};

template <typename T, int M, int NS> struct ScanLds {
    static constexpr int C = Geo<T>::C;
    static constexpr int PAD = Atom<T>::kPad;
    static constexpr int ldw = C + PAD;      // XT [NS][ldw]
    static constexpr int lds = NS + PAD;     // snapshot tile [M][lds]
    // We [M][C] has no padding: its 8-element groups are XOR-swizzled by the row instead (we_off), which
    // keeps the fragment reads of 16 rows off each other's banks just as well and, with the decays at
    // one word per slot, brings a workgroup under a third of a CU's LDS: three are resident instead of
    // two, which is what lets 640 scan workgroups (d = 640, or five heads) run as one round.
    static constexpr int GW = C / 8;         // groups per row
    __device__ static __forceinline__ int we_off(int i, int t8) { return i * C + (((t8 >> 3) ^ (i & (GW - 1))) << 3); }
    // one set per parity of the chunk's position in the walk: a set is written while the other is read
    static constexpr size_t szW = sizeof(T) * M * C, szX = sizeof(T) * NS * ldw, szS = sizeof(T) * M * lds;
    static constexpr size_t oW = 0;
    static constexpr size_t oX = oW + szW;
    static constexpr size_t oSn = oX + szX;
    static constexpr size_t oDec = oSn + szS;             // chunk decays, fp32 [M]
    static constexpr size_t set = oDec + sizeof(float) * M;
    static constexpr size_t bytes = 2 * set;
};

// MODE 0: one workgroup walks a whole sequence.  A sequence of many chunks leaves the chip waiting on
// that one chain, so long sequences are cut into segments of seg_chunks chunks and walked in two
// launches: MODE 1 walks every segment but the last of the walk from a zero start, without snapshots,
// and leaves what the segment adds (sumY) and its total decay (sumD); MODE 2 walks every segment for
// real, starting from the memory its predecessors leave behind, which it gets by running the
// recurrence over their summaries (at most max_seg - 1 steps of an element-wise update).
template <typename T, int M, int NS, bool REVERSE, int MODE>
__global__ __launch_bounds__(Geo<T>::NT, (M > 64 ? 1 : 2)) void scan_kernel(ChunkMap cm, int H, int d_k, int d_v, int n_seqs,
                                                          ScanArgs<T> a)
{
    using L = ScanLds<T, M, NS>;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT, NW = Geo<T>::NW;
    constexpr int MI = M / 16, NI = NS / (16 * NW);
    constexpr int WVEC = M * C / 8, SVEC = M * NS / 8;
    constexpr int WV = (WVEC + NT - 1) / NT, SV = (SVEC + NT - 1) / NT;
    extern __shared__ __align__(16) unsigned char smem[];
    auto We = [&](int b) { return reinterpret_cast<T *>(smem + b * L::set + L::oW); };
    auto XT = [&](int b) { return reinterpret_cast<T *>(smem + b * L::set + L::oX); };
    auto Sn = [&](int b) { return reinterpret_cast<T *>(smem + b * L::set + L::oSn); };
    auto Dec = [&](int b) { return reinterpret_cast<float *>(smem + b * L::set + L::oDec); };

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4, g8 = (lane >> 4) * 8;
    const int D = d_k + d_v;
    const int nsl = D / NS;
    // XCD-aware placement: consecutive workgroup ids go round-robin over the 8 XCDs.  The slices of one
    // (sequence, head, segment) share W and dec, so a whole group of slices is put on one XCD (one L2),
    // and successive groups on successive XCDs (the segments of a long sequence, of which a packed
    // batch may hold few, then spread over the whole chip).
    const int nseg_grid = (MODE == 0) ? 1 : a.max_seg;
    const int ngroups = H * n_seqs * nseg_grid;
    int slice, group;
    if ((ngroups & 7) == 0) {
        const int x = blockIdx.x & 7, t = blockIdx.x >> 3;
        slice = t % nsl;
        group = (t / nsl) * 8 + x;
    } else {
        slice = blockIdx.x % nsl;
        group = blockIdx.x / nsl;
    }
    // A group is (segment of a sequence, head), heads fastest.  The segments are numbered densely,
    // sequence after sequence; a packed batch has fewer of them than the grid provides for (their
    // number is only known on the device), and the surplus sits at the end of the numbering, so the
    // real ones are spread evenly over the XCDs.
    const int h = group % H, dense = group / H;
    int s, seg;
    if (MODE == 0) {
        s = dense; seg = 0;
    } else if (cm.seg_base) {
        if (dense >= cm.seg_base[n_seqs]) return;   // uniform over the workgroup
        int lo = 0, hi = n_seqs - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (cm.seg_base[mid] <= dense) lo = mid; else hi = mid - 1;
        }
        s = lo; seg = dense - cm.seg_base[lo];
    } else {
        s = dense / nseg_grid; seg = dense % nseg_grid;
    }
    const int col0 = slice * NS;
    const bool isK = col0 < d_k;
    const T *src = isK ? a.xk : a.xv;
    const bool phi = isK ? a.phi_k : a.phi_v;
    const int dsrc = isK ? d_k : d_v;
    const int c0 = isK ? col0 : col0 - d_k;
    const size_t wpart = (a.w_parts == 2 && !isK) ? (size_t)M * C : 0;

    int chunk0, nch_seq, tok0, ntok;
    seq_lookup(cm, s, chunk0, nch_seq, tok0, ntok);
    const int wcol = wave * 16 * NI;
    // the chunks this workgroup walks: [first, first + nch) of the sequence
    int first = 0, nch = nch_seq, nseg = 1;
    if (MODE != 0) {
        nseg = max(1, (nch_seq + a.seg_chunks - 1) / a.seg_chunks);
        first = seg * a.seg_chunks;
        nch = min(a.seg_chunks, nch_seq - first);
        const int last_of_walk = REVERSE ? 0 : nseg - 1;
        if (seg >= nseg || (MODE == 1 && seg == last_of_walk)) return;   // uniform over the workgroup
        if (nch_seq == 0) nch = 0;   // a sequence without tokens still hands its initial memory through (MODE 2)
    }
    const bool starts_walk = (MODE == 0) || seg == (REVERSE ? nseg - 1 : 0);
    const bool ends_walk = (MODE == 0) || seg == (REVERSE ? 0 : nseg - 1);

    f32x4 acc[MI][NI];
    {
        const float *S0 = isK ? a.initK : a.initV;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = mi * 16 + g4 + j, c = c0 + wcol + ni * 16 + r;
                    acc[mi][ni][j] = (MODE != 1 && S0) ? S0[(((size_t)s * H + h) * M + i) * dsrc + c] : 0.f;
                }
        if (MODE == 2 && !starts_walk) {
            // the memory at the start of this segment: the recurrence over the summaries of the segments
            // walked before it, acc <- Diag(sumD) acc + sumY, in walk order
            const int npre = REVERSE ? nseg - 1 - seg : seg;
            for (int u = 0; u < npre; ++u) {
                const int sg = REVERSE ? nseg - 1 - u : u;
                const size_t rec = ((size_t)s * a.max_seg + sg) * H + h;
                const float *Y = a.sumY + rec * M * D + col0;
                const float *Dd = a.sumD + (rec * nsl + slice) * M;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    const f32x4 dd = *reinterpret_cast<const f32x4 *>(Dd + mi * 16 + g4);
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc[mi][ni][j] = dd[j] * acc[mi][ni][j] + Y[(size_t)(mi * 16 + g4 + j) * D + wcol + ni * 16 + r];
                }
            }
        }
        // Let these loads land before the loop's prefetches are issued: otherwise the first use of the
        // accumulator inside the loop has to wait for "everything older", which the compiler can only
        // express as "everything", and that would drain the prefetches in every iteration.
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0) only
    }
    f32x4 dprod[MI];   // MODE 1: product of the chunk decays, rows as in acc
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) dprod[mi] = f32x4{1.f, 1.f, 1.f, 1.f};

    // Operands of one chunk, staged in registers: the loads of the next two chunks are in flight
    // while the current one multiplies (one chunk ahead does not cover the memory latency of a
    // loaded chip, and the chain over the chunks is the only sequential part of the method).
    struct Stage {
        Raw8<T> wreg[WV];
        TokTile<T, C, NS, NT> xt;   // transposed (and swizzled) when it enters LDS
        float dec;                  // decay of slot tid (threads < M)
    };
    auto fetch = [&](Stage &st, int n) {
        const size_t ch = (size_t)(chunk0 + n) * H + h;
        st.dec = a.dec[ch * M + (tid & (M - 1))];
        const T *Wg = a.W + ch * a.w_parts * M * C + wpart;
#pragma unroll
        for (int u = 0; u < WV; ++u) {
            const int idx = tid + NT * u;
            st.wreg[u].load(Wg + (size_t)(idx < WVEC ? idx : 0) * 8);
        }
        const int len = min(C, ntok - n * C);
        const T *Xg = src + ((size_t)(tok0 + n * C) * H + h) * dsrc + c0;
        st.xt.template load<true>(Xg, (size_t)H * dsrc, len, NS, tid);
    };
    // accumulator -> LDS tile [m][cols] -> whole rows of the record's key or value part
    auto snapshot_to_lds = [&](int b) {
        T *dstl = Sn(b);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    dstl[(mi * 16 + g4 + j) * L::lds + wcol + ni * 16 + r] = from_f32<T>(acc[mi][ni][j]);
    };
    auto snapshot_to_global = [&](T *rec, int b) {   // rec: start of the record
        static_assert(NS == kSnapTile, "one workgroup owns one tile of the record");
        T *dst = rec + (isK ? a.lay.oK : a.lay.oV) + (size_t)(c0 / kSnapTile) * (M * kSnapTile);   // contiguous [M][NS]
        const T *srcl = Sn(b);
        // LDS reads first (clamped, unconditional), then the stores: no read sits under a branch
        Raw8<T> x[SV];
#pragma unroll
        for (int u = 0; u < SV; ++u) {
            const int idx = min(tid + NT * u, SVEC - 1), i = idx / (NS / 8), cg = idx - i * (NS / 8);
            x[u].load(srcl + i * L::lds + cg * 8);
        }
#pragma unroll
        for (int u = 0; u < SV; ++u) {
            const int idx = tid + NT * u;
            if (SVEC % NT == 0 || idx < SVEC) x[u].store(dst + (size_t)idx * 8);   // read back by the next kernel: cached
        }
    };
    // staged registers -> LDS set b (W as is, X transposed)
    auto stage_to_lds = [&](const Stage &st, int b) {
        T *w = We(b);
#pragma unroll
        for (int u = 0; u < WV; ++u) {
            const int idx = tid + NT * u;
            if (idx < WVEC) {
                const int i = idx / (C / 8), tg = idx - i * (C / 8);
                st.wreg[u].store(w + L::we_off(i, tg * 8));
            }
        }
        if (phi) st.xt.template store_transposed<true>(XT(b), L::ldw, NS, tid);
        else st.xt.store_transposed(XT(b), L::ldw, NS, tid);
        Dec(b)[tid & (M - 1)] = st.dec;   // every thread stores (slots have NT/M writers of the same value): no branch around a loaded value
    };
    // position in the walk -> chunk; positions past the end repeat the last chunk, so that refills can be
    // issued unconditionally (a refill under a branch makes the number of loads in flight unknown to the
    // compiler, which then waits for all of them wherever it needs one)
    auto chunk_of = [&](int it) { it = min(it, nch - 1); return first + (REVERSE ? nch - 1 - it : it); };

    // The walk, software-pipelined with ONE barrier per chunk.  At the top of step `it` LDS set it%2
    // holds the operands of chunk `it` (written during the previous step) and the snapshot tile of
    // the other set holds the memory the previous chunk started from.  The step
    //   - sends that previous snapshot to global memory,
    //   - snapshots the accumulator (the memory chunk `it` starts from) into its own set,
    //   - applies S <- Diag(dec) S + W X with fragments read from its own set,
    //   - writes the operands of chunk it+1 (register stage `nx`) into the other set and refills
    //     that stage with chunk it+3,
    // so only the accumulator update lies on the chain from one chunk to the next; everything
    // else rides beside it.  A set is rewritten two steps after it was read, with a barrier between.
    auto step = [&](Stage &nx, int it) {
        const int b = it & 1;
        if (MODE != 1) {
            if (it > 0) snapshot_to_global(a.snap + ((size_t)(chunk0 + chunk_of(it - 1)) * H + h) * a.lay.stride, b ^ 1);
            snapshot_to_lds(b);
        }
        typename Atom<T>::Frag af[C / 32][MI], bf[C / 32][NI];
        const T *w = We(b), *x = XT(b);
#pragma unroll
        for (int ks = 0; ks < C / 32; ++ks) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) af[ks][mi] = Atom<T>::load(w + L::we_off(mi * 16 + r, ks * 32 + g8));
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                bf[ks][ni] = Atom<T>::load(x + xt_off<C>(wcol + ni * 16 + r, ks * 32 + g8, L::ldw));
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const f32x4 dcur = *reinterpret_cast<const f32x4 *>(Dec(b) + mi * 16 + g4);
            if (MODE == 1) dprod[mi] *= dcur;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) acc[mi][ni] *= dcur;
        }
#pragma unroll
        for (int ks = 0; ks < C / 32; ++ks)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) Atom<T>::mma(acc[mi][ni], af[ks][mi], bf[ks][ni]);
        stage_to_lds(nx, b ^ 1);
    };
    // (the scheduling fences keep the compiler from hoisting a stage's refill above the LDS stores
    // that read its registers: it would then load into other registers and copy them back at the
    // end of the trip, which means waiting for loads that were only just issued)
    Stage sa, sb;
    if (nch > 0) {
        fetch(sa, chunk_of(0));
        fetch(sb, chunk_of(1));
        stage_to_lds(sa, 0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(sa, chunk_of(2));
        __syncthreads();
    }
    int it = 0;
    for (; it + 1 < nch; it += 2) {   // two steps per trip: each stage keeps its own registers
        step(sb, it);                 // operands in set 0; sb holds chunk it+1
        __builtin_amdgcn_sched_barrier(0);
        fetch(sb, chunk_of(it + 3));
        __syncthreads();
        step(sa, it + 1);             // operands in set 1; sa holds chunk it+2
        __builtin_amdgcn_sched_barrier(0);
        fetch(sa, chunk_of(it + 4));
        __syncthreads();
    }
    if (it < nch) {
        step(sb, it);
        __syncthreads();
        ++it;
    }
    if (MODE != 1 && nch > 0)
        snapshot_to_global(a.snap + ((size_t)(chunk0 + chunk_of(nch - 1)) * H + h) * a.lay.stride, (nch - 1) & 1);
    if (MODE == 1) {   // what this segment adds and how much it decays, for its successors
        const size_t rec = ((size_t)s * a.max_seg + seg) * H + h;
        float *Y = a.sumY + rec * M * D + col0;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int j = 0; j < 4; ++j) Y[(size_t)(mi * 16 + g4 + j) * D + wcol + ni * 16 + r] = acc[mi][ni][j];
        if (wave == 0 && r == 0) {
            float *Dd = a.sumD + (rec * nsl + slice) * M;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) *reinterpret_cast<f32x4 *>(Dd + mi * 16 + g4) = dprod[mi];
        }
        return;
    }
    if (!ends_walk) return;
    // accumulator after the last chunk
    float *ST = isK ? a.outK : a.outV;
    if (ST) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = mi * 16 + g4 + j, c = c0 + wcol + ni * 16 + r;
                    ST[(((size_t)s * H + h) * M + i) * dsrc + c] = acc[mi][ni][j];
                }
    }
    if (a.outJ) {
        __syncthreads();   // the last snapshot tile may still be on its way out
        snapshot_to_lds(0);
        __syncthreads();
        snapshot_to_global(a.outJ + ((size_t)s * H + h) * a.lay.stride, 0);
    }
}

// ---------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------
template <typename T, int M>
static hipError_t launch_gates_tm(const Plan &pl, const Work &w, const float *g, const float *sin, float tau,
                                  hipStream_t st)
{
    const ChunkMap cm = make_chunk_map(pl, w);
    KernelTimer kt(kSlotGates, st);
    if (sin || tau > 0.f)
        hipLaunchKernelGGL((gate_kernel<T, M, true>), dim3(pl.chunk_slots, pl.H), dim3(Geo<T>::NT), 0, st, cm, pl.H, g,
                           sin, tau, (T *)w.Wf, w.dec);
    else
        hipLaunchKernelGGL((gate_kernel<T, M, false>), dim3(pl.chunk_slots, pl.H), dim3(Geo<T>::NT), 0, st, cm, pl.H, g,
                           sin, 0.f, (T *)w.Wf, w.dec);
    return hipGetLastError();
}

hipError_t launch_gates(const Plan &pl, const Work &w, const float *g, const float *sin, float tau, hipStream_t st)
{
#define GSA_GATES(T)                                                   \
    switch (pl.m) {                                                    \
    case 16: return launch_gates_tm<T, 16>(pl, w, g, sin, tau, st);         \
    case 32: return launch_gates_tm<T, 32>(pl, w, g, sin, tau, st);         \
    case 128: return launch_gates_tm<T, 128>(pl, w, g, sin, tau, st);       \
    default: return launch_gates_tm<T, 64>(pl, w, g, sin, tau, st);         \
    }
    if (pl.dtype == 0) { GSA_GATES(float) }
    GSA_GATES(bf16_t)
#undef GSA_GATES
}

template <typename T, int M, int NS, bool REVERSE, int MODE>
static hipError_t run_scan_mode(const Plan &pl, const ChunkMap &cm, const ScanArgs<T> &a, int slot, hipStream_t st)
{
    auto kern = scan_kernel<T, M, NS, REVERSE, MODE>;
    const size_t lds = ScanLds<T, M, NS>::bytes;
    GSA_HIP_TRY(allow_lds(kern, lds));
    const int total = (pl.d_k + pl.d_v) / NS * pl.H * pl.n_seqs * (MODE == 0 ? 1 : a.max_seg);
    KernelTimer kt(slot, st);
    hipLaunchKernelGGL(kern, dim3(total), dim3(Geo<T>::NT), lds, st, cm, pl.H, pl.d_k, pl.d_v, pl.n_seqs, a);
    return hipGetLastError();
}

template <typename T, int M, int NS, bool REVERSE>
static hipError_t run_scan(const Plan &pl, const ChunkMap &cm, const ScanArgs<T> &a, hipStream_t st)
{
    const int slot = REVERSE ? kSlotScanBwd : kSlotScanFwd;
    if (a.max_seg <= 1) return run_scan_mode<T, M, NS, REVERSE, 0>(pl, cm, a, slot, st);
    GSA_HIP_TRY((run_scan_mode<T, M, NS, REVERSE, 1>(pl, cm, a, kSlotScanSummary, st)));
    return run_scan_mode<T, M, NS, REVERSE, 2>(pl, cm, a, slot, st);
}

template <typename T, int M>
static hipError_t launch_scan_tm(const Plan &pl, const Work &w, const ScanIo &io, hipStream_t st)
{
    const ChunkMap cm = make_chunk_map(pl, w);
    ScanArgs<T> a;
    a.W = static_cast<const T *>(io.reverse ? w.Wr : w.Wf);
    a.w_parts = io.reverse ? 2 : 1;
    a.dec = w.dec;
    a.xk = static_cast<const T *>(io.xk);
    a.xv = static_cast<const T *>(io.xv);
    a.phi_k = io.phi_k;
    a.phi_v = io.phi_v;
    a.initK = io.initK;
    a.initV = io.initV;
    a.snap = static_cast<T *>(io.reverse ? w.E : w.S);
    a.lay = pl.lay;
    a.outK = io.outK;
    a.outV = io.outV;
    a.outJ = static_cast<T *>(io.outJ);
    a.seg_chunks = pl.seg_chunks;
    a.max_seg = pl.max_seg;
    a.sumY = w.sumY;
    a.sumD = w.sumD;
    // 64-column slices: several workgroups per CU, so that their dependent chains overlap
    if (io.reverse) return run_scan<T, M, 64, true>(pl, cm, a, st);
    return run_scan<T, M, 64, false>(pl, cm, a, st);
}

hipError_t launch_scan(const Plan &pl, const Work &w, const ScanIo &io, hipStream_t st)
{
#define GSA_SCAN(T)                                                   \
    switch (pl.m) {                                                   \
    case 16: return launch_scan_tm<T, 16>(pl, w, io, st);             \
    case 32: return launch_scan_tm<T, 32>(pl, w, io, st);             \
    case 128: return launch_scan_tm<T, 128>(pl, w, io, st);             \
    default: return launch_scan_tm<T, 64>(pl, w, io, st);             \
    }
    if (pl.dtype == 0) { GSA_SCAN(float) }
    GSA_SCAN(bf16_t)
#undef GSA_SCAN
}

}  // namespace gsa
