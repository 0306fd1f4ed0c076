// Chunk-level device routines shared by the forward output kernel and the backward
// kernels: the gated "scores" contraction that both GLA passes of GSA reduce to.
//
// Gate handling (paper, Appendix A: the chunkwise form divides by cumulative decays,
// which overflows; GLA's remedy is a secondary chunking).  Here rows of a chunk are
// grouped in blocks of 16 tokens, one wave per block.  For row block I the reference
// is the cumulative log gate just before the block, Gref_I, and
//     exp(G_t - G_r) = exp(G_t - Gref_I) * exp(Gref_I - G_r).
// The first factor is <= 1.  The second is <= 1 for every earlier block and, inside
// the diagonal block, bounded by the decay across 16 tokens.  If that decay exceeds
// e^80 for some slot (alpha < 0.007 sustained over a block; not reachable with the
// paper's sigmoid^(1/8) gates) the diagonal block is evaluated pair by pair with the
// unfactored exponent instead.
#pragma once
#include "gsa_common.h"

namespace gsa {

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// True when the factored form is not safe for the 16-token block starting at row rowb:
// some slot decays by more than e^kExpClamp across the block.  Wave-uniform.
template <int M>
__device__ __forceinline__ bool block_unsafe(const float *Gs, int ldg, int rowb, int lane)
{
    float drop = 0.f;
    for (int i = lane; i < M; i += kWave) {
        const float gref = rowb ? Gs[(rowb - 1) * ldg + i] : 0.f;
        drop = fmaxf(drop, gref - Gs[(rowb + 15) * ldg + i]);
    }
    return wave_max(drop) > kExpClamp;
}

// Split-contraction bookkeeping.  The chunk kernels contract over the head dimension with
// every wave taking a slice of that dimension for ALL row blocks of the chunk (so each
// operand byte is loaded by exactly one wave, in whole 128-byte lines), and then sum the
// per-wave partial accumulators so that wave w ends up with the totals of row block w.
// acc[rb][cb] are D fragments; the first CAUSAL column blocks are only needed for cb <= rb.
// Red: LDS, NW*NB*64 f32x4 (fragments are exchanged lane for lane, so any wave's layout
// is every wave's layout).  w must be wave-uniform.  Contains barriers: all threads of the
// workgroup must call it.
// RPR row blocks are exchanged per round (RPR divides NW): fewer, fuller rounds need fewer barriers
// and keep more waves busy adding, at the price of a larger buffer, reduce_fragments<..>() * NW * 64 f32x4.
template <int NW, int NB, int CAUSAL, int RPR> constexpr int reduce_fragments()
{
    int worst = 0;
    for (int rb0 = 0; rb0 < NW; rb0 += RPR) {
        int n = 0;
        for (int rb = rb0; rb < rb0 + RPR; ++rb)
            for (int cb = 0; cb < NB; ++cb)
                if (!(cb < CAUSAL && cb > rb)) ++n;
        worst = n > worst ? n : worst;
    }
    return worst;
}

template <int NW, int NB, int CAUSAL, int RPR = 1>
__device__ __forceinline__ void reduce_row_blocks(f32x4 (&own)[NB], const f32x4 (&acc)[NW][NB], f32x4 *Red, int lane,
                                                  int w)
{
    static_assert(NW % RPR == 0, "row blocks per round");
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) own[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Per round: every wave posts its partials of the round's row blocks, each block's owner adds
    // them in wave order.  (Register arrays are indexed by constants only; the wave index enters
    // through LDS addresses.)  Slot numbers count the posted fragments of a round in (rb, cb) order.
#pragma unroll
    for (int rb0 = 0; rb0 < NW; rb0 += RPR) {
        int slot = 0;
#pragma unroll
        for (int rb = rb0; rb < rb0 + RPR; ++rb)
#pragma unroll
            for (int cb = 0; cb < NB; ++cb)
                if (!(cb < CAUSAL && cb > rb)) { Red[(slot * NW + w) * kWave + lane] = acc[rb][cb]; ++slot; }
        __syncthreads();
        slot = 0;
#pragma unroll
        for (int rb = rb0; rb < rb0 + RPR; ++rb)
#pragma unroll
            for (int cb = 0; cb < NB; ++cb) {
                if (cb < CAUSAL && cb > rb) continue;
                if (w == rb) {
                    f32x4 x = Red[(slot * NW) * kWave + lane];
#pragma unroll
                    for (int u = 1; u < NW; ++u) x += Red[(slot * NW + u) * kWave + lane];
                    own[cb] = x;
                }
                ++slot;
            }
        __syncthreads();
    }
}

// Write-intensity tiles of one chunk, referenced to the END of each token's own 16-token block:
//   V[kk][i] = s_kk[i] * exp(G_end(kk)[i] - G_kk[i])  <= 1        (G_end = cumulative gate at the block's last token)
// stored transposed, Vt[i][kk] (operand of contractions over tokens); plus the decay across each block,
//   Rb[b][i] = exp(G_end(b)[i] - G_end(b-1)[i]).
// With these, the weight between a token of row block w and an EARLIER block's token needs no
// exponential of its own: exp(G_t - G_kk) = exp(G_t - G_start(w)) * prod of Rb over the blocks in
// between * exp(G_end(kk) - G_kk), every factor <= 1 (nothing to clamp).  One (block, slot) pair
// per thread and pass; no barrier inside.
template <typename T, int M, int C>
__device__ __forceinline__ void build_write_tiles(const float *Gs, const float *Ss, int ldg, T *Vt, int ldv, float *Rb,
                                                  int tid)
{
    constexpr int CI = C / 16, NT = Geo<T>::NT;
    for (int idx = tid; idx < CI * M; idx += NT) {
        const int b = idx / M, i = idx - b * M;
        const float gend = Gs[(16 * b + 15) * ldg + i];
        const float gstart = b ? Gs[(16 * b - 1) * ldg + i] : 0.f;
        Rb[b * M + i] = __expf(gend - gstart);
        float x[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int kk = 16 * b + e;
            x[e] = Ss[kk * ldg + i] * __expf(gend - Gs[kk * ldg + i]);
        }
        float lo[8], hi[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { lo[e] = x[e]; hi[e] = x[8 + e]; }
        store8<T>(Vt + i * ldv + 16 * b, lo);
        store8<T>(Vt + i * ldv + 16 * b + 8, hi);
    }
}

// For this wave's row block (rows t = rowb .. rowb+15), in D layout (lane holds slot
// i = 16*ni + lane%16, rows t = rowb + 4*(lane/16) + j):
//
//   out[ni][j] = exp(G_t[i]) * <X_t, St[i]>  +  sum_{r<=t} <X_t, Y_r> s_r[i] exp(G_t[i]-G_r[i])
//
// i.e. the inter-chunk plus intra-chunk parts of one gated pass whose gate sits on the
// slot side (pass 1 of Eq. (gsa-2pass) with X=q, Y=k, St=Kt; its mirror in the backward
// with X=dO, Y=v, St=Vt).  X, Y: [len][d] rows in global memory (row stride ldx elements);
// St: one part of a memory snapshot (M slots, d columns, tiled as StateLayout describes).
// The contraction over d reads its operand fragments straight from global memory (each lane 16
// bytes of one row; no staging).  It is split over the waves in steps of 64 columns, wave w taking steps w, w+NW, ...: a wave asks for the two
// halves of a 128-byte line in consecutive instructions, so each line crosses the
// memory system once.  The partial sums meet through Red (see reduce_row_blocks; Red may
// alias As).  d must be a multiple of 64.
// The gate tiles Gs, Ss are produced in here as well (from g: [len][M] fp32, row stride gld;
// `tot`: scratch of NT floats): the gate loads are issued after the contraction and land during
// the reduction, and the tiles are written once the reduction buffer is dead, so Red may alias
// Gs and Ss too.  As [C][lda] is left holding the causally masked X Y^T rounded to T, and the tiles
// of build_write_tiles are left in Vt, Rb for the caller's own use.
// All threads of the workgroup must call it.
// GEN: general form; sin = write intensities [len][M] (layout of g) or NULL for 1 - exp(g).
// RPR: row blocks per round of the reduction (Red must hold reduce_fragments<..., RPR>() * NW * 64 f32x4).
// HINT: which operands are loaded with the non-temporal hint (kHintX | kHintY | kHintSt) -- those the
// caller knows nobody reads again soon.  Both halves of every 128-byte line are asked for by the
// same wave in the same step, so a hinted line is never dropped between its two readers.
constexpr int kHintX = 1, kHintY = 2, kHintSt = 4;
// phi (general form only): which of X, Y get the feature map after the load (kHintX | kHintY bits).
template <typename T, int M, int C, bool GEN = false, int RPR = 1, int HINT = 0>
__device__ __forceinline__ void gated_scores(float (&out)[M / 16][4], bool &unsafe, float *Gs, float *Ss, int ldg,
                                             float *tot, const float *g, size_t gld, T *As, int lda, T *Vt, int ldv,
                                             float *Rb, f32x4 *Red, const T *X, const T *Y,
                                             size_t ldx, int d, const T *St, int len, int tid,
                                             const float *sin = nullptr, float gate_tau = 0.f, int phi = 0)
{
    constexpr int MI = M / 16, CI = C / 16, NW = CI, NB = CI + MI;
    const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g4 = (lane >> 4) * 4, g8 = (lane >> 4) * 8;
    const int rowb = 16 * w;

    f32x4 accA[CI], accZ[MI];
    {
        f32x4 acc[NW][NB];   // [row block][Y blocks | St blocks]
#pragma unroll
        for (int rb = 0; rb < NW; ++rb)
#pragma unroll
            for (int cb = 0; cb < NB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
        // Rows past the end of a ragged chunk are read as copies of its last row: they stay finite
        // and only ever produce rows of the result that are not stored or that meet zero weights.
        uint32_t xo[CI], so[MI];
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) xo[ni] = (uint32_t)min(ni * 16 + r, len - 1) * (uint32_t)ldx + g8;
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) so[ni] = (uint32_t)(ni * 16 + r) * kSnapTile + g8;
        typedef typename Atom<T>::Frag Frag;
        // a wave takes 64 columns at a time: the two halves of every 128-byte line are asked for by the
        // same wave in consecutive instructions
        for (int kk = 64 * w; kk < d; kk += 64 * NW) {
            Frag fx[2][CI], fy[2][CI], fs[2][MI];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int k0 = kk + 32 * hh;
#pragma unroll
                for (int ni = 0; ni < CI; ++ni) fx[hh][ni] = (HINT & kHintX) ? Atom<T>::load_nt(X + xo[ni] + k0) : Atom<T>::load(X + xo[ni] + k0);
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int k0 = kk + 32 * hh;
#pragma unroll
                for (int ni = 0; ni < CI; ++ni) fy[hh][ni] = (HINT & kHintY) ? Atom<T>::load_nt(Y + xo[ni] + k0) : Atom<T>::load(Y + xo[ni] + k0);
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int k0 = kk + 32 * hh;
#pragma unroll
                for (int ni = 0; ni < MI; ++ni) fs[hh][ni] = (HINT & kHintSt) ? Atom<T>::load_nt(St + so[ni] + snap_col<M>(k0)) : Atom<T>::load(St + so[ni] + snap_col<M>(k0));
            }
            __builtin_amdgcn_sched_barrier(0);
            if (GEN && phi) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                    for (int ni = 0; ni < CI; ++ni) {
                        if (phi & kHintX) swish_frag<T>(fx[hh][ni]);
                        if (phi & kHintY) swish_frag<T>(fy[hh][ni]);
                    }
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int rb = 0; rb < NW; ++rb) {
#pragma unroll
                    for (int cb = 0; cb <= rb; ++cb) Atom<T>::mma(acc[rb][cb], fx[hh][rb], fy[hh][cb]);
#pragma unroll
                    for (int ni = 0; ni < MI; ++ni) Atom<T>::mma(acc[rb][CI + ni], fx[hh][rb], fs[hh][ni]);
                }
        }
        GatePrep<M, Geo<T>::NT, C, GEN> gp;
        gp.load(g, gld, len, tid, sin, gate_tau);
        f32x4 own[NB];
        reduce_row_blocks<NW, NB, CI, RPR>(own, acc, Red, lane, w);
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) accA[ni] = own[ni];
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) accZ[ni] = own[CI + ni];
        gp.finish(Gs, Ss, ldg, tot, len, tid);
    }
    // causally masked X Y^T, as an operand
#pragma unroll
    for (int ni = 0; ni < CI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j, rr = ni * 16 + r;
            As[t * lda + rr] = from_f32<T>((ni <= w && rr <= t) ? accA[ni][j] : 0.f);
        }
    build_write_tiles<T, M, C>(Gs, Ss, ldg, Vt, ldv, Rb, tid);
    __syncthreads();
    unsafe = block_unsafe<M>(Gs, ldg, rowb, lane);
    // ---- earlier row blocks, through the end-referenced tile: `run` walks its reference from the chunk
    // start (where it is the inter-chunk term) to the start of this wave's block, one block at a time
    f32x4 run[MI];
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) run[ni] = accZ[ni];
    for (int bp = 0; bp < w; ++bp) {
        const typename Atom<T>::Frag16 a = Atom<T>::load16(As + (rowb + r) * lda + bp * 16 + g4);
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) {
            const float dec = Rb[bp * M + ni * 16 + r];
            run[ni] *= dec;
            const typename Atom<T>::Frag16 bfr = Atom<T>::load16(Vt + (ni * 16 + r) * ldv + bp * 16 + g4);
            Atom<T>::mma16(run[ni], a, bfr);
        }
    }
    // ---- this wave's own block: operand generated here, referenced to the block's start
    float gref[MI];
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) gref[ni] = rowb ? Gs[(rowb - 1) * ldg + ni * 16 + r] : 0.f;
    if (!unsafe) {
        const typename Atom<T>::Frag16 a = Atom<T>::load16(As + (rowb + r) * lda + rowb + g4);
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) {
            const int i = ni * 16 + r;
            typename Atom<T>::Frag16 bfr;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int kk = rowb + g4 + e;
                bfr[e] = from_f32<T>(Ss[kk * ldg + i] * __expf(fminf(gref[ni] - Gs[kk * ldg + i], kExpClamp)));
            }
            Atom<T>::mma16(run[ni], a, bfr);
        }
    }
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) {
        const int i = ni * 16 + r;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            const float G = Gs[t * ldg + i];
            float val = __expf(G - gref[ni]) * run[ni][j];
            if (unsafe) {
                float sum = 0.f;
                for (int rr = rowb; rr <= t; ++rr)
                    sum += to_f32(As[t * lda + rr]) * Ss[rr * ldg + i] * __expf(G - Gs[rr * ldg + i]);
                val += sum;
            }
            out[ni][j] = val;
        }
    }
}

// Eight consecutive floats of an LDS row (16-byte aligned).
__device__ __forceinline__ void lds_row8(float (&x)[8], const float *p)
{
    const f32x4 lo = *reinterpret_cast<const f32x4 *>(p);
    const f32x4 hi = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[e] = lo[e]; x[4 + e] = hi[e]; }
}

// The eight slots i0 .. i0+7 a lane contributes to a contraction over the (padded) slot axis,
// and whether they exist: with M < KM the padding lanes re-read the last eight real slots and
// are masked, so that no LDS read sits under a per-lane branch.
template <int M, int KM> struct SlotSpan {
    int i0;
    bool live;
    __device__ __forceinline__ SlotSpan(int k) : i0((M < KM) ? min(k, M - 8) : k), live((M >= KM) || (k < M)) {}
};

// Gate reference of row block rowb (cumulative log gate just before it) for slots i0 .. i0+7.
__device__ __forceinline__ void gate_ref8(float (&gref)[8], const float *Gs, int ldg, int rowb, int i0)
{
    lds_row8(gref, Gs + (rowb ? rowb - 1 : 0) * ldg + i0);
#pragma unroll
    for (int e = 0; e < 8; ++e) gref[e] = rowb ? gref[e] : 0.f;
}

// B fragment  b[e] = s_rr[i0+e] * exp(gref[e] - G_rr[i0+e])  (clamped; zero where !live).
template <typename T>
__device__ __forceinline__ typename Atom<T>::Frag write_frag(const float *Gs, const float *Ss, int ldg, int rr, int i0,
                                                             bool live, const float (&gref)[8])
{
    float sv[8], gv[8];
    lds_row8(sv, Ss + rr * ldg + i0);
    lds_row8(gv, Gs + rr * ldg + i0);
    typename Atom<T>::Frag b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x = sv[e] * __expf(fminf(gref[e] - gv[e], kExpClamp));
        b[e] = from_f32<T>(live ? x : 0.f);
    }
    return b;
}

// Row block w of the pair-weight matrix, for column blocks ni <= w:
//   acc[ni][j] = sum_i Wa[t][i] s_r[i] exp(G_t[i] - G_r[i]),  t = rowb + 4*(lane/16) + j, r = 16*ni + lane%16
// where the caller supplies Wa pre-multiplied by exp(G_t - Gref_w) as an LDS tile of T
// ([C][ldp], slots padded with zeros to KM).  Entries with r > t are returned as computed
// (the caller masks).  When the block is unsafe the diagonal atom is left at zero and the
// caller adds pair_weights_exact.
template <typename T, int M, int C, int KM>
__device__ __forceinline__ void pair_weights(f32x4 (&acc)[C / 16], const T *Wa, int ldp, const float *Gs,
                                             const float *Ss, int ldg, bool unsafe, int lane, int w)
{
    constexpr int CI = C / 16;
    const int r = lane & 15, g8 = (lane >> 4) * 8;
    const int rowb = 16 * w;
#pragma unroll
    for (int ni = 0; ni < CI; ++ni) acc[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < KM; k0 += 32) {
        const typename Atom<T>::Frag a = Atom<T>::load(Wa + (rowb + r) * ldp + k0 + g8);
        const SlotSpan<M, KM> sp(k0 + g8);
        float gref[8];
        gate_ref8(gref, Gs, ldg, rowb, sp.i0);
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) {
            if (ni > w || (unsafe && ni == w)) continue;   // wave-uniform
            const typename Atom<T>::Frag b = write_frag<T>(Gs, Ss, ldg, ni * 16 + r, sp.i0, sp.live, gref);
            Atom<T>::mma(acc[ni], a, b);
        }
    }
}

// Diagonal atom of the pair-weight matrix without factoring:
//   out[j] = sum_i Wf[t][i] s_r[i] exp(G_t[i] - G_r[i])   for r = rowb + lane%16 <= t, else 0
// Wf: LDS tile [C][ldw] of the ungated weights (fp32 or T).
template <int M, typename TW>
__device__ __forceinline__ f32x4 pair_weights_exact(const TW *Wf, int ldw, const float *Gs, const float *Ss, int ldg,
                                                    int lane, int rowb)
{
    const int r = lane & 15, g4 = (lane >> 4) * 4;
    const int rr = rowb + r;
    f32x4 out = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int t = rowb + g4 + j;
        if (rr > t) continue;
        float sum = 0.f;
        for (int i = 0; i < M; ++i)
            sum += to_f32(Wf[t * ldw + i]) * Ss[rr * ldg + i] * __expf(Gs[t * ldg + i] - Gs[rr * ldg + i]);
        out[j] = sum;
    }
    return out;
}

// Stores a C x ncols tile held in LDS (Os, row stride ldo) to global rows of `ld` elements,
// 8 elements per thread, rows >= len skipped.  NTS: with the non-temporal hint (final outputs).
template <typename T, bool NTS = false>
__device__ __forceinline__ void store_tile(T *dst, size_t ld, const T *Os, int ldo, int rows, int ncols, int len,
                                           int tid, int nthreads)
{
    const int vpr = ncols >> 3;
    for (int idx = tid; idx < rows * vpr; idx += nthreads) {
        const int t = idx / vpr, c = (idx - t * vpr) << 3;
        if (t >= len) continue;
        const T *s = Os + t * ldo + c;
        T *d = dst + (size_t)t * ld + c;
        if (NTS) {
            __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(s), reinterpret_cast<f32x4 *>(d));
            if (sizeof(T) == 4) __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(s + 4), reinterpret_cast<f32x4 *>(d + 4));
        } else {
            *reinterpret_cast<f32x4 *>(d) = *reinterpret_cast<const f32x4 *>(s);
            if (sizeof(T) == 4) *reinterpret_cast<f32x4 *>(d + 4) = *reinterpret_cast<const f32x4 *>(s + 4);
        }
    }
}

// Softmax over the M slots of each chunk row, from scores in global memory into an fp32
// LDS tile Pf[C][ld]; four threads per row.  Rows >= len get zeros.  Also copies a second
// [len][M] array (same global layout) into Df.  Needs NT = 4*C threads.  load() only issues
// the (clamped, unconditional) loads, so that it can be called ahead of other work.
template <int M, int C> struct SoftmaxRows {
    static constexpr int Q = M / 4;
    float zv[Q], dv[Q];
    __device__ __forceinline__ void load(const float *z, const float *dz, size_t gld, int len, int tid)
    {
        const int t = tid >> 2, sub = tid & 3;
        const size_t row = (size_t)min(t, len - 1) * gld;
#pragma unroll
        for (int u = 0; u < Q; ++u) zv[u] = z[row + sub + 4 * u];
#pragma unroll
        for (int u = 0; u < Q; ++u) dv[u] = dz[row + sub + 4 * u];
    }
    __device__ __forceinline__ void finish(float *Pf, float *Df, int ld, int len, int tid)
    {
        const int t = tid >> 2, sub = tid & 3;
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < Q; ++u) mx = fmaxf(mx, zv[u]);
        mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
        float sum = 0.f;
#pragma unroll
        for (int u = 0; u < Q; ++u) { zv[u] = __expf(zv[u] - mx); sum += zv[u]; }
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        const float inv = (t < len) ? 1.f / sum : 0.f;
#pragma unroll
        for (int u = 0; u < Q; ++u) Pf[t * ld + sub + 4 * u] = zv[u] * inv;
#pragma unroll
        for (int u = 0; u < Q; ++u) Df[t * ld + sub + 4 * u] = (t < len) ? dv[u] : 0.f;
    }
    // The same with an element-wise read-out p = f(z) in place of the softmax.
    __device__ __forceinline__ void finish_elementwise(int readout, float *Pf, float *Df, int ld, int len, int tid)
    {
        const int t = tid >> 2, sub = tid & 3;
#pragma unroll
        for (int u = 0; u < Q; ++u) Pf[t * ld + sub + 4 * u] = (t < len) ? readout_value(readout, zv[u]) : 0.f;
#pragma unroll
        for (int u = 0; u < Q; ++u) Df[t * ld + sub + 4 * u] = (t < len) ? dv[u] : 0.f;
    }
};

}  // namespace gsa
