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

// For this wave's row block (rows t = rowb .. rowb+15), in D layout (lane holds slot
// i = 16*ni + lane%16, rows t = rowb + 4*(lane/16) + j):
//
//   out[ni][j] = exp(G_t[i]) * <X_t, St[i]>  +  sum_{r<=t} <X_t, Y_r> s_r[i] exp(G_t[i]-G_r[i])
//
// i.e. the inter-chunk plus intra-chunk parts of one gated pass whose gate sits on the
// slot side (pass 1 of Eq. (gsa-2pass) with X=q, Y=k, St=Kt; its mirror in the backward
// with X=dO, Y=v, St=Vt).  X, Y: [len][d] rows in global memory (row stride ldx elements);
// St: [M][d] rows of T (stride ldst).  The contraction over d reads its operand fragments
// straight from global memory (each lane 16 bytes of one row; no LDS, no barriers), so the
// loads of many k-steps and of several resident workgroups are in flight together.
// LDS: Gs, Ss filled by gate_prep; As [C][lda] is left holding the causally masked X Y^T
// rounded to T.  All threads of the workgroup must call it.
template <typename T, int M, int C>
__device__ __forceinline__ void gated_scores(float (&out)[M / 16][4], bool &unsafe, const float *Gs, const float *Ss,
                                             int ldg, T *As, int lda, const T *X, const T *Y, size_t ldx, int d,
                                             const T *St, size_t ldst, int len, int tid)
{
    constexpr int MI = M / 16, CI = C / 16;
    const int lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4, g8 = (lane >> 4) * 8;
    const int rowb = 16 * w;

    f32x4 accA[CI], accZ[MI];
#pragma unroll
    for (int ni = 0; ni < CI; ++ni) accA[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) accZ[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        // Rows past the end of a ragged chunk are read as copies of its last row: they stay finite
        // and only ever produce rows of the result that are not stored or that meet zero weights.
        const T *xa = X + (size_t)min(rowb + r, len - 1) * ldx + g8;
        const T *yb[CI], *sb[MI];
#pragma unroll
        for (int ni = 0; ni < CI; ++ni) yb[ni] = Y + (size_t)min(ni * 16 + r, len - 1) * ldx + g8;
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) sb[ni] = St + (size_t)(ni * 16 + r) * ldst + g8;
        typedef typename Atom<T>::Frag Frag;
        Frag a0, a1, y0[CI], y1[CI], s0[MI], s1[MI];
        auto fetch = [&](int k0, Frag &fa, Frag (&fy)[CI], Frag (&fs)[MI]) {
            fa = Atom<T>::load(xa + k0);
#pragma unroll
            for (int ni = 0; ni < CI; ++ni) fy[ni] = Atom<T>::load(yb[ni] + k0);
#pragma unroll
            for (int ni = 0; ni < MI; ++ni) fs[ni] = Atom<T>::load(sb[ni] + k0);
        };
        auto multiply = [&](const Frag &fa, const Frag (&fy)[CI], const Frag (&fs)[MI]) {
#pragma unroll
            for (int ni = 0; ni < CI; ++ni) Atom<T>::mma(accA[ni], fa, fy[ni]);
#pragma unroll
            for (int ni = 0; ni < MI; ++ni) Atom<T>::mma(accZ[ni], fa, fs[ni]);
        };
        // two register sets: the loads of the next 32 columns are in flight while these multiply
        fetch(0, a0, y0, s0);
        for (int k0 = 0; k0 < d; k0 += 64) {   // d is a multiple of 64
            fetch(k0 + 32, a1, y1, s1);
            multiply(a0, y0, s0);
            if (k0 + 64 < d) fetch(k0 + 64, a0, y0, s0);
            multiply(a1, y1, s1);
        }
    }
    // causally masked X Y^T, as an operand
#pragma unroll
    for (int ni = 0; ni < CI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j, rr = ni * 16 + r;
            As[t * lda + rr] = from_f32<T>((ni <= w && rr <= t) ? accA[ni][j] : 0.f);
        }
    __syncthreads();
    unsafe = block_unsafe<M>(Gs, ldg, rowb, lane);
    const int kend = unsafe ? rowb : rowb + 16;   // tokens the factored contraction covers
    f32x4 accI[MI];
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) accI[ni] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < kend; k0 += 32) {
        const typename Atom<T>::Frag a = Atom<T>::load(As + (rowb + r) * lda + k0 + g8);
#pragma unroll
        for (int ni = 0; ni < MI; ++ni) {
            const int i = ni * 16 + r;
            const float gref = rowb ? Gs[(rowb - 1) * ldg + i] : 0.f;
            typename Atom<T>::Frag b;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int kk = k0 + g8 + e;
                float val = 0.f;
                if (kk < kend) val = Ss[kk * ldg + i] * __expf(fminf(gref - Gs[kk * ldg + i], kExpClamp));
                b[e] = from_f32<T>(val);
            }
            Atom<T>::mma(accI[ni], a, b);
        }
    }
#pragma unroll
    for (int ni = 0; ni < MI; ++ni) {
        const int i = ni * 16 + r;
        const float gref = rowb ? Gs[(rowb - 1) * ldg + i] : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = rowb + g4 + j;
            const float G = Gs[t * ldg + i];
            float val = __expf(G) * accZ[ni][j] + __expf(G - gref) * accI[ni][j];
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
                    const float gref = rowb ? Gs[(rowb - 1) * ldg + i] : 0.f;
                    val = Ss[rr * ldg + i] * __expf(fminf(gref - Gs[rr * ldg + i], kExpClamp));
                }
                b[e] = from_f32<T>(val);
            }
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
// 8 elements per thread, rows >= len skipped.
template <typename T>
__device__ __forceinline__ void store_tile(T *dst, size_t ld, const T *Os, int ldo, int rows, int ncols, int len,
                                           int tid, int nthreads)
{
    const int vpr = ncols >> 3;
    for (int idx = tid; idx < rows * vpr; idx += nthreads) {
        const int t = idx / vpr, c = (idx - t * vpr) << 3;
        if (t >= len) continue;
        const T *s = Os + t * ldo + c;
        T *d = dst + (size_t)t * ld + c;
        *reinterpret_cast<f32x4 *>(d) = *reinterpret_cast<const f32x4 *>(s);
        if (sizeof(T) == 4) *reinterpret_cast<f32x4 *>(d + 4) = *reinterpret_cast<const f32x4 *>(s + 4);
    }
}

// Softmax over the M slots of each chunk row, from scores in global memory into an fp32
// LDS tile Pf[C][ld]; four threads per row.  Rows >= len get zeros.  Optionally copies a
// second [len][M] array (same global layout) into Df.  Needs NT = 4*C threads.
template <int M, int C>
__device__ __forceinline__ void softmax_rows(float *Pf, float *Df, int ld, const float *z, const float *dz, size_t gld,
                                             int len, int tid)
{
    constexpr int Q = M / 4;
    const int t = tid >> 2, sub = tid & 3;
    float zv[Q];
    float mx = -INFINITY;
    const size_t row = (size_t)min(t, len - 1) * gld;   // clamped: the load is unconditional
#pragma unroll
    for (int u = 0; u < Q; ++u) {
        zv[u] = z[row + sub + 4 * u];
        mx = fmaxf(mx, zv[u]);
    }
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
    if (Df) {
        float dv[Q];
#pragma unroll
        for (int u = 0; u < Q; ++u) dv[u] = dz[row + sub + 4 * u];
#pragma unroll
        for (int u = 0; u < Q; ++u) Df[t * ld + sub + 4 * u] = (t < len) ? dv[u] : 0.f;
    }
}

}  // namespace gsa
