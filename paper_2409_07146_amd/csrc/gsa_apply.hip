// The wide contractions of Gated Slot Attention: every output of width d_k or d_v is
//
//     out[C x cols] = A_tok[C x C] X[C x cols]  +  A_slot[C x m] St[m x cols]
//
// per (chunk, head): the intra-chunk term contracts a small token-by-token matrix with a token
// tensor of the chunk, the inter-chunk term contracts a small token-by-slot matrix with a slot
// memory (paper, Appendix A, Eq. (gla-chunk): intra and inter parts).  The small matrices are
// produced by the chunk kernels and are tiny next to the [tokens x d] tensors, so this kernel
// is where the bytes move:
//
//     forward  o  = A2   V  + (p e^G)      Vt_start
//     backward dq = Bm   K  + (dz e^G)     Kt_start      (Bm and dz carry the softmax scale)
//              dk = Bm^T Q  + (s e^{G_C-G}) E_k
//              dv = A2^T dO + (s e^{G_C-G}) E_v
//
// One workgroup per (column slice, chunk, head, output).  Both wide operands arrive with the
// column index fastest (token rows; slot rows inside the tiles the scans store) while the
// matrix cores want the contraction index fastest, so each is loaded with whole-row 16-byte
// loads and transposed on its way into LDS (XOR-swizzled so the transposing stores spread over
// all banks).  One LDS tile serves the slot operand, then the token operand, then the output
// tile; the two small matrices are staged once per workgroup.  ~37 KB of LDS per workgroup, so
// several workgroups are resident per CU and their loads overlap.
//
// With the feature map on q, k, v (Section 3.3; the PHI instantiation) the token operand gets
// phi(x) = x sigmoid(x) on its way into LDS where it is one of q, k, v, and the three backward
// outputs leave multiplied by phi'(raw) of the tensor they are the gradient of.
#include "gsa_chunk.h"
#include "gsa_launch.h"

namespace gsa {

template <typename T> struct ApplyOne {
    const T *A_tok;       // [chunk][H][C][C]
    const T *A_slot;      // [chunk][H][C][KM]
    const T *xtok;        // [tokens][H][d]
    const T *xslot;       // record base + offset of the part: M slots x d columns per (chunk, head), tiled
    long long xs_stride;  // elements per (chunk, head) record
    T *out;               // [tokens][H][d]
    int d;
    bool phi_tok;         // feature map on xtok on its way into LDS
    const T *raw;         // [tokens][H][d] or NULL: out leaves multiplied by the feature map's slope at raw
    T *act;               // output epilogue (EPI): Swish(out) [tokens][H][d], or NULL
    float *ssq;           // output epilogue (EPI): [tokens][H][slices] sums of squares of act over each column slice, or NULL
};
template <typename T> struct ApplyArgs { ApplyOne<T> one[3]; };

template <typename T, int M> struct ApplyLds {
    static constexpr int C = Geo<T>::C;
    static constexpr int PAD = Atom<T>::kPad;
    static constexpr int NS = (sizeof(T) == 2) ? 128 : 64;
    static constexpr int KM = (M < 32) ? 32 : M;
    static constexpr int lda = C + PAD, ldo = NS + PAD, lds = KM + PAD, ldm = M + PAD;
    static constexpr size_t szX = sizeof(T) * NS * (lda > ldm ? lda : ldm), szO = sizeof(T) * C * ldo;
    static constexpr size_t oAt = szX > szO ? szX : szO;          // A_tok  [C][lda]
    static constexpr size_t oAs = oAt + sizeof(T) * C * lda;      // A_slot [C][lds]
    static constexpr size_t bytes = oAs + sizeof(T) * C * lds;
};

// PHI: compiled with the feature-map options (ApplyOne::phi_tok, ApplyOne::raw); the plain calls run
// PHI = false, where those fields are ignored.
// EPI: the layer's output epilogue (Section 3.3: the layer applies RMSNorm(Swish(.)) to the operator's
// output).  The output tile leaves as it is (when ApplyOne::out is given) and as act = Swish(out), computed
// from the stored (rounded) out; the sum of squares of the stored act over this workgroup's columns goes to
// ssq[token][head][slice], so that the norm that follows needs no pass of its own over the tensor for its
// statistic (it adds the slices' partial sums and scales).  Plain calls run EPI = false.
template <typename T, int M, bool PHI, bool EPI>
__global__ __launch_bounds__(Geo<T>::NT) void apply_kernel(ChunkMap cm, int H, ApplyArgs<T> args)
{
    using L = ApplyLds<T, M>;
    constexpr int C = Geo<T>::C, NT = Geo<T>::NT, NW = Geo<T>::NW;
    constexpr int KM = (M < 32) ? 32 : M;
    constexpr int CI = C / 16, NIo = L::NS / (16 * NW);
    __shared__ __align__(16) unsigned char smem[L::bytes];
    T *XT = reinterpret_cast<T *>(smem);
    T *Os = reinterpret_cast<T *>(smem);

    // XCD-aware placement: consecutive workgroup ids go round-robin over the 8 XCDs, each with its own
    // L2.  The column slices of one (chunk, head, output) share the two small matrices, so they are
    // given ids that land on the same XCD (each XCD takes a contiguous range of logical ids); without
    // this every slice fetches its own copy through a different L2.
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    {
        const unsigned nx = gridDim.x, ny = gridDim.y, total = nx * ny * gridDim.z;
        if ((total & 7u) == 0) {
            unsigned lin = blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z);
            lin = (lin & 7u) * (total >> 3) + (lin >> 3);
            bx = lin % nx;
            by = (lin / nx) % ny;
            bz = lin / (nx * ny);
            if (PHI) {
                // the outputs of one (chunk, head, slice) next to each other as well: the dq workgroup's
                // token tile (k) is the dk workgroup's raw tile and the other way round, so the second
                // of them finds it in this XCD's L2
                const unsigned nout = gridDim.z / (unsigned)H;
                const unsigned which = (lin / nx) % nout, rest = lin / (nx * nout);
                by = rest % ny;
                bz = (rest / ny) + which * (unsigned)H;
            }
        }
    }
    ChunkInfo ci;
    if (!chunk_lookup(cm, by, ci)) return;
    const int h = bz % H, which = bz / H;
    const ApplyOne<T> &a = args.one[which];
    const int cs = bx * L::NS;
    if (cs >= a.d) return;
    const int ncols = min(L::NS, a.d - cs);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g4 = (lane >> 4) * 4, g8 = (lane >> 4) * 8;
    const size_t ch = (size_t)by * H + h;
    const size_t tokh = (size_t)ci.tok0 * H + h;
    const int wcol = 16 * NIo * w;
    const bool active = wcol < ncols;

    // every global load of the workgroup is issued here, in the order the data is needed; the two wide
    // operands are this workgroup's alone and the output is final, so all three stream (non-temporal):
    // measured 112 -> 103 us for the backward launch, and the chunk kernels running next find more of
    // their own data still cached
    TokTile<T, M, L::NS, NT> ts;   // the slot memory's column slice, rows = slots
    ts.template load_snapshot<true>(a.xslot + ch * a.xs_stride, cs, ncols, tid);
    TokTile<T, C, L::NS, NT> tt;   // the token tensor's column slice
    tt.template load<!PHI>(a.xtok + tokh * a.d + cs, (size_t)H * a.d, ci.len, ncols, tid);   // PHI: shared, see above
    // the raw values under this workgroup's output tile, in the thread mapping of the final store
    constexpr int OV = C * (L::NS / 8), OPER = (OV + NT - 1) / NT;
    Raw8<T> rawv[PHI ? OPER : 1];
    const bool chain = PHI && a.raw != nullptr;
    if (chain) {
        const int vpr = ncols >> 3;
#pragma unroll
        for (int u = 0; u < OPER; ++u) {
            const int idx = min(tid + u * NT, C * vpr - 1), t = min(idx / vpr, ci.len - 1), c = (idx - (idx / vpr) * vpr) << 3;
            rawv[PHI ? u : 0].load(a.raw + tokh * a.d + cs + (size_t)t * H * a.d + c);
        }
    }
    // the two small matrices go through LDS: every wave needs all of both
    T *Ats = reinterpret_cast<T *>(smem + L::oAt), *Ass = reinterpret_cast<T *>(smem + L::oAs);
    {
        const T *At = a.A_tok + ch * C * C, *As = a.A_slot + ch * C * KM;
        constexpr int VT = C * C / 8, VS = C * KM / 8;
        Raw8<T> xt[(VT + NT - 1) / NT], xs[(VS + NT - 1) / NT];
#pragma unroll
        for (int u = 0; u < (VT + NT - 1) / NT; ++u) xt[u].load(At + (size_t)min(tid + u * NT, VT - 1) * 8);
#pragma unroll
        for (int u = 0; u < (VS + NT - 1) / NT; ++u) xs[u].load(As + (size_t)min(tid + u * NT, VS - 1) * 8);
#pragma unroll
        for (int u = 0; u < (VT + NT - 1) / NT; ++u) {
            const int idx = tid + u * NT, t = idx / (C / 8), c8 = (idx - t * (C / 8)) * 8;
            if (idx < VT) xt[u].store(Ats + t * L::lda + c8);
        }
#pragma unroll
        for (int u = 0; u < (VS + NT - 1) / NT; ++u) {
            const int idx = tid + u * NT, t = idx / (KM / 8), c8 = (idx - t * (KM / 8)) * 8;
            if (idx < VS) xs[u].store(Ass + t * L::lds + c8);
        }
    }
    ts.store_transposed(XT, L::ldm, ncols, tid);
    __syncthreads();
    f32x4 acc[CI][NIo];
    zero_acc(acc);
    if (active) {
#pragma unroll
        for (int ks = 0; ks < KM / 32; ++ks) {
            typename Atom<T>::Frag af[CI], bf[NIo];
#pragma unroll
            for (int mi = 0; mi < CI; ++mi) af[mi] = Atom<T>::load(Ass + (mi * 16 + r) * L::lds + ks * 32 + g8);
            const SlotSpan<M, KM> sp(ks * 32 + g8);   // padded slots re-read real ones and are zeroed
#pragma unroll
            for (int ni = 0; ni < NIo; ++ni) {
                const typename Atom<T>::Frag f = Atom<T>::load(XT + xt_off<M>(wcol + ni * 16 + r, sp.i0, L::ldm));
                const typename Atom<T>::Frag z = Atom<T>::zero();
                bf[ni] = sp.live ? f : z;
            }
#pragma unroll
            for (int mi = 0; mi < CI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NIo; ++ni) Atom<T>::mma(acc[mi][ni], af[mi], bf[ni]);
        }
    }
    __syncthreads();   // the slot tile is dead: the token tile takes its place
    if (PHI && a.phi_tok) tt.template store_transposed<true>(XT, L::lda, ncols, tid);
    else tt.store_transposed(XT, L::lda, ncols, tid);
    __syncthreads();
    if (active) {
#pragma unroll
        for (int k0 = 0; k0 < C; k0 += 32) {
            typename Atom<T>::Frag af[CI], bf[NIo];
#pragma unroll
            for (int mi = 0; mi < CI; ++mi) af[mi] = Atom<T>::load(Ats + (mi * 16 + r) * L::lda + k0 + g8);
#pragma unroll
            for (int ni = 0; ni < NIo; ++ni)
                bf[ni] = Atom<T>::load(XT + xt_off<C>(wcol + ni * 16 + r, k0 + g8, L::lda));
#pragma unroll
            for (int mi = 0; mi < CI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NIo; ++ni) Atom<T>::mma(acc[mi][ni], af[mi], bf[ni]);
        }
    }
    __syncthreads();   // the token tile is dead: its space becomes the output tile
    if (active) {
#pragma unroll
        for (int mi = 0; mi < CI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NIo; ++ni)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    Os[(mi * 16 + g4 + j) * L::ldo + wcol + ni * 16 + r] = from_f32<T>(acc[mi][ni][j]);
    }
    __syncthreads();
    if (chain) {
        // out = tile * phi'(raw): same walk as store_tile, one 8-element piece per thread and step
        const int vpr = ncols >> 3;
        T *dst = a.out + tokh * a.d + cs;
#pragma unroll
        for (int u = 0; u < OPER; ++u) {
            const int idx = tid + u * NT, t = idx / vpr, c = (idx - t * vpr) << 3;
            if (idx < C * vpr && t < ci.len) {
                Raw8<T> x;
                x.load(Os + t * L::ldo + c);
                Raw8<T> y;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    y.set(e, from_f32<T>((float)x.get(e) * swish_slope((float)rawv[PHI ? u : 0].get(e))));
                y.store_nt(dst + (size_t)t * H * a.d + c);
            }
        }
        return;
    }
    if (EPI) {
        // same walk as store_tile: consecutive threads take consecutive 8-element pieces of a row, so the
        // vpr threads of a row are neighbours in one wave and meet by shuffles
        const int vpr = ncols >> 3;   // 8 or 16 pieces per row
        const int nslices = (a.d + L::NS - 1) / L::NS;
        constexpr int OV = C * (L::NS / 8), OPER = (OV + NT - 1) / NT;
#pragma unroll
        for (int u = 0; u < OPER; ++u) {
            const int idx = tid + u * NT, t = idx / vpr, c = (idx - t * vpr) << 3;
            const bool live = idx < C * vpr && t < ci.len;
            Raw8<T> x;
            x.load(Os + min(t, C - 1) * L::ldo + c);
            Raw8<T> y;
            float sq = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const T ye = from_f32<T>(swish_value((float)x.get(e)));
                y.set(e, ye);
                sq += (float)ye * (float)ye;
            }
            sq = live ? sq : 0.f;
            for (int o = 1; o < vpr; o <<= 1) sq += __shfl_xor(sq, o, 64);
            if (live) {
                const size_t off = tokh * a.d + cs + (size_t)t * H * a.d + c;
                if (a.out) x.store_nt(a.out + off);
                if (a.act) y.store_nt(a.act + off);
                if (a.ssq && c == 0) a.ssq[(tokh + (size_t)t * H) * nslices + bx] = sq;
            }
        }
        return;
    }
    store_tile<T, true>(a.out + tokh * a.d + cs, (size_t)H * a.d, Os, L::ldo, C, ncols, ci.len, tid, NT);
}

int apply_slice_cols(int dtype) { return dtype == 0 ? ApplyLds<float, 64>::NS : ApplyLds<bf16_t, 64>::NS; }

template <typename T, int M>
static hipError_t launch_apply_tm(const Plan &pl, const Work &w, const ApplyIo *io, int n, int slot, hipStream_t st)
{
    const ChunkMap cm = make_chunk_map(pl, w);
    ApplyArgs<T> args;
    int dmax = 0;
    for (int i = 0; i < 3; ++i) {
        const ApplyIo &s = io[i < n ? i : 0];
        ApplyOne<T> &o = args.one[i];
        o.A_tok = static_cast<const T *>(s.A_tok);
        o.A_slot = static_cast<const T *>(s.A_slot);
        o.xtok = static_cast<const T *>(s.xtok);
        o.xslot = static_cast<const T *>(s.xslot_rec) + s.xslot_off;
        o.xs_stride = s.xslot_stride;
        o.out = static_cast<T *>(s.out);
        o.d = s.d;
        o.phi_tok = s.phi_tok;
        o.raw = static_cast<const T *>(s.raw);
        o.act = static_cast<T *>(s.act);
        o.ssq = s.ssq;
        if (i < n && s.d > dmax) dmax = s.d;
    }
    constexpr int NS = ApplyLds<T, M>::NS;
    dim3 grid((dmax + NS - 1) / NS, pl.chunk_slots, pl.H * n);
    KernelTimer kt(slot, st);
    const bool epi = io[0].act != nullptr || io[0].ssq != nullptr;   // forward only
    if (epi && pl.phi) hipLaunchKernelGGL((apply_kernel<T, M, true, true>), grid, dim3(Geo<T>::NT), 0, st, cm, pl.H, args);
    else if (epi) hipLaunchKernelGGL((apply_kernel<T, M, false, true>), grid, dim3(Geo<T>::NT), 0, st, cm, pl.H, args);
    else if (pl.phi) hipLaunchKernelGGL((apply_kernel<T, M, true, false>), grid, dim3(Geo<T>::NT), 0, st, cm, pl.H, args);
    else hipLaunchKernelGGL((apply_kernel<T, M, false, false>), grid, dim3(Geo<T>::NT), 0, st, cm, pl.H, args);
    return hipGetLastError();
}

hipError_t launch_apply(const Plan &pl, const Work &w, const ApplyIo *io, int n, int slot, hipStream_t st)
{
#define GSA_APPLY(T)                                                        \
    switch (pl.m) {                                                         \
    case 16: return launch_apply_tm<T, 16>(pl, w, io, n, slot, st);         \
    case 32: return launch_apply_tm<T, 32>(pl, w, io, n, slot, st);         \
    case 128: return launch_apply_tm<T, 128>(pl, w, io, n, slot, st);         \
    default: return launch_apply_tm<T, 64>(pl, w, io, n, slot, st);         \
    }
    if (pl.dtype == 0) { GSA_APPLY(float) }
    GSA_APPLY(bf16_t)
#undef GSA_APPLY
}

}  // namespace gsa
