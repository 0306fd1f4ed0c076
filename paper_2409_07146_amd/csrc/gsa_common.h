// Device-side building blocks shared by the libgsa kernels (gfx950 / CDNA4, wave64).
//
// Everything here is written in terms of one matrix-core atom: a 16x16 fp32
// accumulator tile updated with a depth-32 contraction.  For bf16 operands that
// is one v_mfma_f32_16x16x32_bf16; for fp32 operands it is eight
// v_mfma_f32_16x16x4_f32.  Both read their operands as "8 consecutive k per
// lane" fragments from LDS tiles stored contraction-index-fastest, so every
// kernel is written once and instantiated for both element types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gsa_layout.h"

namespace gsa {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;
constexpr int kSub = 16;            // row block inside a chunk sharing one gate reference
constexpr float kGateFloor = -30.f; // log-gates below this are treated as this
constexpr float kExpClamp = 80.f;   // largest exponent a factored gate may carry in fp32

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }

// ----------------------------------------------------------------------------
// Matrix-core atom.
//   A fragment: lane l holds A[row = l%16][k = 8*(l/16) + e], e = 0..7
//   B fragment: lane l holds B[k = 8*(l/16) + e][col = l%16]
//   D tile    : lane l holds D[row = 4*(l/16) + j][col = l%16], j = 0..3
// ----------------------------------------------------------------------------
template <typename T> struct Atom;

template <> struct Atom<bf16_t> {
    typedef bf16x8 Frag;
    static constexpr int kPad = 8;  // elements of padding that keep rows 16-byte aligned
    __device__ static __forceinline__ Frag load(const bf16_t *p) { return *reinterpret_cast<const Frag *>(p); }
    __device__ static __forceinline__ Frag load_nt(const bf16_t *p) { return __builtin_nontemporal_load(reinterpret_cast<const Frag *>(p)); }
    __device__ static __forceinline__ Frag zero() { Frag f; for (int e = 0; e < 8; ++e) f[e] = (bf16_t)0.f; return f; }
    __device__ static __forceinline__ void mma(f32x4 &c, const Frag &a, const Frag &b) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    // depth-16 form: lane l holds row l%16 and the four contraction indices 4*(l/16) .. +3
    typedef bf16x4 Frag16;
    __device__ static __forceinline__ Frag16 load16(const bf16_t *p) { return *reinterpret_cast<const Frag16 *>(p); }
    __device__ static __forceinline__ void mma16(f32x4 &c, const Frag16 &a, const Frag16 &b) {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        c = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
    }
};

template <> struct Atom<float> {
    typedef f32x8 Frag;
    static constexpr int kPad = 4;
    __device__ static __forceinline__ Frag load(const float *p) {
        const f32x4 lo = *reinterpret_cast<const f32x4 *>(p);
        const f32x4 hi = *reinterpret_cast<const f32x4 *>(p + 4);
        Frag f;
        f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3];
        f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3];
        return f;
    }
    __device__ static __forceinline__ Frag load_nt(const float *p) {
        const f32x4 lo = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        const f32x4 hi = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + 4));
        Frag f;
        f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3];
        f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3];
        return f;
    }
    __device__ static __forceinline__ Frag zero() { Frag f; for (int e = 0; e < 8; ++e) f[e] = 0.f; return f; }
    __device__ static __forceinline__ void mma(f32x4 &c, const Frag &a, const Frag &b) {
        // instruction e contracts k = {e, 8+e, 16+e, 24+e}: lane group l/16 supplies k = 8*(l/16)+e
#pragma unroll
        for (int e = 0; e < 8; ++e) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], c, 0, 0, 0);
    }
    // depth-16 form: lane l holds row l%16 and the four contraction indices 4*(l/16) .. +3
    typedef f32x4 Frag16;
    __device__ static __forceinline__ Frag16 load16(const float *p) { return *reinterpret_cast<const Frag16 *>(p); }
    __device__ static __forceinline__ void mma16(f32x4 &c, const Frag16 &a, const Frag16 &b) {
#pragma unroll
        for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], c, 0, 0, 0);
    }
};

// Chunk geometry per element type: one wave per 16-token row block.  fp32 tiles are
// twice as large in LDS, so the fp32 path uses half the chunk.
template <typename T> struct Geo {
    static constexpr int C = (sizeof(T) == 2) ? 64 : 32;   // tokens per chunk
    static constexpr int NW = C / kSub;                    // waves per workgroup
    static constexpr int NT = NW * kWave;                  // threads per workgroup
};
inline int chunk_of_dtype(int dtype) { return dtype == 0 ? Geo<float>::C : Geo<bf16_t>::C; }

// acc[MI][NI] += A[16*mi + r][k] * B[16*ni + r][k] summed over k in [0,K), K a multiple of 32.
// A and B are LDS tiles stored [row][k] with row strides lda, ldb (elements).
template <typename T, int MI, int NI>
__device__ __forceinline__ void gemm_nt(f32x4 (&acc)[MI][NI], const T *A, int lda, const T *B, int ldb,
                                        int K, int lane)
{
    const int r = lane & 15, g8 = (lane >> 4) * 8;
    for (int k0 = 0; k0 < K; k0 += 32) {
        typename Atom<T>::Frag a[MI], b[NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) a[mi] = Atom<T>::load(A + (mi * 16 + r) * lda + k0 + g8);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) b[ni] = Atom<T>::load(B + (ni * 16 + r) * ldb + k0 + g8);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) Atom<T>::mma(acc[mi][ni], a[mi], b[ni]);
    }
}

template <int MI, int NI> __device__ __forceinline__ void zero_acc(f32x4 (&acc)[MI][NI])
{
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// ----------------------------------------------------------------------------
// Global -> LDS staging.  Sources are rows of `cols` elements (cols % 8 == 0),
// row r at src + r*gld.  Rows >= nvalid are filled with zeros.
// ----------------------------------------------------------------------------
template <typename Tin> struct Vec8;
template <> struct Vec8<bf16_t> {
    float v[8];
    __device__ __forceinline__ void load(const bf16_t *p) {
        const bf16x8 x = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (float)x[e];
    }
};
template <> struct Vec8<float> {
    float v[8];
    __device__ __forceinline__ void load(const float *p) {
        const f32x4 lo = *reinterpret_cast<const f32x4 *>(p);
        const f32x4 hi = *reinterpret_cast<const f32x4 *>(p + 4);
        v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
        v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
    }
};

template <typename T> __device__ __forceinline__ void store8(T *dst, const float (&v)[8]);
template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t *dst, const float (&v)[8]) {
    bf16x8 x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (bf16_t)v[e];
    *reinterpret_cast<bf16x8 *>(dst) = x;
}
template <> __device__ __forceinline__ void store8<float>(float *dst, const float (&v)[8]) {
    *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4 *>(dst + 4) = f32x4{v[4], v[5], v[6], v[7]};
}

// Non-temporal forms (load_nt / store_nt below and on the atom): for data a kernel touches once and
// nobody reads again soon.  Such traffic then streams through the caches instead of displacing lines
// that the co-resident workgroups or the next kernel still want.  Which accesses carry the hint was
// decided by measurement, access by access: the decode memories, the apply kernel's wide operands and
// outputs and the scans' token tiles gain; the chunk kernels' operands and the scans' snapshot stores
// (read back by the next kernel) lose.
// Eight elements held as loaded (no conversion): the unit of register prefetching.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
    bf16x8 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const bf16x8 *>(p); }
    __device__ __forceinline__ void store(bf16_t *p) const { *reinterpret_cast<bf16x8 *>(p) = v; }
    __device__ __forceinline__ void load_nt(const bf16_t *p) { v = __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(p)); }
    __device__ __forceinline__ void store_nt(bf16_t *p) const { __builtin_nontemporal_store(v, reinterpret_cast<bf16x8 *>(p)); }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)0.f;
    }
    __device__ __forceinline__ bf16_t get(int e) const { return v[e]; }
    __device__ __forceinline__ void set(int e, bf16_t x) { v[e] = x; }
    __device__ __forceinline__ void keep(bool live) {   // zero unless live, by register select
        bf16x8 z;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (bf16_t)0.f;
        v = live ? v : z;
    }
};
template <> struct Raw8<float> {
    f32x4 lo, hi;
    __device__ __forceinline__ void load(const float *p) {
        lo = *reinterpret_cast<const f32x4 *>(p);
        hi = *reinterpret_cast<const f32x4 *>(p + 4);
    }
    __device__ __forceinline__ void store(float *p) const {
        *reinterpret_cast<f32x4 *>(p) = lo;
        *reinterpret_cast<f32x4 *>(p + 4) = hi;
    }
    __device__ __forceinline__ void load_nt(const float *p) {
        lo = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        hi = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + 4));
    }
    __device__ __forceinline__ void store_nt(float *p) const {
        __builtin_nontemporal_store(lo, reinterpret_cast<f32x4 *>(p));
        __builtin_nontemporal_store(hi, reinterpret_cast<f32x4 *>(p + 4));
    }
    __device__ __forceinline__ void zero() { lo = f32x4{0.f, 0.f, 0.f, 0.f}; hi = lo; }
    __device__ __forceinline__ float get(int e) const { return e < 4 ? lo[e] : hi[e - 4]; }
    __device__ __forceinline__ void set(int e, float x) { if (e < 4) lo[e] = x; else hi[e - 4] = x; }
    __device__ __forceinline__ void keep(bool live) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        lo = live ? lo : z;
        hi = live ? hi : z;
    }
};

// four consecutive elements of one row, from fp32
__device__ __forceinline__ void store4(bf16_t *p, float a, float b, float c, float d)
{
    bf16x4 x;
    x[0] = (bf16_t)a; x[1] = (bf16_t)b; x[2] = (bf16_t)c; x[3] = (bf16_t)d;
    *reinterpret_cast<bf16x4 *>(p) = x;
}
__device__ __forceinline__ void store4(float *p, float a, float b, float c, float d)
{
    *reinterpret_cast<f32x4 *>(p) = f32x4{a, b, c, d};
}

// dst[r][c] = src[r][c]   (dst row stride ld)
template <typename T, typename Tin>
__device__ __forceinline__ void stage_rows(T *dst, int ld, const Tin *src, size_t gld, int rows, int cols,
                                           int nvalid, int tid, int nthreads)
{
    const int vpr = cols >> 3;
    for (int idx = tid; idx < rows * vpr; idx += nthreads) {
        const int r = idx / vpr, c = (idx - r * vpr) << 3;
        Vec8<Tin> x;
        if (r < nvalid) x.load(src + (size_t)r * gld + c);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x.v[e] = 0.f;
        }
        store8<T>(dst + r * ld + c, x.v);
    }
}

// dst[c][r] = src[r][c]   (dst row stride ld >= rows): the transposed view that lets a
// contraction over tokens read 8 consecutive tokens per lane.
template <typename T, typename Tin>
__device__ __forceinline__ void stage_cols(T *dst, int ld, const Tin *src, size_t gld, int rows, int cols,
                                           int nvalid, int tid, int nthreads)
{
    const int vpr = cols >> 3;
    for (int idx = tid; idx < rows * vpr; idx += nthreads) {
        // consecutive threads take consecutive 16-byte pieces of a row: global loads coalesce
        const int r = idx / vpr, c = (idx - r * vpr) << 3;
        Vec8<Tin> x;
        if (r < nvalid) x.load(src + (size_t)r * gld + c);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x.v[e] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[(c + e) * ld + r] = from_f32<T>(x.v[e]);
    }
}

// ----------------------------------------------------------------------------
// Chunk map: which tokens a chunk covers.  Batch form: arithmetic.  Packed form:
// a table the prepare kernel writes into the workspace.
// ----------------------------------------------------------------------------
struct ChunkMap {
    const int32_t *table;   // packed: [4 * n_chunk_slots] = {seq, tok0, len, index in seq}; batch: NULL
    const int32_t *seq_tab; // packed: [4 * n_seqs] = {first chunk id, number of chunks, first token, tokens}
    const int32_t *seg_base; // packed: [n_seqs + 1] running count of scan segments before each sequence
    int32_t T;              // batch: tokens per sequence
    int32_t chunk;          // tokens per chunk (C in Appendix A)
    int32_t chunks_per_seq; // batch: ceil(T / chunk)
    int32_t n_chunk_slots;  // upper bound on the number of chunks (grid size)
};

struct ChunkInfo { int seq, tok0, len, idx; };

__device__ __forceinline__ bool chunk_lookup(const ChunkMap &cm, int c, ChunkInfo &ci)
{
    if (cm.table) {
        ci.seq = cm.table[4 * c + 0];
        ci.tok0 = cm.table[4 * c + 1];
        ci.len = cm.table[4 * c + 2];
        ci.idx = cm.table[4 * c + 3];
        return ci.len > 0;
    }
    ci.seq = c / cm.chunks_per_seq;
    ci.idx = c - ci.seq * cm.chunks_per_seq;
    const int off = ci.idx * cm.chunk;
    ci.tok0 = ci.seq * cm.T + off;
    ci.len = min(cm.chunk, cm.T - off);
    return true;
}

// Which (chunk, head) a workgroup of a chunk-parallel kernel takes, for a grid of
// (n_chunk_slots, H) workgroups dispatched x-fastest.  Workgroups are handed out so that all
// sequences and heads advance through their chunks together, newest_first = from the last chunk
// of every sequence backwards: a kernel that follows a scan then starts on the snapshots the scan
// wrote last, which are the ones still sitting in the memory-side cache.
__device__ __forceinline__ void chunk_order(const ChunkMap &cm, int H, bool newest_first, int &chunk, int &head)
{
    const int b = blockIdx.y * gridDim.x + blockIdx.x;
    if (cm.table) {
        const int c = b / H;
        head = b - c * H;
        chunk = newest_first ? cm.n_chunk_slots - 1 - c : c;
        return;
    }
    const int n = cm.chunks_per_seq, per = (cm.n_chunk_slots / n) * H;   // per: (sequence, head) pairs
    const int rank = b / per, rem = b - rank * per;
    const int seq = rem / H;
    head = rem - seq * H;
    chunk = seq * n + (newest_first ? n - 1 - rank : rank);
}

// First chunk id, number of chunks and first token of sequence s.
__device__ __forceinline__ void seq_lookup(const ChunkMap &cm, int s, int &chunk0, int &nchunks, int &tok0, int &ntok)
{
    if (cm.seq_tab) {
        chunk0 = cm.seq_tab[4 * s + 0];
        nchunks = cm.seq_tab[4 * s + 1];
        tok0 = cm.seq_tab[4 * s + 2];
        ntok = cm.seq_tab[4 * s + 3];
    } else {
        chunk0 = s * cm.chunks_per_seq;
        nchunks = cm.chunks_per_seq;
        tok0 = s * cm.T;
        ntok = cm.T;
    }
}

// ----------------------------------------------------------------------------
// Gate preparation for one chunk (Algorithm 1, chunk_cumsum, plus the write
// intensity): from g[len][M] (global, row stride gld) fill
//   Gs[t][i] = sum_{j<=t} max(g_j[i], floor)      chunk-local inclusive cumulative log gate
//   Ss[t][i] = 1 - exp(g_t[i])                    write intensity (0 on padded rows)
// Rows t >= len are padded with g = 0.  Needs blockDim.x = NT threads, NT % M == 0,
// C % (NT/M) == 0, and `tot` scratch of NT floats.  Ends with a __syncthreads().
// ----------------------------------------------------------------------------
// log gate from a gate logit: logsigmoid(u) / tau = -(log(1 + exp(-|u|)) + max(-u, 0)) / tau, and its slope
__device__ __forceinline__ float log_gate_from_logit(float u, float tau)
{
    return -(log1pf(__expf(-fabsf(u))) + fmaxf(-u, 0.f)) / tau;
}
__device__ __forceinline__ float log_gate_slope(float u, float tau) { return 1.f / ((1.f + __expf(u)) * tau); }

// GEN: the general form, in which the write intensity may come from an array of its own
// (sin: [len][M] fp32, same layout as g; NULL = 1 - exp(g) as above), and the array g may hold gate
// LOGITS u instead of log gates: with tau > 0 the log gate is logsigmoid(u) / tau, the layer's gate
// alpha = sigmoid(W x)^(1/tau) of Section 3.3 (tau = 0: g is the log gate itself).
template <int M, int NT, int C, bool GEN = false> struct GatePrep {
    static constexpr int P = NT / M;     // token partitions
    static constexpr int TP = C / P;     // tokens per partition
    static_assert(NT % M == 0 && C % P == 0, "gate_prep partitioning");
    float gv[TP];
    float sv[GEN ? TP : 1];
    bool given = false;
    float tau = 0.f;
    // Issues the loads (rows clamped into the chunk).  May be called well before finish() so that
    // other work hides the latency.
    __device__ __forceinline__ void load(const float *g, size_t gld, int len, int tid, const float *sin = nullptr,
                                         float gate_tau = 0.f)
    {
        if (GEN) tau = gate_tau;
        const int i = tid % M, part = tid / M;
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) gv[tt] = g[(size_t)min(part * TP + tt, len - 1) * gld + i];
        if (GEN && sin) {   // uniform over the grid
            given = true;
#pragma unroll
            for (int tt = 0; tt < (GEN ? TP : 1); ++tt) sv[tt] = sin[(size_t)min(part * TP + tt, len - 1) * gld + i];
        }
    }
    // Fills Gs, Ss.  Contains barriers (all threads must call it) and ends with one.
    __device__ __forceinline__ void finish(float *Gs, float *Ss, int ldg, float *tot, int len, int tid) const
    {
        const int i = tid % M, part = tid / M;
        float run = 0.f;
#pragma unroll
        for (int tt = 0; tt < TP; ++tt) {
            const int t = part * TP + tt;
            float graw = gv[tt];
            if (GEN && tau > 0.f) graw = log_gate_from_logit(graw, tau);
            const float x = (t < len) ? fmaxf(graw, kGateFloor) : 0.f;
            run += x;
            Gs[t * ldg + i] = run;
            float sx = -expm1f(x);
            if (GEN && given) sx = sv[GEN ? tt : 0];
            Ss[t * ldg + i] = (t < len) ? sx : 0.f;
        }
        tot[part * M + i] = run;
        __syncthreads();
        float off = 0.f;
        for (int pp = 0; pp < part; ++pp) off += tot[pp * M + i];
        if (part > 0) {
#pragma unroll 4
            for (int tt = 0; tt < TP; ++tt) Gs[(part * TP + tt) * ldg + i] += off;
        }
        __syncthreads();
    }
};

template <int M, int NT, int C, bool GEN = false>
__device__ __forceinline__ void gate_prep(float *Gs, float *Ss, int ldg, float *tot, const float *g, size_t gld,
                                          int len, int tid, const float *sin = nullptr, float gate_tau = 0.f)
{
    GatePrep<M, NT, C, GEN> gp;
    gp.load(g, gld, len, tid, sin, gate_tau);
    gp.finish(Gs, Ss, ldg, tot, len, tid);
}

// ----------------------------------------------------------------------------
// Read-outs: how the slot scores z become the read weights p.  Softmax over the slots is the
// method's own (Eq. (gsa)); the element-wise ones are the ablations of Section 4 (no softmax,
// Swish, ReLU, ReLU squared).  Values match gsa_readout in the C header.
// ----------------------------------------------------------------------------
enum Readout { kReadSoftmax = 0, kReadIdentity = 1, kReadSwish = 2, kReadRelu = 3, kReadRelu2 = 4 };

__device__ __forceinline__ float readout_value(int ro, float z)
{
    const float sg = 1.f / (1.f + __expf(-z)), zp = fmaxf(z, 0.f);
    return ro == kReadIdentity ? z : ro == kReadSwish ? z * sg : ro == kReadRelu ? zp : zp * zp;
}
__device__ __forceinline__ float readout_slope(int ro, float z)
{
    const float sg = 1.f / (1.f + __expf(-z));
    return ro == kReadIdentity ? 1.f : ro == kReadSwish ? sg + z * sg * (1.f - sg) : ro == kReadRelu ? (z > 0.f ? 1.f : 0.f)
                                                                                               : 2.f * fmaxf(z, 0.f);
}

// ----------------------------------------------------------------------------
// Feature map on q, k, v (Section 3.3: the layer feeds phi(W x) with phi = Swish into the operator).
// With the option on, the q, k, v arguments hold the raw projections and every kernel applies
// phi(x) = x sigmoid(x) to what it has just loaded, in registers: the values are rounded to the I/O
// type once more (they are matrix-core operands), and dq, dk, dv leave multiplied by the slope at
// the raw value.  The arithmetic runs under the loads that are still in flight, which is what makes
// this cheaper than a pass of its own over the three tensors.
// ----------------------------------------------------------------------------
__device__ __forceinline__ float swish_value(float x) { return x * __builtin_amdgcn_rcpf(1.f + __expf(-x)); }
__device__ __forceinline__ float swish_slope(float x)
{
    const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-x));
    return sg * (1.f + x * (1.f - sg));
}
template <typename T> __device__ __forceinline__ void swish_frag(typename Atom<T>::Frag &f)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = from_f32<T>(swish_value((float)f[e]));
}

// Fragment straight from global memory: 8 consecutive elements of one row.  Loads in this
// library are never placed under a data-dependent branch (the compiler would have to wait for
// each one before leaving the branch, which serialises them): callers clamp the row index into
// the valid range so the load is always legal, and rows past the end are zeroed by a register
// select here -- or left as finite duplicates of the last row where they only ever meet zero
// weights.
template <typename T>
__device__ __forceinline__ typename Atom<T>::Frag gfrag(const T *p, bool live)
{
    const typename Atom<T>::Frag f = Atom<T>::load(p);
    const typename Atom<T>::Frag z = Atom<T>::zero();
    return live ? f : z;
}

// ----------------------------------------------------------------------------
// Transposed token tile in LDS: XT[c][t] for c < ncols, t < C, row stride C + kPad,
// with the 8-token blocks of row c XOR-swizzled by (c/8) so that the transposing writes
// (one thread owns two adjacent tokens of 8 consecutive columns) spread over all banks
// and fragment reads stay 16-byte aligned.
// ----------------------------------------------------------------------------
template <int C> __device__ __forceinline__ int xt_off(int c, int t, int ld)
{
    constexpr int NB = C / 8;
    return c * ld + ((((t >> 3) ^ (c >> 3)) & (NB - 1)) << 3) + (t & 7);
}

// Token tile held in registers between the global load and the transposing LDS write.
// The tile is C tokens x NCOLS columns; thread (tid) owns row pairs and 8-column groups.
template <typename T, int C, int NCOLS, int NT> struct TokTile {
    static constexpr int NVEC = (C / 2) * (NCOLS / 8);          // (row pair, column group) items
    static constexpr int PER = (NVEC + NT - 1) / NT;
    Raw8<T> a[PER], b[PER];
    bool la[PER], lb[PER];   // whether the row really exists (else it is written as zeros)
    // src: row 0 of the tile, column 0 of the slice; rows >= len read as zero; columns >= ncols skipped.
    // Only issues the loads: the masking of missing rows is left to store_transposed, so that nothing
    // here waits for the data (a select right after the load would stall the wave for the full memory
    // latency before it could issue anything else).
    template <bool NTL = false>
    __device__ __forceinline__ void load(const T *src, size_t gld, int len, int ncols, int tid)
    {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            int idx = tid + NT * u;
            const bool in = idx < NVEC;
            idx = in ? idx : 0;
            const int rp = idx / (NCOLS / 8);
            int cg = idx - rp * (NCOLS / 8);
            const bool ok = in && cg * 8 < ncols;
            cg = ok ? cg : 0;
            const int r0 = min(2 * rp, len - 1), r1 = min(2 * rp + 1, len - 1);
            if (NTL) { a[u].load_nt(src + (size_t)r0 * gld + cg * 8); b[u].load_nt(src + (size_t)r1 * gld + cg * 8); }
            else { a[u].load(src + (size_t)r0 * gld + cg * 8); b[u].load(src + (size_t)r1 * gld + cg * 8); }
            la[u] = ok && 2 * rp < len;
            lb[u] = ok && 2 * rp + 1 < len;
        }
    }
    // The same for a column slice of one part of a memory snapshot (C slots, all present; the part is
    // tiled by kSnapTile columns): col0 = first column of the slice.
    template <bool NTL = false>
    __device__ __forceinline__ void load_snapshot(const T *part, int col0, int ncols, int tid)
    {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            int idx = tid + NT * u;
            const bool in = idx < NVEC;
            idx = in ? idx : 0;
            const int rp = idx / (NCOLS / 8);
            int cg = idx - rp * (NCOLS / 8);
            const bool ok = in && cg * 8 < ncols;
            cg = ok ? cg : 0;
            const T *p = part + snap_col<C>(col0 + cg * 8);
            if (NTL) { a[u].load_nt(p + (2 * rp) * kSnapTile); b[u].load_nt(p + (2 * rp + 1) * kSnapTile); }
            else { a[u].load(p + (2 * rp) * kSnapTile); b[u].load(p + (2 * rp + 1) * kSnapTile); }
            la[u] = lb[u] = ok;
        }
    }
    // PHI: with the feature map applied on the way (see swish_value)
    template <bool PHI = false>
    __device__ __forceinline__ void store_transposed(T *XT, int ld, int ncols, int tid) const
    {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int idx = tid + NT * u;
            const int rp = idx / (NCOLS / 8), cg = idx - rp * (NCOLS / 8);
            if (idx < NVEC && cg * 8 < ncols) {
                Raw8<T> x = a[u], y = b[u];
                x.keep(la[u]);
                y.keep(lb[u]);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    // two 2-byte stores: measured faster here than one packed 4-byte store
                    T *dst = XT + xt_off<C>(cg * 8 + e, 2 * rp, ld);
                    dst[0] = PHI ? from_f32<T>(swish_value((float)x.get(e))) : x.get(e);
                    dst[1] = PHI ? from_f32<T>(swish_value((float)y.get(e))) : y.get(e);
                }
            }
        }
    }
};

// Reduce over the 16 lanes that share l/16 (the 16 columns of one D-tile row).
__device__ __forceinline__ float row16_max(float x)
{
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float row16_sum(float x)
{
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) x += __shfl_xor(x, o, 64);
    return x;
}

}  // namespace gsa
