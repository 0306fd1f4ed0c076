// Single-token recurrent step of Gated Slot Attention (paper, Eq. (gsa); Figure 1).
//
// One workgroup per (batch, head) memory pair.  The step moves 2*m*(d_k+d_v)
// fp32 values (read + write back) and does ~10 flops per value, so it is bound
// by HBM bandwidth: the kernel issues every state load up front (16-byte loads,
// a whole row per wave so rows stay contiguous), updates in registers, and
// writes back with the same mapping.  Reductions (row dots for the slot scores,
// the slot-weighted sum for the output) go through wave shuffles and LDS in a
// fixed order, so results are bitwise reproducible.
#include "gsa_common.h"
#include "gsa_internal.h"

namespace gsa {

constexpr int kDecThreads = 1024;
constexpr int kDecWaves = kDecThreads / kWave;

template <typename T> __device__ __forceinline__ f32x4 load4(const T *p);
template <> __device__ __forceinline__ f32x4 load4<float>(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
template <> __device__ __forceinline__ f32x4 load4<bf16_t>(const bf16_t *p) {
    const bf16x4 x = *reinterpret_cast<const bf16x4 *>(p);
    return f32x4{(float)x[0], (float)x[1], (float)x[2], (float)x[3]};
}

// M: slots.  NV: float4 column groups per lane per row = ceil(max(d_k,d_v) / 256).
// EARLY_V: issue the value-memory loads before the key-memory arithmetic.
//
// Each wave owns M/16 slots (rows of both memories).  It updates its key rows, gets their
// scores by wave reductions, and folds its value rows into a partial output with a softmax
// that is local to the wave (its own maximum and sum); the 16 partial outputs are merged at the
// end with the usual rescaling.  So there is a single barrier, at the end, and no wave waits for
// another before its stores are issued.  No load sits under a data-dependent branch: column
// indices past the width are clamped and the lanes masked by register selects.
template <typename T, int M, int NV, bool EARLY_V>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(int d_k, int d_v, float scale,
                                                             const T *__restrict__ q, const T *__restrict__ k,
                                                             const T *__restrict__ v, const float *__restrict__ g,
                                                             float *__restrict__ Kst, float *__restrict__ Vst,
                                                             T *__restrict__ o)
{
    static_assert(M % kDecWaves == 0, "slots must split evenly over the waves");
    constexpr int R = M / kDecWaves;  // rows (slots) per wave
    extern __shared__ float smem[];
    float *ms = smem;                 // [kDecWaves][2] wave maximum and sum
    float *part = smem + 128;         // [kDecWaves][d_v] partial outputs

    const int bh = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float *Kb = Kst + (size_t)bh * M * d_k;
    float *Vb = Vst + (size_t)bh * M * d_v;
    const T *qb = q + (size_t)bh * d_k, *kb = k + (size_t)bh * d_k, *vb = v + (size_t)bh * d_v;
    const float *gb = g + (size_t)bh * M;

    int colk[NV], colv[NV];
    bool okk[NV], okv[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int col = 4 * (lane + 64 * j);
        okk[j] = col < d_k;
        okv[j] = col < d_v;
        colk[j] = okk[j] ? col : d_k - 4;
        colv[j] = okv[j] ? col : d_v - 4;
    }
    f32x4 Kr[R][NV], Vr[R][NV];
    // ---- issue the memory loads
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
        for (int j = 0; j < NV; ++j)
            Kr[rr][j] = *reinterpret_cast<const f32x4 *>(Kb + (size_t)(wave * R + rr) * d_k + colk[j]);
    if (EARLY_V) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int j = 0; j < NV; ++j)
                Vr[rr][j] = *reinterpret_cast<const f32x4 *>(Vb + (size_t)(wave * R + rr) * d_v + colv[j]);
    }
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    f32x4 qv[NV], kv[NV], vv[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        qv[j] = load4<T>(qb + colk[j]);
        kv[j] = load4<T>(kb + colk[j]);
        vv[j] = load4<T>(vb + colv[j]);
        qv[j] = okk[j] ? qv[j] : zero4;   // masked lanes contribute nothing to the row dots
    }
    float a[R], s[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const float gv = fmaxf(gb[wave * R + rr], kGateFloor);
        a[rr] = __expf(gv);
        s[rr] = -expm1f(gv);
    }
    // ---- key memories: update, write back, slot scores
    float z[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = wave * R + rr;
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            f32x4 x = Kr[rr][j];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[e] = a[rr] * x[e] + s[rr] * kv[j][e];
                dot += x[e] * qv[j][e];
            }
            if (okk[j]) *reinterpret_cast<f32x4 *>(Kb + (size_t)row * d_k + colk[j]) = x;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
        z[rr] = scale * dot;
    }
    if (!EARLY_V) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int j = 0; j < NV; ++j)
                Vr[rr][j] = *reinterpret_cast<const f32x4 *>(Vb + (size_t)(wave * R + rr) * d_v + colv[j]);
    }
    // ---- wave-local softmax weights
    float mw = z[0];
#pragma unroll
    for (int rr = 1; rr < R; ++rr) mw = fmaxf(mw, z[rr]);
    float sw = 0.f, e[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) { e[rr] = __expf(z[rr] - mw); sw += e[rr]; }
    // ---- value memories: update, write back, partial output
    f32x4 acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = zero4;
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = wave * R + rr;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            f32x4 x = Vr[rr][j];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                x[c] = a[rr] * x[c] + s[rr] * vv[j][c];
                acc[j][c] += e[rr] * x[c];
            }
            if (okv[j]) *reinterpret_cast<f32x4 *>(Vb + (size_t)row * d_v + colv[j]) = x;
        }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j)
        if (okv[j]) *reinterpret_cast<f32x4 *>(part + (size_t)wave * d_v + colv[j]) = acc[j];
    if (lane == 0) { ms[2 * wave] = mw; ms[2 * wave + 1] = sw; }
    __syncthreads();
    // ---- merge the 16 wave-local softmaxes
    float mx = ms[0];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) mx = fmaxf(mx, ms[2 * w]);
    float fw[kDecWaves], den = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) { fw[w] = __expf(ms[2 * w] - mx); den += fw[w] * ms[2 * w + 1]; }
    const float inv = 1.f / den;
    for (int c = tid; c < d_v; c += kDecThreads) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) sum += fw[w] * part[(size_t)w * d_v + c];
        o[(size_t)bh * d_v + c] = from_f32<T>(sum * inv);
    }
}

template <typename T, int M, int NV>
static hipError_t launch_decode_nv(int BH, int d_k, int d_v, float scale, const void *q, const void *k,
                                   const void *v, const float *g, float *K, float *V, void *o, hipStream_t st)
{
    const size_t lds = (128 + (size_t)kDecWaves * d_v) * sizeof(float);
    constexpr bool early = (NV * (M / kDecWaves) <= 8);
    auto kern = decode_kernel<T, M, NV, early>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    KernelTimer kt(kSlotDecode, st);
    hipLaunchKernelGGL(kern, dim3(BH), dim3(kDecThreads), lds, st, d_k, d_v, scale, (const T *)q, (const T *)k,
                       (const T *)v, g, K, V, (T *)o);
    return hipGetLastError();
}

template <typename T, int M>
static hipError_t launch_decode_m(int BH, int d_k, int d_v, float scale, const void *q, const void *k,
                                  const void *v, const float *g, float *K, float *V, void *o, hipStream_t st)
{
    const int dmax = d_k > d_v ? d_k : d_v;
    const int nv = (dmax + 255) / 256;
    switch (nv) {
    case 1: return launch_decode_nv<T, M, 1>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    case 2: return launch_decode_nv<T, M, 2>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    case 3: return launch_decode_nv<T, M, 3>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    default: return launch_decode_nv<T, M, 4>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    }
}

template <typename T>
static hipError_t launch_decode_t(int BH, int d_k, int d_v, int m, float scale, const void *q, const void *k,
                                  const void *v, const float *g, float *K, float *V, void *o, hipStream_t st)
{
    switch (m) {
    case 16: return launch_decode_m<T, 16>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    case 32: return launch_decode_m<T, 32>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    case 64: return launch_decode_m<T, 64>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    default: return launch_decode_m<T, 128>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, st);
    }
}

hipError_t launch_decode(int BH, int d_k, int d_v, int m, int dtype, float scale, const void *q, const void *k,
                         const void *v, const float *g, float *K, float *V, void *o, hipStream_t st)
{
    if (dtype == 0) return launch_decode_t<float>(BH, d_k, d_v, m, scale, q, k, v, g, K, V, o, st);
    return launch_decode_t<bf16_t>(BH, d_k, d_v, m, scale, q, k, v, g, K, V, o, st);
}

}  // namespace gsa
