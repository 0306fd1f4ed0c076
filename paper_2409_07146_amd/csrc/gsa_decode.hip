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
template <typename T, int M, int NV, bool EARLY_V>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(int d_k, int d_v, float scale,
                                                             const T *__restrict__ q, const T *__restrict__ k,
                                                             const T *__restrict__ v, const float *__restrict__ g,
                                                             float *__restrict__ Kst, float *__restrict__ Vst,
                                                             T *__restrict__ o)
{
    constexpr int R = (M + kDecWaves - 1) / kDecWaves;  // rows (slots) per wave
    extern __shared__ float smem[];
    float *zs = smem;                 // [M] scores
    float *part = smem + 128;         // [kDecWaves][d_v] partial outputs

    const int bh = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float *Kb = Kst + (size_t)bh * M * d_k;
    float *Vb = Vst + (size_t)bh * M * d_v;
    const T *qb = q + (size_t)bh * d_k, *kb = k + (size_t)bh * d_k, *vb = v + (size_t)bh * d_v;
    const float *gb = g + (size_t)bh * M;

    f32x4 Kr[R][NV], Vr[R][NV];
    // ---- issue the memory loads
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = wave * R + rr;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int col = 4 * (lane + 64 * j);
            Kr[rr][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (row < M && col < d_k) Kr[rr][j] = *reinterpret_cast<const f32x4 *>(Kb + (size_t)row * d_k + col);
        }
    }
    if (EARLY_V) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int row = wave * R + rr;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int col = 4 * (lane + 64 * j);
                Vr[rr][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (row < M && col < d_v) Vr[rr][j] = *reinterpret_cast<const f32x4 *>(Vb + (size_t)row * d_v + col);
            }
        }
    }
    f32x4 qv[NV], kv[NV], vv[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int col = 4 * (lane + 64 * j);
        qv[j] = kv[j] = vv[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (col < d_k) { qv[j] = load4<T>(qb + col); kv[j] = load4<T>(kb + col); }
        if (col < d_v) vv[j] = load4<T>(vb + col);
    }
    float a[R], s[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = wave * R + rr;
        const float gv = (row < M) ? fmaxf(gb[row], kGateFloor) : 0.f;
        a[rr] = __expf(gv);
        s[rr] = -expm1f(gv);
    }
    // ---- key memories: update, write back, slot scores
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = wave * R + rr;
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int col = 4 * (lane + 64 * j);
            f32x4 x = Kr[rr][j];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[e] = a[rr] * x[e] + s[rr] * kv[j][e];
                dot += x[e] * qv[j][e];
            }
            if (row < M && col < d_k) *reinterpret_cast<f32x4 *>(Kb + (size_t)row * d_k + col) = x;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
        if (lane == 0 && row < M) zs[row] = scale * dot;
    }
    if (!EARLY_V) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int row = wave * R + rr;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int col = 4 * (lane + 64 * j);
                Vr[rr][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (row < M && col < d_v) Vr[rr][j] = *reinterpret_cast<const f32x4 *>(Vb + (size_t)row * d_v + col);
            }
        }
    }
    // ---- value memories: update and write back (independent of the scores)
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = wave * R + rr;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int col = 4 * (lane + 64 * j);
#pragma unroll
            for (int e = 0; e < 4; ++e) Vr[rr][j][e] = a[rr] * Vr[rr][j][e] + s[rr] * vv[j][e];
            if (row < M && col < d_v) *reinterpret_cast<f32x4 *>(Vb + (size_t)row * d_v + col) = Vr[rr][j];
        }
    }
    __syncthreads();
    // ---- softmax over the slots (every wave computes it; M <= 128)
    float z0 = (lane < M) ? zs[lane] : -INFINITY;
    float z1 = (lane + 64 < M) ? zs[lane + 64] : -INFINITY;
    float mx = fmaxf(z0, z1);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float e0 = (lane < M) ? __expf(z0 - mx) : 0.f;
    float e1 = (lane + 64 < M) ? __expf(z1 - mx) : 0.f;
    float den = e0 + e1;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) den += __shfl_xor(den, off, 64);
    const float inv = 1.f / den;
    // ---- output: slot-weighted sum of the updated value memories
    f32x4 acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int row = wave * R + rr;
        const float pe = (row < 64) ? __shfl(e0, row & 63, 64) : __shfl(e1, row & 63, 64);
        const float p = (row < M) ? pe * inv : 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][e] += p * Vr[rr][j][e];
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int col = 4 * (lane + 64 * j);
        if (col < d_v) *reinterpret_cast<f32x4 *>(part + (size_t)wave * d_v + col) = acc[j];
    }
    __syncthreads();
    for (int c = tid; c < d_v; c += kDecThreads) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) sum += part[(size_t)w * d_v + c];
        o[(size_t)bh * d_v + c] = from_f32<T>(sum);
    }
}

template <typename T, int M, int NV>
static hipError_t launch_decode_nv(int BH, int d_k, int d_v, float scale, const void *q, const void *k,
                                   const void *v, const float *g, float *K, float *V, void *o, hipStream_t st)
{
    const size_t lds = (128 + (size_t)kDecWaves * d_v) * sizeof(float);
    constexpr bool early = (NV * ((M + kDecWaves - 1) / kDecWaves) <= 8);
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
