// Single-token recurrent step of Gated Slot Attention (paper, Eq. (gsa); Figure 1).
//
// One workgroup per (batch, head) memory pair.  The step moves 2*m*(d_k+d_v)
// fp32 values (read + write back) and does ~10 flops per value, so it is bound
// by HBM bandwidth: the kernel issues every state load up front (16-byte loads,
// a whole row per wave so rows stay contiguous), updates in registers, and
// writes back with the same mapping.  Reductions (row dots for the slot scores,
// the slot-weighted sum for the output) go through wave shuffles and LDS in a
// fixed order, so results are bitwise reproducible.
//
// With few memory pairs (small batches) one workgroup per pair leaves most of the chip idle
// and the step is bound by what one compute unit can stream.  The split form spreads a pair
// over several workgroups, each covering some of the slots; each writes its unnormalised partial
// output with its own softmax maximum and sum to a workspace, and a second, tiny kernel merges
// the partials of a pair in a fixed order.  No workgroup waits for another.  (With many pairs the
// one-workgroup form is the faster one again.)
#include <mutex>

#include "gsa_common.h"
#include "gsa_internal.h"

// The memories are read once and written once per step and are not touched again until the next
// step of the same layer: their loads and stores carry the non-temporal hint, so they stream
// through the caches instead of displacing each other (measured: 30.4 -> 26.4 us per step at 256
// pairs when the states of successive calls differ, as they do across the layers of a model).
#define GSA_LD(p) __builtin_nontemporal_load(p)
#define GSA_ST(x, p) __builtin_nontemporal_store(x, p)
namespace gsa {

constexpr int kDecThreads = 1024;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr int kSplitWaves = 4;                    // waves (= slot rows) per workgroup of the split form
constexpr int kSplitPairsMax = 64;                // up to this many memory pairs: one slot row per wave (measured crossover)

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
// end with the usual rescaling.  There are two barriers: one between the loads of the memories and
// the first store (see there), one before the merge.  No load sits under a data-dependent branch: column
// indices past the width are clamped and the lanes masked by register selects.
//
// PIECES > 0 (split form): a pair is spread over PIECES workgroups of NWAVES waves, each covering
// M/PIECES slots (blockIdx.x = pair * PIECES + piece); instead of the output the workgroup writes to
// `scratch`, per pair [PIECES][2] (maximum, sum) followed by [PIECES][d_v] (unnormalised partial output).
// GEN: the general form (write intensities from `sin` when given; opts: read-out in the low byte and
// kFeatureMapBit for the feature map on q, k, v; gate logits with gate_tau > 0); the plain calls run
// GEN = false, where none of this is compiled in.
template <typename T, int M, int NV, bool EARLY_V, int NWAVES, int PIECES, bool GEN>
__global__ __launch_bounds__(NWAVES * kWave) void decode_kernel(int d_k, int d_v, float scale,
                                                               const T *__restrict__ q, const T *__restrict__ k,
                                                               const T *__restrict__ v, const float *__restrict__ g,
                                                               float *__restrict__ Kst, float *__restrict__ Vst,
                                                               T *__restrict__ o, float *__restrict__ scratch,
                                                               const float *__restrict__ sin, int opts,
                                                               float gate_tau)
{
    const int readout = opts & kReadoutMask;
    constexpr bool SPLIT = PIECES > 0;
    constexpr int NSPLIT = SPLIT ? PIECES : 1;
    static_assert(M % (NWAVES * NSPLIT) == 0, "slots must split evenly over the workgroups and their waves");
    constexpr int R = M / (NWAVES * NSPLIT);    // rows (slots) per wave
    constexpr int NTHREADS = NWAVES * kWave;
    extern __shared__ float smem[];
    float *ms = smem;                 // [NWAVES][2] wave maximum and sum
    float *part = smem + 128;         // [NWAVES][d_v] partial outputs

    const int bh = blockIdx.x / NSPLIT, piece = blockIdx.x % NSPLIT;
    const int tid = threadIdx.x, lane = tid & 63, wave0 = tid >> 6;
    const int wave = piece * NWAVES + wave0;      // index of this wave's first slot row, in units of R rows
    float *Kb = Kst + (size_t)bh * M * d_k;
    float *Vb = Vst + (size_t)bh * M * d_v;
    const T *qb = q + (size_t)bh * d_k, *kb = k + (size_t)bh * d_k, *vb = v + (size_t)bh * d_v;
    const float *gb = g + (size_t)bh * M;
    // write intensities of their own (gsa_decode_step_ex) or NULL; the load below is unconditional
    // (from g when there are none) and a register select decides
    const float *sb = ((GEN && sin) ? sin : g) + (size_t)bh * M;

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
    // ---- the small operands first
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    f32x4 qv[NV], kv[NV], vv[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        qv[j] = load4<T>(qb + colk[j]);
        kv[j] = load4<T>(kb + colk[j]);
        vv[j] = load4<T>(vb + colv[j]);
    }
    float graw[R], sraw[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        graw[rr] = gb[wave * R + rr];
        sraw[rr] = GEN ? sb[wave * R + rr] : 0.f;
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- then the memories
    f32x4 Kr[R][NV], Vr[R][NV];
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
        for (int j = 0; j < NV; ++j)
            Kr[rr][j] = GSA_LD(reinterpret_cast<const f32x4 *>(Kb + (size_t)(wave * R + rr) * d_k + colk[j]));
    if (EARLY_V) {
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int j = 0; j < NV; ++j)
                Vr[rr][j] = GSA_LD(reinterpret_cast<const f32x4 *>(Vb + (size_t)(wave * R + rr) * d_v + colv[j]));
    }
    __builtin_amdgcn_sched_barrier(0);
    // Every wave of the workgroup has all its memory rows before any of them stores: the chip then reads
    // for a while and writes for a while instead of mixing the two all the time, which the memory
    // system serves measurably faster (26.5 -> 23.7 us per step at 256 pairs).
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NV; ++j) qv[j] = okk[j] ? qv[j] : zero4;   // masked lanes contribute nothing to the row dots
    if (GEN && (opts & kFeatureMapBit)) {
#pragma unroll
        for (int j = 0; j < NV; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                qv[j][e] = swish_value(qv[j][e]);
                kv[j][e] = swish_value(kv[j][e]);
                vv[j][e] = swish_value(vv[j][e]);
            }
    }
    float a[R], s[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const float gv = fmaxf((GEN && gate_tau > 0.f) ? log_gate_from_logit(graw[rr], gate_tau) : graw[rr], kGateFloor);
        a[rr] = __expf(gv);
        s[rr] = (GEN && sin) ? sraw[rr] : -expm1f(gv);
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
            if (okk[j]) GSA_ST(x, reinterpret_cast<f32x4 *>(Kb + (size_t)row * d_k + colk[j]));
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
                Vr[rr][j] = GSA_LD(reinterpret_cast<const f32x4 *>(Vb + (size_t)(wave * R + rr) * d_v + colv[j]));
    }
    // ---- wave-local softmax weights (an element-wise read-out instead: weights f(z), maximum 0 and sum 0,
    // so that the merges below add the partial outputs as they are and skip the normalisation)
    const bool soft = !GEN || readout == kReadSoftmax;
    float mw = z[0];
#pragma unroll
    for (int rr = 1; rr < R; ++rr) mw = fmaxf(mw, z[rr]);
    mw = soft ? mw : 0.f;
    float sw = 0.f, e[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        e[rr] = soft ? __expf(z[rr] - mw) : readout_value(readout, z[rr]);
        sw += soft ? e[rr] : 0.f;
    }
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
            if (okv[j]) GSA_ST(x, reinterpret_cast<f32x4 *>(Vb + (size_t)row * d_v + colv[j]));
        }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j)
        if (okv[j]) *reinterpret_cast<f32x4 *>(part + (size_t)wave0 * d_v + colv[j]) = acc[j];
    if (lane == 0) { ms[2 * wave0] = mw; ms[2 * wave0 + 1] = sw; }
    __syncthreads();
    // ---- merge the wave-local softmaxes of the workgroup
    float mx = ms[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) mx = fmaxf(mx, ms[2 * w]);
    float fw[NWAVES], den = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) { fw[w] = __expf(ms[2 * w] - mx); den += fw[w] * ms[2 * w + 1]; }
    if (SPLIT) {
        float *sp = scratch + (size_t)bh * NSPLIT * (d_v + 2);
        if (tid == 0) { sp[2 * piece] = mx; sp[2 * piece + 1] = den; }
        float *po = sp + 2 * NSPLIT + (size_t)piece * d_v;
        for (int c = tid; c < d_v; c += NTHREADS) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < NWAVES; ++w) sum += fw[w] * part[(size_t)w * d_v + c];
            po[c] = sum;
        }
        return;
    }
    const float inv = soft ? 1.f / den : 1.f;
    for (int c = tid; c < d_v; c += NTHREADS) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NWAVES; ++w) sum += fw[w] * part[(size_t)w * d_v + c];
        o[(size_t)bh * d_v + c] = from_f32<T>(sum * inv);
    }
}

// Second kernel of the split form: merges the NSPLIT partial outputs of a pair (each with its
// softmax maximum and sum) in index order.  One wave per (256 columns, pair); every load is
// issued before the first use, so the kernel costs one trip to memory.
template <typename T> __device__ __forceinline__ void store4_as(T *p, const f32x4 &x);
template <> __device__ __forceinline__ void store4_as<float>(float *p, const f32x4 &x) { *reinterpret_cast<f32x4 *>(p) = x; }
template <> __device__ __forceinline__ void store4_as<bf16_t>(bf16_t *p, const f32x4 &x) {
    *reinterpret_cast<bf16x4 *>(p) = bf16x4{(bf16_t)x[0], (bf16_t)x[1], (bf16_t)x[2], (bf16_t)x[3]};
}

template <typename T, int NSPLIT>
__global__ __launch_bounds__(kWave) void decode_merge_kernel(int d_v, const float *__restrict__ scratch, T *__restrict__ o,
                                                             int readout)
{
    const int bh = blockIdx.y, col = 4 * (blockIdx.x * kWave + threadIdx.x);
    const bool ok = col < d_v;
    const int c = ok ? col : d_v - 4;
    const float *sp = scratch + (size_t)bh * NSPLIT * (d_v + 2);
    const float *po = sp + 2 * NSPLIT + c;
    float mj[NSPLIT], lj[NSPLIT];
    f32x4 pj[NSPLIT];
#pragma unroll
    for (int j = 0; j < NSPLIT; ++j) { mj[j] = sp[2 * j]; lj[j] = sp[2 * j + 1]; }
#pragma unroll
    for (int j = 0; j < NSPLIT; ++j) pj[j] = *reinterpret_cast<const f32x4 *>(po + (size_t)j * d_v);
    float mx = mj[0];
#pragma unroll
    for (int j = 1; j < NSPLIT; ++j) mx = fmaxf(mx, mj[j]);
    float den = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NSPLIT; ++j) {
        const float f = __expf(mj[j] - mx);
        den += f * lj[j];
        acc += f * pj[j];
    }
    acc *= (readout == kReadSoftmax) ? 1.f / den : 1.f;
    if (ok) store4_as<T>(o + (size_t)bh * d_v + col, acc);
}

template <typename T, int M, int NV>
static hipError_t launch_decode_nv(int BH, int d_k, int d_v, float scale, const void *q, const void *k,
                                   const void *v, const float *g, float *K, float *V, void *o, float *scratch,
                                   const float *sin, int opts, float gate_tau, hipStream_t st)
{
    if (scratch && BH <= kSplitPairsMax) {
        // few pairs: m/4 workgroups of four waves per pair (one slot row per wave)
        constexpr int pieces = M / kSplitWaves;
        const size_t lds = (128 + (size_t)kSplitWaves * d_v) * sizeof(float);
        // opts is non-zero for a read-out other than the softmax and for the feature map
        const bool gen = sin != nullptr || opts != kReadSoftmax || gate_tau > 0.f;
        auto kern = gen ? decode_kernel<T, M, NV, true, kSplitWaves, pieces, true>
                        : decode_kernel<T, M, NV, true, kSplitWaves, pieces, false>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        {
            KernelTimer kt(kSlotDecode, st);
            hipLaunchKernelGGL(kern, dim3(BH * pieces), dim3(kSplitWaves * kWave), lds, st, d_k, d_v, scale,
                               (const T *)q, (const T *)k, (const T *)v, g, K, V, (T *)o, scratch, sin, opts,
                               gate_tau);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        KernelTimer kt(kSlotDecodeMerge, st);
        const dim3 mgrid((d_v + 4 * kWave - 1) / (4 * kWave), BH);
        hipLaunchKernelGGL((decode_merge_kernel<T, pieces>), mgrid, dim3(kWave), 0, st, d_v, scratch, (T *)o, opts & kReadoutMask);
        return hipGetLastError();
    }
    const size_t lds = (128 + (size_t)kDecWaves * d_v) * sizeof(float);
    constexpr bool early = (NV * (M / kDecWaves) <= 8);
    const bool gen = sin != nullptr || opts != kReadSoftmax || gate_tau > 0.f;
    auto kern = gen ? decode_kernel<T, M, NV, early, kDecWaves, 0, true> : decode_kernel<T, M, NV, early, kDecWaves, 0, false>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    KernelTimer kt(kSlotDecode, st);
    hipLaunchKernelGGL(kern, dim3(BH), dim3(kDecThreads), lds, st, d_k, d_v, scale, (const T *)q, (const T *)k,
                       (const T *)v, g, K, V, (T *)o, static_cast<float *>(nullptr), sin, opts, gate_tau);
    return hipGetLastError();
}

template <typename T, int M>
static hipError_t launch_decode_m(int BH, int d_k, int d_v, float scale, const void *q, const void *k,
                                  const void *v, const float *g, float *K, float *V, void *o, float *scratch,
                                  const float *sin, int opts, float gate_tau, hipStream_t st)
{
    const int dmax = d_k > d_v ? d_k : d_v;
    const int nv = (dmax + 255) / 256;
    switch (nv) {
    case 1: return launch_decode_nv<T, M, 1>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    case 2: return launch_decode_nv<T, M, 2>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    case 3: return launch_decode_nv<T, M, 3>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    default: return launch_decode_nv<T, M, 4>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    }
}

template <typename T>
static hipError_t launch_decode_t(int BH, int d_k, int d_v, int m, float scale, const void *q, const void *k,
                                  const void *v, const float *g, float *K, float *V, void *o, float *scratch,
                                  const float *sin, int opts, float gate_tau, hipStream_t st)
{
    switch (m) {
    case 16: return launch_decode_m<T, 16>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    case 32: return launch_decode_m<T, 32>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    case 64: return launch_decode_m<T, 64>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    default: return launch_decode_m<T, 128>(BH, d_k, d_v, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    }
}

// Floats of workspace the split form needs for BH pairs (0: the split form is not used at this size).
size_t decode_scratch_floats(int BH, int d_v, int m)
{
    if (BH > kSplitPairsMax) return 0;
    return (size_t)BH * (m / kSplitWaves) * (d_v + 2);
}

// ---------------------------------------------------------------------------------------
// Scratch memory of the split form for callers that cannot allocate (gsa_decode_step_static): a
// file-scope device array, one copy per GPU, held until the process ends.  In host code the array's
// name is only a handle; its device address is asked for once per device with that device current
// (static_scratch below) and only that address is ever passed on.
// ---------------------------------------------------------------------------------------
constexpr size_t kStaticScratchFloats = (size_t)1 << 20;   // 4 MiB
static __device__ __align__(256) float scratch_static[kStaticScratchFloats];

size_t decode_static_scratch_floats() { return kStaticScratchFloats; }

hipError_t decode_static_scratch(float **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static float *addr[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch_static));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = static_cast<float *>(p);
    }
    *ptr = addr[dev];
    return hipSuccess;
}

hipError_t launch_decode(int BH, int d_k, int d_v, int m, int dtype, float scale, const void *q, const void *k,
                         const void *v, const float *g, float *K, float *V, void *o, float *scratch, const float *sin,
                         int opts, float gate_tau, hipStream_t st)
{
    if (dtype == 0) return launch_decode_t<float>(BH, d_k, d_v, m, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
    return launch_decode_t<bf16_t>(BH, d_k, d_v, m, scale, q, k, v, g, K, V, o, scratch, sin, opts, gate_tau, st);
}

}  // namespace gsa
