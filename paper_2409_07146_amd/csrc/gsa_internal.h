// Host-side declarations shared by the libgsa translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace gsa {

// Everything a launcher needs to know about one problem, resolved on the host.
struct Plan {
    int32_t B, T, H, d_k, d_v, m, dtype;
    float scale;
    const int32_t *cu_seqlens;  // device, or NULL
    int32_t n_seqs;             // sequences (B in batch form)
    int64_t tokens;             // B*T
    int32_t chunk;              // tokens per chunk for this dtype
    int32_t chunk_slots;        // upper bound on chunks (exact in batch form)
    // workspace offsets in bytes (256-byte aligned); 0-sized parts share an offset
    size_t off_table, off_seqtab, off_S, off_SF, off_E, off_dz, off_dgf, total_fwd, total_bwd;
};

// Workspace views handed to the launchers.
struct Work {
    int32_t *table;   // [4*chunk_slots] packed form only
    int32_t *seqtab;  // [4*n_seqs]     packed form only
    float *S;         // [chunk_slots][H][m][d_k+d_v] memories at the start of each chunk
    float *SF;        // [n_seqs][H][m][d_k+d_v] memories after the last token (backward only)
    float *E;         // same shape as S: gradient of the memories at the end of each chunk
    float *dz;        // [tokens][H][m]
    float *dgf;       // [tokens][H][m]
};

// Kernel slots of the optional per-kernel event timing (gsa_profile_*).
enum KernelSlot { kSlotPrepare = 0, kSlotScanFwd, kSlotOutFwd, kSlotBwdDz, kSlotScanBwd, kSlotBwdMain, kSlotDecode,
                  kNumKernelSlots };

// Brackets one kernel launch with events on its stream when timing is enabled; otherwise a no-op.
class KernelTimer {
public:
    KernelTimer(int slot, hipStream_t st);
    ~KernelTimer();
    KernelTimer(const KernelTimer &) = delete;
    KernelTimer &operator=(const KernelTimer &) = delete;
private:
    int slot_;
    hipStream_t st_;
    void *start_;
};

hipError_t launch_prepare(const Plan &pl, const Work &w, hipStream_t st);

hipError_t launch_fwd(const Plan &pl, const Work &w, const void *q, const void *k, const void *v, const float *g,
                      const float *K0, const float *V0, void *o, float *z_saved, float *KT, float *VT,
                      hipStream_t st);

hipError_t launch_bwd(const Plan &pl, const Work &w, const void *q, const void *k, const void *v, const float *g,
                      const float *K0, const float *V0, const float *z_saved, const void *dO, const float *dKT,
                      const float *dVT, void *dq, void *dk, void *dv, float *dg, float *dK0, float *dV0,
                      hipStream_t st);

hipError_t launch_decode(int BH, int d_k, int d_v, int m, int dtype, float scale, const void *q, const void *k,
                         const void *v, const float *g, float *K, float *V, void *o, hipStream_t st);

}  // namespace gsa
