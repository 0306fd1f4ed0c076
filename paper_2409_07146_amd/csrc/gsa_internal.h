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
    size_t off_table, off_seqtab, off_Wf, off_dec, off_S, off_SF, off_Wr, off_E, off_dz, off_dgf, total_fwd,
        total_bwd;
};

// Workspace views handed to the launchers.
struct Work {
    int32_t *table;   // [4*chunk_slots] packed form only
    int32_t *seqtab;  // [4*n_seqs]     packed form only
    void *Wf;         // [chunk_slots][H][m][C]    forward scan weights s*exp(G_C-G)          (I/O dtype)
    float *dec;       // [chunk_slots][H][m]       chunk decay exp(G_C)
    void *S;          // [chunk_slots][H][m][d_k+d_v] memories at the start of each chunk     (I/O dtype)
    void *SF;         // [n_seqs][H][m][d_k+d_v]   memories after the last token (backward)   (I/O dtype)
    void *Wr;         // [chunk_slots][H][2][m][C] reverse scan weights                       (I/O dtype)
    void *E;          // same shape as S: gradient of the memories at the end of each chunk   (I/O dtype)
    float *dz;        // [tokens][H][m]
    float *dgf;       // [tokens][H][m]
};

// Kernel slots of the optional per-kernel event timing (gsa_profile_*).
enum KernelSlot { kSlotPrepare = 0, kSlotGates, kSlotScanFwd, kSlotOutFwd, kSlotBwdDz, kSlotScanBwd, kSlotBwdMain,
                  kSlotDecode, kNumKernelSlots };

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

// Forward-scan weights and chunk decays from the log gates (chunk-parallel).
hipError_t launch_gates(const Plan &pl, const Work &w, const float *g, hipStream_t st);

// One scan over the chunks of every sequence.  Forward: x = (k, v), init = (K0, V0), snapshots go
// to Work::S, weights come from Work::Wf.  Reverse: x = (q, dO), init = (dKT, dVT), snapshots go
// to Work::E, weights come from Work::Wr.  outK/outV (fp32, API layout) and outJ (I/O dtype,
// joint layout) receive the accumulator after the last chunk; each may be NULL.
struct ScanIo {
    const void *xk, *xv;
    const float *initK, *initV;
    float *outK, *outV;
    void *outJ;
    bool reverse;
};
hipError_t launch_scan(const Plan &pl, const Work &w, const ScanIo &io, hipStream_t st);

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
