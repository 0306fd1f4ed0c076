// Host-side declarations shared by the libgsa translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gsa_layout.h"

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
    int32_t seg_chunks, max_seg;   // long sequences: chunks per scan segment, segments provided per sequence (1 = off)
    // workspace offsets in bytes (256-byte aligned); 0-sized parts share an offset
    size_t off_table, off_seqtab, off_segbase, off_Wf, off_dec, off_S, off_tA, off_tP, off_sumY, off_sumD, total_fwd;
    size_t off_SF, off_Wr, off_E, off_dz, off_dgf, off_tB, off_tBT, off_tA2T, off_tAvT, off_tSbe, total_bwd;
    // layout of every memory snapshot record (elements); see gsa_layout.h
    StateLayout lay;
    // variants (gsa_fwd_ex / gsa_bwd_ex): write intensity as an input of its own, element-wise read-outs
    const float *s_in = nullptr;   // [B,T,H,m] device, or NULL for s = 1 - exp(g)
    float *ds_out = nullptr;       // backward: gradient of s_in
    int32_t readout = 0;           // Readout
    float gate_tau = 0.f;          // > 0: g holds gate logits, the log gate is logsigmoid(g) / gate_tau
    int32_t phi = 0;               // 1: q, k, v hold raw projections, the kernels apply the Swish feature map
    bool keep = false;             // the forward leaves tables, scan weights, S and SF for the backward (no recomputation)
    // forward output epilogue (gsa_fwd_act): y = Swish(o) and per-slice sums of squares of y beside (or instead of) o
    void *act_out = nullptr;       // [B,T,H,d_v] I/O dtype, or NULL
    float *act_ssq = nullptr;      // [B,T,H,ceil(d_v / slice)] fp32, or NULL
    bool general() const { return s_in != nullptr || readout != 0 || gate_tau > 0.f || phi != 0; }
    int opts() const { return readout | (phi ? kFeatureMapBit : 0); }   // what the device kernels take
};

// Workspace views handed to the launchers.
struct Work {
    int32_t *table;   // [4*chunk_slots] packed form only
    int32_t *seqtab;  // [4*n_seqs]     packed form only
    int32_t *segbase; // [n_seqs+1]     packed form only: scan segments before each sequence
    // per (chunk, head) records, element type = I/O dtype unless noted; KM = max(m, 32)
    void *Wf;         // [m][C]      forward scan weights s*exp(G_C-G)
    float *dec;       // [m]         chunk decay exp(G_C)                                  (fp32)
    void *S;          // memory at the start of the chunk (Plan::lay)
    void *tA;         // [C][C]      forward: pair weights A2;  backward: scale*Bm
    void *tP;         // [C][KM]     forward: p*exp(G);         backward: scale*dz*exp(G)
    void *SF;         // per (sequence, head): memory after the last token (Plan::lay)
    void *Wr;         // [2][m][C]   reverse scan weights
    void *E;          // gradient of the memory at the end of the chunk (Plan::lay)
    void *tBT;        // [C][C]      scale*Bm^T
    void *tA2T;       // [C][C]      A2^T
    void *tAvT;       // [C][C]      (dO_t . v_r)^T, causally masked
    void *tSbe;       // [C][KM]     s*exp(G_C-G)
    float *sumY, *sumD;   // scan segment summaries (fp32), see gsa_scan.hip
    float *dz;        // [tokens][H][m]                                                     (fp32)
    float *dgf;       // [tokens][H][m]   z*dz + p*dp                                       (fp32)
};

// Kernel slots of the optional per-kernel event timing (gsa_profile_*).
enum KernelSlot { kSlotPrepare = 0, kSlotGates, kSlotScanFwd, kSlotChunkFwd, kSlotApplyFwd, kSlotChunkDz, kSlotScanBwd,
                  kSlotChunkIntra, kSlotApplyBwd, kSlotDecode, kSlotDecodeMerge, kSlotCopyProbe, kSlotScanSummary, kNumKernelSlots };

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
hipError_t launch_gates(const Plan &pl, const Work &w, const float *g, const float *sin, float tau, hipStream_t st);

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
    bool phi_k = false, phi_v = false;   // feature map on xk / xv as they are loaded
};
hipError_t launch_scan(const Plan &pl, const Work &w, const ScanIo &io, hipStream_t st);

// The wide contractions out = A_tok X + A_slot St for up to three outputs in one
// launch (see gsa_apply.hip).  xslot_rec + xslot_off points at a memory block [m][d] of the first
// (chunk, head) record; records are xslot_stride elements apart.
struct ApplyIo {
    const void *A_tok, *A_slot, *xtok, *xslot_rec;
    long long xslot_off, xslot_stride;
    void *out;
    int d;
    bool phi_tok = false;        // feature map on xtok as it is loaded
    const void *raw = nullptr;   // [tokens][H][d] or NULL: out is multiplied by the feature map's slope at raw
    // output epilogue (forward): act = Swish(out) as stored, ssq[token][head][slice] = sum over the slice's
    // columns of act^2; out itself may then be NULL (not written)
    void *act = nullptr;
    float *ssq = nullptr;
};
// Columns per workgroup of the apply kernel (= columns per partial sum of squares of the output epilogue).
int apply_slice_cols(int dtype);
hipError_t launch_apply(const Plan &pl, const Work &w, const ApplyIo *io, int n, int slot, hipStream_t st);

hipError_t launch_fwd(const Plan &pl, const Work &w, const void *q, const void *k, const void *v, const float *g,
                      const float *K0, const float *V0, void *o, float *z_saved, float *KT, float *VT,
                      hipStream_t st);

hipError_t launch_bwd(const Plan &pl, const Work &w, const void *q, const void *k, const void *v, const float *g,
                      const float *K0, const float *V0, const float *z_saved, const void *dO, const float *dKT,
                      const float *dVT, void *dq, void *dk, void *dv, float *dg, float *dK0, float *dV0,
                      hipStream_t st);

// scratch: NULL (one workgroup per pair) or decode_scratch_floats(...) floats (split form, small BH).
// opts: Readout in the low byte, kFeatureMapBit.
hipError_t launch_decode(int BH, int d_k, int d_v, int m, int dtype, float scale, const void *q, const void *k,
                         const void *v, const float *g, float *K, float *V, void *o, float *scratch, const float *sin,
                         int opts, float gate_tau, hipStream_t st);
size_t decode_scratch_floats(int BH, int d_v, int m);
// The library's own scratch array for the split form (one per GPU, never freed): its capacity, and its
// address on the current device (looked up on the first call per device; allocates nothing).
size_t decode_static_scratch_floats();
hipError_t decode_static_scratch(float **ptr);

}  // namespace gsa
