// Helpers for the .hip launchers: chunk-map construction and error plumbing.
#pragma once
#include "gsa_common.h"
#include "gsa_internal.h"

namespace gsa {

inline ChunkMap make_chunk_map(const Plan &pl, const Work &w)
{
    ChunkMap cm;
    const bool packed = pl.cu_seqlens != nullptr;
    cm.table = packed ? w.table : nullptr;
    cm.seq_tab = packed ? w.seqtab : nullptr;
    cm.seg_base = packed ? w.segbase : nullptr;
    cm.T = pl.T;
    cm.chunk = pl.chunk;
    cm.chunks_per_seq = (pl.T + pl.chunk - 1) / pl.chunk;
    cm.n_chunk_slots = pl.chunk_slots;
    return cm;
}

#define GSA_HIP_TRY(expr)                         \
    do {                                          \
        hipError_t _e = (expr);                   \
        if (_e != hipSuccess) return _e;          \
    } while (0)

template <typename K> inline hipError_t allow_lds(K kern, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

}  // namespace gsa
