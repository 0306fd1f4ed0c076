// Layout descriptor of the per-chunk memory snapshots kept in the workspace.
#pragma once
#include <hip/hip_runtime.h>

namespace gsa {

// A snapshot of the joint memory [Kt | Vt] (or of its gradient) is one record per (chunk, head)
// or per (sequence, head): the key part followed by the value part.  Each part is stored as
// tiles of kSnapTile columns, tile after tile, every tile [m][kSnapTile] with the column
// fastest: element (slot i, column c) of a part sits at
//     (c / kSnapTile) * m * kSnapTile + i * kSnapTile + c % kSnapTile.
// A scan workgroup owns one tile and writes it as one contiguous block (rows of a [m][d] array
// would be 128-byte pieces a kilobyte apart, which the memory system serves measurably slower);
// a contraction over the head dimension still finds 8 consecutive columns of a slot in one
// 16-byte piece, and the apply kernel, which contracts over the slots, transposes the column
// slice it needs on its way into LDS.  Offsets are in elements from the start of the record.
constexpr int kSnapTile = 64;

// Chunks per segment when the scans cut long sequences into segments: the length at which one
// workgroup's chain over the chunks no longer dominates the launch (measured: 32 chunks).
constexpr int kSegChunks = 32;

// The device kernels take the read-out and the feature-map switch in one int: the Readout value in
// the low byte, this bit for "q, k, v are raw projections: apply the feature map to them".
constexpr int kFeatureMapBit = 0x100;
constexpr int kReadoutMask = 0xff;

struct StateLayout {
    long long stride;   // elements per record
    long long oK, oV;   // key part, value part
};

// Offset of columns k0 .. k0+7 (k0 % 8 == 0) of slot 0 inside a part with m slots.
template <int M> __device__ __forceinline__ unsigned snap_col(int k0)
{
    return (unsigned)(k0 / kSnapTile) * (unsigned)(M * kSnapTile) + (unsigned)(k0 % kSnapTile);
}

}  // namespace gsa
