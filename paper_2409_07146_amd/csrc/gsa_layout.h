// Layout descriptor of the per-chunk memory snapshots kept in the workspace.
#pragma once

namespace gsa {

// A snapshot of the joint memory [Kt | Vt] (or of its gradient) is one record per (chunk, head)
// or per (sequence, head): the key part [m][d_k] followed by the value part [m][d_v], rows =
// slots, head dimension fastest.  That is the orientation a contraction over the head dimension
// reads directly; the apply kernel, which contracts over the slots, transposes the column slice
// it needs on its way into LDS.  Offsets are in elements from the start of the record.
struct StateLayout {
    long long stride;   // elements per record
    long long oK, oV;   // key part, value part
};


}  // namespace gsa
