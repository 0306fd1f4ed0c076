// Layout descriptor of the per-chunk memory snapshots kept in the workspace.
#pragma once

namespace gsa {

// Where the pieces of a per-chunk memory snapshot live.  A snapshot of the joint memory
// [Kt | Vt] is stored as up to four blocks per (chunk, head): the key and value parts in
// natural layout ([m][d], what a contraction over d reads) and/or transposed ([d][m], what
// a contraction over the slots reads).  Offsets are in elements from the start of the
// (chunk, head) record; -1 = block not stored.
struct StateLayout {
    long long stride;            // elements per (chunk, head)
    long long oKn, oVn, oKt, oVt;
};


}  // namespace gsa
