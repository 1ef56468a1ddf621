// Host interface of the one-launch forward (stream_fwd.hpp), compiled in its own translation
// unit.
#pragma once

#include <hip/hip_runtime.h>

#include <vector>

#include "stream_fwd.hpp"

namespace castling {

// The task lists of the eight queues for `units` units: queue x serves units x, x + 8, ...;
// per unit `cr` reduce chunks, `ncs` combine slices and `ca` apply chunks (reduce and combine
// only with the linear branch), the reduce chunks of the unit `lookahead` places further on
// dealt between the apply chunks of the current one; `nw` filter-table tasks go first, spread
// over the queues.  Every task comes after the tasks it waits for.
void build_stream_tasks(int units, int cr, int ca, int ncs, int nw, int lookahead, bool lin,
                        std::vector<uint32_t>& tasks, uint32_t (&queue_off)[kStreamQueues + 1]);

// Sets the kernel's LDS attribute and returns in *blocks_per_cu how many workgroups of it a
// compute unit holds (0 if it cannot run).
hipError_t stream_forward_prepare(int ks, bool lin, bool dw, bool half, int* blocks_per_cu);

hipError_t stream_forward_launch(int ks, bool lin, bool dw, bool half, const StreamArgs& a, int blocks,
                                 hipStream_t s);

}  // namespace castling
