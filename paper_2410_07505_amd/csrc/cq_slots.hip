// Slots of library-owned device state, one per stream.
//
// The quantize kernel combines its per-block zero counts in a word of static device memory that
// is zero between launches and is cleared again by the last block to finish, so that no clearing
// kernel has to run before it.  Calls on one stream are ordered and can
// share a piece; calls on different streams may run at the same time and must not.  Each stream
// handle seen is therefore given a slot of its own, for the life of the process.
#include <mutex>

#include "cq_kernels.h"

namespace cq {

int stream_slot(hipStream_t stream) {
    // the per-thread default stream is one handle for many real streams: no slot
    if (stream == hipStreamPerThread) return -1;
    static std::mutex mu;
    static hipStream_t seen[kStateSlots];
    static int n_seen = 0;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < n_seen; ++i)
        if (seen[i] == stream) return i;
    if (n_seen == kStateSlots) return -1;       // callers fall back to the path that clears first
    seen[n_seen] = stream;
    return n_seen++;
}

}  // namespace cq
