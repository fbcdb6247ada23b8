// Level 1 of the top-k selection (topk.hip), done where the scores are produced: a streaming
// kernel of the Full layer keeps its rows' group-mean scores in LDS until its loop is over, so
// on their way out it also counts them per top-12-bits of their order-preserving key -- a
// binning that needs no score range -- in a workgroup histogram in LDS, and adds the non-empty
// bins to the histogram of its (batch, KV head) in memory.  When the streaming kernel ends,
// that histogram is complete and the selection kernel starts at "find the threshold bin".
#pragma once
#include "device_util.h"

namespace hylra {

constexpr int kScoreBins = 4096;

DEVI void hist_add(int* s_hist, float score) { atomicAdd(&s_hist[ordered_key(score) >> 20], 1); }

// NT threads clear / flush; a thread flushes the bins it cleared, so only the additions in
// between need a barrier on either side.  The flush reads all of a thread's bins before its
// first conditional add, so that the LDS reads are in flight together.
template <int NT>
DEVI void hist_zero(int* s_hist) {
    static_assert(kScoreBins % NT == 0, "bins per thread");
#pragma unroll
    for (int j = 0; j < kScoreBins / NT; ++j) s_hist[threadIdx.x + j * NT] = 0;
}
template <int NT>
DEVI void hist_flush(const int* s_hist, int* __restrict__ ghist) {
    int n[kScoreBins / NT];
#pragma unroll
    for (int j = 0; j < kScoreBins / NT; ++j) n[j] = s_hist[threadIdx.x + j * NT];
#pragma unroll
    for (int j = 0; j < kScoreBins / NT; ++j)
        if (n[j]) atomicAdd(ghist + threadIdx.x + j * NT, n[j]);
}

}  // namespace hylra
