// Step plan of early-exit decoding with KV recomputation (Section 4; cap on the deferred list: Appendix D.3):
// the host arithmetic on a sequence's fill watermarks, free of any device state so that it can be checked on
// a machine without a GPU.  filled[s] = number of positions whose K and V are present in every layer of
// segment s (segment 0 = layers up to the first exit, ..., the last = layers above the last exit);
// filled[0] >= filled[1] >= ... always, and the deferred ("pending") tokens are the positions
// [filled[last], filled[0]).
#pragma once
#include <cstdint>

namespace ee {
namespace plan {

inline int pending(const int32_t* filled, int n_seg) { return filled[0] - filled[n_seg - 1]; }

// A step starts at full depth with the exits switched off once the deferred list has reached the cap
// (max_pending <= 0: there is no cap and no step is ever forced).
inline bool forced(const int32_t* filled, int n_seg, int max_pending) {
    return max_pending > 0 && pending(filled, n_seg) >= max_pending;
}

// Positions that pass through segment `seg` in a step whose current token sits at position p (p < 0: a flush,
// which has no current token): [lo, hi] inclusive.  Resumed rows enter where their KV is missing; re-fed rows
// (the paper's wording: the deferred tokens are included in the current forward pass) enter at layer 1.
inline void rows(const int32_t* filled, int n_seg, int seg, int p, bool refeed, int* lo, int* hi) {
    *lo = refeed ? filled[n_seg - 1] : filled[seg];
    *hi = p >= 0 ? p : filled[0] - 1;
}

// The step of the token at position p ended in segment `reached` (an exit fired there, or it is the last one):
// every segment up to it now holds K and V of all positions up to p.
inline void commit(int32_t* filled, int reached, int p) {
    for (int k = 0; k <= reached; ++k) filled[k] = p + 1;
}

// After a flush nothing is pending.
inline void flushed(int32_t* filled, int n_seg) {
    for (int k = 1; k < n_seg; ++k) filled[k] = filled[0];
}

}  // namespace plan
}  // namespace ee
