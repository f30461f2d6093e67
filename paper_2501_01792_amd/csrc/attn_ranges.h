// How the attention kernels share the token positions of all (sequence, head) pairs among wavefronts,
// and how the merge finds the partials of a pair (Eq. 4 split over the token axis).  Plain integer
// arithmetic, callable from host and device code, so that it can be checked on a CPU.
//
// The positions form one line of `total` entries, pair-major.  Wavefront w of W takes the range
// [range_begin(w), range_begin(w + 1)); for every pair it meets it writes one partial at slot (w + pair).
// The merge of a pair reads slots owner(first position) + pair .. owner(last position) + pair, which are
// exactly the slots written for it PROVIDED no range between two working wavefronts is empty, i.e.
// W <= total: effective_waves() enforces that where `total` is only known on the device.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define HK_HOST_DEVICE __host__ __device__
#else
#define HK_HOST_DEVICE
#endif

namespace hk {
namespace ranges {

// First position of the range of wavefront w when `total` positions are cut into W ranges.
HK_HOST_DEVICE inline int64_t range_begin(int64_t w, int64_t total, int64_t W) { return (w * total) / W; }

// Wavefronts that take part when the line turns out to have `total` positions and the launch holds W.
HK_HOST_DEVICE inline int effective_waves(int W, int64_t total) { return total < (int64_t)W ? (int)(total > 0 ? total : 0) : W; }

// Wavefront whose range holds position x (0 <= x < total, 1 <= W <= total): the last one whose range
// begins at or before x.
HK_HOST_DEVICE inline int owner(int64_t x, int64_t total, int W)
{
    int64_t w = (x * W) / total;
    while (w + 1 < W && range_begin(w + 1, total, W) <= x) ++w;
    while (w > 0 && range_begin(w, total, W) > x) --w;
    return (int)w;
}

}  // namespace ranges
}  // namespace hk
