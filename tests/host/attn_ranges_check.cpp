// Host check of the slot bookkeeping shared by the attention kernels (csrc/attn_ranges.h): replays, with
// plain loops, which partial slots the wavefronts of a launch write and which slots the merge of every
// (request, head) pair reads, and counts reads of slots nobody wrote and slots written twice.
//   usage: attn_ranges_check H W clamp len_0 len_1 ...     (clamp = 1: the kernels' effective_waves; 0: none)
// prints: "<unwritten reads> <double writes> <pairs checked> <working wavefronts>"
#include "../../paper_2501_01792_amd/csrc/attn_ranges.h"

#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

int main(int argc, char **argv)
{
    if (argc < 5) return 2;
    const int H = atoi(argv[1]);
    int W = atoi(argv[2]);
    const bool clamp = atoi(argv[3]) != 0;
    std::vector<int64_t> len, cu(1, 0);
    for (int i = 4; i < argc; ++i) { len.push_back(atoll(argv[i])); cu.push_back(cu.back() + len.back()); }
    const int B = (int)len.size();
    const int64_t total = (int64_t)H * cu[B];
    if (clamp) W = hk::ranges::effective_waves(W, total);
    std::map<int64_t, int> written;                       // slot -> times written
    long double_writes = 0;
    for (int w = 0; w < W && total > 0; ++w) {
        int64_t p = hk::ranges::range_begin(w, total, W);
        const int64_t p_end = hk::ranges::range_begin(w + 1, total, W);
        int r = 0;
        while (p < p_end) {                               // one partial per pair the range meets
            while (p >= (int64_t)H * cu[r + 1]) ++r;
            const int64_t base = (int64_t)H * cu[r];
            const int h = (int)((p - base) / len[r]);
            const int64_t pair_end = base + (int64_t)(h + 1) * len[r];
            const int64_t slot = (int64_t)w + (int64_t)r * H + h;
            if (written[slot]++ > 0) ++double_writes;
            p = p_end < pair_end ? p_end : pair_end;
        }
    }
    long unwritten = 0, pairs = 0;
    for (int r = 0; r < B; ++r)
        for (int h = 0; h < H && len[r] > 0 && total > 0 && W > 0; ++h) {
            const int64_t lo = (int64_t)H * cu[r] + (int64_t)h * len[r], hi = lo + len[r] - 1;
            const int w_first = hk::ranges::owner(lo, total, W), w_last = hk::ranges::owner(hi, total, W);
            for (int w = w_first; w <= w_last; ++w)
                if (written.find((int64_t)w + (int64_t)r * H + h) == written.end()) ++unwritten;
            ++pairs;
        }
    printf("%ld %ld %ld %d\n", unwritten, double_writes, pairs, W);
    return 0;
}
