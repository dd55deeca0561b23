// Host-side lockstep harness for the sampling kernel's all-slots-at-once Floyd rule (csrc/zg_floyd.h), compiled
// with g++ by tests/test_floyd_parallel_rule.py.  For every candidate sequence of the given (deg, F) pairs it runs
// floyd_position for all F lanes of a group and compares the positions with the CPU checker's sequential
// zgo_floyd_resolve.
//
// The lanes of a wavefront exchange values in lockstep; here the lanes run one after another, so the harness
// replays the group several times: an exchange returns what the partner lane handed in at the same exchange of
// the previous replay.  The k-th exchange is right from replay k+1 on (it only depends on earlier exchanges), so
// after (number of exchanges + 1) replays every lane has seen exactly what a lockstep run would have shown it.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "zg_floyd.h"
#include "zg_oracle.h"

namespace {

struct ReplayGroup {
    int width;                                     // lanes of the group (a power of two >= F, as in the kernel)
    const uint32_t *cands;                         // every lane's candidate (handed in before the rule runs)
    std::vector<std::vector<int>> prev_flag, cur_flag; // [exchange][lane]
    std::vector<int> prev_any, cur_any;            // [exchange]
    int lane = 0, k_flag = 0, k_any = 0;

    uint32_t candidate_of(uint32_t j, uint32_t) const { return cands[j]; }
    bool flag_of(uint32_t j, bool mine)
    {
        if ((int)cur_flag.size() <= k_flag) cur_flag.resize(k_flag + 1, std::vector<int>(width, 0));
        cur_flag[k_flag][lane] = mine ? 1 : 0;
        const bool r = k_flag < (int)prev_flag.size() && prev_flag[k_flag][j] != 0;
        ++k_flag;
        return r;
    }
    bool any(bool b)
    {
        if ((int)cur_any.size() <= k_any) cur_any.resize(k_any + 1, 0);
        cur_any[k_any] |= b ? 1 : 0;
        const bool r = k_any < (int)prev_any.size() ? prev_any[k_any] != 0 : true; // unknown yet: keep going
        ++k_any;
        return r;
    }
    void begin_lane(int l) { lane = l; k_flag = k_any = 0; }
    void end_replay()
    {
        prev_flag.swap(cur_flag);
        prev_any.swap(cur_any);
        cur_flag.clear();
        cur_any.clear();
    }
};

// positions of all F slots by the parallel rule
void parallel_positions(int64_t deg, int F, const int64_t *t, int64_t *pos)
{
    int width = 4;
    while (width < F) width *= 2;
    std::vector<uint32_t> cand(width);
    for (int l = 0; l < width; ++l) cand[l] = l < F ? (uint32_t)t[l] : (uint32_t)l; // idle lanes hold their lane number
    ReplayGroup grp;
    grp.width = width;
    grp.cands = cand.data();
    const int replays = 2 * F + 2; // F rounds of (flag_of, any) at most
    for (int r = 0; r < replays; ++r) {
        for (int l = 0; l < width; ++l) {
            grp.begin_lane(l);
            const bool active = l < F;
            const uint32_t p = zg::floyd_position(grp, (uint32_t)l, (uint32_t)F, (uint32_t)deg, active, cand[l]);
            if (r == replays - 1 && l < F) pos[l] = p;
        }
        grp.end_replay();
    }
}

} // namespace

int main(int argc, char **argv)
{
    long cases = 0, bad = 0;
    for (int a = 1; a + 1 < argc; a += 2) {
        const int64_t deg = atoll(argv[a]);
        const int F = atoi(argv[a + 1]);
        if (F < 1 || F > 64 || deg <= F) return 2;
        std::vector<int64_t> t(F, 0), want(F), got(F);
        for (;;) { // odometer over t_j in [0, deg-F+j]
            zgo_floyd_resolve(deg, F, t.data(), want.data());
            parallel_positions(deg, F, t.data(), got.data());
            ++cases;
            if (want != got) {
                if (++bad <= 5) {
                    fprintf(stderr, "deg=%lld F=%d t=", (long long)deg, F);
                    for (int j = 0; j < F; ++j) fprintf(stderr, "%lld ", (long long)t[j]);
                    fprintf(stderr, "\n");
                }
            }
            int j = F - 1;
            while (j >= 0 && ++t[j] > deg - F + j) t[j--] = 0;
            if (j < 0) break;
        }
    }
    printf("%ld %ld\n", cases, bad);
    return bad ? 1 : 0;
}
