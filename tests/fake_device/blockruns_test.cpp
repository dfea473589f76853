// The shim's block allocator against a bitmap: random allocations and releases; first fit means the
// lowest run that is long enough; released neighbours must merge, so that the number of free runs
// always equals the number of maximal zero runs of the bitmap.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "blockruns.hpp"

int main(int argc, char **argv) {
    const uint64_t seed = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 1;
    uint64_t rng = seed * 0x9E3779B97F4A7C15ull + 1;
    auto rnd = [&]() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return rng; };
    const uint64_t N = 200 + seed % 57;
    nixie::BlockRuns runs(N);
    std::vector<int> used(N, 0);
    std::vector<std::pair<uint64_t, uint64_t>> live;
    for (int step = 0; step < 20000; step++) {
        if (live.empty() || rnd() % 3) {
            const uint64_t n = 1 + rnd() % 12;
            uint64_t want = nixie::BlockRuns::kNone;          // brute force: lowest position with n zeros
            for (uint64_t i = 0; i + n <= N && want == nixie::BlockRuns::kNone; i++) {
                bool ok = true;
                for (uint64_t j = i; j < i + n; j++) ok = ok && !used[j];
                if (ok) want = i;
            }
            const uint64_t got = runs.find(n);
            if (got != want) { std::printf("step %d: find(%llu) = %llu, bitmap says %llu\n", step, (unsigned long long)n, (unsigned long long)got, (unsigned long long)want); return 1; }
            if (got == nixie::BlockRuns::kNone) continue;
            runs.take(got, n);
            for (uint64_t j = got; j < got + n; j++) used[j] = 1;
            live.push_back({got, n});
        } else {
            const size_t k = rnd() % live.size();
            runs.give(live[k].first, live[k].second);
            for (uint64_t j = live[k].first; j < live[k].first + live[k].second; j++) used[j] = 0;
            live[k] = live.back();
            live.pop_back();
        }
        uint64_t zeros = 0, zero_runs = 0;
        for (uint64_t i = 0; i < N; i++) {
            zeros += !used[i];
            zero_runs += !used[i] && (i == 0 || used[i - 1]);
        }
        if (runs.free_blocks() != zeros || runs.runs() != zero_runs) {
            std::printf("step %d: %llu free blocks in %zu runs, bitmap has %llu in %llu\n", step, (unsigned long long)runs.free_blocks(),
                        runs.runs(), (unsigned long long)zeros, (unsigned long long)zero_runs);
            return 1;
        }
    }
    if (runs.find(0) != nixie::BlockRuns::kNone) return 1;
    std::printf("ok seed %llu\n", (unsigned long long)seed);
    return 0;
}
