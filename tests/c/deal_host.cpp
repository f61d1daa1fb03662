// Host-side check of the allocator that deals a launch's workgroups out to its GEMMs
// (csrc/tl_deal.hpp): every job gets at least one workgroup and no more than it has tiles, the
// counts add up to the workgroups available whenever the jobs hold that many tiles, equal jobs get
// equal shares, a costlier job never gets fewer workgroups than a cheaper one of the same size,
// and no single move of a workgroup from one job to another shortens the longest run.
#include "tl_deal.hpp"

#include <cstdio>
#include <cstdlib>
#include <vector>

using namespace tl;

static int fail(const char* what, int a, int b)
{
    std::printf("FAILED: %s (%d, %d)\n", what, a, b);
    return 1;
}

static double makespan(const DealModel& m, const std::vector<DealJob>& jobs, const std::vector<int>& wg)
{
    double t = 0.0;
    for (size_t j = 0; j < jobs.size(); ++j) {
        const double c = deal_run_cost(m, jobs[j], wg[j]);
        if (c > t) t = c;
    }
    return t;
}

int main()
{
    const DealModel m{3, true, 2.1, 0.43};
    unsigned s = 12345u;
    auto rnd = [&](unsigned n) { s = s * 1664525u + 1013904223u; return (s >> 8) % n; };
    for (int trial = 0; trial < 400; ++trial) {
        const int count = 1 + int(rnd(32));
        std::vector<DealJob> jobs(count);
        long total = 0;
        for (auto& j : jobs) {
            j.tiles = 1 + int(rnd(trial % 3 == 0 ? 8 : 2000));
            j.passes = 1 + int(rnd(3));
            j.start_up = 0.15 * double(1 + rnd(16)) + (j.passes > 1 ? 1.5 : 0.0);
            total += j.tiles;
        }
        const int cap = 256;
        const int G = total < cap ? int(total) : cap;
        if (G < count) continue;                            // the launchers never ask for fewer groups than jobs
        std::vector<int> wg(count, -1);
        deal_workgroups(m, jobs.data(), count, G, wg.data());
        int used = 0;
        for (int j = 0; j < count; ++j) {
            if (wg[j] < 1) return fail("a job without a workgroup", trial, j);
            if (wg[j] > jobs[j].tiles) return fail("more workgroups than tiles", trial, j);
            used += wg[j];
        }
        if (used != G) return fail("counts do not add up", used, G);
        // no single move helps
        const double t0 = makespan(m, jobs, wg);
        for (int a = 0; a < count; ++a)
            for (int b = 0; b < count; ++b) {
                if (a == b || wg[a] <= 1 || wg[b] >= jobs[b].tiles) continue;
                std::vector<int> w2 = wg;
                --w2[a]; ++w2[b];
                if (makespan(m, jobs, w2) < t0 - 1e-9) return fail("a single move shortens the longest run", trial, a * 100 + b);
            }
    }
    // equal jobs, equal shares; and the sweep of the benchmark: five jobs of 256 tiles and five of 896,
    // 1, 2, 4, 8, 16 rows each
    {
        std::vector<DealJob> jobs(8, DealJob{500, 1, 0.15});
        std::vector<int> wg(8);
        deal_workgroups(m, jobs.data(), 8, 256, wg.data());
        for (int j = 0; j < 8; ++j)
            if (wg[j] != 32) return fail("equal jobs, unequal shares", j, wg[j]);
    }
    {
        std::vector<DealJob> jobs;
        for (int tiles : {256, 896})
            for (int rows : {1, 2, 4, 8, 16}) jobs.push_back(DealJob{tiles, 1, 0.15 * rows});
        std::vector<int> wg(jobs.size());
        deal_workgroups(m, jobs.data(), int(jobs.size()), 256, wg.data());
        for (int half = 0; half < 2; ++half)
            for (int i = 1; i < 5; ++i)
                if (wg[5 * half + i] < wg[5 * half + i - 1]) return fail("more rows, fewer workgroups", half, i);
        for (int i = 0; i < 5; ++i)
            if (wg[5 + i] <= wg[i]) return fail("more tiles, not more workgroups", i, wg[i]);
    }
    std::printf("ok\n");
    return 0;
}
