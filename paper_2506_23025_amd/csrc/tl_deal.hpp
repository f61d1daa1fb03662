// Dealing out the workgroups of one launch to the GEMMs it carries (host side), shared by the
// weight-streaming kernels of both packed formats.
//
// A workgroup serves one job and walks a run of consecutive 16-row tiles of its matrix, in items
// of up to t_max tiles.  Its time, in units of an average tile, is
//     passes x (time of the run + start-up),
// where an item costs its latency and its barrier once (item_first for its first tile, tile_extra
// for each further one) and the start-up is what a workgroup does before its first tile (fetching
// the activation rows, building the operands).  Bisection on a common finishing time gives the
// fewest workgroups each job needs; spare workgroups go to the job with the costliest run.
#pragma once

namespace tl {

struct DealJob {
    int tiles;          // 16-row tiles of the job's matrix
    int passes;         // passes over K of a workgroup of this job
    double start_up;    // start-up of a pass, in tiles
};

struct DealModel {
    int t_max;          // tiles per item
    bool item_cost;     // count items (false: a run costs its tiles)
    double item_first;  // cost of the first tile of an item, in average tiles
    double tile_extra;  // cost of each further tile of an item
};

inline double deal_run_time(const DealModel& m, int run)
{
    if (!m.item_cost) return double(run);
    // a run of 4 goes as 2 + 2 when items hold 3
    const int items = run <= m.t_max ? 1 : ((m.t_max == 3 && run == 4) ? 2 : (run + m.t_max - 1) / m.t_max);
    return m.item_first * double(items) + m.tile_extra * double(run - items);
}

inline double deal_run_cost(const DealModel& m, const DealJob& j, int w)
{
    return double(j.passes) * (deal_run_time(m, (j.tiles + w - 1) / w) + j.start_up);
}

// fewest workgroups that finish job j by tau
inline int deal_groups_for(const DealModel& m, const DealJob& j, double tau)
{
    const double per = tau / double(j.passes) - j.start_up;
    // longest run that fits: from the estimate with whole items, a few steps up or down
    const double per_tile = m.item_cost ? (m.item_first + m.tile_extra * double(m.t_max - 1)) / double(m.t_max) : 1.0;
    int run = int(per / per_tile);
    if (run < 1) run = 1;
    if (run > j.tiles) run = j.tiles;
    while (run > 1 && deal_run_time(m, run) > per) --run;
    while (run < j.tiles && deal_run_time(m, run + 1) <= per) ++run;
    if (deal_run_time(m, run) > per) return j.tiles;
    const int w = (j.tiles + run - 1) / run;
    return w < 1 ? 1 : (w > j.tiles ? j.tiles : w);
}

// wg[j] >= 1 workgroups for job j, G in all when the jobs hold at least G tiles (fewer jobs than G)
inline void deal_workgroups(const DealModel& m, const DealJob* jobs, int count, int G, int* wg)
{
    double lo = 0.0, hi = 0.0;
    for (int j = 0; j < count; ++j) { const double c = deal_run_cost(m, jobs[j], 1); if (c > hi) hi = c; }
    for (int it = 0; it < 24; ++it) {
        const double mid = 0.5 * (lo + hi);
        int need = 0;
        for (int j = 0; j < count; ++j) need += deal_groups_for(m, jobs[j], mid);
        if (need <= G) hi = mid; else lo = mid;
    }
    int used = 0;
    for (int j = 0; j < count; ++j) { wg[j] = deal_groups_for(m, jobs[j], hi); used += wg[j]; }
    while (used < G) {                                     // spare groups: shorten the costliest run
        int best = -1;
        for (int j = 0; j < count; ++j)
            if (wg[j] < jobs[j].tiles &&
                (best < 0 || deal_run_cost(m, jobs[j], wg[j]) > deal_run_cost(m, jobs[best], wg[best]))) best = j;
        if (best < 0) break;
        ++wg[best]; ++used;
    }
    while (used > G) {                                     // cannot happen unless there are more jobs than groups
        int best = -1;
        for (int j = 0; j < count; ++j)
            if (wg[j] > 1 &&
                (best < 0 || deal_run_cost(m, jobs[j], wg[j]) < deal_run_cost(m, jobs[best], wg[best]))) best = j;
        if (best < 0) break;
        --wg[best]; --used;
    }
}

}  // namespace tl
