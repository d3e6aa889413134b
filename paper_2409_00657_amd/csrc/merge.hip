// Micrograph merging (paper section 5.3): host-side bookkeeping only - which time step to
// merge away, how its root vertices are re-dealt, and the epoch-time examination that decides
// how many steps to merge.  No device work: these calls read and write HOST memory.
#include "common.hpp"

using namespace hopgnn;

extern "C" int32_t hopgnn_merge_min_step(const int64_t* counts, int32_t n_models, int32_t n_steps) {
    if (counts == nullptr || n_models < 1 || n_steps < 1) return -1;
    int32_t best = 0;
    int64_t best_total = -1;
    for (int32_t t = 0; t < n_steps; ++t) {
        int64_t total = 0;
        for (int32_t m = 0; m < n_models; ++m) {
            if (counts[(int64_t)m * n_steps + t] < 0) return -1;
            total += counts[(int64_t)m * n_steps + t];
        }
        if (best_total < 0 || total < best_total) {
            best_total = total;
            best = t;
        }
    }
    return best;
}

extern "C" int32_t hopgnn_merge_apply(int64_t* counts, int32_t n_models, int32_t n_steps, int32_t ts) {
    if (counts == nullptr || n_models < 1 || n_steps < 2 || ts < 0 || ts >= n_steps) return -1;
    const int32_t others = n_steps - 1;
    for (int32_t m = 0; m < n_models; ++m) {
        int64_t* row = counts + (int64_t)m * n_steps;
        const int64_t c = row[ts], share = c / others, extra = c % others;
        int32_t k = 0;   // position among the remaining steps, in step order
        for (int32_t t = 0; t < n_steps; ++t) {
            if (t == ts) continue;
            row[t] += share + (k < extra ? 1 : 0);
            ++k;
        }
    }
    // drop column ts: compact every row to n_steps - 1 entries, rows stay contiguous
    int64_t w = 0;
    for (int32_t m = 0; m < n_models; ++m)
        for (int32_t t = 0; t < n_steps; ++t)
            if (t != ts) counts[w++] = counts[(int64_t)m * n_steps + t];
    return others;
}

extern "C" hopgnn_status hopgnn_merge_ctl_init(hopgnn_merge_ctl* ctl, int32_t n_servers) {
    if (ctl == nullptr || n_servers < 1) return HOPGNN_EINVAL;
    ctl->n_steps = n_servers;
    ctl->settled = n_servers == 1 ? 1 : 0;
    ctl->epochs_seen = 0;
    ctl->prev_time = 0.0;
    return HOPGNN_OK;
}

extern "C" int32_t hopgnn_merge_ctl_report(hopgnn_merge_ctl* ctl, double epoch_time) {
    if (ctl == nullptr || !(epoch_time >= 0.0)) return -1;
    ctl->epochs_seen += 1;
    if (ctl->settled) return ctl->n_steps;
    if (ctl->epochs_seen == 1) {            // first epoch: the unmerged baseline; examination starts
        ctl->prev_time = epoch_time;        // with the second epoch, one step merged
        ctl->n_steps -= 1;
        return ctl->n_steps;
    }
    if (epoch_time < ctl->prev_time) {      // the last merge paid off: keep it, try one more
        ctl->prev_time = epoch_time;
        if (ctl->n_steps > 1) {
            ctl->n_steps -= 1;
        } else {
            ctl->settled = 1;
        }
    } else {                                // it did not: back to the pattern before it, for good
        ctl->n_steps += 1;
        ctl->settled = 1;
    }
    return ctl->n_steps;
}
