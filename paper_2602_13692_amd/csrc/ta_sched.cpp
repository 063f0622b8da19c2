// Program-aware scheduling tick (ThunderAgent Sec. 4.3): decayed capacity check per backend,
// Pause by S_pause, Restore by S_restore from one global waiting queue.  Host code.
#include <algorithm>
#include <cmath>
#include <vector>

#include "ta_sched.h"

namespace {

struct Policy {
    double hi, lo, base;
};

// tokens a program counts for in the capacity check
double weight_of(const ta_program& p, const Policy& pol) {
    const double c = static_cast<double>(p.context);
    if (p.phase == TA_PHASE_REASONING) return c;
    return c * std::pow(pol.base, -static_cast<double>(p.acting_time));
}

double load_of(const ta_program* programs, int32_t n, int32_t backend, const Policy& pol) {
    double total = 0.0;
    for (int32_t i = 0; i < n; ++i)
        if (programs[i].status == TA_STATUS_ACTIVE && programs[i].backend == backend)
            total += weight_of(programs[i], pol);
    return total;
}

double score(const ta_program& p, int favoured_phase) {
    return 1.0 / static_cast<double>(p.context) + (p.phase == favoured_phase ? 1.0 : 0.0);
}

bool valid(const ta_sched_config* c, const ta_program* programs, int32_t n, int32_t n_backends) {
    if (!(c->capacity_tokens >= 0.0) || !std::isfinite(c->capacity_tokens)) return false;
    if (!(c->lambda_max >= 0.0) || !std::isfinite(c->lambda_max)) return false;
    if (!(c->lambda_min >= 0.0) || !std::isfinite(c->lambda_min)) return false;
    if (!(c->decay_base >= 1.0) || !std::isfinite(c->decay_base)) return false;
    for (int32_t i = 0; i < n; ++i) {
        const ta_program& p = programs[i];
        if (p.context < 1) return false;
        if (p.phase != TA_PHASE_REASONING && p.phase != TA_PHASE_ACTING) return false;
        if (p.status != TA_STATUS_ACTIVE && p.status != TA_STATUS_PAUSED && p.status != TA_STATUS_TERMINATED)
            return false;
        if (p.status == TA_STATUS_ACTIVE && (p.backend < 0 || p.backend >= n_backends)) return false;
        if (!(p.acting_time >= 0.0f) || !std::isfinite(p.acting_time)) return false;
    }
    return true;
}

}  // namespace

extern "C" int ta_sched_tick(const ta_sched_config* config, ta_program* programs, int32_t n_programs,
                             int32_t n_backends, int32_t* paused_ids, int32_t* n_paused,
                             int32_t* restored_ids, int32_t* restored_backends, int32_t* n_restored) {
    if (!config || !n_paused || !n_restored || n_programs < 0 || n_backends < 0) return TA_ERR_INVALID_ARG;
    if (n_programs > 0 && (!programs || !paused_ids || !restored_ids || !restored_backends))
        return TA_ERR_INVALID_ARG;
    if (!valid(config, programs, n_programs, n_backends)) return TA_ERR_INVALID_ARG;
    const Policy pol{config->lambda_max * config->capacity_tokens, config->lambda_min * config->capacity_tokens,
                     config->decay_base};
    int32_t np = 0, nr = 0;

    // Pause: shed the highest S_pause until the backend is back under the high watermark
    for (int32_t b = 0; b < n_backends; ++b) {
        while (load_of(programs, n_programs, b, pol) > pol.hi) {
            int32_t victim = -1;
            for (int32_t i = 0; i < n_programs; ++i) {
                const ta_program& p = programs[i];
                if (p.status != TA_STATUS_ACTIVE || p.backend != b) continue;
                if (victim < 0) { victim = i; continue; }
                const double s = score(p, TA_PHASE_ACTING), best = score(programs[victim], TA_PHASE_ACTING);
                if (s > best || (s == best && p.id < programs[victim].id)) victim = i;
            }
            if (victim < 0) break;
            programs[victim].status = TA_STATUS_PAUSED;
            programs[victim].backend = -1;
            paused_ids[np++] = programs[victim].id;
        }
    }

    // Restore: the global waiting queue in descending S_restore
    std::vector<int32_t> queue;
    for (int32_t i = 0; i < n_programs; ++i)
        if (programs[i].status == TA_STATUS_PAUSED) queue.push_back(i);
    std::stable_sort(queue.begin(), queue.end(), [&](int32_t a, int32_t b) {
        const double sa = score(programs[a], TA_PHASE_REASONING), sb = score(programs[b], TA_PHASE_REASONING);
        if (sa != sb) return sa > sb;
        return programs[a].id < programs[b].id;
    });
    std::vector<double> loads(static_cast<size_t>(n_backends));
    for (int32_t i : queue) {
        for (int32_t b = 0; b < n_backends; ++b) loads[static_cast<size_t>(b)] = load_of(programs, n_programs, b, pol);
        int32_t best = -1;
        double best_room = 0.0;
        for (int32_t b = 0; b < n_backends; ++b) {
            const double room = pol.hi - loads[static_cast<size_t>(b)];
            if (loads[static_cast<size_t>(b)] < pol.lo && (best < 0 || room > best_room)) {
                best = b;
                best_room = room;
            }
        }
        if (best >= 0 && loads[static_cast<size_t>(best)] + weight_of(programs[i], pol) <= pol.hi) {
            programs[i].status = TA_STATUS_ACTIVE;
            programs[i].backend = best;
            restored_ids[nr] = programs[i].id;
            restored_backends[nr] = best;
            ++nr;
        }
    }
    *n_paused = np;
    *n_restored = nr;
    return TA_OK;
}
