// Trace-driven simulator of the program-aware policy over several backends (ThunderAgent
// Sec. 4.1 and 4.3: the program table, the periodic decision, the global waiting queue; App. B:
// workflows with tool calls of heavy-tailed latency).  Host code.  It turns every decision into
// an ordered list of events (evict, restore, prefill, decode, release) with the pool pages they
// concern, so that a driver can carry them out with the device calls of ta.h.
#include <algorithm>
#include <new>
#include <vector>

#include "ta_sched.h"

namespace {

constexpr int32_t kPage = 16;

int32_t pages_of(int64_t tokens) { return static_cast<int32_t>((tokens + kPage - 1) / kPage); }

struct Workflow {
    int32_t turn = 0;          // index of the current reasoning turn
    int32_t tokens_left = 0;   // tokens still to decode in it
    int32_t tool_left = 0;     // ticks until the running tool returns
    int32_t pending = 0;       // tool-output tokens waiting to be prefilled
};

}  // namespace

struct ta_sim {
    ta_sim_config cfg;
    std::vector<ta_program> table;
    std::vector<Workflow> flow;
    std::vector<int32_t> turn_tokens, tool_ticks, tool_tokens;
    std::vector<std::vector<int32_t>> pages;      // per program, logical order
    std::vector<std::vector<int32_t>> free_pages; // per backend, taken from the back
    std::vector<ta_sim_event> events;
    std::vector<int32_t> slots;
    std::vector<int32_t> paused_ids, restored_ids, restored_backends;

    int32_t trace(const std::vector<int32_t>& a, int32_t p, int32_t turn) const {
        return a[static_cast<size_t>(p) * cfg.n_turns + turn];
    }

    void emit(int32_t kind, int32_t p, int32_t backend, int32_t tokens, const int32_t* s, size_t n) {
        ta_sim_event e{};
        e.kind = kind;
        e.program = p;
        e.backend = backend;
        e.tokens = tokens;
        e.context = table[p].context;
        e.first_slot = static_cast<int32_t>(slots.size());
        e.n_slots = static_cast<int32_t>(n);
        slots.insert(slots.end(), s, s + n);
        events.push_back(e);
    }

    // the program's pages go back to its backend's free list
    void give_up_pages(int32_t kind, int32_t p) {
        const int32_t b = table[p].backend;
        emit(kind, p, b, table[p].context, pages[p].data(), pages[p].size());
        if (b >= 0)
            for (auto it = pages[p].rbegin(); it != pages[p].rend(); ++it) free_pages[b].push_back(*it);
        pages[p].clear();
    }

    double pause_score(int32_t p) const {
        return 1.0 / static_cast<double>(table[p].context) + (table[p].phase == TA_PHASE_ACTING ? 1.0 : 0.0);
    }

    // Makes `need` pages free on backend b by reclaiming idle caches (see ta_sched.h): only
    // programs waiting for a tool are candidates, and programs flagged in `served` are not
    // touched.  Returns false when that is not possible.
    bool make_room(int32_t b, int32_t need, const std::vector<char>& served) {
        while (static_cast<int32_t>(free_pages[b].size()) < need) {
            int32_t victim = -1;
            for (int32_t i = 0; i < cfg.n_programs; ++i) {
                if (table[i].status != TA_STATUS_ACTIVE || table[i].backend != b || served[i]) continue;
                if (table[i].phase != TA_PHASE_ACTING) continue;
                if (victim < 0 || pause_score(i) > pause_score(victim)) victim = i;   // ties: lower id
            }
            if (victim < 0) return false;
            give_up_pages(TA_SIM_EVICT_FORCED, victim);
            table[victim].status = TA_STATUS_PAUSED;
            table[victim].backend = -1;
        }
        return true;
    }

    // Takes `n` pages from backend b's free list onto the tail of p's page list; returns the
    // index of the first new page in pages[p].
    size_t take_pages(int32_t p, int32_t b, int32_t n) {
        const size_t first = pages[p].size();
        for (int32_t i = 0; i < n; ++i) {
            pages[p].push_back(free_pages[b].back());
            free_pages[b].pop_back();
        }
        return first;
    }

    void release(int32_t p) {
        give_up_pages(TA_SIM_RELEASE, p);
        table[p].status = TA_STATUS_TERMINATED;
        table[p].backend = -1;
    }

    // Grows an active program to new_context tokens; `kind` says why.  A program that cannot
    // get its pages leaves the backend itself.
    void grow(int32_t kind, int32_t p, int32_t new_context, int32_t tokens) {
        const int32_t b = table[p].backend;
        const int32_t need = pages_of(new_context) - static_cast<int32_t>(pages[p].size());
        std::vector<char> served(static_cast<size_t>(cfg.n_programs), 0);
        served[p] = 1;
        if (need > 0 && !make_room(b, need, served)) {
            give_up_pages(TA_SIM_EVICT_FORCED, p);
            table[p].status = TA_STATUS_PAUSED;
            table[p].backend = -1;
            return;
        }
        const size_t first = take_pages(p, b, need > 0 ? need : 0);
        table[p].context = new_context;
        emit(kind, p, b, tokens, pages[p].data() + first, pages[p].size() - first);
    }

    void tick() {
        events.clear();
        slots.clear();
        const int32_t n = cfg.n_programs;
        // 1. tools
        for (int32_t p = 0; p < n; ++p) {
            if (table[p].status == TA_STATUS_TERMINATED || table[p].phase != TA_PHASE_ACTING) continue;
            table[p].acting_time += static_cast<float>(cfg.time_per_tick);
            if (--flow[p].tool_left > 0) continue;
            flow[p].pending = trace(tool_tokens, p, flow[p].turn);
            flow[p].turn += 1;
            flow[p].tokens_left = flow[p].turn < cfg.n_turns ? trace(turn_tokens, p, flow[p].turn) : 0;
            table[p].phase = TA_PHASE_REASONING;
            table[p].acting_time = 0.0f;
        }
        // 2. the policy
        int32_t np = 0, nr = 0;
        std::vector<int32_t> before(static_cast<size_t>(n));
        for (int32_t p = 0; p < n; ++p) before[p] = table[p].backend;
        ta_sched_tick(&cfg.sched, table.data(), n, cfg.n_backends, paused_ids.data(), &np, restored_ids.data(),
                      restored_backends.data(), &nr);
        std::vector<char> served(static_cast<size_t>(n), 0);
        for (int32_t i = 0; i < nr; ++i) served[restored_ids[i]] = 1;
        for (int32_t i = 0; i < np; ++i) {
            const int32_t p = paused_ids[i];
            const int32_t now = table[p].backend;           // -1, or a new backend if the tick restored it at once
            table[p].backend = before[p];                   // the pages sit in the pool it was paused on
            give_up_pages(TA_SIM_EVICT, p);
            table[p].backend = now;
        }
        for (int32_t i = 0; i < nr; ++i) {
            const int32_t p = restored_ids[i], b = restored_backends[i];
            const int32_t need = pages_of(table[p].context);
            if (!make_room(b, need, served)) {              // no room after all: back to the waiting queue
                table[p].status = TA_STATUS_PAUSED;
                table[p].backend = -1;
                served[p] = 0;
                continue;
            }
            take_pages(p, b, need);
            emit(TA_SIM_RESTORE, p, b, table[p].context, pages[p].data(), pages[p].size());
        }
        auto running = [&](int32_t p) {
            return table[p].status == TA_STATUS_ACTIVE && table[p].phase == TA_PHASE_REASONING;
        };
        // 3. tool output waiting to be prefilled
        for (int32_t p = 0; p < n; ++p) {
            if (!running(p) || flow[p].pending == 0) continue;
            const int64_t new_context = int64_t(table[p].context) + flow[p].pending;
            if (new_context > cfg.max_context) {
                release(p);
                continue;
            }
            const int32_t tokens = flow[p].pending;
            grow(TA_SIM_PREFILL, p, static_cast<int32_t>(new_context), tokens);
            if (table[p].status == TA_STATUS_ACTIVE) flow[p].pending = 0;
        }
        // 4. decode steps
        for (int32_t step = 0; step < cfg.steps_per_tick; ++step)
            for (int32_t p = 0; p < n; ++p) {
                if (!running(p) || flow[p].pending != 0 || flow[p].tokens_left == 0) continue;
                if (table[p].context + 1 > cfg.max_context) {
                    release(p);
                    continue;
                }
                grow(TA_SIM_DECODE, p, table[p].context + 1, step);
                if (table[p].status == TA_STATUS_ACTIVE) flow[p].tokens_left -= 1;
            }
        // 5. finished turns
        for (int32_t p = 0; p < n; ++p) {
            if (!running(p) || flow[p].pending != 0 || flow[p].tokens_left != 0) continue;
            if (flow[p].turn >= cfg.n_turns) {
                release(p);
                continue;
            }
            table[p].phase = TA_PHASE_ACTING;
            table[p].acting_time = 0.0f;
            flow[p].tool_left = trace(tool_ticks, p, flow[p].turn);
        }
    }
};

extern "C" {

ta_sim* ta_sim_create(const ta_sim_config* config, const int32_t* initial_context, const int32_t* turn_tokens,
                      const int32_t* tool_ticks, const int32_t* tool_tokens) {
    if (!config || !initial_context || !turn_tokens || !tool_ticks || !tool_tokens) return nullptr;
    const ta_sim_config& c = *config;
    if (c.n_programs < 1 || c.n_backends < 1 || c.n_turns < 1 || c.pool_pages < 1 || c.steps_per_tick < 0 ||
        c.max_context < 1 || !(c.time_per_tick >= 0.0))
        return nullptr;
    const size_t cells = static_cast<size_t>(c.n_programs) * c.n_turns;
    for (int32_t p = 0; p < c.n_programs; ++p)
        if (initial_context[p] < 1 || initial_context[p] > c.max_context) return nullptr;
    for (size_t i = 0; i < cells; ++i)
        if (turn_tokens[i] < 1 || tool_ticks[i] < 1 || tool_tokens[i] < 1) return nullptr;
    ta_sim* s = new (std::nothrow) ta_sim();
    if (!s) return nullptr;
    s->cfg = c;
    s->table.resize(c.n_programs);
    s->flow.resize(c.n_programs);
    s->pages.resize(c.n_programs);
    s->free_pages.resize(c.n_backends);
    s->paused_ids.resize(c.n_programs);
    s->restored_ids.resize(c.n_programs);
    s->restored_backends.resize(c.n_programs);
    s->turn_tokens.assign(turn_tokens, turn_tokens + cells);
    s->tool_ticks.assign(tool_ticks, tool_ticks + cells);
    s->tool_tokens.assign(tool_tokens, tool_tokens + cells);
    for (int32_t b = 0; b < c.n_backends; ++b)
        for (int32_t page = c.pool_pages - 1; page >= 0; --page) s->free_pages[b].push_back(page);   // page 0 goes first
    for (int32_t p = 0; p < c.n_programs; ++p) {
        ta_program& t = s->table[p];
        t.id = p;
        t.context = initial_context[p];
        t.backend = -1;
        t.phase = TA_PHASE_REASONING;
        t.status = TA_STATUS_PAUSED;
        t.acting_time = 0.0f;
        s->flow[p].tokens_left = turn_tokens[static_cast<size_t>(p) * c.n_turns];
    }
    // a configuration the policy itself rejects is rejected here
    int32_t np = 0, nr = 0;
    std::vector<ta_program> probe = s->table;
    if (ta_sched_tick(&s->cfg.sched, probe.data(), c.n_programs, c.n_backends, s->paused_ids.data(), &np,
                      s->restored_ids.data(), s->restored_backends.data(), &nr) != TA_OK) {
        delete s;
        return nullptr;
    }
    return s;
}

void ta_sim_destroy(ta_sim* sim) { delete sim; }

int ta_sim_tick(ta_sim* sim, int32_t* n_events, int32_t* n_slots) {
    if (!sim || !n_events || !n_slots) return TA_ERR_INVALID_ARG;
    sim->tick();
    *n_events = static_cast<int32_t>(sim->events.size());
    *n_slots = static_cast<int32_t>(sim->slots.size());
    return TA_OK;
}

int ta_sim_fetch(const ta_sim* sim, ta_sim_event* events, int32_t* slots) {
    if (!sim || (!events && !sim->events.empty()) || (!slots && !sim->slots.empty())) return TA_ERR_INVALID_ARG;
    std::copy(sim->events.begin(), sim->events.end(), events);
    std::copy(sim->slots.begin(), sim->slots.end(), slots);
    return TA_OK;
}

int ta_sim_programs(const ta_sim* sim, ta_program* out) {
    if (!sim || !out) return TA_ERR_INVALID_ARG;
    std::copy(sim->table.begin(), sim->table.end(), out);
    return TA_OK;
}

int32_t ta_sim_page_table(const ta_sim* sim, int32_t program, int32_t* out, int32_t max_pages) {
    if (!sim || program < 0 || program >= sim->cfg.n_programs || max_pages < 0 || (max_pages > 0 && !out)) return -1;
    const std::vector<int32_t>& pg = sim->pages[program];
    const size_t n = std::min(pg.size(), static_cast<size_t>(max_pages));
    std::copy(pg.begin(), pg.begin() + n, out);
    return static_cast<int32_t>(pg.size());
}

}  // extern "C"
