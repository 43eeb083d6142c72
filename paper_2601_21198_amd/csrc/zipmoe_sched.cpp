// Cache-affinity scheduling of the reconstruction tasks of one sparse layer: ZipMoE (arXiv 2601.21198)
// Sec. 3.3 "Cache-Affinity Scheduler" (task partition, block construction), App. A (Alg. 1, the
// compute-dominant test, work-conserving execution in block priority order) and App. B (charged time,
// lower bounds on the optimum).  Host only, double precision.
//
// The timeline of a priority list is computed resource by resource, because the dependencies only run one
// way: the I/O thread depends on nothing, the decompression threads only on E-chunk arrivals, the GPU
// stream on both.
#include "zipmoe.h"

#include <algorithm>
#include <cmath>
#include <functional>
#include <new>
#include <queue>
#include <utility>
#include <vector>

namespace {

struct Problem {
    const zm_sched_task *tasks;
    int n_tasks;
    const double *p;
    int n_experts;
    zm_sched_costs k;
};

struct Blocks {
    std::vector<int32_t> order;       // task indices, highest priority first
    std::vector<int32_t> end;         // end position of each block
};

struct Outcome {
    zm_sched_result totals{};
    std::vector<double> worker_end;
    std::vector<zm_sched_event> events;
};

inline bool decodes(const zm_sched_task &t) { return t.needs_decode != 0; }
inline bool type_one(const zm_sched_task &t) { return decodes(t) && t.needs_sm != 0; }
inline bool reads_e(const zm_sched_task &t) { return decodes(t) && t.needs_e != 0; }

bool valid(const Problem &q)
{
    if (!q.tasks || !q.p || q.n_tasks < 0 || q.n_experts < 0) return false;
    const double c[4] = {q.k.sm_read, q.k.e_read, q.k.decompress, q.k.recover};
    for (double x : c)
        if (!(x >= 0.0) || !std::isfinite(x)) return false;
    if (q.k.threads < 1 || q.k.shards < 1) return false;
    for (int j = 0; j < q.n_tasks; ++j)
        if (q.tasks[j].expert < 0 || q.tasks[j].expert >= q.n_experts) return false;
    for (int n = 0; n < q.n_experts; ++n)
        if (!(q.p[n] >= 0.0) || !std::isfinite(q.p[n])) return false;
    return true;
}

// The timeline of the listed tasks.  `keep_events` is off while blocks are being built.
void run(const Problem &q, const Blocks &b, bool keep_events, Outcome &out)
{
    const int K = q.k.shards, L = q.k.threads;
    const int n_listed = static_cast<int>(b.order.size());
    out.events.clear();
    auto note = [&](int kind, int task, int chunk, int unit, double s, double e) {
        if (keep_events) out.events.push_back(zm_sched_event{kind, task, chunk, unit, s, e});
    };

    // I/O thread: back to back; per block the E-chunks of its tasks, then the SM-chunks.
    std::vector<std::vector<double>> e_at(n_listed);
    std::vector<double> sm_at(n_listed, 0.0);
    double t = 0.0;
    int begin = 0;
    for (int32_t stop : b.end) {
        for (int pos = begin; pos < stop; ++pos) {
            if (!reads_e(q.tasks[b.order[pos]])) continue;
            e_at[pos].resize(K);
            for (int i = 0; i < K; ++i) {
                note(ZM_OP_E_READ, b.order[pos], i, 0, t, t + q.k.e_read);
                t = t + q.k.e_read;
                e_at[pos][i] = t;
            }
        }
        for (int pos = begin; pos < stop; ++pos) {
            if (!type_one(q.tasks[b.order[pos]])) continue;
            note(ZM_OP_SM_READ, b.order[pos], 0, 0, t, t + q.k.sm_read);
            t = t + q.k.sm_read;
            sm_at[pos] = t;
        }
        begin = stop;
    }
    out.totals.io_end = t;

    // Decompression threads.  Operations are numbered in priority order: id = rank * K + chunk over the
    // positions that decode.  Those that wait for a read arrive in the order the I/O thread runs them,
    // which is their priority order too, so one cursor walks them; those with nothing to read are ready
    // from the start.
    std::vector<int> dec_pos;
    for (int pos = 0; pos < n_listed; ++pos)
        if (decodes(q.tasks[b.order[pos]])) dec_pos.push_back(pos);
    const long n_ops = static_cast<long>(dec_pos.size()) * K;
    std::priority_queue<long, std::vector<long>, std::greater<long>> ready;
    std::vector<long> arriving;
    arriving.reserve(static_cast<size_t>(n_ops));
    for (size_t r = 0; r < dec_pos.size(); ++r)
        for (int i = 0; i < K; ++i) {
            const long id = static_cast<long>(r) * K + i;
            if (e_at[dec_pos[r]].empty()) ready.push(id); else arriving.push_back(id);
        }
    auto arrival = [&](long id) { return e_at[dec_pos[id / K]][id % K]; };
    size_t cursor = 0;
    using Slot = std::pair<double, int>;               // (free at, thread)
    std::priority_queue<Slot, std::vector<Slot>, std::greater<Slot>> threads;
    for (int w = 0; w < L; ++w) threads.push(Slot(0.0, w));
    out.worker_end.assign(L, 0.0);
    std::vector<double> decoded_at(n_listed, 0.0);
    double charge = 0.0;
    for (long done = 0; done < n_ops; ++done) {
        const Slot slot = threads.top();
        threads.pop();
        double now = slot.first;
        while (cursor < arriving.size() && arrival(arriving[cursor]) <= now) ready.push(arriving[cursor++]);
        if (ready.empty()) {                            // nothing has arrived: wait for the next read to end
            now = arrival(arriving[cursor]);
            while (cursor < arriving.size() && arrival(arriving[cursor]) <= now) ready.push(arriving[cursor++]);
        }
        const long id = ready.top();
        ready.pop();
        const int pos = dec_pos[id / K];
        charge += now - slot.first;
        const double end = now + q.k.decompress;
        note(ZM_OP_DECOMPRESS, b.order[pos], static_cast<int>(id % K), slot.second, now, end);
        threads.push(Slot(end, slot.second));
        out.worker_end[slot.second] = end;
        decoded_at[pos] = std::max(decoded_at[pos], end);
    }
    out.totals.charge = charge;

    // GPU stream.  Items in priority order: the recovery of each decoding position, and each expert's
    // execution right behind the expert's last position.
    struct Item { int pos; int kind; int id; double ready; bool known; bool placed; };
    std::vector<Item> items;
    std::vector<int> last_pos(q.n_experts, -1), waiting(q.n_experts, 0);
    std::vector<double> expert_ready(q.n_experts, 0.0);
    for (int pos = 0; pos < n_listed; ++pos) {
        const zm_sched_task &tk = q.tasks[b.order[pos]];
        last_pos[tk.expert] = pos;
        if (decodes(tk)) ++waiting[tk.expert];
    }
    for (int pos = 0; pos < n_listed; ++pos) {
        const zm_sched_task &tk = q.tasks[b.order[pos]];
        if (decodes(tk)) items.push_back(Item{pos, ZM_OP_RECOVER, pos, std::max(decoded_at[pos], sm_at[pos]), true, false});
        if (last_pos[tk.expert] == pos) items.push_back(Item{pos, ZM_OP_EXECUTE, tk.expert, 0.0, waiting[tk.expert] == 0, false});
    }
    double gpu = 0.0;
    for (size_t placed = 0; placed < items.size(); ++placed) {
        Item *pick = nullptr;
        double soonest = 0.0;
        bool any = false;
        for (Item &it : items) {
            if (it.placed || !it.known) continue;
            if (it.ready <= gpu) { pick = &it; break; }
            if (!any || it.ready < soonest) { soonest = it.ready; any = true; }
        }
        double now = gpu;
        if (!pick) {
            now = soonest;
            for (Item &it : items)
                if (!it.placed && it.known && it.ready <= now) { pick = &it; break; }
        }
        pick->placed = true;
        if (pick->kind == ZM_OP_RECOVER) {
            const int task = b.order[pick->id];
            const int n = q.tasks[task].expert;
            gpu = now + q.k.recover;
            note(ZM_OP_RECOVER, task, 0, 0, now, gpu);
            expert_ready[n] = std::max(expert_ready[n], gpu);
            if (--waiting[n] == 0)
                for (Item &it : items)
                    if (it.kind == ZM_OP_EXECUTE && it.id == n) { it.ready = expert_ready[n]; it.known = true; }
        } else {
            gpu = now + q.p[pick->id];
            note(ZM_OP_EXECUTE, pick->id, 0, 0, now, gpu);
        }
    }
    out.totals.makespan = gpu;
}

bool compute_dominant(const Outcome &o, const zm_sched_costs &k)
{
    std::vector<double> ends(o.worker_end);
    std::sort(ends.begin(), ends.end());
    const int top = std::min(k.threads, k.shards);
    for (int l = 1; l <= top; ++l)
        if (!(ends[l - 1] - o.totals.io_end >= l * k.e_read)) return false;
    return true;
}

// Sec. 3.3 "Task Partition": one class in priority order.
std::vector<int32_t> sorted_class(const Problem &q, bool want_type_one)
{
    std::vector<int32_t> v;
    for (int j = 0; j < q.n_tasks; ++j)
        if (type_one(q.tasks[j]) == want_type_one) v.push_back(j);
    std::stable_sort(v.begin(), v.end(), [&](int32_t a, int32_t b) {
        const int ea = q.tasks[a].expert, eb = q.tasks[b].expert;
        if (q.p[ea] != q.p[eb]) return q.p[ea] > q.p[eb];
        if (ea != eb) return ea < eb;
        return a < b;
    });
    return v;
}

void build(const Problem &q, Blocks &done)
{
    std::vector<int32_t> one = sorted_class(q, true), two = sorted_class(q, false);
    size_t at_one = 0, at_two = 0;
    done.order.clear();
    done.end.clear();
    Outcome now, trial;
    Blocks work;
    while (at_one < one.size()) {
        const size_t base = done.order.size();          // where the open block starts
        work = done;
        work.order.push_back(one[at_one++]);
        work.end.push_back(static_cast<int32_t>(work.order.size()));
        while (at_one < one.size() || at_two < two.size()) {
            run(q, work, false, now);
            if (compute_dominant(now, q.k)) break;
            const int32_t j = at_two < two.size() ? two[at_two++] : one[at_one++];
            const double limit = now.totals.charge + 1e-12 * (1.0 + now.totals.charge);
            const size_t len = work.order.size() - base;
            work.end.back() += 1;
            bool placed = false;
            for (size_t pos = 0; pos <= len && !placed; ++pos) {
                work.order.insert(work.order.begin() + base + pos, j);
                run(q, work, false, trial);
                placed = trial.totals.charge <= limit;
                if (!placed) work.order.erase(work.order.begin() + base + pos);
            }
            if (placed) continue;
            bool has_two = false;
            for (size_t i = base; i < work.order.size(); ++i) has_two = has_two || !type_one(q.tasks[work.order[i]]);
            const double pj = q.p[q.tasks[j].expert];
            size_t at = work.order.size();
            for (size_t i = work.order.size(); i-- > base;) {
                const zm_sched_task &o = q.tasks[work.order[i]];
                if (type_one(o) != has_two && q.p[o.expert] >= pj) { at = i + 1; break; }
            }
            work.order.insert(work.order.begin() + at, j);
        }
        done = work;
    }
    if (at_two < two.size()) {
        done.order.insert(done.order.end(), two.begin() + at_two, two.end());
        done.end.push_back(static_cast<int32_t>(done.order.size()));
    }
}

}  // namespace

extern "C" {

int zm_sched_build(const zm_sched_task *tasks, int n_tasks, const double *expert_time, int n_experts,
                   const zm_sched_costs *costs, int32_t *order_out, int32_t *block_end_out, int *n_blocks_out)
{
    if (!costs || !order_out || !block_end_out || !n_blocks_out) return ZM_E_ARG;
    const Problem q{tasks, n_tasks, expert_time, n_experts, *costs};
    if (!valid(q)) return ZM_E_ARG;
    try {
        Blocks b;
        build(q, b);
        std::copy(b.order.begin(), b.order.end(), order_out);
        std::copy(b.end.begin(), b.end.end(), block_end_out);
        *n_blocks_out = static_cast<int>(b.end.size());
    } catch (const std::bad_alloc &) {
        return ZM_E_NOMEM;
    }
    return ZM_OK;
}

int zm_sched_simulate(const zm_sched_task *tasks, int n_tasks, const double *expert_time, int n_experts,
                      const zm_sched_costs *costs, const int32_t *order, const int32_t *block_end, int n_blocks,
                      zm_sched_result *result, double *worker_end_out,
                      zm_sched_event *events_out, size_t events_cap, size_t *n_events_out)
{
    if (!costs || !result || n_blocks < 0 || (n_blocks > 0 && (!order || !block_end))) return ZM_E_ARG;
    const Problem q{tasks, n_tasks, expert_time, n_experts, *costs};
    if (!valid(q)) return ZM_E_ARG;
    try {
        Blocks b;
        int32_t prev = 0;
        for (int i = 0; i < n_blocks; ++i) {
            if (block_end[i] < prev || block_end[i] > n_tasks) return ZM_E_ARG;
            prev = block_end[i];
            b.end.push_back(prev);
        }
        std::vector<char> seen(static_cast<size_t>(n_tasks), 0);
        for (int32_t pos = 0; pos < prev; ++pos) {
            if (order[pos] < 0 || order[pos] >= n_tasks || seen[order[pos]]) return ZM_E_ARG;
            seen[order[pos]] = 1;
            b.order.push_back(order[pos]);
        }
        Outcome o;
        run(q, b, events_out != nullptr || n_events_out != nullptr, o);
        *result = o.totals;
        if (worker_end_out) std::copy(o.worker_end.begin(), o.worker_end.end(), worker_end_out);
        if (n_events_out) *n_events_out = o.events.size();
        if (events_out) std::copy(o.events.begin(), o.events.begin() + std::min(events_cap, o.events.size()), events_out);
    } catch (const std::bad_alloc &) {
        return ZM_E_NOMEM;
    }
    return ZM_OK;
}

int zm_sched_lower_bounds(const zm_sched_task *tasks, int n_tasks, const double *expert_time, int n_experts,
                          const zm_sched_costs *costs, double bounds_out[4])
{
    if (!costs || !bounds_out) return ZM_E_ARG;
    const Problem q{tasks, n_tasks, expert_time, n_experts, *costs};
    if (!valid(q)) return ZM_E_ARG;
    try {
        const int K = costs->shards;
        const int width = std::min(K, costs->threads);
        const int rounds = (K + width - 1) / width;
        double io = 0.0, work = 0.0, chain = 0.0, exec = 0.0;
        std::vector<char> named(static_cast<size_t>(n_experts), 0);
        for (int j = 0; j < n_tasks; ++j) {
            const zm_sched_task &t = tasks[j];
            const double p = expert_time[t.expert];
            if (!named[t.expert]) { named[t.expert] = 1; exec += p; }
            if (!decodes(t)) { chain = std::max(chain, p); continue; }
            const double e_reads = reads_e(t) ? K * costs->e_read : 0.0;
            const double reads = e_reads + (type_one(t) ? costs->sm_read : 0.0);
            // the last chunk cannot be decoded before it has arrived; the busiest thread cannot start
            // before the first one has
            const double decoded = reads_e(t) ? std::max(e_reads + costs->decompress, costs->e_read + rounds * costs->decompress)
                                              : rounds * costs->decompress;
            io += reads;
            work += K * costs->decompress;
            chain = std::max(chain, std::max(decoded, reads) + costs->recover + p);
        }
        bounds_out[0] = io;
        bounds_out[1] = work / costs->threads;
        bounds_out[2] = exec;
        bounds_out[3] = chain;
    } catch (const std::bad_alloc &) {
        return ZM_E_NOMEM;
    }
    return ZM_OK;
}

}  // extern "C"
