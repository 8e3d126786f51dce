// Host planner: prefix programs -> trees -> labels -> pools -> executor work lists.
//
// Paper: Background / Visual Reasoning Programs (a function sequence plus fixed arities gives a
// unique tree, assembled depth first); Methods / Improved topological sort (label = distance from
// the root, pool equal labels, at most p calls per pool) and Standard topological sort (queue per
// program, b x s grid run column by column); Discussion (batching by dependency depth, as
// TensorFlow Fold does: label = one more than the deepest argument).  Results / IEP asks for exactly this code to be
// multithreaded native code because in the authors' Python it took over half of the run time.
//
// No GPU call in this file: it can be built and tested on a machine without a GPU.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <new>
#include <thread>

#include "plan_internal.h"

namespace dynb {

static thread_local std::string g_error;

void set_error(const std::string& msg) { g_error = msg; }

int fail(int code, const std::string& msg)
{
    g_error = msg;
    return code;
}

namespace {

struct Frame {
    int32_t node;     // position inside the example
    uint8_t filled;   // arguments already started
    uint8_t arity;
};

// Parses example `ex`; fills root distance, dependency depth, children and queue position.
// Returns false if the sequence is not exactly one complete tree.
bool parse_example(const int32_t* prog, int32_t base, int32_t len, const uint8_t* arity,
                   int32_t n_types, int32_t* rootdist, int32_t* depdepth, int32_t* child0, int32_t* child1,
                   int32_t* queue_pos, std::vector<Frame>& stack)
{
    if (len <= 0) return false;
    stack.clear();
    int32_t done = 0;
    for (int32_t pos = 0; pos < len; ++pos) {
        const int32_t t = prog[base + pos];
        if (t < 0 || t >= n_types) return false;
        const int32_t id = base + pos;
        child0[id] = child1[id] = -1;
        if (pos == 0) {
            rootdist[id] = 0;
        } else {
            if (stack.empty()) return false;              // tokens left after the tree closed
            Frame& par = stack.back();
            const int32_t pid = base + par.node;
            (par.filled == 0 ? child0 : child1)[pid] = id;
            ++par.filled;
            rootdist[id] = rootdist[pid] + 1;
        }
        if (arity[t] == 0) {
            queue_pos[id] = done++;
            depdepth[id] = 0;
            // every enclosing function whose last argument just closed enters the queue too;
            // its arguments' depths are final by then
            while (!stack.empty() && stack.back().filled == stack.back().arity) {
                const int32_t fid = base + stack.back().node;
                queue_pos[fid] = done++;
                int32_t deepest = depdepth[child0[fid]];
                if (child1[fid] >= 0) deepest = std::max(deepest, depdepth[child1[fid]]);
                depdepth[fid] = deepest + 1;
                stack.pop_back();
            }
        } else {
            stack.push_back(Frame{pos, 0, arity[t]});
        }
    }
    return stack.empty();
}

}  // namespace
}  // namespace dynb

using dynb::fail;

namespace {

// Pools and executor work lists from labels, arguments and roots (p->level, type, child0, child1,
// root).  `example` maps a node to its example, `queue_pos` is the per-example post-order position
// (only read by the naive schedule), `shared` says that a node may have several consumers.
void build_lists(dynb_plan* p, const uint8_t* arity, const int32_t* prog_off, const std::vector<int32_t>& example,
                 const std::vector<int32_t>& queue_pos, bool balance, bool shared)
{
    const int32_t B = p->B, N = p->N, D = p->D, n_types = p->n_types, mode = p->mode;
    const bool improved = (mode == DYNB_SCHED_IMPROVED), by_depth = (mode == DYNB_SCHED_DEPTH);
    if (shared) balance = false;                     // the pull-forward pass assumes one consumer per node
    // ---- pools: stable counting sort of node ids by (execution step, function id)
    p->members.resize(N); p->in0.resize(N); p->in1.resize(N); p->out.resize(N);
    if (mode == DYNB_SCHED_NAIVE) {
        // one pool per node, example by example in queue order
        for (int32_t i = 0; i < B; ++i) {
            const int32_t base = prog_off[i], len = prog_off[i + 1] - base;
            for (int32_t j = 0; j < len; ++j) p->members[base + queue_pos[base + j]] = base + j;
        }
        p->b_level.resize(N); p->b_type.resize(N); p->b_start.resize(N); p->b_count.assign(N, 1);
        for (int32_t s = 0; s < N; ++s) {
            const int32_t n = p->members[s];
            p->b_level[s] = p->level[n]; p->b_type[s] = p->type[n]; p->b_start[s] = s;
        }
    } else {
        const size_t n_keys = size_t(D) * size_t(n_types);
        std::vector<int32_t> hist(n_keys + 1, 0);
        auto key = [&](int32_t n) {
            const int32_t step = improved ? D - 1 - p->level[n] : p->level[n];
            return size_t(step) * n_types + size_t(p->type[n]);
        };
        for (int32_t n = 0; n < N; ++n) ++hist[key(n) + 1];
        for (size_t q = 0; q < n_keys; ++q) {
            if (hist[q + 1] > 0) {
                const int32_t step = int32_t(q / n_types);
                p->b_level.push_back(improved ? D - 1 - step : step);
                p->b_type.push_back(int32_t(q % n_types));
                p->b_start.push_back(hist[q]);
                p->b_count.push_back(hist[q + 1]);
            }
            hist[q + 1] += hist[q];
        }
        for (int32_t n = 0; n < N; ++n) p->members[hist[key(n)]++] = n;   // ascending ids inside a pool
    }
    for (int32_t s = 0; s < N; ++s) {
        const int32_t n = p->members[s];
        p->in0[s] = p->child0[n]; p->in1[s] = p->child1[n]; p->out[s] = n;
    }

    // ---- executor work lists: items in execution order, launch groups, slots
    // 1. launch group of every compute node, in the logical order of the pools
    p->node_launch.assign(N, -1);
    std::vector<int32_t> order;                       // compute nodes in execution order
    int32_t n_launch = 0;
    {
        int32_t cur_label = -1;
        for (int32_t s = 0; s < N; ++s) {
            const int32_t n = p->members[s];
            if (arity[p->type[n]] == 0) continue;
            if (arity[p->type[n]] == 2) p->has_binary = true;
            if (mode == DYNB_SCHED_NAIVE || p->level[n] != cur_label) { ++n_launch; cur_label = p->level[n]; }
            p->node_launch[n] = n_launch - 1;
            order.push_back(n);
        }
    }
    const int32_t n_compute = int32_t(order.size());
    auto is_compute = [&](int32_t c) { return c >= 0 && arity[p->type[c]] > 0; };

    // 2. optional balancing of the improved sort.  A label only fixes the LATEST launch group a
    // node may run in; a node whose arguments finish early can run earlier.  Launch groups with
    // more nodes than the chip has CUs (256) cost a second round, so nodes are pulled forward out
    // of such groups into earlier groups that have idle CUs (earliest deadline first).  The paper
    // mentions in its Discussion that the execution order could be optimised and leaves it aside.
    if (improved && balance && n_launch > 1) {
        const int32_t S = n_launch;
        constexpr int32_t CUS = 256, HALF_CUS = 128;
        std::vector<int32_t> remaining(S, 0), pending(N, 0), ready_at(N, 0), assigned(N, -1), parent(N, -1);
        for (int32_t n : order) {
            ++remaining[p->node_launch[n]];
            for (int32_t c : {p->child0[n], p->child1[n]})
                if (is_compute(c)) { ++pending[n]; parent[c] = n; }
        }
        // `order` is grouped by deadline already.  Size classes of the executor: up to 128 nodes a
        // group runs with two CUs per node, up to 256 with one, beyond that in two rounds.
        std::vector<int32_t> first_of(S + 1, 0);
        for (int32_t n : order) ++first_of[p->node_launch[n] + 1];
        for (int32_t L = 0; L < S; ++L) first_of[L + 1] += first_of[L];
        std::vector<int32_t> size_at(S, 0);             // nodes currently scheduled in a group
        std::vector<char> gives(S, 0);                  // groups above the smallest size class
        std::vector<int32_t> givers;
        for (int32_t L = 0; L < S; ++L)
            if (remaining[L] > HALF_CUS) { gives[L] = 1; givers.push_back(L); }
        std::vector<std::vector<int32_t>> ready(S);
        for (int32_t L : givers) ready[L].reserve(remaining[L]);
        for (int32_t n : order)
            if (pending[n] == 0 && gives[p->node_launch[n]]) ready[p->node_launch[n]].push_back(n);
        auto assign = [&](int32_t n, int32_t s) {
            assigned[n] = s;
            ++size_at[s];
            --remaining[p->node_launch[n]];
            const int32_t q = parent[n];
            if (q >= 0) {
                ready_at[q] = std::max(ready_at[q], s + 1);
                if (--pending[q] == 0 && gives[p->node_launch[q]]) ready[p->node_launch[q]].push_back(q);
            }
        };
        // pass 0: every node at its deadline unless it is pulled forward out of a group wider than
        // the chip (those come down to 256); earlier groups are filled up to their size class
        for (int32_t s = 0; s < S; ++s) {
            for (int32_t i = first_of[s]; i < first_of[s + 1]; ++i)
                if (assigned[order[i]] < 0) assign(order[i], s);
            const int32_t here = size_at[s];
            const int32_t cap = here <= HALF_CUS ? HALF_CUS : (here <= CUS ? CUS : here);
            for (int32_t L : givers) {
                if (size_at[s] >= cap) break;
                if (L <= s || remaining[L] <= CUS) continue;
                auto& pool = ready[L];
                size_t keep = 0;
                for (size_t i = 0; i < pool.size(); ++i) {
                    const int32_t n = pool[i];
                    if (size_at[s] < cap && remaining[L] > CUS && ready_at[n] <= s) assign(n, s);
                    else pool[keep++] = n;
                }
                pool.resize(keep);
            }
        }
        // pass 1: with the room that is left below 128, bring groups of 129..256 nodes down to 128,
        // earliest deadline first (ready_at is a safe upper bound: arguments only ever move earlier)
        std::vector<std::vector<int32_t>> at(S);
        for (int32_t L : givers)
            if (size_at[L] > HALF_CUS && size_at[L] <= CUS) at[L].reserve(size_at[L]);
        for (int32_t n : order) {
            const int32_t L = assigned[n];
            if (size_at[L] > HALF_CUS && size_at[L] <= CUS) at[L].push_back(n);
        }
        for (int32_t s = 0; s < S; ++s) {
            if (size_at[s] >= HALF_CUS) continue;
            for (int32_t L : givers) {
                if (size_at[s] >= HALF_CUS) break;
                if (L <= s || size_at[L] <= HALF_CUS || size_at[L] > CUS) continue;
                auto& pool = at[L];
                size_t keep = 0;
                for (size_t i = 0; i < pool.size(); ++i) {
                    const int32_t n = pool[i];
                    if (size_at[s] < HALF_CUS && size_at[L] > HALF_CUS && ready_at[n] <= s) {
                        assigned[n] = s; ++size_at[s]; --size_at[L];
                    } else pool[keep++] = n;
                }
                pool.resize(keep);
            }
        }
        for (int32_t n : order) p->node_launch[n] = assigned[n];
        // execution order: launch group, then function id (weights stay hot), then node id
        std::vector<int32_t> start(size_t(S) * n_types + 1, 0);
        auto key = [&](int32_t n) { return size_t(p->node_launch[n]) * n_types + size_t(p->type[n]); };
        for (int32_t n : order) ++start[key(n) + 1];
        for (size_t q = 0; q + 1 < start.size(); ++q) start[q + 1] += start[q];
        std::vector<int32_t> sorted(order.size());
        for (int32_t n = 0; n < N; ++n)                       // ascending node id inside a (group, function) run
            if (p->node_launch[n] >= 0) sorted[start[key(n)]++] = n;
        order.swap(sorted);
    }

    // 3. slots and items
    std::vector<int32_t> slot(N, -1);
    {
        // Root-distance labels put every argument exactly one label below its consumer, so two
        // alternating halves suffice.  Balanced and dependency-depth plans keep a result for several
        // groups: they recycle slots through a free list once the consuming group has been issued.
        // A shared node lives until its last consumer has been issued (use counts).
        // One dependency-driven launch per batch has no label boundary after which a slot could be reused:
        // every result keeps a slot of its own.
        const bool own_slots = p->persistent || p->keep;
        const bool pingpong = improved && !balance && !shared && !own_slots;
        const bool recycle = ((improved && balance) || by_depth || shared) && !own_slots;
        std::vector<int32_t> uses;
        if (recycle) {
            uses.assign(N, 0);
            for (int32_t n : order)
                for (int32_t c : {p->child0[n], p->child1[n]})
                    if (c >= 0) ++uses[c];
        }
        int32_t maxw = 0, running = 0;
        std::vector<int32_t> rank_in_level(D, 0);
        if (pingpong) {
            std::vector<int32_t> width(D, 0);
            for (int32_t n : order) ++width[p->level[n]];
            for (int32_t l = 0; l < D; ++l) maxw = std::max(maxw, width[l]);
        }
        std::vector<int32_t> free_slots, release;     // balanced plans recycle slots through a free list
        p->items.reserve(n_compute);
        int32_t cur = -1;
        for (int32_t n : order) {
            if (p->node_launch[n] != cur) {
                // slots of arguments consumed by the previous group may be reused from here on
                free_slots.insert(free_slots.end(), release.begin(), release.end());
                release.clear();
                p->launches.push_back(dynb_launch{int32_t(p->items.size()), 0, 0});
                cur = p->node_launch[n];
            }
            const bool is_root = (n == p->root[example[n]]);
            if (pingpong) {
                // arguments of a label-l node all sit at label l+1: two alternating halves suffice
                slot[n] = (p->level[n] & 1) * maxw + rank_in_level[p->level[n]]++;
            } else if (!is_root) {
                if (recycle && !free_slots.empty()) { slot[n] = free_slots.back(); free_slots.pop_back(); }
                else slot[n] = running++;
            }
            auto src = [&](int32_t c) -> int32_t {
                if (c < 0) return 0;
                if (!is_compute(c)) return -1 - example[c];
                if (recycle && --uses[c] == 0) release.push_back(slot[c]);
                return slot[c];
            };
            dynb_item it;
            it.src0 = src(p->child0[n]);
            it.src1 = src(p->child1[n]);
            it.dst = is_root ? -1 - example[n] : slot[n];
            it.type = p->type[n];
            ++p->launches.back().count;
            if (arity[it.type] == 2) p->launches.back().any_binary = 1;
            p->items.push_back(it);
            p->item_node.push_back(n);
        }
        p->n_slots = pingpong ? 2 * maxw : running;
        for (const auto& l : p->launches) p->max_launch = std::max(p->max_launch, l.count);
    }
    // 3b. routes of the backward pass: the gradient with respect to an argument goes to the item that evaluated
    // it, or to a numbered SCENE leaf (summed per example afterwards, in leaf order)
    if (p->keep) {
        std::vector<int32_t> item_of(N, -1), leaf_of(N, -1);
        for (size_t i = 0; i < p->item_node.size(); ++i) item_of[p->item_node[i]] = int32_t(i);
        p->leaf_first.assign(size_t(B) + 1, 0);
        int32_t n_leaf = 0;
        for (int32_t n = 0; n < N; ++n) {                   // node ids ascend example by example
            if (arity[p->type[n]] == 0) leaf_of[n] = n_leaf++;
            p->leaf_first[example[n] + 1] = n_leaf;
        }
        for (int32_t e = 0; e < B; ++e) p->leaf_first[e + 1] = std::max(p->leaf_first[e + 1], p->leaf_first[e]);
        auto route = [&](int32_t c) -> int32_t { return c < 0 ? 0 : (item_of[c] >= 0 ? item_of[c] : -1 - leaf_of[c]); };
        p->grad_dst0.resize(p->items.size()); p->grad_dst1.resize(p->items.size());
        for (size_t i = 0; i < p->items.size(); ++i) {
            const int32_t n = p->item_node[i];
            p->grad_dst0[i] = route(p->child0[n]);
            p->grad_dst1[i] = route(p->child1[n]);
        }
        p->root_item.resize(B);
        for (int32_t e = 0; e < B; ++e) p->root_item[e] = item_of[p->root[e]];
        // the items of every function in execution order (counting sort): a function's parameter gradients are
        // summed over this list
        p->fn_first.assign(size_t(p->n_types) + 1, 0);
        for (const dynb_item& it : p->items) ++p->fn_first[size_t(it.type) + 1];
        for (int32_t t = 0; t < p->n_types; ++t) p->fn_first[t + 1] += p->fn_first[t];
        p->fn_items.resize(p->items.size());
        std::vector<int32_t> at(p->fn_first.begin(), p->fn_first.end() - 1);
        for (size_t i = 0; i < p->items.size(); ++i) p->fn_items[at[p->items[i].type]++] = int32_t(i);
        // units of the parameter-gradient kernel
        // (every function has its groups, also those without a gradient of that kind: their sum is zero; the
        // conv1x1 groups exist only if the batch uses a two-argument function at all)
        for (int32_t mode = 0; mode < (p->has_binary ? 3 : 2); ++mode)
            for (int32_t t = 0; t < p->n_types; ++t) {
                const bool has_units = arity[t] != 0 && (mode != 2 || arity[t] == 2);
                const int32_t lo = p->fn_first[t], hi = has_units ? p->fn_first[t + 1] : lo;
                for (int32_t part = 0; part < (mode == 2 ? 2 : 3); ++part) {
                    dynb_wg_group g{mode, t, part, int32_t(p->wg_units.size()), 0, 0, 0, 0};
                    for (int32_t b = lo; b < hi; b += DYNB_WG_CHUNK) {
                        p->wg_units.push_back(dynb_wg_unit{mode, t, part, b, std::min(hi, b + DYNB_WG_CHUNK), 0, 0, 0});
                        ++g.n_units;
                    }
                    p->wg_groups.push_back(g);                     // a function without items has no units: its gradient is zero
                }
            }
        // Order in which workgroups take the units: chunks with the most items first (a short tail), and the parts of
        // one chunk (its kernel rows / arguments read the same maps) 8 workgroups apart: consecutive workgroups go
        // to the chip's 8 dies in turn, so those parts run on one die at the same time and share its L2.
        struct Chunk { int32_t first_group, n_parts, chunk, work; };
        std::vector<Chunk> chunks;
        for (size_t gi = 0; gi < p->wg_groups.size();) {
            const dynb_wg_group& g0 = p->wg_groups[gi];
            const int32_t n_parts = g0.mode == 2 ? 2 : 3;
            for (int32_t c = 0; c < g0.n_units; ++c) {
                const dynb_wg_unit& u = p->wg_units[g0.first_unit + c];
                chunks.push_back(Chunk{int32_t(gi), n_parts, c, (u.end - u.begin) * (g0.mode == 2 ? 1 : 3)});
            }
            gi += size_t(n_parts);
        }
        std::stable_sort(chunks.begin(), chunks.end(), [](const Chunk& a, const Chunk& b) {
            return a.n_parts != b.n_parts ? a.n_parts > b.n_parts : a.work > b.work;
        });
        p->wg_order.clear();
        for (size_t b0 = 0; b0 < chunks.size(); b0 += 8)
            for (int32_t part = 0; part < 3; ++part)
                for (size_t x = b0; x < std::min(chunks.size(), b0 + 8); ++x)
                    if (part < chunks[x].n_parts)
                        p->wg_order.push_back(p->wg_groups[size_t(chunks[x].first_group) + part].first_unit + chunks[x].chunk);
    }
    // 4. units of work of the dependency-driven launch, in claim order = execution order of the items
    // (arguments always come earlier in it).  Groups that leave half of the chip idle are run with two
    // workgroups per node (upper and lower half of the map), like the per-label executor does.
    if (p->persistent) {
        p->tickets.reserve(2 * p->items.size());
        for (const auto& l : p->launches)
            for (int32_t i = l.start; i < l.start + l.count; ++i) {
                if (l.count <= 128) { p->tickets.push_back(4 * i + 1); p->tickets.push_back(4 * i + 2); }
                else p->tickets.push_back(4 * i);
            }
    }
    for (int32_t i = 0; i < B; ++i)
        if (arity[p->type[p->root[i]]] == 0) p->leaf_roots.push_back(i);
}

}  // namespace

extern "C" const char* dynb_last_error(void) { return dynb::g_error.c_str(); }

extern "C" int dynbatch_plan(const int32_t* prog, const int32_t* prog_off, int32_t B,
                             const uint8_t* arity, int32_t n_types, uint32_t flags, dynb_plan** out)
{
    if (out) *out = nullptr;
    if (!prog || !prog_off || !arity || !out) return fail(DYNB_E_INVAL, "dynbatch_plan: NULL argument");
    if (B <= 0 || n_types <= 0) return fail(DYNB_E_INVAL, "dynbatch_plan: B and n_types must be positive");
    if (flags & ~uint32_t(DYNB_SCHED_MASK | DYNB_PLAN_BALANCE | DYNB_PLAN_THROUGHPUT | DYNB_PLAN_PERSISTENT | DYNB_PLAN_KEEP)) return fail(DYNB_E_UNSUPPORTED, "dynbatch_plan: unknown flag bits");
    const int32_t mode = int32_t(flags & DYNB_SCHED_MASK);
    // one dependency-driven launch per batch sizes its units of work by the balanced launch groups
    const bool persistent = (flags & DYNB_PLAN_PERSISTENT) != 0 && mode != DYNB_SCHED_NAIVE;
    const bool balance = (flags & DYNB_PLAN_BALANCE) != 0 || persistent;
    for (int32_t t = 0; t < n_types; ++t)
        if (arity[t] > 2)
            return fail(DYNB_E_UNSUPPORTED, "dynbatch_plan: function " + std::to_string(t) + " has arity > 2");
    if (prog_off[0] != 0) return fail(DYNB_E_INVAL, "dynbatch_plan: prog_off[0] must be 0");
    for (int32_t i = 0; i < B; ++i)
        if (prog_off[i + 1] < prog_off[i]) return fail(DYNB_E_INVAL, "dynbatch_plan: prog_off must not decrease");

    dynb_plan* p = new (std::nothrow) dynb_plan;
    if (!p) return fail(DYNB_E_NOMEM, "dynbatch_plan: out of host memory");
    try {
        const int32_t N = prog_off[B];
        p->B = B; p->N = N; p->n_types = n_types; p->mode = mode;
        p->throughput = (flags & DYNB_PLAN_THROUGHPUT) != 0;
        p->persistent = persistent;
        p->keep = (flags & DYNB_PLAN_KEEP) != 0;
        p->arity.assign(arity, arity + n_types);
        p->level.resize(N); p->type.assign(prog, prog + N);
        p->child0.resize(N); p->child1.resize(N); p->root.resize(B);
        std::vector<int32_t> rootdist(N), depdepth(N), queue_pos(N), example(N);

        // ---- trees: examples are independent, so large batches are parsed by several threads
        std::atomic<int32_t> first_bad(B);
        auto work = [&](int32_t lo, int32_t hi) {
            std::vector<dynb::Frame> stack;
            stack.reserve(64);
            for (int32_t i = lo; i < hi; ++i) {
                const int32_t base = prog_off[i], len = prog_off[i + 1] - base;
                bool ok = dynb::parse_example(prog, base, len, arity, n_types, rootdist.data(), depdepth.data(),
                                              p->child0.data(), p->child1.data(), queue_pos.data(), stack);
                if (!ok) {
                    int32_t cur = first_bad.load();
                    while (i < cur && !first_bad.compare_exchange_weak(cur, i)) {}
                    continue;
                }
                p->root[i] = base;
                for (int32_t j = 0; j < len; ++j) example[base + j] = i;
            }
        };
        unsigned nthr = 1;
        if (N >= (1 << 15)) nthr = std::min<unsigned>(std::max(1u, std::thread::hardware_concurrency()), 16u);
        nthr = std::min<unsigned>(nthr, unsigned(B));
        if (nthr <= 1) {
            work(0, B);
        } else {
            std::vector<std::thread> pool;
            for (unsigned k = 0; k < nthr; ++k)
                pool.emplace_back(work, int32_t(int64_t(B) * k / nthr), int32_t(int64_t(B) * (k + 1) / nthr));
            for (auto& th : pool) th.join();
        }
        if (first_bad.load() < B) {
            const int32_t i = first_bad.load();
            delete p;
            return fail(DYNB_E_MALFORMED, "dynbatch_plan: example " + std::to_string(i) +
                                              " is not a complete prefix tree");
        }

        // ---- labels
        const bool improved = (mode == DYNB_SCHED_IMPROVED), by_depth = (mode == DYNB_SCHED_DEPTH);
        int32_t D = 0;
        for (int32_t n = 0; n < N; ++n) {
            p->level[n] = improved ? rootdist[n] : by_depth ? depdepth[n] : queue_pos[n];
            D = std::max(D, p->level[n] + 1);
        }
        p->D = D;

        build_lists(p, arity, prog_off, example, queue_pos, balance, false);
    } catch (const std::bad_alloc&) {
        delete p;
        return fail(DYNB_E_NOMEM, "dynbatch_plan: out of host memory");
    }
    *out = p;
    return DYNB_OK;
}

namespace {

// Labels of one dependency graph (nodes [base, base + n), argument indices local to the example).
// Returns false if it is malformed: a function id or argument index out of range, an argument
// count that differs from the arity, a cycle, or a node the root does not depend on.
bool label_graph(const int32_t* type, const int32_t* arg0, const int32_t* arg1, int32_t base, int32_t n,
                 int32_t root, const uint8_t* arity, int32_t n_types, int32_t* rootdist, int32_t* depdepth,
                 int32_t* queue_pos, std::vector<int32_t>& post, std::vector<int32_t>& stack, std::vector<uint8_t>& state)
{
    if (n <= 0 || root < 0 || root >= n) return false;
    for (int32_t j = 0; j < n; ++j) {
        const int32_t t = type[base + j], a = arg0[base + j], b = arg1[base + j];
        if (t < 0 || t >= n_types || a < -1 || a >= n || b < -1 || b >= n) return false;
        if ((a >= 0) + (b >= 0) != arity[t] || (b >= 0 && a < 0)) return false;
    }
    // depth-first from the root with an explicit stack: state 0 unseen, 1 open (on the path), 2 closed;
    // a node enters `post` when all its arguments are closed
    post.clear(); stack.clear(); state.assign(size_t(n), 0);
    stack.push_back(root);
    while (!stack.empty()) {
        const int32_t j = stack.back();
        if (state[j] == 2) { stack.pop_back(); continue; }
        if (state[j] == 0) {
            state[j] = 1;
            for (int32_t a : {arg1[base + j], arg0[base + j]}) {
                if (a < 0) continue;
                if (state[a] == 1) return false;                  // back edge: a cycle
                if (state[a] == 0) stack.push_back(a);
            }
        } else {                                                  // arguments done
            state[j] = 2;
            queue_pos[base + j] = int32_t(post.size());
            post.push_back(j);
            stack.pop_back();
        }
    }
    if (int32_t(post.size()) != n) return false;                  // some node does not feed the root
    for (int32_t j : post) {                                      // arguments before consumers
        int32_t d = 0;
        for (int32_t a : {arg0[base + j], arg1[base + j]})
            if (a >= 0) d = std::max(d, depdepth[base + a] + 1);
        depdepth[base + j] = d;
    }
    for (int32_t j = 0; j < n; ++j) rootdist[base + j] = -1;
    rootdist[base + root] = 0;
    for (auto it = post.rbegin(); it != post.rend(); ++it)        // consumers before arguments: longest path
        for (int32_t a : {arg0[base + *it], arg1[base + *it]})
            if (a >= 0) rootdist[base + a] = std::max(rootdist[base + a], rootdist[base + *it] + 1);
    return true;
}

}  // namespace

extern "C" int dynbatch_plan_dag(const int32_t* type, const int32_t* arg0, const int32_t* arg1, const int32_t* node_off,
                                 const int32_t* root, int32_t B, const uint8_t* arity, int32_t n_types,
                                 uint32_t flags, dynb_plan** out)
{
    if (out) *out = nullptr;
    if (!type || !arg0 || !arg1 || !node_off || !root || !arity || !out)
        return fail(DYNB_E_INVAL, "dynbatch_plan_dag: NULL argument");
    if (B <= 0 || n_types <= 0) return fail(DYNB_E_INVAL, "dynbatch_plan_dag: B and n_types must be positive");
    if (flags & ~uint32_t(DYNB_SCHED_MASK | DYNB_PLAN_BALANCE | DYNB_PLAN_THROUGHPUT | DYNB_PLAN_PERSISTENT | DYNB_PLAN_KEEP))
        return fail(DYNB_E_UNSUPPORTED, "dynbatch_plan_dag: unknown flag bits");
    const int32_t mode = int32_t(flags & DYNB_SCHED_MASK);
    if (mode != DYNB_SCHED_IMPROVED && mode != DYNB_SCHED_DEPTH)
        return fail(DYNB_E_UNSUPPORTED, "dynbatch_plan_dag: graphs are scheduled by root distance or dependency depth only");
    for (int32_t t = 0; t < n_types; ++t)
        if (arity[t] > 2)
            return fail(DYNB_E_UNSUPPORTED, "dynbatch_plan_dag: function " + std::to_string(t) + " has arity > 2");
    if (node_off[0] != 0) return fail(DYNB_E_INVAL, "dynbatch_plan_dag: node_off[0] must be 0");
    for (int32_t i = 0; i < B; ++i)
        if (node_off[i + 1] < node_off[i]) return fail(DYNB_E_INVAL, "dynbatch_plan_dag: node_off must not decrease");

    dynb_plan* p = new (std::nothrow) dynb_plan;
    if (!p) return fail(DYNB_E_NOMEM, "dynbatch_plan_dag: out of host memory");
    try {
        const int32_t N = node_off[B];
        p->B = B; p->N = N; p->n_types = n_types; p->mode = mode;
        p->throughput = (flags & DYNB_PLAN_THROUGHPUT) != 0;
        p->persistent = (flags & DYNB_PLAN_PERSISTENT) != 0;
        p->keep = (flags & DYNB_PLAN_KEEP) != 0;
        p->shared_nodes = true;
        p->arity.assign(arity, arity + n_types);
        p->level.resize(N); p->type.assign(type, type + N);
        p->child0.resize(N); p->child1.resize(N); p->root.resize(B);
        std::vector<int32_t> rootdist(N), depdepth(N), queue_pos(N), example(N), post, stack;
        std::vector<uint8_t> state;
        for (int32_t i = 0; i < B; ++i) {
            const int32_t base = node_off[i], n = node_off[i + 1] - base;
            if (!label_graph(type, arg0, arg1, base, n, root[i], arity, n_types, rootdist.data(), depdepth.data(),
                             queue_pos.data(), post, stack, state)) {
                delete p;
                return fail(DYNB_E_MALFORMED, "dynbatch_plan_dag: example " + std::to_string(i) +
                                                  " is not a well-formed dependency graph");
            }
            p->root[i] = base + root[i];
            for (int32_t j = 0; j < n; ++j) {
                example[base + j] = i;
                p->child0[base + j] = arg0[base + j] >= 0 ? base + arg0[base + j] : -1;
                p->child1[base + j] = arg1[base + j] >= 0 ? base + arg1[base + j] : -1;
            }
        }
        int32_t D = 0;
        for (int32_t n = 0; n < N; ++n) {
            p->level[n] = mode == DYNB_SCHED_IMPROVED ? rootdist[n] : depdepth[n];
            D = std::max(D, p->level[n] + 1);
        }
        p->D = D;
        build_lists(p, arity, node_off, example, queue_pos, false, true);
    } catch (const std::bad_alloc&) {
        delete p;
        return fail(DYNB_E_NOMEM, "dynbatch_plan_dag: out of host memory");
    }
    *out = p;
    return DYNB_OK;
}

extern "C" int dynbatch_plan_view(const dynb_plan* p, dynb_plan_view* v)
{
    if (!p || !v) return fail(DYNB_E_INVAL, "dynbatch_plan_view: NULL argument");
    v->n_examples = p->B;
    v->n_nodes = p->N;
    v->n_levels = p->D;
    v->n_buckets = int32_t(p->b_level.size());
    v->n_compute_nodes = int32_t(p->items.size());
    v->n_launches = int32_t(p->launches.size());
    v->max_launch_nodes = p->max_launch;
    v->n_slots = p->n_slots;
    v->node_launch = p->node_launch.data();
    v->node_level = p->level.data();
    v->node_type = p->type.data();
    v->child0 = p->child0.data();
    v->child1 = p->child1.data();
    v->root = p->root.data();
    v->bucket_level = p->b_level.data();
    v->bucket_type = p->b_type.data();
    v->bucket_start = p->b_start.data();
    v->bucket_count = p->b_count.data();
    v->members = p->members.data();
    v->in0 = p->in0.data();
    v->in1 = p->in1.data();
    v->out = p->out.data();
    v->item_node = p->item_node.data();
    v->n_tickets = int32_t(p->tickets.size());
    v->tickets = p->tickets.data();
    v->grad_dst0 = p->keep ? p->grad_dst0.data() : nullptr;
    v->grad_dst1 = p->keep ? p->grad_dst1.data() : nullptr;
    v->fn_first = p->keep ? p->fn_first.data() : nullptr;
    v->fn_items = p->keep ? p->fn_items.data() : nullptr;
    v->n_types = p->n_types;
    v->n_wg_units = int32_t(p->wg_units.size());
    static_assert(sizeof(dynb_wg_unit) == 8 * sizeof(int32_t), "a unit is eight integers");
    v->wg_units = p->wg_units.empty() ? nullptr : reinterpret_cast<const int32_t*>(p->wg_units.data());
    v->wg_order = p->wg_order.empty() ? nullptr : p->wg_order.data();
    return DYNB_OK;
}

extern "C" void dynbatch_plan_free(dynb_plan* p) { delete p; }
