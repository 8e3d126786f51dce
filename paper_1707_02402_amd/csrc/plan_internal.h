// Internal representation of a plan, shared by the host planner and the GPU executor.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "dynbatch.h"

// One module evaluation as the kernels see it.  src/dst >= 0 name a workspace slot; a negative
// value v names example -1-v: as a source its feature map (the SCENE output), as a destination
// its row of the output tensor (the node is that example's root).
struct dynb_item {
    int32_t src0;
    int32_t src1;   // unused for unary functions
    int32_t dst;
    int32_t type;
};

struct dynb_launch {
    int32_t start;       // first item
    int32_t count;
    int32_t any_binary;  // some item of the group is a two-argument function (the kernels take the conv1x1 path)
};

// mode 0: second conv3x3 (part = kernel row), 1: first conv3x3 (part = kernel row), 2: conv1x1 (part = argument)
constexpr int DYNB_WG_CHUNK = 16;
struct dynb_wg_unit { int32_t mode, type, part, begin, end, pad0, pad1, pad2; };     // items fn_items[begin .. end)
struct dynb_wg_group { int32_t mode, type, part, first_unit, n_units, pad0, pad1, pad2; };

struct dynb_plan {
    int32_t B = 0, N = 0, D = 0, n_types = 0, mode = 0;
    std::vector<uint8_t> arity;
    std::vector<int32_t> level, type, child0, child1, root;
    std::vector<int32_t> b_level, b_type, b_start, b_count, members, in0, in1, out;
    std::vector<int32_t> node_launch;    // launch group that executes each node (-1 for SCENE leaves)
    std::vector<dynb_item> items;        // execution order
    std::vector<dynb_launch> launches;
    std::vector<int32_t> leaf_roots;     // examples whose whole program is one SCENE token
    int32_t n_slots = 0, max_launch = 0;
    bool has_binary = false;
    bool throughput = false;             // DYNB_PLAN_THROUGHPUT: most work per CU instead of lowest latency
    bool persistent = false;             // DYNB_PLAN_PERSISTENT: one dependency-driven launch per batch
    std::vector<int32_t> item_node;      // node id of every item
    // DYNB_PLAN_PERSISTENT: units of work in the order workgroups claim them: 4 * item + part, part 0 = the
    // whole node, 1 / 2 = its upper / lower half.  Every unit of a node's arguments precedes the node's units.
    std::vector<int32_t> tickets;
    // DYNB_PLAN_KEEP: where the backward pass sends the gradient of an item's arguments, and the SCENE leaves.
    // grad_dst0/1[item] >= 0: item that evaluates the argument; -1 - l: SCENE leaf number l (leaves are numbered
    // example by example, in node order); unused entries are 0.
    bool keep = false;
    bool shared_nodes = false;           // built by dynbatch_plan_dag: a node may have several consumers
    std::vector<int32_t> grad_dst0, grad_dst1;
    std::vector<int32_t> leaf_first;     // [B+1] leaves of example e are leaf_first[e] .. leaf_first[e+1]
    std::vector<int32_t> root_item;      // [B] item that evaluates the example's root, -1 if the root is a SCENE leaf
    std::vector<int32_t> fn_first;       // [n_types+1] the items of function t are fn_items[fn_first[t] .. fn_first[t+1])
    std::vector<int32_t> fn_items;       // item indices grouped by function, ascending inside a function
    // Work list of the parameter-gradient kernel: a function's items are cut into chunks of at most DYNB_WG_CHUNK so that
    // the units fill the chip evenly; a unit sums one chunk for one (convolution, kernel row or argument).
    std::vector<dynb_wg_unit> wg_units;  // grouped: the chunks of one (mode, function, part) are consecutive
    std::vector<dynb_wg_group> wg_groups;
    std::vector<int32_t> wg_order;       // unit indices, longest chunks first: the order in which workgroups take them
    std::vector<char> image;             // host image of the device buffer, filled by dynbatch_plan_upload
    void* dev_buf = nullptr;             // set by dynbatch_plan_upload
    size_t dev_bytes = 0;
};

// Device buffer of an uploaded plan: items | ids of single-SCENE examples | arity table | tickets | the backward
// pass's tables (DYNB_PLAN_KEEP), each part padded to 256 bytes.
inline size_t dynb_align256(size_t v) { return (v + 255) & ~size_t(255); }
inline size_t dynb_plan_items_bytes(const dynb_plan* p) { return dynb_align256(p->items.size() * sizeof(dynb_item)); }
inline size_t dynb_plan_leaf_bytes(const dynb_plan* p) { return dynb_align256(p->leaf_roots.size() * sizeof(int32_t)); }
inline size_t dynb_plan_arity_offset(const dynb_plan* p) { return dynb_plan_items_bytes(p) + dynb_plan_leaf_bytes(p); }
inline size_t dynb_plan_arity_bytes(const dynb_plan* p) { return dynb_align256(p->arity.size()); }
inline size_t dynb_plan_ticket_bytes(const dynb_plan* p) { return dynb_align256(p->tickets.size() * sizeof(int32_t)); }
struct dynb_keep_tables { size_t gdst0, gdst1, leaf_first, root_item, fn_items, units, groups, order, end; };   // byte offsets
inline dynb_keep_tables dynb_plan_keep_tables(const dynb_plan* p)
{
    dynb_keep_tables t;
    size_t o = dynb_plan_arity_offset(p) + dynb_plan_arity_bytes(p) + dynb_plan_ticket_bytes(p);
    auto take = [&](size_t bytes) { const size_t at = o; o += p->keep ? dynb_align256(bytes) : 0; return at; };
    t.gdst0 = take(p->grad_dst0.size() * 4);
    t.gdst1 = take(p->grad_dst1.size() * 4);
    t.leaf_first = take(p->leaf_first.size() * 4);
    t.root_item = take(p->root_item.size() * 4);
    t.fn_items = take(p->fn_items.size() * 4);
    t.units = take(p->wg_units.size() * sizeof(dynb_wg_unit));
    t.groups = take(p->wg_groups.size() * sizeof(dynb_wg_group));
    t.order = take(p->wg_order.size() * 4);
    t.end = o;
    return t;
}

// Workspace of dynbatch_execute on the fused kernels' shape (bf16, C = 128, 14 x 14), in this order:
//   slots | module weights in fragment order (w3a, w3b: 9 taps, w1: 2 halves; 128 x 128 bf16 per tap and function)
//   | DYNB_PLAN_PERSISTENT: ready[n_slots], ticket counter, status word
//   | DYNB_PLAN_KEEP: mid of every item, then u of every item (written for two-argument functions), for the backward pass
inline size_t dynb_fast_map_bytes() { return size_t(14) * 14 * 128 * 2; }
inline size_t dynb_fast_packed_weight_bytes(int n_types) { return size_t(n_types) * (9 + 9 + 2) * 128 * 128 * 2; }
inline size_t dynb_fast_sync_offset(const dynb_plan* p)
{
    return dynb_align256(size_t(p->n_slots) * dynb_fast_map_bytes()) + dynb_align256(dynb_fast_packed_weight_bytes(p->n_types));
}
inline size_t dynb_fast_sync_bytes(const dynb_plan* p) { return p->persistent ? dynb_align256((size_t(p->n_slots) + 2) * sizeof(int32_t)) : 0; }
inline size_t dynb_fast_keep_offset(const dynb_plan* p) { return dynb_fast_sync_offset(p) + dynb_fast_sync_bytes(p); }
inline size_t dynb_fast_keep_bytes(const dynb_plan* p) { return p->keep ? dynb_align256(2 * p->items.size() * dynb_fast_map_bytes()) : 0; }

namespace dynb {
void set_error(const std::string& msg);
int fail(int code, const std::string& msg);
}  // namespace dynb
