// Cost-sorted, XCD-aware work lists for packed variable-length causal attention.
//
// The paper balances mixed-length sequences across pipelines with a cost model
// evaluated on the CPU while the GPU is busy (Appendix "Scenario-specific
// Planning", mixed-length case).  Inside one GPU the same long tail appears
// again: under the causal mask q tile t of a sequence visits t+1 key tiles, so
// one 16K sequence holds most of a pack's work.  The list built here is the
// on-device analogue: every (sequence, tile, head) is an item with a known cost,
// and the order in which workgroups pick items up is planned on the host, once
// per pack, and reused by every layer and both passes.
//
// Placement follows the chip: workgroups are handed to the 8 XCDs round-robin by
// workgroup index and every XCD has its own L2.  Items that stream the same K/V
// (all q tiles and all query heads of one (sequence, kv head)) are therefore kept
// in the same queue (= the same XCD) and adjacent in it, so that one tile's K/V
// fetch is an L2 hit for its neighbours.  Chains heavier than a fraction of the
// total are cut into segments so that queues can be balanced; segments go to the
// least-loaded queue, heaviest first (longest-processing-time rule), and a queue
// runs its segments in order of their most expensive item.
#include "schedule.hpp"

#include <algorithm>
#include <numeric>
#include <queue>

namespace hspmd {

std::string check_pack(const int32_t* cu, int32_t num_seqs, int32_t hq, int32_t hkv) {
    if (!cu) return "cu_seqlens is NULL";
    if (num_seqs < 0) return "num_seqs is negative";
    if (hq <= 0 || hkv <= 0) return "head counts must be positive";
    if (hq % hkv != 0) return "local_q_heads must be a multiple of local_kv_heads (cut an uneven share on KV-group boundaries)";
    if (cu[0] != 0) return "cu_seqlens[0] must be 0";
    for (int32_t i = 0; i < num_seqs; ++i)
        if (cu[i + 1] < cu[i]) return "cu_seqlens must be non-decreasing";
    return std::string();
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int64_t item_cost(hspmd_list_kind kind, int32_t seq_len, int32_t tile, int32_t group) {
    if (kind == HSPMD_LIST_DKV) {
        const int64_t first_row = (int64_t)tile * kDkvKTile;          // rows r >= first key of the tile
        if (first_row >= seq_len) return 0;
        return ceil_div(seq_len - first_row, kDkvQTile) * group;
    }
    const int64_t last_key = std::min<int64_t>(seq_len, (int64_t)(tile + 1) * kFwdQTile);
    if ((int64_t)tile * kFwdQTile >= seq_len) return 0;
    return ceil_div(last_key, kFwdKTile);
}

namespace {
struct Segment {
    int64_t cost = 0;
    int64_t first_cost = 0;
    int64_t order = 0;                 // creation index: keeps ties deterministic
    std::vector<hspmd_work_item> items;
};
}  // namespace

// The two orders without placement: used only to measure what the default order buys.
static std::vector<hspmd_work_item> build_plain_list(hspmd_list_kind kind, const int32_t* cu, int32_t num_seqs,
                                                     int32_t hq, int32_t hkv, hspmd_order order) {
    const int32_t group = hq / hkv;
    const int tile_rows = (kind == HSPMD_LIST_DKV) ? kDkvKTile : kFwdQTile;
    const int32_t heads = (kind == HSPMD_LIST_DKV) ? hkv : hq;
    std::vector<hspmd_work_item> out;
    for (int32_t s = 0; s < num_seqs; ++s) {
        const int32_t len = cu[s + 1] - cu[s];
        if (len <= 0) continue;
        const int32_t n_tiles = (int32_t)ceil_div(len, tile_rows);
        for (int32_t t = 0; t < n_tiles; ++t)
            for (int32_t h = 0; h < heads; ++h) out.push_back({cu[s], len, t, h});
    }
    if (order == HSPMD_ORDER_COST)
        std::stable_sort(out.begin(), out.end(), [&](const hspmd_work_item& a, const hspmd_work_item& b) {
            return item_cost(kind, a.seq_len, a.tile, group) > item_cost(kind, b.seq_len, b.tile, group);
        });
    return out;
}

std::vector<hspmd_work_item> build_work_list(hspmd_list_kind kind, const int32_t* cu, int32_t num_seqs,
                                             int32_t hq, int32_t hkv, int32_t num_queues, hspmd_order order) {
    if (order != HSPMD_ORDER_XCD_COST) return build_plain_list(kind, cu, num_seqs, hq, hkv, order);
    const int32_t group = hq / hkv;
    const int tile_rows = (kind == HSPMD_LIST_DKV) ? kDkvKTile : kFwdQTile;

    // 1. chains: all items that share one (sequence, kv head), most expensive first
    std::vector<std::vector<hspmd_work_item>> chains;
    int64_t total_cost = 0;
    for (int32_t s = 0; s < num_seqs; ++s) {
        const int32_t len = cu[s + 1] - cu[s];
        if (len <= 0) continue;
        const int32_t n_tiles = (int32_t)ceil_div(len, tile_rows);
        for (int32_t g = 0; g < hkv; ++g) {
            std::vector<hspmd_work_item> chain;
            if (kind == HSPMD_LIST_DKV) {
                for (int32_t t = 0; t < n_tiles; ++t) chain.push_back({cu[s], len, t, g});
            } else {
                for (int32_t t = n_tiles - 1; t >= 0; --t)
                    for (int32_t h = g * group; h < (g + 1) * group; ++h) chain.push_back({cu[s], len, t, h});
            }
            for (const auto& it : chain) total_cost += item_cost(kind, it.seq_len, it.tile, group);
            chains.push_back(std::move(chain));
        }
    }
    if (chains.empty()) return {};

    // 2. cut chains into segments no heavier than 1/(4 * queues) of the total
    const int64_t cap = std::max<int64_t>(1, total_cost / ((int64_t)num_queues * 4));
    std::vector<Segment> segments;
    for (auto& chain : chains) {
        Segment seg;
        for (const auto& it : chain) {
            const int64_t c = item_cost(kind, it.seq_len, it.tile, group);
            if (!seg.items.empty() && seg.cost + c > cap) {
                seg.order = (int64_t)segments.size();
                segments.push_back(std::move(seg));
                seg = Segment();
            }
            if (seg.items.empty()) seg.first_cost = c;
            seg.items.push_back(it);
            seg.cost += c;
        }
        if (!seg.items.empty()) {
            seg.order = (int64_t)segments.size();
            segments.push_back(std::move(seg));
        }
    }

    // 3. longest-processing-time assignment of segments to queues
    std::vector<size_t> by_cost(segments.size());
    std::iota(by_cost.begin(), by_cost.end(), 0);
    std::stable_sort(by_cost.begin(), by_cost.end(),
                     [&](size_t a, size_t b) { return segments[a].cost > segments[b].cost; });
    using Load = std::pair<int64_t, int32_t>;  // (load, queue)
    std::priority_queue<Load, std::vector<Load>, std::greater<Load>> loads;
    for (int32_t x = 0; x < num_queues; ++x) loads.push({0, x});
    std::vector<std::vector<size_t>> queue_segments(num_queues);
    for (size_t idx : by_cost) {
        Load l = loads.top();
        loads.pop();
        queue_segments[l.second].push_back(idx);
        l.first += segments[idx].cost;
        loads.push(l);
    }

    // 4. inside a queue: segments by their most expensive item, then creation order
    std::vector<std::vector<hspmd_work_item>> queues(num_queues);
    size_t longest = 0;
    for (int32_t x = 0; x < num_queues; ++x) {
        auto& segs = queue_segments[x];
        std::stable_sort(segs.begin(), segs.end(), [&](size_t a, size_t b) {
            if (segments[a].first_cost != segments[b].first_cost) return segments[a].first_cost > segments[b].first_cost;
            return segments[a].order < segments[b].order;
        });
        for (size_t idx : segs)
            queues[x].insert(queues[x].end(), segments[idx].items.begin(), segments[idx].items.end());
        longest = std::max(longest, queues[x].size());
    }

    // 5. interleave: slot p belongs to queue p % num_queues; pad short queues
    std::vector<hspmd_work_item> out(longest * (size_t)num_queues, hspmd_work_item{0, 0, -1, 0});
    for (int32_t x = 0; x < num_queues; ++x)
        for (size_t i = 0; i < queues[x].size(); ++i) out[i * (size_t)num_queues + (size_t)x] = queues[x][i];
    return out;
}

}  // namespace hspmd
