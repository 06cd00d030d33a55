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

// Steps 2-5 of the placement, shared by the packed and the block lists: cut chains into segments, assign the
// segments to queues by the longest-processing-time rule, order each queue, interleave the queues.
template <typename Item, typename Cost>
static std::vector<Item> place_chains(std::vector<std::vector<Item>>& chains, int64_t total_cost, int32_t num_queues,
                                      Cost cost_of, Item pad) {
    struct Seg {
        int64_t cost = 0;
        int64_t first_cost = 0;
        int64_t order = 0;                 // creation index: keeps ties deterministic
        std::vector<Item> items;
    };
    if (chains.empty()) return {};
    // 2. cut chains into segments no heavier than 1/(4 * queues) of the total
    const int64_t cap = std::max<int64_t>(1, total_cost / ((int64_t)num_queues * 4));
    std::vector<Seg> segments;
    for (auto& chain : chains) {
        Seg seg;
        for (const auto& it : chain) {
            // an item that only writes zeros (block variant) still occupies a workgroup slot: weight 1, so that
            // such items spread over the queues instead of piling up in one
            const int64_t c = std::max<int64_t>(1, cost_of(it));
            if (!seg.items.empty() && seg.cost + c > cap) {
                seg.order = (int64_t)segments.size();
                segments.push_back(std::move(seg));
                seg = Seg();
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
    std::vector<std::vector<Item>> queues(num_queues);
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
    std::vector<Item> out(longest * (size_t)num_queues, pad);
    for (int32_t x = 0; x < num_queues; ++x)
        for (size_t i = 0; i < queues[x].size(); ++i) out[i * (size_t)num_queues + (size_t)x] = queues[x][i];
    return out;
}

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
    return place_chains<hspmd_work_item>(
        chains, total_cost, num_queues, [&](const hspmd_work_item& it) { return item_cost(kind, it.seq_len, it.tile, group); },
        hspmd_work_item{0, 0, -1, 0});
}

// ------------------------------------------------------------------------------ cost model
// The paper's planner dispatches mixed-length sequences with a cost model evaluated on the CPU (Appendix
// "Scenario-specific Planning", mixed-length case); this is the per-operator predictor for the attention
// kernels of this library.  Fitted by relative least squares to 40 packs per head_dim: mean absolute error
// 6-8 %, at most 15-32 % (on packs that take about a hundred microseconds).
PassCost pass_cost_coefficients(hspmd_list_kind kind, int32_t head_dim) {
    static const PassCost k128[3] = {{13.1, 1.655, 10.37}, {7.6, 2.168, 18.64}, {24.8, 1.620, 11.66}};
    static const PassCost k64[3] = {{13.1, 1.045, 6.22}, {7.6, 1.239, 9.02}, {18.5, 1.062, 6.41}};
    return (head_dim == 64 ? k64 : k128)[(int)kind];
}

double estimate_pass_us(hspmd_list_kind kind, const int32_t* cu, int32_t num_seqs, int32_t hq, int32_t hkv, int32_t head_dim) {
    const std::vector<hspmd_work_item> list = build_work_list(kind, cu, num_seqs, hq, hkv, kNumXcd);
    if (list.empty()) return 0.0;
    const PassCost c = pass_cost_coefficients(kind, head_dim);
    const int32_t group = hq / hkv;
    // workgroups resident per XCD: 32 compute units, two workgroups each in the forward and dQ passes, one in dK/dV
    const double slots = kind == HSPMD_LIST_DKV ? 32.0 : 64.0;
    double queue_weight[kNumXcd] = {0};
    double heaviest = 0.0;
    for (size_t p = 0; p < list.size(); ++p) {
        if (list[p].tile < 0) continue;
        const double w = (double)item_cost(kind, list[p].seq_len, list[p].tile, group) * c.step_us + c.item_us;
        queue_weight[p % kNumXcd] += w;
        heaviest = std::max(heaviest, w);
    }
    double worst = 0.0;
    for (double w : queue_weight) worst = std::max(worst, w);
    return c.launch_us + std::max(worst / slots, heaviest);
}

// ------------------------------------------------------------------------------ block variant
std::string check_block_pack(const int32_t* cu_q, const int32_t* cu_k, const int32_t* q_pos, const int32_t* k_pos,
                             int32_t num_seqs, int32_t hq, int32_t hkv) {
    if (!cu_q || !cu_k) return "cu_seqlens is NULL";
    if (num_seqs < 0) return "num_seqs is negative";
    if (num_seqs > 0 && (!q_pos || !k_pos)) return "chunk positions are NULL";
    if (hq <= 0 || hkv <= 0) return "head counts must be positive";
    if (hq % hkv != 0) return "local_q_heads must be a multiple of local_kv_heads (cut an uneven share on KV-group boundaries)";
    if (cu_q[0] != 0 || cu_k[0] != 0) return "cu_seqlens[0] must be 0";
    for (int32_t i = 0; i < num_seqs; ++i) {
        if (cu_q[i + 1] < cu_q[i] || cu_k[i + 1] < cu_k[i]) return "cu_seqlens must be non-decreasing";
        if (q_pos[i] < 0 || k_pos[i] < 0) return "chunk positions must be non-negative";
        // positions of the last row / key must stay in int32 together with the tile arithmetic
        if ((int64_t)q_pos[i] + (cu_q[i + 1] - cu_q[i]) > (int64_t)1 << 30 ||
            (int64_t)k_pos[i] + (cu_k[i + 1] - cu_k[i]) > (int64_t)1 << 30)
            return "chunk position + length above 2^30";
    }
    return std::string();
}

int64_t block_item_cost(hspmd_list_kind kind, const hspmd_block_item& it, int32_t group) {
    if (kind == HSPMD_LIST_DKV) {
        // rows r >= key0 - offset see the tile's first key
        if ((int64_t)it.tile * kDkvKTile >= it.k_len) return 0;
        const int64_t first_row = std::max<int64_t>(0, (int64_t)it.tile * kDkvKTile - it.offset);
        const int64_t first_qt = first_row / kDkvQTile;
        const int64_t n_qt = ceil_div(it.q_len, kDkvQTile);
        return std::max<int64_t>(0, n_qt - first_qt) * group;
    }
    if ((int64_t)it.tile * kFwdQTile >= it.q_len) return 0;
    const int64_t last_row = std::min<int64_t>(it.q_len, (int64_t)(it.tile + 1) * kFwdQTile);   // exclusive
    const int64_t kv_end = std::max<int64_t>(0, std::min<int64_t>(it.k_len, last_row + it.offset));
    return ceil_div(kv_end, kFwdKTile);
}

std::vector<hspmd_block_item> build_block_list(hspmd_list_kind kind, const int32_t* cu_q, const int32_t* cu_k,
                                               const int32_t* q_pos, const int32_t* k_pos, int32_t num_seqs,
                                               int32_t hq, int32_t hkv, int32_t num_queues) {
    const int32_t group = hq / hkv;
    std::vector<std::vector<hspmd_block_item>> chains;
    int64_t total_cost = 0;
    for (int32_t s = 0; s < num_seqs; ++s) {
        const int32_t q_len = cu_q[s + 1] - cu_q[s], k_len = cu_k[s + 1] - cu_k[s];
        const int32_t rows = (kind == HSPMD_LIST_DKV) ? k_len : q_len;     // rows of the outputs the list owns
        if (rows <= 0) continue;
        const int tile_rows = (kind == HSPMD_LIST_DKV) ? kDkvKTile : kFwdQTile;
        const int32_t n_tiles = (int32_t)ceil_div(rows, tile_rows);
        const hspmd_block_item proto{cu_q[s], q_len, cu_k[s], k_len, q_pos[s] - k_pos[s], 0, 0, q_pos[s]};
        for (int32_t g = 0; g < hkv; ++g) {
            std::vector<hspmd_block_item> chain;
            auto add = [&](int32_t tile, int32_t head) {
                hspmd_block_item it = proto;
                it.tile = tile;
                it.head = head;
                chain.push_back(it);
            };
            if (kind == HSPMD_LIST_DKV) {
                for (int32_t t = 0; t < n_tiles; ++t) add(t, g);
            } else {
                for (int32_t t = n_tiles - 1; t >= 0; --t)
                    for (int32_t h = g * group; h < (g + 1) * group; ++h) add(t, h);
            }
            // most expensive first inside a chain (with a shift the cost is still monotone in the tile index)
            for (const auto& it : chain) total_cost += block_item_cost(kind, it, group);
            chains.push_back(std::move(chain));
        }
    }
    return place_chains<hspmd_block_item>(
        chains, total_cost, num_queues, [&](const hspmd_block_item& it) { return block_item_cost(kind, it, group); },
        hspmd_block_item{0, 0, 0, 0, 0, -1, 0, 0});
}

}  // namespace hspmd
