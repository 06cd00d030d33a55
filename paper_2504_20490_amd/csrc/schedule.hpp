// Host-side construction of the cost-sorted work lists (no GPU code in here).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/hspmd_attn.h"

namespace hspmd {

// Tile geometry shared by the scheduler and the kernels.
constexpr int kFwdQTile = 128;   // q rows per forward / dQ work item (4 waves x 32 rows)
constexpr int kFwdKTile = 64;    // keys per inner step of the forward / dQ kernels
constexpr int kDkvKTile = 128;   // keys per dK/dV work item (4 waves x 32 keys)
constexpr int kDkvQTile = 64;    // q rows per inner step of the dK/dV kernel
constexpr int kNumXcd = 8;       // XCDs of an MI355X: workgroup p lands on XCD p % 8

// Validates cu_seqlens / head counts; returns an empty string when fine.
std::string check_pack(const int32_t* cu, int32_t num_seqs, int32_t hq, int32_t hkv);

// Cost (number of inner steps) of one item.
int64_t item_cost(hspmd_list_kind kind, int32_t seq_len, int32_t tile, int32_t group);

// Builds the launch-ordered list (see hspmd_attn_schedule in the public header).
std::vector<hspmd_work_item> build_work_list(hspmd_list_kind kind, const int32_t* cu, int32_t num_seqs,
                                             int32_t hq, int32_t hkv, int32_t num_queues,
                                             hspmd_order order = HSPMD_ORDER_XCD_COST);

// ---- cost model: predicted kernel times (microseconds) of the three passes for a pack.
// Every item of a pass's work list weighs steps * step_us + item_us; the pass takes launch_us plus the weight
// of its heaviest queue divided by the workgroups resident per XCD (and not less than its heaviest item).
struct PassCost {
    double launch_us, step_us, item_us;
};
// coefficients fitted to measurements on MI355X (fit_cost_model.py refits them); head_dim = the tile width, 64 or 128
PassCost pass_cost_coefficients(hspmd_list_kind kind, int32_t head_dim);
double estimate_pass_us(hspmd_list_kind kind, const int32_t* cu, int32_t num_seqs, int32_t hq, int32_t hkv, int32_t head_dim);

// ---- block variant (one step of context-parallel attention): per sequence a query chunk and a key chunk
// with positions inside the sequence; key j is visible to row r iff j <= r + (q_pos - k_pos).
std::string check_block_pack(const int32_t* cu_q, const int32_t* cu_k, const int32_t* q_pos, const int32_t* k_pos,
                             int32_t num_seqs, int32_t hq, int32_t hkv);

// Cost (number of inner steps) of one block item; 0 when the item only writes zeros.
int64_t block_item_cost(hspmd_list_kind kind, const hspmd_block_item& item, int32_t group);

// Launch-ordered list of the block variant: same placement rules as build_work_list.  Every tile that owns
// output rows gets an item, also when nothing is visible to it (it then writes zeros).
std::vector<hspmd_block_item> build_block_list(hspmd_list_kind kind, const int32_t* cu_q, const int32_t* cu_k,
                                               const int32_t* q_pos, const int32_t* k_pos, int32_t num_seqs,
                                               int32_t hq, int32_t hkv, int32_t num_queues);

}  // namespace hspmd
