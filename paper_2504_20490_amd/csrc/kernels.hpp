// Kernel parameter blocks and host-callable launchers (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hspmd_attn.h"

namespace hspmd {

struct FwdParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    uint16_t* o;
    float* lse;
    const hspmd_work_item* items;
    const hspmd_block_item* block_items;   // block variant only (items is then unused)
    float* o_f32;                  // block variant only: partial O as fp32 [Tq, Hq, d] (o is then unused)
    int64_t q_stride, kv_stride;   // token strides in elements
    int64_t total_tokens;          // query tokens (rows of lse)
    int32_t q_heads, group;
    int32_t head_dim;              // elements per head in memory (a multiple of 8, at most the kernel's tile width)
    float scale_log2;              // softmax_scale * log2(e)
    int32_t num_items;             // slots of the work list (padding included)
    int32_t* queue;                // this pass's draw counters (ItemQueue), zero between launches
};

struct BwdParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const uint16_t* o;
    const uint16_t* d_o;
    const float* lse;
    float* negd;                   // workspace: -D[Hq, T], D = rowsum(dO * O)
    float* nlse;                   // workspace: -lse / scale [Hq, T] (the logsumexp in units of raw scores)
    float* ninf_pad;               // workspace: 16 floats holding -inf
    void* dq;
    void* dk;
    void* dv;
    const hspmd_work_item* items;
    const hspmd_block_item* block_items;   // block variant only (items is then unused)
    int64_t q_stride, kv_stride;
    int64_t total_tokens;          // query tokens (rows of lse, D)
    int32_t q_heads, kv_heads, group;
    int32_t head_dim;              // elements per head in memory (a multiple of 8, at most the kernel's tile width)
    int32_t grad_f32;              // 1: gradients are fp32, 0: bf16
    int32_t dq_accumulate;         // block variant only: dq += this block's share (fp32) instead of dq = ...
    const float* rope_table;       // may be NULL: (cos, sin) pairs [position][head_dim / 2]; dq and dk
                                   // then leave as gradients with respect to the q and k BEFORE the rotary embedding
    float scale;                   // softmax_scale
    float scale_log2;              // softmax_scale * log2(e)
    int32_t num_items;             // slots of the current pass's work list (padding included)
    int32_t* queue;                // the current pass's draw counters (ItemQueue), zero between launches
};

// The kernels exist for tile widths 64 and 128 (LDS rows, MFMA contraction); a head_dim below the tile width runs
// on the next width up: register fragments are zero beyond head_dim, LDS pad columns repeat a valid chunk.
inline int tile_width(int head_dim) { return head_dim <= 64 ? 64 : 128; }
// 16-column steps of a contraction over head_dim that hold data; the kernels of tile width 128 also exist with 7
// steps (head_dim 97 .. 112, such as the 104 of the paper's 32B model), which skip the step that is all padding
inline int contraction_steps(int head_dim) { return (head_dim + 15) / 16; }

// Workgroups that a persistent kernel starts: as many as the current device holds at once at `per_cu` workgroups per
// compute unit, and not more than the list has slots (the list length is a multiple of the queue count).
int persistent_grid(int64_t num_items, int per_cu);

// `block`: the items are hspmd_block_item (separate query / key chunks, shifted causal mask)
hipError_t launch_fwd(const FwdParams& p, int head_dim, int64_t num_items, bool block, hipStream_t stream);
hipError_t launch_bwd_dsum(const BwdParams& p, int head_dim, hipStream_t stream);
hipError_t launch_bwd_dq(const BwdParams& p, int head_dim, int64_t num_items, bool block, hipStream_t stream);
hipError_t launch_bwd_dkv(const BwdParams& p, int head_dim, int64_t num_items, bool block, hipStream_t stream);

// merge of two partial results of the same rows over disjoint key sets (fp32 O [T, Hq, d], LSE [Hq, T]):
// out = a (+) b; out may alias a.  out_bf16 (may be NULL) also receives the merged O rounded to bf16.
struct MergeParams {
    const float* o_a;
    const float* lse_a;
    const float* o_b;
    const float* lse_b;
    float* o_out;
    float* lse_out;
    uint16_t* o_out_bf16;
    int64_t total_tokens;
    int32_t q_heads, head_dim;
};
hipError_t launch_merge(const MergeParams& p, hipStream_t stream);

// rotary position embedding (RoPE, rotate-half pairing) of the q and k of a pack, walking the forward work list
struct RopeParams {
    const uint16_t* q;
    const uint16_t* k;
    uint16_t* q_out;
    uint16_t* k_out;
    const float* table;            // (cos, sin) pairs [position][head_dim / 2]
    const hspmd_work_item* items;  // packed plans: forward list, every (q tile, q head) once
    const hspmd_block_item* block_items;   // block plans: forward list (query chunks) or dK/dV list (key chunks)
    int64_t q_stride, kv_stride, q_out_stride, kv_out_stride;   // token strides in elements
    int32_t q_heads, group, head_dim;
    float sin_sign;                // +1: rotate, -1: rotate back
};
hipError_t launch_rope_table(float* table, int32_t positions, int32_t head_dim, double base, hipStream_t stream);
hipError_t launch_rope_qk(const RopeParams& p, int64_t num_items, hipStream_t stream);
// block plans: `keys` selects the key chunks (p.block_items = dK/dV list) or the query chunks (forward list)
hipError_t launch_rope_block(const RopeParams& p, int64_t num_items, bool keys, hipStream_t stream);

// matrix-core rate probe: `grid` workgroups of kProbeThreads threads, each wave issues 16 * rounds MFMAs and
// every thread writes one float to out[grid * kProbeThreads]
constexpr int kProbeMaxGrid = 4096;
constexpr int kProbeThreads = 256;
int probe_grid(int compute_units);
hipError_t launch_mfma_probe(float* out, int64_t rounds, int grid, bool varied_operands, hipStream_t stream);
// the variants of hspmd_probe_mfma_rate (mode = hspmd_probe_mode)
int probe_mode_grid(int mode, int compute_units);
hipError_t launch_mfma_probe_mode(int mode, float* out, int64_t rounds, int grid, hipStream_t stream);

}  // namespace hspmd
