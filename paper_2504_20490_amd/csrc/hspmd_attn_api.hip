// C-ABI entry points of libhspmd_attn: argument validation, plan management, launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <new>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/hspmd_attn.h"
#include "kernels.hpp"
#include "schedule.hpp"

namespace hspmd {

// compute units of the current device (queried once per device)
int persistent_grid(int64_t num_items, int per_cu) {
    static std::mutex mutex;
    static std::map<int, int> compute_units;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    int cus = 0;
    {
        std::lock_guard<std::mutex> lock(mutex);
        auto it = compute_units.find(dev);
        if (it == compute_units.end()) {
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 0;
            compute_units[dev] = cus;
        } else {
            cus = it->second;
        }
    }
    // a multiple of the queue count, like the list length
    const int64_t resident = (int64_t)(cus * per_cu / kNumXcd) * kNumXcd;
    return (int)std::min<int64_t>(num_items, std::max<int64_t>(resident, kNumXcd));
}

}  // namespace hspmd

namespace {

thread_local std::string g_last_error;

hspmd_status fail(hspmd_status code, const std::string& what) {
    g_last_error = what;
    return code;
}

hspmd_status fail_hip(hipError_t e, const char* where) {
    g_last_error = std::string(where) + ": " + hipGetErrorString(e);
    return HSPMD_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// rows are moved in 16-byte chunks; the kernels exist for tile widths 64 and 128 and pad up to the next one
bool supported_head_dim(int32_t head_dim) { return head_dim >= 8 && head_dim <= 128 && head_dim % 8 == 0; }

// ---- optional per-kernel event timing ------------------------------------------------------
struct ProfileRecord {
    int kernel;
    hipEvent_t start, stop;
};
// The switch is read on every launch from any thread; the records and the event pool are shared by all
// threads and guarded by one mutex (taken only while timing is on).
std::atomic<bool> g_profile_on{false};
std::mutex g_profile_mutex;
std::vector<ProfileRecord> g_records;
std::vector<hipEvent_t> g_event_pool;

hipError_t take_event(hipEvent_t* ev) {   // g_profile_mutex held
    if (!g_event_pool.empty()) {
        *ev = g_event_pool.back();
        g_event_pool.pop_back();
        return hipSuccess;
    }
    return hipEventCreate(ev);
}

// Runs `launch` on `stream`; when profiling is on, brackets it with two events.
template <typename F>
hipError_t timed_launch(int kernel, hipStream_t stream, F&& launch) {
    if (!g_profile_on.load(std::memory_order_relaxed)) return launch();
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    ProfileRecord r{kernel, nullptr, nullptr};
    hipError_t e = take_event(&r.start);
    if (e != hipSuccess) return e;
    e = take_event(&r.stop);
    if (e != hipSuccess) return e;
    e = hipEventRecord(r.start, stream);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    e = hipEventRecord(r.stop, stream);
    if (e != hipSuccess) return e;
    g_records.push_back(r);
    return hipSuccess;
}

// Upload of a plan's work lists.  It goes through a copy stream of the library's own (one per device, created on
// first use, default priority, not synchronising with the NULL stream) and waits for that stream only: the
// caller's compute stream is never waited on, so building the plan of the next micro-batch overlaps the kernels
// of the current one.  The copy has completed when this returns; kernels launched afterwards on any stream see it.
std::mutex g_copy_stream_mutex;
std::map<int, hipStream_t> g_copy_streams;

hipError_t upload_blocking(void* dst, const void* src, size_t bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    hipStream_t copy = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_copy_stream_mutex);
        auto it = g_copy_streams.find(dev);
        if (it == g_copy_streams.end()) {
            e = hipStreamCreateWithFlags(&copy, hipStreamNonBlocking);
            if (e != hipSuccess) return e;
            g_copy_streams[dev] = copy;
        } else {
            copy = it->second;
        }
    }
    e = hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, copy);
    if (e == hipSuccess) e = hipStreamSynchronize(copy);
    return e;
}

// waits for the recorded events, hands every launch's elapsed time to `sink(kernel, ms)` and forgets the records
template <typename Sink>
hspmd_status drain_profile_records(Sink&& sink) {
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    hspmd_status rc = HSPMD_OK;
    for (const ProfileRecord& r : g_records) {
        hipError_t e = hipEventSynchronize(r.stop);
        float t = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&t, r.start, r.stop);
        if (e == hipSuccess) sink(r.kernel, (double)t);
        else rc = fail_hip(e, "profile read");
        g_event_pool.push_back(r.start);
        g_event_pool.push_back(r.stop);
    }
    g_records.clear();
    return rc;
}

}  // namespace

// One copy of a plan's work lists on the device.  A plan owns a small ring of these: a refill
// (hspmd_attn_plan_update) writes the slot that was used longest ago while launches that read the current one may
// still be running, and waits (on the host) only for the event that the last launch reading THAT slot recorded.
struct ListSlot {
    void* block = nullptr;          // device memory
    size_t capacity = 0;            // bytes
    hipEvent_t last_use = nullptr;  // recorded on the launch stream after a launch that reads the slot
    bool recorded = false;
};
constexpr int kPlanSlots = 3;
// the draw counters of one pass (16 int32) in units of list items
constexpr size_t kCounterItems = 16 * sizeof(int32_t) / sizeof(hspmd_work_item);
constexpr size_t kCounterBlockItems = 16 * sizeof(int32_t) / sizeof(hspmd_block_item);

struct hspmd_attn_plan {
    int32_t num_seqs = 0;
    int32_t q_heads = 0, kv_heads = 0, head_dim = 0;
    int64_t total_tokens = 0;
    int32_t max_position = 0;      // positions inside a sequence that the plan's tokens occupy: 0 .. max_position-1
    int64_t count[3] = {0, 0, 0};
    hspmd_work_item* items[3] = {nullptr, nullptr, nullptr};   // device; three views into the current slot
    hspmd_order order = HSPMD_ORDER_XCD_COST;
    // block variant (hspmd_attn_block_plan_create): total_tokens counts query tokens
    bool is_block = false;
    int64_t total_kv_tokens = 0;
    hspmd_block_item* block_items[3] = {nullptr, nullptr, nullptr};
    int32_t* queue[3] = {nullptr, nullptr, nullptr};   // device: draw counters of the three passes (zero between launches)
    // device copies of the lists
    ListSlot slots[kPlanSlots];
    int current = 0;
    mutable std::mutex use_mutex;   // launches from several threads record the current slot's event
};

namespace {

// Marks the plan's current slot as read by work just enqueued on `stream` (a later refill of that slot waits for
// it).  Nothing is recorded while the stream is being captured into a graph: a plan that a graph replays must not be
// refilled while the graph may run, and that is the caller's to ensure.
hipError_t mark_use(const hspmd_attn_plan* plan, hipStream_t stream) {
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (stream != nullptr) {
        const hipError_t e = hipStreamIsCapturing(stream, &capturing);
        if (e != hipSuccess) return e;
    }
    if (capturing != hipStreamCaptureStatusNone) return hipSuccess;
    std::lock_guard<std::mutex> lock(plan->use_mutex);
    ListSlot& slot = const_cast<hspmd_attn_plan*>(plan)->slots[plan->current];
    if (!slot.last_use) return hipSuccess;
    const hipError_t e = hipEventRecord(slot.last_use, stream);
    if (e == hipSuccess) slot.recorded = true;
    return e;
}

// Puts `bytes` of host data into the plan's next slot and makes it the current one.  Steady state (the slot has been
// used before and is large enough): no allocation, no free, no device-wide synchronisation -- one wait for that
// slot's own last launch (long finished when the ring has gone round) and one copy on the library's copy stream.
hspmd_status install_lists(hspmd_attn_plan* plan, const void* host, size_t bytes, bool first) {
    const int next = first ? 0 : (plan->current + 1) % kPlanSlots;
    ListSlot& slot = plan->slots[next];
    hipError_t e = hipSuccess;
    if (slot.recorded) {
        e = hipEventSynchronize(slot.last_use);
        if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize(work list slot)");
        slot.recorded = false;
    }
    if (!slot.last_use) {
        e = hipEventCreateWithFlags(&slot.last_use, hipEventDisableTiming);
        if (e != hipSuccess) return fail_hip(e, "hipEventCreate(work list slot)");
    }
    if (bytes > slot.capacity) {
        // grow only, with headroom, so that packs of similar size stop allocating after the first few refills
        if (slot.block) {
            e = hipFree(slot.block);
            slot.block = nullptr;
            slot.capacity = 0;
            if (e != hipSuccess) return fail_hip(e, "hipFree(work lists)");
        }
        const size_t want = first ? bytes : bytes + bytes / 4;
        e = hipMalloc(&slot.block, want);
        if (e != hipSuccess) return fail_hip(e, "hipMalloc(work lists)");
        slot.capacity = want;
    }
    if (bytes > 0) {
        e = upload_blocking(slot.block, host, bytes);
        if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync(work lists)");
    }
    plan->current = next;
    return HSPMD_OK;
}

// Builds the three packed lists of a pack on the host (forward and dQ share one copy) and installs them.
hspmd_status fill_packed_plan(hspmd_attn_plan* plan, const int32_t* cu, int32_t num_seqs, bool first) {
    std::vector<hspmd_work_item> all;
    size_t offset[3] = {0, 0, 0};
    int64_t count[3] = {0, 0, 0};
    try {
        for (int kind = 0; kind < 3; ++kind) {
            if (kind == HSPMD_LIST_DQ) {
                // same items, costs and order as the forward list: one copy serves both passes
                count[kind] = count[HSPMD_LIST_FWD];
                offset[kind] = offset[HSPMD_LIST_FWD];
                continue;
            }
            const std::vector<hspmd_work_item> list = hspmd::build_work_list(
                (hspmd_list_kind)kind, cu, num_seqs, plan->q_heads, plan->kv_heads, hspmd::kNumXcd, plan->order);
            count[kind] = (int64_t)list.size();
            offset[kind] = all.size();
            all.insert(all.end(), list.begin(), list.end());
        }
    } catch (const std::bad_alloc&) {
        return fail(HSPMD_ERR_INVALID_ARG, "out of host memory while building the work lists");
    }
    // behind the lists: the draw counters of the three passes, uploaded as zeros (one list item = 16 bytes = 4 counters)
    const size_t counters_at = all.size();
    try {
        all.resize(all.size() + 3 * kCounterItems, hspmd_work_item{0, 0, 0, 0});
    } catch (const std::bad_alloc&) {
        return fail(HSPMD_ERR_INVALID_ARG, "out of host memory while building the work lists");
    }
    if (hspmd_status rc = install_lists(plan, all.data(), all.size() * sizeof(hspmd_work_item), first)) return rc;
    for (int kind = 0; kind < 3; ++kind)
        plan->queue[kind] = reinterpret_cast<int32_t*>(static_cast<hspmd_work_item*>(plan->slots[plan->current].block) +
                                                       counters_at + kind * kCounterItems);
    plan->num_seqs = num_seqs;
    plan->total_tokens = cu[num_seqs];
    plan->max_position = 0;
    for (int32_t i = 0; i < num_seqs; ++i) plan->max_position = std::max(plan->max_position, cu[i + 1] - cu[i]);
    for (int kind = 0; kind < 3; ++kind) {
        plan->count[kind] = count[kind];
        plan->items[kind] = count[kind] > 0 ? static_cast<hspmd_work_item*>(plan->slots[plan->current].block) + offset[kind]
                                            : nullptr;
    }
    return HSPMD_OK;
}

hspmd_status fill_block_plan(hspmd_attn_plan* plan, const int32_t* cu_q, const int32_t* cu_k, const int32_t* q_pos,
                             const int32_t* k_pos, int32_t num_seqs, bool first) {
    std::vector<hspmd_block_item> all;
    size_t offset[3] = {0, 0, 0};
    int64_t count[3] = {0, 0, 0};
    try {
        for (int kind = 0; kind < 3; ++kind) {
            if (kind == HSPMD_LIST_DQ) {
                count[kind] = count[HSPMD_LIST_FWD];
                offset[kind] = offset[HSPMD_LIST_FWD];
                continue;
            }
            const std::vector<hspmd_block_item> list = hspmd::build_block_list(
                (hspmd_list_kind)kind, cu_q, cu_k, q_pos, k_pos, num_seqs, plan->q_heads, plan->kv_heads, hspmd::kNumXcd);
            count[kind] = (int64_t)list.size();
            offset[kind] = all.size();
            all.insert(all.end(), list.begin(), list.end());
        }
    } catch (const std::bad_alloc&) {
        return fail(HSPMD_ERR_INVALID_ARG, "out of host memory while building the work lists");
    }
    const size_t counters_at = all.size();
    try {
        all.resize(all.size() + 3 * kCounterBlockItems, hspmd_block_item{0, 0, 0, 0, 0, 0, 0, 0});
    } catch (const std::bad_alloc&) {
        return fail(HSPMD_ERR_INVALID_ARG, "out of host memory while building the work lists");
    }
    if (hspmd_status rc = install_lists(plan, all.data(), all.size() * sizeof(hspmd_block_item), first)) return rc;
    for (int kind = 0; kind < 3; ++kind)
        plan->queue[kind] = reinterpret_cast<int32_t*>(static_cast<hspmd_block_item*>(plan->slots[plan->current].block) +
                                                       counters_at + kind * kCounterBlockItems);
    plan->num_seqs = num_seqs;
    plan->total_tokens = cu_q[num_seqs];
    plan->total_kv_tokens = cu_k[num_seqs];
    plan->max_position = 0;
    for (int32_t i = 0; i < num_seqs; ++i)
        plan->max_position = std::max(plan->max_position, std::max(q_pos[i] + (cu_q[i + 1] - cu_q[i]),
                                                                   k_pos[i] + (cu_k[i + 1] - cu_k[i])));
    for (int kind = 0; kind < 3; ++kind) {
        plan->count[kind] = count[kind];
        plan->block_items[kind] =
            count[kind] > 0 ? static_cast<hspmd_block_item*>(plan->slots[plan->current].block) + offset[kind] : nullptr;
    }
    return HSPMD_OK;
}

}  // namespace

extern "C" {

const char* hspmd_last_error(void) { return g_last_error.c_str(); }

int32_t hspmd_attn_tile_rows(hspmd_list_kind kind) {
    return kind == HSPMD_LIST_DKV ? hspmd::kDkvKTile : hspmd::kFwdQTile;
}

hspmd_status hspmd_build_cu_seqlens(const int32_t* lengths, int32_t num_seqs, int32_t* cu_seqlens,
                                    int32_t* max_seqlen, int64_t* total_tokens) {
    if (num_seqs < 0) return fail(HSPMD_ERR_INVALID_ARG, "num_seqs is negative");
    if (!cu_seqlens || (!lengths && num_seqs > 0)) return fail(HSPMD_ERR_INVALID_ARG, "null pointer");
    int64_t running = 0;
    int32_t longest = 0;
    cu_seqlens[0] = 0;
    for (int32_t i = 0; i < num_seqs; ++i) {
        if (lengths[i] < 0) return fail(HSPMD_ERR_INVALID_ARG, "negative sequence length");
        running += lengths[i];
        if (running > std::numeric_limits<int32_t>::max())
            return fail(HSPMD_ERR_INVALID_ARG, "total token count exceeds INT32_MAX");
        cu_seqlens[i + 1] = (int32_t)running;
        if (lengths[i] > longest) longest = lengths[i];
    }
    if (max_seqlen) *max_seqlen = longest;
    if (total_tokens) *total_tokens = running;
    return HSPMD_OK;
}

hspmd_status hspmd_attn_schedule_ordered(hspmd_list_kind kind, hspmd_order order, const int32_t* cu_seqlens,
                                         int32_t num_seqs, int32_t local_q_heads, int32_t local_kv_heads,
                                         int32_t num_queues, hspmd_work_item* items, int64_t capacity, int64_t* count) {
    if (kind != HSPMD_LIST_FWD && kind != HSPMD_LIST_DQ && kind != HSPMD_LIST_DKV)
        return fail(HSPMD_ERR_INVALID_ARG, "unknown list kind");
    if (order != HSPMD_ORDER_XCD_COST && order != HSPMD_ORDER_NATURAL && order != HSPMD_ORDER_COST)
        return fail(HSPMD_ERR_INVALID_ARG, "unknown order");
    if (!count) return fail(HSPMD_ERR_INVALID_ARG, "count is NULL");
    if (num_queues < 1) return fail(HSPMD_ERR_INVALID_ARG, "num_queues must be >= 1");
    if (capacity < 0 || (capacity > 0 && !items)) return fail(HSPMD_ERR_INVALID_ARG, "items is NULL");
    const std::string why = hspmd::check_pack(cu_seqlens, num_seqs, local_q_heads, local_kv_heads);
    if (!why.empty()) return fail(HSPMD_ERR_INVALID_ARG, why);
    std::vector<hspmd_work_item> list;
    try {
        list = hspmd::build_work_list(kind, cu_seqlens, num_seqs, local_q_heads, local_kv_heads, num_queues, order);
    } catch (const std::bad_alloc&) {
        return fail(HSPMD_ERR_INVALID_ARG, "out of host memory while building the work list");
    }
    *count = (int64_t)list.size();
    if (capacity == 0) return HSPMD_OK;
    if ((int64_t)list.size() > capacity) return fail(HSPMD_ERR_INVALID_ARG, "items buffer too small");
    if (!list.empty()) std::memcpy(items, list.data(), list.size() * sizeof(hspmd_work_item));
    return HSPMD_OK;
}

hspmd_status hspmd_attn_schedule(hspmd_list_kind kind, const int32_t* cu_seqlens, int32_t num_seqs,
                                 int32_t local_q_heads, int32_t local_kv_heads, int32_t num_queues,
                                 hspmd_work_item* items, int64_t capacity, int64_t* count) {
    return hspmd_attn_schedule_ordered(kind, HSPMD_ORDER_XCD_COST, cu_seqlens, num_seqs, local_q_heads, local_kv_heads,
                                       num_queues, items, capacity, count);
}

hspmd_status hspmd_attn_plan_create_ordered(const int32_t* cu_seqlens_host, int32_t num_seqs, int32_t local_q_heads,
                                            int32_t local_kv_heads, int32_t head_dim, hspmd_order order,
                                            void* stream, hspmd_attn_plan** out) {
    if (!out) return fail(HSPMD_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    const std::string why = hspmd::check_pack(cu_seqlens_host, num_seqs, local_q_heads, local_kv_heads);
    if (!why.empty()) return fail(HSPMD_ERR_INVALID_ARG, why);
    if (!supported_head_dim(head_dim)) return fail(HSPMD_ERR_UNSUPPORTED, "head_dim must be a multiple of 8 between 8 and 128");
    if (order != HSPMD_ORDER_XCD_COST && order != HSPMD_ORDER_NATURAL && order != HSPMD_ORDER_COST)
        return fail(HSPMD_ERR_INVALID_ARG, "unknown order");
    hspmd_attn_plan* plan = new (std::nothrow) hspmd_attn_plan();
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "out of host memory");
    plan->q_heads = local_q_heads;
    plan->kv_heads = local_kv_heads;
    plan->head_dim = head_dim;
    plan->order = order;
    (void)stream;   // kept in the signature; the upload uses the library's copy stream
    if (hspmd_status rc = fill_packed_plan(plan, cu_seqlens_host, num_seqs, true)) {
        const std::string why_failed = g_last_error;
        hspmd_attn_plan_destroy(plan);
        g_last_error = why_failed;
        return rc;
    }
    *out = plan;
    return HSPMD_OK;
}

hspmd_status hspmd_attn_plan_create(const int32_t* cu_seqlens_host, int32_t num_seqs, int32_t local_q_heads,
                                    int32_t local_kv_heads, int32_t head_dim, void* stream,
                                    hspmd_attn_plan** out) {
    return hspmd_attn_plan_create_ordered(cu_seqlens_host, num_seqs, local_q_heads, local_kv_heads, head_dim,
                                          HSPMD_ORDER_XCD_COST, stream, out);
}

hspmd_status hspmd_attn_plan_update(hspmd_attn_plan* plan, const int32_t* cu_seqlens_host, int32_t num_seqs) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    if (plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was made by hspmd_attn_block_plan_create");
    const std::string why = hspmd::check_pack(cu_seqlens_host, num_seqs, plan->q_heads, plan->kv_heads);
    if (!why.empty()) return fail(HSPMD_ERR_INVALID_ARG, why);
    return fill_packed_plan(plan, cu_seqlens_host, num_seqs, false);
}

hspmd_status hspmd_attn_block_plan_update(hspmd_attn_plan* plan, const int32_t* cu_q_host, const int32_t* cu_k_host,
                                          const int32_t* q_pos_host, const int32_t* k_pos_host, int32_t num_seqs) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    if (!plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was not made by hspmd_attn_block_plan_create");
    const std::string why =
        hspmd::check_block_pack(cu_q_host, cu_k_host, q_pos_host, k_pos_host, num_seqs, plan->q_heads, plan->kv_heads);
    if (!why.empty()) return fail(HSPMD_ERR_INVALID_ARG, why);
    return fill_block_plan(plan, cu_q_host, cu_k_host, q_pos_host, k_pos_host, num_seqs, false);
}

hspmd_status hspmd_attn_plan_destroy(hspmd_attn_plan* plan) {
    if (!plan) return HSPMD_OK;
    hspmd_status rc = HSPMD_OK;
    for (ListSlot& slot : plan->slots) {
        if (slot.block) {
            const hipError_t e = hipFree(slot.block);   // waits for the device: launches that read the slot have ended
            if (e != hipSuccess) rc = fail_hip(e, "hipFree(work lists)");
        }
        if (slot.last_use) {
            const hipError_t e = hipEventDestroy(slot.last_use);
            if (e != hipSuccess) rc = fail_hip(e, "hipEventDestroy(work list slot)");
        }
    }
    delete plan;
    return rc;
}

int64_t hspmd_attn_plan_total_tokens(const hspmd_attn_plan* plan) { return plan ? plan->total_tokens : -1; }

int64_t hspmd_attn_plan_num_items(const hspmd_attn_plan* plan, hspmd_list_kind kind) {
    if (!plan || kind < 0 || kind > 2) return -1;
    return plan->count[kind];
}

size_t hspmd_attn_bwd_workspace_bytes(const hspmd_attn_plan* plan) {
    if (!plan) return 0;
    // -D [Hq,T], -LSE/scale [Hq,T], and 16 floats of -inf
    return (2 * (size_t)plan->q_heads * (size_t)plan->total_tokens + 16) * sizeof(float);
}

static hspmd_status check_strides(const hspmd_attn_plan* plan, int64_t q_token_stride, int64_t kv_token_stride) {
    if (q_token_stride < (int64_t)plan->q_heads * plan->head_dim || q_token_stride % 8 != 0)
        return fail(HSPMD_ERR_INVALID_ARG, "q_token_stride must be a multiple of 8 and >= local_q_heads*head_dim");
    if (kv_token_stride < (int64_t)plan->kv_heads * plan->head_dim || kv_token_stride % 8 != 0)
        return fail(HSPMD_ERR_INVALID_ARG, "kv_token_stride must be a multiple of 8 and >= local_kv_heads*head_dim");
    return HSPMD_OK;
}

// softmax_scale <= 0 selects 1/sqrt(head_dim).  A positive scale must be finite and lie in [2^-60, 2^60]: the backward
// carries the logsumexp in units of raw scores (lse / scale), which must neither overflow nor fall into the
// denormal range of fp32.
static hspmd_status resolve_scale(float softmax_scale, int32_t head_dim, float* scale) {
    if (!(softmax_scale <= 0.f)) {
        if (!std::isfinite(softmax_scale)) return fail(HSPMD_ERR_INVALID_ARG, "softmax_scale is not finite");
        if (softmax_scale < 0x1p-60f || softmax_scale > 0x1p60f)
            return fail(HSPMD_ERR_INVALID_ARG, "a positive softmax_scale must lie in [2^-60, 2^60]");
    }
    *scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)head_dim);
    return HSPMD_OK;
}

hspmd_status hspmd_attn_varlen_fwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                   int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                   void* o, float* lse, void* stream) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    if (plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was made by hspmd_attn_block_plan_create");
    if (plan->total_tokens == 0) return HSPMD_OK;
    if (!q || !k || !v || !o || !lse) return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
        return fail(HSPMD_ERR_INVALID_ARG, "q, k, v, o must be 16-byte aligned");
    if (hspmd_status rc = check_strides(plan, q_token_stride, kv_token_stride)) return rc;
    float scale = 0.f;
    if (hspmd_status rc = resolve_scale(softmax_scale, plan->head_dim, &scale)) return rc;
    hspmd::FwdParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.v = static_cast<const uint16_t*>(v);
    p.o = static_cast<uint16_t*>(o);
    p.lse = lse;
    p.items = plan->items[HSPMD_LIST_FWD];
    p.q_stride = q_token_stride;
    p.kv_stride = kv_token_stride;
    p.total_tokens = plan->total_tokens;
    p.q_heads = plan->q_heads;
    p.group = plan->q_heads / plan->kv_heads;
    p.head_dim = plan->head_dim;
    p.scale_log2 = scale * 1.4426950408889634f;
    p.num_items = (int32_t)plan->count[HSPMD_LIST_FWD];
    p.queue = plan->queue[HSPMD_LIST_FWD];
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t e = timed_launch(0, s, [&] { return hspmd::launch_fwd(p, plan->head_dim, plan->count[HSPMD_LIST_FWD], false, s); });
    if (e != hipSuccess) return fail_hip(e, "forward launch");
    if (const hipError_t m = mark_use(plan, s)) return fail_hip(m, "hipEventRecord(work list slot)");
    return HSPMD_OK;
}

// rope_table == NULL: plain backward
static hspmd_status varlen_bwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v, const void* o,
                               const float* lse, const void* d_o, int64_t q_token_stride, int64_t kv_token_stride,
                               float softmax_scale, void* dq, void* dk, void* dv, hspmd_grad_dtype grad_dtype,
                               const float* rope_table, void* workspace, size_t workspace_bytes, void* stream,
                               bool timed = true) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    if (plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was made by hspmd_attn_block_plan_create");
    if (grad_dtype != HSPMD_GRAD_BF16 && grad_dtype != HSPMD_GRAD_F32)
        return fail(HSPMD_ERR_UNSUPPORTED, "grad_dtype must be HSPMD_GRAD_BF16 or HSPMD_GRAD_F32");
    if (plan->total_tokens == 0) return HSPMD_OK;
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || !workspace)
        return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(dq) ||
        !aligned16(dk) || !aligned16(dv) || !aligned16(workspace))
        return fail(HSPMD_ERR_INVALID_ARG, "tensors and workspace must be 16-byte aligned");
    if (hspmd_status rc = check_strides(plan, q_token_stride, kv_token_stride)) return rc;
    if (workspace_bytes < hspmd_attn_bwd_workspace_bytes(plan))
        return fail(HSPMD_ERR_WORKSPACE_TOO_SMALL, "workspace smaller than hspmd_attn_bwd_workspace_bytes(plan)");
    float scale = 0.f;
    if (hspmd_status rc = resolve_scale(softmax_scale, plan->head_dim, &scale)) return rc;
    hspmd::BwdParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.v = static_cast<const uint16_t*>(v);
    p.o = static_cast<const uint16_t*>(o);
    p.d_o = static_cast<const uint16_t*>(d_o);
    p.lse = lse;
    p.negd = static_cast<float*>(workspace);
    p.nlse = p.negd + (size_t)plan->q_heads * (size_t)plan->total_tokens;
    p.ninf_pad = p.nlse + (size_t)plan->q_heads * (size_t)plan->total_tokens;
    p.dq = dq;
    p.dk = dk;
    p.dv = dv;
    p.q_stride = q_token_stride;
    p.kv_stride = kv_token_stride;
    p.total_tokens = plan->total_tokens;
    p.q_heads = plan->q_heads;
    p.kv_heads = plan->kv_heads;
    p.group = plan->q_heads / plan->kv_heads;
    p.head_dim = plan->head_dim;
    p.grad_f32 = grad_dtype == HSPMD_GRAD_F32 ? 1 : 0;
    p.rope_table = rope_table;
    p.scale = scale;
    p.scale_log2 = scale * 1.4426950408889634f;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // D = rowsum(dO * O) is computed by the dQ pass itself (every (row, head) belongs to exactly one of its items)
    p.items = plan->items[HSPMD_LIST_DQ];
    auto dq_pass = [&] { return hspmd::launch_bwd_dq(p, plan->head_dim, plan->count[HSPMD_LIST_DQ], false, s); };
    hipError_t e = timed ? timed_launch(2, s, dq_pass) : dq_pass();
    if (e != hipSuccess) return fail_hip(e, "backward dQ launch");
    p.items = plan->items[HSPMD_LIST_DKV];
    auto dkv_pass = [&] { return hspmd::launch_bwd_dkv(p, plan->head_dim, plan->count[HSPMD_LIST_DKV], false, s); };
    e = timed ? timed_launch(3, s, dkv_pass) : dkv_pass();
    if (e != hipSuccess) return fail_hip(e, "backward dK/dV launch");
    if (const hipError_t m = mark_use(plan, s)) return fail_hip(m, "hipEventRecord(work list slot)");
    return HSPMD_OK;
}

hspmd_status hspmd_attn_varlen_bwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                   const void* o, const float* lse, const void* d_o,
                                   int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                   void* dq, void* dk, void* dv, hspmd_grad_dtype grad_dtype,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    return varlen_bwd(plan, q, k, v, o, lse, d_o, q_token_stride, kv_token_stride, softmax_scale, dq, dk, dv, grad_dtype,
                      nullptr, workspace, workspace_bytes, stream);
}

// ---- backward with the library's own workspace: for callers that cannot allocate -------------------------------
// The row statistics that the dQ pass leaves for the dK/dV pass live in a fixed device array instead of a buffer
// from the caller.  In host code the array's name is only a handle for hipGetSymbolAddress: the device address is
// looked up once per device and kept; the kernels get that address like any other workspace pointer.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[HSPMD_STATIC_WORKSPACE_BYTES];

namespace {
std::mutex g_scratch_mutex;
std::map<int, void*> g_scratch_address;   // per device: each GPU holds its own copy of the array

hipError_t static_workspace(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    auto it = g_scratch_address.find(dev);
    if (it == g_scratch_address.end()) {
        void* address = nullptr;
        e = hipGetSymbolAddress(&address, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!address) return hipErrorInvalidSymbol;
        it = g_scratch_address.emplace(dev, address).first;
    }
    *out = it->second;
    return hipSuccess;
}
}  // namespace

hspmd_status hspmd_attn_varlen_bwd_static_ws(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                             const void* o, const float* lse, const void* d_o, int64_t q_token_stride,
                                             int64_t kv_token_stride, float softmax_scale, void* dq, void* dk, void* dv,
                                             hspmd_grad_dtype grad_dtype, void* stream) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    const size_t need = hspmd_attn_bwd_workspace_bytes(plan);
    if (need > (size_t)HSPMD_STATIC_WORKSPACE_BYTES)
        return fail(HSPMD_ERR_WORKSPACE_TOO_SMALL,
                    "local_q_heads * total_tokens exceeds what the library's fixed workspace holds "
                    "(HSPMD_STATIC_WORKSPACE_BYTES); use hspmd_attn_varlen_bwd with a workspace of the caller's");
    void* workspace = nullptr;
    const hipError_t e = static_workspace(&workspace);
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(static workspace)");
    // Per-kernel timing creates events on first use; this entry point must not create anything, so it launches
    // untimed whatever the switch says.
    return varlen_bwd(plan, q, k, v, o, lse, d_o, q_token_stride, kv_token_stride, softmax_scale, dq, dk, dv, grad_dtype,
                      nullptr, workspace, (size_t)HSPMD_STATIC_WORKSPACE_BYTES, stream, /*timed=*/false);
}

// ---- rotary position embedding ---------------------------------------------------------------------------------

static hspmd_status check_rope_table(const hspmd_attn_plan* plan, const float* table, int32_t table_positions) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    if (plan->total_tokens == 0 && plan->total_kv_tokens == 0) return HSPMD_OK;
    if (!table) return fail(HSPMD_ERR_INVALID_ARG, "rope table is NULL");
    if (!aligned16(table)) return fail(HSPMD_ERR_INVALID_ARG, "rope table must be 16-byte aligned");
    if (table_positions < plan->max_position)
        return fail(HSPMD_ERR_INVALID_ARG, "rope table has fewer positions than the plan's tokens occupy");
    return HSPMD_OK;
}

size_t hspmd_rope_table_bytes(int32_t positions, int32_t head_dim) {
    if (positions < 0 || !supported_head_dim(head_dim)) return 0;
    return (size_t)positions * (size_t)(head_dim / 2) * 2 * sizeof(float);
}

hspmd_status hspmd_rope_table(float* table, int32_t positions, int32_t head_dim, double base, void* stream) {
    if (positions < 0) return fail(HSPMD_ERR_INVALID_ARG, "positions is negative");
    if (!supported_head_dim(head_dim)) return fail(HSPMD_ERR_UNSUPPORTED, "head_dim must be a multiple of 8 between 8 and 128");
    if (!(base > 0.0) || !std::isfinite(base)) return fail(HSPMD_ERR_INVALID_ARG, "base must be positive and finite");
    if (positions == 0) return HSPMD_OK;
    if (!table) return fail(HSPMD_ERR_INVALID_ARG, "table is NULL");
    if (!aligned16(table)) return fail(HSPMD_ERR_INVALID_ARG, "table must be 16-byte aligned");
    const hipError_t e = hspmd::launch_rope_table(table, positions, head_dim, base, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "rope table launch");
    return HSPMD_OK;
}

hspmd_status hspmd_rope_qk(const hspmd_attn_plan* plan, const void* q, const void* k, int64_t q_token_stride,
                           int64_t kv_token_stride, void* q_out, void* k_out, int64_t q_out_token_stride,
                           int64_t kv_out_token_stride, const float* table, int32_t table_positions, int32_t inverse,
                           void* stream) {
    if (hspmd_status rc = check_rope_table(plan, table, table_positions)) return rc;
    if (plan->total_tokens == 0 && plan->total_kv_tokens == 0) return HSPMD_OK;
    if ((plan->total_tokens > 0 && (!q || !q_out)) || ((plan->is_block ? plan->total_kv_tokens : plan->total_tokens) > 0 && (!k || !k_out)))
        return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned16(q) || !aligned16(k) || !aligned16(q_out) || !aligned16(k_out))
        return fail(HSPMD_ERR_INVALID_ARG, "q, k, q_out, k_out must be 16-byte aligned");
    if (hspmd_status rc = check_strides(plan, q_token_stride, kv_token_stride)) return rc;
    if (hspmd_status rc = check_strides(plan, q_out_token_stride, kv_out_token_stride)) return rc;
    hspmd::RopeParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.q_out = static_cast<uint16_t*>(q_out);
    p.k_out = static_cast<uint16_t*>(k_out);
    p.table = table;
    p.items = plan->items[HSPMD_LIST_FWD];
    p.q_stride = q_token_stride;
    p.kv_stride = kv_token_stride;
    p.q_out_stride = q_out_token_stride;
    p.kv_out_stride = kv_out_token_stride;
    p.q_heads = plan->q_heads;
    p.group = plan->q_heads / plan->kv_heads;
    p.head_dim = plan->head_dim;
    p.sin_sign = inverse ? -1.f : 1.f;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->is_block) {
        // query chunks through the forward list, key chunks through the dK/dV list
        p.block_items = plan->block_items[HSPMD_LIST_FWD];
        hipError_t e = timed_launch(4, s, [&] { return hspmd::launch_rope_block(p, plan->count[HSPMD_LIST_FWD], false, s); });
        if (e != hipSuccess) return fail_hip(e, "rope launch (query chunks)");
        p.block_items = plan->block_items[HSPMD_LIST_DKV];
        e = timed_launch(4, s, [&] { return hspmd::launch_rope_block(p, plan->count[HSPMD_LIST_DKV], true, s); });
        if (e != hipSuccess) return fail_hip(e, "rope launch (key chunks)");
        if (const hipError_t m = mark_use(plan, s)) return fail_hip(m, "hipEventRecord(work list slot)");
        return HSPMD_OK;
    }
    const hipError_t e = timed_launch(4, s, [&] { return hspmd::launch_rope_qk(p, plan->count[HSPMD_LIST_FWD], s); });
    if (e != hipSuccess) return fail_hip(e, "rope launch");
    if (const hipError_t m = mark_use(plan, s)) return fail_hip(m, "hipEventRecord(work list slot)");
    return HSPMD_OK;
}

hspmd_status hspmd_attn_varlen_bwd_rope(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                        const void* o, const float* lse, const void* d_o, int64_t q_token_stride,
                                        int64_t kv_token_stride, float softmax_scale, void* dq, void* dk, void* dv,
                                        hspmd_grad_dtype grad_dtype, const float* table, int32_t table_positions,
                                        void* workspace, size_t workspace_bytes, void* stream) {
    if (plan && plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was made by hspmd_attn_block_plan_create");
    if (hspmd_status rc = check_rope_table(plan, table, table_positions)) return rc;
    return varlen_bwd(plan, q, k, v, o, lse, d_o, q_token_stride, kv_token_stride, softmax_scale, dq, dk, dv, grad_dtype,
                      table, workspace, workspace_bytes, stream);
}

hspmd_status hspmd_attn_estimate_ms(const int32_t* cu_seqlens, int32_t num_seqs, int32_t local_q_heads,
                                    int32_t local_kv_heads, int32_t head_dim, double* fwd_ms, double* bwd_ms) {
    if (!fwd_ms || !bwd_ms) return fail(HSPMD_ERR_INVALID_ARG, "null pointer");
    const std::string why = hspmd::check_pack(cu_seqlens, num_seqs, local_q_heads, local_kv_heads);
    if (!why.empty()) return fail(HSPMD_ERR_INVALID_ARG, why);
    if (!supported_head_dim(head_dim)) return fail(HSPMD_ERR_UNSUPPORTED, "head_dim must be a multiple of 8 between 8 and 128");
    try {
        head_dim = hspmd::tile_width(head_dim);   // a narrower head runs on the next tile width up
        *fwd_ms = hspmd::estimate_pass_us(HSPMD_LIST_FWD, cu_seqlens, num_seqs, local_q_heads, local_kv_heads, head_dim) * 1e-3;
        *bwd_ms = (hspmd::estimate_pass_us(HSPMD_LIST_DQ, cu_seqlens, num_seqs, local_q_heads, local_kv_heads, head_dim) +
                   hspmd::estimate_pass_us(HSPMD_LIST_DKV, cu_seqlens, num_seqs, local_q_heads, local_kv_heads, head_dim)) * 1e-3;
    } catch (const std::bad_alloc&) {
        return fail(HSPMD_ERR_INVALID_ARG, "out of host memory while building the work lists");
    }
    return HSPMD_OK;
}

// ------------------------------------------------------------------------------ block variant
hspmd_status hspmd_attn_block_schedule(hspmd_list_kind kind, const int32_t* cu_q, const int32_t* cu_k,
                                       const int32_t* q_pos, const int32_t* k_pos, int32_t num_seqs,
                                       int32_t local_q_heads, int32_t local_kv_heads, int32_t num_queues,
                                       hspmd_block_item* items, int64_t capacity, int64_t* count) {
    if (kind != HSPMD_LIST_FWD && kind != HSPMD_LIST_DQ && kind != HSPMD_LIST_DKV)
        return fail(HSPMD_ERR_INVALID_ARG, "unknown list kind");
    if (!count) return fail(HSPMD_ERR_INVALID_ARG, "count is NULL");
    if (num_queues < 1) return fail(HSPMD_ERR_INVALID_ARG, "num_queues must be >= 1");
    if (capacity < 0 || (capacity > 0 && !items)) return fail(HSPMD_ERR_INVALID_ARG, "items is NULL");
    const std::string why = hspmd::check_block_pack(cu_q, cu_k, q_pos, k_pos, num_seqs, local_q_heads, local_kv_heads);
    if (!why.empty()) return fail(HSPMD_ERR_INVALID_ARG, why);
    std::vector<hspmd_block_item> list;
    try {
        list = hspmd::build_block_list(kind, cu_q, cu_k, q_pos, k_pos, num_seqs, local_q_heads, local_kv_heads, num_queues);
    } catch (const std::bad_alloc&) {
        return fail(HSPMD_ERR_INVALID_ARG, "out of host memory while building the work list");
    }
    *count = (int64_t)list.size();
    if (capacity == 0) return HSPMD_OK;
    if ((int64_t)list.size() > capacity) return fail(HSPMD_ERR_INVALID_ARG, "items buffer too small");
    if (!list.empty()) std::memcpy(items, list.data(), list.size() * sizeof(hspmd_block_item));
    return HSPMD_OK;
}

hspmd_status hspmd_attn_block_plan_create(const int32_t* cu_q_host, const int32_t* cu_k_host, const int32_t* q_pos_host,
                                          const int32_t* k_pos_host, int32_t num_seqs, int32_t local_q_heads,
                                          int32_t local_kv_heads, int32_t head_dim, void* stream, hspmd_attn_plan** out) {
    if (!out) return fail(HSPMD_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    const std::string why =
        hspmd::check_block_pack(cu_q_host, cu_k_host, q_pos_host, k_pos_host, num_seqs, local_q_heads, local_kv_heads);
    if (!why.empty()) return fail(HSPMD_ERR_INVALID_ARG, why);
    if (!supported_head_dim(head_dim)) return fail(HSPMD_ERR_UNSUPPORTED, "head_dim must be a multiple of 8 between 8 and 128");
    hspmd_attn_plan* plan = new (std::nothrow) hspmd_attn_plan();
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "out of host memory");
    plan->is_block = true;
    plan->q_heads = local_q_heads;
    plan->kv_heads = local_kv_heads;
    plan->head_dim = head_dim;
    (void)stream;   // kept in the signature; the upload uses the library's copy stream
    if (hspmd_status rc = fill_block_plan(plan, cu_q_host, cu_k_host, q_pos_host, k_pos_host, num_seqs, true)) {
        const std::string why_failed = g_last_error;
        hspmd_attn_plan_destroy(plan);
        g_last_error = why_failed;
        return rc;
    }
    *out = plan;
    return HSPMD_OK;
}

int64_t hspmd_attn_plan_total_kv_tokens(const hspmd_attn_plan* plan) {
    if (!plan) return -1;
    return plan->is_block ? plan->total_kv_tokens : plan->total_tokens;
}

hspmd_status hspmd_attn_block_fwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                  int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                  float* o_partial, float* lse_partial, void* stream) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    if (!plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was not made by hspmd_attn_block_plan_create");
    if (plan->total_tokens == 0) return HSPMD_OK;
    if (!q || !o_partial || !lse_partial || (plan->total_kv_tokens > 0 && (!k || !v)))
        return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o_partial))
        return fail(HSPMD_ERR_INVALID_ARG, "q, k, v, o_partial must be 16-byte aligned");
    if (hspmd_status rc = check_strides(plan, q_token_stride, kv_token_stride)) return rc;
    float scale = 0.f;
    if (hspmd_status rc = resolve_scale(softmax_scale, plan->head_dim, &scale)) return rc;
    hspmd::FwdParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.v = static_cast<const uint16_t*>(v);
    p.o_f32 = o_partial;
    p.lse = lse_partial;
    p.block_items = plan->block_items[HSPMD_LIST_FWD];
    p.q_stride = q_token_stride;
    p.kv_stride = kv_token_stride;
    p.total_tokens = plan->total_tokens;
    p.q_heads = plan->q_heads;
    p.group = plan->q_heads / plan->kv_heads;
    p.head_dim = plan->head_dim;
    p.scale_log2 = scale * 1.4426950408889634f;
    p.num_items = (int32_t)plan->count[HSPMD_LIST_FWD];
    p.queue = plan->queue[HSPMD_LIST_FWD];
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t e = timed_launch(0, s, [&] { return hspmd::launch_fwd(p, plan->head_dim, plan->count[HSPMD_LIST_FWD], true, s); });
    if (e != hipSuccess) return fail_hip(e, "block forward launch");
    if (const hipError_t m = mark_use(plan, s)) return fail_hip(m, "hipEventRecord(work list slot)");
    return HSPMD_OK;
}

hspmd_status hspmd_attn_merge(int64_t total_tokens, int32_t local_q_heads, int32_t head_dim, const float* o_a,
                              const float* lse_a, const float* o_b, const float* lse_b, float* o_out, float* lse_out,
                              void* o_out_bf16, void* stream) {
    if (total_tokens < 0 || local_q_heads <= 0) return fail(HSPMD_ERR_INVALID_ARG, "bad token or head count");
    if (!supported_head_dim(head_dim)) return fail(HSPMD_ERR_UNSUPPORTED, "head_dim must be a multiple of 8 between 8 and 128");
    if (total_tokens == 0) return HSPMD_OK;
    if (!o_a || !lse_a || !o_b || !lse_b || !o_out || !lse_out) return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned16(o_a) || !aligned16(o_b) || !aligned16(o_out) || !aligned16(o_out_bf16))
        return fail(HSPMD_ERR_INVALID_ARG, "O tensors must be 16-byte aligned");
    if (o_out == o_b || lse_out == lse_b) return fail(HSPMD_ERR_INVALID_ARG, "the output may alias operand a only");
    hspmd::MergeParams p{};
    p.o_a = o_a; p.lse_a = lse_a; p.o_b = o_b; p.lse_b = lse_b;
    p.o_out = o_out; p.lse_out = lse_out;
    p.o_out_bf16 = static_cast<uint16_t*>(o_out_bf16);
    p.total_tokens = total_tokens;
    p.q_heads = local_q_heads;
    p.head_dim = head_dim;
    const hipError_t e = hspmd::launch_merge(p, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "merge launch");
    return HSPMD_OK;
}

// rope_table == NULL: plain block backward
static hspmd_status block_bwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v, const void* o,
                              const float* lse, const void* d_o, int64_t q_token_stride, int64_t kv_token_stride,
                              float softmax_scale, float* dq, int32_t dq_accumulate, float* dk, float* dv,
                              int32_t reuse_statistics, const float* rope_table, void* workspace, size_t workspace_bytes,
                              void* stream) {
    if (!plan) return fail(HSPMD_ERR_INVALID_ARG, "plan is NULL");
    if (!plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was not made by hspmd_attn_block_plan_create");
    if (plan->total_tokens == 0 && plan->total_kv_tokens == 0) return HSPMD_OK;
    if (!workspace) return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (plan->total_tokens > 0 && (!q || !d_o || !dq || (!reuse_statistics && (!o || !lse))))
        return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (plan->total_kv_tokens > 0 && (!k || !v || !dk || !dv)) return fail(HSPMD_ERR_INVALID_ARG, "null tensor pointer");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(dq) ||
        !aligned16(dk) || !aligned16(dv) || !aligned16(workspace))
        return fail(HSPMD_ERR_INVALID_ARG, "tensors and workspace must be 16-byte aligned");
    if (hspmd_status rc = check_strides(plan, q_token_stride, kv_token_stride)) return rc;
    if (workspace_bytes < hspmd_attn_bwd_workspace_bytes(plan))
        return fail(HSPMD_ERR_WORKSPACE_TOO_SMALL, "workspace smaller than hspmd_attn_bwd_workspace_bytes(plan)");
    float scale = 0.f;
    if (hspmd_status rc = resolve_scale(softmax_scale, plan->head_dim, &scale)) return rc;
    hspmd::BwdParams p{};
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k);
    p.v = static_cast<const uint16_t*>(v);
    p.o = static_cast<const uint16_t*>(o);
    p.d_o = static_cast<const uint16_t*>(d_o);
    p.lse = lse;
    p.negd = static_cast<float*>(workspace);
    p.nlse = p.negd + (size_t)plan->q_heads * (size_t)plan->total_tokens;
    p.ninf_pad = p.nlse + (size_t)plan->q_heads * (size_t)plan->total_tokens;
    p.dq = dq;
    p.dk = dk;
    p.dv = dv;
    p.q_stride = q_token_stride;
    p.kv_stride = kv_token_stride;
    p.total_tokens = plan->total_tokens;
    p.q_heads = plan->q_heads;
    p.kv_heads = plan->kv_heads;
    p.group = plan->q_heads / plan->kv_heads;
    p.head_dim = plan->head_dim;
    p.grad_f32 = 1;
    p.dq_accumulate = dq_accumulate ? 1 : 0;
    p.rope_table = rope_table;
    p.scale = scale;
    p.scale_log2 = scale * 1.4426950408889634f;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    if (!reuse_statistics && plan->total_tokens > 0) {
        e = timed_launch(1, s, [&] { return hspmd::launch_bwd_dsum(p, plan->head_dim, s); });
        if (e != hipSuccess) return fail_hip(e, "backward D launch");
    }
    p.block_items = plan->block_items[HSPMD_LIST_DQ];
    e = timed_launch(2, s, [&] { return hspmd::launch_bwd_dq(p, plan->head_dim, plan->count[HSPMD_LIST_DQ], true, s); });
    if (e != hipSuccess) return fail_hip(e, "block backward dQ launch");
    p.block_items = plan->block_items[HSPMD_LIST_DKV];
    e = timed_launch(3, s, [&] { return hspmd::launch_bwd_dkv(p, plan->head_dim, plan->count[HSPMD_LIST_DKV], true, s); });
    if (e != hipSuccess) return fail_hip(e, "block backward dK/dV launch");
    if (const hipError_t m = mark_use(plan, s)) return fail_hip(m, "hipEventRecord(work list slot)");
    return HSPMD_OK;
}

hspmd_status hspmd_attn_block_bwd(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                  const void* o, const float* lse, const void* d_o,
                                  int64_t q_token_stride, int64_t kv_token_stride, float softmax_scale,
                                  float* dq, int32_t dq_accumulate, float* dk, float* dv, int32_t reuse_statistics,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    return block_bwd(plan, q, k, v, o, lse, d_o, q_token_stride, kv_token_stride, softmax_scale, dq, dq_accumulate, dk, dv,
                     reuse_statistics, nullptr, workspace, workspace_bytes, stream);
}

hspmd_status hspmd_attn_block_bwd_rope(const hspmd_attn_plan* plan, const void* q, const void* k, const void* v,
                                       const void* o, const float* lse, const void* d_o, int64_t q_token_stride,
                                       int64_t kv_token_stride, float softmax_scale, float* dq, int32_t dq_accumulate,
                                       float* dk, float* dv, int32_t reuse_statistics, const float* table,
                                       int32_t table_positions, void* workspace, size_t workspace_bytes, void* stream) {
    if (plan && !plan->is_block) return fail(HSPMD_ERR_INVALID_ARG, "plan was not made by hspmd_attn_block_plan_create");
    if (hspmd_status rc = check_rope_table(plan, table, table_positions)) return rc;
    return block_bwd(plan, q, k, v, o, lse, d_o, q_token_stride, kv_token_stride, softmax_scale, dq, dq_accumulate, dk, dv,
                     reuse_statistics, table, workspace, workspace_bytes, stream);
}

hspmd_status hspmd_profile_enable(int32_t on) {
    g_profile_on.store(on != 0, std::memory_order_relaxed);
    return HSPMD_OK;
}

hspmd_status hspmd_profile_read(double* ms, int64_t* launches) {
    if (!ms || !launches) return fail(HSPMD_ERR_INVALID_ARG, "null pointer");
    return drain_profile_records([&](int kernel, double t) {
        ms[kernel] += t;
        launches[kernel] += 1;
    });
}

hspmd_status hspmd_profile_read_stats(double* sum_ms, int64_t* launches, double* min_ms, double* median_ms) {
    if (!sum_ms || !launches || !min_ms || !median_ms) return fail(HSPMD_ERR_INVALID_ARG, "null pointer");
    std::vector<double> samples[HSPMD_NUM_KERNELS];
    const hspmd_status rc = drain_profile_records([&](int kernel, double t) { samples[kernel].push_back(t); });
    for (int k = 0; k < HSPMD_NUM_KERNELS; ++k) {
        std::vector<double>& v = samples[k];
        sum_ms[k] = 0.0;
        launches[k] = (int64_t)v.size();
        min_ms[k] = median_ms[k] = 0.0;
        if (v.empty()) continue;
        std::sort(v.begin(), v.end());
        for (double t : v) sum_ms[k] += t;
        min_ms[k] = v.front();
        median_ms[k] = v.size() % 2 ? v[v.size() / 2] : 0.5 * (v[v.size() / 2 - 1] + v[v.size() / 2]);
    }
    return rc;
}

size_t hspmd_probe_scratch_bytes(void) { return (size_t)hspmd::kProbeMaxGrid * hspmd::kProbeThreads * sizeof(float); }

static hspmd_status probe_mfma(int64_t mfma_per_wave, bool varied_operands, void* scratch_out, size_t scratch_bytes,
                               void* stream, double* tflops) {
    if (!scratch_out || !tflops) return fail(HSPMD_ERR_INVALID_ARG, "null pointer");
    if (mfma_per_wave <= 0) return fail(HSPMD_ERR_INVALID_ARG, "mfma_per_wave must be positive");
    if (scratch_bytes < hspmd_probe_scratch_bytes()) return fail(HSPMD_ERR_WORKSPACE_TOO_SMALL, "probe scratch too small");
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return fail_hip(e, "device query");
    const int grid = hspmd::probe_grid(cus);
    if (grid <= 0 || grid > hspmd::kProbeMaxGrid) return fail(HSPMD_ERR_UNSUPPORTED, "unexpected compute unit count");
    const int64_t rounds = (mfma_per_wave + 15) / 16;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t start = nullptr, stop = nullptr;
    e = hipEventCreate(&start);
    if (e == hipSuccess) e = hipEventCreate(&stop);
    if (e == hipSuccess) e = hspmd::launch_mfma_probe((float*)scratch_out, rounds, grid, varied_operands, s);   // untimed
    if (e == hipSuccess) e = hipEventRecord(start, s);
    if (e == hipSuccess) e = hspmd::launch_mfma_probe((float*)scratch_out, rounds, grid, varied_operands, s);
    if (e == hipSuccess) e = hipEventRecord(stop, s);
    if (e == hipSuccess) e = hipEventSynchronize(stop);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, start, stop);
    if (start) (void)hipEventDestroy(start);
    if (stop) (void)hipEventDestroy(stop);
    if (e != hipSuccess) return fail_hip(e, "mfma probe");
    // one 32x32x16 MFMA = 2 * 32 * 32 * 16 flops; 4 waves per workgroup
    const double flops = (double)grid * 4.0 * (double)(rounds * 16) * 32768.0;
    *tflops = ms > 0.f ? flops / ((double)ms * 1e-3) / 1e12 : 0.0;
    return HSPMD_OK;
}

hspmd_status hspmd_probe_mfma_rate(hspmd_probe_mode mode, int64_t mfma_per_wave, void* scratch_out, size_t scratch_bytes,
                                   void* stream, double* tflops) {
    if (mode < HSPMD_PROBE_32X32X16_CONSTANT || mode > HSPMD_PROBE_IDLE_1024) return fail(HSPMD_ERR_INVALID_ARG, "unknown probe mode");
    if (!scratch_out || !tflops) return fail(HSPMD_ERR_INVALID_ARG, "null pointer");
    if (mfma_per_wave <= 0) return fail(HSPMD_ERR_INVALID_ARG, "mfma_per_wave must be positive");
    if (scratch_bytes < hspmd_probe_scratch_bytes()) return fail(HSPMD_ERR_WORKSPACE_TOO_SMALL, "probe scratch too small");
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return fail_hip(e, "device query");
    const int grid = hspmd::probe_mode_grid(mode, cus);
    if (grid <= 0 || grid > hspmd::kProbeMaxGrid) return fail(HSPMD_ERR_UNSUPPORTED, "unexpected compute unit count");
    const int64_t rounds = (mfma_per_wave + 15) / 16;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t start = nullptr, stop = nullptr;
    e = hipEventCreate(&start);
    if (e == hipSuccess) e = hipEventCreate(&stop);
    if (e == hipSuccess) e = hspmd::launch_mfma_probe_mode(mode, (float*)scratch_out, rounds, grid, s);   // untimed
    if (e == hipSuccess) e = hipEventRecord(start, s);
    if (e == hipSuccess) e = hspmd::launch_mfma_probe_mode(mode, (float*)scratch_out, rounds, grid, s);
    if (e == hipSuccess) e = hipEventRecord(stop, s);
    if (e == hipSuccess) e = hipEventSynchronize(stop);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, start, stop);
    if (start) (void)hipEventDestroy(start);
    if (stop) (void)hipEventDestroy(stop);
    if (e != hipSuccess) return fail_hip(e, "mfma probe");
    // a round = 16 products 32x32x16 (or 32 products 16x16x32) = 16 * 2 * 32 * 32 * 16 flops; 4 waves per workgroup
    const double flops = (double)grid * 4.0 * (double)(rounds * 16) * 32768.0;
    *tflops = ms > 0.f ? flops / ((double)ms * 1e-3) / 1e12 : 0.0;
    return HSPMD_OK;
}

hspmd_status hspmd_probe_mfma_tflops(int64_t mfma_per_wave, void* scratch_out, size_t scratch_bytes, void* stream,
                                     double* tflops) {
    return probe_mfma(mfma_per_wave, false, scratch_out, scratch_bytes, stream, tflops);
}

hspmd_status hspmd_probe_mfma_tflops_varied(int64_t mfma_per_wave, void* scratch_out, size_t scratch_bytes, void* stream,
                                            double* tflops) {
    return probe_mfma(mfma_per_wave, true, scratch_out, scratch_bytes, stream, tflops);
}

const char* hspmd_kernel_name(int32_t kernel) {
    static const char* const names[HSPMD_NUM_KERNELS] = {"fwd_kernel", "bwd_dsum_kernel", "bwd_dq_kernel",
                                                         "bwd_dkv_kernel", "rope_qk_kernel"};
    return (kernel >= 0 && kernel < HSPMD_NUM_KERNELS) ? names[kernel] : nullptr;
}

}  // extern "C"
