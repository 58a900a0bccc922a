// Host side of the C ABI: argument validation, static sizes, workspace layout, entry points.
#include <cmath>
#include <cstring>
#include <mutex>

#include "common.h"
#include "schedule.h"

namespace capmoe {

int validate(const moe_desc_t* d) {
    if (!d) return MOE_ERR_INVALID_ARG;
    if (d->n_tokens < 0 || d->d_model < 1 || d->n_experts < 1 || d->top_k < 1 || d->d_hidden < 1 ||
        d->device_groups < 1)
        return MOE_ERR_INVALID_ARG;
    if (d->overselect < 0 || (d->max_experts != 0 && d->max_experts != 1)) return MOE_ERR_INVALID_ARG;
    if ((int64_t)d->top_k + d->overselect > d->n_experts) return MOE_ERR_INVALID_ARG;
    if (d->n_tokens % d->device_groups != 0 || d->n_experts % d->device_groups != 0) return MOE_ERR_INVALID_ARG;
    if (d->mode < MOE_MODE_NONE || d->mode > MOE_MODE_EXPANDED_DROP) return MOE_ERR_INVALID_ARG;
    if (d->capacity_scope < MOE_SCOPE_LOCAL || d->capacity_scope > MOE_SCOPE_GLOBAL_DEVICE) return MOE_ERR_INVALID_ARG;
    if (d->dtype != MOE_DTYPE_F32 && d->dtype != MOE_DTYPE_BF16) return MOE_ERR_INVALID_ARG;
    if (d->metric < MOE_METRIC_SCORE || d->metric > MOE_METRIC_RANDOM) return MOE_ERR_INVALID_ARG;
    if (std::isnan(d->gamma) || d->gamma < 0.0) return MOE_ERR_INVALID_ARG;
    if (d->n_experts > kMaxExperts || d->top_k + d->overselect > kMaxTopK) return MOE_ERR_UNSUPPORTED;
    const int slots = d->top_k + d->overselect + (d->mode == MOE_MODE_EXPANDED_DROP ? d->n_experts / d->device_groups : 0);
    if (slots > 255) return MOE_ERR_UNSUPPORTED;
    if ((int64_t)d->n_tokens * d->n_experts >= (int64_t)1 << 30) return MOE_ERR_UNSUPPORTED;
    if ((int64_t)d->n_tokens * slots >= (int64_t)1 << 31) return MOE_ERR_UNSUPPORTED;
    // rows are moved in 16-byte pieces
    const int per16 = d->dtype == MOE_DTYPE_BF16 ? 8 : 4;
    if (d->d_model % per16 != 0) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

Sizes derive(const moe_desc_t& d) {
    Sizes s;
    const bool local = d.capacity_scope == MOE_SCOPE_LOCAL || d.capacity_scope == MOE_SCOPE_LOCAL_DEVICE;
    const bool per_device = d.capacity_scope == MOE_SCOPE_LOCAL_DEVICE || d.capacity_scope == MOE_SCOPE_GLOBAL_DEVICE;
    s.n_blocks = local ? d.device_groups : 1;
    s.seg_tokens = d.n_tokens / s.n_blocks;
    s.group_experts = d.n_experts / d.device_groups;
    s.group_tokens = d.n_tokens / d.device_groups;
    s.span = per_device ? s.group_experts : 1;
    const long long seg_pairs = (long long)s.seg_tokens * s.span;  // most pairs a segment can hold
    if (d.mode == MOE_MODE_NONE || (std::isinf(d.gamma) && d.gamma > 0)) {
        s.cap = (int)seg_pairs;
    } else {
        // capacity as in Alg. 1: gamma times (N*k), divided by E, truncated; for a device budget the
        // numerator carries the n_l experts of the device (Sec. 5.2); never above what the segment holds
        const double c =
            d.gamma * (double)((long long)s.seg_tokens * (long long)d.top_k * s.span) / (double)d.n_experts;
        if (!(c > 0.0))
            s.cap = 0;
        else if (c >= (double)seg_pairs)
            s.cap = (int)seg_pairs;
        else
            s.cap = (int)c;
    }
    s.list_k = d.top_k + d.overselect;
    s.slots = s.list_k + (d.mode == MOE_MODE_EXPANDED_DROP ? s.group_experts : 0);
    const int64_t by_tokens = (int64_t)d.n_tokens * (s.slots < d.n_experts ? s.slots : d.n_experts);
    const int64_t by_capacity = (int64_t)s.n_blocks * (d.n_experts / s.span) * s.cap;
    s.max_rows = by_tokens < by_capacity ? by_tokens : by_capacity;
    s.elem = d.dtype == MOE_DTYPE_BF16 ? 2 : 4;
    return s;
}

DropWorkspace drop_workspace(const moe_desc_t& d, const Sizes& s, void* base) {
    DropWorkspace w;
    char* p = (char*)base;
    size_t off = 0;
    const size_t ne = (size_t)d.n_tokens * d.n_experts;
    const size_t segs = (size_t)s.n_blocks * d.n_experts;
    w.key_t = (uint32_t*)(p + off);
    off += align256(ne * 4);
    w.slot_t = (uint8_t*)(p + off);
    off += align256(ne);
    w.seg_tau = (uint32_t*)(p + off);
    off += align256(segs * 4);
    w.seg_need = (int32_t*)(p + off);
    off += align256(segs * 4);
    w.bytes = off;
    return w;
}

FfnWorkspace ffn_workspace(const moe_desc_t& d, const Sizes& s, void* base) {
    FfnWorkspace w;
    char* p = (char*)base;
    size_t off = 0;
    const bool bf16 = d.dtype == MOE_DTYPE_BF16;
    w.big.tile_m = bf16 ? kFfnTileM : kFfnTileMF32;

    w.big.max_tiles = (int)(s.max_rows / w.big.tile_m) + d.n_experts;
    w.small.tile_m = kFfnTileSmall;
    w.small_max = bf16 ? kFfnSmallMax : 0;
    // remainders: one per expert at most
    w.small.max_tiles = bf16 ? d.n_experts * (kFfnSmallMax / kFfnTileSmall) : 0;
    w.small.max_launch = w.small.max_tiles;
    w.big.max_launch = w.big.max_tiles;

    w.hidden = p + off;
    off += align256((size_t)(s.max_rows > 0 ? s.max_rows : 1) * d.d_hidden * s.elem);
    // both kinds in one list (the gate/up GEMM's order)
    w.all.tile_m = 0;
    w.all.max_tiles = w.big.max_tiles + w.small.max_tiles;
    w.all.max_launch = w.all.max_tiles;
    for (TileList* t : {&w.big, &w.small, &w.all}) {
        const size_t n = align256((size_t)(t->max_tiles > 0 ? t->max_tiles : 1) * 4);
        t->expert = (int32_t*)(p + off);
        off += n;
        t->row0 = (int32_t*)(p + off);
        off += n;
        t->rows = (int32_t*)(p + off);
        off += n;
        t->count = (int32_t*)(p + off);
        off += 256;
    }
    w.split_hdr = nullptr;
    w.split_counter = nullptr;
    w.split_partial = nullptr;
    if (bf16) {
        w.split_hdr = (int32_t*)(p + off);
        off += 256;
        w.split_counter = (int32_t*)(p + off);
        off += align256((size_t)4 * kFfnSplitUnits * 4);
        w.split_partial = (float*)(p + off);
        off += align256((size_t)kFfnSplitUnits * (kFfnTileM + kFfnTileSmall) * 256 * 4);
    }
    w.bytes = off;
    return w;
}

thread_local moe_profile_t* t_profile = nullptr;

int compute_units() {
    static std::atomic<int> cus[kMaxDevices] = {};
    const int dev = current_device();
    int c = cus[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        if (hipDeviceGetAttribute(&c, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || c <= 0) c = 256;
        cus[dev].store(c, std::memory_order_relaxed);
    }
    return c;
}

// gathered: the first GEMM fetches its rows from the unpermuted x (moe_dispatch_ffn): the bf16 kernels address x
// through one buffer descriptor with 32-bit byte offsets, so x must stay below 4 GiB
static int ffn_shape_supported(const moe_desc_t& d, bool gathered) {
    if (d.dtype != MOE_DTYPE_BF16) return MOE_OK;
    if (d.d_model % 128 != 0 || d.d_hidden % 128 != 0) return MOE_ERR_UNSUPPORTED;
    if (gathered && (uint64_t)d.n_tokens * (uint64_t)d.d_model >= (1ull << 31)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

}  // namespace capmoe

using namespace capmoe;

static bool misaligned16(const void* p) { return ((uintptr_t)p & 15) != 0; }

// Scratch memory of moe_route_topk_static: the split-K partial sums of the router GEMM, for callers that can
// neither allocate nor pass a workspace.  One copy per GPU, held from the moment the library is loaded on it.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// the current device's copy of `scratch` (looked up once per device, with that device current)
static int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MOE_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}

static int route_topk_impl(const moe_desc_t* desc, const void* x, const float* w_router, const float* bias,
                   int use_given_logits, float* logits, float* scores, int32_t* topk_idx, float* topk_score,
                   void* workspace, size_t workspace_bytes, void* stream) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    if (desc->n_tokens == 0) return MOE_OK;  // nothing to route; empty arrays may be null
    if (!logits || !scores || !topk_idx || !topk_score) return MOE_ERR_INVALID_ARG;
    if (!use_given_logits && (!x || !w_router)) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const float* partial = nullptr;
    int ksplit = 1;
    if (!use_given_logits) {
        const RouteWorkspace ws = route_workspace(*desc, workspace);
        if (ws.use_mfma) {
            if (ws.bytes > 0) {
                if (!workspace) return MOE_ERR_INVALID_ARG;
                if (workspace_bytes < ws.bytes) return MOE_ERR_WORKSPACE_TOO_SMALL;
                if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
            }
            if (misaligned16(x) || misaligned16(w_router)) return MOE_ERR_INVALID_ARG;
            if (launch_router_mfma(*desc, ws, x, w_router, bias, logits, st) != hipSuccess) return MOE_ERR_HIP;
            if (ws.ksplit > 1) {
                partial = ws.partial;
                ksplit = ws.ksplit;
            }
        } else if (launch_router_logits(*desc, x, w_router, bias, logits, st) != hipSuccess) {
            return MOE_ERR_HIP;
        }
    }
    if (launch_softmax_topk(*desc, logits, partial, ksplit, bias, scores, topk_idx, topk_score, st) != hipSuccess)
        return MOE_ERR_HIP;
    return MOE_OK;
}

// schedule != nullptr: the drop also builds the tile schedule of the expert GEMMs (moe_layer_forward)
static int capacity_drop_impl(const moe_desc_t* desc, const float* scores, const int32_t* topk_idx,
                              const uint8_t* token_class, uint32_t seed, int32_t* expert_count, int32_t* seg_count,
                              int32_t* expert_offset, int32_t* row_token, float* row_weight, int32_t* pair_row,
                              void* workspace, size_t workspace_bytes, const FfnScheduleArgs* schedule, void* stream) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    if (!expert_count || !seg_count || !expert_offset || !workspace) return MOE_ERR_INVALID_ARG;
    const Sizes s = derive(*desc);
    // arrays that are empty for this descriptor may be null
    if (desc->n_tokens > 0 && (!scores || !topk_idx || !pair_row)) return MOE_ERR_INVALID_ARG;
    if (s.max_rows > 0 && (!row_token || !row_weight)) return MOE_ERR_INVALID_ARG;
    if (s.max_rows >= (int64_t)1 << 31) return MOE_ERR_UNSUPPORTED;
    // the kernels fetch top-k lists, score rows and keys in 16-byte pieces
    if (misaligned16(scores) || misaligned16(topk_idx) || misaligned16(pair_row)) return MOE_ERR_INVALID_ARG;
    const DropWorkspace ws = drop_workspace(*desc, s, workspace);
    if (workspace_bytes < ws.bytes) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
    if (launch_capacity_drop(*desc, s, ws, scores, topk_idx, token_class, seed, expert_count, seg_count, expert_offset,
                             row_token, row_weight, pair_row, schedule, (hipStream_t)stream) != hipSuccess)
        return MOE_ERR_HIP;
    return MOE_OK;
}

extern "C" {

const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported shape or type";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MOE_ERR_HIP: return "HIP launch failed";
        case MOE_ERR_SCRATCH_LIMIT: return "problem needs more scratch memory than the built-in buffer holds";
        default: return "unknown status";
    }
}

int moe_profile_attach(moe_profile_t* table) {
    t_profile = table;
    return MOE_OK;
}

int moe_query(const moe_desc_t* desc, int32_t* cap, int32_t* slots_per_token, int64_t* max_rows,
              size_t* workspace_bytes) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    const Sizes s = derive(*desc);
    if (s.max_rows >= (int64_t)1 << 31) return MOE_ERR_UNSUPPORTED;
    if (cap) *cap = s.cap;
    if (slots_per_token) *slots_per_token = s.slots;
    if (max_rows) *max_rows = s.max_rows;
    if (workspace_bytes) {
        const size_t a = drop_workspace(*desc, s, nullptr).bytes;
        const size_t b = ffn_workspace(*desc, s, nullptr).bytes;
        const size_t c = route_workspace(*desc, nullptr).bytes;
        *workspace_bytes = a > b ? (a > c ? a : c) : (b > c ? b : c);
    }
    return MOE_OK;
}

int moe_ffn_schedule_query(const moe_desc_t* desc, const int32_t* expert_count, int compute_units, int32_t* tiles,
                           int32_t* header) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    if (!expert_count || !tiles || !header || compute_units < 8 || compute_units > 4096) return MOE_ERR_INVALID_ARG;
    const Sizes s = derive(*desc);
    if (s.max_rows >= (int64_t)1 << 31) return MOE_ERR_UNSUPPORTED;
    int64_t rows = 0;
    for (int e = 0; e < desc->n_experts; ++e) {
        if (expert_count[e] < 0) return MOE_ERR_INVALID_ARG;
        rows += expert_count[e];
    }
    if (rows > s.max_rows) return MOE_ERR_INVALID_ARG;
    ffn_schedule_on_host(*desc, ffn_workspace(*desc, s, nullptr), expert_count, compute_units, tiles, header);
    return MOE_OK;
}

int moe_route_topk(const moe_desc_t* desc, const void* x, const float* w_router, const float* bias,
                   int use_given_logits, float* logits, float* scores, int32_t* topk_idx, float* topk_score,
                   void* workspace, size_t workspace_bytes, void* stream) {
    return route_topk_impl(desc, x, w_router, bias, use_given_logits, logits, scores, topk_idx, topk_score, workspace,
                           workspace_bytes, stream);
}

int moe_route_topk_static(const moe_desc_t* desc, const void* x, const float* w_router, const float* bias,
                          int use_given_logits, float* logits, float* scores, int32_t* topk_idx, float* topk_score,
                          void* stream) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    // the size check comes before anything touches the device: a refusal enqueues nothing
    if (!use_given_logits && route_workspace(*desc, nullptr).bytes > kStaticScratchBytes) return MOE_ERR_SCRATCH_LIMIT;
    void* ptr = nullptr;
    const int st = static_scratch(&ptr);
    if (st != MOE_OK) return st;
    return route_topk_impl(desc, x, w_router, bias, use_given_logits, logits, scores, topk_idx, topk_score, ptr,
                           kStaticScratchBytes, stream);
}

int moe_capacity_drop_ranked(const moe_desc_t* desc, const float* scores, const int32_t* topk_idx,
                             const uint8_t* token_class, uint32_t seed, int32_t* expert_count, int32_t* seg_count,
                             int32_t* expert_offset, int32_t* row_token, float* row_weight, int32_t* pair_row,
                             void* workspace, size_t workspace_bytes, void* stream) {
    return capacity_drop_impl(desc, scores, topk_idx, token_class, seed, expert_count, seg_count, expert_offset,
                              row_token, row_weight, pair_row, workspace, workspace_bytes, nullptr, stream);
}

int moe_capacity_drop(const moe_desc_t* desc, const float* scores, const int32_t* topk_idx, int32_t* expert_count,
                      int32_t* seg_count, int32_t* expert_offset, int32_t* row_token, float* row_weight,
                      int32_t* pair_row, void* workspace, size_t workspace_bytes, void* stream) {
    return moe_capacity_drop_ranked(desc, scores, topk_idx, nullptr, 0u, expert_count, seg_count, expert_offset,
                                    row_token, row_weight, pair_row, workspace, workspace_bytes, stream);
}

int moe_dispatch(const moe_desc_t* desc, const void* x, const int32_t* expert_offset, const int32_t* row_token,
                 void* xp, void* stream) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    const Sizes s = derive(*desc);
    if (s.max_rows == 0) return MOE_OK;  // no row can survive
    if (!x || !expert_offset || !row_token || !xp) return MOE_ERR_INVALID_ARG;
    if (misaligned16(x) || misaligned16(xp)) return MOE_ERR_INVALID_ARG;
    if (launch_dispatch(*desc, s, x, expert_offset, row_token, xp, (hipStream_t)stream) != hipSuccess)
        return MOE_ERR_HIP;
    return MOE_OK;
}

static int grouped_ffn_impl(const moe_desc_t* desc, const void* a, const int32_t* row_token,
                            const int32_t* expert_offset, const void* w_gate, const void* w_up, const void* w_down,
                            void* yp, void* workspace, size_t workspace_bytes, bool schedule_ready, void* stream) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    if (!a || !expert_offset || !w_gate || !w_up || !w_down || !yp || !workspace) return MOE_ERR_INVALID_ARG;
    if (misaligned16(a) || misaligned16(w_gate) || misaligned16(w_up) || misaligned16(w_down) || misaligned16(yp))
        return MOE_ERR_INVALID_ARG;
    const int sh = ffn_shape_supported(*desc, row_token != nullptr);
    if (sh != MOE_OK) return sh;
    const Sizes s = derive(*desc);
    const FfnWorkspace ws = ffn_workspace(*desc, s, workspace);
    if (workspace_bytes < ws.bytes) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
    if (s.max_rows == 0) return MOE_OK;
    if (launch_grouped_ffn(*desc, s, ws, a, row_token, expert_offset, w_gate, w_up, w_down, yp, schedule_ready,
                           (hipStream_t)stream) !=
        hipSuccess)
        return MOE_ERR_HIP;
    return MOE_OK;
}

int moe_grouped_ffn(const moe_desc_t* desc, const void* xp, const int32_t* expert_offset, const void* w_gate,
                    const void* w_up, const void* w_down, void* yp, void* workspace, size_t workspace_bytes,
                    void* stream) {
    return grouped_ffn_impl(desc, xp, nullptr, expert_offset, w_gate, w_up, w_down, yp, workspace, workspace_bytes,
                            false, stream);
}

int moe_dispatch_ffn(const moe_desc_t* desc, const void* x, const int32_t* expert_offset, const int32_t* row_token,
                     const void* w_gate, const void* w_up, const void* w_down, void* yp, void* workspace,
                     size_t workspace_bytes, void* stream) {
    if (!row_token) return MOE_ERR_INVALID_ARG;
    return grouped_ffn_impl(desc, x, row_token, expert_offset, w_gate, w_up, w_down, yp, workspace, workspace_bytes,
                            false, stream);
}

int moe_combine(const moe_desc_t* desc, const void* yp, const float* row_weight, const int32_t* pair_row, void* y,
                void* stream) {
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    if (desc->n_tokens == 0) return MOE_OK;
    if (!yp || !row_weight || !pair_row || !y) return MOE_ERR_INVALID_ARG;
    if (misaligned16(yp) || misaligned16(y)) return MOE_ERR_INVALID_ARG;
    const Sizes s = derive(*desc);
    if (launch_combine(*desc, s, yp, row_weight, pair_row, y, (hipStream_t)stream) != hipSuccess) return MOE_ERR_HIP;
    return MOE_OK;
}

int moe_layer_forward(const moe_desc_t* desc, const void* x, const float* w_router, const float* bias,
                      const void* w_gate, const void* w_up, const void* w_down, const uint8_t* token_class,
                      uint32_t seed, float* logits, float* scores, int32_t* topk_idx, float* topk_score,
                      int32_t* expert_count, int32_t* seg_count, int32_t* expert_offset, int32_t* row_token,
                      float* row_weight, int32_t* pair_row, void* yp, void* y, void* workspace,
                      size_t workspace_bytes, void* stream) {
    // every check of the four calls first, so that a refusal leaves nothing enqueued
    const int v = validate(desc);
    if (v != MOE_OK) return v;
    const Sizes s = derive(*desc);
    if (s.max_rows >= (int64_t)1 << 31) return MOE_ERR_UNSUPPORTED;
    if (!expert_count || !seg_count || !expert_offset || !workspace) return MOE_ERR_INVALID_ARG;
    if (((uintptr_t)workspace & 255) != 0) return MOE_ERR_INVALID_ARG;
    size_t need = drop_workspace(*desc, s, nullptr).bytes;
    const size_t need_route = route_workspace(*desc, nullptr).bytes;
    if (need_route > need) need = need_route;
    if (desc->n_tokens > 0) {
        if (!x || !w_router || !logits || !scores || !topk_idx || !topk_score || !pair_row || !yp || !y || !row_weight)
            return MOE_ERR_INVALID_ARG;
        if (misaligned16(x) || misaligned16(w_router) || misaligned16(yp) || misaligned16(y)) return MOE_ERR_INVALID_ARG;
    }
    if (s.max_rows > 0) {
        if (!row_token || !row_weight || !w_gate || !w_up || !w_down || !yp) return MOE_ERR_INVALID_ARG;
        if (misaligned16(w_gate) || misaligned16(w_up) || misaligned16(w_down) || misaligned16(yp))
            return MOE_ERR_INVALID_ARG;
        const int sh = ffn_shape_supported(*desc, true);
        if (sh != MOE_OK) return sh;
        const size_t need_ffn = ffn_workspace(*desc, s, nullptr).bytes;
        if (need_ffn > need) need = need_ffn;
    }
    if (workspace_bytes < need) return MOE_ERR_WORKSPACE_TOO_SMALL;
    int st = moe_route_topk(desc, x, w_router, bias, 0, logits, scores, topk_idx, topk_score, workspace,
                            workspace_bytes, stream);
    if (st != MOE_OK) return st;
    // The tile schedule of the expert GEMMs lives in the workspace behind the hidden activations.  Where that
    // place lies beyond what the drop itself uses of the workspace, the drop builds the schedule in the launch
    // that finishes the plan and the GEMMs start without a schedule kernel of their own.
    FfnScheduleArgs schedule;
    bool fold = false;
    if (s.max_rows > 0) {
        const FfnWorkspace fw = ffn_workspace(*desc, s, workspace);
        fold = (size_t)((const char*)fw.big.expert - (const char*)workspace) >= drop_workspace(*desc, s, nullptr).bytes;
        if (fold) schedule = ffn_schedule_args(*desc, fw, compute_units());
    }
    st = capacity_drop_impl(desc, scores, topk_idx, token_class, seed, expert_count, seg_count, expert_offset, row_token,
                            row_weight, pair_row, workspace, workspace_bytes, fold ? &schedule : nullptr, stream);
    if (st != MOE_OK) return st;
    if (s.max_rows > 0) {
        st = grouped_ffn_impl(desc, x, row_token, expert_offset, w_gate, w_up, w_down, yp, workspace, workspace_bytes,
                              fold, stream);
        if (st != MOE_OK) return st;
    }
    return moe_combine(desc, yp, row_weight, pair_row, y, stream);
}

}  // extern "C"
