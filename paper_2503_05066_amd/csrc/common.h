// Internal declarations shared by the capmoe translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "capmoe.h"

namespace capmoe {

constexpr int kMaxExperts = 256;  // expert ids fit a byte (slot tables), one LDS histogram row per expert
constexpr int kMaxTopK = 64;
constexpr int kWave = 64;

// Tile heights of the expert GEMMs; the tile schedule in the workspace is built for these.
constexpr int kFfnTileM = 256;      // bf16 MFMA kernels, compute-bound tiles
constexpr int kFfnTileSmall = 64;   // bf16 MFMA kernels, tail of an expert with at most 64 rows left
constexpr int kFfnSmallMax = 64;    // a remainder of up to this many rows is one small tile (larger: a partly filled big tile)
constexpr int kFfnTileMF32 = 16;    // fp32 fallback kernels (tiny layers)

inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

// Static sizes derived from a descriptor (host side).
struct Sizes {
    int n_blocks;      // capacity blocks B
    int seg_tokens;    // tokens per capacity segment
    int cap;           // capacity per segment (per expert, or per device for the device scopes)
    int span;          // experts that share one capacity: 1, or E/G for the device scopes
    int slots;         // S
    int list_k;        // k + overselect: width of topk_idx
    int64_t max_rows;  // P_max
    int group_experts; // m = E / G
    int group_tokens;  // N / G
    size_t elem;       // bytes per element of desc->dtype
};

int validate(const moe_desc_t* d);
Sizes derive(const moe_desc_t& d);

// Workspace layout of moe_capacity_drop.
struct DropWorkspace {
    uint32_t* key_t;    // [E,N]  candidate key (score bits + 1) or 0, expert-major
    uint8_t* slot_t;    // [E,N]  slot of the pair in the token's candidate list
    uint32_t* seg_tau;  // [B*E]  threshold key of the segment
    int32_t* seg_need;  // [B*E]  how many candidates equal to the threshold are kept
    size_t bytes;
};
DropWorkspace drop_workspace(const moe_desc_t& d, const Sizes& s, void* base);

// Workspace layout of moe_route_topk (bf16 activations: router GEMM on the matrix cores, split over K).
struct RouteWorkspace {
    bool use_mfma;    // false: fp32 activations or an unsupported width, plain fp32 kernel, no workspace
    int ksplit;       // K slices; > 1: partial sums go to `partial` and the softmax kernel adds them
    float* partial;   // [ksplit,N,E]
    size_t bytes;
};
RouteWorkspace route_workspace(const moe_desc_t& d, void* base);

// Workspace layout of moe_grouped_ffn.
// Big work items left over after an XCD's last full round are cut along K into units that run side by side.
constexpr int kFfnSplitUnits = 256;      // most units of cut items in one launch (32 per XCD), also most cut items
constexpr int kFfnSplitMaxSlices = 8;    // most units per item
constexpr int kFfnSplitMinSlabs = 16;    // fewest 64-wide K slabs per unit
constexpr int kFfnSplitMinK = 128;       // GEMMs with fewer K slabs are never cut: a unit costs a fixed ~30 us on top of
                                         // its slabs (partial tile out, ticket, the sum), an item of 64 slabs only 100 us
constexpr int kFfnSplitHdr = 8;          // ints per GEMM in the schedule's header
constexpr int kFfnJointMinRounds = 8;    // work items per compute unit from which an uncut GEMM walks the joint tile
                                         // list (measured: 16 and 20 rounds gain 2 %, 3 rounds lose 7 %, 5 neither)
constexpr int kFfnRowPieces = kFfnTileM / kFfnTileSmall;  // short-tile blocks that cover one big item
constexpr int kFfnJointPoolRounds = 1;   // rounds of work items at the end of the joint order that any XCD may take
struct TileList {
    int32_t* expert;  // [max_tiles]
    int32_t* row0;    // [max_tiles] first row of the tile
    int32_t* rows;    // [max_tiles] valid rows in the tile
    int32_t* count;   // [1]
    int max_tiles;    // capacity of the arrays
    int max_launch;   // most tiles a launch can find in the list, per column block
    int tile_m;
};
struct FfnWorkspace {
    void* hidden;    // [P_max, h] activations silu(gate)*up in desc->dtype
    TileList big;    // full-height row tiles, and remainders above small_max rows
    TileList small;  // short row tiles covering remainders of at most small_max rows (bf16 only)
    TileList all;    // both kinds in one list, expert by expert (bf16 only; tile_m unused)
    int small_max;
    int32_t* split_hdr;      // [2 GEMMs][kFfnSplitHdr]: big items per XCD that are cut along K and units per item,
                             // the same for the short items, whether the GEMM walks the joint list (bf16 only)
    int32_t* split_counter;  // [2 GEMMs][2][kFfnSplitUnits] one ticket per cut item (big, short); a GEMM that walks the
                             // joint list is never cut and counts the shared items of its end in its first ticket
    float* split_partial;    // [kFfnSplitUnits][256 x 256] fp32 partial tiles of big items, then
                             // [kFfnSplitUnits][64 x 256] of short ones (the GEMMs run one after the other)
    size_t bytes;
};
FfnWorkspace ffn_workspace(const moe_desc_t& d, const Sizes& s, void* base);

// The caller's profile table (moe_profile_attach), per host thread; ProfileScope records the table's events
// around one launch and counts the launch.  The library keeps only this pointer, never the table.
extern thread_local moe_profile_t* t_profile;
struct ProfileScope {
    int id;
    hipStream_t st;
    ProfileScope(int id_, hipStream_t st_) : id(id_), st(st_) {
        if (t_profile) {
            if (t_profile->start[id]) (void)hipEventRecord((hipEvent_t)t_profile->start[id], st);
            t_profile->launches[id] += 1;
        }
    }
    ~ProfileScope() {
        if (t_profile && t_profile->stop[id]) (void)hipEventRecord((hipEvent_t)t_profile->stop[id], st);
    }
};

// What the library remembers per device (kernel attributes already set, the compute-unit count): one bit or
// one slot per device ordinal, written with atomics, so that any thread may call on any device.
constexpr int kMaxDevices = 64;
inline int current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
    return dev;
}
// Runs `configure` on the first call for the current device (twice at worst, when two threads race: setting a
// kernel attribute again is harmless); `seen` is one word per kernel, one bit per device.
template <class F>
inline void once_per_device(std::atomic<uint64_t>& seen, F&& configure) {
    const uint64_t bit = 1ull << current_device();
    if (!(seen.load(std::memory_order_acquire) & bit)) {
        configure();
        seen.fetch_or(bit, std::memory_order_release);
    }
}
int compute_units();  // of the current device

struct FfnScheduleArgs;  // schedule.h

// Launchers (each returns a hipError_t from hipGetLastError after its launches).
hipError_t launch_router_logits(const moe_desc_t& d, const void* x, const float* w, const float* bias, float* logits,
                                hipStream_t st);
hipError_t launch_router_mfma(const moe_desc_t& d, const RouteWorkspace& ws, const void* x, const float* w,
                              const float* bias, float* logits, hipStream_t st);
// partial != nullptr: logits[t,e] = bias[e] + sum over the ksplit slices of partial, written before use
hipError_t launch_softmax_topk(const moe_desc_t& d, float* logits, const float* partial, int ksplit, const float* bias,
                               float* scores, int32_t* topk_idx, float* topk_score, hipStream_t st);
hipError_t launch_capacity_drop(const moe_desc_t& d, const Sizes& s, const DropWorkspace& ws, const float* scores,
                                const int32_t* topk_idx, const uint8_t* token_class, uint32_t seed,
                                int32_t* expert_count, int32_t* seg_count,
                                int32_t* expert_offset, int32_t* row_token, float* row_weight, int32_t* pair_row,
                                const FfnScheduleArgs* schedule, hipStream_t st);
hipError_t launch_dispatch(const moe_desc_t& d, const Sizes& s, const void* x, const int32_t* expert_offset,
                           const int32_t* row_token, void* xp, hipStream_t st);
hipError_t launch_combine(const moe_desc_t& d, const Sizes& s, const void* yp, const float* row_weight,
                          const int32_t* pair_row, void* y, hipStream_t st);
hipError_t launch_grouped_ffn(const moe_desc_t& d, const Sizes& s, const FfnWorkspace& ws, const void* xp,
                              const int32_t* row_token, const int32_t* expert_offset, const void* w_gate,
                              const void* w_up, const void* w_down, void* yp, bool schedule_ready, hipStream_t st);
// schedule != nullptr (launch_capacity_drop): the drop also builds the tile schedule of the expert GEMMs;
// schedule_ready (launch_grouped_ffn): it has been built that way, no schedule kernel is launched
FfnScheduleArgs ffn_schedule_args(const moe_desc_t& d, const FfnWorkspace& ws, int cus);
void ffn_schedule_on_host(const moe_desc_t& d, const FfnWorkspace& ws, const int32_t* expert_count, int cus,
                          int32_t* tiles, int32_t* header);

}  // namespace capmoe
