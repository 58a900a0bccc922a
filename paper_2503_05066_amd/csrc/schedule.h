// Tile schedule of the expert GEMMs: turns the per-expert row offsets of a dispatch plan into lists of row tiles
// and decides which work items are cut along K.  One wavefront builds it: the schedule kernel of
// moe_grouped_ffn, or the block of the capacity-drop kernels that knows every expert's row count when the
// whole layer is enqueued by one call (the plan and its schedule then leave the same launch).
#pragma once

#include "common.h"

namespace capmoe {

// Expert e with c rows gets floor(c / big) full tiles; a remainder above small_max rows becomes one
// more (partly filled) big tile, a smaller one is cut into ceil(remainder / small) short tiles, which
// run the same loop on 64-row blocks (few rows per weight byte: memory-bound work).
//
// A GEMM runs its big work items (row tiles x column blocks) in rounds of one item per compute unit, and
// every XCD (an eighth of the compute units with an L2 of its own) gets a contiguous eighth of them.  The
// items left over after an XCD's last full round would hold that XCD for a whole item time with most of
// its compute units idle, so each of them is cut along K into `slices` units that run side by side: a unit
// multiplies its share of the K slabs and writes its fp32 partial tile to the workspace, and the unit of an
// item that finishes last (an integer ticket per item) adds the partial tiles in slice order and writes the
// output tile: no floating-point atomics, the same bits run to run.  The cut depends on the GEMM's
// column-block count and K, so each of the two GEMMs gets its own header.
//
// A GEMM that is never cut walks either the two lists one after the other (big items first, short ones at the
// end) or the joint list, in which an expert's short tiles follow its big ones.  In a long launch of compute-bound
// big items the joint order hides the short items' weight streaming behind matrix work; in a launch of a few
// rounds, big items that start late because short ones went first are the longer end.  The schedule picks the
// joint order from kFfnJointMinRounds items per compute unit on.
struct SplitArgs {
    int32_t* hdr;      // [kFfnSplitHdr]: big items per XCD that are cut (taken from the end of the XCD's share) and
                       // units per item, then the same for the short items, then 1 if the GEMM walks the joint list,
                       // then how many items at the end of that list the XCDs share out by a counter (counter[0]),
                       // then how many big items at the end of an XCD's share run as row pieces
    int32_t* counter;  // [2 * kFfnSplitUnits] tickets (big, short), zeroed here before every launch
    int ncol_big;      // column blocks of the GEMM's big items; 0: never cut
    int ncol_small;    // column blocks of its short items
    int slabs;         // K slabs of the GEMM
};
struct TileListArgs {
    int32_t *b_expert, *b_row0, *b_rows, *b_count, *s_expert, *s_row0, *s_rows, *s_count;
    int b_max, s_max;
    // both kinds in one list, expert by expert (an expert's big tiles, then its short ones); a short tile's row
    // count carries kShortTileFlag.  u_max == 0: not written.
    int32_t *u_expert, *u_row0, *u_rows, *u_count;
    int u_max;
};
constexpr int kShortTileFlag = 1 << 16;  // above every tile height

struct ExpertTiles {
    int lo, rows, nb, ns;
};
// Tile heights are powers of two (big = 1 << big_sh, small = 1 << small_sh): a single wave runs this kernel,
// every dependent instruction counts, and a division by a run-time value is forty of them.
__host__ __device__ inline ExpertTiles expert_tiles(int lo, int hi, int big_sh, int small_sh, int small_max) {
    ExpertTiles t;
    t.lo = lo;
    t.rows = hi - lo;
    const int full = t.rows >> big_sh, rem = t.rows - (full << big_sh);
    const bool rem_small = rem > 0 && rem <= small_max;
    t.nb = full + (rem > 0 && !rem_small ? 1 : 0);
    t.ns = rem_small ? (rem + (1 << small_sh) - 1) >> small_sh : 0;
    return t;
}

// inclusive scan of two counters over the wave
__device__ inline void wave_scan2(int& a, int& b) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int oa = __shfl_up(a, off, kWave), ob = __shfl_up(b, off, kWave);
        if (lane >= off) {
            a += oa;
            b += ob;
        }
    }
}

// How an XCD's share of `items_per_xcd` items of one kind is cut: the last `cut` of them into `slices` units each.
// cus_per_xcd compute units run one item each per round; the units of the cut items may occupy unit_cus of them
// side by side; a unit keeps at least kFfnSplitMinSlabs slabs.
__host__ __device__ inline void split_rule(int items_per_xcd, int cus_per_xcd, int unit_cus, int slabs, int& cut,
                                           int& slices) {
    cut = 0;
    slices = 1;
    if (items_per_xcd <= 0 || cus_per_xcd <= 0 || slabs < kFfnSplitMinK) return;
    if (cus_per_xcd > kFfnSplitUnits / 8) cus_per_xcd = kFfnSplitUnits / 8;
    if (unit_cus > cus_per_xcd) unit_cus = cus_per_xcd;
    const int left = items_per_xcd % cus_per_xcd;
    if (left == 0) return;
    int s = unit_cus / left;
    if (s < 2 && cus_per_xcd / left >= 2) s = 2;  // halves still beat whole items at the end of a launch
    if (s > kFfnSplitMaxSlices) s = kFfnSplitMaxSlices;
    if (s > slabs / kFfnSplitMinSlabs) s = slabs / kFfnSplitMinSlabs;
    if (s < 2) return;
    cut = left;
    slices = s;
}

// The header of one GEMM (kFfnSplitHdr ints, see SplitArgs::hdr) from the number of big and short row tiles:
// every decision of the schedule that depends on the plan.  joint_list: the joint tile list is written (bf16);
// short_tiles: the short-tile configuration exists.  Host and device run the same code (the host copy answers
// moe_ffn_schedule_query).
__host__ __device__ inline void ffn_schedule_header(int nb, int ns, int ncol_big, int ncol_small, int slabs, int cus,
                                                    bool joint_list, bool short_tiles, int32_t* hdr) {
    const long long items[2] = {(long long)nb * ncol_big, (long long)ns * ncol_small};
    const int per_xcd = cus >> 3;
    int chunk[2] = {0, 0};
    for (int which = 0; which < 2; ++which)
        if (items[which] > 0 && items[which] < (1ll << 30)) chunk[which] = (int)((items[which] + 7) >> 3);
    // The units of the big items start first; when the XCD also has short items to run after them, those
    // units take only the big items' share of the tail's work (a short item counted as half a big one),
    // so that short items start at once on the other compute units and both kinds end together.
    const int left_big = per_xcd > 0 ? chunk[0] % per_xcd : 0;
    const int big_cus = chunk[1] > 0 ? per_xcd * 2 * left_big / (2 * left_big + chunk[1]) : per_xcd;
    for (int which = 0; which < 2; ++which) {
        int cut = 0, slices = 1;
        split_rule(chunk[which], per_xcd, which == 0 ? big_cus : per_xcd, slabs, cut, slices);
        hdr[2 * which] = cut;
        hdr[2 * which + 1] = slices;
    }
    const long long joint_items = (long long)(nb + ns) * ncol_big;
    hdr[4] = joint_list && ns > 0 && slabs < kFfnSplitMinK && joint_items >= (long long)kFfnJointMinRounds * cus;
    // the end of the joint order that the XCDs share out among themselves as they get free
    hdr[5] = hdr[4] ? kFfnJointPoolRounds * cus : 0;
    // Big items left over after the XCD's last full round, in a GEMM too short in K to be cut there: run
    // as row pieces (four short-tile blocks each) when those and the XCD's short items fit in one round
    // together, which then takes half an item's time instead of a whole one.
    const int left_over = per_xcd > 0 && chunk[0] > per_xcd ? chunk[0] % per_xcd : 0;
    hdr[6] = !hdr[4] && slabs < kFfnSplitMinK && short_tiles && left_over > 0 &&
                     left_over * kFfnRowPieces + chunk[1] <= per_xcd
                 ? left_over
                 : 0;
    hdr[7] = 0;
}

// Everything the schedule needs besides the row offsets (passed by value to a kernel).
struct FfnScheduleArgs {
    int enabled;  // 0: the kernel that carries these arguments builds no schedule
    int E, big_sh, small_sh, small_max, cus;
    TileListArgs L;
    SplitArgs first, second;
};

// Builds the schedule from expert_offset[0..E] (global memory or LDS).  Called by all 64 lanes of one wave.
__device__ inline void build_ffn_schedule(const int32_t* expert_offset, const FfnScheduleArgs& a) {
    const int E = a.E, big_sh = a.big_sh, small_sh = a.small_sh, small_max = a.small_max, cus = a.cus;
    const TileListArgs& L = a.L;
    const SplitArgs& first = a.first;
    const SplitArgs& second = a.second;
    const int lane = threadIdx.x & (kWave - 1);
    const int big = 1 << big_sh, small = 1 << small_sh;
    // Every lane's experts, fetched once, and one scan per 64 experts: the kernel is a chain of latencies
    // (a dependent global load costs a microsecond, a wave scan half of one), so nothing is done twice.
    constexpr int kChunks = kMaxExperts / kWave;
    int nt_b = 0, nt_s = 0;
    int lo[kChunks], hi[kChunks];
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
        const int e = c * kWave + lane;
        lo[c] = e < E ? expert_offset[e] : 0;
        hi[c] = e < E ? expert_offset[e + 1] : 0;
    }
    // tickets of both GEMMs start at zero
    for (int i = lane; i < 2 * kFfnSplitUnits; i += kWave) {
        if (first.counter) first.counter[i] = 0;
        if (second.counter) second.counter[i] = 0;
    }
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
        if (c * kWave >= E) continue;  // the same for every lane
        const int e = c * kWave + lane;
        const ExpertTiles x = expert_tiles(lo[c], hi[c], big_sh, small_sh, small_max);
        int ib = x.nb, is = x.ns;
        wave_scan2(ib, is);
        const int start_b = nt_b + ib - x.nb, start_s = nt_s + is - x.ns;
        nt_b += __shfl(ib, kWave - 1, kWave);
        nt_s += __shfl(is, kWave - 1, kWave);
        const int start_u = start_b + start_s;
        for (int i = 0; i < x.nb; ++i) {
            const int idx = start_b + i;
            const int left = x.rows - i * big;
            if (idx < L.b_max) {
                L.b_expert[idx] = e;
                L.b_row0[idx] = x.lo + i * big;
                L.b_rows[idx] = left < big ? left : big;
            }
            if (start_u + i < L.u_max) {
                L.u_expert[start_u + i] = e;
                L.u_row0[start_u + i] = x.lo + i * big;
                L.u_rows[start_u + i] = left < big ? left : big;
            }
        }
        const int full = x.rows >> big_sh, rem = x.rows - (full << big_sh);
        for (int i = 0; i < x.ns; ++i) {
            const int idx = start_s + i;
            if (idx < L.s_max) {
                L.s_expert[idx] = e;
                L.s_row0[idx] = x.lo + full * big + i * small;
                const int left = rem - i * small;
                L.s_rows[idx] = left < small ? left : small;
            }
            const int ui = start_u + x.nb + i;
            if (ui < L.u_max) {
                L.u_expert[ui] = e;
                L.u_row0[ui] = x.lo + full * big + i * small;
                const int left = rem - i * small;
                L.u_rows[ui] = (left < small ? left : small) + kShortTileFlag;
            }
        }
    }
    if (lane == 0) {
        const int nb = nt_b < L.b_max ? nt_b : L.b_max, ns = nt_s < L.s_max ? nt_s : L.s_max;
        *L.b_count = nb;
        *L.s_count = ns;
        *L.u_count = nb + ns < L.u_max ? nb + ns : L.u_max;
        for (const SplitArgs* sp : {&first, &second}) {
            if (!sp->hdr) continue;
            ffn_schedule_header(nb, ns, sp->ncol_big, sp->ncol_small, sp->slabs, cus, L.u_max > 0, L.s_max > 0, sp->hdr);
        }
    }
}

}  // namespace capmoe
