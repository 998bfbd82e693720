// Host-side bookkeeping shared by the entry points: context, workspace layout.
// Nothing here runs on the device.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../../include/sja.h"

namespace sja {

constexpr int kWave = 64;

// ---- tiling constants shared by host launch code and kernels -------------
constexpr int kFitBlock = 128;        // threads per fit block, one job per thread
constexpr int kFitMaxChunk = 512;     // most sorted gap positions one fit block walks
constexpr int kFitWindow = 16;        // atoms per job staged ahead in LDS (power of two)
constexpr int kFitPeriod = 32;        // steps between window top-ups (multiple of 4)
constexpr int kMaxClasses = 64;       // distinct capacities served by the table-driven path
constexpr int kSelBlock = 256;        // threads per select block, one job per thread
constexpr int kSelGapChunk = 64;      // sorted gap positions walked by one select block
constexpr int kGapTile = 4096;        // gaps sorted together in LDS when the gaps are ordered
constexpr int kListSplits = 40;       // most pieces one capacity class's small windows are split into

// One partial arg-max per (job tile, gap): 32 bytes.
struct SelPartial {
    unsigned long long hi;   // 0 = no candidate; else 1 + (tier << 62 | score)
    unsigned long long lo;   // secondary score (MIXED: F), else 0
    int32_t job;
    int32_t cut;
    int64_t pad;
};

// Gap plan header written by k_gap_plan (device memory, int32 each).
enum { kPlanClasses = 0, kPlanChunks = 1, kPlanTabled = 2, kPlanSubBlocks = 3, kPlanListBlocks = 4, kPlanMarks = 5, kPlanWords = 8 };

// Byte offsets of the private tables inside the caller's workspace.
struct Layout {
    size_t atom_dp, atom_db;               // [S+8] int2 each: (dur, peak) and (dur, boundary)
    size_t n_atoms;                        // [J] int32
    size_t first_dp;                       // [J] int2: a job's first atom (duration, peak), INT32_MAX twice if none
    size_t atom_area, pre_area;            // area score only: int64 area under the envelope per atom / per segment
    size_t gap_rank, gap_order;            // [G] int32
    size_t gap_tile_key, gap_tile_idx;     // [ceil(G / kGapTile) * kGapTile] uint64 / int32: gaps sorted tile by tile
    size_t gap_w, gap_c, gap_run_end;      // [G+16] int32, in sorted order
    size_t gap_cls;                        // [G+16] int32: capacity class of a sorted position
    size_t bits_table;                     // [kMaxClasses * ceil(J/32)] uint32: per class and job word, the jobs whose first atom fits the capacity
    size_t gap_row;                        // [G+16] int64: element offset of a gap's cut row
    size_t plan;                           // [kPlanWords] int32 header
    size_t class_begin, class_chunk0, class_sub0;   // [kMaxClasses+1] int32
    size_t class_marks;                    // [kMaxClasses+1] int32: first positions of the capacity runs, unordered
    size_t class_dmax;                     // [kMaxClasses] int32: largest first-atom duration among the jobs that fit the class
    size_t chunk_begin, chunk_end, chunk_class, chunk_sub;  // [chunk_bound] int32
    size_t sub_begin, sub_end, sub_class;  // [sub_bound] int32
    size_t start_tab;                      // [chunk_bound * J] int32: per chunk of the stepping kernels
    size_t sub_tab;                        // [sub_bound * J] int32: per sub-block, built by sja_resolve for its lists
    size_t ncap_tab;                       // [kMaxClasses * J] int32
    size_t sel_part;                       // [ceil(J/kSelBlock) * G] SelPartial
    size_t res_cand_job, res_cand_cut;     // [G] int32
    size_t res_cand_score;                 // [G] int64
    size_t res_active;                     // [G] uint8
    size_t res_claim;                      // [J] uint64
    size_t res_counters;                   // [16] int32
    // list-driven grant path
    size_t g_abase;                        // [J+2] int32
    size_t g_scan_tmp;                     // tile sums of the scans
    size_t g_key_hi, g_key_lo;             // [atom_cap] uint64
    size_t g_perm0, g_perm1, g_rank;       // [atom_cap] uint32
    size_t g_hist;                         // [256 * tiles] int32, tiles of the larger of the two sorts
    size_t g_ekey0, g_ekey1;               // [entry_cap] uint64: list entries (block : rank : lane range)
    size_t g_rec;                          // [entry_cap] uint4: the sorted lists as records
    size_t g_atom_ja, g_ranked;            // [atom_cap] int2: (job, atom) by atom id and by rank
    size_t lb_begin, lb_end, lb_sub;       // [list_bound] int32: grant-list blocks (pieces of sub-blocks)
    size_t lb_off;                         // [sub_bound+2] int32: first list block of a sub-block
    size_t g_list_off;                     // [list_bound+2] int32
    size_t g_held;                         // 2 x held_bitmap_words(J) uint32: jobs held before a round, two alternating copies
    size_t g_state;                        // [list_bound * 64] int4: pointer, candidate job, candidate atom, flag | gap << 2
    size_t g_cnt_lost, g_cnt_cand;         // [min(G,J)+4] int32
    int64_t atom_cap, entry_cap;
    size_t total;
};

inline size_t align_up(size_t x) { return (x + 255) & ~size_t(255); }

// Sorted gap positions per fit block: large enough to amortise a block's
// set-up, small enough that a small batch still spreads over the chip.
inline int fit_chunk_len(int64_t G, int64_t J)
{
    const int64_t tiles = (J + kFitBlock - 1) / kFitBlock;
    int gc = kFitMaxChunk;
    while (gc > 32 && tiles * ((G + gc - 1) / gc) < 2048) gc >>= 1;
    return gc;
}

inline int64_t fit_chunk_bound(int64_t G, int64_t J)
{
    const int gc = fit_chunk_len(G, J);
    return (G + gc - 1) / gc + kMaxClasses;
}

// Sub-blocks: runs of at most 64 sorted positions inside one capacity class;
// the start tables and the grant lists are kept per sub-block.
inline int fit_sub_len(int64_t G, int64_t J) { const int gc = fit_chunk_len(G, J); return gc < 64 ? gc : 64; }

inline int64_t fit_sub_bound(int64_t G, int64_t J)
{
    const int sb = fit_sub_len(G, J);
    return (G + sb - 1) / sb + kMaxClasses;
}

// Grant-list blocks: the sub-blocks, those that span a wide range of small
// windows cut into pieces (at most kListSplits per capacity class).
inline int64_t list_block_bound(int64_t G, int64_t J) { return fit_sub_bound(G, J) + int64_t(kMaxClasses) * kListSplits; }

// Words of one held-job bitmap: one bit per job, padded to whole 16-byte loads.
inline int held_bitmap_words(int64_t n_jobs) { return int(((n_jobs + 31) / 32 + 3) / 4 * 4); }

inline Layout make_layout(int64_t G, int64_t J, int64_t S)
{
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.atom_dp = take(size_t(S + 8) * 8);
    L.atom_db = take(size_t(S + 8) * 8);
    L.n_atoms = take(size_t(J) * 4);
    L.first_dp = take(size_t(J) * 8);
    L.atom_area = take(size_t(S + 8) * 8);
    L.pre_area = take(size_t(S + 8) * 8);
    L.gap_rank = take(size_t(G) * 4);
    L.gap_order = take(size_t(G) * 4);
    const size_t gap_tiles = size_t((G + kGapTile - 1) / kGapTile);
    L.gap_tile_key = take(gap_tiles * kGapTile * 8);
    L.gap_tile_idx = take(gap_tiles * kGapTile * 4);
    L.gap_w = take(size_t(G + 16) * 4);
    L.gap_c = take(size_t(G + 16) * 4);
    L.gap_run_end = take(size_t(G + 16) * 4);
    L.gap_cls = take(size_t(G + 16) * 4);
    L.bits_table = take(size_t(kMaxClasses) * size_t((J + 31) / 32) * 4);
    L.gap_row = take(size_t(G + 16) * 8);
    L.plan = take(kPlanWords * 4);
    L.class_begin = take((kMaxClasses + 1) * 4);
    L.class_chunk0 = take((kMaxClasses + 1) * 4);
    L.class_sub0 = take((kMaxClasses + 1) * 4);
    L.class_marks = take((kMaxClasses + 1) * 4);
    L.class_dmax = take(kMaxClasses * 4);
    const size_t cb = size_t(fit_chunk_bound(G, J));
    const size_t ub = size_t(fit_sub_bound(G, J));
    L.chunk_begin = take(cb * 4);
    L.chunk_end = take(cb * 4);
    L.chunk_class = take(cb * 4);
    L.chunk_sub = take(cb * 4);
    L.sub_begin = take(ub * 4);
    L.sub_end = take(ub * 4);
    L.sub_class = take(ub * 4);
    L.start_tab = take(cb * size_t(J) * 4);
    L.sub_tab = take(ub * size_t(J) * 4);
    L.ncap_tab = take(size_t(kMaxClasses) * size_t(J) * 4);
    size_t job_tiles = size_t((J + kSelBlock - 1) / kSelBlock);
    L.sel_part = take(job_tiles * size_t(G) * sizeof(SelPartial));
    L.res_cand_job = take(size_t(G) * 4);
    L.res_cand_cut = take(size_t(G) * 4);
    L.res_cand_score = take(size_t(G) * 8);
    L.res_active = take(size_t(G));
    L.res_claim = take(size_t(J) * 8);
    L.res_counters = take(64);
    L.atom_cap = S + 8;
    const size_t lb = size_t(list_block_bound(G, J));
    L.entry_cap = int64_t(ub + 128) * J + 2 * S + 8;
    const size_t ac = size_t(L.atom_cap), ec = size_t(L.entry_cap);
    const size_t hist_ints = 256 * ((ec + 4095) / 4096);      // ec >= ac: the atom sort fits too
    L.g_abase = take(size_t(J + 2) * 4);
    L.g_scan_tmp = take(((hist_ints + 2047) / 2048 + size_t(J) / 2048 + lb / 2048 + 16) * 4);
    L.g_key_hi = take(ac * 8);
    L.g_key_lo = take(ac * 8);
    L.g_perm0 = take(ac * 4);
    L.g_perm1 = take(ac * 4);
    L.g_rank = take(ac * 4);
    L.g_hist = take(hist_ints * 4);
    L.g_ekey0 = take(ec * 8);
    L.g_ekey1 = take(ec * 8);
    L.g_rec = take(ec * 16);
    L.g_atom_ja = take(ac * 8);
    L.g_ranked = take(ac * 8);
    L.lb_begin = take(lb * 4);
    L.lb_end = take(lb * 4);
    L.lb_sub = take(lb * 4);
    L.lb_off = take((ub + 2) * 4);
    L.g_list_off = take((lb + 2) * 4);
    L.g_state = take(lb * size_t(kWave) * 16);
    L.g_held = take(2 * size_t(held_bitmap_words(J)) * 4);
    const size_t rounds_cap = size_t(G < J ? G : J) + 4;
    L.g_cnt_lost = take(rounds_cap * 4);
    L.g_cnt_cand = take(rounds_cap * 4);
    L.total = off;
    return L;
}

}  // namespace sja

struct sja_ctx {
    int device;
    char *ws;
    size_t ws_bytes;
    char err[256];

    // state left by sja_prepare_profiles
    bool prepared;
    int32_t n_jobs;
    int64_t n_segments;
    const int64_t *seg_off;
    const int32_t *dur;
    const int32_t *mem;
    const uint8_t *safe;
    int32_t *pre_dur;
    int32_t *pre_peak;
    int32_t *prev_safe;

    // admission limits: as set by sja_set_limits, and as the last prepare applied them
    bool limits_on, limits_used;
    sja_limits limits, limits_applied;
    const int32_t *lim_power, *lim_deadline;
    const int32_t *used_power, *used_deadline;

    // how F is read (sja_set_score), and how the last prepare built the tables
    int score_mode, score_used;

    // hysteresis rule: as set by sja_set_hysteresis, and as the last prepare applied it
    int32_t hyst_n_caps, hyst_min_gain, hyst_cap[SJA_MAX_CAPS];
    int32_t hyst_used_n_caps, hyst_used_min_gain, hyst_used_cap[SJA_MAX_CAPS];

    // optional timing of the pair-evaluation kernel
    bool timing;
    bool timed;
    hipEvent_t ev_start, ev_stop;

    // how sja_resolve runs its rounds (sja_set_resolve_mode)
    int resolve_mode;

    // state left by sja_fit (planned and fitted) or sja_fit_select (planned only: no cut matrix)
    bool planned;
    bool fitted;
    int32_t n_gaps;
    const int32_t *cut;
};
