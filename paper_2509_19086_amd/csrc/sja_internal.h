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
constexpr int kFitBlock = 256;        // threads per fit block, one job per thread
constexpr int kFitGapChunk = 256;     // sorted gap positions walked by one fit block
constexpr int kSelBlock = 256;        // threads per select block, one job per thread
constexpr int kSelGapChunk = 128;     // sorted gap positions walked by one select block

// One partial arg-max per (job tile, gap): 32 bytes.
struct SelPartial {
    unsigned long long hi;   // 0 = no candidate; else 1 + (tier << 62 | score)
    unsigned long long lo;   // secondary score (MIXED: F), else 0
    int32_t job;
    int32_t cut;
    int64_t pad;
};

// Byte offsets of the private tables inside the caller's workspace.
struct Layout {
    size_t atom_dur, atom_peak, atom_bnd;  // [S] int32 each: per-job compacted safe cuts
    size_t n_atoms;                        // [J] int32
    size_t gap_rank, gap_order;            // [G] int32
    size_t gap_w, gap_c;                   // [G] int32, in sorted order
    size_t sel_part;                       // [ceil(J/kSelBlock) * G] SelPartial
    size_t res_cand_job, res_cand_cut;     // [G] int32
    size_t res_cand_score;                 // [G] int64
    size_t res_active;                     // [G] uint8
    size_t res_claim;                      // [J] uint64
    size_t res_counters;                   // [4] int32
    size_t total;
};

inline size_t align_up(size_t x) { return (x + 255) & ~size_t(255); }

inline Layout make_layout(int64_t G, int64_t J, int64_t S)
{
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.atom_dur = take(size_t(S) * 4);
    L.atom_peak = take(size_t(S) * 4);
    L.atom_bnd = take(size_t(S) * 4);
    L.n_atoms = take(size_t(J) * 4);
    L.gap_rank = take(size_t(G) * 4);
    L.gap_order = take(size_t(G) * 4);
    L.gap_w = take(size_t(G) * 4);
    L.gap_c = take(size_t(G) * 4);
    size_t job_tiles = size_t((J + kSelBlock - 1) / kSelBlock);
    L.sel_part = take(job_tiles * size_t(G) * sizeof(SelPartial));
    L.res_cand_job = take(size_t(G) * 4);
    L.res_cand_cut = take(size_t(G) * 4);
    L.res_cand_score = take(size_t(G) * 8);
    L.res_active = take(size_t(G));
    L.res_claim = take(size_t(J) * 8);
    L.res_counters = take(64);
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
    const int32_t *pre_dur;
    const int32_t *pre_peak;

    // optional timing of the pair-evaluation kernel
    bool timing;
    bool timed;
    hipEvent_t ev_start, ev_stop;

    // state left by sja_fit
    bool fitted;
    int32_t n_gaps;
    const int32_t *cut;
};
