// Fused fit -> select: the per-gap policy arg-max straight from the atom
// tables, without a (gap, job) matrix in between (Sec. 3.5: a subjob only
// comes into being at its grant, so all a gap needs from the jobs' replies is
// the best one).
//
// The stepping is that of the pair-evaluation kernel: lanes run along jobs,
// waves step through sorted gap positions of one capacity class, each lane
// advances a merge pointer through its job's atoms (staged in an LDS window
// that is topped up once per period).  Instead of storing the cut, a lane that
// passes an atom recomputes its key F * weight from the atom's (duration,
// peak).  Along the sorted positions of a class a job's key never decreases,
// so the wave's arg-max is a running one: only a key that changed and reaches
// the wave's best can move it.  After every period the waves of a block
// combine their bests per position and the block leaves one partial per (job
// tile, gap); k_fused_reduce finishes the arg-max and turns the winning atom
// into its boundary.
#pragma once

#include "k_fit.h"
#include "k_grant.h"

namespace sja {

constexpr int kFusedBlock = kSelBlock;     // the partials are laid out per tile of kSelBlock jobs
constexpr int kFusedWindow = 8;
constexpr int kFusedPeriod = 32;

__device__ __forceinline__ bool fused_better(unsigned long long hi_a, unsigned long long lo_a, int j_a,
                                             unsigned long long hi_b, unsigned long long lo_b, int j_b)
{
    if (hi_a != hi_b) return hi_a > hi_b;
    if (lo_a != lo_b) return lo_a > lo_b;
    return j_a < j_b;
}

__device__ __forceinline__ unsigned long long fused_readlane_u64(unsigned long long v, int l)
{
    const unsigned int lo = __builtin_amdgcn_readlane(int(uint32_t(v)), l);
    const unsigned int hi = __builtin_amdgcn_readlane(int(uint32_t(v >> 32)), l);
    return (static_cast<unsigned long long>(hi) << 32) | lo;
}

// Eight waves per SIMD (64 registers, a few spilled) beat the 94 registers the
// compiler takes by itself: the stepping loop is bound by latency (1.5 against 2.1 ms).
// AREA: the key's F is the atom's area under the envelope (a second window of
// 64-bit values beside the (duration, peak) one) instead of duration x peak.
template <int BLOCK, int CAP, int PERIOD, bool MIXED, bool AREA>
__global__ __launch_bounds__(BLOCK) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_fit_select(
    int n_jobs, int n_gaps, int chunk_bound, PolicyDev pol, const int64_t *__restrict__ seg_off,
    const int2 *__restrict__ atom_dp, const long long *__restrict__ atom_area,
    const int32_t *__restrict__ n_atoms,
    const int32_t *__restrict__ plan, const int32_t *__restrict__ chunk_begin,
    const int32_t *__restrict__ chunk_end, const int32_t *__restrict__ chunk_class,
    const int32_t *__restrict__ chunk_sub, const int32_t *__restrict__ start_tab,
    const int32_t *__restrict__ ncap_tab, const int32_t *__restrict__ gap_w,
    const int32_t *__restrict__ gap_c, const int32_t *__restrict__ gap_order,
    const int32_t *__restrict__ gap_run_end, const int32_t *__restrict__ wait,
    const uint8_t *__restrict__ sla_class,
    const int32_t *__restrict__ job_held, const uint8_t *__restrict__ gap_active,
    SelPartial *__restrict__ part)
{
    static_assert((CAP & (CAP - 1)) == 0 && BLOCK % kWave == 0 && PERIOD <= 64, "tile shape");
    constexpr int WAVES = BLOCK / kWave;
    __shared__ int2 win[CAP][BLOCK];
    __shared__ long long win_area[AREA ? CAP : 1][AREA ? BLOCK : 1];
    // per wave and period: the steps at which its running best changed, with the new best
    __shared__ unsigned long long e_hi[WAVES][PERIOD + 1];
    __shared__ unsigned long long e_lo[WAVES][PERIOD + 1];
    __shared__ int e_lane[WAVES][PERIOD + 1];
    __shared__ int e_atoms[WAVES][PERIOD + 1];
    __shared__ int e_step[WAVES][PERIOD + 1];
    __shared__ int e_count[WAVES];

    const int xcd = blockIdx.x & 7;
    const int k = blockIdx.x >> 3;
    const int job_tile = (k / chunk_bound) * 8 + xcd;
    const int chunk = k % chunk_bound;
    if (job_tile * BLOCK >= n_jobs || chunk >= plan[kPlanChunks]) return;
    const bool tabled = plan[kPlanTabled] != 0;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int j_raw = job_tile * BLOCK + tid;
    const bool live = j_raw < n_jobs;
    const int j = live ? j_raw : n_jobs - 1;
    const bool usable = live && !(job_held && job_held[j] >= 0);
    const int64_t base = seg_off[j];
    const int n = usable ? n_atoms[j] : 0;
    const int2 *dp = atom_dp + base;
    const long long *da = atom_area + base;        // read with AREA only
    unsigned long long mult = 1, tier = 0;
    job_policy(pol, wait, sla_class, j, mult, tier);
    const int s_begin = chunk_begin[chunk], s_end = chunk_end[chunk];

    int n_cap = 0;   // atoms the current capacity class can reach
    int a = 0;       // atoms whose running duration fits the current window
    int hi = 0;      // atoms [a, hi) are staged in the LDS window
    int nd = 0, np = 0;      // atom a     (meaningful while a < hi)
    int nd2 = 0, np2 = 0;    // atom a + 1 (meaningful while a + 1 < hi)
    unsigned long long key_hi = 0, key_lo = 0;   // key of atom a - 1, 0 while a == 0
    int c_cur = 0;
    unsigned long long dry_mask = 0;
    // the wave's running best, the same values in every lane
    unsigned long long best_hi = 0, best_lo = 0;
    int best_lane = kWave, best_atoms = 0;
    int q_now = 0;       // step of the current period (for the change list)
    int n_events = 0;    // entries of this wave's change list (the same in every lane)
    int q_noted = -1;    // step of the list's last entry
    auto uniform64 = [](unsigned long long v) {
        const unsigned int lo = __builtin_amdgcn_readfirstlane(int(uint32_t(v)));
        const unsigned int hi = __builtin_amdgcn_readfirstlane(int(uint32_t(v >> 32)));
        return (static_cast<unsigned long long>(hi) << 32) | lo;
    };
    auto note = [&]() {
        // at most one entry per step: a second change in the same step overwrites the first
        if (n_events > 0 && q_noted == q_now) --n_events;
        q_noted = q_now;
        if (lane == 0) {
            e_step[wave][n_events] = q_now;
            e_hi[wave][n_events] = best_hi;
            e_lo[wave][n_events] = best_lo;
            e_lane[wave][n_events] = best_lane;
            e_atoms[wave][n_events] = best_atoms;
        }
        ++n_events;
    };

    auto key_from = [&](unsigned long long F) {
        key_hi = ((tier << 62) | times_mult(F, mult)) + 1ull;
        key_lo = MIXED ? F : 0ull;
    };
    // key of the atom just passed: a - 1, whose window slot is still intact (a top-up writes at most
    // up to atom a + CAP - 1)
    auto key_of = [&](int d, int p) {
        if (AREA) key_from((unsigned long long)win_area[(a - 1) & (CAP - 1)][tid]);
        else key_from(rect_of(d, p));
    };
    // a key changed in the lanes of `ch` (those that can matter): move the running best
    auto challenge = [&](bool in) {
        unsigned long long ch = __ballot(in);
        if (!ch) return;
        if (__popcll(ch) > 4) {
            unsigned long long bh = in ? key_hi : 0ull, bl = in ? key_lo : 0ull;
            int bj = in ? lane : kWave;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const unsigned long long oh = (unsigned long long)__shfl_xor((long long)bh, d, kWave);
                const unsigned long long ol = (unsigned long long)__shfl_xor((long long)bl, d, kWave);
                const int oj = __shfl_xor(bj, d, kWave);
                if (fused_better(oh, ol, oj, bh, bl, bj)) { bh = oh; bl = ol; bj = oj; }
            }
            // the best of the changed keys replaces the running best if it beats it, or if it is the
            // best lane's own new key; a best lane that changed without being this maximum is beaten by it
            const bool own = (ch >> (best_lane & (kWave - 1))) & 1ull && best_lane < kWave;
            if (own || fused_better(bh, bl, bj, best_hi, best_lo, best_lane)) {
                best_hi = uniform64(bh); best_lo = uniform64(bl); best_lane = __builtin_amdgcn_readfirstlane(bj);
                best_atoms = __builtin_amdgcn_readlane(a, best_lane & (kWave - 1));
                note();
            }
        } else {
            bool moved = false;
            while (ch) {
                const int l = __ffsll((long long)ch) - 1;
                ch &= ch - 1;
                const unsigned long long kh = fused_readlane_u64(key_hi, l);
                const unsigned long long kl = MIXED ? fused_readlane_u64(key_lo, l) : 0ull;
                if (l == best_lane || fused_better(kh, kl, l, best_hi, best_lo, best_lane)) {
                    best_hi = kh; best_lo = kl; best_lane = l;
                    best_atoms = __builtin_amdgcn_readlane(a, l);
                    moved = true;
                }
            }
            if (moved) note();
        }
    };
    auto init = [&](int s) {
        c_cur = gap_c[s];
        if (!usable) {
            n_cap = 0; a = 0;
        } else if (tabled) {
            a = start_tab[int64_t(chunk) * n_jobs + j];
            n_cap = ncap_tab[int64_t(chunk_class[chunk]) * n_jobs + j];
        } else {
            n_cap = upper_bound_peak(dp, n, c_cur);
            a = upper_bound_dur(dp, n_cap, gap_w[s]);
        }
        key_hi = 0; key_lo = 0;
        if (a > 0) {
            if (AREA) {
                key_from((unsigned long long)da[a - 1]);
            } else {
                const int2 v = dp[a - 1];
                key_from(rect_of(v.x, v.y));
            }
        }
        hi = a;
        best_hi = 0; best_lo = 0; best_lane = kWave; best_atoms = 0;
        note();
        challenge(a > 0);
    };
    auto reload = [&]() {
        const int2 x = win[a & (CAP - 1)][tid]; nd = x.x; np = x.y;
        const int2 y = win[(a + 1) & (CAP - 1)][tid]; nd2 = y.x; np2 = y.y;
    };
    auto topup = [&]() {
        const int want = min(a + CAP, n_cap);
        int2 v[CAP];
#pragma unroll
        for (int t = 0; t < CAP; ++t)
            if (hi + t < want) v[t] = dp[hi + t];
#pragma unroll
        for (int t = 0; t < CAP; ++t)
            if (hi + t < want) win[(hi + t) & (CAP - 1)][tid] = v[t];
        if (AREA) {
            for (int idx = hi; idx < want; ++idx) win_area[idx & (CAP - 1)][tid] = da[idx];
        }
        hi = max(hi, want);
        reload();
    };
    // One step: move every lane past the atoms that window w has reached and keep the
    // running best (q = step within the period).
    auto step = [&](int w, int q) {
        bool adv = a < hi && nd <= w;
        if (__any(adv)) {
            bool changed = false;
            int ld = 0, lp = 0;                  // (duration, peak) of the last atom passed
            do {
                if (adv) { ld = nd; lp = np; ++a; nd = nd2; np = np2; changed = true; }
                {
                    const int2 y = win[(a + 1) & (CAP - 1)][tid];
                    nd2 = y.x; np2 = y.y;
                }
                if (__ballot(a == hi) & dry_mask) {
                    // a window ran dry inside a period: refill at once (rare)
                    if (a == hi && hi < n_cap) {
                        // with AREA one slot stays back: atom a - 1 shares its slot with atom a + CAP - 1
                        const int want = min(a + CAP - (AREA ? 1 : 0), n_cap);
                        for (int idx = hi; idx < want; ++idx) {
                            win[idx & (CAP - 1)][tid] = dp[idx];
                            if (AREA) win_area[idx & (CAP - 1)][tid] = da[idx];
                        }
                        hi = want;
                        reload();
                    }
                    dry_mask = __ballot(hi < n_cap);
                }
                adv = a < hi && nd <= w;
            } while (__any(adv));
            q_now = q;
            if (changed) key_of(ld, lp);         // once per step, for the last atom passed
            challenge(changed && key_hi >= best_hi);
        }
    };

    for (int s0 = s_begin; s0 < s_end; s0 += PERIOD) {
        const int s1 = min(s_end, s0 + PERIOD);
        n_events = 0;
        q_now = 0;
        q_noted = -1;
        if (s0 == s_begin || gap_c[s0] != c_cur) init(s0); else note();     // the list starts with the best so far
        topup();
        dry_mask = __ballot(hi < n_cap);
        if (s1 - s0 == PERIOD && gap_run_end[s0] >= s1) {
#pragma unroll
            for (int u4 = 0; u4 < PERIOD; u4 += 4) {
                const int wv[4] = {gap_w[s0 + u4], gap_w[s0 + u4 + 1], gap_w[s0 + u4 + 2], gap_w[s0 + u4 + 3]};
#pragma unroll
                for (int u = 0; u < 4; ++u) step(wv[u], u4 + u);
            }
        } else {
            for (int s = s0; s < s1; ++s) {
                q_now = s - s0;
                if (gap_c[s] != c_cur) { init(s); topup(); dry_mask = __ballot(hi < n_cap); }
                step(gap_w[s], s - s0);
            }
        }
        if (lane == 0) e_count[wave] = n_events;
        __syncthreads();
        // one partial per position of this period: the best of the block's waves at that step
        for (int q = tid; q < s1 - s0; q += BLOCK) {
            const int g = gap_order[s0 + q];
            const bool on = !gap_active || gap_active[g];
            unsigned long long bh = 0, bl = 0;
            int bj = INT32_MAX, ba = 0;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) {
                const int ne = e_count[w];
                int e = 0;                                   // the last change at or before step q
                for (int i = 1; i < ne && e_step[w][i] <= q; ++i) e = i;
                const unsigned long long oh = on ? e_hi[w][e] : 0ull, ol = e_lo[w][e];
                const int oj = oh ? job_tile * BLOCK + w * kWave + e_lane[w][e] : INT32_MAX;
                if (fused_better(oh, ol, oj, bh, bl, bj)) { bh = oh; bl = ol; bj = oj; ba = e_atoms[w][e]; }
            }
            SelPartial out;
            out.hi = bh; out.lo = bl; out.job = bh ? bj : -1; out.cut = bh ? ba : -1; out.pad = 0;
            part[int64_t(job_tile) * n_gaps + g] = out;
        }
        __syncthreads();
    }
}

// Final arg-max over the job tiles; the winner's atom count becomes its boundary.
__global__ void k_fused_reduce(int n_gaps, int n_job_tiles, const SelPartial *__restrict__ part,
                               const int64_t *__restrict__ seg_off, const int2 *__restrict__ atom_db,
                               int32_t *__restrict__ cand_job, int32_t *__restrict__ cand_cut,
                               int64_t *__restrict__ cand_score)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_gaps) return;
    unsigned long long bh = 0, bl = 0;
    int bj = INT32_MAX, ba = -1;
    for (int t = 0; t < n_job_tiles; ++t) {
        const SelPartial p = part[int64_t(t) * n_gaps + g];
        const int pj = p.hi ? p.job : INT32_MAX;
        if (fused_better(p.hi, p.lo, pj, bh, bl, bj)) { bh = p.hi; bl = p.lo; bj = pj; ba = p.cut; }
    }
    cand_job[g] = bh ? bj : -1;
    cand_cut[g] = bh ? atom_db[seg_off[bj] + ba - 1].y : -1;
    cand_score[g] = bh ? int64_t((bh - 1ull) & ((1ull << 62) - 1ull)) : 0;
}

}  // namespace sja
