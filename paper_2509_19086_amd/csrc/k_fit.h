// K2: fit for every (gap, job) pair (Sec. 3.8 admissibility in the envelope
// form of Sec. 3.9; the longest safe fragment is preferred), plus the small
// kernels that order the gaps and plan the launch.
//
// Over a job's atoms (its safe cuts after the progress point) both the running
// duration D and the running peak P are non-decreasing, so for a gap (W, C)
//     cut = boundary of atom  min(#{D <= W}, #{P <= C}) - 1      (or -1).
// Gaps are sorted by (C, W).  Inside a run of equal C the second count is a
// per-job constant and the first only grows with the sorted position, so a
// lane that owns one job walks a merge pointer through that job's atoms while
// the wave steps through gap positions and stores one coalesced 256-byte piece
// of a cut row per step.  The kernel is bound by those row stores; everything
// else is arranged so that the stepping loop issues no global load:
//   - the atoms a lane may cross next sit in a small circular LDS window that
//     is topped up from global memory once per period of steps;
//   - where a chunk of gap positions starts inside a job's atom list comes from
//     a table built by k_fit_starts (one sequential walk per job and capacity
//     class) instead of a per-chunk binary search;
//   - gap windows and row offsets arrive through wide scalar loads.
#pragma once

#include "sja_internal.h"

namespace sja {

// --------------------------------------------------------------------------
// Gap ordering: rank sort by (C, W, index); exact and deterministic.
// --------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long gap_key(int w, int c)
{
    return (static_cast<unsigned long long>(static_cast<uint32_t>(c) ^ 0x80000000u) << 32) |
           (static_cast<uint32_t>(w) ^ 0x80000000u);
}

__global__ void k_fill_i32(int32_t *p, int64_t n, int32_t v)
{
    int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

constexpr int kRankSpan = 2048;  // gaps compared against per block in k_gap_rank

__global__ __launch_bounds__(256) void k_gap_rank(int n_gaps, const int32_t *__restrict__ W,
                                                  const int32_t *__restrict__ C,
                                                  int32_t *__restrict__ rank)
{
    __shared__ unsigned long long tile[256];
    const int g = blockIdx.x * 256 + threadIdx.x;
    const unsigned long long mine = g < n_gaps ? gap_key(W[g], C[g]) : 0ull;
    const int h_begin = blockIdx.y * kRankSpan;
    const int h_end = min(n_gaps, h_begin + kRankSpan);
    int r = 0;
    for (int h0 = h_begin; h0 < h_end; h0 += 256) {
        const int h = h0 + threadIdx.x;
        __syncthreads();
        tile[threadIdx.x] = h < h_end ? gap_key(W[h], C[h]) : ~0ull;
        __syncthreads();
        const int n = min(256, h_end - h0);
        for (int t = 0; t < n; ++t) {
            const unsigned long long other = tile[t];
            r += (other < mine) || (other == mine && (h0 + t) < g);
        }
    }
    if (g < n_gaps && r) atomicAdd(&rank[g], r);
}

// Sorted copies of the gaps plus, per sorted position, the element offset of
// the gap's cut row.
__global__ void k_gap_scatter(int n_gaps, int n_jobs, const int32_t *__restrict__ W,
                              const int32_t *__restrict__ C, const int32_t *__restrict__ rank,
                              int32_t *__restrict__ order, int32_t *__restrict__ ws,
                              int32_t *__restrict__ cs, int64_t *__restrict__ row)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_gaps) return;
    const int r = rank[g];
    order[r] = g;
    ws[r] = W[g];
    cs[r] = C[g];
    row[r] = int64_t(g) * n_jobs;
}

// run_end[s] = first sorted position after s whose capacity differs.
__global__ void k_gap_run_end(int n_gaps, const int32_t *__restrict__ cs, int32_t *__restrict__ run_end)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_gaps) return;
    const int c = cs[s];
    int lo = s + 1, hi = n_gaps;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (cs[mid] <= c) lo = mid + 1; else hi = mid;
    }
    run_end[s] = lo;
}

// One block.  Finds the capacity classes (runs of equal C) and cuts the sorted
// positions into chunks of at most gc.  With at most kMaxClasses classes the
// chunks never straddle a class and the table-driven path is used; otherwise
// chunks are plain slices and the fit kernel searches for itself.
__global__ __launch_bounds__(1024) void k_gap_plan(int n_gaps, int gc, int sb, int chunk_bound,
                                                   int sub_bound, const int32_t *__restrict__ cs,
                                                   int32_t *plan, int32_t *class_begin,
                                                   int32_t *class_chunk0, int32_t *class_sub0,
                                                   int32_t *chunk_begin, int32_t *chunk_end,
                                                   int32_t *chunk_class, int32_t *chunk_sub,
                                                   int32_t *sub_begin, int32_t *sub_end,
                                                   int32_t *sub_class, int32_t *gap_cls)
{
    __shared__ int s_cnt[1024];
    __shared__ int s_classes, s_chunks, s_tabled, s_subs;
    const int t = threadIdx.x;
    const int span = (n_gaps + 1023) / 1024;
    const int lo = min(n_gaps, t * span), hi = min(n_gaps, lo + span);
    int cnt = 0;
    for (int s = lo; s < hi; ++s) cnt += (s == 0) || (cs[s] != cs[s - 1]);
    s_cnt[t] = cnt;
    __syncthreads();
    if (t == 0) {
        int acc = 0;
        for (int i = 0; i < 1024; ++i) { const int c = s_cnt[i]; s_cnt[i] = acc; acc += c; }
        s_classes = acc;
        s_tabled = acc <= kMaxClasses;
    }
    __syncthreads();
    const int n_classes = s_classes;
    const bool tabled = s_tabled != 0;
    {   // capacity class of every sorted position
        int k = s_cnt[t];
        for (int s = lo; s < hi; ++s) {
            k += (s == 0) || (cs[s] != cs[s - 1]);
            gap_cls[s] = k - 1;
        }
    }
    if (tabled) {
        int k = s_cnt[t];
        for (int s = lo; s < hi; ++s)
            if ((s == 0) || (cs[s] != cs[s - 1])) class_begin[k++] = s;
        if (t == 0) class_begin[n_classes] = n_gaps;
    }
    __syncthreads();
    if (t == 0) {
        int q = 0, u = 0;
        if (tabled) {
            for (int c = 0; c < n_classes; ++c) {
                class_chunk0[c] = q;
                class_sub0[c] = u;
                const int len = class_begin[c + 1] - class_begin[c];
                q += (len + gc - 1) / gc;
                u += (len + sb - 1) / sb;
            }
            class_chunk0[n_classes] = q;
            class_sub0[n_classes] = u;
        } else {
            q = (n_gaps + gc - 1) / gc;
        }
        s_chunks = min(q, chunk_bound);
        s_subs = min(u, sub_bound);
        plan[kPlanClasses] = n_classes;
        plan[kPlanChunks] = s_chunks;
        plan[kPlanTabled] = tabled ? 1 : 0;
        plan[kPlanSubBlocks] = s_subs;
    }
    __syncthreads();
    const int n_chunks = s_chunks;
    for (int q = t; q < n_chunks; q += 1024) {
        if (tabled) {
            int c = 0;
            while (c + 1 < n_classes && class_chunk0[c + 1] <= q) ++c;
            const int b = class_begin[c] + (q - class_chunk0[c]) * gc;
            chunk_begin[q] = b;
            chunk_end[q] = min(class_begin[c + 1], b + gc);
            chunk_class[q] = c;
            chunk_sub[q] = class_sub0[c] + (q - class_chunk0[c]) * (gc / sb);
        } else {
            chunk_begin[q] = q * gc;
            chunk_end[q] = min(n_gaps, q * gc + gc);
            chunk_class[q] = -1;
            chunk_sub[q] = 0;
        }
    }
    const int n_subs = s_subs;
    for (int u = t; u < n_subs; u += 1024) {
        int c = 0;
        while (c + 1 < n_classes && class_sub0[c + 1] <= u) ++c;
        const int b = class_begin[c] + (u - class_sub0[c]) * sb;
        sub_begin[u] = b;
        sub_end[u] = min(class_begin[c + 1], b + sb);
        sub_class[u] = c;
    }
}

// --------------------------------------------------------------------------
// Start tables (table-driven path).  Thread (job j, class c) walks the job's
// atoms once, in order, against the windows of the first gap of each of the
// class's sub-blocks (runs of `sb` sorted positions; a chunk is a whole number
// of them), ascending:
//   start[u][j] = #atoms usable by the first gap of sub-block u
//   ncap[c][j]  = #atoms any gap of class c can reach (peak <= C_c and
//                 duration <= the class's largest window)
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fit_starts(
    int n_jobs, int sb, const int32_t *__restrict__ plan, const int32_t *__restrict__ class_begin,
    const int32_t *__restrict__ class_sub0, const int32_t *__restrict__ gap_w,
    const int32_t *__restrict__ gap_c, const int64_t *__restrict__ seg_off,
    const int2 *__restrict__ atom_dp, const int32_t *__restrict__ n_atoms,
    int32_t *__restrict__ start_tab, int32_t *__restrict__ ncap_tab)
{
    const int c = blockIdx.y;
    if (!plan[kPlanTabled] || c >= plan[kPlanClasses]) return;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_jobs) return;
    const int pos_b = class_begin[c], pos_e = class_begin[c + 1];
    const int cap = gap_c[pos_b];
    const int w_max = gap_w[pos_e - 1];
    const int q0 = class_sub0[c], qe = class_sub0[c + 1];
    const int2 *dp = atom_dp + seg_off[j];
    const int n = n_atoms[j];

    int q = q0;
    int w_q = gap_w[pos_b];
    int reach = n;
    bool done = false;
    for (int b0 = 0; b0 < n && !done; b0 += 4) {
        int2 v[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = dp[b0 + t];      // the tables carry 8 entries of padding
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int idx = b0 + t;
            if (done) continue;
            if (idx >= n || v[t].y > cap || v[t].x > w_max) {
                done = true;
                reach = idx;
            } else {
                while (q < qe && v[t].x > w_q) {
                    start_tab[int64_t(q) * n_jobs + j] = idx;
                    ++q;
                    if (q < qe) w_q = gap_w[pos_b + (q - q0) * sb];
                }
            }
        }
    }
    for (; q < qe; ++q) start_tab[int64_t(q) * n_jobs + j] = reach;
    ncap_tab[int64_t(c) * n_jobs + j] = reach;
}

// --------------------------------------------------------------------------
// The pair-evaluation kernel.
// --------------------------------------------------------------------------
__device__ __forceinline__ int upper_bound_peak(const int2 *__restrict__ a, int n, int v)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid].y <= v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ int upper_bound_dur(const int2 *__restrict__ a, int n, int v)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid].x <= v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// s_waitcnt vmcnt(0): every global load and store of this wave has completed.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0f70); }

template <int BLOCK, int CAP, int PERIOD>
__global__ __launch_bounds__(BLOCK) void k_fit_main(
    int n_jobs, int chunk_bound, const int64_t *__restrict__ seg_off,
    const int2 *__restrict__ atom_dp, const int2 *__restrict__ atom_db,
    const int32_t *__restrict__ n_atoms, const int32_t *__restrict__ plan,
    const int32_t *__restrict__ chunk_begin, const int32_t *__restrict__ chunk_end,
    const int32_t *__restrict__ chunk_class, const int32_t *__restrict__ chunk_sub,
    const int32_t *__restrict__ start_tab,
    const int32_t *__restrict__ ncap_tab, const int32_t *__restrict__ gap_w,
    const int32_t *__restrict__ gap_c, const int64_t *__restrict__ gap_row,
    const int32_t *__restrict__ gap_run_end, int32_t *__restrict__ cut)
{
    static_assert((CAP & (CAP - 1)) == 0 && PERIOD % 4 == 0 && BLOCK % kWave == 0, "tile shape");
    __shared__ int2 win[CAP][BLOCK];

    // Blocks of one job tile sit on one XCD (block ids are dealt round-robin
    // over the 8 XCDs): its atoms and tables stay in that XCD's L2.
    const int xcd = blockIdx.x & 7;
    const int k = blockIdx.x >> 3;
    const int job_tile = (k / chunk_bound) * 8 + xcd;
    const int chunk = k % chunk_bound;
    if (job_tile * BLOCK >= n_jobs || chunk >= plan[kPlanChunks]) return;
    const bool tabled = plan[kPlanTabled] != 0;
    const int tid = threadIdx.x;
    const int j_raw = job_tile * BLOCK + tid;
    const bool live = j_raw < n_jobs;
    const int j = live ? j_raw : n_jobs - 1;   // spare lanes shadow the last job: same value, same address
    const int64_t base = seg_off[j];
    const int n = n_atoms[j];
    const int2 *dp = atom_dp + base;
    const int2 *db = atom_db + base;
    const int s_begin = chunk_begin[chunk], s_end = chunk_end[chunk];

    int n_cap = 0;   // atoms the current capacity class can reach
    int a = 0;       // atoms whose running duration fits the current window
    int hi = 0;      // atoms [a, hi) are staged in the LDS window
    int cur = -1;    // boundary of atom a-1, or -1
    int nd = 0, nb = 0;     // atom a     (meaningful while a < hi)
    int nd2 = 0, nb2 = 0;   // atom a + 1 (meaningful while a + 1 < hi)
    int c_cur = 0;
    unsigned long long dry_mask = 0;   // lanes with hi < n_cap: reaching hi may leave atoms unpassed

    auto init = [&](int s) {
        c_cur = gap_c[s];
        if (tabled) {
            a = start_tab[int64_t(chunk_sub[chunk]) * n_jobs + j];
            n_cap = ncap_tab[int64_t(chunk_class[chunk]) * n_jobs + j];
        } else {
            n_cap = upper_bound_peak(dp, n, c_cur);
            a = upper_bound_dur(dp, n_cap, gap_w[s]);
        }
        cur = a > 0 ? db[a - 1].y : -1;
        hi = a;
    };
    auto reload = [&]() {
        const int2 x = win[a & (CAP - 1)][tid]; nd = x.x; nb = x.y;
        const int2 y = win[(a + 1) & (CAP - 1)][tid]; nd2 = y.x; nb2 = y.y;
    };
    auto topup = [&]() {
        const int want = min(a + CAP, n_cap);
        int2 v[CAP];
#pragma unroll
        for (int t = 0; t < CAP; ++t)
            if (hi + t < want) v[t] = db[hi + t];
#pragma unroll
        for (int t = 0; t < CAP; ++t)
            if (hi + t < want) win[(hi + t) & (CAP - 1)][tid] = v[t];
        hi = max(hi, want);
        reload();
    };
    constexpr unsigned ROW = BLOCK * sizeof(int2);     // bytes per window slot row (a power of two)
    static_assert((ROW & (ROW - 1)) == 0, "BLOCK must be a power of two");
    const unsigned lds_lane = unsigned(tid) * unsigned(sizeof(int2));
    // One step: move every lane past the atoms that window w has reached, then
    // store.  The body is predicated rather than branched per lane, and the next
    // two atoms of each lane sit in registers, so no LDS answer is needed before
    // the loop condition is known; it repeats only while some lane passes a
    // further atom.
    auto step = [&](int w, int64_t row) {
        bool adv = a < hi && nd <= w;
        if (__any(adv)) {
            do {
                cur = adv ? nb : cur;
                a += adv ? 1 : 0;
                nd = adv ? nd2 : nd;
                nb = adv ? nb2 : nb;
                {   // atom a + 1 from the circular window: slot = (a + 1) mod CAP
                    const unsigned off = (unsigned(a) * ROW + (ROW + lds_lane)) & (CAP * ROW - 1u);
                    const int2 y = *reinterpret_cast<const int2 *>(reinterpret_cast<const char *>(&win[0][0]) + off);
                    nd2 = y.x; nb2 = y.y;
                }
                if (__ballot(a == hi) & dry_mask) {
                    // a window ran dry inside a period: refill at once (rare)
                    if (a == hi && hi < n_cap) {
                        const int want = min(a + CAP, n_cap);
                        for (int idx = hi; idx < want; ++idx) win[idx & (CAP - 1)][tid] = db[idx];
                        hi = want;
                        reload();
                    }
                    dry_mask = __ballot(hi < n_cap);
                    wait_vmem();
                }
                adv = a < hi && nd <= w;
            } while (__any(adv));
        }
        (cut + row)[j] = cur;
    };

    for (int s0 = s_begin; s0 < s_end; s0 += PERIOD) {
        const int s1 = min(s_end, s0 + PERIOD);
        if (s0 == s_begin || gap_c[s0] != c_cur) init(s0);
        topup();
        dry_mask = __ballot(hi < n_cap);
        wait_vmem();   // below, until the next period, no global load is pending
        if (s1 - s0 == PERIOD && gap_run_end[s0] >= s1) {
#pragma unroll
            for (int u4 = 0; u4 < PERIOD; u4 += 4) {
                const int wv[4] = {gap_w[s0 + u4], gap_w[s0 + u4 + 1], gap_w[s0 + u4 + 2], gap_w[s0 + u4 + 3]};
                const int64_t rv[4] = {gap_row[s0 + u4], gap_row[s0 + u4 + 1], gap_row[s0 + u4 + 2],
                                       gap_row[s0 + u4 + 3]};
#pragma unroll
                for (int u = 0; u < 4; ++u) step(wv[u], rv[u]);
            }
        } else {
            for (int s = s0; s < s1; ++s) {
                if (gap_c[s] != c_cur) { init(s); topup(); dry_mask = __ballot(hi < n_cap); wait_vmem(); }
                step(gap_w[s], gap_row[s]);
            }
        }
    }
}

// --------------------------------------------------------------------------
// Interest rows.  A job answers a gap with interest exactly when its first
// atom fits (running duration and running peak only grow along the atoms), so
// bit j of a gap's row is D_first(j) <= W && P_first(j) <= C.  Per (capacity
// class, 32-job word) a small table holds the word of jobs whose first atom
// fits the capacity and the smallest and largest first duration among them:
// a window at or above the largest gives that word, one below the smallest
// gives 0, and only windows in between (a few hundred ticks at the bottom of a
// class) look at the 32 jobs one by one.  One thread per (gap, word); a wave
// stores 256 contiguous bytes of a row.
// --------------------------------------------------------------------------
__device__ __forceinline__ int4 bits_word_entry(int n_jobs, int j0, int c, const int2 *__restrict__ first_dp)
{
    int2 f[32];
#pragma unroll
    for (int b = 0; b < 32; ++b) f[b] = first_dp[min(j0 + b, n_jobs - 1)];
    uint32_t fits = 0;
    int d_min = INT32_MAX, d_max = INT32_MIN;
#pragma unroll
    for (int b = 0; b < 32; ++b) {
        if (j0 + b < n_jobs && f[b].y <= c && f[b].x != INT32_MAX) {
            fits |= 1u << b;
            d_min = min(d_min, f[b].x);
            d_max = max(d_max, f[b].x);
        }
    }
    return make_int4(int(fits), d_min, d_max, 0);
}

// table[c][word] for the classes of the table-driven plan
__global__ __launch_bounds__(256) void k_bits_table(int n_jobs, int words, const int32_t *__restrict__ plan,
                                                    const int32_t *__restrict__ class_begin,
                                                    const int32_t *__restrict__ gap_c,
                                                    const int2 *__restrict__ first_dp, int4 *__restrict__ table)
{
    const int word = blockIdx.x * blockDim.x + threadIdx.x;
    const int c = blockIdx.y;
    if (!plan[kPlanTabled] || c >= plan[kPlanClasses] || word >= words) return;
    table[int64_t(c) * words + word] = bits_word_entry(n_jobs, word * 32, gap_c[class_begin[c]], first_dp);
}

constexpr int kBitsRows = 8;       // gaps per block

// Rows are taken in the caller's gap order, so the blocks write the interest
// matrix front to back.
__global__ __launch_bounds__(256) void k_fit_bits(int n_jobs, int n_gaps, int words,
                                                  const int32_t *__restrict__ plan,
                                                  const int2 *__restrict__ first_dp,
                                                  const int4 *__restrict__ table,
                                                  const int32_t *__restrict__ gap_rank,
                                                  const int32_t *__restrict__ gap_cls,
                                                  const int32_t *__restrict__ gap_w,
                                                  const int32_t *__restrict__ gap_c,
                                                  uint32_t *__restrict__ bits)
{
    const int word = blockIdx.x * blockDim.x + threadIdx.x;
    if (word >= words) return;
    const bool tabled = plan[kPlanTabled] != 0;
    const int j0 = word * 32;
    const int g_begin = blockIdx.y * kBitsRows, g_end = min(n_gaps, g_begin + kBitsRows);
    int pos[kBitsRows];
#pragma unroll
    for (int r = 0; r < kBitsRows; ++r) pos[r] = gap_rank[min(g_begin + r, n_gaps - 1)];
    int cls = -1;
    int4 e = make_int4(0, INT32_MAX, INT32_MIN, 0);
#pragma unroll
    for (int r = 0; r < kBitsRows; ++r) {
        const int g = g_begin + r;
        if (g >= g_end) break;
        const int s = pos[r];
        const int w = gap_w[s];
        if (tabled) {
            const int c = gap_cls[s];
            if (c != cls) { cls = c; e = table[int64_t(c) * words + word]; }
        } else {
            e = bits_word_entry(n_jobs, j0, gap_c[s], first_dp);
        }
        uint32_t v = 0;
        if (w >= e.z) {
            v = uint32_t(e.x);
        } else if (w >= e.y) {
            for (int b = 0; b < 32; ++b)
                if ((uint32_t(e.x) >> b) & 1u) v |= (first_dp[j0 + b].x <= w ? 1u : 0u) << b;
        }
        bits[int64_t(g) * words + word] = v;
    }
}

}  // namespace sja
