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

// Rank of every gap in the order (C, W, index), in two steps: tiles of
// kGapTile gaps are sorted in LDS (bitonic network over (key, index) pairs, which
// are all distinct, so the order is total and the result exact), then every gap
// adds up, over all tiles, how many pairs of the tile precede its own (a binary
// search in the tile, staged in LDS; its position, inside its own tile).
constexpr int kGapSortThreads = 1024;
constexpr int kGapRankBlock = 256;

__device__ __forceinline__ bool gap_pair_less(unsigned long long ka, int ia, unsigned long long kb, int ib)
{
    return ka < kb || (ka == kb && ia < ib);
}

__global__ __launch_bounds__(kGapSortThreads) void k_gap_tile_sort(int n_gaps, const int32_t *__restrict__ W,
                                                                   const int32_t *__restrict__ C,
                                                                   unsigned long long *__restrict__ tile_key,
                                                                   int32_t *__restrict__ tile_idx, int32_t *plan,
                                                                   int32_t *class_dmax)
{
    __shared__ unsigned long long s_key[kGapTile];
    __shared__ int s_idx[kGapTile];
    if (blockIdx.x == 0) {     // counters that later kernels of the sequence add to
        if (threadIdx.x == 0) plan[kPlanMarks] = 0;
        if (threadIdx.x < kMaxClasses) class_dmax[threadIdx.x] = INT32_MIN;
    }
    const int base = blockIdx.x * kGapTile;
    for (int i = threadIdx.x; i < kGapTile; i += kGapSortThreads) {
        const int g = base + i;
        s_key[i] = g < n_gaps ? gap_key(W[g], C[g]) : ~0ull;      // padding sorts last (index beyond every gap)
        s_idx[i] = g < n_gaps ? g : INT32_MAX;
    }
    __syncthreads();
    for (int k = 2; k <= kGapTile; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < kGapTile / 2; t += kGapSortThreads) {
                const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1));     // the t-th index with bit j clear
                const int hi = lo | j;
                const bool up = (lo & k) == 0;
                const unsigned long long ka = s_key[lo], kb = s_key[hi];
                const int ia = s_idx[lo], ib = s_idx[hi];
                if (gap_pair_less(kb, ib, ka, ia) == up) {
                    s_key[lo] = kb; s_idx[lo] = ib;
                    s_key[hi] = ka; s_idx[hi] = ia;
                }
            }
            __syncthreads();
        }
    }
    for (int i = threadIdx.x; i < kGapTile; i += kGapSortThreads) {
        tile_key[base + i] = s_key[i];
        tile_idx[base + i] = s_idx[i];
    }
}

// One thread per entry of the sorted tiles.  rank[g] = number of gaps that precede g; the
// gap's window, capacity, index and the element offset of its cut row go to that position of
// the sorted copies.
__global__ __launch_bounds__(kGapRankBlock) void k_gap_rank(int n_gaps, int n_jobs, int n_tiles,
                                                            const unsigned long long *__restrict__ tile_key,
                                                            const int32_t *__restrict__ tile_idx,
                                                            const int32_t *__restrict__ W,
                                                            const int32_t *__restrict__ C,
                                                            int32_t *__restrict__ rank, int32_t *__restrict__ order,
                                                            int32_t *__restrict__ ws, int32_t *__restrict__ cs,
                                                            int64_t *__restrict__ row)
{
    __shared__ unsigned long long s_key[kGapTile];
    __shared__ int s_idx[kGapTile];
    const int e = blockIdx.x * kGapRankBlock + threadIdx.x;       // entry of the sorted tiles
    const int own = e / kGapTile;
    const unsigned long long key = tile_key[e];
    const int idx = tile_idx[e];
    int r = e - own * kGapTile;                                    // pairs of its own tile before it
    for (int t = 0; t < n_tiles; ++t) {
        if (t == own) continue;                                    // uniform over the block: kGapTile % kGapRankBlock == 0
        __syncthreads();
        for (int i = threadIdx.x; i < kGapTile; i += kGapRankBlock) {
            s_key[i] = tile_key[t * kGapTile + i];
            s_idx[i] = tile_idx[t * kGapTile + i];
        }
        __syncthreads();
        int lo = 0, hi = kGapTile;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (gap_pair_less(s_key[mid], s_idx[mid], key, idx)) lo = mid + 1; else hi = mid;
        }
        r += lo;
    }
    if (idx < n_gaps) {
        rank[idx] = r;
        order[r] = idx;
        ws[r] = W[idx];
        cs[r] = C[idx];
        row[r] = int64_t(idx) * n_jobs;
    }
}

// Capacity classes = runs of equal C in the sorted order.  k_gap_marks appends the
// first position of every run to a short list (a count beyond kMaxClasses only
// says "too many": then the plan is not table-driven); k_gap_plan, every block
// for itself, puts the list in order and derives the classes from it, then the
// blocks share the per-position and per-chunk work.  The counters these kernels
// add to are cleared by k_gap_tile_sort, the first kernel of the sequence.
__global__ __launch_bounds__(256) void k_gap_marks(int n_gaps, const int32_t *__restrict__ cs, int32_t *plan,
                                                   int32_t *__restrict__ marks)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_gaps) return;
    if (s == 0 || cs[s] != cs[s - 1]) {
        const int i = atomicAdd(&plan[kPlanMarks], 1);
        if (i <= kMaxClasses) marks[i] = s;
    }
}

// Chunks: at most gc sorted positions; sub-blocks: at most sb.  With at most
// kMaxClasses classes neither straddles a class and the table-driven path is
// used; otherwise chunks are plain slices and the stepping kernels search for
// themselves.  Also: the class of every sorted position and run_end[s] = the
// first position after s whose capacity differs.
__global__ __launch_bounds__(256) void k_gap_plan(int n_gaps, int gc, int sb, int chunk_bound, int sub_bound,
                                                  const int32_t *__restrict__ cs, const int32_t *__restrict__ marks,
                                                  int32_t *plan, int32_t *class_begin,
                                                  int32_t *class_chunk0, int32_t *class_sub0,
                                                  int32_t *chunk_begin, int32_t *chunk_end,
                                                  int32_t *chunk_class, int32_t *chunk_sub,
                                                  int32_t *sub_begin, int32_t *sub_end,
                                                  int32_t *sub_class, int32_t *__restrict__ gap_cls,
                                                  int32_t *__restrict__ run_end)
{
    static_assert(kMaxClasses <= kWave, "one wave scans the classes");
    __shared__ int s_begin[kMaxClasses + 1], s_chunk0[kMaxClasses + 1], s_sub0[kMaxClasses + 1];
    const int t = threadIdx.x;
    const int n_marks = plan[kPlanMarks];
    const bool tabled = n_marks <= kMaxClasses;
    const int n_classes = n_marks;
    int n_chunks = 0, n_subs = 0;
    if (tabled) {
        if (t < kWave) {
            // the marks in ascending order (each lane counts the marks below its own), then the
            // first chunk and the first sub-block of every class by a scan over the class lengths
            const int mine = t < n_classes ? marks[t] : INT32_MAX;
            int r = 0;
#pragma unroll 8
            for (int i = 0; i < kWave; ++i) r += __builtin_amdgcn_readlane(mine, i) < mine;
            if (t < n_classes) s_begin[r] = mine;
            if (t == 0) s_begin[n_classes] = n_gaps;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int len = t < n_classes ? s_begin[t + 1] - s_begin[t] : 0;
            const int nq = (len + gc - 1) / gc, nu = (len + sb - 1) / sb;
            int iq = nq, iu = nu;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const int oq = __shfl_up(iq, d, kWave), ou = __shfl_up(iu, d, kWave);
                if (t >= d) { iq += oq; iu += ou; }
            }
            if (t < n_classes) { s_chunk0[t] = iq - nq; s_sub0[t] = iu - nu; }
            if (t == kWave - 1) { s_chunk0[n_classes] = iq; s_sub0[n_classes] = iu; }
        }
        __syncthreads();
        n_chunks = min(s_chunk0[n_classes], chunk_bound);
        n_subs = min(s_sub0[n_classes], sub_bound);
    } else {
        n_chunks = min((n_gaps + gc - 1) / gc, chunk_bound);
    }
    if (blockIdx.x == 0) {
        if (tabled && t <= n_classes) {
            class_begin[t] = s_begin[t];
            class_chunk0[t] = s_chunk0[t];
            class_sub0[t] = s_sub0[t];
        }
        if (t == 0) {
            plan[kPlanClasses] = n_classes;
            plan[kPlanChunks] = n_chunks;
            plan[kPlanTabled] = tabled ? 1 : 0;
            plan[kPlanSubBlocks] = n_subs;
        }
    }
    const int gid = blockIdx.x * blockDim.x + t, stride = gridDim.x * blockDim.x;
    auto class_of = [&](const int *first, int v) {      // last class whose first item is <= v
        int lo = 0, hi = n_classes;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (first[mid] <= v) lo = mid; else hi = mid;
        }
        return lo;
    };
    for (int s = gid; s < n_gaps; s += stride) {
        if (tabled) {
            const int c = class_of(s_begin, s);
            gap_cls[s] = c;
            run_end[s] = s_begin[c + 1];
        } else {
            const int c = cs[s];
            int lo = s + 1, hi = n_gaps;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (cs[mid] <= c) lo = mid + 1; else hi = mid;
            }
            run_end[s] = lo;
        }
    }
    for (int q = gid; q < n_chunks; q += stride) {
        if (tabled) {
            const int c = class_of(s_chunk0, q);
            const int b = s_begin[c] + (q - s_chunk0[c]) * gc;
            chunk_begin[q] = b;
            chunk_end[q] = min(s_begin[c + 1], b + gc);
            chunk_class[q] = c;
            chunk_sub[q] = s_sub0[c] + (q - s_chunk0[c]) * (gc / sb);
        } else {
            chunk_begin[q] = q * gc;
            chunk_end[q] = min(n_gaps, q * gc + gc);
            chunk_class[q] = -1;
            chunk_sub[q] = 0;
        }
    }
    for (int u = gid; u < n_subs; u += stride) {
        const int c = class_of(s_sub0, u);
        const int b = s_begin[c] + (u - s_sub0[c]) * sb;
        sub_begin[u] = b;
        sub_end[u] = min(s_begin[c + 1], b + sb);
        sub_class[u] = c;
    }
}

// --------------------------------------------------------------------------
// Start tables (table-driven path).  A row is a run of sorted positions of one
// capacity class: the chunks of the stepping kernels (the table sja_fit and
// sja_fit_select need) or the finer sub-blocks (the table the grant lists are
// built from).
//   start[row][j] = #atoms of job j usable by the first gap of the row
//   ncap[c][j]    = #atoms any gap of class c can reach (peak <= C_c and
//                   duration <= the class's largest window); null: not wanted
// A block takes kStartsJobs consecutive jobs: their atoms go to LDS once
// (coalesced), then every lane keeps one of the jobs (lane % kStartsJobs) and
// the lanes run along the classes and along the rows, each lane with a binary
// search of its own: both counts are "how many atoms have a running duration
// (peak) of at most x", and both sequences ascend.  A wave's store is then four
// rows of sixteen consecutive jobs, 64 bytes each (a wave per job, lanes along
// the rows, wrote every value into a cache line of its own: 0.6 ms for the 565
// sub-block rows of the Stress workload against 0.14).
// --------------------------------------------------------------------------
constexpr int kStartsAtoms = 512;           // atoms of a job kept in LDS (more: the rest is read from memory)
constexpr int kStartsJobs = 8;              // consecutive jobs of a block
constexpr int kStartsRows = 1024;           // rows whose window and class are kept in LDS

__global__ __launch_bounds__(256) void k_fit_starts(
    int n_jobs, int rows_word, const int32_t *__restrict__ plan, const int32_t *__restrict__ class_begin,
    const int32_t *__restrict__ row_begin, const int32_t *__restrict__ row_class, const int32_t *__restrict__ gap_w,
    const int32_t *__restrict__ gap_c, const int64_t *__restrict__ seg_off,
    const int2 *__restrict__ atom_dp, const int32_t *__restrict__ n_atoms,
    int32_t *__restrict__ start_tab, int32_t *__restrict__ ncap_tab)
{
    constexpr int GROUPS = 256 / kStartsJobs;                  // rows (or classes) a block takes per step
    __shared__ int2 s_at[kStartsJobs][kStartsAtoms + 1];       // padded: equal places of different jobs in different banks
    __shared__ int s_n[kStartsJobs];
    __shared__ int s_roww[kStartsRows];
    __shared__ int s_rowc[kStartsRows];
    __shared__ int s_cap[kMaxClasses], s_wmax[kMaxClasses];
    __shared__ int s_ncap[kMaxClasses][kStartsJobs];
    if (!plan[kPlanTabled]) return;
    const int n_classes = plan[kPlanClasses], n_rows = plan[rows_word];
    const int tid = threadIdx.x;
    for (int q = tid; q < min(n_rows, kStartsRows); q += 256) {
        s_roww[q] = gap_w[row_begin[q]];
        s_rowc[q] = row_class[q];
    }
    if (tid < n_classes) {
        s_cap[tid] = gap_c[class_begin[tid]];
        s_wmax[tid] = gap_w[class_begin[tid + 1] - 1];
    }
    const int j0 = blockIdx.x * kStartsJobs;
    {
        // staging: GROUPS threads per job
        const int jl = tid / GROUPS, sub = tid % GROUPS, j = j0 + jl;
        int n = 0;
        if (j < n_jobs) {
            n = n_atoms[j];
            // eight loads in flight per thread: one trip per 8 * GROUPS atoms, not one per GROUPS
            const int2 *src = atom_dp + seg_off[j];
            const int lim = min(n, kStartsAtoms);
            for (int a0 = sub; a0 < lim; a0 += 8 * GROUPS) {
                int2 v[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) v[t] = src[min(a0 + t * GROUPS, lim - 1)];
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (a0 + t * GROUPS < lim) s_at[jl][a0 + t * GROUPS] = v[t];
            }
        }
        if (sub == 0) s_n[jl] = n;
    }
    __syncthreads();
    const int jl = tid % kStartsJobs, group = tid / kStartsJobs, j = j0 + jl;
    const bool live = j < n_jobs;
    const int n = s_n[jl];
    const int2 *dp = atom_dp + (live ? seg_off[j] : 0);
    auto atom = [&](int a) { return a < kStartsAtoms ? s_at[jl][a] : dp[a]; };
    auto count_dur = [&](int w) {               // atoms with running duration <= w
        int lo = 0, hi = n;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (atom(mid).x <= w) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    for (int c = group; c < n_classes; c += GROUPS) {
        const int cap = s_cap[c];
        int lo = 0, hi = n;                     // atoms with running peak <= cap
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (atom(mid).y <= cap) lo = mid + 1; else hi = mid;
        }
        const int reach = min(lo, count_dur(s_wmax[c]));
        s_ncap[c][jl] = reach;
        if (ncap_tab && live) ncap_tab[int64_t(c) * n_jobs + j] = reach;
    }
    __syncthreads();
    for (int q = group; q < n_rows; q += GROUPS) {
        const int w = q < kStartsRows ? s_roww[q] : gap_w[row_begin[q]];
        const int c = q < kStartsRows ? s_rowc[q] : row_class[q];
        const int v = min(count_dur(w), s_ncap[c][jl]);
        if (live) start_tab[int64_t(q) * n_jobs + j] = v;
    }
}

// --------------------------------------------------------------------------
// Interest rows.  A job answers a gap with interest exactly when its first
// atom fits (running duration and running peak only grow along the atoms), so
// bit j of a gap's row is D_first(j) <= W && P_first(j) <= C.  Per capacity
// class a table holds, for every 32-job word, the jobs whose first atom fits the
// capacity, and the largest first duration among all of those: a gap whose
// window reaches that duration gets the class's words as they are (a row copy);
// the few gaps below it (the bottom of every class in the sorted order) and all
// gaps of a plan without class tables are evaluated job by job, lanes along
// jobs, one ballot per 64 jobs.  A block takes kBitsRows sorted positions and
// 1024 words of their rows.
// --------------------------------------------------------------------------
// table[c][word] and dmax[c] for the classes of the table-driven plan (dmax is
// cleared by k_gap_tile_sort)
__global__ __launch_bounds__(256) void k_bits_table(int n_jobs, int words, const int32_t *__restrict__ plan,
                                                    const int32_t *__restrict__ class_begin,
                                                    const int32_t *__restrict__ gap_c,
                                                    const int2 *__restrict__ first_dp, uint32_t *__restrict__ table,
                                                    int32_t *class_dmax)
{
    const int word = blockIdx.x * blockDim.x + threadIdx.x;
    const int c = blockIdx.y;
    if (!plan[kPlanTabled] || c >= plan[kPlanClasses]) return;
    const int cap = gap_c[class_begin[c]];
    uint32_t fits = 0;
    int d_max = INT32_MIN;
    if (word < words) {
        int2 f[32];
#pragma unroll
        for (int b = 0; b < 32; ++b) f[b] = first_dp[min(word * 32 + b, n_jobs - 1)];
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            if (word * 32 + b < n_jobs && f[b].y <= cap && f[b].x != INT32_MAX) {
                fits |= 1u << b;
                d_max = max(d_max, f[b].x);
            }
        }
        table[int64_t(c) * words + word] = fits;
    }
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) d_max = max(d_max, __shfl_xor(d_max, d, kWave));
    if ((threadIdx.x & (kWave - 1)) == 0 && d_max != INT32_MIN) atomicMax(&class_dmax[c], d_max);
}

constexpr int kBitsRows = 16;      // sorted gap positions per block
constexpr int kBitsWords = 4;      // consecutive 32-job words per thread

struct BitsArgs {
    uint32_t *bits;
    const int2 *first_dp;
    const uint32_t *table;
    const int32_t *class_dmax;
    const int32_t *gap_order;
    const int32_t *gap_cls;
    int n_gaps, words;
};

__global__ __launch_bounds__(256) void k_fit_bits(BitsArgs B, int n_jobs, const int32_t *__restrict__ plan,
                                                  const int32_t *__restrict__ gap_w, const int32_t *__restrict__ gap_c)
{
    __shared__ int s_dmax[kMaxClasses];
    const int words = B.words;
    const int col_tiles = (words + 256 * kBitsWords - 1) / (256 * kBitsWords);
    const int ct = int(blockIdx.x % unsigned(col_tiles)), rt = int(blockIdx.x / unsigned(col_tiles));
    const int tid = threadIdx.x;
    const int w0 = (ct * 256 + tid) * kBitsWords;
    const int s_begin = rt * kBitsRows, s_end = min(B.n_gaps, s_begin + kBitsRows);
    if (s_begin >= s_end) return;
    const bool tabled = plan[kPlanTabled] != 0;
    if (tid < kMaxClasses) s_dmax[tid] = B.class_dmax[tid];
    const int nw = max(0, min(kBitsWords, words - w0));
    const bool wide = nw == kBitsWords && (words % kBitsWords) == 0 &&      // 16-byte aligned row pieces
                      (reinterpret_cast<uintptr_t>(B.bits) & 15u) == 0;
    // the rows of this block (uniform over the block, so these sit in scalar registers)
    int gq[kBitsRows], wq[kBitsRows], cq[kBitsRows], kq[kBitsRows];
#pragma unroll
    for (int r = 0; r < kBitsRows; ++r) {
        const int s = min(s_begin + r, s_end - 1);
        gq[r] = B.gap_order[s];
        wq[r] = gap_w[s];
        cq[r] = gap_c[s];
        kq[r] = tabled ? B.gap_cls[s] : 0;
    }
    __syncthreads();
    if (tabled) {
        // a gap whose window reaches the class's largest first duration gets the class's words; the
        // gaps below it are k_fit_bits_low's
        int cls = -1;
        uint32_t e[kBitsWords] = {0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < kBitsRows; ++r) {
            if (s_begin + r >= s_end) break;
            const int c = kq[r];
            if (wq[r] < s_dmax[c] || nw <= 0) continue;
            if (c != cls) {
                cls = c;
#pragma unroll
                for (int i = 0; i < kBitsWords; ++i)
                    if (i < nw) e[i] = B.table[int64_t(c) * words + w0 + i];
            }
            uint32_t *dst = B.bits + int64_t(gq[r]) * words + w0;
            if (wide) {
                *reinterpret_cast<uint4 *>(dst) = make_uint4(e[0], e[1], e[2], e[3]);
            } else {
#pragma unroll
                for (int i = 0; i < kBitsWords; ++i)
                    if (i < nw) dst[i] = e[i];
            }
        }
        return;
    }
    // no class tables: job by job, lanes along the jobs of this block's words, a 64-job ballot per
    // wave and row
    const int lane = tid & (kWave - 1);
    const int j_begin = ct * 256 * kBitsWords * 32;
    const int j_end = min(n_jobs, j_begin + 256 * kBitsWords * 32);
    constexpr int AHEAD = 8;       // first atoms asked for together: the loop is a chain of memory trips otherwise
    for (int jb = j_begin + (tid - lane); jb < j_end; jb += 256 * AHEAD) {      // jb: first job of this wave's first 64
        int2 f[AHEAD];
#pragma unroll
        for (int k = 0; k < AHEAD; ++k) f[k] = B.first_dp[min(jb + k * 256 + lane, n_jobs - 1)];
#pragma unroll
        for (int k = 0; k < AHEAD; ++k) {
            const int j0 = jb + k * 256;
            if (j0 >= j_end) break;                                             // uniform over the wave
            const bool real = j0 + lane < n_jobs && f[k].x != INT32_MAX;
#pragma unroll
            for (int r = 0; r < kBitsRows; ++r) {
                if (s_begin + r >= s_end) break;
                const unsigned long long m = __ballot(real && f[k].x <= wq[r] && f[k].y <= cq[r]);
                uint32_t *dst = B.bits + int64_t(gq[r]) * words + (j0 >> 5);
                if (lane == 0) dst[0] = uint32_t(m);
                if (lane == 32 && (j0 >> 5) + 1 < words) dst[1] = uint32_t(m >> 32);
            }
        }
    }
}

// The rows at the bottom of a class: windows below the class's largest first
// duration.  A block takes kLowRows sorted positions and 256 words of their rows
// and leaves at once when none of the positions is such a row (the usual case
// wherever windows are long against first durations).  Otherwise a thread
// fetches the first durations of its word's 32 jobs once and compares them with
// every such window in turn; a wave stores 256 contiguous bytes of a row per step.
constexpr int kLowRows = 32;

__global__ __launch_bounds__(256) void k_fit_bits_low(BitsArgs B, int n_jobs, const int32_t *__restrict__ plan,
                                                      const int32_t *__restrict__ gap_w)
{
    __shared__ int s_w[kLowRows], s_g[kLowRows], s_c[kLowRows];
    __shared__ unsigned s_low;
    if (!plan[kPlanTabled]) return;
    const int words = B.words;
    const int word = blockIdx.x * blockDim.x + threadIdx.x;
    const int s_begin = blockIdx.y * kLowRows;
    if (threadIdx.x < kWave) {
        const int s = s_begin + int(threadIdx.x);
        bool low = false;
        if (threadIdx.x < kLowRows && s < B.n_gaps) {
            const int w = gap_w[s], c = B.gap_cls[s];
            low = w < B.class_dmax[c];
            s_w[threadIdx.x] = w;
            s_c[threadIdx.x] = c;
            s_g[threadIdx.x] = B.gap_order[s];
        }
        const unsigned long long m = __ballot(low);
        if (threadIdx.x == 0) s_low = unsigned(m);
    }
    __syncthreads();
    unsigned todo = s_low;                               // uniform over the block
    if (!todo) return;
    const bool live = word < words;
    int d[32];
#pragma unroll
    for (int b = 0; b < 32; ++b) d[b] = B.first_dp[min(word * 32 + b, n_jobs - 1)].x;
    int cls = -1;
    uint32_t fits = 0;
    while (todo) {
        const int r = __ffs(int(todo)) - 1;
        todo &= todo - 1;
        const int w = s_w[r], c = s_c[r];
        if (c != cls) {
            cls = c;
            fits = live ? B.table[int64_t(c) * words + word] : 0u;
        }
        uint32_t le = 0;
#pragma unroll
        for (int b = 0; b < 32; ++b) le |= (d[b] <= w ? 1u : 0u) << b;
        if (live) B.bits[int64_t(s_g[r]) * words + word] = le & fits;
    }
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
            a = start_tab[int64_t(chunk) * n_jobs + j];
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
        __builtin_nontemporal_store(cur, cut + row + j);      // written once, read by a later kernel: keep it out of the caches
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

// Measurement aid, no step of the method: the store stream of k_fit_main with nothing
// computed.  Same grid, same block -> (job tile, chunk) mapping, same walk over the
// chunk's sorted positions, one 256-byte piece of a cut row per wave and step, the
// same non-temporal stores; the value stored is the lane's job index.  Its duration
// is what the memory system allows for this address pattern.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_store_reference(int n_jobs, int chunk_bound, const int32_t *__restrict__ plan,
                                                           const int32_t *__restrict__ chunk_begin,
                                                           const int32_t *__restrict__ chunk_end,
                                                           const int64_t *__restrict__ gap_row, int32_t *__restrict__ cut)
{
    const int xcd = blockIdx.x & 7;
    const int k = blockIdx.x >> 3;
    const int job_tile = (k / chunk_bound) * 8 + xcd;
    const int chunk = k % chunk_bound;
    if (job_tile * BLOCK >= n_jobs || chunk >= plan[kPlanChunks]) return;
    const int j_raw = job_tile * BLOCK + threadIdx.x;
    const int j = j_raw < n_jobs ? j_raw : n_jobs - 1;
    const int s_begin = chunk_begin[chunk], s_end = chunk_end[chunk];
    for (int s = s_begin; s < s_end; ++s) __builtin_nontemporal_store(j, cut + gap_row[s] + j);
}

}  // namespace sja
