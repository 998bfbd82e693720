// K4, list-driven: conflict rounds without re-scanning the pair matrix.
//
// The rounds are inherently sequential (a round's selections depend on the
// grants of the round before) and a large batch needs thousands of them, so a
// round must cost next to nothing.  What a gap needs in a round is "my best job
// that no gap holds yet".  Every gap ranks jobs by the same per-atom policy key
// (an atom is a safe cut of a job; the key depends on the job and on the cut,
// not on the gap), and in sorted gap order an atom is the answer of a job for
// one contiguous range of positions.  So:
//   1. all reachable atoms are ranked once by policy key (stable radix passes:
//      key descending, job id ascending);
//   2. for every list block (<= 64 sorted gap positions of one capacity class
//      whose windows are of similar length) the atoms some position of it would
//      get are listed in rank order, each with the range of lanes (positions)
//      it applies to;
//   3. a round is one small kernel: a wave per list block, a lane per gap; a
//      lane that lost walks on through its block's list to the next entry that
//      covers it and whose job is not held, and claims that job with an
//      atomicMax of (round, ~gap index), the claims of a thread block merged
//      first; the next round's kernel first checks who won.  Claims carry the
//      round number, so nothing is ever reset and a claim made in the current
//      round is not mistaken for a hold.  In the early rounds, where lanes
//      pass hundreds of records of jobs that were just taken, the waves
//      also keep the held jobs as a bitmap (see grant_step).
#pragma once

#include "k_sort.h"

namespace sja {

constexpr int kEntryLaneBits = 13;      // low bits of a list entry: lane range lo (6), hi (7)

struct PolicyDev {
    int policy;
    int wait_scale;
    int w0, w1, w2;
    int class0_override;
};

// Per-job multiplier and tier of the policy key: key = (tier, F * mult [, F]).
__device__ __forceinline__ void job_policy(const PolicyDev &pol, const int32_t *wait,
                                           const uint8_t *sla_class, int j,
                                           unsigned long long &mult, unsigned long long &tier)
{
    const int cls = sla_class ? sla_class[j] : 0;
    const long long wt = wait ? wait[j] : 0;
    mult = 1;
    tier = 0;
    switch (pol.policy) {
    case SJA_POLICY_FAIRNESS: mult = (unsigned long long)(pol.wait_scale + wt); break;
    case SJA_POLICY_SLA:
        mult = (unsigned long long)(cls == 0 ? pol.w0 : (cls == 1 ? pol.w1 : pol.w2));
        tier = (pol.class0_override && cls == 0) ? 1 : 0;
        break;
    case SJA_POLICY_MIXED:
        mult = (unsigned long long)(pol.wait_scale + wt);
        tier = (unsigned long long)(2 - cls);
        break;
    default: break;
    }
}

// F = duration x peak and F x multiplier with as few of the (slow) 32-bit integer
// multiplies as the value ranges allow: durations, peaks and multipliers are
// non-negative and fit 32 bits, and a score stays below 2^62.
__device__ __forceinline__ unsigned long long rect_of(int dur, int peak)
{
    return static_cast<unsigned long long>(uint32_t(dur)) * uint32_t(peak);
}

__device__ __forceinline__ unsigned long long times_mult(unsigned long long F, unsigned long long mult)
{
    const uint32_t m = uint32_t(mult);            // wait_scale + wait, or an SLA weight: below 2^32
    return static_cast<unsigned long long>(uint32_t(F)) * m +
           (static_cast<unsigned long long>(uint32_t(F >> 32) * m) << 32);
}

// reach[j] = atoms of job j that some capacity class can reach; reach[n_jobs] = 0.
__global__ void k_reach(int n_jobs, const int32_t *__restrict__ plan, const int32_t *__restrict__ ncap_tab,
                        int32_t *__restrict__ reach)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j > n_jobs) return;
    int r = 0;
    if (j < n_jobs && plan[kPlanTabled]) {
        const int n_classes = plan[kPlanClasses];
        for (int c = 0; c < n_classes; ++c) r = max(r, ncap_tab[int64_t(c) * n_jobs + j]);
    }
    reach[j] = r;
}

// One wave per job: inverted policy keys of its reachable atoms (ascending sort
// of the inverted key = descending key) and the identity permutation.
__global__ __launch_bounds__(256) void k_atom_keys(
    int n_jobs, PolicyDev pol, const int64_t *__restrict__ seg_off, const int2 *__restrict__ atom_dp,
    const long long *__restrict__ atom_area, const int32_t *__restrict__ abase, const int32_t *__restrict__ wait,
    const uint8_t *__restrict__ sla_class, unsigned long long *__restrict__ key_hi,
    unsigned long long *__restrict__ key_lo, uint32_t *__restrict__ perm, int2 *__restrict__ atom_ja)
{
    const int j = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (j >= n_jobs) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int a0 = abase[j], n = abase[j + 1] - a0;
    const int64_t base = seg_off[j];
    const int2 *dp = atom_dp + base;
    unsigned long long mult, tier;
    job_policy(pol, wait, sla_class, j, mult, tier);
    const bool mixed = pol.policy == SJA_POLICY_MIXED;
    for (int a = lane; a < n; a += kWave) {
        const int2 v = dp[a];
        const unsigned long long F = atom_area ? (unsigned long long)atom_area[base + a]
                                               : (unsigned long long)v.x * (unsigned long long)v.y;
        key_hi[a0 + a] = ~((tier << 62) | (F * mult));
        key_lo[a0 + a] = ~(mixed ? F : 0ull);
        perm[a0 + a] = uint32_t(a0 + a);
        atom_ja[a0 + a] = make_int2(j, a);
    }
}

// rank of every atom, and the (job, atom) that holds each rank
__global__ void k_rank_from_perm(const int32_t *n_ptr, const uint32_t *__restrict__ perm,
                                 const int2 *__restrict__ atom_ja, uint32_t *__restrict__ rank,
                                 int2 *__restrict__ ranked)
{
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < *n_ptr) {
        const uint32_t a = perm[i];
        rank[a] = uint32_t(i);
        ranked[i] = atom_ja[a];
    }
}

// Number of entries of sorted w[0..len) that are < d, known to be at least `from`.
__device__ __forceinline__ int count_less(const int *w, int len, int d, int from = 0)
{
    int lo = from, hi = len;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (w[mid] < d) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Grant-list blocks.  A list serves its gaps well when most of its records
// cover most of its lanes; a sub-block that starts at a very small window and
// ends at a much larger one is therefore cut into pieces, each ending before
// the first window beyond 1.5 * (its first window) + 64.
__device__ __forceinline__ int list_piece_end(const int32_t *__restrict__ gap_w, int b, int e)
{
    const int64_t w0 = max(gap_w[b], 0);
    const int64_t limit = w0 + (w0 >> 1) + 64;
    int p = b + 1;
    while (p < e && int64_t(gap_w[p]) <= limit) ++p;
    return p;
}

// Pieces per sub-block (an exclusive scan turns them into lb_off).
__global__ void k_list_blocks_count(int n_slots, const int32_t *__restrict__ plan,
                                    const int32_t *__restrict__ sub_begin, const int32_t *__restrict__ sub_end,
                                    const int32_t *__restrict__ gap_w, int32_t *lb_off)
{
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n_slots) return;
    int cnt = 0;
    if (plan[kPlanTabled] && u < plan[kPlanSubBlocks]) {
        const int e = sub_end[u];
        for (int b = sub_begin[u]; b < e; b = list_piece_end(gap_w, b, e)) ++cnt;
    }
    lb_off[u] = cnt;
}

__global__ void k_list_blocks_write(int lb_cap, const int32_t *__restrict__ plan,
                                    const int32_t *__restrict__ sub_begin, const int32_t *__restrict__ sub_end,
                                    const int32_t *__restrict__ gap_w, const int32_t *__restrict__ lb_off,
                                    int32_t *lb_begin, int32_t *lb_end, int32_t *lb_sub)
{
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (!plan[kPlanTabled] || u >= plan[kPlanSubBlocks]) return;
    int v = lb_off[u];
    const int e = sub_end[u];
    for (int b = sub_begin[u]; b < e && v < lb_cap; ++v) {
        const int p = list_piece_end(gap_w, b, e);
        lb_begin[v] = b;
        lb_end[v] = p;
        lb_sub[v] = u;
        b = p;
    }
}

// Entries of the lists.  Thread (list block v, job j) visits the atoms of j
// that some position of v gets: atom a applies to lanes [lo, hi) where lo is
// the first position whose window reaches D_a and hi the first one that
// already reaches atom a+1.  Every entry is one 64-bit word, v : rank : hi (7
// bits) : lo (6 bits); where it is stored does not matter (the sort orders
// them); entries beyond entry_cap are counted but not stored.
// A block takes kEmitTiles tiles of 256 jobs for one list block.  Each tile is
// visited once: the entries go to a buffer in LDS as they are found (the lanes
// of a wave that find one in the same step of the visit take their places with
// one addition); once the buffer is half full, and after the last tile, the
// block reserves room in the output with one addition to the running total
// (additions to one word are served one after the other: one per wave made
// this kernel three times slower) and copies the buffer out with coalesced
// stores.  Entries that find the buffer full go straight to the output, a
// wave's step at a time.
constexpr int kEmitTiles = 8;
constexpr int kEmitBuffer = 3072;     // entries staged in LDS (24 KB: six blocks per compute unit)

template <typename Sink>
__device__ __forceinline__ void list_visit(const int2 *__restrict__ dp, const int *s_w, int len, int a_first, int n_cap,
                                           Sink &&sink)
{
    const int a_begin = max(a_first - 1, 0);
    if (a_begin >= n_cap) return;
    // an atom's range ends where the next one's begins: one search per atom
    int lo = a_begin < a_first ? 0 : count_less(s_w, len, dp[a_begin].x);
    for (int a = a_begin; a < n_cap && lo < len; ++a) {
        const int hi = a + 1 < n_cap ? count_less(s_w, len, dp[a + 1].x, lo) : len;    // durations ascend
        if (hi > lo) sink(a, lo, hi);
        lo = hi;
    }
}

__global__ __launch_bounds__(256) void k_list_emit(
    int n_jobs, int rank_bits, int job_shift, int lb_cap, long long entry_cap, const int32_t *__restrict__ plan, const int32_t *__restrict__ lb_begin,
    const int32_t *__restrict__ lb_end, const int32_t *__restrict__ lb_sub, const int32_t *__restrict__ sub_class,
    const int32_t *__restrict__ gap_w, const int64_t *__restrict__ seg_off,
    const int2 *__restrict__ atom_dp, const int32_t *__restrict__ start_tab,
    const int32_t *__restrict__ ncap_tab, const int32_t *__restrict__ abase,
    const uint32_t *__restrict__ rank, int32_t *sub_count, unsigned long long *total,
    unsigned long long *__restrict__ ekey)
{
    __shared__ int s_w[64];
    __shared__ unsigned long long s_buf[kEmitBuffer];
    __shared__ int s_cursor, s_all;
    __shared__ unsigned long long s_base;
    const int u = blockIdx.y;                  // list block
    if (!plan[kPlanTabled] || u >= min(plan[kPlanListBlocks], lb_cap)) return;
    const int b0 = lb_begin[u], len = lb_end[u] - b0;
    if (threadIdx.x < 64) s_w[threadIdx.x] = threadIdx.x < len ? gap_w[b0 + threadIdx.x] : INT32_MAX;
    if (threadIdx.x == 0) { s_cursor = 0; s_all = 0; }
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1);
    const int sub = lb_sub[u];
    const int cls = sub_class[sub];
    const int j0 = blockIdx.x * (kEmitTiles * 256) + threadIdx.x;
    const unsigned long long head = (unsigned long long)u << rank_bits;
    for (int it = 0; it < kEmitTiles; ++it) {
        const int j = j0 + it * 256;
        if (j < n_jobs) {
            int af = start_tab[int64_t(sub) * n_jobs + j];
            const int nc = ncap_tab[int64_t(cls) * n_jobs + j];
            const int2 *dp = atom_dp + seg_off[j];
            // the table holds the count at the sub-block's first position; a later piece starts further on
            while (af < nc && dp[af].x <= s_w[0]) ++af;
            const int a0 = abase[j];
            // the job rides above the sorted bits when there is room for it (job_shift >= 0)
            const unsigned long long rider = job_shift >= 0 ? (unsigned long long)uint32_t(j) << job_shift : 0ull;
            list_visit(dp, s_w, len, af, nc, [&](int a, int lo, int hi) {
                const unsigned long long key = rider | ((head | rank[a0 + a]) << kEntryLaneBits) | (unsigned long long)((hi << 6) | lo);
                // the lanes of this wave that are at this point together
                const unsigned long long peers = __ballot(true);
                const int n_peers = __popcll(peers);
                const int mine = __builtin_amdgcn_mbcnt_hi(uint32_t(peers >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(peers), 0u));
                int at = 0;
                if (mine == 0) at = atomicAdd(&s_cursor, n_peers);
                at = __builtin_amdgcn_readlane(at, __ffsll((long long)peers) - 1) + mine;
                if (at < kEmitBuffer) {
                    s_buf[at] = key;
                } else {
                    // the buffer is full: this step's surplus goes straight out
                    const unsigned long long over = __ballot(true);
                    unsigned long long to = 0;
                    if (lane == __ffsll((long long)over) - 1) to = atomicAdd(total, (unsigned long long)__popcll(over));
                    to = __shfl(to, __ffsll((long long)over) - 1, kWave) + __popcll(over & lanes_below(lane));
                    if ((long long)to < entry_cap) ekey[to] = key;
                }
            });
        }
        __syncthreads();
        const int found = s_cursor;                           // entries since the last copy, surplus included
        __syncthreads();                                      // everybody has read it before anybody adds to it again
        if (found < kEmitBuffer / 2 && it + 1 < kEmitTiles) continue;       // uniform over the block
        const int staged = min(found, kEmitBuffer);
        if (threadIdx.x == 0) {
            s_all += found;
            s_base = staged ? atomicAdd(total, (unsigned long long)staged) : 0ull;
        }
        __syncthreads();
        const unsigned long long out0 = s_base;
        for (int i = threadIdx.x; i < staged; i += 256)
            if ((long long)(out0 + i) < entry_cap) ekey[out0 + i] = s_buf[i];
        __syncthreads();
        if (threadIdx.x == 0) s_cursor = 0;
        __syncthreads();
    }
    if (threadIdx.x == 0 && s_all) atomicAdd(&sub_count[u], s_all);
}

__device__ __forceinline__ unsigned long long claim_of(int round, int g)
{
    return (static_cast<unsigned long long>(round) << 32) | (0xffffffffu - uint32_t(g));
}

// Sorted entries as 16-byte records (job, rank, lo | hi << 8, 0): one load per entry.
__global__ void k_list_pack(const int32_t *n_ptr, const unsigned long long *__restrict__ ekey, KeyRecords out)
{
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= *n_ptr) return;
    out.rec[i] = key_record(out, ekey[i]);
}

// One round for one list block (one wave, one lane per gap position).  First
// the outcome of round k-1: a gap whose candidate job carries the gap's own
// claim word has won (the grant is final), otherwise it lost.  Then, if
// `propose`, every lane that still needs a job walks on from its own pointer to
// the first entry that covers it and whose job is not held, and claims it.
// st = (pointer, candidate job, rank of the candidate atom, flag) with flag 0 = active,
// 1 = granted, 2 = no candidate left (in memory the flag shares its word with
// the gap index).
//
// The lanes of a wave walk together: per round trip the wave reads kSweep chunks
// of 64 records, starting at the chunk of its lowest pointer still looking, and
// the claim words of those that cover a lane still looking.  A lane passes the
// records of its block that cover other lanes only (a job's other cuts), so
// most rounds some lane of most waves has more than one record to look at; a
// first look at the lane's own next record alone, with the joint walk behind it
// when that was not the one, made nine rounds in ten two trips longer.  The
// first chunks are asked for before the wave knows who won round k-1 (nearly
// every open lane lost), so they travel beside that check's claim word.
constexpr int kSweep = 2;        // chunks of 64 records the wave reads per trip (3: 1.7 ms slower per Stress resolve, 4: 3.7 ms)
constexpr int kSweepHeld = 8;  // the same with the held bitmap: no claim words to fetch, so a wider trip costs little
constexpr int kRoundBlock = 256; // threads per block of the round kernel
constexpr int kBlockClaims = 256; // claims a block merges in LDS per round
constexpr int kClaimTurns = 4;    // jobs whose claims a wave merges over its lanes before the rest are sent singly

constexpr int kHeldMaxWords = 4096;   // words of the held-job bitmap a block keeps in LDS (jobs / 32)
constexpr int kHeldRounds = 512;      // rounds that keep and read the bitmap

__device__ __forceinline__ bool held_bit(const uint32_t *s_held, uint32_t job)
{
    return (s_held[job >> 5] >> (job & 31u)) & 1u;
}

// HELD (the early rounds, where lanes pass hundreds of records of jobs that were
// just taken): the wave asks a bitmap in LDS which jobs were held before this
// round, instead of fetching a claim word per record, so a trip is one memory
// trip, not two; only the record a lane settles on has its claim word fetched.
// Two bitmaps alternate: a round reads one and writes only the other
// (held_next), so nothing it reads changes under it.  A job named in round k is
// held from round k+1 on, whoever wins it: the gaps naming it set its bit in the
// bitmap round k+1 reads, and its winner, when it learns in round k+1 that it
// won, sets it in the other one, after which both carry it.
template <bool HELD>
__device__ __forceinline__ void grant_step(int round, bool propose, int lane, int g, int list_begin, int list_end,
                                           const uint4 *__restrict__ rec, unsigned long long *claim, int4 &st,
                                           bool &lost, bool &cand, int *s_n, int *s_job,
                                           unsigned long long *s_word, const uint32_t *s_held,
                                           uint32_t *held_next)
{
    constexpr int SW = HELD ? kSweepHeld : kSweep;
    lost = false;
    cand = false;
    // the first chunks, for every lane that is open now
    const bool open_now = st.w == 0 && propose && st.x < list_end;
    int e0 = wave_min_dpp(open_now ? st.x : 0x7fffffff);
    bool ahead = e0 != 0x7fffffff;                 // rr holds the chunks from c0 on
    int c0 = ahead ? list_begin + ((e0 - list_begin) & ~(kWave - 1)) : 0;
    uint4 rr[SW];
    if (ahead) {
#pragma unroll
        for (int k = 0; k < SW; ++k) rr[k] = rec[min(c0 + k * kWave + lane, list_end - 1)];
    }
    if (st.w == 0 && st.y >= 0) {
        if (claim[st.y] == claim_of(round - 1, g)) {               // won: final
            st.w = 1;
            if (HELD) atomicOr(&held_next[uint32_t(st.y) >> 5], 1u << (uint32_t(st.y) & 31u));
        } else {
            lost = true;
        }
    }
    int cand_job = -1;
    unsigned long long cand_word = 0;      // the candidate job's claim word as the walk saw it
    const bool walking = st.w == 0 && propose;
    int e = st.x, found = -1, found_j = -1, found_a = -1;
    bool by_bitmap = false;                // found with HELD: the claim word is still to fetch
    bool looking = walking && e < list_end;
    // HELD: the chunks behind the ones being looked at are asked for before the look starts (a wave
    // whose lanes' pointers lie thousands of records apart takes window after window, and a lane
    // that finds nothing goes on exactly there), so their trip overlaps the look.  Always issued,
    // at clamped addresses: a load that may be skipped makes every later wait a wait for all.
    uint4 rn[HELD ? SW : 1];
    int c_next = -1;
    for (;;) {
        const unsigned long long need = __ballot(looking);
        if (!need) break;
        if (!ahead) {
            e0 = wave_min_dpp(looking ? e : 0x7fffffff);    // the wave's lowest pointer still looking
            c0 = list_begin + ((e0 - list_begin) & ~(kWave - 1));
            if (HELD && c0 == c_next) {
#pragma unroll
                for (int k = 0; k < SW; ++k) rr[k] = rn[k];
            } else {
#pragma unroll
                for (int k = 0; k < SW; ++k) rr[k] = rec[min(c0 + k * kWave + lane, list_end - 1)];
            }
        }
        ahead = false;
        if (HELD) {
            c_next = c0 + SW * kWave;
#pragma unroll
            for (int k = 0; k < SW; ++k) rn[k] = rec[min(c_next + k * kWave + lane, list_end - 1)];
        }
        // claim words only of records that cover some lane still looking
        const int all_lo = __ffsll((long long)need) - 1, all_hi = 63 - __clzll((long long)need);
        unsigned long long cw[HELD ? 1 : SW];      // the claim words; HELD asks the bitmap instead
        bool open_job[HELD ? SW : 1];
        if (HELD) {
#pragma unroll
            for (int k = 0; k < SW; ++k) open_job[k] = !held_bit(s_held, rr[k].x);
        } else {
            // every lane loads (the others word 0, one request per wave) so that the loads of all
            // chunks are issued back to back: a load that may be skipped makes the next one wait for it
            bool worth[SW];
#pragma unroll
            for (int k = 0; k < SW; ++k) worth[k] = int(rr[k].z & 255u) <= all_hi && int(rr[k].z >> 8) > all_lo;
#pragma unroll
            for (int k = 0; k < SW; ++k) cw[k] = claim[worth[k] ? rr[k].x : 0u];
#pragma unroll
            for (int k = 0; k < SW; ++k) cw[k] = worth[k] ? cw[k] : ~0ull;
        }
        const bool here = looking && e < c0 + SW * kWave;
        int hit = -1, hj = 0, ha = 0;
        unsigned int hw_lo = 0, hw_hi = 0;
#pragma unroll
        for (int k = 0; k < SW; ++k) {
            // lanes this chunk can serve: still looking, and standing before its end (the pointers of
            // a wave of the early rounds lie thousands of records apart: most lanes `here` only
            // start in a later chunk of the window, and nothing in this one is for them)
            const bool elig = here && hit < 0 && e < c0 + (k + 1) * kWave;
            const unsigned long long still = __ballot(elig);
            if (!still) continue;
            // records worth a look: free, and covering some lane that can take one here
            const int need_lo = __ffsll((long long)still) - 1;
            const int need_hi = 63 - __clzll((long long)still);
            const uint32_t stamp = HELD ? 0u : uint32_t(cw[HELD ? 0 : k] >> 32);
            const bool not_held = HELD ? open_job[HELD ? k : 0] : (stamp == 0 || (stamp >= uint32_t(round) && stamp != 0xffffffffu));
            const bool free_rec = c0 + k * kWave + lane < list_end && not_held &&
                                  int(rr[k].z & 255u) <= need_hi && int(rr[k].z >> 8) > need_lo;
            unsigned long long fm = __ballot(free_rec);
            int hk = -1;
            while (fm) {
                const int t = __ffsll((long long)fm) - 1;
                fm &= fm - 1;
                const unsigned int z = __builtin_amdgcn_readlane(rr[k].z, t);
                const bool h = elig && hk < 0 && c0 + k * kWave + t >= e && lane >= int(z & 255u) &&
                               lane < int(z >> 8);
                if (__any(h)) {
                    // record t's job, atom and claim word straight from lane t's registers
                    const int tj = __builtin_amdgcn_readlane(int(rr[k].x), t), ta = __builtin_amdgcn_readlane(int(rr[k].y), t);
                    // (with HELD the claim word of the record a lane settles on is fetched afterwards)
                    const unsigned int t_lo = HELD ? 0u : __builtin_amdgcn_readlane(int(uint32_t(cw[HELD ? 0 : k])), t);
                    const unsigned int t_hi = HELD ? 0u : __builtin_amdgcn_readlane(int(uint32_t(cw[HELD ? 0 : k] >> 32)), t);
                    if (h) { hk = t; hit = k * kWave + t; hj = tj; ha = ta; hw_lo = t_lo; hw_hi = t_hi; }
                }
                if (!__any(elig && hk < 0)) break;
            }
        }
        if (here) {
            if (hit >= 0) {
                found = c0 + hit; found_j = hj; found_a = ha;
                cand_word = (static_cast<unsigned long long>(hw_hi) << 32) | hw_lo;
                by_bitmap = HELD;
                looking = false;
            } else {
                e = c0 + SW * kWave;
                looking = e < list_end;
            }
        }
    }
    if (HELD && by_bitmap) cand_word = claim[found_j];      // what this round's earlier claims left there
    if (walking) {
        if (found >= 0) {
            st = make_int4(found + 1, found_j, found_a, 0);
            cand = true;
            cand_job = found_j;
        } else {
            st = make_int4(list_end, -1, -1, 2);
        }
    }
    // Claims.  Most gaps of a batch name the same few jobs in a round, so the
    // lanes of a wave that name one job first agree on their lowest gap index,
    // and a claim that the job's word (as the walk read it) already beats is not
    // made.  The wave's claims go to the block's list (s_n, s_job, s_word); the
    // block merges them before anything is sent (a claim that finds the list
    // full is sent at once).
    unsigned long long todo = __ballot(cand);
    for (int turn = 0; todo; ++turn) {
        if (turn == kClaimTurns) {
            // a wave of the early rounds, whose lanes name dozens of different jobs: one turn of
            // this loop per job costs more than the claims it merges, so the rest go out as they are
            if ((todo >> lane) & 1ull) {
                const unsigned long long word = claim_of(round, g);
                if (cand_word < word) {
                    atomicMax(&claim[cand_job], word);
                    if (HELD) atomicOr(&held_next[uint32_t(cand_job) >> 5], 1u << (uint32_t(cand_job) & 31u));
                }
            }
            break;
        }
        const int leader = __ffsll((long long)todo) - 1;
        const int job = __builtin_amdgcn_readlane(cand_job, leader);
        const bool mine = cand && cand_job == job;
        const unsigned int best = 0xffffffffu - uint32_t(wave_min_dpp(mine ? g : 0x7fffffff));   // larger = lower gap index
        if (lane == leader) {
            const unsigned long long word = (static_cast<unsigned long long>(round) << 32) | best;
            if (cand_word < word) {
                const int slot = atomicAdd(s_n, 1);
                if (slot < kBlockClaims) {
                    s_job[slot] = job;
                    s_word[slot] = word;
                } else {
                    atomicMax(&claim[job], word);
                    if (HELD) atomicOr(&held_next[uint32_t(job) >> 5], 1u << (uint32_t(job) & 31u));
                }
            }
        }
        todo &= ~__ballot(mine);
    }
}

// One round per launch, several list blocks per thread block.  Hundreds of
// waves name the same few jobs in a round and atomics on one word are served
// one after the other, so the waves of a block first merge their claims in LDS
// and the block sends one atomicMax per job.  A round leaves two flags: somebody
// lost (round k-1), somebody selected (round k); the host only asks those two
// questions.
// n_lb, the number of list blocks, comes as an argument (the host has read it
// back to size its launches): the state and the block's list bounds are all a
// wave has to wait for before it can ask for its records and its claim word.
// The arguments a wave needs first come first: the library is built so that
// the leading 16 dwords of a kernel's arguments are in scalar registers when
// the wave starts, and the state load does not wait for an argument load.
template <bool HELD>
__global__ __launch_bounds__(kRoundBlock) void k_grant_round(
    int4 *state, const int32_t *__restrict__ list_off, const uint4 *__restrict__ rec, unsigned long long *claim,
    int round, int propose, int n_lb, int held_words, uint32_t *held, const int32_t *__restrict__ lb_begin,
    const int32_t *__restrict__ lb_end, const int32_t *__restrict__ gap_order, int32_t *cnt_lost, int32_t *cnt_cand)
{
    __shared__ int s_n;
    __shared__ int s_job[kBlockClaims];
    __shared__ unsigned long long s_word[kBlockClaims];
    __shared__ uint4 s_held4[HELD ? kHeldMaxWords / 4 : 1];
    const uint32_t *s_held = reinterpret_cast<const uint32_t *>(s_held4);
    uint32_t *held_next = nullptr;
    const int u = blockIdx.x * (kRoundBlock / kWave) + (threadIdx.x / kWave);
    const int lane = threadIdx.x & (kWave - 1);
    // The state of a gap lives at (list block, lane) and carries the gap's index, so
    // that its load needs none of the block tables and travels together with them.
    const int slot = u * kWave + lane;
    int4 raw = make_int4(0, -1, -1, 2);
    int list_begin = 0, list_end = 0;
    if (u < n_lb) {
        raw = state[slot];               // round 1 reads what an earlier resolve left and replaces it below
        list_begin = list_off[u];
        list_end = list_off[u + 1];
    }
    if (HELD) {
        // the bitmap travels together with the state; held_words is a multiple of 4 and at most
        // kHeldMaxWords, and the two bitmaps lie back to back
        const uint4 *src = reinterpret_cast<const uint4 *>(held + size_t(round & 1) * held_words);
        for (int i = threadIdx.x; i < held_words / 4; i += kRoundBlock) s_held4[i] = src[i];
        held_next = held + size_t((round + 1) & 1) * held_words;
    }
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    if (u < n_lb) {
        if (round == 1) {
            const int b0 = lb_begin[u];
            const bool valid = lane < lb_end[u] - b0;
            raw = make_int4(list_begin, -1, -1, valid ? (gap_order[b0 + lane] << 2) : 2);
        }
        const int g = raw.w >> 2;
        int4 st = make_int4(raw.x, raw.y, raw.z, raw.w & 3);
        const int4 before = st;
        bool lost, cand;
        grant_step<HELD>(round, propose != 0, lane, g, list_begin, list_end, rec, claim, st, lost, cand, &s_n, s_job,
                         s_word, s_held, held_next);
        if (st.x != before.x || st.w != before.w || round == 1) state[slot] = make_int4(st.x, st.y, st.z, st.w | (g << 2));
        if (__ballot(lost) && lane == 0) cnt_lost[round - 1] = 1;
        if (__ballot(cand) && lane == 0) cnt_cand[round] = 1;
    }
    __syncthreads();
    const int n = min(s_n, kBlockClaims);
    if (n <= kWave) {
        // the usual case, a handful of claims: one lane of the first wave per claim, the others'
        // claims read from their lanes (a loop over the list in LDS pays two dependent LDS trips
        // per entry, at the very end of every round)
        if (threadIdx.x < kWave) {
            const bool valid = lane < n;
            const int job = valid ? s_job[lane] : -1;
            const unsigned long long word = valid ? s_word[lane] : 0ull;
            unsigned long long best = word;
            bool first = valid;
            for (int k = 0; k < n; ++k) {
                const int jk = __builtin_amdgcn_readlane(job, k);
                const unsigned long long wk =
                    (static_cast<unsigned long long>(uint32_t(__builtin_amdgcn_readlane(int(uint32_t(word >> 32)), k))) << 32) |
                    uint32_t(__builtin_amdgcn_readlane(int(uint32_t(word)), k));
                if (jk == job) {
                    best = max(best, wk);
                    first = first && k >= lane;
                }
            }
            if (first) {
                atomicMax(&claim[job], best);
                if (HELD) atomicOr(&held_next[uint32_t(job) >> 5], 1u << (uint32_t(job) & 31u));
            }
        }
        return;
    }
    for (int i = threadIdx.x; i < n; i += kRoundBlock) {
        const int job = s_job[i];
        unsigned long long word = s_word[i];
        bool first = true;
        for (int k = 0; k < n; ++k) {
            if (s_job[k] == job) {
                word = max(word, s_word[k]);
                first = first && k >= i;
            }
        }
        if (first) {
            atomicMax(&claim[job], word);
            if (HELD) atomicOr(&held_next[uint32_t(job) >> 5], 1u << (uint32_t(job) & 31u));
        }
    }
}

// Gap positions that are neither granted nor out of candidates.  Every round that
// does not end the process grants at least one of them, so this bounds the rounds
// that can still follow; the host sizes its next batch of launches with it.
__global__ __launch_bounds__(1024) void k_count_open(int lb_cap, const int32_t *__restrict__ plan,
                                                     const int4 *__restrict__ state, int32_t *out)
{
    __shared__ int s_sum[1024 / kWave];
    const int n = min(plan[kPlanListBlocks], lb_cap) * kWave;
    int c = 0;
    for (int i = threadIdx.x; i < n; i += 1024) c += (state[i].w & 3) == 0;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) c += __shfl_xor(c, d, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) s_sum[threadIdx.x / kWave] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int i = 0; i < 1024 / kWave; ++i) t += s_sum[i];
        out[0] = t;
    }
}

// After the last round: the grants themselves.  A granted position still holds
// its winning job and the rank of the winning atom in its state; `ranked` turns
// the rank into the atom.
__global__ void k_grant_finish(int lb_cap, PolicyDev pol, const int32_t *__restrict__ plan,
                               const int4 *__restrict__ state, const int2 *__restrict__ ranked,
                               const int64_t *__restrict__ seg_off,
                               const int2 *__restrict__ atom_dp, const int2 *__restrict__ atom_db,
                               const long long *__restrict__ atom_area,
                               const int32_t *__restrict__ wait, const uint8_t *__restrict__ sla_class,
                               int32_t *grant_job, int32_t *grant_cut, int64_t *grant_score,
                               int32_t *job_gap)
{
    const int slot = blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= min(plan[kPlanListBlocks], lb_cap) * kWave) return;
    const int4 st = state[slot];
    if ((st.w & 3) != 1) return;
    const int g = st.w >> 2, j = st.y;
    const int atom = ranked[st.z].y;
    const int64_t base = seg_off[j];
    const int2 v = atom_dp[base + atom];
    unsigned long long mult, tier;
    job_policy(pol, wait, sla_class, j, mult, tier);
    grant_job[g] = j;
    grant_cut[g] = atom_db[base + atom].y;
    const unsigned long long F = atom_area ? (unsigned long long)atom_area[base + atom]
                                           : (unsigned long long)v.x * (unsigned long long)v.y;
    grant_score[g] = int64_t(F * mult);
    job_gap[j] = g;
}

}  // namespace sja
