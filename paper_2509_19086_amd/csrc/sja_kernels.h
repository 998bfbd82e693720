// Device kernels (gfx950, wave64) for the four steps of a scheduling tick.
// Integer-only; no matrix cores: nothing here is a dense contraction.
#pragma once

#include "sja_internal.h"

namespace sja {

// --------------------------------------------------------------------------
// wave64 helpers
// --------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ unsigned long long lanes_below(int lane)
{
    return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// Lane i receives lane i - n of its row of 16 (n = 1, 2, 4, 8), or lane 15 of the
// row before it (rows 1 and 3) / lane 31 (rows 2 and 3); lanes with no source
// keep `identity`.  These run in the vector ALU's own data path (DPP), not
// through the LDS crossbar as a shuffle does.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_from(int identity, int v)
{
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;
constexpr int kDppWaveShr1 = 0x138;       // lane i receives lane i - 1 across the whole wave; lane 0 keeps `identity`

// Inclusive scans over the 64 lanes of a wave: four shifts inside each row of
// 16, then the row totals handed on to the rows after them.
__device__ __forceinline__ int wave_scan_add(int v)
{
    v += dpp_from<kDppRowShr1, 0xf>(0, v);
    v += dpp_from<kDppRowShr2, 0xf>(0, v);
    v += dpp_from<kDppRowShr4, 0xf>(0, v);
    v += dpp_from<kDppRowShr8, 0xf>(0, v);
    v += dpp_from<kDppRowBcast15, 0xa>(0, v);
    v += dpp_from<kDppRowBcast31, 0xc>(0, v);
    return v;
}

__device__ __forceinline__ int wave_scan_max_dpp(int v)
{
    v = max(v, dpp_from<kDppRowShr1, 0xf>(INT32_MIN, v));
    v = max(v, dpp_from<kDppRowShr2, 0xf>(INT32_MIN, v));
    v = max(v, dpp_from<kDppRowShr4, 0xf>(INT32_MIN, v));
    v = max(v, dpp_from<kDppRowShr8, 0xf>(INT32_MIN, v));
    v = max(v, dpp_from<kDppRowBcast15, 0xa>(INT32_MIN, v));
    v = max(v, dpp_from<kDppRowBcast31, 0xc>(INT32_MIN, v));
    return v;
}

// The smallest value over all 64 lanes (which must all be active), the same in
// every lane: the scan's last lane holds it.
__device__ __forceinline__ int wave_min_dpp(int v)
{
    v = min(v, dpp_from<kDppRowShr1, 0xf>(INT32_MAX, v));
    v = min(v, dpp_from<kDppRowShr2, 0xf>(INT32_MAX, v));
    v = min(v, dpp_from<kDppRowShr4, 0xf>(INT32_MAX, v));
    v = min(v, dpp_from<kDppRowShr8, 0xf>(INT32_MAX, v));
    v = min(v, dpp_from<kDppRowBcast15, 0xa>(INT32_MAX, v));
    v = min(v, dpp_from<kDppRowBcast31, 0xc>(INT32_MAX, v));
    return __builtin_amdgcn_readlane(v, kWave - 1);
}

// Lane `src`'s value, `src` the same in every lane: read from the registers
// (v_readlane), not sent through the LDS crossbar as a shuffle is.
__device__ __forceinline__ int lane_value(int v, int src)
{
    return __builtin_amdgcn_readlane(v, src);
}
__device__ __forceinline__ long long lane_value(long long v, int src)
{
    const unsigned int lo = uint32_t(__builtin_amdgcn_readlane(int(uint32_t((unsigned long long)v)), src));
    const unsigned int hi = uint32_t(__builtin_amdgcn_readlane(int(uint32_t((unsigned long long)v >> 32)), src));
    return (long long)(((unsigned long long)hi << 32) | lo);
}

// Inclusive wave scan of (sum, max, max) triples.
__device__ __forceinline__ void wave_scan_add_max_max(int &s, int &m, int &l, int lane)
{
    (void)lane;
    s = wave_scan_add(s);
    m = wave_scan_max_dpp(m);
    l = wave_scan_max_dpp(l);
}

// --------------------------------------------------------------------------
// K1  per-job segmented scans from the progress point (Sec. 3.9: evaluate the
// envelope on demand from the job's current state).  One wave per job walks
// the remaining segments 64 at a time with coalesced SoA loads and a carry.
// Besides the caller-visible prefixes it compacts the job's safe boundaries
// ("atoms": running duration, running peak and boundary index at each safe
// cut after the progress point) into the workspace at the job's segment base,
// as (duration, peak) and (duration, boundary) pairs.
// --------------------------------------------------------------------------
// Admission limits applied while the atoms are compacted (Sec. 4.3: bounds on
// a subjob's duration; Sec. 4.4: peak power under a cap, completion by a
// deadline).  Each test is monotone along a job's boundaries, or can only turn
// the answer of a pair into a decline, so an atom that fails one is of no use
// to any gap and is left out; the kernels downstream never see the limits.
struct JobLimits {
    int tau_min;                 // shortest subjob that may be offered, the job's end excepted
    int tau_max;                 // longest subjob that may be offered
    int power_cap;               // bound on the running power peak (with a power trace)
    int now;                     // deadline[j] - now bounds the duration (with deadlines)
    const int32_t *power;        // per segment, or null
    const int32_t *deadline;     // per job, or null
};

// Hysteresis on subdivision (Sec. 3.9, safeguard ii: a shorter fragment is accepted
// only for a minimum gain in slack).  The capacity set of the same section,
// ascending; n_caps = 0 switches the rule off.
constexpr int kMaxCaps = 32;
struct Hysteresis {
    int n_caps;
    int min_gain;
    int cap[kMaxCaps];
};

__device__ __forceinline__ void wave_scan_max(int &q, int lane)
{
    (void)lane;
    q = wave_scan_max_dpp(q);
}

// The rule as a remap of one job's atoms, run by the wave that has just compacted
// them.  A gap's plain answer is its last fitting atom a; with cover(x) = the
// smallest capacity of the set >= x, the rule prefers the longest earlier atom
// whose peak maps to a capacity at least min_gain below cover(P(a)) (any covered
// atom when P(a) itself has no cover).  Peaks ascend along the atoms, so that atom
// is found by a search for the threshold capacity, and it depends on a alone: the
// boundary each atom reports (atom_db[].y) and the F it is scored with (atom_f[])
// are overwritten with those of its target, and every kernel downstream reads
// them as it reads any other atom.  atom_f holds the areas under the envelope on
// entry when f_is_area, and is filled with duration x peak otherwise.
// Chunks go from the job's last atom down and each lane loads its target's values
// before it stores its own, so no atom is read after it was overwritten.
__device__ __forceinline__ void hysteresis_remap(const Hysteresis &h, int lane, int64_t base, int count,
                                                 const int2 *__restrict__ atom_dp, int2 *atom_db,
                                                 long long *atom_f, bool f_is_area)
{
    const int2 *dp = atom_dp + base;
    for (int c0 = ((count - 1) / kWave) * kWave; c0 >= 0; c0 -= kWave) {
        const int a = c0 + lane;
        const bool valid = a < count;
        int src = a;
        if (valid) {
            const int peak = dp[a].y;
            bool covered = false;
            long long room = 0;                          // cover(P(a)) - min_gain
            for (int i = 0; i < h.n_caps; ++i)
                if (!covered && h.cap[i] >= peak) {
                    covered = true;
                    room = (long long)h.cap[i] - h.min_gain;
                }
            bool any = false;
            int thr = 0;                                 // the largest capacity worth moving to
            for (int i = 0; i < h.n_caps; ++i)
                if (!covered || h.cap[i] <= room) {
                    any = true;
                    thr = h.cap[i];
                }
            if (any) {
                int lo = 0, hi = a;                      // atoms [0, lo) have peak <= thr
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (dp[mid].y <= thr) lo = mid + 1;
                    else hi = mid;
                }
                if (lo > 0) src = lo - 1;
            }
        }
        int boundary = 0;
        long long f = 0;
        if (valid) {
            boundary = atom_db[base + src].y;
            if (f_is_area) {
                f = atom_f[base + src];
            } else {
                const int2 v = dp[src];
                f = (long long)((unsigned long long)uint32_t(v.x) * uint32_t(v.y));
            }
        }
        if (valid) {
            atom_db[base + a].y = boundary;
            atom_f[base + a] = f;
        }
    }
}

// After prepare_job / prepare_job_wide of the same wave: make the wave's own atom
// stores visible to its other lanes, then apply the rule.
__device__ __forceinline__ void hysteresis_after_prepare(const Hysteresis &h, int j, int lane, int64_t base,
                                                         const int2 *atom_dp, int2 *atom_db,
                                                         const int32_t *n_atoms, long long *atom_f,
                                                         bool f_is_area)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    const int count = n_atoms[j];
    hysteresis_remap(h, lane, base, count, atom_dp, atom_db, atom_f, f_is_area);
}

// Inclusive wave scan of 64-bit sums.
__device__ __forceinline__ void wave_scan_add64(long long &v, int lane)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const long long o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
}

// One wave walks job j's segments from boundary p to the job's end.  With
// pre_area / atom_area (both or neither) it also keeps the running area under
// the envelope, sum of dur * mem, per segment and per atom.
template <bool LIMITED>
__device__ __forceinline__ void prepare_job(
    const JobLimits &lim, long long *__restrict__ pre_area, long long *__restrict__ atom_area,
    int j, int lane, int64_t base, int L, int p, const int32_t *__restrict__ dur,
    const int32_t *__restrict__ mem, const uint8_t *__restrict__ safe, int32_t *__restrict__ pre_dur,
    int32_t *__restrict__ pre_peak, int32_t *__restrict__ prev_safe,
    int2 *__restrict__ atom_dp, int2 *__restrict__ atom_db, int32_t *__restrict__ n_atoms,
    int2 *__restrict__ first_dp)
{
    int carry_sum = 0, carry_peak = INT32_MIN, carry_last = -1, count = 0;
    int first_d = INT32_MAX, first_p = INT32_MAX;     // the first atom, if there is one
    int d_hi = INT32_MAX, carry_pow = INT32_MIN;
    long long carry_area = 0;
    if (LIMITED) {
        d_hi = lim.tau_max;
        if (lim.deadline) {
            const int64_t room = int64_t(lim.deadline[j]) - lim.now;
            if (room < d_hi) d_hi = room < 0 ? -1 : int(room);
        }
    }
    // the next 64 segments are asked for before the current ones are scanned, so the scans
    // and stores of one step cover the memory trip of the next
    int n_dur = 0, n_mem = 0, n_pow = INT32_MIN;
    uint8_t n_safe = 0;
    auto fetch = [&](int k0) {
        const int k = k0 + lane;
        if (k < L) {
            n_dur = dur[base + k];
            n_mem = mem[base + k];
            n_safe = safe[base + k];
            if (LIMITED && lim.power) n_pow = lim.power[base + k];
        }
    };
    fetch(p);
    for (int k0 = p; k0 < L; k0 += kWave) {
        const int k = k0 + lane;
        const bool valid = k < L;
        int s = 0, m = INT32_MIN, l = -1;
        bool flag = false;
        const int c_pow = n_pow;
        if (valid) {
            s = n_dur;
            m = n_mem;
            flag = (n_safe != 0) || (k + 1 == L);
            l = flag ? k + 1 : -1;
        }
        if (k0 + kWave < L) fetch(k0 + kWave);
        long long ar = 0;
        if (pre_area) {
            ar = valid ? (long long)s * (long long)m : 0ll;
            wave_scan_add64(ar, lane);
            ar += carry_area;
            if (valid) pre_area[base + k] = ar;
            carry_area = lane_value(ar, kWave - 1);
        }
        wave_scan_add_max_max(s, m, l, lane);
        s += carry_sum;
        m = max(m, carry_peak);
        l = max(l, carry_last);
        if (valid) {
            pre_dur[base + k] = s;
            pre_peak[base + k] = m;
            prev_safe[base + k] = l;
        }
        if (LIMITED) {
            bool keep = flag && s <= d_hi && (s >= lim.tau_min || k + 1 == L);
            if (lim.power) {
                int q = valid ? c_pow : INT32_MIN;
                wave_scan_max(q, lane);
                q = max(q, carry_pow);
                keep = keep && q <= lim.power_cap;
                carry_pow = lane_value(q, kWave - 1);
            }
            flag = keep;
        }
        const unsigned long long mask = __ballot(flag);
        if (count == 0 && mask) {
            const int src = __ffsll((long long)mask) - 1;
            first_d = lane_value(s, src);
            first_p = lane_value(m, src);
        }
        if (flag) {
            const int idx = count + __popcll(mask & lanes_below(lane));
            atom_dp[base + idx] = make_int2(s, m);
            atom_db[base + idx] = make_int2(s, k + 1);
            if (atom_area) atom_area[base + idx] = ar;
        }
        count += __popcll(mask);
        carry_sum = lane_value(s, kWave - 1);
        carry_peak = lane_value(m, kWave - 1);
        carry_last = lane_value(l, kWave - 1);
    }
    if (lane == 0) {
        n_atoms[j] = count;
        first_dp[j] = make_int2(first_d, first_p);
    }
}

// The same walk for the plain case (no admission limits, no area score), four
// consecutive segments per lane: 256 segments per step, 16-byte loads and stores,
// a lane-local scan of its four values plus one wave scan of the lane totals.  With
// one segment per lane a step is a memory trip for 64 segments, and the trips,
// not the bytes, bound the kernel.
struct __attribute__((packed, aligned(4))) Int4U {      // a 16-byte group of ints at any 4-byte boundary
    int v[4];
};

__device__ __forceinline__ void prepare_job_wide(
    int j, int lane, int64_t base, int L, int p, const int32_t *__restrict__ dur,
    const int32_t *__restrict__ mem, const uint8_t *__restrict__ safe, int32_t *__restrict__ pre_dur,
    int32_t *__restrict__ pre_peak, int32_t *__restrict__ prev_safe,
    int2 *__restrict__ atom_dp, int2 *__restrict__ atom_db, int32_t *__restrict__ n_atoms,
    int2 *__restrict__ first_dp)
{
    constexpr int PER = 4, STEP = PER * kWave;
    int carry_sum = 0, carry_peak = INT32_MIN, carry_last = -1, count = 0;
    int first_d = INT32_MAX, first_p = INT32_MAX;
    int nd[PER], nm[PER];
    uint32_t nf = 0;
    auto fetch = [&](int k0) {
        const int k = k0 + PER * lane;
        if (k + PER <= L) {
            const Int4U d4 = *reinterpret_cast<const Int4U *>(dur + base + k);
            const Int4U m4 = *reinterpret_cast<const Int4U *>(mem + base + k);
            uint32_t f4;
            __builtin_memcpy(&f4, safe + base + k, 4);
#pragma unroll
            for (int i = 0; i < PER; ++i) { nd[i] = d4.v[i]; nm[i] = m4.v[i]; }
            nf = f4;
        } else {
            nf = 0;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const bool in = k + i < L;
                nd[i] = in ? dur[base + k + i] : 0;
                nm[i] = in ? mem[base + k + i] : INT32_MIN;
                nf |= (in && safe[base + k + i] != 0 ? 1u : 0u) << (8 * i);
            }
        }
    };
    fetch(p);
    for (int k0 = p; k0 < L; k0 += STEP) {
        const int k = k0 + PER * lane;
        int s[PER], m[PER], l[PER];
        bool flag[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const bool valid = k + i < L;
            flag[i] = valid && (((nf >> (8 * i)) & 0xffu) != 0 || k + i + 1 == L);
            s[i] = valid ? nd[i] : 0;
            m[i] = valid ? nm[i] : INT32_MIN;
            l[i] = flag[i] ? k + i + 1 : -1;
        }
        if (k0 + STEP < L) fetch(k0 + STEP);
        // lane-local inclusive scans, then the lanes before this one
#pragma unroll
        for (int i = 1; i < PER; ++i) {
            s[i] += s[i - 1];
            m[i] = max(m[i], m[i - 1]);
            l[i] = max(l[i], l[i - 1]);
        }
        int ts = wave_scan_add(s[PER - 1]), tm = wave_scan_max_dpp(m[PER - 1]), tl = wave_scan_max_dpp(l[PER - 1]);
        const int tot_s = lane_value(ts, kWave - 1), tot_m = lane_value(tm, kWave - 1), tot_l = lane_value(tl, kWave - 1);
        // exclusive over lanes = inclusive of the lane before
        int es = dpp_from<kDppWaveShr1, 0xf>(0, ts), em = dpp_from<kDppWaveShr1, 0xf>(INT32_MIN, tm);
        int el = dpp_from<kDppWaveShr1, 0xf>(-1, tl);
        es += carry_sum;
        em = max(em, carry_peak);
        el = max(el, carry_last);
        int nflag = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            s[i] += es;
            m[i] = max(m[i], em);
            l[i] = max(l[i], el);
            nflag += flag[i] ? 1 : 0;
        }
        if (k + PER <= L) {
            Int4U o;
#pragma unroll
            for (int i = 0; i < PER; ++i) o.v[i] = s[i];
            *reinterpret_cast<Int4U *>(pre_dur + base + k) = o;
#pragma unroll
            for (int i = 0; i < PER; ++i) o.v[i] = m[i];
            *reinterpret_cast<Int4U *>(pre_peak + base + k) = o;
#pragma unroll
            for (int i = 0; i < PER; ++i) o.v[i] = l[i];
            *reinterpret_cast<Int4U *>(prev_safe + base + k) = o;
        } else {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                if (k + i < L) {
                    pre_dur[base + k + i] = s[i];
                    pre_peak[base + k + i] = m[i];
                    prev_safe[base + k + i] = l[i];
                }
            }
        }
        // atoms: the flagged boundaries, compacted in order
        const int incl = wave_scan_add(nflag);
        const int total = lane_value(incl, kWave - 1);
        int idx = count + incl - nflag;
        if (count == 0 && total > 0) {
            // the first atom of the job: the lowest lane with a flag, its first flagged value
            const unsigned long long has = __ballot(nflag > 0);
            const int src = __ffsll((long long)has) - 1;
            int fd = 0, fp = 0;
            bool got = false;
#pragma unroll
            for (int i = 0; i < PER; ++i)
                if (!got && flag[i]) { fd = s[i]; fp = m[i]; got = true; }
            first_d = lane_value(fd, src);
            first_p = lane_value(fp, src);
        }
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (flag[i]) {
                atom_dp[base + idx] = make_int2(s[i], m[i]);
                atom_db[base + idx] = make_int2(s[i], k + i + 1);
                ++idx;
            }
        }
        count += total;
        carry_sum += tot_s;
        carry_peak = max(carry_peak, tot_m);
        carry_last = max(carry_last, tot_l);
    }
    if (lane == 0) {
        n_atoms[j] = count;
        first_dp[j] = make_int2(first_d, first_p);
    }
}

template <bool LIMITED>
__global__ __launch_bounds__(256) void k_prepare(
    JobLimits lim, Hysteresis hyst, long long *__restrict__ pre_area, long long *__restrict__ atom_area, int n_jobs, const int64_t *__restrict__ seg_off, const int32_t *__restrict__ dur,
    const int32_t *__restrict__ mem, const uint8_t *__restrict__ safe,
    const int32_t *__restrict__ progress, int32_t *__restrict__ pre_dur,
    int32_t *__restrict__ pre_peak, int32_t *__restrict__ prev_safe,
    int2 *__restrict__ atom_dp, int2 *__restrict__ atom_db, int32_t *__restrict__ n_atoms,
    int2 *__restrict__ first_dp)
{
    const int lane = lane_id();
    const int j = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (j >= n_jobs) return;
    const int64_t base = seg_off[j];
    const int L = int(seg_off[j + 1] - base);
    int p = progress[j];
    p = p < 0 ? 0 : (p > L ? L : p);
    if (!LIMITED && !pre_area)
        prepare_job_wide(j, lane, base, L, p, dur, mem, safe, pre_dur, pre_peak, prev_safe, atom_dp, atom_db, n_atoms, first_dp);
    else
        prepare_job<LIMITED>(lim, pre_area, pre_area ? atom_area : nullptr, j, lane, base, L, p, dur, mem, safe, pre_dur, pre_peak, prev_safe, atom_dp,
                             atom_db, n_atoms, first_dp);
    if (hyst.n_caps > 0)
        hysteresis_after_prepare(hyst, j, lane, base, atom_dp, atom_db, n_atoms, atom_area, pre_area != nullptr);
}

// --------------------------------------------------------------------------
// Tick advance (Sec. 3.1 / 3.5: the parent resumes from its last completed
// fragment).  A grant counts when the two tables point at each other and the
// cut lies in (progress, L]; anything else is treated as no grant.
// --------------------------------------------------------------------------
__device__ __forceinline__ bool grant_holds(int g, int j, int n_gaps, int n_jobs,
                                            const int64_t *__restrict__ seg_off,
                                            const int32_t *__restrict__ grant_job,
                                            const int32_t *__restrict__ grant_cut,
                                            const int32_t *__restrict__ job_gap,
                                            const int32_t *__restrict__ progress, int &cut_out)
{
    if (g < 0 || g >= n_gaps || j < 0 || j >= n_jobs) return false;
    if (grant_job[g] != j || job_gap[j] != g) return false;
    const int L = int(seg_off[j + 1] - seg_off[j]);
    int p = progress[j];
    p = p < 0 ? 0 : (p > L ? L : p);
    const int c = grant_cut[g];
    cut_out = c;
    return c > p && c <= L;
}

__global__ __launch_bounds__(64) void k_fill_i64(int n, int64_t value, int64_t *__restrict__ out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = value;
}

// The tick's totals over gaps: filled area of the grants (from the running
// duration and peak at the granted boundary, before progress moves), offered
// area, number of grants.  One atomic per block and counter.
__global__ __launch_bounds__(256) void k_advance_gaps(
    int n_gaps, int n_jobs, const int64_t *__restrict__ seg_off, const int32_t *__restrict__ pre_dur,
    const int32_t *__restrict__ pre_peak, const int32_t *__restrict__ W, const int32_t *__restrict__ C,
    const int32_t *__restrict__ grant_job, const int32_t *__restrict__ grant_cut,
    const int32_t *__restrict__ job_gap, const int32_t *__restrict__ progress,
    unsigned long long *__restrict__ metrics)
{
    __shared__ unsigned long long s_sum[3][256 / kWave];
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long filled = 0, offered = 0, grants = 0;
    if (g < n_gaps) {
        const int w = W[g], c = C[g];
        offered = (unsigned long long)(w > 0 ? w : 0) * (unsigned long long)(c > 0 ? c : 0);
        const int j = grant_job[g];
        int cut;
        if (grant_holds(g, j, n_gaps, n_jobs, seg_off, grant_job, grant_cut, job_gap, progress, cut)) {
            const int64_t k = seg_off[j] + cut - 1;
            filled = (unsigned long long)pre_dur[k] * (unsigned long long)pre_peak[k];
            grants = 1;
        }
    }
    for (int d = kWave / 2; d > 0; d >>= 1) {
        filled += __shfl_xor(filled, d, kWave);
        offered += __shfl_xor(offered, d, kWave);
        grants += __shfl_xor(grants, d, kWave);
    }
    const int wave = threadIdx.x / kWave;
    if (lane_id() == 0) {
        s_sum[0][wave] = filled;
        s_sum[1][wave] = offered;
        s_sum[2][wave] = grants;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        unsigned long long t = 0;
        for (int i = 0; i < 256 / kWave; ++i) t += s_sum[threadIdx.x][i];
        if (t) atomicAdd(&metrics[threadIdx.x], t);
    }
}

// Slack-minimising capacity mapping (Sec. 3.9): per granted gap the smallest
// capacity of an ascending set that covers the granted subjob's memory peak.
__global__ __launch_bounds__(256) void k_cover(
    int n_gaps, int n_jobs, const int64_t *__restrict__ seg_off, const int32_t *__restrict__ pre_peak,
    const int32_t *__restrict__ C, const int32_t *__restrict__ grant_job,
    const int32_t *__restrict__ grant_cut, int n_caps, const int32_t *__restrict__ cap_set,
    int32_t *__restrict__ cover, int32_t *__restrict__ slack)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_gaps) return;
    int cov = -1, sl = 0;
    const int j = grant_job[g];
    if (j >= 0 && j < n_jobs) {
        const int64_t base = seg_off[j];
        const int cut = grant_cut[g];
        if (cut >= 1 && cut <= int(seg_off[j + 1] - base)) {
            const int peak = pre_peak[base + cut - 1];
            int lo = 0, hi = n_caps;                  // first capacity >= peak
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (cap_set[mid] < peak) lo = mid + 1; else hi = mid;
            }
            if (lo < n_caps) {
                cov = cap_set[lo];
                sl = C[g] - cov;
            }
        }
    }
    cover[g] = cov;
    slack[g] = sl;
}

// One wave per job: a granted job moves to its cut, stops waiting and has its
// running tables and atoms rebuilt from there; any other unfinished job waits
// wait_step longer.  metrics[3] counts the jobs with nothing left afterwards.
template <bool LIMITED>
__global__ __launch_bounds__(256) void k_advance_jobs(
    JobLimits lim, Hysteresis hyst, long long *__restrict__ pre_area, long long *__restrict__ atom_area, int n_gaps, int n_jobs, const int64_t *__restrict__ seg_off, const int32_t *__restrict__ dur,
    const int32_t *__restrict__ mem, const uint8_t *__restrict__ safe,
    const int32_t *__restrict__ grant_job, const int32_t *__restrict__ grant_cut,
    const int32_t *__restrict__ job_gap, int32_t *__restrict__ progress, int32_t *__restrict__ wait,
    int wait_step, int32_t *__restrict__ pre_dur, int32_t *__restrict__ pre_peak,
    int32_t *__restrict__ prev_safe, int2 *__restrict__ atom_dp, int2 *__restrict__ atom_db,
    int32_t *__restrict__ n_atoms, int2 *__restrict__ first_dp, unsigned long long *__restrict__ metrics)
{
    __shared__ int s_done[256 / kWave];
    const int lane = lane_id();
    const int wave = threadIdx.x / kWave;
    const int j = blockIdx.x * (blockDim.x / kWave) + wave;
    int done = 0;
    if (j < n_jobs) {
        const int64_t base = seg_off[j];
        const int L = int(seg_off[j + 1] - base);
        int p = progress[j];
        int cut;
        // every lane evaluates the same scalars, so the branch is uniform over the wave
        if (grant_holds(job_gap[j], j, n_gaps, n_jobs, seg_off, grant_job, grant_cut, job_gap, progress, cut)) {
            p = cut;
            if (!LIMITED && !pre_area)
                prepare_job_wide(j, lane, base, L, p, dur, mem, safe, pre_dur, pre_peak, prev_safe, atom_dp, atom_db, n_atoms,
                                 first_dp);
            else
                prepare_job<LIMITED>(lim, pre_area, pre_area ? atom_area : nullptr, j, lane, base, L, p, dur, mem, safe, pre_dur, pre_peak, prev_safe,
                                     atom_dp, atom_db, n_atoms, first_dp);
            if (hyst.n_caps > 0)
                hysteresis_after_prepare(hyst, j, lane, base, atom_dp, atom_db, n_atoms, atom_area, pre_area != nullptr);
            if (lane == 0) {
                progress[j] = p;
                if (wait) wait[j] = 0;
            }
        } else if (p < L && wait && lane == 0) {
            const int64_t t = int64_t(wait[j]) + wait_step;
            wait[j] = t > INT32_MAX ? INT32_MAX : int32_t(t);
        }
        done = p >= L;
    }
    if (lane == 0) s_done[wave] = done;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long t = 0;
        for (int i = 0; i < 256 / kWave; ++i) t += s_done[i];
        if (t) atomicAdd(&metrics[3], t);
    }
}

}  // namespace sja

#include "k_fit.h"
#include "k_grant.h"
#include "k_fused.h"

namespace sja {

// --------------------------------------------------------------------------
// Input check (no step of the method): the data-dependent assumptions the
// other kernels make and do not test.  One wave per job; reads stay inside
// [0, n_segments) whatever the offsets say.  Bits as in the header.
// --------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_validate(
    int n_jobs, int64_t n_segments, const int64_t *__restrict__ seg_off, const int32_t *__restrict__ dur,
    const int32_t *__restrict__ mem, const int32_t *__restrict__ progress, bool with_policy, PolicyDev pol,
    const int32_t *__restrict__ wait, const uint8_t *__restrict__ sla_class, uint32_t *__restrict__ problems)
{
    const int lane = lane_id();
    const int j = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (j >= n_jobs) return;
    uint32_t bad = 0;
    const int64_t b = seg_off[j], e = seg_off[j + 1];
    if (b < 0 || e < b || e > n_segments || (j == 0 && b != 0) || (j == n_jobs - 1 && e != n_segments) ||
        e - b > INT32_MAX) {
        bad |= SJA_BAD_OFFSETS;
    } else {
        const int L = int(e - b);
        const int p = progress[j];
        if (p < 0 || p > L) bad |= SJA_BAD_PROGRESS;
        long long sum = 0;
        int peak = 0;
        for (int k = lane; k < L; k += kWave) {
            const int d = dur[b + k], m = mem[b + k];
            if (d < 1) bad |= SJA_BAD_DURATION;
            if (m < 0) bad |= SJA_BAD_MEMORY;
            sum += d > 0 ? d : 0;
            peak = max(peak, m);
        }
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            sum += __shfl_xor(sum, d, kWave);
            peak = max(peak, __shfl_xor(peak, d, kWave));
        }
        if (sum > INT32_MAX) bad |= SJA_BAD_DURATION_SUM;
        if (with_policy) {
            const int cls = sla_class ? sla_class[j] : 0;
            const bool uses_class = pol.policy == SJA_POLICY_SLA || pol.policy == SJA_POLICY_MIXED;
            const bool uses_wait = pol.policy == SJA_POLICY_FAIRNESS || pol.policy == SJA_POLICY_MIXED;
            if (uses_class && cls > 2) bad |= SJA_BAD_CLASS;
            if (uses_wait && wait[j] < 0) bad |= SJA_BAD_WAIT;
            if (!(bad & (SJA_BAD_CLASS | SJA_BAD_WAIT | SJA_BAD_DURATION_SUM))) {
                // no subjob of the job fills more than (whole duration) x (largest memory)
                unsigned long long mult, tier;
                job_policy(pol, wait, sla_class, j, mult, tier);
                const unsigned long long F = (unsigned long long)sum * (unsigned long long)peak;   // < 2^62
                const unsigned long long limit = 1ull << 62;
                if (mult != 0 && F >= (limit + mult - 1) / mult) bad |= SJA_BAD_SCORE_RANGE;
            }
        }
    }
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) bad |= __shfl_xor(int(bad), d, kWave);
    if (lane == 0 && bad) atomicOr(problems, bad);
}

// --------------------------------------------------------------------------
// K3  policy arg-max per gap (Sec. 3.5 phase 3).  Lanes run along jobs and
// walk a chunk of gap positions in the sorted order of the last fit, so a
// job's cut -- and with it F = duration * peak -- rarely changes from one
// position to the next and is kept in registers.  Per gap each wave reduces
// its 64 candidates, waves combine through LDS, and each block leaves one
// partial per (job tile, gap); k_select_reduce finishes the arg-max.
// Key order: hi desc, lo desc, job asc.
// --------------------------------------------------------------------------
__device__ __forceinline__ bool key_better(unsigned long long hi_a, unsigned long long lo_a, int j_a,
                                           unsigned long long hi_b, unsigned long long lo_b, int j_b)
{
    if (hi_a != hi_b) return hi_a > hi_b;
    if (lo_a != lo_b) return lo_a > lo_b;
    return j_a < j_b;
}

// The key of every prefix of every job, ((tier << 62) | F * multiplier) + 1, once
// per call: the stepping kernel below then fetches a finished key where a job's
// cut changes instead of (duration, peak) and three 64-bit multiplies per lane.
// One wave per job; the kernel moves 16 bytes per segment and runs at the rate
// of a copy (a wave running along four neighbouring jobs as one stretch, so that
// the shortest jobs fill it, was no faster).  Prefixes before a job's progress
// hold whatever the prefix arrays hold there; no cut points at them.
template <bool AREA>
__global__ __launch_bounds__(256) void k_select_keys(
    int n_jobs, PolicyDev pol, const int64_t *__restrict__ seg_off, const int32_t *__restrict__ pre_dur,
    const int32_t *__restrict__ pre_peak, const long long *__restrict__ pre_area,
    const int32_t *__restrict__ wait, const uint8_t *__restrict__ sla_class,
    unsigned long long *__restrict__ seg_key)
{
    const int lane = lane_id();
    const int j = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (j >= n_jobs) return;
    const int64_t base = seg_off[j];
    const int L = int(seg_off[j + 1] - base);
    unsigned long long mult, tier;
    job_policy(pol, wait, sla_class, j, mult, tier);
    for (int k = lane; k < L; k += kWave) {
        const unsigned long long F = AREA ? (unsigned long long)pre_area[base + k] : rect_of(pre_dur[base + k], pre_peak[base + k]);
        seg_key[base + k] = ((tier << 62) | times_mult(F, mult)) + 1ull;
    }
}

// Steps reduced together by one wave (see k_select_pass).
constexpr int kSelBatch = 8;

template <bool MIXED>
__global__ __launch_bounds__(kSelBlock) void k_select_pass(
    int n_jobs, int n_gaps, int n_chunks, PolicyDev pol, const int64_t *__restrict__ seg_off,
    const unsigned long long *__restrict__ seg_key, const int32_t *__restrict__ cut, const int32_t *__restrict__ gap_order,
    const int32_t *__restrict__ wait, const uint8_t *__restrict__ sla_class,
    const int32_t *__restrict__ job_held, const uint8_t *__restrict__ gap_active,
    SelPartial *__restrict__ part)
{
    constexpr int WAVES = kSelBlock / kWave;
    constexpr int ROW = kWave + 1;                       // padded: a column read hits distinct banks
    __shared__ unsigned long long s_key[WAVES][kSelBatch][ROW];   // one batch of per-lane keys per wave
    __shared__ unsigned long long s_mult[WAVES][kWave];           // per-lane score multiplier (MIXED ties)
    __shared__ unsigned long long s_hi[WAVES][kSelGapChunk];
    __shared__ int s_job[WAVES][kSelGapChunk];

    const int xcd = blockIdx.x & 7;
    const int k = blockIdx.x >> 3;
    const int job_tile = (k / n_chunks) * 8 + xcd;
    const int chunk = k % n_chunks;
    if (job_tile * kSelBlock >= n_jobs) return;
    const int j = job_tile * kSelBlock + threadIdx.x;
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    const int wave_job0 = job_tile * kSelBlock + wave * kWave;

    bool usable = j < n_jobs;
    int64_t base = 0;
    unsigned long long mult = 1, tier = 0;
    if (usable) {
        if (job_held && job_held[j] >= 0) usable = false;
        base = seg_off[j];
        if (MIXED) job_policy(pol, wait, sla_class, j, mult, tier);    // the multiplier, for ties only
    }
    s_mult[wave][lane] = mult;

    const int s_begin = chunk * kSelGapChunk;
    const int s_end = min(n_gaps, s_begin + kSelGapChunk);
    int last_cut = -1;
    unsigned long long hi = 0;
    // secondary score of a key (MIXED: F = score / multiplier), only needed to break ties
    auto second = [&](unsigned long long key, int src) -> unsigned long long {
        return MIXED ? ((key - 1ull) & ((1ull << 62) - 1ull)) / s_mult[wave][src] : 0ull;
    };
    // the cuts of one batch of steps (cut rows are read coalesced)
    auto load_cuts = [&](int s0, int (&out)[kSelBatch]) {
        const int n_step = min(kSelBatch, s_end - s0);
#pragma unroll
        for (int t = 0; t < kSelBatch; ++t) {
            out[t] = -1;
            if (t < n_step && usable) {
                const int g = gap_order[s0 + t];
                if (!gap_active || gap_active[g]) out[t] = cut[int64_t(g) * n_jobs + j];
            }
        }
    };
    int cv_next[kSelBatch];
    load_cuts(s_begin, cv_next);
    for (int s0 = s_begin; s0 < s_end; s0 += kSelBatch) {
        const int n_step = min(kSelBatch, s_end - s0);
        // phase 1: every lane's key for each step of the batch
        int cv[kSelBatch];
#pragma unroll
        for (int t = 0; t < kSelBatch; ++t) cv[t] = cv_next[t];
        // a job's cut rarely changes from one sorted position to the next: only the changes
        // gather the prefix's key, all of a batch's gathers in flight together
        unsigned long long kv[kSelBatch];
        bool fresh[kSelBatch];
        int prev = last_cut;
#pragma unroll
        for (int t = 0; t < kSelBatch; ++t) {
            const int c = cv[t];
            fresh[t] = c >= 0 && c != prev;
            if (fresh[t]) kv[t] = seg_key[base + c - 1];
            prev = c >= 0 ? c : prev;
        }
        last_cut = prev;
        // the next batch's cuts travel together with this batch's gathers
        if (s0 + kSelBatch < s_end) load_cuts(s0 + kSelBatch, cv_next);
#pragma unroll
        for (int t = 0; t < kSelBatch; ++t) {
            if (fresh[t]) hi = kv[t];
            s_key[wave][t][lane] = cv[t] >= 0 ? hi : 0ull;
        }
        // the keys just written are read by other lanes of this wave: order the two
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // phase 2: lane l reduces step (l % 16) over lanes [16 * (l / 16), +16), then the four
        // quarter results of a step are combined across lanes l, l+16, l+32, l+48
        const int t = lane & (kSelBatch - 1), q = lane / kSelBatch;
        unsigned long long bh = 0;
        int bsrc = kWave;
#pragma unroll
        for (int i = 0; i < kSelBatch; ++i) {
            const int src = q * kSelBatch + i;
            const unsigned long long oh = s_key[wave][t][src];
            bool better = oh > bh;
            if (MIXED && oh == bh && oh != 0) better = second(oh, src) > second(bh, bsrc);
            if (better) { bh = oh; bsrc = src; }     // equal keys keep the lower lane = lower job id
        }
#pragma unroll
        for (int d = kSelBatch; d < kWave; d <<= 1) {
            const unsigned long long oh = __shfl_xor(bh, d, kWave);
            const int osrc = __shfl_xor(bsrc, d, kWave);
            bool better = oh > bh || (oh == bh && osrc < bsrc);
            if (MIXED && oh == bh && oh != 0) {
                const unsigned long long fo = second(oh, osrc), fb = second(bh, bsrc);
                better = fo > fb || (fo == fb && osrc < bsrc);
            }
            if (better) { bh = oh; bsrc = osrc; }
        }
        // the winner's secondary score is a 64-bit division: it is left to the end, where it is
        // needed once per position (and per tie between waves), not once per wave and batch
        if (lane < n_step) {
            const int slot = s0 - s_begin + lane;
            s_hi[wave][slot] = bh; s_job[wave][slot] = bh ? wave_job0 + bsrc : INT32_MAX;
        }
    }
    __syncthreads();
    // secondary score of wave w's winner (its multiplier sits in that wave's row of s_mult)
    auto second_of = [&](unsigned long long key, int w, int job) -> unsigned long long {
        return MIXED ? ((key - 1ull) & ((1ull << 62) - 1ull)) / s_mult[w][job - (job_tile * kSelBlock + w * kWave)] : 0ull;
    };
    for (int slot = threadIdx.x; slot < s_end - s_begin; slot += kSelBlock) {
        unsigned long long bh = s_hi[0][slot];
        int bj = bh ? s_job[0][slot] : INT32_MAX, bw = 0;
#pragma unroll
        for (int w = 1; w < WAVES; ++w) {
            const unsigned long long oh = s_hi[w][slot];
            const int oj = oh ? s_job[w][slot] : INT32_MAX;
            bool better = oh > bh;
            // equal keys: the larger secondary score, then the lower job, which is the earlier wave's
            if (MIXED && oh == bh && oh != 0) better = second_of(oh, w, oj) > second_of(bh, bw, bj);
            if (better) { bh = oh; bj = oj; bw = w; }
        }
        const unsigned long long bl = (MIXED && bh) ? second_of(bh, bw, bj) : 0ull;
        const int g = gap_order[s_begin + slot];
        // the winner's cut, fetched here for all of the block's positions at once (inside the
        // stepping loop it would be one more memory trip per batch)
        const int bc = bh ? cut[int64_t(g) * n_jobs + bj] : -1;
        SelPartial out;
        out.hi = bh; out.lo = bl; out.job = bh ? bj : -1; out.cut = bh ? bc : -1; out.pad = 0;
        part[int64_t(job_tile) * n_gaps + g] = out;
    }
}

__global__ void k_select_reduce(int n_gaps, int n_job_tiles, const SelPartial *__restrict__ part,
                                int32_t *__restrict__ cand_job, int32_t *__restrict__ cand_cut,
                                int64_t *__restrict__ cand_score)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= n_gaps) return;
    unsigned long long bh = 0, bl = 0;
    int bj = INT32_MAX, bc = -1;
    for (int t = 0; t < n_job_tiles; ++t) {
        const SelPartial p = part[int64_t(t) * n_gaps + g];
        const int pj = p.hi ? p.job : INT32_MAX;
        if (key_better(p.hi, p.lo, pj, bh, bl, bj)) { bh = p.hi; bl = p.lo; bj = pj; bc = p.cut; }
    }
    cand_job[g] = bh ? bj : -1;
    cand_cut[g] = bh ? bc : -1;
    cand_score[g] = bh ? int64_t((bh - 1ull) & ((1ull << 62) - 1ull)) : 0;
}

// --------------------------------------------------------------------------
// K4  conflict rounds.  A round is: select over the still-active gaps with
// the held jobs masked (kernels above), k_claim (each candidate job records
// the lowest-index gap that named it, stamped with the round so that no reset
// is needed), k_commit (winners become grants, losers stay active).
// --------------------------------------------------------------------------
__global__ void k_resolve_init(int n_gaps, int n_jobs, int32_t *grant_job, int32_t *grant_cut,
                               int64_t *grant_score, int32_t *job_gap, uint8_t *active,
                               unsigned long long *claim)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_gaps) { grant_job[i] = -1; grant_cut[i] = -1; grant_score[i] = 0; active[i] = 1; }
    if (i < n_jobs) { job_gap[i] = -1; claim[i] = 0ull; }
}

__device__ __forceinline__ unsigned long long claim_word(int round, int g)
{
    return (static_cast<unsigned long long>(round) << 32) | (0xffffffffu - uint32_t(g));
}

__global__ void k_claim(int n_gaps, int round, const uint8_t *__restrict__ active,
                        const int32_t *__restrict__ cand_job, unsigned long long *claim,
                        int32_t *counters)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g == 0) { counters[0] = 0; counters[1] = 0; }
    if (g >= n_gaps || !active[g]) return;
    const int j = cand_job[g];
    if (j >= 0) atomicMax(&claim[j], claim_word(round, g));
}

__global__ void k_commit(int n_gaps, int round, uint8_t *active, const int32_t *__restrict__ cand_job,
                         const int32_t *__restrict__ cand_cut, const int64_t *__restrict__ cand_score,
                         const unsigned long long *__restrict__ claim, int32_t *grant_job,
                         int32_t *grant_cut, int64_t *grant_score, int32_t *job_gap,
                         int32_t *counters)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    bool cand = false, lost = false;
    if (g < n_gaps && active[g]) {
        const int j = cand_job[g];
        if (j >= 0) {
            cand = true;
            if (claim[j] == claim_word(round, g)) {
                grant_job[g] = j;
                grant_cut[g] = cand_cut[g];
                grant_score[g] = cand_score[g];
                job_gap[j] = g;
                active[g] = 0;
            } else {
                lost = true;
            }
        }
    }
    const unsigned long long mc = __ballot(cand), ml = __ballot(lost);
    if (lane_id() == 0) {
        if (mc) atomicAdd(&counters[0], __popcll(mc));
        if (ml) atomicAdd(&counters[1], __popcll(ml));
    }
}

}  // namespace sja
