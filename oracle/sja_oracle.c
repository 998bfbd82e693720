/*
 * TEST INFRASTRUCTURE -- plain CPU oracle for batched gap-job fit evaluation
 * and slot grant (Scheduler-Driven Job Atomization).
 *
 * This file is the slow, obviously-correct statement of what the GPU library
 * computes.  It shares no code, header, table or helper with the GPU path and
 * is only ever called from the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg.  Nothing in the product may link or call it.
 *
 * Model (integer realisation of the paper's definitions):
 *   - A job's profile is a piecewise-constant envelope U(t) (Sec. 3.9): segment
 *     k of job j lasts dur[k] >= 1 ticks at mem[k] MiB.  Boundary b lies before
 *     segment b; boundary L is the job's end.  safe[k] flags boundary k+1 as a
 *     subjob boundary (Sec. 3.7); the end is always one, whatever its flag.
 *   - A subjob is the run of segments [p, cut) starting at the job's progress
 *     point p (Sec. 3.1, 3.5: the parent resumes from the last completed
 *     fragment).  For an offered gap (W, C) (Sec. 3.5: time interval plus slice
 *     capacity) it is admissible when its duration is <= W and max U over it is
 *     <= C (Sec. 3.8 admissibility, in the envelope form of Sec. 3.9).
 *   - The job answers with the longest admissible subjob ending on a safe
 *     boundary (Sec. 3.9: prefer longer fragments), or declines (cut = -1).
 *   - The scheduler picks one interested job per gap by policy (Sec. 3.5, 4.2)
 *     and conflicts are settled in rounds so that a job holds at most one gap.
 *   - Between ticks a granted job moves its progress point to the granted
 *     boundary, the others wait longer (sjo_advance; pinned against a brute
 *     force over the raw segments and the invariants of a chain of ticks).
 *
 * All sums and products are int64; a product that would overflow int64 makes
 * the call return SJO_ERR_OVERFLOW.  The outer loops over gaps may be split
 * over host threads (rows are independent); the per-pair code is the plain
 * definition.
 *
 * Pins (tests, CPU only): library routines (cumsum / running max /
 * searchsorted), closed forms for constant profiles, a from-scratch brute
 * force in another language on tiny inputs, and the fit / grant invariants.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SJO_OK 0
#define SJO_ERR_ARG (-1)
#define SJO_ERR_OVERFLOW (-2)
#define SJO_ERR_NOMEM (-3)

enum { SJO_EFFICIENCY = 0, SJO_FAIRNESS = 1, SJO_SLA = 2, SJO_MIXED = 3 };

typedef struct {
    int32_t policy;
    int32_t wait_scale;      /* fairness: score = F * (wait_scale + wait)      */
    int32_t sla_weight[3];   /* SLA: score = F * sla_weight[class]             */
    int32_t class0_override; /* SLA: any class-0 job beats every other class   */
    int32_t max_rounds;      /* resolve: 0 = until stable                      */
} sjo_params;

int sjo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void sjo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------
 * Prepare: for each job, from its progress point p, the running duration
 * D(b) = sum dur[p..b-1], running peak P(b) = max mem[p..b-1] and the last
 * safe boundary in (p, b], for b = p+1..L, stored at entry k = b-1.
 * Entries before the progress point are left untouched.
 * ---------------------------------------------------------------------- */
int sjo_prepare(int32_t n_jobs, const int64_t *seg_off, const int32_t *dur,
                const int32_t *mem, const uint8_t *safe, const int32_t *progress,
                int64_t *pre_dur, int64_t *pre_peak, int32_t *prev_safe)
{
    if (n_jobs < 0) return SJO_ERR_ARG;
    for (int32_t j = 0; j < n_jobs; ++j) {
        int64_t base = seg_off[j];
        int64_t L = seg_off[j + 1] - base;
        int64_t p = progress[j];
        if (L < 0 || p < 0 || p > L) return SJO_ERR_ARG;
        int64_t sum = 0, peak = 0;
        int32_t last = -1;
        for (int64_t b = p + 1; b <= L; ++b) {
            int64_t k = base + b - 1;
            sum += dur[k];
            if (b == p + 1 || mem[k] > peak) peak = mem[k];
            if (b == L || safe[k]) last = (int32_t)b;
            pre_dur[k] = sum;
            pre_peak[k] = peak;
            prev_safe[k] = last;
        }
    }
    return SJO_OK;
}

/* ------------------------------------------------------------------------
 * Area under the envelope from the progress point: pre_area[k] = sum over
 * segments p..k of dur * mem, the memory-time a subjob ending after segment k
 * really uses (the alternative reading of "filled capacity-time"; the default
 * is the rectangle duration * peak).
 * ---------------------------------------------------------------------- */
int sjo_area(int32_t n_jobs, const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
             const int32_t *progress, int64_t *pre_area)
{
    if (n_jobs < 0) return SJO_ERR_ARG;
    for (int32_t j = 0; j < n_jobs; ++j) {
        int64_t base = seg_off[j];
        int64_t L = seg_off[j + 1] - base;
        int64_t p = progress[j];
        if (L < 0 || p < 0 || p > L) return SJO_ERR_ARG;
        int64_t area = 0;
        for (int64_t k = base + p; k < base + L; ++k) {
            int64_t term;
            if (__builtin_mul_overflow((int64_t)dur[k], (int64_t)mem[k], &term) ||
                __builtin_add_overflow(area, term, &area)) return SJO_ERR_OVERFLOW;
            pre_area[k] = area;
        }
    }
    return SJO_OK;
}

/* ------------------------------------------------------------------------
 * Optional admission limits on top of the gap's own window and capacity:
 *   - a power trace with a cap in force for the tick: the subjob's peak power
 *     must stay <= power_cap (Sec. 4.4, energy-aware admission: the same
 *     max-over-the-window test on a second channel);
 *   - a deadline per job: the subjob has to complete by it, i.e. its duration
 *     is <= deadline[j] - now, the gaps of a tick starting at `now`
 *     (Sec. 4.4, deadline-aware admission);
 *   - framework-level bounds on a subjob's duration (Sec. 4.3, granularity):
 *     at most tau_max, and at least tau_min unless the subjob runs to the
 *     job's end (a job's tail must be allowed to finish).
 * A NULL limits pointer, a NULL power trace or a NULL deadline array switches
 * the corresponding tests off.
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t tau_min;   /* >= 0 */
    int32_t tau_max;   /* >= 0 */
    int32_t power_cap;
    int32_t now;
} sjo_limits;

/* ------------------------------------------------------------------------
 * Fit for one (gap, job) pair: walk boundaries forward from the progress
 * point while the subjob still fits, remembering the last safe boundary that
 * may be offered.  The running duration and the running peaks never decrease,
 * so the first violation of an upper bound ends the walk.  Returns the cut (or
 * -1) and, for an interested pair, the subjob's duration and memory peak.
 * ---------------------------------------------------------------------- */
static int32_t fit_pair(int64_t L, int64_t p, const int32_t *dur, const int32_t *mem,
                        const uint8_t *safe, int64_t W, int64_t C, const sjo_limits *lim,
                        const int32_t *power, const int32_t *deadline_j,
                        int64_t *out_dur, int64_t *out_peak)
{
    int64_t sum = 0, peak = 0, ppeak = 0;
    int32_t cut = -1;
    int64_t cut_dur = 0, cut_peak = 0;
    for (int64_t b = p + 1; b <= L; ++b) {
        int64_t k = b - 1;
        sum += dur[k];
        if (b == p + 1 || mem[k] > peak) peak = mem[k];
        if (power && (b == p + 1 || power[k] > ppeak)) ppeak = power[k];
        if (sum > W || peak > C) break;
        if (lim) {
            if (sum > lim->tau_max) break;
            if (power && ppeak > lim->power_cap) break;
            if (deadline_j && sum > (int64_t)*deadline_j - lim->now) break;
        }
        if (b == L || safe[k]) {
            if (lim && b != L && sum < lim->tau_min) continue;
            cut = (int32_t)b;
            cut_dur = sum;
            cut_peak = peak;
        }
    }
    if (out_dur) *out_dur = cut_dur;
    if (out_peak) *out_peak = cut_peak;
    return cut;
}

/* cut[g*J + j] for every pair; interest_bits (may be NULL) holds bit j%32 of
 * word g*ceil(J/32) + j/32 set iff the job is interested in the gap. */
int sjo_fit_limited(int32_t n_gaps, int32_t n_jobs, const int64_t *seg_off, const int32_t *dur,
                    const int32_t *mem, const uint8_t *safe, const int32_t *progress,
                    const int32_t *W, const int32_t *C, const sjo_limits *lim, const int32_t *power,
                    const int32_t *deadline, int32_t *cut, uint32_t *interest_bits)
{
    if (n_gaps < 0 || n_jobs < 0) return SJO_ERR_ARG;
    if (lim && (lim->tau_min < 0 || lim->tau_max < 0)) return SJO_ERR_ARG;
    int64_t words = ((int64_t)n_jobs + 31) / 32;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t g = 0; g < n_gaps; ++g) {
        int32_t *row = cut + (int64_t)g * n_jobs;
        uint32_t *bits = interest_bits ? interest_bits + (int64_t)g * words : NULL;
        if (bits) memset(bits, 0, (size_t)words * sizeof(uint32_t));
        for (int32_t j = 0; j < n_jobs; ++j) {
            int64_t base = seg_off[j];
            int64_t L = seg_off[j + 1] - base;
            int32_t c = fit_pair(L, progress[j], dur + base, mem + base, safe + base,
                                 W[g], C[g], lim, power ? power + base : NULL,
                                 deadline ? deadline + j : NULL, NULL, NULL);
            row[j] = c;
            if (bits && c >= 0) bits[j >> 5] |= (uint32_t)1 << (j & 31);
        }
    }
    return SJO_OK;
}

int sjo_fit(int32_t n_gaps, int32_t n_jobs, const int64_t *seg_off, const int32_t *dur,
            const int32_t *mem, const uint8_t *safe, const int32_t *progress,
            const int32_t *W, const int32_t *C, int32_t *cut, uint32_t *interest_bits)
{
    return sjo_fit_limited(n_gaps, n_jobs, seg_off, dur, mem, safe, progress, W, C, NULL, NULL, NULL,
                           cut, interest_bits);
}

/* The same evaluation on a list of sampled pairs (gap_idx[i], job_idx[i]). */
int sjo_fit_pairs_limited(int64_t n_pairs, const int32_t *gap_idx, const int32_t *job_idx,
                          const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                          const uint8_t *safe, const int32_t *progress, const int32_t *W,
                          const int32_t *C, const sjo_limits *lim, const int32_t *power,
                          const int32_t *deadline, int32_t *cut, int64_t *sub_dur, int64_t *sub_peak)
{
    if (n_pairs < 0) return SJO_ERR_ARG;
    if (lim && (lim->tau_min < 0 || lim->tau_max < 0)) return SJO_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_pairs; ++i) {
        int32_t g = gap_idx[i], j = job_idx[i];
        int64_t base = seg_off[j];
        int64_t L = seg_off[j + 1] - base;
        int64_t d = 0, pk = 0;
        cut[i] = fit_pair(L, progress[j], dur + base, mem + base, safe + base,
                          W[g], C[g], lim, power ? power + base : NULL,
                          deadline ? deadline + j : NULL, &d, &pk);
        if (sub_dur) sub_dur[i] = d;
        if (sub_peak) sub_peak[i] = pk;
    }
    return SJO_OK;
}

int sjo_fit_pairs(int64_t n_pairs, const int32_t *gap_idx, const int32_t *job_idx,
                  const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                  const uint8_t *safe, const int32_t *progress, const int32_t *W,
                  const int32_t *C, int32_t *cut, int64_t *sub_dur, int64_t *sub_peak)
{
    return sjo_fit_pairs_limited(n_pairs, gap_idx, job_idx, seg_off, dur, mem, safe, progress, W, C,
                                 NULL, NULL, NULL, cut, sub_dur, sub_peak);
}

/* ------------------------------------------------------------------------
 * Hysteresis on subdivision (Sec. 3.9, safeguard ii): a job prefers its longest
 * fitting fragment and accepts a shorter one only for a minimum gain in slack.
 * The paper names the rule and gives no formula; the reading taken here:
 *   - cover(x) = the smallest capacity of the set (ascending) that is >= x,
 *     +infinity if there is none (the mapping of the same section);
 *   - b* = the cut of the fit without hysteresis (limits included), the longest
 *     fragment the pair admits; a pair without one stays a decline;
 *   - a boundary b with p < b < b* that may be offered (safe, and not shorter
 *     than tau_min under limits; every upper bound holds for it because it
 *     holds for b* and the running sums and peaks never decrease) is "worth
 *     the subdivision" if cover(P(b)) is finite and lies at least min_gain below
 *     cover(P(b*)) (any finite cover counts when cover(P(b*)) is infinite);
 *   - the cut is the longest boundary worth the subdivision, b* if none is.
 * min_gain >= 1; an empty set (n_caps = 0) switches the rule off.
 * ---------------------------------------------------------------------- */
#define SJO_NO_COVER INT64_MAX

static int64_t cover_of(int64_t x, int32_t n_caps, const int32_t *cap_set)
{
    for (int32_t i = 0; i < n_caps; ++i)
        if (cap_set[i] >= x) return cap_set[i];
    return SJO_NO_COVER;
}

static int32_t fit_pair_hysteresis(int64_t L, int64_t p, const int32_t *dur, const int32_t *mem,
                                   const uint8_t *safe, int64_t W, int64_t C, const sjo_limits *lim,
                                   const int32_t *power, const int32_t *deadline_j, int32_t n_caps,
                                   const int32_t *cap_set, int64_t min_gain,
                                   int64_t *out_dur, int64_t *out_peak)
{
    int64_t d_star = 0, p_star = 0;
    int32_t b_star = fit_pair(L, p, dur, mem, safe, W, C, lim, power, deadline_j, &d_star, &p_star);
    int32_t cut = b_star;
    int64_t cut_dur = d_star, cut_peak = p_star;
    if (b_star >= 0 && n_caps > 0) {
        int64_t cov_star = cover_of(p_star, n_caps, cap_set);
        int64_t sum = 0, peak = 0;
        for (int64_t b = p + 1; b < b_star; ++b) {
            int64_t k = b - 1;
            sum += dur[k];
            if (b == p + 1 || mem[k] > peak) peak = mem[k];
            if (!safe[k]) continue;
            if (lim && sum < lim->tau_min) continue;
            int64_t cov = cover_of(peak, n_caps, cap_set);
            if (cov == SJO_NO_COVER) continue;
            if (cov_star != SJO_NO_COVER && cov_star - cov < min_gain) continue;
            cut = (int32_t)b;
            cut_dur = sum;
            cut_peak = peak;
        }
    }
    if (out_dur) *out_dur = cut_dur;
    if (out_peak) *out_peak = cut_peak;
    return cut;
}

static int hysteresis_args_ok(int32_t n_caps, const int32_t *cap_set, int32_t min_gain)
{
    if (n_caps < 0 || (n_caps > 0 && (!cap_set || min_gain < 1))) return 0;
    for (int32_t i = 1; i < n_caps; ++i)
        if (cap_set[i] < cap_set[i - 1]) return 0;
    return 1;
}

/* The cut matrix and interest bits of sjo_fit_limited under the hysteresis rule
 * (lim, power, deadline may be NULL as there). */
int sjo_fit_hysteresis(int32_t n_gaps, int32_t n_jobs, const int64_t *seg_off, const int32_t *dur,
                       const int32_t *mem, const uint8_t *safe, const int32_t *progress,
                       const int32_t *W, const int32_t *C, const sjo_limits *lim, const int32_t *power,
                       const int32_t *deadline, int32_t n_caps, const int32_t *cap_set, int32_t min_gain,
                       int32_t *cut, uint32_t *interest_bits)
{
    if (n_gaps < 0 || n_jobs < 0) return SJO_ERR_ARG;
    if (lim && (lim->tau_min < 0 || lim->tau_max < 0)) return SJO_ERR_ARG;
    if (!hysteresis_args_ok(n_caps, cap_set, min_gain)) return SJO_ERR_ARG;
    int64_t words = ((int64_t)n_jobs + 31) / 32;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t g = 0; g < n_gaps; ++g) {
        int32_t *row = cut + (int64_t)g * n_jobs;
        uint32_t *bits = interest_bits ? interest_bits + (int64_t)g * words : NULL;
        if (bits) memset(bits, 0, (size_t)words * sizeof(uint32_t));
        for (int32_t j = 0; j < n_jobs; ++j) {
            int64_t base = seg_off[j];
            int64_t L = seg_off[j + 1] - base;
            int32_t c = fit_pair_hysteresis(L, progress[j], dur + base, mem + base, safe + base,
                                            W[g], C[g], lim, power ? power + base : NULL,
                                            deadline ? deadline + j : NULL, n_caps, cap_set, min_gain,
                                            NULL, NULL);
            row[j] = c;
            if (bits && c >= 0) bits[j >> 5] |= (uint32_t)1 << (j & 31);
        }
    }
    return SJO_OK;
}

/* The same on sampled pairs, with the chosen subjob's duration and peak. */
int sjo_fit_pairs_hysteresis(int64_t n_pairs, const int32_t *gap_idx, const int32_t *job_idx,
                             const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                             const uint8_t *safe, const int32_t *progress, const int32_t *W,
                             const int32_t *C, const sjo_limits *lim, const int32_t *power,
                             const int32_t *deadline, int32_t n_caps, const int32_t *cap_set,
                             int32_t min_gain, int32_t *cut, int64_t *sub_dur, int64_t *sub_peak)
{
    if (n_pairs < 0) return SJO_ERR_ARG;
    if (lim && (lim->tau_min < 0 || lim->tau_max < 0)) return SJO_ERR_ARG;
    if (!hysteresis_args_ok(n_caps, cap_set, min_gain)) return SJO_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_pairs; ++i) {
        int32_t g = gap_idx[i], j = job_idx[i];
        int64_t base = seg_off[j];
        int64_t L = seg_off[j + 1] - base;
        int64_t d = 0, pk = 0;
        cut[i] = fit_pair_hysteresis(L, progress[j], dur + base, mem + base, safe + base, W[g], C[g],
                                     lim, power ? power + base : NULL, deadline ? deadline + j : NULL,
                                     n_caps, cap_set, min_gain, &d, &pk);
        if (sub_dur) sub_dur[i] = d;
        if (sub_peak) sub_peak[i] = pk;
    }
    return SJO_OK;
}

/* ------------------------------------------------------------------------
 * Slack-minimising capacity mapping (Sec. 3.9): for each granted gap, the
 * smallest capacity of the set (ascending, n_caps entries) that covers the
 * granted subjob's memory peak, and the slack left against the gap's own
 * capacity.  cover = -1 and slack = 0 for an ungranted gap; cover = -1 and
 * slack = 0 too when no capacity of the set covers the peak.
 * ---------------------------------------------------------------------- */
int sjo_cover(int32_t n_gaps, const int64_t *seg_off, const int64_t *pre_peak, const int32_t *C,
              const int32_t *grant_job, const int32_t *grant_cut, int32_t n_caps,
              const int32_t *cap_set, int32_t *cover, int32_t *slack)
{
    if (n_gaps < 0 || n_caps < 0) return SJO_ERR_ARG;
    for (int32_t i = 1; i < n_caps; ++i)
        if (cap_set[i] < cap_set[i - 1]) return SJO_ERR_ARG;
    for (int32_t g = 0; g < n_gaps; ++g) {
        cover[g] = -1;
        slack[g] = 0;
        int32_t j = grant_job[g];
        if (j < 0) continue;
        int64_t peak = pre_peak[seg_off[j] + grant_cut[g] - 1];
        for (int32_t i = 0; i < n_caps; ++i) {
            if (cap_set[i] >= peak) {
                cover[g] = cap_set[i];
                slack[g] = C[g] - cap_set[i];
                break;
            }
        }
    }
    return SJO_OK;
}

/* ------------------------------------------------------------------------
 * Policy key of an interested pair.  F = duration * peak of the subjob (the
 * capacity-time rectangle it fills).  Larger key wins; equal keys go to the
 * lower job id.  The reported score is the key's primary score term.
 * ---------------------------------------------------------------------- */
typedef struct { int64_t k0, k1, k2; } sjo_key;

static int key_greater(const sjo_key *a, const sjo_key *b)
{
    if (a->k0 != b->k0) return a->k0 > b->k0;
    if (a->k1 != b->k1) return a->k1 > b->k1;
    return a->k2 > b->k2;
}

static int make_key(const sjo_params *pp, int64_t F, int64_t wait, int32_t cls, sjo_key *key)
{
    int64_t s;
    switch (pp->policy) {
    case SJO_EFFICIENCY:
        key->k0 = 0; key->k1 = F; key->k2 = 0;
        return SJO_OK;
    case SJO_FAIRNESS:
        if (__builtin_mul_overflow(F, (int64_t)pp->wait_scale + wait, &s)) return SJO_ERR_OVERFLOW;
        key->k0 = 0; key->k1 = s; key->k2 = 0;
        return SJO_OK;
    case SJO_SLA:
        if (cls < 0 || cls > 2) return SJO_ERR_ARG;
        if (__builtin_mul_overflow(F, (int64_t)pp->sla_weight[cls], &s)) return SJO_ERR_OVERFLOW;
        key->k0 = (pp->class0_override && cls == 0) ? 1 : 0; key->k1 = s; key->k2 = 0;
        return SJO_OK;
    case SJO_MIXED:
        if (cls < 0 || cls > 2) return SJO_ERR_ARG;
        if (__builtin_mul_overflow(F, (int64_t)pp->wait_scale + wait, &s)) return SJO_ERR_OVERFLOW;
        key->k0 = 2 - cls; key->k1 = s; key->k2 = F;
        return SJO_OK;
    default:
        return SJO_ERR_ARG;
    }
}

/* Select for one gap: linear scan over jobs in id order, keeping a candidate
 * only when its key is strictly greater (so the lowest id wins ties). */
static int select_gap(const sjo_params *pp, int32_t n_jobs, const int32_t *cut_row,
                      const int64_t *seg_off, const int64_t *pre_dur, const int64_t *pre_peak,
                      const int64_t *pre_area, const int32_t *wait, const uint8_t *sla_class, const int32_t *job_held,
                      int32_t *cand_job, int32_t *cand_cut, int64_t *cand_score)
{
    sjo_key best = {0, 0, 0};
    int32_t bj = -1, bc = -1;
    for (int32_t j = 0; j < n_jobs; ++j) {
        int32_t c = cut_row[j];
        if (c < 0) continue;
        if (job_held && job_held[j] >= 0) continue;
        int64_t k = seg_off[j] + c - 1;
        sjo_key key;
        int64_t F;
        if (pre_area) F = pre_area[k];
        else if (__builtin_mul_overflow(pre_dur[k], pre_peak[k], &F)) return SJO_ERR_OVERFLOW;
        int rc = make_key(pp, F, wait ? wait[j] : 0, sla_class ? sla_class[j] : 0, &key);
        if (rc != SJO_OK) return rc;
        if (bj < 0 || key_greater(&key, &best)) { best = key; bj = j; bc = c; }
    }
    *cand_job = bj;
    *cand_cut = bc;
    *cand_score = bj >= 0 ? best.k1 : 0;
    return SJO_OK;
}

/* Per-gap policy arg-max over interested, un-held jobs.  pre_dur / pre_peak are
 * sjo_prepare's outputs (looked up at the cut).  pre_area (may be NULL) switches
 * the filled capacity-time F from the rectangle duration * peak to the area
 * under the envelope, sjo_area's output.  job_held (may be NULL): a job
 * with job_held[j] >= 0 is skipped.  gap_active (may be NULL): a gap with
 * gap_active[g] == 0 gets cand_job = cand_cut = -1, cand_score = 0. */
int sjo_select(int32_t n_gaps, int32_t n_jobs, const int32_t *cut, const int64_t *seg_off,
               const int64_t *pre_dur, const int64_t *pre_peak, const int64_t *pre_area, const sjo_params *pp,
               const int32_t *wait, const uint8_t *sla_class, const int32_t *job_held,
               const uint8_t *gap_active, int32_t *cand_job, int32_t *cand_cut,
               int64_t *cand_score)
{
    if (n_gaps < 0 || n_jobs < 0 || !pp) return SJO_ERR_ARG;
    if (pp->policy < 0 || pp->policy > 3) return SJO_ERR_ARG;
    int err = SJO_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t g = 0; g < n_gaps; ++g) {
        if (gap_active && !gap_active[g]) {
            cand_job[g] = -1; cand_cut[g] = -1; cand_score[g] = 0;
            continue;
        }
        int rc = select_gap(pp, n_jobs, cut + (int64_t)g * n_jobs, seg_off, pre_dur, pre_peak, pre_area,
                            wait, sla_class, job_held, &cand_job[g], &cand_cut[g],
                            &cand_score[g]);
        if (rc != SJO_OK) {
#pragma omp critical
            err = rc;
        }
    }
    return err;
}

/* ------------------------------------------------------------------------
 * Resolve: deterministic rounds.  Every ungranted gap selects among the jobs
 * no gap holds yet; each selected job keeps the lowest-index gap that chose
 * it, and that grant is final; the other gaps that chose it try again next
 * round.  Stops when a round finds no candidate at all or leaves no loser.
 * rounds_stable[0] = rounds in which a select was run, rounds_stable[1] = 1
 * if the process ended by itself, 0 if the round cap cut it short.
 * ---------------------------------------------------------------------- */
int sjo_resolve(int32_t n_gaps, int32_t n_jobs, const int32_t *cut, const int64_t *seg_off,
                const int64_t *pre_dur, const int64_t *pre_peak, const int64_t *pre_area, const sjo_params *pp,
                const int32_t *wait, const uint8_t *sla_class, int32_t *grant_job,
                int32_t *grant_cut, int64_t *grant_score, int32_t *job_gap,
                int32_t *rounds_stable)
{
    if (n_gaps < 0 || n_jobs < 0 || !pp || pp->max_rounds < 0) return SJO_ERR_ARG;
    int32_t *cj = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_gaps ? n_gaps : 1));
    int32_t *cc = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_gaps ? n_gaps : 1));
    int64_t *cs = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_gaps ? n_gaps : 1));
    uint8_t *active = (uint8_t *)malloc((size_t)(n_gaps ? n_gaps : 1));
    if (!cj || !cc || !cs || !active) { free(cj); free(cc); free(cs); free(active); return SJO_ERR_NOMEM; }

    for (int32_t g = 0; g < n_gaps; ++g) { grant_job[g] = -1; grant_cut[g] = -1; grant_score[g] = 0; }
    for (int32_t j = 0; j < n_jobs; ++j) job_gap[j] = -1;

    int64_t cap = pp->max_rounds > 0 ? pp->max_rounds
                                     : (int64_t)(n_gaps < n_jobs ? n_gaps : n_jobs) + 1;
    int32_t rounds = 0, stable = 0;
    int rc = SJO_OK;
    for (int64_t r = 1; r <= cap; ++r) {
        for (int32_t g = 0; g < n_gaps; ++g) active[g] = grant_job[g] < 0;
        rc = sjo_select(n_gaps, n_jobs, cut, seg_off, pre_dur, pre_peak, pre_area, pp, wait, sla_class,
                        job_gap, active, cj, cc, cs);
        if (rc != SJO_OK) break;
        ++rounds;
        int64_t n_cand = 0, n_lost = 0;
        /* gaps in increasing index order: the first gap that names a job keeps it */
        for (int32_t g = 0; g < n_gaps; ++g) {
            int32_t j = cj[g];
            if (j < 0) continue;
            ++n_cand;
            if (job_gap[j] < 0) {
                job_gap[j] = g;
                grant_job[g] = j; grant_cut[g] = cc[g]; grant_score[g] = cs[g];
            } else {
                ++n_lost;
            }
        }
        if (n_cand == 0 || n_lost == 0) { stable = 1; break; }
    }
    rounds_stable[0] = rounds;
    rounds_stable[1] = stable;
    free(cj); free(cc); free(cs); free(active);
    return rc;
}

/* ------------------------------------------------------------------------
 * Advance to the next tick (Sec. 3.1 / 3.5: a parent job resumes from its last
 * completed fragment; the metrics are those the paper plans to report in its
 * evaluation, Sec. 5: utilisation, queueing delay, rejections).
 * For every job that holds a gap: progress = the granted cut, wait = 0.  Every
 * other job that still has segments left waits wait_step longer (saturating at
 * INT32_MAX); a finished job keeps its wait.  wait may be NULL.
 * pre_dur / pre_peak are sjo_prepare's outputs for the progress points BEFORE
 * the advance.  metrics[0] = sum over granted gaps of duration * peak of the
 * granted subjob, metrics[1] = sum over all gaps of max(W,0) * max(C,0),
 * metrics[2] = number of grants, metrics[3] = jobs with nothing left after the
 * advance.
 * ---------------------------------------------------------------------- */
int sjo_advance(int32_t n_gaps, int32_t n_jobs, const int64_t *seg_off, const int64_t *pre_dur,
                const int64_t *pre_peak, const int32_t *W, const int32_t *C,
                const int32_t *grant_job, const int32_t *grant_cut, const int32_t *job_gap,
                int32_t *progress, int32_t *wait, int32_t wait_step, int64_t *metrics)
{
    if (n_gaps < 0 || n_jobs < 0 || wait_step < 0 || !metrics) return SJO_ERR_ARG;
    int64_t filled = 0, offered = 0, grants = 0, finished = 0;
    for (int32_t g = 0; g < n_gaps; ++g) {
        int64_t w = W[g] > 0 ? W[g] : 0, c = C[g] > 0 ? C[g] : 0;
        offered += w * c;
        int32_t j = grant_job[g];
        if (j < 0) continue;
        if (j >= n_jobs || job_gap[j] != g) return SJO_ERR_ARG;
        int64_t k = seg_off[j] + grant_cut[g] - 1;
        if (grant_cut[g] <= progress[j] || k >= seg_off[j + 1]) return SJO_ERR_ARG;
        filled += pre_dur[k] * pre_peak[k];
        ++grants;
    }
    for (int32_t j = 0; j < n_jobs; ++j) {
        int64_t L = seg_off[j + 1] - seg_off[j];
        int32_t g = job_gap[j];
        if (g >= 0) {
            if (g >= n_gaps || grant_job[g] != j) return SJO_ERR_ARG;
            progress[j] = grant_cut[g];
            if (wait) wait[j] = 0;
        } else if (progress[j] < L && wait) {
            int64_t w = (int64_t)wait[j] + wait_step;
            wait[j] = w > INT32_MAX ? INT32_MAX : (int32_t)w;
        }
        if (progress[j] >= L) ++finished;
    }
    metrics[0] = filled; metrics[1] = offered; metrics[2] = grants; metrics[3] = finished;
    return SJO_OK;
}

