/*
 * sja.h -- C ABI of the batched gap-job fit / slot-grant engine for one
 * scheduling tick of Scheduler-Driven Job Atomization (MI355X, gfx950).
 *
 * One tick of the paper's three-phase protocol (Sec. 3.5), evaluated for every
 * advertised gap and every waiting job at once:
 *
 *   sja_set_limits        optional admission limits applied by the next prepare:
 *                         power trace under a cap, per-job deadline (Sec. 4.4),
 *                         minimum / maximum subjob duration (Sec. 4.3)
 *   sja_set_hysteresis    optional rule on subdivision applied by the next
 *                         prepare: a shorter fragment only for a minimum gain in
 *                         slack (Sec. 3.9)
 *   sja_prepare_profiles  per-job running duration / running peak / last safe
 *                         boundary from the job's progress point (the on-demand
 *                         evaluation of the envelope U(t), Sec. 3.9)
 *   sja_fit               job -> scheduler reply for every (gap, job) pair:
 *                         the longest safe subjob that fits, or decline
 *                         (Sec. 3.5 phase 2, Sec. 3.8 admissibility, Sec. 3.9)
 *   sja_select            scheduler policy arg-max per gap (Sec. 3.5 phase 3)
 *   sja_fit_select        the two above in one pass, without the pair matrix
 *   sja_resolve           grants, with conflicts settled in rounds so that a job
 *                         holds at most one gap (Sec. 3.1 / 3.5: fragments of a
 *                         job are sequential from one progress point)
 *   sja_cover             smallest capacity of a set that covers each grant
 *                         (Sec. 3.9)
 *   sja_advance           end of the tick: granted jobs move to their cut and
 *                         only their tables are rebuilt (Sec. 3.1 / 3.5)
 * Beside the method: sja_validate (input preconditions, checked on the device),
 * sja_prepare_profiles_static (the prepare for callers that cannot allocate),
 * sja_set_score, sja_set_resolve_mode, and two measurement aids
 * (sja_enable_timing / sja_last_fit_kernel_ms, sja_store_reference).
 *
 * Conventions
 *   - Every array argument is a DEVICE pointer owned by the caller, unless the
 *     comment says "host".  The library never frees or reallocates them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call except sja_resolve only enqueues work and returns; outputs
 *     are valid once the stream has been synchronised.  sja_resolve runs a
 *     data-dependent number of rounds and synchronises the stream before it
 *     returns.
 *   - The context remembers the pointers and sizes handed to the previous
 *     call of the sequence prepare -> fit -> select / resolve: the arrays of
 *     sja_prepare_profiles must stay alive and unchanged until the last
 *     sja_fit / sja_select / sja_resolve that uses them, and the `cut` matrix
 *     of sja_fit until the last sja_select / sja_resolve.  Calling out of
 *     order returns SJA_ERR_STATE.
 *   - All scratch lives in one caller-owned workspace (sja_set_workspace);
 *     the library itself allocates no device memory.
 *   - Return value: SJA_OK (0) or a negative sja_status.  Arguments that can
 *     be checked on the host (null pointers, negative sizes, bad enum values,
 *     workspace too small) are rejected before any device work is enqueued.
 *     No exception or abort crosses this boundary.
 *
 * Profile model.  Job j owns segments seg_off[j] .. seg_off[j+1]-1 (CSR).
 * Segment k lasts dur[k] >= 1 ticks at mem[k] >= 0 MiB.  Boundaries of a job
 * with L segments are numbered 0..L; boundary b lies before segment b, boundary
 * L is the job's end.  safe[k] != 0 flags boundary k+1 (within the job) as a
 * subjob boundary (Sec. 3.7); the end counts as one whatever its flag.
 * progress[j] in [0, L] is the boundary the job has completed up to.
 *
 * Data-dependent preconditions (not checked by these calls; sja_validate
 * checks them on the device and reports problem bits): seg_off non-decreasing with
 * seg_off[0] == 0 and seg_off[n_jobs] == n_segments; 0 <= progress[j] <= L_j;
 * dur >= 1; mem >= 0; per job, the sum of durations fits int32; every policy
 * score term (see sja_params: F, or F times its weight) is below 2^62 (the
 * arg-max packs a two-bit tier above it).
 */
#ifndef SJA_H
#define SJA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sja_ctx sja_ctx; /* opaque; host-side bookkeeping only */

typedef enum {
    SJA_OK = 0,
    SJA_ERR_NULL = -1,      /* a required pointer is NULL                      */
    SJA_ERR_SIZE = -2,      /* a size is negative or beyond the supported max  */
    SJA_ERR_POLICY = -3,    /* bad policy enum or policy parameter             */
    SJA_ERR_STATE = -4,     /* call out of sequence                            */
    SJA_ERR_OVERFLOW = -5,  /* G*J or a byte count does not fit                */
    SJA_ERR_WORKSPACE = -6, /* workspace missing, misaligned or too small      */
    SJA_ERR_HIP = -7,       /* a HIP runtime call failed (see sja_last_error)  */
    SJA_ERR_NOT_IMPLEMENTED = -8
} sja_status;

typedef enum {
    SJA_POLICY_EFFICIENCY = 0, /* key = F                                           */
    SJA_POLICY_FAIRNESS = 1,   /* key = F * (wait_scale + wait[j])                  */
    SJA_POLICY_SLA = 2,        /* key = (class-0 tier, F * sla_weight[class[j]])    */
    SJA_POLICY_MIXED = 3       /* key = (2 - class[j], F * (wait_scale + wait[j]), F) */
} sja_policy;

/*
 * Policy parameters (Sec. 3.5: the scheduler picks by its allocation policy;
 * Sec. 4.2: a lightweight selection among interested jobs).  F is the
 * capacity-time rectangle a subjob fills: its duration times its peak memory.
 * Keys compare lexicographically, larger wins, equal keys go to the lower job
 * id.  The score reported for a candidate is the key's score term (F, or the
 * weighted F).
 */
typedef struct {
    int32_t policy;          /* sja_policy                                        */
    int32_t wait_scale;      /* > 0; 1000 reproduces F * (1 + wait/1000) exactly  */
    int32_t sla_weight[3];   /* >= 0; per SLA class 0,1,2 (class 0 = most urgent) */
    int32_t class0_override; /* SLA: nonzero = any class-0 job beats other classes */
    int32_t max_rounds;      /* sja_resolve: >= 0; 0 = run until stable           */
} sja_params;

/* Largest sizes the library accepts. */
#define SJA_MAX_JOBS 16777216      /* 2^24 */
#define SJA_MAX_GAPS 1048576       /* 2^20 */
#define SJA_MAX_SEGMENTS 2147483647 /* 2^31-1 */

/* Creates a context bound to HIP device `device_id`.  Touches no device.
 * *out (host) receives the context; free it with sja_destroy. */
int sja_create(sja_ctx **out, int device_id);
int sja_destroy(sja_ctx *ctx);

/* Bytes of workspace needed for a tick of this size (0 on invalid sizes). */
size_t sja_workspace_bytes(int64_t n_gaps, int64_t n_jobs, int64_t n_segments);

/* Hands the library a caller-owned device buffer (256-byte aligned).  It must
 * stay alive while the context uses it and may be replaced between ticks.
 * Its contents are private to the library between sja_prepare_profiles and
 * the last call of that tick. */
int sja_set_workspace(sja_ctx *ctx, void *dev_ptr, size_t bytes);

/* Static string for a status code; last error text of a context (host). */
const char *sja_status_string(int status);
const char *sja_last_error(const sja_ctx *ctx);

/*
 * Which quantity the policies score as the "filled capacity-time" F of a
 * subjob (the paper names the notion and leaves its formula open):
 *   SJA_SCORE_RECTANGLE  duration x peak memory: the rectangle the subjob's
 *                        footprint occupies in the gap (the default)
 *   SJA_SCORE_AREA       sum of dur x mem over the subjob's segments: the area
 *                        under its memory envelope, never above the rectangle
 * Takes effect at the next sja_prepare_profiles (which then also keeps running
 * area tables in the workspace) and holds for the sja_select, sja_fit_select,
 * sja_resolve and sja_advance calls on top of it.  Keys, tie rules and the
 * score bound are unchanged.  SJA_ERR_SIZE for any other value.
 */
typedef enum {
    SJA_SCORE_RECTANGLE = 0,
    SJA_SCORE_AREA = 1
} sja_score;
int sja_set_score(sja_ctx *ctx, int score);

/*
 * Admission limits on top of each gap's own window and capacity.  All are off
 * in a new context.
 *   - power trace with a cap (Sec. 4.4, energy-aware admission: the subjob's
 *     peak power over its lifetime stays within the cap; the same test as the
 *     memory fit, on a second channel).  The cap is the one in force for the
 *     tick, shared by its gaps.
 *   - deadline per job (Sec. 4.4, deadline-aware admission: only subjobs that
 *     complete by the deadline; the gaps of a tick start at `now`, so the
 *     subjob's duration must be <= deadline[j] - now).
 *   - duration bounds (Sec. 4.3, granularity: minimum and maximum subjob
 *     duration enforced by the framework): at most tau_max, and at least
 *     tau_min unless the subjob runs to the job's end.
 * With limits, cut[g][j] is the largest safe boundary whose subjob passes the
 * gap's tests and all of these.
 */
typedef struct {
    int32_t tau_min;   /* >= 0; 0 = no lower bound                         */
    int32_t tau_max;   /* >= 0; INT32_MAX = no upper bound                 */
    int32_t power_cap; /* used only with a power trace                     */
    int32_t now;       /* used only with deadlines                         */
} sja_limits;

/*
 * Sets (limits != NULL) or clears (limits == NULL) the admission limits.
 * `limits` is a host pointer and is copied.  power [n_segments] int32 (power of
 * each profile segment) and deadline [n_jobs] int32 are device arrays sized for
 * the NEXT sja_prepare_profiles, or NULL to leave that test out; they must stay
 * alive and unchanged while that prepare's tables are in use.  The limits take
 * effect at the next sja_prepare_profiles; sja_advance keeps applying the ones
 * its prepare used, `now` included (to move `now`, set the limits and prepare
 * again).  SJA_ERR_SIZE for a negative tau_min or tau_max.  Touches no device.
 */
int sja_set_limits(sja_ctx *ctx, const sja_limits *limits, const int32_t *power,
                   const int32_t *deadline);

/*
 * Hysteresis on subdivision (Sec. 3.9, safeguard ii: a minimum gain in slack is
 * required before a further subdivision is accepted; otherwise the longer, more
 * stable fragment is preferred).  The paper names the rule without a formula;
 * the reading built here, with cover(x) = the smallest capacity of cap_set that
 * is >= x (Sec. 3.9's slack-minimising mapping), +infinity if there is none:
 *   for a pair (gap, job) let b* be the cut without the rule (limits included).
 *   A boundary b, progress < b < b*, that may be offered (a safe boundary, not
 *   shorter than tau_min under limits) is worth the subdivision if cover(P(b)) is
 *   finite and cover(P(b*)) - cover(P(b)) >= min_gain (any finite cover counts
 *   when cover(P(b*)) is infinite).  cut[g][j] is the longest boundary worth the
 *   subdivision, and b* if none is.  A decline stays a decline, so the interest
 *   bits do not change.
 * Every call that reports or scores a subjob (sja_fit, sja_select,
 * sja_fit_select, sja_resolve, sja_cover on their grants, sja_advance) then
 * works with the cut the rule chose.
 *   n_caps in [0, SJA_MAX_CAPS]; 0 switches the rule off (the state of a new
 *   context) and ignores the other arguments.
 *   cap_set [n_caps] int32, HOST pointer, ascending; copied.
 *   min_gain >= 1, in the units of the capacities.
 * Takes effect at the next sja_prepare_profiles and is kept by the sja_advance
 * calls on top of it.  SJA_ERR_SIZE for n_caps out of range, min_gain < 1 or a
 * set that does not ascend; SJA_ERR_NULL for a missing set.  Touches no device.
 */
#define SJA_MAX_CAPS 32
int sja_set_hysteresis(sja_ctx *ctx, int32_t n_caps, const int32_t *cap_set, int32_t min_gain);

/*
 * Per-job segmented scans from the progress point (Sec. 3.9: segmentation is
 * evaluated on demand from the job's current state).  For each job j with
 * p = progress[j] and each boundary b = p+1 .. L_j, at entry k = seg_off[j]+b-1:
 *   pre_dur[k]   = dur[p] + ... + dur[b-1]            (running duration D_j(b))
 *   pre_peak[k]  = max(mem[p], ..., mem[b-1])         (running peak P_j(b))
 *   prev_safe[k] = largest safe boundary in (p, b], or -1 if there is none
 * Entries of segments before the progress point are not written.
 * Also builds the library's private per-job tables in the workspace.
 *   seg_off [n_jobs+1] int64, dur/mem [n_segments] int32, safe [n_segments]
 *   uint8, progress [n_jobs] int32; outputs [n_segments] int32 each.
 * Needs a workspace sized for (any n_gaps, n_jobs, n_segments).
 */
int sja_prepare_profiles(sja_ctx *ctx, void *stream, int32_t n_jobs, int64_t n_segments,
                         const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                         const uint8_t *safe, const int32_t *progress, int32_t *pre_dur,
                         int32_t *pre_peak, int32_t *prev_safe);

/*
 * sja_prepare_profiles for callers that cannot allocate device memory, not even
 * a workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same outputs, same errors; the library's
 * private tables go into a scratch array built into the library (file-scope
 * device memory of SJA_STATIC_SCRATCH_BYTES per GPU, held by every GPU the
 * library runs on until the process ends) instead of the caller's workspace,
 * and that array then IS the context's workspace for the rest of the tick:
 * sja_fit, sja_fit_select, sja_select, sja_resolve, sja_cover and sja_advance
 * work on it as usual and return SJA_ERR_WORKSPACE when their own tables for
 * that many gaps do not fit into it.  The context stays on the built-in scratch
 * until sja_set_workspace hands it another buffer.
 *   - Limit: SJA_ERR_SIZE, before any device work, unless
 *     sja_workspace_bytes(0, n_jobs, n_segments) <= SJA_STATIC_SCRATCH_BYTES.
 *   - Calls no hipMalloc / hipFree and no allocating library routine.
 *   - One array per GPU, shared by every context and every call on that GPU and
 *     never cleared: nothing in it has to start at zero (each call rewrites all
 *     that it later reads), but two ticks that overlap on one GPU, from two
 *     contexts or two streams, race on it.  Run them one after the other.
 */
#define SJA_STATIC_SCRATCH_BYTES (64u << 20) /* 64 MiB */
int sja_prepare_profiles_static(sja_ctx *ctx, void *stream, int32_t n_jobs, int64_t n_segments,
                                const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                                const uint8_t *safe, const int32_t *progress, int32_t *pre_dur,
                                int32_t *pre_peak, int32_t *prev_safe);

/*
 * Fit evaluation for every (gap, job) pair (Sec. 3.5 phase 2; Sec. 3.8: a
 * subjob is admissible on capacity C over its lifetime if its demand stays
 * <= C; Sec. 3.9: max of U over the window <= c, longer fragments preferred).
 *   cut[g*n_jobs + j] = largest boundary b in (progress[j], L_j] that is safe,
 *                       with D_j(b) <= W[g] and P_j(b) <= C[g]; -1 = decline.
 *   interest_bits[g*ceil(n_jobs/32) + j/32] bit (j%32) = (cut >= 0); may be NULL.
 * W, C [n_gaps] int32 (a negative W or C fits nothing).  Uses the profiles of
 * the last sja_prepare_profiles.  cut is row-major by gap: one row holds one
 * gap's replies.
 */
int sja_fit(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *W, const int32_t *C,
            int32_t *cut, uint32_t *interest_bits);

/*
 * Policy arg-max per gap over the interested jobs of the last sja_fit
 * (Sec. 3.5 phase 3).  A job with job_held[j] >= 0 is skipped (job_held may be
 * NULL = none held); a gap with gap_active[g] == 0 gets no candidate
 * (gap_active may be NULL = all active).  wait [n_jobs] int32 and sla_class
 * [n_jobs] uint8 (values 0..2) are required by the policies that read them
 * (FAIRNESS/MIXED: wait; SLA/MIXED: sla_class) and may be NULL otherwise.
 *   cand_job[g]   winning job id, or -1 if no candidate
 *   cand_cut[g]   its cut (-1 if none)
 *   cand_score[g] its score term (0 if none)
 */
int sja_select(sja_ctx *ctx, void *stream, const sja_params *params, const int32_t *wait,
               const uint8_t *sla_class, const int32_t *job_held, const uint8_t *gap_active,
               int32_t *cand_job, int32_t *cand_cut, int64_t *cand_score);

/*
 * sja_fit followed by sja_select in one pass that never writes the (gap, job)
 * replies down (Sec. 3.5: subjob state comes into being only at a grant, and
 * the scheduler only needs the best reply per gap).  Arguments are
 * those of sja_fit (n_gaps, W, C) and of sja_select (params, wait, sla_class,
 * job_held, gap_active, cand_*), with the same meaning, layout and results:
 * cand_job / cand_cut / cand_score equal what sja_select would report after
 * sja_fit on the same inputs.  No cut matrix and no interest rows exist
 * afterwards: sja_select needs a sja_fit of its own; sja_resolve works (its
 * candidate lists need no matrix, and where they cannot run - more than 64
 * distinct capacities, the lists are built per capacity class - its scanning
 * rounds evaluate the pairs again each round instead of reading a matrix).
 * Only enqueues work.
 * With sja_enable_timing the events bracket this call's stepping kernel.
 */
int sja_fit_select(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *W, const int32_t *C,
                   const sja_params *params, const int32_t *wait, const uint8_t *sla_class,
                   const int32_t *job_held, const uint8_t *gap_active, int32_t *cand_job,
                   int32_t *cand_cut, int64_t *cand_score);

/*
 * Grants with conflict resolution in deterministic rounds (Sec. 3.5: one job
 * is granted per slot; Sec. 3.1 / 3.5: a job's fragments are sequential, so it
 * can hold one gap per tick).  Round: every ungranted gap selects among the
 * jobs no gap holds yet; each selected job keeps the lowest-index gap that
 * selected it and that grant is final; the other gaps reselect next round.
 * Ends when a round finds no candidate or leaves no loser, or after
 * params->max_rounds rounds (then the last round's losers stay ungranted).
 *   grant_job/grant_cut [n_gaps] int32 (-1 = ungranted), grant_score [n_gaps]
 *   int64 (0 = ungranted), job_gap [n_jobs] int32 (gap held by the job or -1),
 *   rounds_used_and_stable [2] int32: rounds in which a selection ran, and 1
 *   if the process ended by itself (0 if the round cap cut it short).
 * Synchronises `stream` before returning.
 */
int sja_resolve(sja_ctx *ctx, void *stream, const sja_params *params, const int32_t *wait,
                const uint8_t *sla_class, int32_t *grant_job, int32_t *grant_cut,
                int64_t *grant_score, int32_t *job_gap, int32_t *rounds_used_and_stable);

/*
 * End of a tick: apply the grants and get the job table ready for the next
 * batch of gaps (Sec. 3.1 / 3.5: a parent job resumes from its last completed
 * fragment; the totals are the quantities Sec. 5 plans to report: utilisation,
 * queueing delay, grants against offers).
 *   W, C [n_gaps]                    the gaps the grants were made for
 *   grant_job, grant_cut [n_gaps]    as sja_resolve left them
 *   job_gap [n_jobs]                 as sja_resolve left it
 *   progress [n_jobs] int32, in/out  a job holding a gap moves to its granted cut
 *   wait [n_jobs] int32, in/out      0 for a job holding a gap; any other job
 *                                    with segments left waits wait_step (>= 0)
 *                                    longer, saturating at 2^31-1; a finished job
 *                                    keeps its value.  May be NULL.
 *   metrics [4] int64, out           [0] sum over grants of duration x peak of the
 *                                    granted subjob, [1] sum over gaps of
 *                                    max(W,0) x max(C,0), [2] grants, [3] jobs with
 *                                    no segment left after the move
 * The running tables of the last sja_prepare_profiles (pre_dur, pre_peak,
 * prev_safe, still owned by the caller, and the library's own per-job tables)
 * are rebuilt for the jobs that moved and left as they are for the others, so
 * the next sja_fit / sja_fit_select needs no sja_prepare_profiles; this call
 * reads dur, mem, safe and seg_off through the pointers given to that call,
 * which must still be alive and unchanged.  `progress` may be the array given
 * to sja_prepare_profiles or a copy of it.  A grant counts when grant_job[g] = j
 * and job_gap[j] = g point at each other and progress[j] < grant_cut[g] <= L_j;
 * any other entry is ignored (no grant).  The cut matrix, candidates and lists
 * of the last fit are stale afterwards: sja_select / sja_resolve need a new
 * sja_fit or sja_fit_select.  Only enqueues work.
 */
int sja_advance(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *W, const int32_t *C,
                const int32_t *grant_job, const int32_t *grant_cut, const int32_t *job_gap,
                int32_t *progress, int32_t *wait, int32_t wait_step, int64_t *metrics);

/*
 * Slack-minimising capacity mapping for the grants (Sec. 3.9: map the granted
 * window to the smallest slice capacity of the set that covers the predicted
 * demand in it).
 *   C, grant_job, grant_cut [n_gaps]  the gaps and the grants of sja_resolve
 *   cap_set [n_caps] int32            the capacity set, ascending (device)
 *   cover [n_gaps] int32, out         smallest cap_set entry >= the memory peak
 *                                     of the granted subjob; -1 if the gap is
 *                                     ungranted or no entry covers the peak
 *   slack [n_gaps] int32, out         C[g] - cover[g]; 0 where cover is -1
 * Reads the running peaks of the last sja_prepare_profiles: call it before
 * sja_advance moves the jobs.  An entry whose job id or cut is out of range
 * counts as ungranted.  A cap_set that does not ascend gives unspecified (but
 * in-range) answers.  Only enqueues work.
 */
int sja_cover(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *C, const int32_t *grant_job,
              const int32_t *grant_cut, int32_t n_caps, const int32_t *cap_set, int32_t *cover,
              int32_t *slack);

/*
 * Input check, no step of the method: the data-dependent preconditions that
 * the calls above assume and do not test themselves.  *problems (device,
 * one uint32) receives the OR of the sja_problem bits found, 0 if none.
 *   seg_off [n_jobs+1], dur, mem [n_segments], progress [n_jobs]: as for
 *   sja_prepare_profiles.  params (host; may be NULL), wait, sla_class: as for
 *   sja_select; with params the policy's per-job inputs are checked too, and
 *   the score bound is tested per job against (whole duration) x (largest
 *   memory) x the job's policy factor, which no subjob's score exceeds.
 * Reads nothing outside the arrays whatever their contents.  Only enqueues work.
 */
typedef enum {
    SJA_BAD_OFFSETS = 1,       /* seg_off does not start at 0, decreases, or does not end at n_segments */
    SJA_BAD_DURATION = 2,      /* a segment lasts less than 1 tick                                      */
    SJA_BAD_MEMORY = 4,        /* a negative memory value                                               */
    SJA_BAD_PROGRESS = 8,      /* a progress point outside [0, L_j]                                     */
    SJA_BAD_DURATION_SUM = 16, /* a job's durations sum to more than 2^31-1                             */
    SJA_BAD_CLASS = 32,        /* an SLA class above 2 under a policy that reads it                     */
    SJA_BAD_WAIT = 64,         /* a negative waiting time under a policy that reads it                  */
    SJA_BAD_SCORE_RANGE = 128  /* a policy score could reach 2^62                                       */
} sja_problem;
int sja_validate(sja_ctx *ctx, void *stream, int32_t n_jobs, int64_t n_segments, const int64_t *seg_off,
                 const int32_t *dur, const int32_t *mem, const int32_t *progress, const sja_params *params,
                 const int32_t *wait, const uint8_t *sla_class, uint32_t *problems);

/*
 * Measurement aid for benchmarks (callers that report the pair-evaluation
 * kernel's own duration rather than the whole call's).  With timing enabled,
 * sja_fit brackets its pair-evaluation kernel with HIP events on `stream`;
 * sja_last_fit_kernel_ms waits for that kernel and stores its duration in
 * *ms_host (host pointer).  SJA_ERR_STATE if no timed sja_fit has run.
 */
int sja_enable_timing(sja_ctx *ctx, int on);
int sja_last_fit_kernel_ms(sja_ctx *ctx, float *ms_host);

/*
 * Measurement aid, no step of the method: writes the (n_gaps x n_jobs) int32
 * matrix `cut` (device) with the launch shape, the block-to-tile mapping and the
 * store stream of sja_fit's pair-evaluation kernel - one 256-byte piece of a
 * row per wave and step, along the sorted gap positions of the last sja_fit or
 * sja_fit_select - but computes nothing: cut[g][j] = j afterwards.  Its
 * duration is what the memory system allows for that address pattern, the
 * ceiling the pair-evaluation kernel is measured against.  Needs the plan of
 * the last sja_fit / sja_fit_select (SJA_ERR_STATE otherwise); if `cut` is the
 * matrix that sja_fit wrote, that matrix is gone and sja_select / matrix rounds
 * need a new sja_fit.  Only enqueues work.
 */
int sja_store_reference(sja_ctx *ctx, void *stream, int32_t *cut);

/*
 * How sja_resolve runs the rounds of Sec. 3.5's grant phase.  Both modes give
 * the same grants, rounds_used and stable flag; they differ in speed only.
 *   SJA_RESOLVE_LISTS   per-gap candidate lists in preference order, one cheap
 *                       launch per round (the default).  Falls back to the
 *                       other mode by itself with more than 64 distinct
 *                       capacities or when the lists would not fit the workspace.
 *   SJA_RESOLVE_MATRIX  every round re-scans the gaps that are still
 *                       ungranted: the rows of the cut matrix after sja_fit,
 *                       the pairs themselves (evaluated again, nothing stored)
 *                       after sja_fit_select.
 *   SJA_RESOLVE_LISTS_LOOKUP  as SJA_RESOLVE_LISTS, but the job of every list
 *                       record is looked up through the record's rank even
 *                       where the list keys have room to carry it: the form
 *                       the lists take by themselves for batches whose block,
 *                       rank and job numbers do not fit one 64-bit key
 *                       together; selectable so that it can be tested at any
 *                       size.
 * SJA_ERR_SIZE for any other value.
 */
typedef enum {
    SJA_RESOLVE_LISTS = 0,
    SJA_RESOLVE_MATRIX = 1,
    SJA_RESOLVE_LISTS_LOOKUP = 2
} sja_resolve_mode;
int sja_set_resolve_mode(sja_ctx *ctx, int mode);

#ifdef __cplusplus
}
#endif
#endif /* SJA_H */
