// C ABI of the gap-job fit / slot-grant engine: argument validation, workspace
// bookkeeping and kernel launches.  See include/sja.h for the contract.
#include "sja_kernels.h"

#include <mutex>
#include <new>
#include <vector>

using namespace sja;

// Built-in scratch for callers that cannot allocate a workspace (see
// sja_prepare_profiles_static).  Every GPU the library runs on holds its own
// copy of this array, at its own address, until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress: kernels are given
// the address that call returns, never the name.
static __device__ __align__(256) unsigned char scratch[SJA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once known
std::mutex g_scratch_mutex;

// Address of the built-in scratch on `device`, which must be the current device.
hipError_t static_scratch(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    hipError_t err = hipSuccess;
    explicit DeviceGuard(int dev)
    {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != dev) {
            err = hipSetDevice(dev);
            switched = (err == hipSuccess);
        }
    }
    ~DeviceGuard()
    {
        if (switched) (void)hipSetDevice(prev);
    }
};

int fail(sja_ctx *ctx, int status, const char *what)
{
    if (ctx) snprintf(ctx->err, sizeof(ctx->err), "%s: %s", sja_status_string(status), what);
    return status;
}

int fail_hip(sja_ctx *ctx, hipError_t e, const char *what)
{
    if (ctx) snprintf(ctx->err, sizeof(ctx->err), "HIP error in %s: %s", what, hipGetErrorString(e));
    return SJA_ERR_HIP;
}

#define SJA_HIP(call, what)                                        \
    do {                                                           \
        hipError_t e__ = (call);                                   \
        if (e__ != hipSuccess) return fail_hip(ctx, e__, what);    \
    } while (0)

template <typename T>
T *ws_ptr(sja_ctx *ctx, size_t off) { return reinterpret_cast<T *>(ctx->ws + off); }

// The per-atom table of F is read while the area score or the hysteresis rule is in force
// (without either an atom's F is its own duration x peak); the per-segment area table only
// with the area score.
const long long *atom_area_of(const sja_ctx *ctx, const Layout &L)
{
    return (ctx->score_used == SJA_SCORE_AREA || ctx->hyst_used_n_caps > 0)
               ? reinterpret_cast<const long long *>(ctx->ws + L.atom_area) : nullptr;
}
const long long *pre_area_of(const sja_ctx *ctx, const Layout &L)
{
    return ctx->score_used == SJA_SCORE_AREA ? reinterpret_cast<const long long *>(ctx->ws + L.pre_area) : nullptr;
}

int check_params(sja_ctx *ctx, const sja_params *p, const int32_t *wait, const uint8_t *sla_class)
{
    if (!p) return fail(ctx, SJA_ERR_NULL, "params");
    if (p->policy < SJA_POLICY_EFFICIENCY || p->policy > SJA_POLICY_MIXED)
        return fail(ctx, SJA_ERR_POLICY, "unknown policy");
    if (p->wait_scale <= 0) return fail(ctx, SJA_ERR_POLICY, "wait_scale must be > 0");
    for (int i = 0; i < 3; ++i)
        if (p->sla_weight[i] < 0) return fail(ctx, SJA_ERR_POLICY, "sla_weight must be >= 0");
    if (p->max_rounds < 0) return fail(ctx, SJA_ERR_POLICY, "max_rounds must be >= 0");
    const bool needs_wait = p->policy == SJA_POLICY_FAIRNESS || p->policy == SJA_POLICY_MIXED;
    const bool needs_class = p->policy == SJA_POLICY_SLA || p->policy == SJA_POLICY_MIXED;
    if (needs_wait && !wait) return fail(ctx, SJA_ERR_NULL, "wait is required by this policy");
    if (needs_class && !sla_class) return fail(ctx, SJA_ERR_NULL, "sla_class is required by this policy");
    return SJA_OK;
}

PolicyDev to_dev(const sja_params *p)
{
    PolicyDev d;
    d.policy = p->policy;
    d.wait_scale = p->wait_scale;
    d.w0 = p->sla_weight[0];
    d.w1 = p->sla_weight[1];
    d.w2 = p->sla_weight[2];
    d.class0_override = p->class0_override;
    return d;
}

// Enqueues the select kernels; outputs may be user or workspace arrays.  The
// per-prefix keys live in the space the list building of sja_resolve uses for
// its atom keys (the two never run at the same time); `keys_ready` says that an
// earlier call with the same policy inputs left them there and nothing has
// written that space since.
int launch_select(sja_ctx *ctx, hipStream_t st, const sja_params *params, const int32_t *wait,
                  const uint8_t *sla_class, const int32_t *job_held, const uint8_t *gap_active,
                  int32_t *cand_job, int32_t *cand_cut, int64_t *cand_score, bool keys_ready = false)
{
    const Layout L = make_layout(ctx->n_gaps, ctx->n_jobs, ctx->n_segments);
    const int G = ctx->n_gaps, J = ctx->n_jobs;
    if (G == 0) return SJA_OK;
    const int job_tiles = (J + kSelBlock - 1) / kSelBlock;
    unsigned long long *seg_key = ws_ptr<unsigned long long>(ctx, L.g_key_hi);
    if (job_tiles > 0 && !keys_ready) {
        const long long *pre_area = pre_area_of(ctx, L);
        auto kern = pre_area ? k_select_keys<true> : k_select_keys<false>;
        hipLaunchKernelGGL(kern, dim3((J + 3) / 4), dim3(256), 0, st, J, to_dev(params), ctx->seg_off, ctx->pre_dur,
                           ctx->pre_peak, pre_area, wait, sla_class, seg_key);
        SJA_HIP(hipGetLastError(), "k_select_keys launch");
    }
    if (job_tiles > 0) {
        const int n_chunks = (G + kSelGapChunk - 1) / kSelGapChunk;
        const int tiles8 = (job_tiles + 7) / 8 * 8;
        const unsigned grid = unsigned(tiles8) * unsigned(n_chunks);
        const bool mixed = params->policy == SJA_POLICY_MIXED;
        auto kern = mixed ? k_select_pass<true> : k_select_pass<false>;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kSelBlock), 0, st, J, G, n_chunks,
                           to_dev(params), ctx->seg_off, seg_key, ctx->cut,
                           ws_ptr<int32_t>(ctx, L.gap_order), wait, sla_class, job_held, gap_active,
                           ws_ptr<SelPartial>(ctx, L.sel_part));
        SJA_HIP(hipGetLastError(), "k_select_pass launch");
    }
    hipLaunchKernelGGL(k_select_reduce, dim3((G + 255) / 256), dim3(256), 0, st, G, job_tiles,
                       ws_ptr<SelPartial>(ctx, L.sel_part), cand_job, cand_cut, cand_score);
    SJA_HIP(hipGetLastError(), "k_select_reduce launch");
    return SJA_OK;
}


// Stable radix passes over bare 64-bit keys (key-only tiles) between two
// buffers, optionally with a 32-bit payload per key.  Only the bytes named in
// byte_mask are sorted on, lowest first (a byte that is the same in every key
// needs no pass).
int radix_sort_keys(sja_ctx *ctx, hipStream_t st, const Layout &L, const int32_t *n_dev, int64_t n_host,
                    unsigned byte_mask, int bit_offset, bool &flip, unsigned long long *const buf[2],
                    uint32_t *const pay[2], const KeyRecords *records = nullptr, bool *records_written = nullptr,
                    int sorted_bits = 64)
{
    // sorted_bits: bits above bit_offset + sorted_bits are not part of the order (a rider) and are masked
    // out of the last digit
    if (records_written) *records_written = false;
    if (n_host <= 0) return SJA_OK;
    int last_byte = -1;         // the pass that finishes the order: with `records` it writes those instead of keys
    for (int b = 0; b < 8; ++b)
        if (((byte_mask >> b) & 1u) && bit_offset + 8 * b < 64) last_byte = b;
    const int n_tiles = int((n_host + kKeyTile - 1) / kKeyTile);
    int32_t *hist = ws_ptr<int32_t>(ctx, L.g_hist);
    int32_t *tmp = ws_ptr<int32_t>(ctx, L.g_scan_tmp);
    for (int b = 0; b < 8; ++b) {
        if (!((byte_mask >> b) & 1u)) continue;
        const int shift = bit_offset + 8 * b;
        if (shift >= 64) break;
        const unsigned long long *src = buf[flip ? 1 : 0];
        unsigned long long *dst = buf[flip ? 0 : 1];
        const int live = sorted_bits - 8 * b;                   // bits of this digit that belong to the order
        if (live <= 0) break;
        const unsigned digit_mask = live >= 8 ? 255u : (1u << live) - 1u;
        hipLaunchKernelGGL(k_keys_hist, dim3(n_tiles), dim3(256), 0, st, src, n_dev, shift, digit_mask, hist, n_tiles);
        SJA_HIP(hipGetLastError(), "k_keys_hist launch");
        SJA_HIP(enqueue_scan(st, hist, int64_t(256) * n_tiles, tmp, nullptr), "radix scan launch");
        if (pay)
            hipLaunchKernelGGL((k_keys_scatter<true, false>), dim3(n_tiles), dim3(256), 0, st, src, dst, pay[flip ? 1 : 0],
                               pay[flip ? 0 : 1], n_dev, shift, digit_mask, hist, n_tiles, KeyRecords{});
        else if (records && b == last_byte) {
            hipLaunchKernelGGL((k_keys_scatter<false, true>), dim3(n_tiles), dim3(256), 0, st, src, dst,
                               static_cast<const uint32_t *>(nullptr), static_cast<uint32_t *>(nullptr), n_dev, shift,
                               digit_mask, hist, n_tiles, *records);
            if (records_written) *records_written = true;
        } else
            hipLaunchKernelGGL((k_keys_scatter<false, false>), dim3(n_tiles), dim3(256), 0, st, src, dst,
                               static_cast<const uint32_t *>(nullptr), static_cast<uint32_t *>(nullptr), n_dev, shift,
                               digit_mask, hist, n_tiles, KeyRecords{});
        SJA_HIP(hipGetLastError(), "k_keys_scatter launch");
        flip = !flip;
    }
    return SJA_OK;
}

int bits_for(int64_t n)
{
    int b = 1;
    while ((int64_t(1) << b) < n) ++b;
    return b;
}

// List-driven conflict rounds.  Returns SJA_OK with *done = true when it
// produced the grants, *done = false when the batch is outside what the lists
// serve (more than kMaxClasses capacities, or more list entries than the
// workspace holds) and the caller must take the matrix-scanning rounds.
int resolve_with_lists(sja_ctx *ctx, hipStream_t st, const Layout &L, const sja_params *params,
                       const int32_t *wait, const uint8_t *sla_class, int32_t *grant_job, int32_t *grant_cut,
                       int64_t *grant_score, int32_t *job_gap, int64_t cap, int32_t result[2], bool *done)
{
    *done = false;
    const int G = ctx->n_gaps, J = ctx->n_jobs;
    const int sub_bound = int(fit_sub_bound(G, J));
    const int lb_bound = int(list_block_bound(G, J));
    const PolicyDev pol = to_dev(params);
    int32_t *plan = ws_ptr<int32_t>(ctx, L.plan);
    int32_t *abase = ws_ptr<int32_t>(ctx, L.g_abase);
    int32_t *tmp = ws_ptr<int32_t>(ctx, L.g_scan_tmp);
    int32_t *counters = ws_ptr<int32_t>(ctx, L.res_counters);      // [0..1] entries (64 bit), [2] atoms, [4..7] key bits
    int32_t *list_off = ws_ptr<int32_t>(ctx, L.g_list_off);
    const int2 *atom_dp = ws_ptr<int2>(ctx, L.atom_dp);
    const int2 *atom_db = ws_ptr<int2>(ctx, L.atom_db);
    const int32_t *sub_begin = ws_ptr<int32_t>(ctx, L.sub_begin), *sub_end = ws_ptr<int32_t>(ctx, L.sub_end);
    const int32_t *sub_class = ws_ptr<int32_t>(ctx, L.sub_class);
    int32_t *lb_begin = ws_ptr<int32_t>(ctx, L.lb_begin), *lb_end = ws_ptr<int32_t>(ctx, L.lb_end);
    int32_t *lb_sub = ws_ptr<int32_t>(ctx, L.lb_sub), *lb_off = ws_ptr<int32_t>(ctx, L.lb_off);
    const int32_t *ncap_tab = ws_ptr<int32_t>(ctx, L.ncap_tab);
    const int32_t *gap_w = ws_ptr<int32_t>(ctx, L.gap_w);
    unsigned long long *key_hi = ws_ptr<unsigned long long>(ctx, L.g_key_hi);
    unsigned long long *key_lo = ws_ptr<unsigned long long>(ctx, L.g_key_lo);
    uint32_t *perm[2] = {ws_ptr<uint32_t>(ctx, L.g_perm0), ws_ptr<uint32_t>(ctx, L.g_perm1)};
    uint32_t *rank = ws_ptr<uint32_t>(ctx, L.g_rank);
    unsigned long long *ekey[2] = {ws_ptr<unsigned long long>(ctx, L.g_ekey0), ws_ptr<unsigned long long>(ctx, L.g_ekey1)};
    int2 *atom_ja = ws_ptr<int2>(ctx, L.g_atom_ja), *ranked = ws_ptr<int2>(ctx, L.g_ranked);

    // 1. list blocks; reachable atoms per job -> compact atom ids
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(256), 0, st, counters, int64_t(16), 0);
    hipLaunchKernelGGL(k_fill_i32, dim3((lb_bound + 2 + 255) / 256), dim3(256), 0, st, list_off, int64_t(lb_bound + 2), 0);
    hipLaunchKernelGGL(k_list_blocks_count, dim3((sub_bound + 1 + 255) / 256), dim3(256), 0, st, sub_bound + 1, plan, sub_begin,
                       sub_end, gap_w, lb_off);
    SJA_HIP(enqueue_scan(st, lb_off, int64_t(sub_bound) + 1, tmp, plan + kPlanListBlocks), "list block scan launch");
    hipLaunchKernelGGL(k_list_blocks_write, dim3((sub_bound + 255) / 256), dim3(256), 0, st, lb_bound, plan, sub_begin,
                       sub_end, gap_w, lb_off, lb_begin, lb_end, lb_sub);
    SJA_HIP(hipGetLastError(), "list block launch");
    // where every sub-block starts in every job's atom list (the fit only keeps this per chunk)
    int32_t *sub_tab = ws_ptr<int32_t>(ctx, L.sub_tab);
    const int starts_jobs = kStartsJobs;
    hipLaunchKernelGGL(k_fit_starts, dim3((J + starts_jobs - 1) / starts_jobs), dim3(256), 0, st, J, int(kPlanSubBlocks), plan,
                       ws_ptr<int32_t>(ctx, L.class_begin), sub_begin, sub_class, gap_w, ws_ptr<int32_t>(ctx, L.gap_c),
                       ctx->seg_off, atom_dp, ws_ptr<int32_t>(ctx, L.n_atoms), sub_tab, static_cast<int32_t *>(nullptr));
    SJA_HIP(hipGetLastError(), "k_fit_starts launch");
    hipLaunchKernelGGL(k_reach, dim3((J + 1 + 255) / 256), dim3(256), 0, st, J, plan, ncap_tab, abase);
    SJA_HIP(hipGetLastError(), "k_reach launch");
    SJA_HIP(enqueue_scan(st, abase, int64_t(J) + 1, tmp, counters + 2), "atom scan launch");
    // policy keys of the atoms and the bytes in which they differ (both only need the device-side counts)
    hipLaunchKernelGGL(k_atom_keys, dim3((J + 3) / 4), dim3(256), 0, st, J, pol, ctx->seg_off, atom_dp,
                       atom_area_of(ctx, L), abase, wait,
                       sla_class, key_hi, key_lo, perm[0], atom_ja);
    SJA_HIP(hipGetLastError(), "k_atom_keys launch");
    hipLaunchKernelGGL(k_key_bits, dim3(256), dim3(256), 0, st, counters + 2, key_hi, key_lo,
                       reinterpret_cast<unsigned long long *>(counters + 4));
    SJA_HIP(hipGetLastError(), "k_key_bits launch");
    int32_t host_plan[kPlanWords] = {0}, host_counters[8] = {0};
    SJA_HIP(hipMemcpyAsync(host_plan, plan, sizeof(host_plan), hipMemcpyDeviceToHost, st), "plan readback");
    SJA_HIP(hipMemcpyAsync(host_counters, counters, sizeof(host_counters), hipMemcpyDeviceToHost, st), "count readback");
    SJA_HIP(hipStreamSynchronize(st), "count synchronise");
    const int64_t n_atoms = host_counters[2];
    const int n_subs = host_plan[kPlanListBlocks];          // list blocks from here on
    if (!host_plan[kPlanTabled] || n_subs > lb_bound || n_atoms > L.atom_cap) return SJA_OK;

    // 2. rank the atoms by policy key (descending key, ascending job id): stable passes over
    //    (inverted key, atom id) pairs, the secondary key first; the entry buffers serve as the
    //    second key buffer, they are not in use yet
    if (n_atoms > 0) {
        unsigned long long bits_hi = 0, bits_lo = 0;
        memcpy(&bits_hi, host_counters + 4, 8);
        memcpy(&bits_lo, host_counters + 6, 8);
        auto bytes_of = [](unsigned long long v) {
            unsigned m = 0;
            for (int b = 0; b < 8; ++b) if ((v >> (8 * b)) & 0xffull) m |= 1u << b;
            return m;
        };
        bool flip = false;      // where the atom ids are: perm[flip]
        int rc = SJA_OK;
        if (params->policy == SJA_POLICY_MIXED) {
            unsigned long long *kb[2] = {key_lo, ekey[0]};
            rc = radix_sort_keys(ctx, st, L, counters + 2, n_atoms, bytes_of(bits_lo), 0, flip, kb, perm);
            if (rc != SJA_OK) return rc;
        }
        // the primary keys in the order reached so far
        unsigned long long *kh[2] = {ekey[1], ekey[0]};
        if (flip) { kh[0] = ekey[0]; kh[1] = ekey[1]; }      // buffer index must follow the id buffers
        hipLaunchKernelGGL(k_gather_keys, dim3(unsigned((n_atoms + 255) / 256)), dim3(256), 0, st, counters + 2, key_hi,
                           perm[flip ? 1 : 0], kh[flip ? 1 : 0]);
        SJA_HIP(hipGetLastError(), "k_gather_keys launch");
        rc = radix_sort_keys(ctx, st, L, counters + 2, n_atoms, bytes_of(bits_hi), 0, flip, kh, perm);
        if (rc != SJA_OK) return rc;
        hipLaunchKernelGGL(k_rank_from_perm, dim3(unsigned((n_atoms + 255) / 256)), dim3(256), 0, st, counters + 2,
                           perm[flip ? 1 : 0], atom_ja, rank, ranked);
        SJA_HIP(hipGetLastError(), "k_rank_from_perm launch");
    }

    // 3. list entries (one pass, counted as they are written), then sorted by (block, rank)
    const int rank_bits = bits_for(n_atoms > 1 ? n_atoms : 2);
    const int sub_bits = bits_for(n_subs > 1 ? n_subs : 2);
    // the job of an entry rides in its key above the sorted bits when the key has room for it:
    // then the pass that writes the records need not look it up through the rank
    const int job_bits = bits_for(J > 1 ? J : 2);
    const bool ride = ctx->resolve_mode != SJA_RESOLVE_LISTS_LOOKUP && kEntryLaneBits + rank_bits + sub_bits + job_bits <= 64;
    const int job_shift = ride ? kEntryLaneBits + rank_bits + sub_bits : -1;
    const dim3 emit_grid((J + 256 * kEmitTiles - 1) / (256 * kEmitTiles), lb_bound);
    hipLaunchKernelGGL(k_list_emit, emit_grid, dim3(256), 0, st, J, rank_bits, job_shift, lb_bound, (long long)L.entry_cap, plan,
                       lb_begin, lb_end, lb_sub, sub_class, gap_w, ctx->seg_off, atom_dp, sub_tab, ncap_tab, abase, rank,
                       list_off, reinterpret_cast<unsigned long long *>(counters), ekey[0]);
    SJA_HIP(hipGetLastError(), "k_list_emit launch");
    long long n_entries = 0;
    SJA_HIP(hipMemcpyAsync(&n_entries, counters, sizeof(n_entries), hipMemcpyDeviceToHost, st), "entry count readback");
    SJA_HIP(hipStreamSynchronize(st), "entry count synchronise");
    if (n_entries > L.entry_cap || n_entries >= (1ll << 31)) return SJA_OK;
    SJA_HIP(enqueue_scan(st, list_off, int64_t(lb_bound) + 2, tmp, nullptr), "list offset scan launch");
    bool eflip = false, packed = false;
    uint4 *rec = ws_ptr<uint4>(ctx, L.g_rec);
    const KeyRecords records{ranked, rec, kEntryLaneBits, rank_bits, job_shift};
    if (n_entries > 0) {
        // the pass that finishes the order writes the 16-byte records straight away
        const int key_bytes = (rank_bits + sub_bits + 7) / 8;
        int rc = radix_sort_keys(ctx, st, L, counters, n_entries, (1u << key_bytes) - 1u, kEntryLaneBits, eflip, ekey,
                                 nullptr, &records, &packed, rank_bits + sub_bits);
        if (rc != SJA_OK) return rc;
    }
    const int fb = eflip ? 1 : 0;
    if (n_entries > 0 && !packed) {
        hipLaunchKernelGGL(k_list_pack, dim3(unsigned((n_entries + 255) / 256)), dim3(256), 0, st, counters, ekey[fb],
                           records);
        SJA_HIP(hipGetLastError(), "k_list_pack launch");
    }

    // 4. rounds
    int32_t *cnt_lost = ws_ptr<int32_t>(ctx, L.g_cnt_lost), *cnt_cand = ws_ptr<int32_t>(ctx, L.g_cnt_cand);
    const int64_t rounds_cap = int64_t(G < J ? G : J) + 4;
    hipLaunchKernelGGL(k_fill_i32, dim3(unsigned((rounds_cap + 255) / 256)), dim3(256), 0, st, cnt_lost, rounds_cap, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(unsigned((rounds_cap + 255) / 256)), dim3(256), 0, st, cnt_cand, rounds_cap, 0);
    SJA_HIP(hipGetLastError(), "counter fill launch");
    const int32_t *gap_order = ws_ptr<int32_t>(ctx, L.gap_order);
    unsigned long long *claim = ws_ptr<unsigned long long>(ctx, L.res_claim);
    int4 *state = ws_ptr<int4>(ctx, L.g_state);
    const int round_grid = (n_subs + kRoundBlock / kWave - 1) / (kRoundBlock / kWave);

    // one launch per round, in batches between looks at the flags
    // the first kHeldRounds rounds keep the held jobs as a bitmap too (two alternating copies), if it fits LDS
    const int held_words = held_bitmap_words(J);
    const bool use_held = held_words <= kHeldMaxWords;
    uint32_t *held = ws_ptr<uint32_t>(ctx, L.g_held);
    if (use_held) {
        hipLaunchKernelGGL(k_fill_i32, dim3((2 * held_words + 255) / 256), dim3(256), 0, st,
                           reinterpret_cast<int32_t *>(held), int64_t(2) * held_words, 0);
        SJA_HIP(hipGetLastError(), "k_fill_i32 launch");
    }
    auto launch_round = [&](int64_t k, int propose) {
        if (use_held && k <= kHeldRounds)
            hipLaunchKernelGGL(k_grant_round<true>, dim3(round_grid), dim3(kRoundBlock), 0, st, state, list_off, rec, claim, int(k), propose, n_subs,
                               held_words, held, lb_begin, lb_end, gap_order, cnt_lost, cnt_cand);
        else
            hipLaunchKernelGGL(k_grant_round<false>, dim3(round_grid), dim3(kRoundBlock), 0, st, state, list_off, rec, claim, int(k), propose, n_subs,
                               0, static_cast<uint32_t *>(nullptr), lb_begin, lb_end, gap_order, cnt_lost, cnt_cand);
        return hipGetLastError();
    };
    std::vector<int32_t> h_lost, h_cand;
    int64_t launched = 0;        // kernels 1..launched have been enqueued
    int64_t next_check = 1;      // first round whose end is not yet decided
    bool finished = false;
    int64_t batch = 64;          // rounds enqueued between looks at the flags; grows, a finished batch costs little
    while (!finished) {
        const int64_t upto = (launched + batch < cap) ? launched + batch : cap;
        if (batch < 1024) batch *= 2;
        for (int64_t k = launched + 1; k <= upto; ++k) SJA_HIP(launch_round(k, 1), "k_grant_round launch");
        if (upto == cap) SJA_HIP(launch_round(cap + 1, 0), "k_grant_round launch");
        launched = upto;
        hipLaunchKernelGGL(k_count_open, dim3(1), dim3(1024), 0, st, lb_bound, plan, state, counters + 12);
        SJA_HIP(hipGetLastError(), "k_count_open launch");
        const int64_t known = (upto == cap) ? cap + 1 : upto;        // kernels that have run
        h_lost.resize(size_t(known + 1));
        h_cand.resize(size_t(known + 1));
        SJA_HIP(hipMemcpyAsync(h_lost.data(), cnt_lost, size_t(known + 1) * 4, hipMemcpyDeviceToHost, st), "round counters");
        SJA_HIP(hipMemcpyAsync(h_cand.data(), cnt_cand, size_t(known + 1) * 4, hipMemcpyDeviceToHost, st), "round counters");
        int32_t h_open = 0;
        SJA_HIP(hipMemcpyAsync(&h_open, counters + 12, 4, hipMemcpyDeviceToHost, st), "open count");
        SJA_HIP(hipStreamSynchronize(st), "round synchronise");
        // every further round grants at least one open position: no point in enqueueing more than that
        if (int64_t(h_open) + 1 < batch) batch = int64_t(h_open) + 1;
        for (int64_t r = next_check; r <= upto; ++r) {
            if (h_cand[size_t(r)] == 0) { result[0] = int32_t(r); result[1] = 1; finished = true; break; }
            if (r + 1 > known) { next_check = r; break; }              // losers of r not counted yet
            if (h_lost[size_t(r)] == 0) { result[0] = int32_t(r); result[1] = 1; finished = true; break; }
            if (r == cap) { result[0] = int32_t(cap); result[1] = 0; finished = true; break; }
            next_check = r + 1;
        }
    }
    hipLaunchKernelGGL(k_grant_finish, dim3(unsigned((int64_t(n_subs) * kWave + 255) / 256)), dim3(256), 0, st, lb_bound, pol,
                       plan, state, ranked, ctx->seg_off, atom_dp, atom_db, atom_area_of(ctx, L), wait, sla_class, grant_job,
                       grant_cut, grant_score,
                       job_gap);
    SJA_HIP(hipGetLastError(), "k_grant_finish launch");
    *done = true;
    return SJA_OK;
}

// Gap ordering, capacity classes, chunk / sub-block plan and the start tables
// for a batch of gaps: everything the stepping kernels need before they run.
int enqueue_gap_plan(sja_ctx *ctx, hipStream_t st, const Layout &L, int32_t n_gaps, const int32_t *W, const int32_t *C)
{
    const int J = ctx->n_jobs;
    const int gc = fit_chunk_len(n_gaps, J);
    const int chunk_bound = int(fit_chunk_bound(n_gaps, J));
    const int sb = fit_sub_len(n_gaps, J);
    const int sub_bound = int(fit_sub_bound(n_gaps, J));
    const dim3 per_gap((n_gaps + 255) / 256), b256(256);
    int32_t *rank = ws_ptr<int32_t>(ctx, L.gap_rank);
    int32_t *gw = ws_ptr<int32_t>(ctx, L.gap_w), *gcap = ws_ptr<int32_t>(ctx, L.gap_c);
    int32_t *plan = ws_ptr<int32_t>(ctx, L.plan);
    const int gap_tiles = (n_gaps + kGapTile - 1) / kGapTile;
    unsigned long long *tile_key = ws_ptr<unsigned long long>(ctx, L.gap_tile_key);
    int32_t *tile_idx = ws_ptr<int32_t>(ctx, L.gap_tile_idx);
    hipLaunchKernelGGL(k_gap_tile_sort, dim3(gap_tiles), dim3(kGapSortThreads), 0, st, n_gaps, W, C, tile_key, tile_idx,
                       plan, ws_ptr<int32_t>(ctx, L.class_dmax));
    SJA_HIP(hipGetLastError(), "k_gap_tile_sort launch");
    hipLaunchKernelGGL(k_gap_rank, dim3(gap_tiles * (kGapTile / kGapRankBlock)), dim3(kGapRankBlock), 0, st, n_gaps, J,
                       gap_tiles, tile_key, tile_idx, W, C, rank, ws_ptr<int32_t>(ctx, L.gap_order), gw, gcap,
                       ws_ptr<int64_t>(ctx, L.gap_row));
    SJA_HIP(hipGetLastError(), "k_gap_rank launch");
    if (J > 0) {
        int32_t *marks = ws_ptr<int32_t>(ctx, L.class_marks);
        hipLaunchKernelGGL(k_gap_marks, per_gap, b256, 0, st, n_gaps, gcap, plan, marks);
        SJA_HIP(hipGetLastError(), "k_gap_marks launch");
        const int plan_blocks = (n_gaps + 255) / 256 < 64 ? (n_gaps + 255) / 256 : 64;
        hipLaunchKernelGGL(k_gap_plan, dim3(plan_blocks), b256, 0, st, n_gaps, gc, sb, chunk_bound, sub_bound, gcap, marks,
                           plan, ws_ptr<int32_t>(ctx, L.class_begin), ws_ptr<int32_t>(ctx, L.class_chunk0),
                           ws_ptr<int32_t>(ctx, L.class_sub0), ws_ptr<int32_t>(ctx, L.chunk_begin),
                           ws_ptr<int32_t>(ctx, L.chunk_end), ws_ptr<int32_t>(ctx, L.chunk_class),
                           ws_ptr<int32_t>(ctx, L.chunk_sub), ws_ptr<int32_t>(ctx, L.sub_begin),
                           ws_ptr<int32_t>(ctx, L.sub_end), ws_ptr<int32_t>(ctx, L.sub_class),
                           ws_ptr<int32_t>(ctx, L.gap_cls), ws_ptr<int32_t>(ctx, L.gap_run_end));
        SJA_HIP(hipGetLastError(), "k_gap_plan launch");
        const int jobs_per_block = kStartsJobs;
        hipLaunchKernelGGL(k_fit_starts, dim3((J + jobs_per_block - 1) / jobs_per_block), b256, 0, st, J, int(kPlanChunks),
                           plan, ws_ptr<int32_t>(ctx, L.class_begin), ws_ptr<int32_t>(ctx, L.chunk_begin),
                           ws_ptr<int32_t>(ctx, L.chunk_class), gw, gcap, ctx->seg_off, ws_ptr<int2>(ctx, L.atom_dp),
                           ws_ptr<int32_t>(ctx, L.n_atoms), ws_ptr<int32_t>(ctx, L.start_tab),
                           ws_ptr<int32_t>(ctx, L.ncap_tab));
        SJA_HIP(hipGetLastError(), "k_fit_starts launch");
    }
    return SJA_OK;
}

JobLimits job_limits(const sja_limits &l, const int32_t *power, const int32_t *deadline)
{
    JobLimits out;
    out.tau_min = l.tau_min;
    out.tau_max = l.tau_max;
    out.power_cap = l.power_cap;
    out.now = l.now;
    out.power = power;
    out.deadline = deadline;
    return out;
}

// The fused fit -> select pass over the planned batch of gaps (the plan of enqueue_gap_plan is in
// the workspace): candidates per gap among the jobs that job_held does not mark, for the gaps that
// gap_active does not switch off.  No cut matrix is read or written.
int launch_fused(sja_ctx *ctx, hipStream_t st, const Layout &L, int32_t n_gaps, const sja_params *params,
                 const int32_t *wait, const uint8_t *sla_class, const int32_t *job_held, const uint8_t *gap_active,
                 int32_t *cand_job, int32_t *cand_cut, int64_t *cand_score, bool timed)
{
    const int J = ctx->n_jobs;
    const int job_tiles = (J + kFusedBlock - 1) / kFusedBlock;
    if (job_tiles > 0) {
        const int chunk_bound = int(fit_chunk_bound(n_gaps, J));
        const int tiles8 = (job_tiles + 7) / 8 * 8;
        const unsigned grid = unsigned(tiles8) * unsigned(chunk_bound);
        const bool mixed = params->policy == SJA_POLICY_MIXED;
        const long long *atom_area = atom_area_of(ctx, L);
        auto kern = atom_area ? (mixed ? k_fit_select<kFusedBlock, kFusedWindow, kFusedPeriod, true, true>
                                       : k_fit_select<kFusedBlock, kFusedWindow, kFusedPeriod, false, true>)
                              : (mixed ? k_fit_select<kFusedBlock, kFusedWindow, kFusedPeriod, true, false>
                                       : k_fit_select<kFusedBlock, kFusedWindow, kFusedPeriod, false, false>);
        if (timed) {
            if (!ctx->ev_start) {
                SJA_HIP(hipEventCreate(&ctx->ev_start), "hipEventCreate");
                SJA_HIP(hipEventCreate(&ctx->ev_stop), "hipEventCreate");
            }
            SJA_HIP(hipEventRecord(ctx->ev_start, st), "hipEventRecord");
        }
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kFusedBlock), 0, st, J, n_gaps, chunk_bound, to_dev(params),
                           ctx->seg_off, ws_ptr<int2>(ctx, L.atom_dp), atom_area, ws_ptr<int32_t>(ctx, L.n_atoms),
                           ws_ptr<int32_t>(ctx, L.plan), ws_ptr<int32_t>(ctx, L.chunk_begin),
                           ws_ptr<int32_t>(ctx, L.chunk_end), ws_ptr<int32_t>(ctx, L.chunk_class),
                           ws_ptr<int32_t>(ctx, L.chunk_sub), ws_ptr<int32_t>(ctx, L.start_tab),
                           ws_ptr<int32_t>(ctx, L.ncap_tab), ws_ptr<int32_t>(ctx, L.gap_w),
                           ws_ptr<int32_t>(ctx, L.gap_c), ws_ptr<int32_t>(ctx, L.gap_order),
                           ws_ptr<int32_t>(ctx, L.gap_run_end), wait, sla_class, job_held, gap_active,
                           ws_ptr<SelPartial>(ctx, L.sel_part));
        SJA_HIP(hipGetLastError(), "k_fit_select launch");
        if (timed) {
            SJA_HIP(hipEventRecord(ctx->ev_stop, st), "hipEventRecord");
            ctx->timed = true;
        }
    }
    hipLaunchKernelGGL(k_fused_reduce, dim3((n_gaps + 255) / 256), dim3(256), 0, st, n_gaps, job_tiles,
                       ws_ptr<SelPartial>(ctx, L.sel_part), ctx->seg_off, ws_ptr<int2>(ctx, L.atom_db), cand_job,
                       cand_cut, cand_score);
    SJA_HIP(hipGetLastError(), "k_fused_reduce launch");
    return SJA_OK;
}

Hysteresis hysteresis_of(int32_t n_caps, int32_t min_gain, const int32_t *cap)
{
    Hysteresis h{};
    h.n_caps = n_caps;
    h.min_gain = min_gain;
    for (int i = 0; i < n_caps; ++i) h.cap[i] = cap[i];
    return h;
}

// sja_prepare_profiles and its variant on the built-in scratch: the same checks and the same
// kernel; only where the private tables live differs.
int prepare_into(sja_ctx *ctx, void *stream, int32_t n_jobs, int64_t n_segments,
                 const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                 const uint8_t *safe, const int32_t *progress, int32_t *pre_dur,
                 int32_t *pre_peak, int32_t *prev_safe, bool on_static_scratch)
{
    ctx->prepared = false;
    ctx->fitted = false;
    ctx->planned = false;
    if (n_jobs < 0 || n_jobs > SJA_MAX_JOBS) return fail(ctx, SJA_ERR_SIZE, "n_jobs");
    if (n_segments < 0 || n_segments > SJA_MAX_SEGMENTS) return fail(ctx, SJA_ERR_SIZE, "n_segments");
    if (!seg_off || !progress) return fail(ctx, SJA_ERR_NULL, "seg_off / progress");
    if (n_segments > 0 && (!dur || !mem || !safe || !pre_dur || !pre_peak || !prev_safe))
        return fail(ctx, SJA_ERR_NULL, "profile or output array");
    const Layout L = make_layout(0, n_jobs, n_segments);
    if (on_static_scratch) {
        if (L.total > size_t(SJA_STATIC_SCRATCH_BYTES))
            return fail(ctx, SJA_ERR_SIZE, "n_jobs / n_segments beyond what the built-in scratch holds "
                                           "(sja_workspace_bytes(0, n_jobs, n_segments) > SJA_STATIC_SCRATCH_BYTES)");
    } else if (!ctx->ws || ctx->ws_bytes < L.total) {
        return fail(ctx, SJA_ERR_WORKSPACE, "workspace too small for prepare");
    }

    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    if (on_static_scratch) {
        void *p = nullptr;
        SJA_HIP(static_scratch(ctx->device, &p), "hipGetSymbolAddress(scratch)");
        ctx->ws = static_cast<char *>(p);
        ctx->ws_bytes = size_t(SJA_STATIC_SCRATCH_BYTES);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_jobs > 0) {
        const int jobs_per_block = 256 / kWave;
        const dim3 grid((n_jobs + jobs_per_block - 1) / jobs_per_block), block(256);
        const bool by_area = ctx->score_mode == SJA_SCORE_AREA;
        const Hysteresis hyst = hysteresis_of(ctx->hyst_n_caps, ctx->hyst_min_gain, ctx->hyst_cap);
        long long *pre_area = by_area ? ws_ptr<long long>(ctx, L.pre_area) : nullptr;
        long long *atom_area = by_area || hyst.n_caps > 0 ? ws_ptr<long long>(ctx, L.atom_area) : nullptr;
        if (ctx->limits_on) {
            const JobLimits lim = job_limits(ctx->limits, ctx->lim_power, ctx->lim_deadline);
            hipLaunchKernelGGL(k_prepare<true>, grid, block, 0, st, lim, hyst, pre_area, atom_area, n_jobs, seg_off, dur, mem, safe, progress,
                               pre_dur, pre_peak, prev_safe, ws_ptr<int2>(ctx, L.atom_dp),
                               ws_ptr<int2>(ctx, L.atom_db), ws_ptr<int32_t>(ctx, L.n_atoms),
                               ws_ptr<int2>(ctx, L.first_dp));
        } else {
            hipLaunchKernelGGL(k_prepare<false>, grid, block, 0, st, JobLimits{}, hyst, pre_area, atom_area, n_jobs, seg_off, dur, mem, safe,
                               progress, pre_dur, pre_peak, prev_safe, ws_ptr<int2>(ctx, L.atom_dp),
                               ws_ptr<int2>(ctx, L.atom_db), ws_ptr<int32_t>(ctx, L.n_atoms),
                               ws_ptr<int2>(ctx, L.first_dp));
        }
        SJA_HIP(hipGetLastError(), "k_prepare launch");
    }
    ctx->limits_used = ctx->limits_on;
    ctx->score_used = ctx->score_mode;
    ctx->hyst_used_n_caps = ctx->hyst_n_caps;
    ctx->hyst_used_min_gain = ctx->hyst_min_gain;
    memcpy(ctx->hyst_used_cap, ctx->hyst_cap, sizeof(ctx->hyst_cap));
    ctx->limits_applied = ctx->limits;
    ctx->used_power = ctx->lim_power;
    ctx->used_deadline = ctx->lim_deadline;
    ctx->n_jobs = n_jobs;
    ctx->n_segments = n_segments;
    ctx->seg_off = seg_off;
    ctx->dur = dur;
    ctx->mem = mem;
    ctx->safe = safe;
    ctx->pre_dur = pre_dur;
    ctx->pre_peak = pre_peak;
    ctx->prev_safe = prev_safe;
    ctx->prepared = true;
    return SJA_OK;
}

}  // namespace

extern "C" {

const char *sja_status_string(int status)
{
    switch (status) {
    case SJA_OK: return "SJA_OK";
    case SJA_ERR_NULL: return "SJA_ERR_NULL";
    case SJA_ERR_SIZE: return "SJA_ERR_SIZE";
    case SJA_ERR_POLICY: return "SJA_ERR_POLICY";
    case SJA_ERR_STATE: return "SJA_ERR_STATE";
    case SJA_ERR_OVERFLOW: return "SJA_ERR_OVERFLOW";
    case SJA_ERR_WORKSPACE: return "SJA_ERR_WORKSPACE";
    case SJA_ERR_HIP: return "SJA_ERR_HIP";
    case SJA_ERR_NOT_IMPLEMENTED: return "SJA_ERR_NOT_IMPLEMENTED";
    default: return "SJA_ERR_UNKNOWN";
    }
}

const char *sja_last_error(const sja_ctx *ctx) { return ctx ? ctx->err : "null context"; }

int sja_create(sja_ctx **out, int device_id)
{
    if (!out) return SJA_ERR_NULL;
    *out = nullptr;
    if (device_id < 0) return SJA_ERR_SIZE;
    sja_ctx *ctx = new (std::nothrow) sja_ctx();
    if (!ctx) return SJA_ERR_WORKSPACE;
    memset(ctx, 0, sizeof(*ctx));
    ctx->device = device_id;
    *out = ctx;
    return SJA_OK;
}

int sja_destroy(sja_ctx *ctx)
{
    if (!ctx) return SJA_ERR_NULL;
    if (ctx->ev_start) (void)hipEventDestroy(ctx->ev_start);
    if (ctx->ev_stop) (void)hipEventDestroy(ctx->ev_stop);
    delete ctx;
    return SJA_OK;
}

size_t sja_workspace_bytes(int64_t n_gaps, int64_t n_jobs, int64_t n_segments)
{
    if (n_gaps < 0 || n_jobs < 0 || n_segments < 0) return 0;
    if (n_gaps > SJA_MAX_GAPS || n_jobs > SJA_MAX_JOBS || n_segments > SJA_MAX_SEGMENTS) return 0;
    return make_layout(n_gaps, n_jobs, n_segments).total;
}

int sja_set_workspace(sja_ctx *ctx, void *dev_ptr, size_t bytes)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!dev_ptr && bytes) return fail(ctx, SJA_ERR_NULL, "workspace pointer");
    if (reinterpret_cast<uintptr_t>(dev_ptr) & 255) return fail(ctx, SJA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    ctx->ws = static_cast<char *>(dev_ptr);
    ctx->ws_bytes = bytes;
    ctx->prepared = false;   // private tables lived in the old workspace
    ctx->fitted = false;
    ctx->planned = false;
    return SJA_OK;
}

int sja_validate(sja_ctx *ctx, void *stream, int32_t n_jobs, int64_t n_segments, const int64_t *seg_off,
                 const int32_t *dur, const int32_t *mem, const int32_t *progress, const sja_params *params,
                 const int32_t *wait, const uint8_t *sla_class, uint32_t *problems)
{
    if (!ctx) return SJA_ERR_NULL;
    if (n_jobs < 0 || n_jobs > SJA_MAX_JOBS) return fail(ctx, SJA_ERR_SIZE, "n_jobs");
    if (n_segments < 0 || n_segments > SJA_MAX_SEGMENTS) return fail(ctx, SJA_ERR_SIZE, "n_segments");
    if (!seg_off || !problems) return fail(ctx, SJA_ERR_NULL, "seg_off / problems");
    if (n_jobs > 0 && !progress) return fail(ctx, SJA_ERR_NULL, "progress");
    if (n_segments > 0 && (!dur || !mem)) return fail(ctx, SJA_ERR_NULL, "dur / mem");
    PolicyDev pol{};
    if (params) {
        const int rc = check_params(ctx, params, wait, sla_class);
        if (rc != SJA_OK) return rc;
        pol = to_dev(params);
    }
    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, reinterpret_cast<int32_t *>(problems), int64_t(1), 0);
    SJA_HIP(hipGetLastError(), "k_fill_i32 launch");
    if (n_jobs > 0) {
        const int jobs_per_block = 256 / kWave;
        hipLaunchKernelGGL(k_validate, dim3((n_jobs + jobs_per_block - 1) / jobs_per_block), dim3(256), 0, st, n_jobs,
                           n_segments, seg_off, dur, mem, progress, params != nullptr, pol, wait, sla_class, problems);
        SJA_HIP(hipGetLastError(), "k_validate launch");
    }
    return SJA_OK;
}

int sja_enable_timing(sja_ctx *ctx, int on)
{
    if (!ctx) return SJA_ERR_NULL;
    ctx->timing = on != 0;
    ctx->timed = false;
    return SJA_OK;
}

int sja_set_resolve_mode(sja_ctx *ctx, int mode)
{
    if (!ctx) return SJA_ERR_NULL;
    if (mode != SJA_RESOLVE_LISTS && mode != SJA_RESOLVE_MATRIX && mode != SJA_RESOLVE_LISTS_LOOKUP)
        return fail(ctx, SJA_ERR_SIZE, "sja_set_resolve_mode: unknown mode");
    ctx->resolve_mode = mode;
    return SJA_OK;
}

int sja_last_fit_kernel_ms(sja_ctx *ctx, float *ms_host)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!ms_host) return fail(ctx, SJA_ERR_NULL, "ms_host");
    if (!ctx->timed) return fail(ctx, SJA_ERR_STATE, "no timed sja_fit has run");
    SJA_HIP(hipEventSynchronize(ctx->ev_stop), "hipEventSynchronize");
    SJA_HIP(hipEventElapsedTime(ms_host, ctx->ev_start, ctx->ev_stop), "hipEventElapsedTime");
    return SJA_OK;
}

int sja_set_score(sja_ctx *ctx, int score)
{
    if (!ctx) return SJA_ERR_NULL;
    if (score != SJA_SCORE_RECTANGLE && score != SJA_SCORE_AREA) return fail(ctx, SJA_ERR_SIZE, "unknown score");
    ctx->score_mode = score;
    return SJA_OK;
}

int sja_set_limits(sja_ctx *ctx, const sja_limits *limits, const int32_t *power, const int32_t *deadline)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!limits) {
        ctx->limits_on = false;
        ctx->lim_power = nullptr;
        ctx->lim_deadline = nullptr;
        return SJA_OK;
    }
    if (limits->tau_min < 0 || limits->tau_max < 0) return fail(ctx, SJA_ERR_SIZE, "tau_min / tau_max");
    ctx->limits = *limits;
    ctx->lim_power = power;
    ctx->lim_deadline = deadline;
    ctx->limits_on = true;
    return SJA_OK;
}

int sja_set_hysteresis(sja_ctx *ctx, int32_t n_caps, const int32_t *cap_set, int32_t min_gain)
{
    if (!ctx) return SJA_ERR_NULL;
    if (n_caps < 0 || n_caps > SJA_MAX_CAPS) return fail(ctx, SJA_ERR_SIZE, "n_caps");
    if (n_caps == 0) {
        ctx->hyst_n_caps = 0;
        return SJA_OK;
    }
    if (!cap_set) return fail(ctx, SJA_ERR_NULL, "cap_set");
    if (min_gain < 1) return fail(ctx, SJA_ERR_SIZE, "min_gain must be >= 1");
    for (int i = 1; i < n_caps; ++i)
        if (cap_set[i] < cap_set[i - 1]) return fail(ctx, SJA_ERR_SIZE, "cap_set must ascend");
    ctx->hyst_n_caps = n_caps;
    ctx->hyst_min_gain = min_gain;
    for (int i = 0; i < n_caps; ++i) ctx->hyst_cap[i] = cap_set[i];
    return SJA_OK;
}

int sja_prepare_profiles(sja_ctx *ctx, void *stream, int32_t n_jobs, int64_t n_segments,
                         const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                         const uint8_t *safe, const int32_t *progress, int32_t *pre_dur,
                         int32_t *pre_peak, int32_t *prev_safe)
{
    if (!ctx) return SJA_ERR_NULL;
    return prepare_into(ctx, stream, n_jobs, n_segments, seg_off, dur, mem, safe, progress, pre_dur, pre_peak,
                        prev_safe, false);
}

int sja_prepare_profiles_static(sja_ctx *ctx, void *stream, int32_t n_jobs, int64_t n_segments,
                                const int64_t *seg_off, const int32_t *dur, const int32_t *mem,
                                const uint8_t *safe, const int32_t *progress, int32_t *pre_dur,
                                int32_t *pre_peak, int32_t *prev_safe)
{
    if (!ctx) return SJA_ERR_NULL;
    return prepare_into(ctx, stream, n_jobs, n_segments, seg_off, dur, mem, safe, progress, pre_dur, pre_peak,
                        prev_safe, true);
}

int sja_fit(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *W, const int32_t *C,
            int32_t *cut, uint32_t *interest_bits)
{
    if (!ctx) return SJA_ERR_NULL;
    ctx->fitted = false;
    ctx->planned = false;
    ctx->timed = false;
    if (!ctx->prepared) return fail(ctx, SJA_ERR_STATE, "sja_fit before sja_prepare_profiles");
    if (n_gaps < 0 || n_gaps > SJA_MAX_GAPS) return fail(ctx, SJA_ERR_SIZE, "n_gaps");
    if (n_gaps > 0 && (!W || !C)) return fail(ctx, SJA_ERR_NULL, "W / C");
    const int J = ctx->n_jobs;
    if (n_gaps > 0 && J > 0 && !cut) return fail(ctx, SJA_ERR_NULL, "cut");
    const Layout L = make_layout(n_gaps, J, ctx->n_segments);
    if (!ctx->ws || ctx->ws_bytes < L.total) return fail(ctx, SJA_ERR_WORKSPACE, "workspace too small for this many gaps");

    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_gaps > 0) {
        const int words = (J + 31) / 32;
        const int chunk_bound = int(fit_chunk_bound(n_gaps, J));
        const dim3 b256(256);
        int32_t *gw = ws_ptr<int32_t>(ctx, L.gap_w), *gcap = ws_ptr<int32_t>(ctx, L.gap_c);
        int32_t *plan = ws_ptr<int32_t>(ctx, L.plan);
        int rc = enqueue_gap_plan(ctx, st, L, n_gaps, W, C);
        if (rc != SJA_OK) return rc;
        if (J > 0) {
            const int job_tiles = (J + kFitBlock - 1) / kFitBlock;
            const int tiles8 = (job_tiles + 7) / 8 * 8;
            const unsigned grid = unsigned(tiles8) * unsigned(chunk_bound);
            if (ctx->timing) {
                if (!ctx->ev_start) {
                    SJA_HIP(hipEventCreate(&ctx->ev_start), "hipEventCreate");
                    SJA_HIP(hipEventCreate(&ctx->ev_stop), "hipEventCreate");
                }
                SJA_HIP(hipEventRecord(ctx->ev_start, st), "hipEventRecord");
            }
            hipLaunchKernelGGL((k_fit_main<kFitBlock, kFitWindow, kFitPeriod>), dim3(grid), dim3(kFitBlock), 0, st,
                               J, chunk_bound, ctx->seg_off, ws_ptr<int2>(ctx, L.atom_dp),
                               ws_ptr<int2>(ctx, L.atom_db), ws_ptr<int32_t>(ctx, L.n_atoms), plan,
                               ws_ptr<int32_t>(ctx, L.chunk_begin), ws_ptr<int32_t>(ctx, L.chunk_end),
                               ws_ptr<int32_t>(ctx, L.chunk_class), ws_ptr<int32_t>(ctx, L.chunk_sub),
                               ws_ptr<int32_t>(ctx, L.start_tab),
                               ws_ptr<int32_t>(ctx, L.ncap_tab), gw, gcap, ws_ptr<int64_t>(ctx, L.gap_row),
                               ws_ptr<int32_t>(ctx, L.gap_run_end), cut);
            SJA_HIP(hipGetLastError(), "k_fit_main launch");
            if (ctx->timing) {
                SJA_HIP(hipEventRecord(ctx->ev_stop, st), "hipEventRecord");
                ctx->timed = true;
            }
            if (interest_bits) {
                uint32_t *table = ws_ptr<uint32_t>(ctx, L.bits_table);
                int32_t *class_dmax = ws_ptr<int32_t>(ctx, L.class_dmax);
                hipLaunchKernelGGL(k_bits_table, dim3((words + 255) / 256, kMaxClasses), b256, 0, st, J, words, plan,
                                   ws_ptr<int32_t>(ctx, L.class_begin), gcap, ws_ptr<int2>(ctx, L.first_dp), table, class_dmax);
                SJA_HIP(hipGetLastError(), "k_bits_table launch");
                BitsArgs bits{};
                bits.bits = interest_bits;
                bits.first_dp = ws_ptr<int2>(ctx, L.first_dp);
                bits.table = table;
                bits.class_dmax = class_dmax;
                bits.gap_order = ws_ptr<int32_t>(ctx, L.gap_order);
                bits.gap_cls = ws_ptr<int32_t>(ctx, L.gap_cls);
                bits.n_gaps = n_gaps;
                bits.words = words;
                const int64_t col_tiles = (words + 256 * kBitsWords - 1) / (256 * kBitsWords);
                const int64_t row_tiles = (n_gaps + kBitsRows - 1) / kBitsRows;
                hipLaunchKernelGGL(k_fit_bits, dim3(unsigned(col_tiles * row_tiles)), b256, 0, st, bits, J, plan, gw, gcap);
                SJA_HIP(hipGetLastError(), "k_fit_bits launch");
                hipLaunchKernelGGL(k_fit_bits_low, dim3((words + 255) / 256, (n_gaps + kLowRows - 1) / kLowRows), b256, 0, st,
                                   bits, J, plan, gw);
                SJA_HIP(hipGetLastError(), "k_fit_bits launch");
            }
        }
    }
    ctx->n_gaps = n_gaps;
    ctx->cut = cut;
    ctx->fitted = true;
    ctx->planned = true;
    return SJA_OK;
}

int sja_store_reference(sja_ctx *ctx, void *stream, int32_t *cut)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!ctx->planned) return fail(ctx, SJA_ERR_STATE, "sja_store_reference before sja_fit or sja_fit_select");
    const int G = ctx->n_gaps, J = ctx->n_jobs;
    if (G > 0 && J > 0 && !cut) return fail(ctx, SJA_ERR_NULL, "cut");
    const Layout L = make_layout(G, J, ctx->n_segments);
    if (!ctx->ws || ctx->ws_bytes < L.total) return fail(ctx, SJA_ERR_WORKSPACE, "workspace too small");
    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int job_tiles = (J + kFitBlock - 1) / kFitBlock;
    if (G > 0 && job_tiles > 0) {
        const int chunk_bound = int(fit_chunk_bound(G, J));
        const int tiles8 = (job_tiles + 7) / 8 * 8;
        hipLaunchKernelGGL(k_store_reference<kFitBlock>, dim3(unsigned(tiles8) * unsigned(chunk_bound)), dim3(kFitBlock), 0, st,
                           J, chunk_bound, ws_ptr<int32_t>(ctx, L.plan), ws_ptr<int32_t>(ctx, L.chunk_begin),
                           ws_ptr<int32_t>(ctx, L.chunk_end), ws_ptr<int64_t>(ctx, L.gap_row), cut);
        SJA_HIP(hipGetLastError(), "k_store_reference launch");
    }
    if (cut == ctx->cut) ctx->fitted = false;      // the matrix of the last sja_fit no longer holds its replies
    return SJA_OK;
}

int sja_fit_select(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *W, const int32_t *C,
                   const sja_params *params, const int32_t *wait, const uint8_t *sla_class,
                   const int32_t *job_held, const uint8_t *gap_active, int32_t *cand_job, int32_t *cand_cut,
                   int64_t *cand_score)
{
    if (!ctx) return SJA_ERR_NULL;
    ctx->fitted = false;
    ctx->planned = false;
    ctx->timed = false;
    if (!ctx->prepared) return fail(ctx, SJA_ERR_STATE, "sja_fit_select before sja_prepare_profiles");
    if (n_gaps < 0 || n_gaps > SJA_MAX_GAPS) return fail(ctx, SJA_ERR_SIZE, "n_gaps");
    if (n_gaps > 0 && (!W || !C)) return fail(ctx, SJA_ERR_NULL, "W / C");
    int rc = check_params(ctx, params, wait, sla_class);
    if (rc != SJA_OK) return rc;
    if (n_gaps > 0 && (!cand_job || !cand_cut || !cand_score)) return fail(ctx, SJA_ERR_NULL, "candidate outputs");
    const int J = ctx->n_jobs;
    const Layout L = make_layout(n_gaps, J, ctx->n_segments);
    if (!ctx->ws || ctx->ws_bytes < L.total) return fail(ctx, SJA_ERR_WORKSPACE, "workspace too small for this many gaps");

    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_gaps > 0) {
        rc = enqueue_gap_plan(ctx, st, L, n_gaps, W, C);
        if (rc != SJA_OK) return rc;
        rc = launch_fused(ctx, st, L, n_gaps, params, wait, sla_class, job_held, gap_active, cand_job, cand_cut,
                          cand_score, ctx->timing);
        if (rc != SJA_OK) return rc;
    }
    ctx->n_gaps = n_gaps;
    ctx->cut = nullptr;
    ctx->planned = true;
    return SJA_OK;
}

int sja_select(sja_ctx *ctx, void *stream, const sja_params *params, const int32_t *wait,
               const uint8_t *sla_class, const int32_t *job_held, const uint8_t *gap_active,
               int32_t *cand_job, int32_t *cand_cut, int64_t *cand_score)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!ctx->fitted) return fail(ctx, SJA_ERR_STATE, "sja_select before sja_fit");
    int rc = check_params(ctx, params, wait, sla_class);
    if (rc != SJA_OK) return rc;
    if (ctx->n_gaps > 0 && (!cand_job || !cand_cut || !cand_score)) return fail(ctx, SJA_ERR_NULL, "candidate outputs");
    const Layout L = make_layout(ctx->n_gaps, ctx->n_jobs, ctx->n_segments);
    if (!ctx->ws || ctx->ws_bytes < L.total) return fail(ctx, SJA_ERR_WORKSPACE, "workspace too small");
    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    return launch_select(ctx, static_cast<hipStream_t>(stream), params, wait, sla_class, job_held,
                         gap_active, cand_job, cand_cut, cand_score);
}

int sja_resolve(sja_ctx *ctx, void *stream, const sja_params *params, const int32_t *wait,
                const uint8_t *sla_class, int32_t *grant_job, int32_t *grant_cut,
                int64_t *grant_score, int32_t *job_gap, int32_t *rounds_used_and_stable)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!ctx->planned) return fail(ctx, SJA_ERR_STATE, "sja_resolve before sja_fit or sja_fit_select");
    int rc = check_params(ctx, params, wait, sla_class);
    if (rc != SJA_OK) return rc;
    const int G = ctx->n_gaps, J = ctx->n_jobs;
    if (G > 0 && (!grant_job || !grant_cut || !grant_score)) return fail(ctx, SJA_ERR_NULL, "grant outputs");
    if (J > 0 && !job_gap) return fail(ctx, SJA_ERR_NULL, "job_gap");
    if (!rounds_used_and_stable) return fail(ctx, SJA_ERR_NULL, "rounds_used_and_stable");
    const Layout L = make_layout(G, J, ctx->n_segments);
    if (!ctx->ws || ctx->ws_bytes < L.total) return fail(ctx, SJA_ERR_WORKSPACE, "workspace too small");

    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    hipStream_t st = static_cast<hipStream_t>(stream);

    int32_t *cand_job = ws_ptr<int32_t>(ctx, L.res_cand_job);
    int32_t *cand_cut = ws_ptr<int32_t>(ctx, L.res_cand_cut);
    int64_t *cand_score = ws_ptr<int64_t>(ctx, L.res_cand_score);
    uint8_t *active = ws_ptr<uint8_t>(ctx, L.res_active);
    unsigned long long *claim = ws_ptr<unsigned long long>(ctx, L.res_claim);
    int32_t *counters = ws_ptr<int32_t>(ctx, L.res_counters);

    const int n_init = G > J ? G : J;
    if (n_init > 0) {
        hipLaunchKernelGGL(k_resolve_init, dim3((n_init + 255) / 256), dim3(256), 0, st, G, J, grant_job,
                           grant_cut, grant_score, job_gap, active, claim);
        SJA_HIP(hipGetLastError(), "k_resolve_init launch");
    }
    // every round that does not end the process grants at least one job, so it
    // ends by itself within min(G, J) + 1 rounds: a larger cap changes nothing
    const int64_t natural = int64_t(G < J ? G : J) + 1;
    const int64_t cap = (params->max_rounds > 0 && params->max_rounds < natural) ? params->max_rounds : natural;
    int32_t result[2] = {0, 0};
    bool done = false;
    if (G > 0 && J > 0 && ctx->resolve_mode != SJA_RESOLVE_MATRIX) {
        rc = resolve_with_lists(ctx, st, L, params, wait, sla_class, grant_job, grant_cut, grant_score, job_gap, cap,
                                result, &done);
        if (rc != SJA_OK) return rc;
    }
    for (int64_t r = 1; !done && r <= cap; ++r) {
        ++result[0];
        int32_t host_counters[2] = {0, 0};
        if (G > 0) {
            // the round's selection over the still-active gaps and un-held jobs: from the cut matrix if
            // sja_fit left one, else by evaluating the pairs again (the fused pass; nothing is stored)
            if (ctx->fitted)
                rc = launch_select(ctx, st, params, wait, sla_class, job_gap, active, cand_job, cand_cut, cand_score,
                                   /*keys_ready=*/r > 1);
            else
                rc = launch_fused(ctx, st, L, G, params, wait, sla_class, job_gap, active, cand_job, cand_cut, cand_score,
                                  false);
            if (rc != SJA_OK) return rc;
            const dim3 grid((G + 255) / 256), block(256);
            hipLaunchKernelGGL(k_claim, grid, block, 0, st, G, int(r), active, cand_job, claim, counters);
            SJA_HIP(hipGetLastError(), "k_claim launch");
            hipLaunchKernelGGL(k_commit, grid, block, 0, st, G, int(r), active, cand_job, cand_cut, cand_score,
                               claim, grant_job, grant_cut, grant_score, job_gap, counters);
            SJA_HIP(hipGetLastError(), "k_commit launch");
            SJA_HIP(hipMemcpyAsync(host_counters, counters, sizeof(host_counters), hipMemcpyDeviceToHost, st),
                    "counter readback");
            SJA_HIP(hipStreamSynchronize(st), "round synchronise");
        }
        if (host_counters[0] == 0 || host_counters[1] == 0) { result[1] = 1; break; }
    }
    SJA_HIP(hipMemcpyAsync(rounds_used_and_stable, result, sizeof(result), hipMemcpyHostToDevice, st),
            "rounds writeback");
    SJA_HIP(hipStreamSynchronize(st), "final synchronise");
    return SJA_OK;
}

int sja_advance(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *W, const int32_t *C,
                const int32_t *grant_job, const int32_t *grant_cut, const int32_t *job_gap, int32_t *progress,
                int32_t *wait, int32_t wait_step, int64_t *metrics)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!ctx->prepared) return fail(ctx, SJA_ERR_STATE, "sja_advance before sja_prepare_profiles");
    if (n_gaps < 0 || n_gaps > SJA_MAX_GAPS) return fail(ctx, SJA_ERR_SIZE, "n_gaps");
    if (wait_step < 0) return fail(ctx, SJA_ERR_SIZE, "wait_step");
    if (n_gaps > 0 && (!W || !C || !grant_job || !grant_cut)) return fail(ctx, SJA_ERR_NULL, "gap arrays");
    const int J = ctx->n_jobs;
    if (J > 0 && (!job_gap || !progress)) return fail(ctx, SJA_ERR_NULL, "job_gap / progress");
    if (!metrics) return fail(ctx, SJA_ERR_NULL, "metrics");
    const Layout L = make_layout(0, J, ctx->n_segments);
    if (!ctx->ws || ctx->ws_bytes < L.total) return fail(ctx, SJA_ERR_WORKSPACE, "workspace too small");

    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the profiles of the granted jobs change: whatever the last fit left no longer describes them
    ctx->fitted = false;
    ctx->planned = false;
    unsigned long long *m = reinterpret_cast<unsigned long long *>(metrics);
    hipLaunchKernelGGL(k_fill_i64, dim3(1), dim3(64), 0, st, 4, int64_t(0), metrics);
    SJA_HIP(hipGetLastError(), "k_fill_i64 launch");
    if (n_gaps > 0) {
        hipLaunchKernelGGL(k_advance_gaps, dim3((n_gaps + 255) / 256), dim3(256), 0, st, n_gaps, J, ctx->seg_off,
                           ctx->pre_dur, ctx->pre_peak, W, C, grant_job, grant_cut, job_gap, progress, m);
        SJA_HIP(hipGetLastError(), "k_advance_gaps launch");
    }
    if (J > 0) {
        const int jobs_per_block = 256 / kWave;
        const dim3 grid((J + jobs_per_block - 1) / jobs_per_block), block(256);
        const bool by_area = ctx->score_used == SJA_SCORE_AREA;
        const Hysteresis hyst = hysteresis_of(ctx->hyst_used_n_caps, ctx->hyst_used_min_gain, ctx->hyst_used_cap);
        long long *pre_area = by_area ? ws_ptr<long long>(ctx, L.pre_area) : nullptr;
        long long *atom_area = by_area || hyst.n_caps > 0 ? ws_ptr<long long>(ctx, L.atom_area) : nullptr;
        if (ctx->limits_used) {
            const JobLimits lim = job_limits(ctx->limits_applied, ctx->used_power, ctx->used_deadline);
            hipLaunchKernelGGL(k_advance_jobs<true>, grid, block, 0, st, lim, hyst, pre_area, atom_area, n_gaps, J, ctx->seg_off, ctx->dur,
                               ctx->mem, ctx->safe, grant_job, grant_cut, job_gap, progress, wait, wait_step,
                               ctx->pre_dur, ctx->pre_peak, ctx->prev_safe, ws_ptr<int2>(ctx, L.atom_dp),
                               ws_ptr<int2>(ctx, L.atom_db), ws_ptr<int32_t>(ctx, L.n_atoms),
                               ws_ptr<int2>(ctx, L.first_dp), m);
        } else {
            hipLaunchKernelGGL(k_advance_jobs<false>, grid, block, 0, st, JobLimits{}, hyst, pre_area, atom_area, n_gaps, J, ctx->seg_off,
                               ctx->dur, ctx->mem, ctx->safe, grant_job, grant_cut, job_gap, progress, wait,
                               wait_step, ctx->pre_dur, ctx->pre_peak, ctx->prev_safe,
                               ws_ptr<int2>(ctx, L.atom_dp), ws_ptr<int2>(ctx, L.atom_db),
                               ws_ptr<int32_t>(ctx, L.n_atoms), ws_ptr<int2>(ctx, L.first_dp), m);
        }
        SJA_HIP(hipGetLastError(), "k_advance_jobs launch");
    }
    return SJA_OK;
}

int sja_cover(sja_ctx *ctx, void *stream, int32_t n_gaps, const int32_t *C, const int32_t *grant_job,
              const int32_t *grant_cut, int32_t n_caps, const int32_t *cap_set, int32_t *cover, int32_t *slack)
{
    if (!ctx) return SJA_ERR_NULL;
    if (!ctx->prepared) return fail(ctx, SJA_ERR_STATE, "sja_cover before sja_prepare_profiles");
    if (n_gaps < 0 || n_gaps > SJA_MAX_GAPS) return fail(ctx, SJA_ERR_SIZE, "n_gaps");
    if (n_caps < 0) return fail(ctx, SJA_ERR_SIZE, "n_caps");
    if (n_gaps > 0 && (!C || !grant_job || !grant_cut || !cover || !slack)) return fail(ctx, SJA_ERR_NULL, "gap arrays");
    if (n_caps > 0 && !cap_set) return fail(ctx, SJA_ERR_NULL, "cap_set");
    DeviceGuard guard(ctx->device);
    SJA_HIP(guard.err, "hipSetDevice");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_gaps > 0) {
        hipLaunchKernelGGL(k_cover, dim3((n_gaps + 255) / 256), dim3(256), 0, st, n_gaps, ctx->n_jobs, ctx->seg_off,
                           ctx->pre_peak, C, grant_job, grant_cut, n_caps, cap_set, cover, slack);
        SJA_HIP(hipGetLastError(), "k_cover launch");
    }
    return SJA_OK;
}

}  // extern "C"
