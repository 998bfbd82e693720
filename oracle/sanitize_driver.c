/*
 * TEST INFRASTRUCTURE: runs oracle/sja_oracle.c under the compiler's address and
 * undefined-behaviour sanitizers.  Built together with sja_oracle.c into one
 * executable (gcc -fsanitize=address,undefined), it reads tiny cases with the
 * answers a from-scratch brute force gave (tests/test_oracle_sanitized.py writes
 * them from oracle/brute.py), calls the oracle's entry points on exactly sized
 * heap buffers, so that any read or write beyond an array ends the run, and
 * compares every output.  Exit status 0: all cases equal and no sanitizer
 * report.  Nothing here is reachable from the GPU library.
 *
 * Case file (text, whitespace separated):
 *   n_cases
 *   per case: J G S policy wait_scale w0 w1 w2 class0_override max_rounds
 *             seg_off[J+1] dur[S] mem[S] safe[S] progress[J] W[G] C[G] wait[J] cls[J]
 *             cut[G*J] cand_job[G] cand_cut[G] cand_score[G]
 *             grant_job[G] grant_cut[G] grant_score[G] job_gap[J] rounds stable
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t policy, wait_scale, sla_weight[3], class0_override, max_rounds;
} sjo_params;

int sjo_prepare(int32_t, const int64_t *, const int32_t *, const int32_t *, const uint8_t *, const int32_t *,
                int64_t *, int64_t *, int32_t *);
int sjo_fit(int32_t, int32_t, const int64_t *, const int32_t *, const int32_t *, const uint8_t *, const int32_t *,
            const int32_t *, const int32_t *, int32_t *, uint32_t *);
int sjo_select(int32_t, int32_t, const int32_t *, const int64_t *, const int64_t *, const int64_t *, const int64_t *,
               const sjo_params *, const int32_t *, const uint8_t *, const int32_t *, const uint8_t *, int32_t *,
               int32_t *, int64_t *);
int sjo_resolve(int32_t, int32_t, const int32_t *, const int64_t *, const int64_t *, const int64_t *, const int64_t *,
                const sjo_params *, const int32_t *, const uint8_t *, int32_t *, int32_t *, int64_t *, int32_t *,
                int32_t *);

static FILE *in;

static long long next_value(void)
{
    long long v;
    if (fscanf(in, "%lld", &v) != 1) { fprintf(stderr, "case file ended early\n"); exit(3); }
    return v;
}

/* exactly n elements (one byte when n == 0 so that malloc returns a pointer) */
#define NEW(type, n) ((type *)malloc((n) > 0 ? sizeof(type) * (size_t)(n) : 1))
#define READ(type, name, n) type *name = NEW(type, n); for (long long i_ = 0; i_ < (n); ++i_) name[i_] = (type)next_value()

static int differ(const char *what, int c, long long i, long long got, long long want)
{
    fprintf(stderr, "case %d: %s[%lld] = %lld, brute force says %lld\n", c, what, i, got, want);
    return 1;
}

int main(int argc, char **argv)
{
    if (argc < 2 || !(in = fopen(argv[1], "r"))) { fprintf(stderr, "usage: %s cases.txt\n", argv[0]); return 2; }
    const int n_cases = (int)next_value();
    int bad = 0;
    for (int c = 0; c < n_cases && !bad; ++c) {
        const int J = (int)next_value(), G = (int)next_value();
        const long long S = next_value();
        sjo_params par;
        par.policy = (int32_t)next_value();
        par.wait_scale = (int32_t)next_value();
        for (int i = 0; i < 3; ++i) par.sla_weight[i] = (int32_t)next_value();
        par.class0_override = (int32_t)next_value();
        par.max_rounds = (int32_t)next_value();
        READ(int64_t, seg_off, J + 1);
        READ(int32_t, dur, S);
        READ(int32_t, mem, S);
        READ(uint8_t, safe, S);
        READ(int32_t, progress, J);
        READ(int32_t, W, G);
        READ(int32_t, C, G);
        READ(int32_t, wait, J);
        READ(uint8_t, cls, J);
        READ(int32_t, want_cut, (long long)G * J);
        READ(int32_t, want_cj, G);
        READ(int32_t, want_cc, G);
        READ(int64_t, want_cs, G);
        READ(int32_t, want_gj, G);
        READ(int32_t, want_gc, G);
        READ(int64_t, want_gs, G);
        READ(int32_t, want_jg, J);
        const int want_rounds = (int)next_value(), want_stable = (int)next_value();

        int64_t *pre_dur = NEW(int64_t, S), *pre_peak = NEW(int64_t, S);
        int32_t *prev_safe = NEW(int32_t, S);
        int32_t *cut = NEW(int32_t, (long long)G * J);
        const int words = (J + 31) / 32;
        uint32_t *bits = NEW(uint32_t, (long long)G * words);
        int32_t *cj = NEW(int32_t, G), *cc = NEW(int32_t, G), *gj = NEW(int32_t, G), *gc = NEW(int32_t, G);
        int64_t *cs = NEW(int64_t, G), *gs = NEW(int64_t, G);
        int32_t *jg = NEW(int32_t, J);
        int32_t rs[2] = {-1, -1};
        for (long long i = 0; i < S; ++i) { pre_dur[i] = -7; pre_peak[i] = -7; prev_safe[i] = -7; }

        int rc = sjo_prepare(J, seg_off, dur, mem, safe, progress, pre_dur, pre_peak, prev_safe);
        if (!rc) rc = sjo_fit(G, J, seg_off, dur, mem, safe, progress, W, C, cut, bits);
        if (!rc) rc = sjo_select(G, J, cut, seg_off, pre_dur, pre_peak, NULL, &par, wait, cls, NULL, NULL, cj, cc, cs);
        if (!rc) rc = sjo_resolve(G, J, cut, seg_off, pre_dur, pre_peak, NULL, &par, wait, cls, gj, gc, gs, jg, rs);
        if (rc) { fprintf(stderr, "case %d: oracle status %d\n", c, rc); bad = 1; }
        for (long long i = 0; i < (long long)G * J && !bad; ++i) {
            if (cut[i] != want_cut[i]) bad = differ("cut", c, i, cut[i], want_cut[i]);
            const int g = (int)(i / J), j = (int)(i % J);
            const int bit = (int)((bits[(long long)g * words + (j >> 5)] >> (j & 31)) & 1u);
            if (!bad && bit != (want_cut[i] >= 0)) bad = differ("interest bit", c, i, bit, want_cut[i] >= 0);
        }
        for (int g = 0; g < G && !bad; ++g) {
            if (cj[g] != want_cj[g]) bad = differ("cand_job", c, g, cj[g], want_cj[g]);
            else if (cc[g] != want_cc[g]) bad = differ("cand_cut", c, g, cc[g], want_cc[g]);
            else if (cs[g] != want_cs[g]) bad = differ("cand_score", c, g, cs[g], want_cs[g]);
            else if (gj[g] != want_gj[g]) bad = differ("grant_job", c, g, gj[g], want_gj[g]);
            else if (gc[g] != want_gc[g]) bad = differ("grant_cut", c, g, gc[g], want_gc[g]);
            else if (gs[g] != want_gs[g]) bad = differ("grant_score", c, g, gs[g], want_gs[g]);
        }
        for (int j = 0; j < J && !bad; ++j)
            if (jg[j] != want_jg[j]) bad = differ("job_gap", c, j, jg[j], want_jg[j]);
        if (!bad && (rs[0] != want_rounds || rs[1] != want_stable)) bad = differ("rounds", c, 0, rs[0], want_rounds);

        free(seg_off); free(dur); free(mem); free(safe); free(progress); free(W); free(C); free(wait); free(cls);
        free(want_cut); free(want_cj); free(want_cc); free(want_cs); free(want_gj); free(want_gc); free(want_gs);
        free(want_jg); free(pre_dur); free(pre_peak); free(prev_safe); free(cut); free(bits); free(cj); free(cc);
        free(gj); free(gc); free(cs); free(gs); free(jg);
    }
    fclose(in);
    if (!bad) printf("%d cases equal, no sanitizer report\n", n_cases);
    return bad;
}
