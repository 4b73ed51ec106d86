/*
 * tessel_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, single-purpose CPU implementation of what the repetend-candidate
 * evaluator must compute, written out from the definitions in the Tessel paper
 * (arXiv 2311.15269).  It shares no code, header, table or constant generator with the
 * HIP library; only tests, the smoke check and the cpu_baseline leg of the benchmark may
 * call it.  Everything is integer arithmetic (Sec. III-A: t_B in Z+, m_B in Z, s_B >= 0).
 *
 * What is a definition and what is a convention:
 *   - constraints (device exclusivity, memory prefix, data dependency): Eq. 1 [1]-[3];
 *   - repetend block set, micro-batch index assignment n_i ("lead"): Eq. 3;
 *   - Property 1 (same-type blocks in increasing micro-batch order) and Property 2
 *     (producer index >= consumer index): Sec. IV-B;
 *   - repetend time t_R incl. compaction of neighbouring repetends: Eq. 4 and the
 *     paragraph below it.  For a fixed per-device order the smallest t_R over all start
 *     times is the smallest integer period T for which the rigidly repeated window
 *     satisfies every constraint; that is what orc_period() computes, by its definition
 *     (binary search on T, Bellman-Ford feasibility of the difference constraints);
 *   - entry memory of the repetend from the index assignment: Sec. IV-B last paragraph;
 *   - lower bound: Alg. 1, GetLowerBound;  tie rule (strict <): Alg. 1;
 *   - warm-up / cool-down block sets: Eq. 5, 6.
 *   Conventions the paper does not fix (candidate index encodings, the seeded sampler,
 *   the deadlock-repair rule, the greedy completion order) are this build's own and are
 *   spelled out next to the function that implements them.
 *
 * Pinned by tests (-m "not gpu"): brute force over integer start vectors on tiny graphs,
 * an independent validity checker, the 1F1B and GPipe closed forms, hand-verified
 * 2-device schedules, invariants (period >= lower bound, lead-shift invariance,
 * monotonicity in M).  orc_complete()'s greedy order has no closed form in general:
 * its output is checked for validity and against the 1F1B/GPipe makespans only.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <pthread.h>

#define ORC_MAX_D   32
#define ORC_MAX_K   64
#define ORC_MAX_NR  16
#define ORC_MAX_N   (ORC_MAX_K * ORC_MAX_NR)
#define ORC_MAX_DEPS 256
#define ORC_MAX_LEADVECS (1 << 20)

enum { ORC_SPACE_FACTORIAL = 0, ORC_SPACE_CANONICAL = 1, ORC_SPACE_SAMPLED_STRICT = 2, ORC_SPACE_SAMPLED_REPAIR = 3 };
enum { ORC_OK = 0, ORC_DUP = 1, ORC_TP_MISMATCH = 2, ORC_PROP2 = 3, ORC_DEADLOCK = 4, ORC_MEM = 5, ORC_NSTATUS = 6 };
enum { ORC_E_OK = 0, ORC_E_INVALID = -1, ORC_E_BAD_DEP = -2, ORC_E_UNBALANCED = -3, ORC_E_TOOBIG = -4, ORC_E_RANGE = -8, ORC_E_NO_SCHEDULE = -10 };

typedef struct {
    int D, K, NR, M;
    int t[ORC_MAX_K], m[ORC_MAX_K];
    uint32_t mask[ORC_MAX_K];
    int ndeps, src[ORC_MAX_DEPS], dst[ORC_MAX_DEPS];
    int space, has_fixed, fixed[ORC_MAX_K];
    uint64_t seed;
    uint32_t step_q16;
    /* derived */
    int ntd[ORC_MAX_D];                 /* number of block types on device d            */
    int td[ORC_MAX_D][ORC_MAX_K];       /* their ids, ascending                         */
    int topo[ORC_MAX_K];                /* types in a topological order of the deps     */
    int LB, UB;
    int nlead;                          /* CANONICAL: number of lead vectors            */
    int8_t *leadtab;                    /* nlead x K                                    */
    uint64_t cdev[ORC_MAX_D];           /* CANONICAL: interleavings per device;
                                           FACTORIAL: n_d!                              */
    uint64_t count;                     /* number of candidates (UINT64_MAX = any)      */
} orc_problem;

typedef struct {
    int status;                         /* ORC_OK or a reject reason                    */
    int period;                         /* T*, valid when status == ORC_OK              */
    int peak[ORC_MAX_D];                /* valid when status is ORC_OK or ORC_MEM       */
    int peak_max;
} orc_score;

typedef struct {
    int leads[ORC_MAX_K];
    int len[ORC_MAX_D];
    int seq[ORC_MAX_D][ORC_MAX_N];      /* block type ids in device order               */
} orc_candidate;

/* Counts the integer max/add/compare steps the period computation performs; read by the
 * benchmark to state "algorithmic operations per candidate". */
static __thread uint64_t orc_ops;

/* ------------------------------------------------------------------ counter-based sampler
 * This build's convention (the paper only says values are "drawn"): a candidate ordinal
 * is mixed with the seed by the SplitMix64 finaliser into two 32-bit keys (a, b); the
 * w-th 32-bit word of the candidate's stream is a MurmurHash3 fmix32 of a + w*golden
 * with b folded in between the two multiplications; each word yields two 16-bit draws,
 * low half first.  A draw u is turned into a digit below `radix` as (u * radix) >> 16. */
static uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}
static uint32_t stream_word(uint32_t a, uint32_t b, uint32_t w)
{
    uint32_t x = a + w * 0x9E3779B9u;
    x ^= x >> 16; x *= 0x85EBCA6Bu;
    x ^= b;
    x ^= x >> 13; x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}
static uint32_t draw16(uint64_t seed, uint64_t ordinal, uint32_t j)
{
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * (ordinal + 1));
    uint32_t a = (uint32_t)z, b = (uint32_t)(z >> 32);
    uint32_t word = stream_word(a, b, j >> 1);
    return (word >> (16 * (j & 1))) & 0xFFFFu;
}
/* exported so that a test can pin the sampler against the worked example of tests/golden/sampler_hand.txt */
uint32_t orc_draw16(uint64_t seed, uint64_t ordinal, uint32_t j) { return draw16(seed, ordinal, j); }

#define DRAW_LEAD_BASE 0u     /* draw j = e            decides the lead step of dependency e   */
#define DRAW_ORD_BASE  128u   /* draw j = 128+32*d+p   picks the p-th block of device d        */

/* ------------------------------------------------------------------ problem set-up */
static uint64_t factorial_or_zero(int n)     /* 0 when n! does not fit in 64 bits */
{
    if (n > 20) return 0;
    uint64_t f = 1;
    for (int i = 2; i <= n; i++) f *= (uint64_t)i;
    return f;
}

/* number of distinct arrangements of a multiset with the given counts; 0 on overflow */
static uint64_t arrangements(const int *cnt, int ntypes)
{
    unsigned __int128 r = 1;
    int placed = 0;
    for (int y = 0; y < ntypes; y++)
        for (int k = 1; k <= cnt[y]; k++) {
            placed++;
            r = r * (unsigned)placed / (unsigned)k;      /* exact: running binomial */
            if (r >> 64) return 0;
        }
    return (uint64_t)r;
}

static void enum_leads(orc_problem *p, int i, int *cur, int *err)
{
    /* lexicographic enumeration, type 0 most significant, of every lead vector with
     * lead_src >= lead_dst on each dependency (Property 2) and minimum 0 (a common shift
     * of all indices is the same repetend). */
    if (*err) return;
    if (i == p->K) {
        int mn = cur[0];
        for (int k = 1; k < p->K; k++) if (cur[k] < mn) mn = cur[k];
        if (mn != 0) return;
        for (int e = 0; e < p->ndeps; e++) if (cur[p->src[e]] < cur[p->dst[e]]) return;
        if (p->nlead >= ORC_MAX_LEADVECS) { *err = ORC_E_TOOBIG; return; }
        for (int k = 0; k < p->K; k++) p->leadtab[(size_t)p->nlead * p->K + k] = (int8_t)cur[k];
        p->nlead++;
        return;
    }
    for (int v = 0; v < p->NR; v++) {
        cur[i] = v;
        /* prune: a dependency between two already assigned types must hold */
        int ok = 1;
        for (int e = 0; e < p->ndeps && ok; e++) {
            int a = p->src[e], b = p->dst[e];
            if (a <= i && b <= i && (a == i || b == i) && cur[a] < cur[b]) ok = 0;
        }
        if (ok) enum_leads(p, i + 1, cur, err);
    }
}

orc_problem *orc_create(int D, int K, int NR, int M, const int *t, const int *m, const uint32_t *mask,
                        int ndeps, const int *src, const int *dst, int space, const int *fixed_leads,
                        uint64_t seed, uint32_t step_q16, int *err)
{
    *err = ORC_E_OK;
    if (D < 1 || D > ORC_MAX_D || K < 1 || K > ORC_MAX_K || NR < 1 || NR > ORC_MAX_NR || ndeps < 0 ||
        ndeps > ORC_MAX_DEPS || space < 0 || space > 3 || step_q16 > 65536u) { *err = ORC_E_INVALID; return NULL; }
    orc_problem *p = (orc_problem *)calloc(1, sizeof *p);
    p->D = D; p->K = K; p->NR = NR; p->M = M; p->space = space; p->seed = seed; p->step_q16 = step_q16;
    for (int i = 0; i < K; i++) {
        if (t[i] < 1 || mask[i] == 0 || (D < 32 && (mask[i] >> D))) { *err = ORC_E_INVALID; free(p); return NULL; }
        p->t[i] = t[i]; p->m[i] = m[i]; p->mask[i] = mask[i];
    }
    p->ndeps = ndeps;
    for (int e = 0; e < ndeps; e++) {
        if (src[e] < 0 || src[e] >= K || dst[e] < 0 || dst[e] >= K || src[e] == dst[e]) { *err = ORC_E_INVALID; free(p); return NULL; }
        p->src[e] = src[e]; p->dst[e] = dst[e];
    }
    /* topological order of the block types (Kahn, smallest id first); a cycle is an error */
    {
        int indeg[ORC_MAX_K] = {0}, done[ORC_MAX_K] = {0}, n = 0;
        for (int e = 0; e < ndeps; e++) indeg[dst[e]]++;
        for (;;) {
            int pick = -1;
            for (int i = 0; i < K; i++) if (!done[i] && indeg[i] == 0) { pick = i; break; }
            if (pick < 0) break;
            done[pick] = 1; p->topo[n++] = pick;
            for (int e = 0; e < ndeps; e++) if (src[e] == pick) indeg[dst[e]]--;
        }
        if (n != K) { *err = ORC_E_BAD_DEP; free(p); return NULL; }
    }
    int sumt = 0;
    for (int i = 0; i < K; i++) sumt += p->t[i];
    p->UB = NR * sumt;
    p->LB = 0;
    for (int d = 0; d < D; d++) {
        int busy = 0, net = 0;
        p->ntd[d] = 0;
        for (int i = 0; i < K; i++) if (mask[i] >> d & 1u) { p->td[d][p->ntd[d]++] = i; busy += t[i]; net += m[i]; }
        if (net != 0) { *err = ORC_E_UNBALANCED; free(p); return NULL; }   /* no steady state otherwise */
        if (NR * busy > p->LB) p->LB = NR * busy;                         /* Alg. 1 GetLowerBound, x N_R */
    }
    if (fixed_leads) {
        if (space == ORC_SPACE_FACTORIAL) { *err = ORC_E_INVALID; free(p); return NULL; }
        p->has_fixed = 1;
        for (int i = 0; i < K; i++) {
            if (fixed_leads[i] < 0 || fixed_leads[i] >= NR) { *err = ORC_E_INVALID; free(p); return NULL; }
            p->fixed[i] = fixed_leads[i];
        }
        for (int e = 0; e < ndeps; e++) if (p->fixed[src[e]] < p->fixed[dst[e]]) { *err = ORC_E_INVALID; free(p); return NULL; }
    }
    /* candidate count */
    if (space == ORC_SPACE_FACTORIAL) {
        unsigned __int128 c = 1;
        for (int d = 0; d < D; d++) {
            p->cdev[d] = factorial_or_zero(p->ntd[d] * NR);
            if (!p->cdev[d]) { *err = ORC_E_TOOBIG; free(p); return NULL; }
            c *= p->cdev[d];
            if (c >> 64) { *err = ORC_E_TOOBIG; free(p); return NULL; }
        }
        p->count = (uint64_t)c;
    } else if (space == ORC_SPACE_CANONICAL) {
        if (p->has_fixed) {
            p->nlead = 1;
            p->leadtab = (int8_t *)malloc((size_t)K);
            for (int i = 0; i < K; i++) p->leadtab[i] = (int8_t)p->fixed[i];
        } else {
            int cur[ORC_MAX_K];
            p->leadtab = (int8_t *)malloc((size_t)ORC_MAX_LEADVECS * K);
            p->nlead = 0;
            enum_leads(p, 0, cur, err);
            if (*err) { free(p->leadtab); free(p); return NULL; }
        }
        unsigned __int128 c = (unsigned)p->nlead;
        for (int d = 0; d < D; d++) {
            int cnt[ORC_MAX_K];
            for (int y = 0; y < p->ntd[d]; y++) cnt[y] = NR;
            p->cdev[d] = arrangements(cnt, p->ntd[d]);
            if (!p->cdev[d]) { *err = ORC_E_TOOBIG; free(p->leadtab); free(p); return NULL; }
            c *= p->cdev[d];
            if (c >> 64) { *err = ORC_E_TOOBIG; free(p->leadtab); free(p); return NULL; }
        }
        p->count = (uint64_t)c;
    } else {
        if (ndeps > 128) { *err = ORC_E_TOOBIG; free(p); return NULL; }
        p->count = UINT64_MAX;
    }
    return p;
}

void orc_destroy(orc_problem *p) { if (p) { free(p->leadtab); free(p); } }
uint64_t orc_candidate_count(const orc_problem *p) { return p->count; }
int orc_lower_bound(const orc_problem *p) { return p->LB; }
int orc_upper_bound(const orc_problem *p) { return p->UB; }
int orc_num_lead_vectors(const orc_problem *p) { return p->nlead; }

/* ------------------------------------------------------------------ candidate decoding */

/* A block of type g, about to run its next occurrence, may be placed when every lag-0
 * producer occurrence has been placed.  With mu_next[x] = lead_x + (occurrences of x placed),
 * the consumer's next occurrence handles micro-batch mu_next[g]; the producer i has handled
 * it already in this window iff mu_next[i] > mu_next[g]; if the micro-batch is below lead_i
 * the producer handled it in the previous window (lag 1) and nothing has to be placed. */
static int producers_placed(const orc_problem *p, const int *leads, const int *placed_cnt, int g)
{
    int mu = leads[g] + placed_cnt[g];
    for (int e = 0; e < p->ndeps; e++) if (p->dst[e] == g) {
        int i = p->src[e];
        if (mu < leads[i]) continue;                       /* lag 1 */
        if (leads[i] + placed_cnt[i] > mu) continue;       /* lag 0, placed */
        return 0;
    }
    return 1;
}

/* Deadlock repair (this build's convention; used only by ORC_SPACE_SAMPLED_REPAIR).
 * Each device keeps its sampled type sequence as a priority list.  Until everything is
 * placed: scan the devices in ascending order and look at the first unplaced entry of each;
 * if its producers are placed and, for a multi-device block, it is the first unplaced entry
 * on all its devices, place it (append to the output order of each of its devices) and
 * restart the scan.  If no device can advance, scan devices ascending and, inside a device,
 * its unplaced entries in list order; place the first whose producers are placed (on all
 * its devices, taking its earliest unplaced entry there) and restart. */
static void repair_orders(const orc_problem *p, orc_candidate *c)
{
    static __thread int rem[ORC_MAX_D][ORC_MAX_N];
    int remlen[ORC_MAX_D], outlen[ORC_MAX_D], cnt[ORC_MAX_K] = {0};
    int total = 0, placed = 0;
    for (int d = 0; d < p->D; d++) {
        remlen[d] = c->len[d]; outlen[d] = 0;
        memcpy(rem[d], c->seq[d], sizeof(int) * (size_t)c->len[d]);
    }
    for (int i = 0; i < p->K; i++) total += p->NR;
    while (placed < total) {
        int pick = -1;
        for (int d = 0; d < p->D && pick < 0; d++) {
            if (!remlen[d]) continue;
            int g = rem[d][0], head_everywhere = 1;
            for (int dd = 0; dd < p->D; dd++)
                if ((p->mask[g] >> dd & 1u) && (!remlen[dd] || rem[dd][0] != g)) head_everywhere = 0;
            if (head_everywhere && producers_placed(p, c->leads, cnt, g)) pick = g;
        }
        for (int d = 0; d < p->D && pick < 0; d++)
            for (int k = 0; k < remlen[d] && pick < 0; k++)
                if (producers_placed(p, c->leads, cnt, rem[d][k])) pick = rem[d][k];
        /* a pick always exists: the unplaced occurrences form a DAG under lag-0 dependencies */
        for (int dd = 0; dd < p->D; dd++) if (p->mask[pick] >> dd & 1u) {
            int k = 0;
            while (rem[dd][k] != pick) k++;
            memmove(&rem[dd][k], &rem[dd][k + 1], sizeof(int) * (size_t)(remlen[dd] - k - 1));
            remlen[dd]--;
            c->seq[dd][outlen[dd]++] = pick;
        }
        cnt[pick]++; placed++;
    }
}

/* Turns a candidate index into (leads, per-device type sequences).  Returns ORC_OK or the
 * structural reject reason (DUP, TP_MISMATCH, PROP2) -- only the FACTORIAL space has any.
 *
 * FACTORIAL (factorial number system per device): device d's slots are listed as
 *   (type ascending, label 0..N_R-1 ascending); index = sum_d r_d * prod_{d'<d} n_d'! with
 *   r_d the lexicographic rank of the device's permutation of that list.  The label of the
 *   first slot of a type in device order is its lead (its n_i of Eq. 3); by Property 1 the
 *   later labels must follow cyclically (lead, lead+1, ... mod N_R), otherwise the index
 *   names the same schedule as another index and is rejected as DUP.
 * CANONICAL: index = r_0 + C_0*(r_1 + C_1*(... (r_{D-1} + C_{D-1}*lead_rank))), r_d the
 *   lexicographic rank of device d's type sequence among the arrangements of its multiset
 *   (each type N_R times, smaller type id first), lead_rank into the table of enum_leads().
 * SAMPLED_*: the index is an ordinal into the counter-based stream above.  Leads: types in
 *   reverse topological order, lead_i = min(N_R-1, max over dependencies i->j of
 *   lead_j + step), step = 1 iff the two types sit on different device sets and draw e is
 *   below step_q16; a type nobody consumes has lead 0.  Orders: for device d, position p,
 *   digit = (draw(128+32d+p) * remaining) >> 16 picks among the remaining blocks listed
 *   (type ascending); only its type matters. */
static int decode(const orc_problem *p, uint64_t index, orc_candidate *c)
{
    const int NR = p->NR;
    if (p->space == ORC_SPACE_FACTORIAL) {
        int dup = 0, tp_mismatch = 0;
        int lead_seen[ORC_MAX_K];
        for (int i = 0; i < p->K; i++) lead_seen[i] = -1;
        for (int d = 0; d < p->D; d++) {
            int n = p->ntd[d] * NR;
            uint64_t r = index % p->cdev[d];
            index /= p->cdev[d];
            int list_t[ORC_MAX_N], list_l[ORC_MAX_N], ln = 0;
            for (int y = 0; y < p->ntd[d]; y++) for (int l = 0; l < NR; l++) { list_t[ln] = p->td[d][y]; list_l[ln] = l; ln++; }
            int first[ORC_MAX_K], seen[ORC_MAX_K];
            for (int i = 0; i < p->K; i++) { first[i] = -1; seen[i] = 0; }
            c->len[d] = n;
            for (int pos = 0; pos < n; pos++) {
                uint64_t f = factorial_or_zero(n - 1 - pos);
                int digit = (int)(r / f);
                r %= f;
                int g = list_t[digit], l = list_l[digit];
                for (int k = digit; k < ln - 1; k++) { list_t[k] = list_t[k + 1]; list_l[k] = list_l[k + 1]; }
                ln--;
                c->seq[d][pos] = g;
                if (first[g] < 0) first[g] = l;
                else if (l != (first[g] + seen[g]) % NR) dup = 1;
                seen[g]++;
            }
            for (int y = 0; y < p->ntd[d]; y++) {
                int g = p->td[d][y];
                if (lead_seen[g] < 0) lead_seen[g] = first[g];
                else if (lead_seen[g] != first[g]) tp_mismatch = 1;
            }
        }
        for (int i = 0; i < p->K; i++) c->leads[i] = lead_seen[i];
        if (dup) return ORC_DUP;                      /* reasons are reported in this order */
        if (tp_mismatch) return ORC_TP_MISMATCH;
        for (int e = 0; e < p->ndeps; e++) if (c->leads[p->src[e]] < c->leads[p->dst[e]]) return ORC_PROP2;
        return ORC_OK;
    }
    if (p->space == ORC_SPACE_CANONICAL) {
        for (int d = 0; d < p->D; d++) {
            uint64_t r = index % p->cdev[d];
            index /= p->cdev[d];
            int cnt[ORC_MAX_K], n = p->ntd[d] * NR;
            for (int y = 0; y < p->ntd[d]; y++) cnt[y] = NR;
            c->len[d] = n;
            for (int pos = 0; pos < n; pos++) {
                for (int y = 0; y < p->ntd[d]; y++) {
                    if (!cnt[y]) continue;
                    cnt[y]--;
                    uint64_t w = arrangements(cnt, p->ntd[d]);
                    if (r < w) { c->seq[d][pos] = p->td[d][y]; break; }
                    r -= w;
                    cnt[y]++;
                }
            }
        }
        for (int i = 0; i < p->K; i++) c->leads[i] = p->leadtab[(size_t)index * p->K + i];
        return ORC_OK;
    }
    /* sampled spaces */
    if (p->has_fixed) {
        for (int i = 0; i < p->K; i++) c->leads[i] = p->fixed[i];
    } else {
        for (int k = p->K - 1; k >= 0; k--) {
            int i = p->topo[k], lead = 0;
            for (int e = 0; e < p->ndeps; e++) if (p->src[e] == i) {
                int j = p->dst[e];
                int step = (p->mask[i] != p->mask[j]) && (draw16(p->seed, index, DRAW_LEAD_BASE + (uint32_t)e) < p->step_q16);
                if (c->leads[j] + step > lead) lead = c->leads[j] + step;
            }
            c->leads[i] = lead > NR - 1 ? NR - 1 : lead;
        }
    }
    for (int d = 0; d < p->D; d++) {
        int cnt[ORC_MAX_K], n = p->ntd[d] * NR;
        for (int y = 0; y < p->ntd[d]; y++) cnt[y] = NR;
        c->len[d] = n;
        for (int pos = 0; pos < n; pos++) {
            uint32_t u = draw16(p->seed, index, DRAW_ORD_BASE + 32u * (uint32_t)d + (uint32_t)pos);
            int digit = (int)((u * (uint32_t)(n - pos)) >> 16);
            int y = 0;
            while (digit >= cnt[y]) { digit -= cnt[y]; y++; }
            cnt[y]--;
            c->seq[d][pos] = p->td[d][y];
        }
    }
    if (p->space == ORC_SPACE_SAMPLED_REPAIR) repair_orders(p, c);
    return ORC_OK;
}

/* ------------------------------------------------------------------ evaluation of one candidate */

typedef struct { int u, v, w, lag; } orc_edge;

typedef struct {
    int n, ne, nlag1;
    orc_edge e[ORC_MAX_N * 2 + ORC_MAX_DEPS * ORC_MAX_NR];
    int order[ORC_MAX_N];               /* a topological order of the lag-0 graph */
} orc_graph;

/* Node (i, q) = q-th occurrence of type i in device order (Property 1) = slot that handles
 * micro-batch lead_i + q + N_R*k in window k.  Dependency i->j with Delta = lead_i - lead_j:
 * consumer (j, q) needs producer (i, q-Delta) of the same window when q >= Delta (lag 0,
 * s_c >= s_p + t_p), else (i, q-Delta+N_R) of the previous window (lag 1, s_c + T >= s_p + t_p).
 * Device exclusivity for a fixed order: consecutive slots lag 0, last -> first lag 1. */
static int build_graph(const orc_problem *p, const orc_candidate *c, orc_graph *g)
{
    const int NR = p->NR;
    g->n = p->K * NR; g->ne = 0; g->nlag1 = 0;
    for (int e = 0; e < p->ndeps; e++) {
        int i = p->src[e], j = p->dst[e], delta = c->leads[i] - c->leads[j];
        for (int q = 0; q < NR; q++) {
            orc_edge *x = &g->e[g->ne++];
            x->v = j * NR + q; x->w = p->t[i];
            if (q >= delta) { x->u = i * NR + q - delta; x->lag = 0; }
            else { x->u = i * NR + q - delta + NR; x->lag = 1; g->nlag1++; }
        }
    }
    for (int d = 0; d < p->D; d++) {
        int cnt[ORC_MAX_K] = {0}, prev = -1, first = -1;
        for (int k = 0; k < c->len[d]; k++) {
            int ty = c->seq[d][k], node = ty * NR + cnt[ty]++;
            if (prev >= 0) { orc_edge *x = &g->e[g->ne++]; x->u = prev; x->v = node; x->w = p->t[prev / NR]; x->lag = 0; }
            else first = node;
            prev = node;
        }
        orc_edge *x = &g->e[g->ne++];
        x->u = prev; x->v = first; x->w = p->t[prev / NR]; x->lag = 1; g->nlag1++;
    }
    /* Kahn on the lag-0 edges; a cycle means the order can never execute */
    int indeg[ORC_MAX_N] = {0}, queue[ORC_MAX_N], qh = 0, qt = 0;
    for (int k = 0; k < g->ne; k++) if (!g->e[k].lag) indeg[g->e[k].v]++;
    for (int v = 0; v < g->n; v++) if (!indeg[v]) queue[qt++] = v;
    while (qh < qt) {
        int u = queue[qh++];
        for (int k = 0; k < g->ne; k++) if (!g->e[k].lag && g->e[k].u == u && --indeg[g->e[k].v] == 0) queue[qt++] = g->e[k].v;
    }
    if (qt != g->n) return 0;
    memcpy(g->order, queue, sizeof(int) * (size_t)g->n);
    return 1;
}

/* incoming edges of every node, nodes in topological order of the lag-0 graph */
typedef struct { int start[ORC_MAX_N + 1]; orc_edge e[ORC_MAX_N * 2 + ORC_MAX_DEPS * ORC_MAX_NR]; } orc_in_edges;

static void group_in_edges(const orc_graph *g, orc_in_edges *in)
{
    int pos = 0;
    for (int k = 0; k < g->n; k++) {
        int v = g->order[k];
        in->start[k] = pos;
        for (int x = 0; x < g->ne; x++) if (g->e[x].v == v) in->e[pos++] = g->e[x];
    }
    in->start[g->n] = pos;
}

/* Least non-negative integer solution of  s_v >= s_u + w - lag*T  for all edges, or 0 if none.
 * Bellman-Ford from s = 0.  Edges are relaxed grouped by head node in topological order of the
 * lag-0 graph, so one pass settles every path that uses no further lag-1 edge; a simple path has
 * at most nlag1 lag-1 edges, hence a pass that still changes something after nlag1+1 passes
 * proves a positive cycle. */
static int feasible(const orc_graph *g, const orc_in_edges *in, int T, int *s)
{
    for (int v = 0; v < g->n; v++) s[v] = 0;
    for (int pass = 0; pass < g->nlag1 + 2; pass++) {
        int changed = 0;
        for (int k = 0; k < g->n; k++) {
            int v = g->order[k];
            for (int x = in->start[k]; x < in->start[k + 1]; x++) {
                int cand = s[in->e[x].u] + in->e[x].w - in->e[x].lag * T;
                orc_ops += 2;
                if (cand > s[v]) { s[v] = cand; changed = 1; }
            }
        }
        if (!changed) return 1;
    }
    return 0;
}

/* Smallest integer period (monotone in T: a larger T only loosens lag-1 constraints).
 * T = UB (all work of the window, serial) is always feasible for a deadlock-free order. */
static int min_period(const orc_problem *p, const orc_graph *g, int *s)
{
    static __thread orc_in_edges in;
    group_in_edges(g, &in);
    int lo = p->LB, hi = p->UB;
    while (lo < hi) {
        int mid = lo + (hi - lo) / 2;
        if (feasible(g, &in, mid, s)) hi = mid; else lo = mid + 1;
    }
    feasible(g, &in, lo, s);
    return lo;
}

/* Memory (Eq. 1 [2]): blocks that ran before the window give entry_d = sum_i m_i*lead_i
 * (type i has already handled micro-batches 0..lead_i-1); then m is added at each block
 * start in device order; the peak is the largest prefix. */
static int memory_peaks(const orc_problem *p, const orc_candidate *c, int *peak)
{
    int worst = 0, first = 1;
    for (int d = 0; d < p->D; d++) {
        int cur = 0, pk = 0;
        for (int y = 0; y < p->ntd[d]; y++) cur += p->m[p->td[d][y]] * c->leads[p->td[d][y]];
        for (int k = 0; k < c->len[d]; k++) {
            cur += p->m[c->seq[d][k]];
            if (k == 0 || cur > pk) pk = cur;
        }
        peak[d] = pk;
        if (first || pk > worst) { worst = pk; first = 0; }
    }
    return worst;
}

static void eval_decoded(const orc_problem *p, const orc_candidate *c, orc_score *out, int *starts)
{
    static __thread orc_graph g;
    static __thread int s[ORC_MAX_N];
    memset(out, 0, sizeof *out);
    for (int e = 0; e < p->ndeps; e++) if (c->leads[p->src[e]] < c->leads[p->dst[e]]) { out->status = ORC_PROP2; return; }
    if (!build_graph(p, c, &g)) { out->status = ORC_DEADLOCK; return; }
    out->peak_max = memory_peaks(p, c, out->peak);
    if (out->peak_max > p->M) { out->status = ORC_MEM; return; }
    out->status = ORC_OK;
    out->period = min_period(p, &g, s);
    if (starts) memcpy(starts, s, sizeof(int) * (size_t)g.n);
}

/* score of candidate `index`; starts (optional) receives the least start times at T*,
 * indexed type*N_R + occurrence */
int orc_eval_index(const orc_problem *p, uint64_t index, orc_score *out, int *starts)
{
    static __thread orc_candidate c;
    if (index >= p->count && p->count != UINT64_MAX) return ORC_E_RANGE;
    int st = decode(p, index, &c);
    if (st != ORC_OK) { memset(out, 0, sizeof *out); out->status = st; return ORC_E_OK; }
    eval_decoded(p, &c, out, starts);
    return ORC_E_OK;
}

/* decoded form of candidate `index`: leads[K], len[D], seq[D][stride] */
int orc_decode_index(const orc_problem *p, uint64_t index, int *status, int *leads, int *len, int *seq, int stride)
{
    static __thread orc_candidate c;
    if (index >= p->count && p->count != UINT64_MAX) return ORC_E_RANGE;
    *status = decode(p, index, &c);
    for (int i = 0; i < p->K; i++) leads[i] = c.leads[i];
    for (int d = 0; d < p->D; d++) {
        len[d] = c.len[d];
        for (int k = 0; k < c.len[d] && k < stride; k++) seq[d * stride + k] = c.seq[d][k];
    }
    return ORC_E_OK;
}

/* an explicitly given candidate (closed-form pins use this) */
int orc_eval_explicit(const orc_problem *p, const int *leads, const int *len, const int *seq, int stride,
                      orc_score *out, int *starts)
{
    static __thread orc_candidate c;
    int cnt[ORC_MAX_K] = {0};
    for (int i = 0; i < p->K; i++) { if (leads[i] < 0 || leads[i] >= p->NR) return ORC_E_INVALID; c.leads[i] = leads[i]; }
    for (int d = 0; d < p->D; d++) {
        if (len[d] != p->ntd[d] * p->NR) return ORC_E_INVALID;
        c.len[d] = len[d];
        for (int k = 0; k < len[d]; k++) {
            int g = seq[d * stride + k];
            if (g < 0 || g >= p->K || !(p->mask[g] >> d & 1u)) return ORC_E_INVALID;
            c.seq[d][k] = g;
            if (d == __builtin_ctz(p->mask[g])) cnt[g]++;
        }
    }
    for (int i = 0; i < p->K; i++) if (cnt[i] != p->NR) return ORC_E_INVALID;
    eval_decoded(p, &c, out, starts);
    return ORC_E_OK;
}

/* the repair rule on explicitly given priority lists (pins its scan order against a worked example):
 * seq_out[D][stride] receives the repaired per-device orders */
int orc_repair_explicit(const orc_problem *p, const int *leads, const int *len, const int *seq, int stride, int *seq_out)
{
    static __thread orc_candidate c;
    int cnt[ORC_MAX_K] = {0};
    for (int i = 0; i < p->K; i++) { if (leads[i] < 0 || leads[i] >= p->NR) return ORC_E_INVALID; c.leads[i] = leads[i]; }
    for (int e = 0; e < p->ndeps; e++) if (leads[p->src[e]] < leads[p->dst[e]]) return ORC_E_INVALID;
    for (int d = 0; d < p->D; d++) {
        if (len[d] != p->ntd[d] * p->NR) return ORC_E_INVALID;
        c.len[d] = len[d];
        for (int k = 0; k < len[d]; k++) {
            int g = seq[d * stride + k];
            if (g < 0 || g >= p->K || !(p->mask[g] >> d & 1u)) return ORC_E_INVALID;
            c.seq[d][k] = g;
            if (d == __builtin_ctz(p->mask[g])) cnt[g]++;
        }
    }
    for (int i = 0; i < p->K; i++) if (cnt[i] != p->NR) return ORC_E_INVALID;
    repair_orders(p, &c);
    for (int d = 0; d < p->D; d++)
        for (int k = 0; k < c.len[d]; k++) seq_out[d * stride + k] = c.seq[d][k];
    return ORC_E_OK;
}

/* feasibility of one period for an explicit candidate (pins the monotone search) */
int orc_feasible_explicit(const orc_problem *p, const int *leads, const int *len, const int *seq, int stride, int T)
{
    static __thread orc_candidate c;
    static __thread orc_graph g;
    static __thread int s[ORC_MAX_N];
    for (int i = 0; i < p->K; i++) c.leads[i] = leads[i];
    for (int d = 0; d < p->D; d++) { c.len[d] = len[d]; for (int k = 0; k < len[d]; k++) c.seq[d][k] = seq[d * stride + k]; }
    static __thread orc_in_edges in;
    if (!build_graph(p, &c, &g)) return -1;
    group_in_edges(&g, &in);
    return feasible(&g, &in, T, s);
}

/* ------------------------------------------------------------------ brute-force sweep + argmin */

typedef struct {
    int period;                          /* best T*, -1 if nothing feasible */
    uint64_t index;                      /* lowest index attaining it (Alg. 1 keeps the first) */
    int peak[ORC_MAX_D];
    int peak_max;
    uint64_t n_evaluated, n_feasible, n_reject[ORC_NSTATUS];
    uint64_t ops;                        /* period-computation steps counted (see orc_ops) */
} orc_result;

static void sweep_range(const orc_problem *p, uint64_t first, uint64_t count, orc_result *r)
{
    memset(r, 0, sizeof *r);
    r->period = -1;
    orc_ops = 0;
    for (uint64_t k = 0; k < count; k++) {
        orc_score sc;
        uint64_t idx = first + k;
        orc_eval_index(p, idx, &sc, NULL);
        r->n_evaluated++;
        if (sc.status != ORC_OK) { r->n_reject[sc.status]++; continue; }
        r->n_feasible++;
        if (r->period < 0 || sc.period < r->period) {          /* strict <: first found wins */
            r->period = sc.period; r->index = idx; r->peak_max = sc.peak_max;
            memcpy(r->peak, sc.peak, sizeof sc.peak);
        }
    }
    r->ops = orc_ops;
}

int orc_sweep(const orc_problem *p, uint64_t first, uint64_t count, orc_result *r)
{
    if (p->count != UINT64_MAX && (first > p->count || count > p->count - first)) return ORC_E_RANGE;
    sweep_range(p, first, count, r);
    return ORC_E_OK;
}

typedef struct { const orc_problem *p; uint64_t first, count; orc_result r; } orc_job;
static void *sweep_thread(void *arg) { orc_job *j = (orc_job *)arg; sweep_range(j->p, j->first, j->count, &j->r); return NULL; }

/* same result as orc_sweep, the range cut into contiguous pieces, one per thread */
int orc_sweep_mt(const orc_problem *p, uint64_t first, uint64_t count, int nthreads, orc_result *r)
{
    if (p->count != UINT64_MAX && (first > p->count || count > p->count - first)) return ORC_E_RANGE;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    orc_job *jobs = (orc_job *)calloc((size_t)nthreads, sizeof *jobs);
    pthread_t *th = (pthread_t *)calloc((size_t)nthreads, sizeof *th);
    uint64_t per = count / (uint64_t)nthreads, extra = count % (uint64_t)nthreads, at = first;
    for (int k = 0; k < nthreads; k++) {
        jobs[k].p = p; jobs[k].first = at; jobs[k].count = per + ((uint64_t)k < extra);
        at += jobs[k].count;
        pthread_create(&th[k], NULL, sweep_thread, &jobs[k]);
    }
    memset(r, 0, sizeof *r);
    r->period = -1;
    for (int k = 0; k < nthreads; k++) {
        pthread_join(th[k], NULL);
        const orc_result *x = &jobs[k].r;
        r->n_evaluated += x->n_evaluated; r->n_feasible += x->n_feasible; r->ops += x->ops;
        for (int s = 0; s < ORC_NSTATUS; s++) r->n_reject[s] += x->n_reject[s];
        if (x->period >= 0 && (r->period < 0 || x->period < r->period)) {     /* pieces ascend in index */
            r->period = x->period; r->index = x->index; r->peak_max = x->peak_max;
            memcpy(r->peak, x->peak, sizeof x->peak);
        }
    }
    free(jobs); free(th);
    return ORC_E_OK;
}

/* per-candidate records: code[k] = T* if feasible else -(reject reason); peakmax[k] */
int orc_score_range(const orc_problem *p, uint64_t first, uint64_t count, int32_t *code, int32_t *peakmax)
{
    if (p->count != UINT64_MAX && (first > p->count || count > p->count - first)) return ORC_E_RANGE;
    for (uint64_t k = 0; k < count; k++) {
        orc_score sc;
        orc_eval_index(p, first + k, &sc, NULL);
        code[k] = sc.status == ORC_OK ? sc.period : -sc.status;
        if (peakmax) peakmax[k] = sc.peak_max;
    }
    return ORC_E_OK;
}

/* ------------------------------------------------------------------ schedule completion
 * Blocks of N micro-batches around R = floor((N - max lead) / N_R) copies of the window.
 * Warm-up = {(i, mu): mu < lead_i}  (Eq. 5 applied to every micro-batch the windows skip),
 * steady  = window k handles mu = lead_i + q + N_R*k,
 * cool-down = {(i, mu): lead_i + N_R*R <= mu < N}  (Eq. 6 likewise).
 * Per-device order = warm-up order, the R windows, cool-down order.  The paper finds the two
 * outer orders with a time-optimal solver; this build's convention is a serial greedy list
 * schedule instead: among the unscheduled blocks of the phase whose producers are scheduled
 * and whose memory delta keeps every device it occupies at or below M, take the one with the
 * smallest (earliest start, micro-batch, type id), the earliest start being the maximum of
 * its devices' free times and its producers' end times; append it.  Start times of window
 * blocks are their earliest ones in the flat order (an ordinary DAG, no lags).
 * Output arrays are indexed type*N + mu.  Returns the makespan or a negative error. */
int orc_complete(const orc_problem *p, const int *leads, const int *len, const int *seq, int stride, int N,
                 int *start /* [K*N] */, int *dev_order /* [D][K*N] as type*N+mu, -1 padded */, int *dev_len /* [D] */)
{
    const int NR = p->NR, K = p->K, D = p->D;
    int maxlead = 0;
    for (int i = 0; i < K; i++) if (leads[i] > maxlead) maxlead = leads[i];
    int R = (N - maxlead) / NR;
    if (N < 1 || R < 1) return ORC_E_RANGE;
    int *end = (int *)malloc(sizeof(int) * (size_t)K * (size_t)N);
    char *done = (char *)calloc((size_t)K * (size_t)N, 1);
    int freeat[ORC_MAX_D] = {0}, cur[ORC_MAX_D] = {0};
    for (int d = 0; d < D; d++) dev_len[d] = 0;
    int rc = 0;
#define PLACE(i_, mu_, st_) do { int i__ = (i_), mu__ = (mu_), st__ = (st_); \
        start[i__ * N + mu__] = st__; end[i__ * N + mu__] = st__ + p->t[i__]; done[i__ * N + mu__] = 1; \
        for (int d__ = 0; d__ < D; d__++) if (p->mask[i__] >> d__ & 1u) { \
            freeat[d__] = st__ + p->t[i__]; cur[d__] += p->m[i__]; \
            dev_order[d__ * K * N + dev_len[d__]++] = i__ * N + mu__; } } while (0)
    for (int phase = 0; phase < 3 && rc == 0; phase++) {
        if (phase == 1) {
            for (int k = 0; k < R && rc == 0; k++) {
                /* one window: place blocks in any topological order that respects the candidate's
                 * device orders; repeat "advance a device whose next block is ready" */
                int pos[ORC_MAX_D] = {0}, cnt[ORC_MAX_K] = {0}, left = K * NR;
                while (left > 0) {
                    int progressed = 0;
                    for (int d = 0; d < D; d++) {
                        if (pos[d] >= len[d]) continue;
                        int i = seq[d * stride + pos[d]], mu = leads[i] + cnt[i] + NR * k, ok = 1, est = 0;
                        for (int dd = 0; dd < D; dd++) if (p->mask[i] >> dd & 1u) {
                            if (pos[dd] >= len[dd] || seq[dd * stride + pos[dd]] != i) ok = 0;
                            if (freeat[dd] > est) est = freeat[dd];
                        }
                        for (int e = 0; e < p->ndeps && ok; e++) if (p->dst[e] == i) {
                            if (!done[p->src[e] * N + mu]) ok = 0;
                            else if (end[p->src[e] * N + mu] > est) est = end[p->src[e] * N + mu];
                        }
                        if (!ok) continue;
                        PLACE(i, mu, est);
                        for (int dd = 0; dd < D; dd++) if (p->mask[i] >> dd & 1u) pos[dd]++;
                        cnt[i]++; left--; progressed = 1;
                    }
                    if (!progressed) { rc = ORC_E_NO_SCHEDULE; break; }
                }
            }
            continue;
        }
        for (;;) {
            int best_i = -1, best_mu = 0, best_est = 0, any_left = 0;
            for (int i = 0; i < K; i++) {
                int lo = phase == 0 ? 0 : leads[i] + NR * R, hi = phase == 0 ? leads[i] : N;
                for (int mu = lo; mu < hi; mu++) {
                    if (done[i * N + mu]) continue;
                    any_left = 1;
                    int ok = 1, est = 0;
                    for (int e = 0; e < p->ndeps && ok; e++) if (p->dst[e] == i) {
                        if (!done[p->src[e] * N + mu]) ok = 0;
                        else if (end[p->src[e] * N + mu] > est) est = end[p->src[e] * N + mu];
                    }
                    for (int d = 0; d < D && ok; d++) if (p->mask[i] >> d & 1u) {
                        if (p->m[i] > 0 && cur[d] + p->m[i] > p->M) ok = 0;
                        if (freeat[d] > est) est = freeat[d];
                    }
                    if (!ok) continue;
                    if (best_i < 0 || est < best_est || (est == best_est && (mu < best_mu || (mu == best_mu && i < best_i)))) {
                        best_i = i; best_mu = mu; best_est = est;
                    }
                }
            }
            if (!any_left) break;
            if (best_i < 0) { rc = ORC_E_NO_SCHEDULE; break; }
            PLACE(best_i, best_mu, best_est);
        }
    }
#undef PLACE
    int makespan = 0;
    if (rc == 0) for (int x = 0; x < K * N; x++) if (end[x] > makespan) makespan = end[x];
    free(end); free(done);
    return rc ? rc : makespan;
}


/* ------------------------------------------------------------------ searched completion
 * The paper orders warm-up and cool-down with a time-optimal solver (Sec. IV-C, Alg. 1); the greedy
 * rule above is one guess.  This build searches a family of such guesses instead: completion
 * candidate `ordinal` perturbs the greedy choice.  Per phase every block type offers its lowest
 * unscheduled micro-batch only (Property 1: blocks of one type run in micro-batch order); an offered
 * block is eligible when its producer's block of the same micro-batch is scheduled and its memory
 * delta fits on all its devices; among the eligible the smallest (earliest start + jitter,
 * micro-batch, type id) is appended at its earliest start.  jitter = 0 for ordinal 0 (the plain
 * greedy schedule) or when the amplitude J is 0; otherwise (draw * (J + 1)) >> 16 with the 16-bit draw
 * number type*N + mu of the counter-based stream keyed by (seed + ORC_COMPLETION_KEY, ordinal).
 * The windows in between are replayed exactly as in orc_complete.  Returns the makespan or an error. */
#define ORC_COMPLETION_KEY 0x632BE59BD9B4E019ULL
int orc_complete_jitter(const orc_problem *p, const int *leads, const int *len, const int *seq, int stride, int N,
                        uint64_t ordinal, int J, int *start, int *dev_order, int *dev_len)
{
    const int NR = p->NR, K = p->K, D = p->D;
    int maxlead = 0;
    for (int i = 0; i < K; i++) if (leads[i] > maxlead) maxlead = leads[i];
    int R = (N - maxlead) / NR;
    if (N < 1 || R < 1 || J < 0 || J > 65535) return ORC_E_RANGE;
    int *end = (int *)malloc(sizeof(int) * (size_t)K * (size_t)N);
    int next[ORC_MAX_K];                 /* per type: the next micro-batch to schedule */
    int freeat[ORC_MAX_D] = {0}, cur[ORC_MAX_D] = {0};
    for (int i = 0; i < K; i++) next[i] = 0;
    for (int d = 0; d < D; d++) dev_len[d] = 0;
    int rc = 0;
    for (int phase = 0; phase < 3 && rc == 0; phase++) {
        if (phase == 1) {                /* R windows, replayed in an executable sequence of the device orders */
            for (int k = 0; k < R && rc == 0; k++) {
                int pos[ORC_MAX_D] = {0}, left = K * NR;
                while (left > 0) {
                    int progressed = 0;
                    for (int d = 0; d < D; d++) {
                        if (pos[d] >= len[d]) continue;
                        int i = seq[d * stride + pos[d]], mu = next[i], ok = 1, est = 0;
                        for (int dd = 0; dd < D; dd++) if (p->mask[i] >> dd & 1u) {
                            if (pos[dd] >= len[dd] || seq[dd * stride + pos[dd]] != i) ok = 0;
                            if (freeat[dd] > est) est = freeat[dd];
                        }
                        for (int e = 0; e < p->ndeps && ok; e++) if (p->dst[e] == i) {
                            if (next[p->src[e]] <= mu) ok = 0;
                            else if (end[p->src[e] * N + mu] > est) est = end[p->src[e] * N + mu];
                        }
                        if (!ok) continue;
                        start[i * N + mu] = est; end[i * N + mu] = est + p->t[i]; next[i]++;
                        for (int dd = 0; dd < D; dd++) if (p->mask[i] >> dd & 1u) {
                            freeat[dd] = est + p->t[i]; cur[dd] += p->m[i]; pos[dd]++;
                            dev_order[dd * K * N + dev_len[dd]++] = i * N + mu;
                        }
                        left--; progressed = 1;
                    }
                    if (!progressed) { rc = ORC_E_NO_SCHEDULE; break; }
                }
            }
            continue;
        }
        for (;;) {
            int best_i = -1, best_mu = 0, best_est = 0, best_key = 0, any_left = 0;
            for (int i = 0; i < K; i++) {
                int hi = phase == 0 ? leads[i] : N, mu = next[i];
                if (mu >= hi) continue;
                any_left = 1;
                int ok = 1, est = 0;
                for (int e = 0; e < p->ndeps && ok; e++) if (p->dst[e] == i) {
                    if (next[p->src[e]] <= mu) ok = 0;
                    else if (end[p->src[e] * N + mu] > est) est = end[p->src[e] * N + mu];
                }
                for (int d = 0; d < D && ok; d++) if (p->mask[i] >> d & 1u) {
                    if (p->m[i] > 0 && cur[d] + p->m[i] > p->M) ok = 0;
                    if (freeat[d] > est) est = freeat[d];
                }
                if (!ok) continue;
                int jitter = 0;
                if (ordinal != 0 && J > 0)
                    jitter = (int)((draw16(p->seed + ORC_COMPLETION_KEY, ordinal, (uint32_t)(i * N + mu)) * (uint32_t)(J + 1)) >> 16);
                int key = est + jitter;
                if (best_i < 0 || key < best_key || (key == best_key && (mu < best_mu || (mu == best_mu && i < best_i)))) {
                    best_i = i; best_mu = mu; best_est = est; best_key = key;
                }
            }
            if (!any_left) break;
            if (best_i < 0) { rc = ORC_E_NO_SCHEDULE; break; }
            start[best_i * N + best_mu] = best_est; end[best_i * N + best_mu] = best_est + p->t[best_i]; next[best_i]++;
            for (int d = 0; d < D; d++) if (p->mask[best_i] >> d & 1u) {
                freeat[d] = best_est + p->t[best_i]; cur[d] += p->m[best_i];
                dev_order[d * K * N + dev_len[d]++] = best_i * N + best_mu;
            }
        }
    }
    int makespan = 0;
    if (rc == 0) for (int d = 0; d < D; d++) if (freeat[d] > makespan) makespan = freeat[d];
    free(end);
    return rc ? rc : makespan;
}

/* makespans of completion candidates first .. first+count-1 (INT32_MAX where no schedule exists) and the
 * lowest ordinal attaining the least one */
int orc_completion_scores(const orc_problem *p, const int *leads, const int *len, const int *seq, int stride, int N,
                          uint64_t first, uint64_t count, int J, int32_t *makespan, uint64_t *best_ordinal)
{
    int *start = (int *)malloc(sizeof(int) * (size_t)p->K * (size_t)N);
    int *order = (int *)malloc(sizeof(int) * (size_t)p->D * (size_t)p->K * (size_t)N);
    int dl[ORC_MAX_D], best = INT32_MAX;
    *best_ordinal = 0;
    for (uint64_t k = 0; k < count; k++) {
        int mk = orc_complete_jitter(p, leads, len, seq, stride, N, first + k, J, start, order, dl);
        if (mk == ORC_E_RANGE) { free(start); free(order); return mk; }
        int32_t v = mk < 0 ? INT32_MAX : mk;
        if (makespan) makespan[k] = v;
        if (v < best) { best = v; *best_ordinal = first + k; }
    }
    free(start); free(order);
    return best == INT32_MAX ? ORC_E_NO_SCHEDULE : best;
}

/* ------------------------------------------------------------------ Alg. 1, the whole search
 * CalMaxInflight (Alg. 1; the paper only says "the maximum number of in-flight micro-batches
 * that can be executed within the memory constraints"): this build's reading.  One micro-batch
 * that runs alone, its blocks in topological order (smallest type id first), holds on device d
 * at most hold_d = the largest prefix sum of m over its blocks on d.  n micro-batches in flight
 * can hold n * hold_d there, so inflights = min over devices with hold_d > 0 of floor(M / hold_d);
 * a problem that holds no memory anywhere is not bounded by memory (returns `unbounded`). */
int orc_max_inflight(const orc_problem *p, int unbounded)
{
    int best = unbounded;
    for (int d = 0; d < p->D; d++) {
        int run = 0, hold = 0;
        for (int k = 0; k < p->K; k++) {
            int i = p->topo[k];
            if (p->mask[i] >> d & 1u) { run += p->m[i]; if (run > hold) hold = run; }
        }
        if (hold > 0 && p->M / hold < best) best = p->M / hold;
    }
    return best;
}

typedef struct {
    int inflights;                       /* CalMaxInflight                                     */
    int lower_bound;                     /* GetLowerBound: max_d sum of t on d, per micro-batch */
    int nr_tried;                        /* window sizes entered                               */
    int best_nr, best_period;            /* incumbent: t_R = best_period / best_nr; 0/-1 = none */
    uint64_t best_index;
    int early_exit;                      /* the lower bound was reached                        */
    int period_nr[ORC_MAX_NR + 1];       /* best T* seen at window size N_R (-1 = none), [0] unused */
    uint64_t index_nr[ORC_MAX_NR + 1];   /* first index attaining it                            */
    uint64_t evaluated_nr[ORC_MAX_NR + 1];
} orc_search_result;

/* Alg. 1 as printed, one candidate at a time: N_R = 1 .. inflights (and <= max_nr), every
 * candidate index of that window size in ascending order (at most max_candidates of them),
 * the incumbent replaced on a strictly smaller repetend time only, return as soon as the lower
 * bound is met.  Repetend times of different window sizes are compared per micro-batch:
 * T_a / N_a < T_b / N_b  <=>  T_a * N_b < T_b * N_a.  The incumbent starts empty instead of
 * at the serial time (a reading: as printed, a problem where nothing beats serial execution
 * would get no schedule at all; whenever something does, both give the same result). */
int orc_search(int D, int K, int M, const int *t, const int *m, const uint32_t *mask,
               int ndeps, const int *src, const int *dst, int space, uint64_t seed, uint32_t step_q16,
               int max_nr, int use_inflight_bound, uint64_t max_candidates, orc_search_result *out)
{
    memset(out, 0, sizeof *out);
    out->best_period = -1;
    for (int n = 0; n <= ORC_MAX_NR; n++) out->period_nr[n] = -1;
    if (max_nr < 1 || max_nr > ORC_MAX_NR) return ORC_E_INVALID;
    int limit = max_nr;
    for (int NR = 1; NR <= limit; NR++) {
        int err;
        orc_problem *p = orc_create(D, K, NR, M, t, m, mask, ndeps, src, dst, space, NULL, seed, step_q16, &err);
        if (!p) return err;
        if (NR == 1) {
            out->lower_bound = p->LB;                        /* N_R = 1: LB is the per-micro-batch bound */
            out->inflights = orc_max_inflight(p, max_nr);          /* no memory held anywhere: no bound beyond max_nr */
            if (use_inflight_bound && out->inflights < limit) limit = out->inflights;
            if (limit < 1) { orc_destroy(p); return ORC_E_OK; }
        }
        out->nr_tried = NR;
        uint64_t n = p->count < max_candidates ? p->count : max_candidates;
        for (uint64_t idx = 0; idx < n; idx++) {
            orc_score sc;
            orc_eval_index(p, idx, &sc, NULL);
            out->evaluated_nr[NR]++;
            if (sc.status != ORC_OK) continue;
            if (out->period_nr[NR] < 0 || sc.period < out->period_nr[NR]) { out->period_nr[NR] = sc.period; out->index_nr[NR] = idx; }
            if (out->best_period >= 0 && (int64_t)sc.period * out->best_nr >= (int64_t)out->best_period * NR) continue;
            out->best_period = sc.period; out->best_nr = NR; out->best_index = idx;
            if (sc.period == NR * out->lower_bound) { out->early_exit = 1; orc_destroy(p); return ORC_E_OK; }
        }
        orc_destroy(p);
    }
    return ORC_E_OK;
}

/* ------------------------------------------------------------------ runtime instantiation (Sec. IV-D)
 * A complete schedule fixes start times and per-device orders; what the devices execute is one
 * global sequence of operations.  Blocks come in ascending start time; blocks that start together
 * are consecutive, devices in ascending order, each device's blocks in its execution order (a block
 * on several devices appears once, with its lowest device).  Every tensor that a consumer needs on a
 * device where the producer did not run is one send/receive pair, treated as a single operation and
 * placed right after the time slot (the group of equal start times) of the block that produces it.
 * This build's reading where the paper is silent: the sender is the lowest device of the producer;
 * pairs of one slot follow the order of their producers in the sequence, then the dependency's
 * position in the problem statement, then the receiving device.
 * op = 5 ints: kind (0 block, 1 pair), block (type*N + mu; for a pair: the producer), src (block:
 * device mask; pair: sender), dst (block: start time; pair: receiver), aux (block: 0; pair: consumer). */
int orc_instantiate(const orc_problem *p, int N, const int *start, const int *dev_order, const int *dev_len, int stride,
                    int *ops, int capacity)
{
    const int K = p->K, D = p->D;
    int nops = 0, emitted = 0, total = K * N;
    char *done = (char *)calloc((size_t)total, 1);
    while (emitted < total) {
        /* next time slot = least start among blocks not emitted yet */
        int slot = -1;
        for (int x = 0; x < total; x++) if (!done[x] && (slot < 0 || start[x] < slot)) slot = start[x];
        int first_of_slot = nops;
        for (int d = 0; d < D; d++)
            for (int k = 0; k < dev_len[d]; k++) {
                int x = dev_order[d * stride + k];
                if (done[x] || start[x] != slot) continue;
                done[x] = 1; emitted++;
                if (nops >= capacity) { free(done); return ORC_E_RANGE; }
                int *o = ops + 5 * nops++;
                o[0] = 0; o[1] = x; o[2] = (int)p->mask[x / N]; o[3] = slot; o[4] = 0;
            }
        int last_of_slot = nops;
        for (int q = first_of_slot; q < last_of_slot; q++) {
            int x = ops[5 * q + 1], i = x / N, mu = x % N;
            for (int e = 0; e < p->ndeps; e++) {
                if (p->src[e] != i) continue;
                int j = p->dst[e], sender = 0;
                while (!(p->mask[i] >> sender & 1u)) sender++;
                for (int v = 0; v < D; v++) {
                    if (!(p->mask[j] >> v & 1u) || (p->mask[i] >> v & 1u)) continue;
                    if (nops >= capacity) { free(done); return ORC_E_RANGE; }
                    int *o = ops + 5 * nops++;
                    o[0] = 1; o[1] = x; o[2] = sender; o[3] = v; o[4] = j * N + mu;
                }
            }
        }
    }
    free(done);
    return nops;
}

uint64_t orc_sizeof_score(void) { return sizeof(orc_score); }
uint64_t orc_sizeof_result(void) { return sizeof(orc_result); }
uint64_t orc_sizeof_search_result(void) { return sizeof(orc_search_result); }
