/*
 * Sequential CPU oracle for the Tsetlin machine hot path (test infrastructure).
 *
 * This file is TEST INFRASTRUCTURE.  It is a deliberately plain, single-threaded
 * restatement of what the paper's method computes, written literal by literal on
 * unpacked booleans, so that it can be checked against the paper by eye.  It is
 * used only by the test-suite, by the smoke check and by the benchmark's
 * "cpu_baseline" leg.  It shares no code, header, table or helper with the HIP
 * library; the product never calls it.
 *
 * Notation follows the paper (Section 2.1): o Boolean features, 2o literals,
 * m classes, n clauses per class, 2N states per Tsetlin automaton (TA), voting
 * margin T, specificity s, q examples.
 *
 * Data conventions of this file
 *   X      uint8  [q][o]        feature values 0/1
 *   y      int32  [q]           class label 0..m-1 (regression mode: target 0..T)
 *   state  int32  [m*n][2o]     TA state 1..2N.  Literal k<o is x_k, literal
 *                               o+k is NOT x_k (Section 2.1, literal set L).
 *   clause g = c*n + j belongs to class c; it has positive polarity iff j is
 *   odd (Section 2.1: "odd indexes positive"; the worked XOR example numbers
 *   clauses from 0 and lets C_1, C_3 vote for y=1).
 *
 * Readings of points the paper leaves open:
 *   - A TA includes its literal iff state > N.  Section 2.2 says the counter is
 *     increased to reinforce Include, so Include must be the upper half.
 *   - An empty clause outputs 1 (empty conjunction, Eq. 1).
 *   - The gate fires iff r * 2T < e * 2^32 for a 32-bit uniform r, i.e. with
 *     probability e/2T, never at e = 0 (Section 2.2: nothing is reinforced once
 *     v reaches T) and always at e = 2T.
 *   - Multi-class: class y_i is trained towards output 1 and one other class,
 *     drawn per (epoch, example), towards output 0.
 *   - The tally refresh of Algorithm 1 (its last five lines) is done for every
 *     visited (clause, example) pair and adds polarity * (o - o*), so that the
 *     tallies converge to the signed sum of Eq. 3 ("eventual consistency").
 *
 * Regression mode (the regression Tsetlin machine of Section 4.1).  The paper
 * measures it but does not restate its update rule; this file follows the rule of
 * the regression TM publication it cites (Abeyrathna et al., 2020), expressed in
 * the quantities of Algorithm 1:
 *   - one bank of n clauses (m = 1), every clause votes +1 (no negative polarity);
 *   - the output is the vote sum clipped to [0, T]; targets are integers y in
 *     [0, T] (the caller scales its continuous target to that range);
 *   - with vc = clip(v, 0, T): nothing happens at vc = y; at vc < y every clause
 *     receives Type I feedback with probability (y - vc)/T, at vc > y Type II
 *     feedback with probability (vc - y)/T.  The draw is the gate's:
 *     fire iff r * T < |y - vc| * 2^32.
 * Everything else (clause evaluation, Type I / II tables, tally refresh, random
 * streams) is shared with classification.
 *
 * What pins this file (tests that run without a GPU): the worked examples, Table 1 and
 * Table 2 of the paper cell by cell, brute force on sets for Eq. 1 - Eq. 3, exact end points
 * and frequencies of the gate, the training loops (synchronous, Algorithm 1 in both loop
 * orders, in batches, under a frozen snapshot) against a restatement in pure Python on sets,
 * the gate / negative-class / initial-state draws against raw Philox words, Philox itself
 * against an independent engine.
 * PARITY UNPINNED against the paper, because it prints nothing to pin them to: the
 * regression rule (otm_gate_regression and role 3 of the loops: taken from the cited
 * publication and pinned only against that rule's own closed forms); the choice of one
 * negative class per example (otm_neg_class), of the initial states (otm_init), of the output
 * of an empty clause, and of refreshing every visited pair (visit); and the accuracy any
 * of the training loops reaches (only compared with each other).
 *
 * Randomness: Philox4x32-10 (Salmon et al., SC'11), key = seed, counter
 *   ( blk | stream<<28 , g , i mod 2^32 , epoch | (i>>32)<<24 ).
 * Streams: 0 initial states, 1 gate, 2 Type I, 3 negative class.
 * A literal k has a "slot" (lw, j): half h = (k >= o), f = k - h*o,
 *   lw = h*ceil(o/32) + f/32, j = f mod 32.
 * Its 16-bit uniform for Type I feedback is
 *   u = sum_{b=0..15} bit_j( word[b mod 4] of block 4*lw + b/4 ) << b.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t  m;      /* classes                     */
    int32_t  n;      /* clauses per class (even)    */
    int32_t  o;      /* Boolean features            */
    int32_t  N;      /* states per action           */
    int32_t  T;      /* voting margin               */
    double   s;      /* specificity                 */
    uint64_t seed;
    int32_t  boost;  /* boost true positives: the strong Type I probability (s-1)/s becomes 1
                        (footnote of Section 2.2) */
    int32_t  regression; /* 1: regression mode (m = 1, y in [0, T]), see above */
} otm_config;

enum { OTM_INIT = 0, OTM_GATE = 1, OTM_TYPE1 = 2, OTM_NEGCLASS = 3 };

/* ---- Philox4x32-10 ---------------------------------------------------- */

void otm_philox(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void draw(const otm_config *cfg, uint32_t stream, uint32_t blk, uint32_t g,
                 uint64_t i, uint32_t epoch, uint32_t out[4])
{
    uint32_t ctr[4], key[2];
    ctr[0] = blk | (stream << 28);
    ctr[1] = g;
    ctr[2] = (uint32_t)(i & 0xffffffffu);
    ctr[3] = epoch | ((uint32_t)(i >> 32) << 24);
    key[0] = (uint32_t)(cfg->seed & 0xffffffffu);
    key[1] = (uint32_t)(cfg->seed >> 32);
    otm_philox(ctr, key, out);
}

/* slot of literal k */
static void slot_of(const otm_config *cfg, int k, int *lw, int *j)
{
    int Wf = (cfg->o + 31) / 32;
    int h = (k >= cfg->o);
    int f = k - h * cfg->o;
    *lw = h * Wf + f / 32;
    *j = f % 32;
}

/* ---- helpers on one example ------------------------------------------- */

/* literal values of one example: lit[k] = x_k, lit[o+k] = 1 - x_k (Section 2.1) */
static void literals(const otm_config *cfg, const uint8_t *x, uint8_t *lit)
{
    for (int k = 0; k < cfg->o; ++k) {
        lit[k] = x[k] ? 1 : 0;
        lit[cfg->o + k] = x[k] ? 0 : 1;
    }
}

/* Eq. 1: conjunction of the included literals */
static int clause_output(const otm_config *cfg, const int32_t *st, const uint8_t *lit)
{
    for (int k = 0; k < 2 * cfg->o; ++k)
        if (st[k] > cfg->N && lit[k] == 0)
            return 0;
    return 1;
}

static int polarity_sign(const otm_config *cfg, int g)
{
    int j = g % cfg->n;
    if (cfg->regression)
        return +1;
    return (j & 1) ? +1 : -1;
}

/* Eq. 3 for one class */
static int32_t vote_sum(const otm_config *cfg, const int32_t *state, const uint8_t *lit, int c)
{
    int32_t v = 0;
    int L = 2 * cfg->o;
    for (int j = 0; j < cfg->n; ++j) {
        int g = c * cfg->n + j;
        v += polarity_sign(cfg, g) * clause_output(cfg, state + (size_t)g * L, lit);
    }
    return v;
}

static int32_t clip(int32_t v, int32_t lo, int32_t hi)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

/* ---- public pieces ---------------------------------------------------- */

/* Initial states: every TA starts at N or N+1 with probability 1/2 each. */
void otm_init(const otm_config *cfg, int32_t *state)
{
    int L = 2 * cfg->o, C = cfg->m * cfg->n;
    for (int g = 0; g < C; ++g)
        for (int k = 0; k < L; ++k) {
            int lw, j;
            uint32_t r[4];
            slot_of(cfg, k, &lw, &j);
            draw(cfg, OTM_INIT, 4u * (uint32_t)lw, (uint32_t)g, 0, 0, r);
            state[(size_t)g * L + k] = cfg->N + (int32_t)((r[0] >> j) & 1u);
        }
}

/* out[i][g] = C_g(X_i)  (Eq. 1) */
void otm_clause_outputs(const otm_config *cfg, const int32_t *state, const uint8_t *X,
                        int64_t q, uint8_t *out)
{
    int L = 2 * cfg->o, C = cfg->m * cfg->n;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    for (int64_t i = 0; i < q; ++i) {
        literals(cfg, X + i * cfg->o, lit);
        for (int g = 0; g < C; ++g)
            out[i * C + g] = (uint8_t)clause_output(cfg, state + (size_t)g * L, lit);
    }
    free(lit);
}

/* sums[i][c] = Eq. 3 per class; clamped to [-T,T] ([0,T] in regression mode) if clamp != 0 */
void otm_class_sums(const otm_config *cfg, const int32_t *state, const uint8_t *X,
                    int64_t q, int clamp, int32_t *sums)
{
    int L = 2 * cfg->o;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    for (int64_t i = 0; i < q; ++i) {
        literals(cfg, X + i * cfg->o, lit);
        for (int c = 0; c < cfg->m; ++c) {
            int32_t v = vote_sum(cfg, state, lit, c);
            sums[i * cfg->m + c] = clamp ? clip(v, cfg->regression ? 0 : -cfg->T, cfg->T) : v;
        }
    }
    free(lit);
}

/* pred[i] = lowest class index with the largest clamped sum; in regression mode the
 * clipped vote sum itself (the prediction in units of 1/T of the target range) */
void otm_predict(const otm_config *cfg, const int32_t *state, const uint8_t *X,
                 int64_t q, int32_t *pred)
{
    int32_t *sums = (int32_t *)malloc(sizeof(int32_t) * (size_t)q * cfg->m);
    otm_class_sums(cfg, state, X, q, 1, sums);
    for (int64_t i = 0; i < q; ++i) {
        int best = 0;
        if (cfg->regression) {
            pred[i] = sums[i];
            continue;
        }
        for (int c = 1; c < cfg->m; ++c)
            if (sums[i * cfg->m + c] > sums[i * cfg->m + best])
                best = c;
        pred[i] = best;
    }
    free(sums);
}

/* the class trained towards output 0 for example i in this epoch */
int32_t otm_neg_class(const otm_config *cfg, uint32_t epoch, int64_t i, int32_t y)
{
    uint32_t r[4];
    draw(cfg, OTM_NEGCLASS, 0, 0, (uint64_t)i, epoch, r);
    int32_t d = (int32_t)(((uint64_t)r[0] * (uint64_t)(cfg->m - 1)) >> 32);
    return d + (d >= y ? 1 : 0);
}

/* Algorithm 1, clip / error / stochastic gate.  target = 1 if this class is
 * being trained towards output 1 for the example.  Returns 1 if feedback fires. */
int otm_gate(const otm_config *cfg, int32_t g, int64_t i, uint32_t epoch, int32_t v, int target)
{
    int32_t vc = clip(v, -cfg->T, cfg->T);
    int32_t e = target ? cfg->T - vc : cfg->T + vc;
    uint32_t r[4];
    draw(cfg, OTM_GATE, 0, (uint32_t)g, (uint64_t)i, epoch, r);
    return (uint64_t)r[0] * (uint64_t)(2 * (int64_t)cfg->T) < ((uint64_t)e << 32);
}

/* Regression mode: which feedback, if any, clause g gives itself on example i whose
 * recorded vote sum is v and whose target is y.  0 none, 1 Type I, 2 Type II. */
int otm_gate_regression(const otm_config *cfg, int32_t g, int64_t i, uint32_t epoch, int32_t v, int32_t y)
{
    int32_t vc = clip(v, 0, cfg->T);
    int32_t e = vc < y ? y - vc : vc - y;
    uint32_t r[4];
    draw(cfg, OTM_GATE, 0, (uint32_t)g, (uint64_t)i, epoch, r);
    if (!((uint64_t)r[0] * (uint64_t)cfg->T < ((uint64_t)e << 32)))
        return 0;
    return vc < y ? 1 : 2;
}

/* threshold of the 16-bit uniform: P(u < thr) = 1/s */
int32_t otm_threshold(const otm_config *cfg)
{
    double t = 65536.0 / cfg->s + 0.5;
    int32_t thr = (int32_t)t; /* floor, t > 0 */
    if (thr < 0) thr = 0;
    if (thr > 65536) thr = 65536;
    return thr;
}

/* Type I feedback (Table 1) to the TA team st[2o] of clause g, given the
 * literal values and the clause output Cout computed before the update. */
void otm_type1(const otm_config *cfg, int32_t *st, const uint8_t *lit, int Cout,
               int32_t g, int64_t i, uint32_t epoch)
{
    int32_t thr = otm_threshold(cfg);
    int cached_lw = -1;
    uint32_t R[16];
    for (int k = 0; k < 2 * cfg->o; ++k) {
        int lw, j;
        slot_of(cfg, k, &lw, &j);
        if (lw != cached_lw) {
            for (int t = 0; t < 4; ++t)
                draw(cfg, OTM_TYPE1, 4u * (uint32_t)lw + (uint32_t)t, (uint32_t)g,
                     (uint64_t)i, epoch, R + 4 * t);
            cached_lw = lw;
        }
        int32_t u = 0;
        for (int b = 0; b < 16; ++b)
            u |= (int32_t)((R[b] >> j) & 1u) << b;
        if (Cout == 1 && lit[k] == 1) {
            /* strong: reward Include / penalise Exclude, probability (s-1)/s,
             * or 1 when true positives are boosted */
            if ((cfg->boost || u >= thr) && st[k] < 2 * cfg->N)
                st[k] += 1;
        } else {
            /* weak: penalise Include / reward Exclude, probability 1/s */
            if (u < thr && st[k] > 1)
                st[k] -= 1;
        }
    }
}

/* Type II feedback (Table 2): penalise Exclude with probability 1 where the
 * clause is 1 and the literal is 0. */
void otm_type2(const otm_config *cfg, int32_t *st, const uint8_t *lit, int Cout)
{
    if (Cout != 1)
        return;
    for (int k = 0; k < 2 * cfg->o; ++k)
        if (lit[k] == 0 && st[k] <= cfg->N)
            st[k] += 1;
}

/* One visit of clause g to example i (body of the loop of Algorithm 1).
 * v_gate is the tally value the gate looks at.  tally_ic points at the live
 * tally of (i, class of g); ostar_gi at the stored previous output.  Either
 * may be NULL (synchronous training keeps neither). Returns 1 if feedback fired. */
static int visit(const otm_config *cfg, int32_t *state, int32_t g, const uint8_t *lit,
                 int64_t i, uint32_t epoch, int role /*0 none,1 target,2 negative,3 regression*/,
                 int32_t y_i, int32_t v_gate, int32_t *tally_ic, uint8_t *ostar_gi)
{
    int L = 2 * cfg->o;
    int32_t *st = state + (size_t)g * L;
    int fired = 0;
    if (role == 3) {
        int kind = otm_gate_regression(cfg, g, i, epoch, v_gate, y_i);
        if (kind != 0) {
            int Cout = clause_output(cfg, st, lit);
            if (kind == 2)
                otm_type2(cfg, st, lit, Cout);
            else
                otm_type1(cfg, st, lit, Cout, g, i, epoch);
            fired = 1;
        }
    } else if (role != 0) {
        int target = (role == 1);
        int p = (polarity_sign(cfg, g) > 0);
        if (otm_gate(cfg, g, i, epoch, v_gate, target)) {
            int Cout = clause_output(cfg, st, lit);
            if (target ^ p)
                otm_type2(cfg, st, lit, Cout);
            else
                otm_type1(cfg, st, lit, Cout, g, i, epoch);
            fired = 1;
        }
    }
    if (ostar_gi) {
        int o_new = clause_output(cfg, st, lit);
        if (o_new != *ostar_gi) {
            *tally_ic += polarity_sign(cfg, g) * (o_new - (int)*ostar_gi);
            *ostar_gi = (uint8_t)o_new;
        }
    }
    return fired;
}

static int role_of(const otm_config *cfg, int c, int32_t y, uint32_t epoch, int64_t i)
{
    if (cfg->regression) return 3;
    if (c == y) return 1;
    if (c == otm_neg_class(cfg, epoch, i, y)) return 2;
    return 0;
}

/* Pre-calculation of the tallies (Section 3.1): ostar[g][i] = C_g(X_i),
 * tally[i][c] = unclamped Eq. 3. */
void otm_sync_tallies(const otm_config *cfg, const int32_t *state, const uint8_t *X,
                      int64_t q, int32_t *tally, uint8_t *ostar)
{
    int L = 2 * cfg->o, C = cfg->m * cfg->n;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    for (int64_t i = 0; i < q; ++i) {
        literals(cfg, X + i * cfg->o, lit);
        for (int c = 0; c < cfg->m; ++c)
            tally[i * cfg->m + c] = 0;
        for (int g = 0; g < C; ++g) {
            int out = clause_output(cfg, state + (size_t)g * L, lit);
            ostar[(size_t)g * q + i] = (uint8_t)out;
            tally[i * cfg->m + g / cfg->n] += polarity_sign(cfg, g) * out;
        }
    }
    free(lit);
}

/* Algorithm 1 under a frozen tally snapshot vhat[q][m]: every clause visits
 * examples i0 .. i0+cnt-1 in order and gates on vhat; refreshes go to the live
 * tally[q][m] and ostar[C][q].  Each clause's result is independent of the
 * others, so any parallel schedule must reproduce it exactly.
 * fired_count (may be NULL) receives the number of fired gates. */
void otm_feedback_step(const otm_config *cfg, int32_t *state, const uint8_t *X,
                       const int32_t *y, int64_t q, const int32_t *vhat, int32_t *tally,
                       uint8_t *ostar, uint32_t epoch, int64_t i0, int64_t cnt,
                       int64_t *fired_count)
{
    int L = 2 * cfg->o, C = cfg->m * cfg->n;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    int64_t fired = 0;
    for (int g = 0; g < C; ++g) {
        int c = g / cfg->n;
        for (int64_t i = i0; i < i0 + cnt && i < q; ++i) {
            literals(cfg, X + i * cfg->o, lit);
            int role = role_of(cfg, c, y[i], epoch, i);
            fired += visit(cfg, state, g, lit, i, epoch, role, y[i], vhat[i * cfg->m + c],
                           &tally[i * cfg->m + c], &ostar[(size_t)g * q + i]);
        }
    }
    if (fired_count) *fired_count = fired;
    free(lit);
}

/* The same frozen-snapshot pass for a chosen subset of clauses only (each
 * clause's trajectory is independent of the others under a frozen snapshot, so
 * a few clauses of a machine too large to run in full can be followed alone).
 * state is the full [C][2o] array; ostar_sub is [n_ids][q], row r belonging to
 * clause ids[r]; the live tally is not kept. */
void otm_feedback_step_subset(const otm_config *cfg, int32_t *state, const uint8_t *X,
                              const int32_t *y, int64_t q, const int32_t *vhat,
                              uint8_t *ostar_sub, uint32_t epoch, int64_t i0, int64_t cnt,
                              const int32_t *ids, int32_t n_ids, int64_t *fired_count)
{
    int L = 2 * cfg->o;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    int64_t fired = 0;
    for (int r = 0; r < n_ids; ++r) {
        int g = ids[r];
        int c = g / cfg->n;
        for (int64_t i = i0; i < i0 + cnt && i < q; ++i) {
            int32_t scratch_tally = 0;
            literals(cfg, X + i * cfg->o, lit);
            int role = role_of(cfg, c, y[i], epoch, i);
            fired += visit(cfg, state, g, lit, i, epoch, role, y[i], vhat[i * cfg->m + c],
                           &scratch_tally, &ostar_sub[(size_t)r * q + i]);
        }
    }
    if (fired_count) *fired_count = fired;
    free(lit);
}

/* out[r][i] = C_{ids[r]}(X_i) for a subset of clauses */
void otm_clause_outputs_subset(const otm_config *cfg, const int32_t *state, const uint8_t *X,
                               int64_t q, const int32_t *ids, int32_t n_ids, uint8_t *out)
{
    int L = 2 * cfg->o;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    for (int64_t i = 0; i < q; ++i) {
        literals(cfg, X + i * cfg->o, lit);
        for (int r = 0; r < n_ids; ++r)
            out[(size_t)r * q + i] = (uint8_t)clause_output(cfg, state + (size_t)ids[r] * L, lit);
    }
    free(lit);
}

/* Sequential execution of Algorithm 1 with live tallies (one legal schedule of
 * the asynchronous method): examples outermost if example_major, else clauses
 * outermost. */
void otm_async_epoch(const otm_config *cfg, int32_t *state, const uint8_t *X,
                     const int32_t *y, int64_t q, int32_t *tally, uint8_t *ostar,
                     uint32_t epoch, int example_major)
{
    int L = 2 * cfg->o, C = cfg->m * cfg->n;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    if (example_major) {
        for (int64_t i = 0; i < q; ++i) {
            literals(cfg, X + i * cfg->o, lit);
            for (int g = 0; g < C; ++g) {
                int c = g / cfg->n;
                int role = role_of(cfg, c, y[i], epoch, i);
                visit(cfg, state, g, lit, i, epoch, role, y[i], tally[i * cfg->m + c],
                      &tally[i * cfg->m + c], &ostar[(size_t)g * q + i]);
            }
        }
    } else {
        for (int g = 0; g < C; ++g) {
            int c = g / cfg->n;
            for (int64_t i = 0; i < q; ++i) {
                literals(cfg, X + i * cfg->o, lit);
                int role = role_of(cfg, c, y[i], epoch, i);
                visit(cfg, state, g, lit, i, epoch, role, y[i], tally[i * cfg->m + c],
                      &tally[i * cfg->m + c], &ostar[(size_t)g * q + i]);
            }
        }
    }
    free(lit);
}

/* The same sequential execution restricted to the batch of examples i0 .. i0+cnt-1
 * (Algorithm 1's batch size b = cnt): with clauses outermost, every clause in turn
 * walks the whole batch before the next clause starts. */
void otm_async_range(const otm_config *cfg, int32_t *state, const uint8_t *X,
                     const int32_t *y, int64_t q, int32_t *tally, uint8_t *ostar,
                     uint32_t epoch, int64_t i0, int64_t cnt, int example_major)
{
    int L = 2 * cfg->o, C = cfg->m * cfg->n;
    int64_t i1 = i0 + cnt < q ? i0 + cnt : q;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    if (example_major) {
        for (int64_t i = i0; i < i1; ++i) {
            literals(cfg, X + i * cfg->o, lit);
            for (int g = 0; g < C; ++g) {
                int c = g / cfg->n;
                int role = role_of(cfg, c, y[i], epoch, i);
                visit(cfg, state, g, lit, i, epoch, role, y[i], tally[i * cfg->m + c],
                      &tally[i * cfg->m + c], &ostar[(size_t)g * q + i]);
            }
        }
    } else {
        for (int g = 0; g < C; ++g) {
            int c = g / cfg->n;
            for (int64_t i = i0; i < i1; ++i) {
                literals(cfg, X + i * cfg->o, lit);
                int role = role_of(cfg, c, y[i], epoch, i);
                visit(cfg, state, g, lit, i, epoch, role, y[i], tally[i * cfg->m + c],
                      &tally[i * cfg->m + c], &ostar[(size_t)g * q + i]);
            }
        }
    }
    free(lit);
}

/* Standard (synchronous) TM training, Section 3.1 first paragraph: examples
 * one by one; the exact vote sum of Eq. 3 is computed from the current
 * clauses before any of them receives feedback. */
void otm_sync_epoch(const otm_config *cfg, int32_t *state, const uint8_t *X,
                    const int32_t *y, int64_t q, uint32_t epoch)
{
    int L = 2 * cfg->o;
    uint8_t *lit = (uint8_t *)malloc((size_t)L);
    for (int64_t i = 0; i < q; ++i) {
        literals(cfg, X + i * cfg->o, lit);
        if (cfg->regression) {
            int32_t v0 = vote_sum(cfg, state, lit, 0);
            for (int j = 0; j < cfg->n; ++j)
                visit(cfg, state, j, lit, i, epoch, 3, y[i], v0, NULL, NULL);
            continue;
        }
        int cls[2];
        cls[0] = y[i];
        cls[1] = otm_neg_class(cfg, epoch, i, y[i]);
        int32_t v[2];
        v[0] = vote_sum(cfg, state, lit, cls[0]);
        v[1] = vote_sum(cfg, state, lit, cls[1]);
        for (int r = 0; r < 2; ++r)
            for (int j = 0; j < cfg->n; ++j)
                visit(cfg, state, cls[r] * cfg->n + j, lit, i, epoch, r + 1, y[i], v[r], NULL, NULL);
    }
    free(lit);
}
