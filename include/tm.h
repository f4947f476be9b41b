/*
 * tm.h - C boundary of the asynchronous Tsetlin machine library for gfx950.
 *
 * The library implements the data-parallel hot path of "Massively Parallel and
 * Asynchronous Tsetlin Machine Architecture Supporting Almost Constant-Time
 * Scaling": clause evaluation over bit-packed literals (Eq. 1), signed voting
 * (Eq. 2 / Eq. 3), per-example voting tallies (Section 3.1) and the
 * decentralised clause update of Algorithm 1 with Type I / Type II feedback
 * (Tables 1 and 2).
 *
 * Symbols follow the paper: o Boolean features, 2o literals, m classes,
 * n clauses per class, C = m*n clauses, 2N states per Tsetlin automaton (TA),
 * voting margin T, specificity s, q examples.  Wf = ceil(o/32).
 *
 * Conventions shared by all entry points
 *   - Every pointer marked "device" is device memory of the GPU named in
 *     tm_config.device and is owned by the caller.  The library never
 *     allocates or frees device memory; it keeps raw pointers between
 *     tm_create / tm_bind_train and tm_destroy and the caller must keep the
 *     buffers alive for that time.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Unless stated otherwise a call only enqueues work on that stream and
 *     returns; results are ready when the stream reaches that point.
 *   - Features are bit-packed by the caller: X is uint32 [q][Wf], feature k of
 *     example i is bit (k & 31) of X[i*Wf + (k >> 5)]; padding bits are 0.
 *   - Clause g = c*n + j belongs to class c and has positive polarity iff j is
 *     odd (Section 2.1).  Literal k < o is x_k, literal o+k is NOT x_k.
 *   - Every function returns TM_OK or a negative error code; nothing is
 *     thrown, printed or aborted.  A handle must not be used from two host
 *     threads at once.
 */
#ifndef TM_H_
#define TM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TM_OK = 0,
    TM_EINVAL = -1, /* bad argument or configuration                        */
    TM_ESTATE = -2, /* call needs bound training data (tm_bind_train) first */
    TM_EHIP = -3,   /* a HIP call failed; see tm_last_hip_error             */
    TM_ELIMIT = -4  /* size outside what the kernels support                */
};

/* Largest supported number of features (2*ceil(o/32) literal words must fit
 * the 64 lanes x 20 register slots of one wavefront). */
#define TM_MAX_FEATURES 20480

typedef struct tm_handle tm_handle; /* opaque */

/* Problem statement of the paper (Section 2.1, Section 2.2, Algorithm 1). */
typedef struct {
    int32_t n_classes;         /* m >= 2 (regression mode: exactly 1)                 */
    int32_t clauses_per_class; /* n, even and >= 2: half positive, half negative      */
    int32_t n_features;        /* o, 1 .. TM_MAX_FEATURES                             */
    int32_t states_per_action; /* N, 1 .. 128; a TA has 2N states, Include iff > N    */
    int32_t T;                 /* voting margin, >= 1                                 */
    double s;                  /* specificity, >= 1.0                                 */
    uint64_t seed;             /* key of the counter-based random generator           */
    int32_t device;            /* HIP device ordinal                                  */
    int32_t boost_true_positive; /* 0/1: strong Type I probability (s-1)/s replaced by 1
                                    (footnote of Section 2.2)                          */
    int32_t regression;        /* 0/1: regression mode, see below                     */
} tm_config;

/* Regression mode (the regression Tsetlin machine measured in Section 4.1; the paper
 * does not restate its update rule, the library follows the regression TM publication
 * it cites).  One bank of n clauses (n_classes = 1) that all vote +1; the output is
 * the vote sum clipped to [0, T]; y holds integer targets 0..T (the caller scales its
 * continuous target to that range).  In Algorithm 1 the error becomes
 * e = |y_i - clip(v_i, 0, T)| and a clause gives itself feedback with probability
 * e/T: Type I where the vote sum lies below the target, Type II where it lies above.
 * Evaluation, Type I / II feedback, tallies and their refresh are those of
 * classification.  tm_class_sums* return the clipped vote sum [q][1]; tm_predict*
 * return the same value in pred. */

/* Size in bytes of the model state buffer for a configuration: one counter of
 * 2N states per Tsetlin automaton, 2o automata per clause (Section 2.2: a TA
 * "team" per clause, states 1..2N), stored bit-sliced (one byte per
 * automaton), plus the include masks the clauses are evaluated from (Eq. 1).
 * Host-only computation.  TM_EINVAL / TM_ELIMIT on a bad configuration. */
int tm_state_bytes(const tm_config *cfg, size_t *out);

/* Size in bytes of the training workspace for q examples.  Section 3.1 gives
 * every training example a voting tally and every clause one bit per example
 * (its previous output); the workspace holds those (int32 [m][q], 1 bit per
 * (clause, example)) plus what the kernels derive from X and the clauses: the
 * transposed copy of X, the literals as bit rows over the examples, literal
 * lists of the clauses, per-class gate lists, per-clause bookkeeping, counters.
 * Host-only computation.  The library cannot check the size of the buffer it
 * is given in tm_bind_train: passing fewer bytes than this is undefined. */
int tm_train_ws_bytes(const tm_config *cfg, int64_t q, size_t *out);

/* Creates a machine whose state lives in state_buf (device, at least
 * tm_state_bytes, 256-byte aligned).  Every TA starts at state N or N+1 with
 * probability 1/2 (the paper does not fix the start).  Enqueues the
 * initialisation on `stream`. */
int tm_create(const tm_config *cfg, void *state_buf, void *stream, tm_handle **out);

/* Frees the host-side handle only (and the timing events it created).  Device
 * buffers - the TA states of Section 2.2, the tallies of Section 3.1 - stay
 * with the caller and keep their contents. */
int tm_destroy(tm_handle *h);

/* Binds a training set: X device uint32 [q][Wf], y device int32 [q] with
 * labels 0..m-1 (regression mode: targets 0..T), ws device workspace of tm_train_ws_bytes(cfg, q) bytes
 * (256-byte aligned).  Builds the transposed copy of X and runs the tally
 * pre-calculation of Section 3.1 (every clause on every example; fills the
 * previous-output bits and the tallies).  Synchronises the stream once to
 * report labels out of range as TM_EINVAL.  q >= 1. */
int tm_bind_train(tm_handle *h, const uint32_t *X, const int32_t *y, int64_t q, void *ws,
                  void *stream);

/* Limits of the random counter (seed, epoch, example, clause, literal block):
 * epoch < 2^24 (tm_fit_epoch, tm_fit_batch and tm_feedback_step return TM_ELIMIT
 * once the epoch counter reaches it, tm_set_epoch refuses it with TM_EINVAL) and
 * example index < 2^30 (checked in tm_bind_train). */

/* One pass of Algorithm 1 with batch size b = q over the bound examples: every
 * clause visits examples 0..q-1 in order, gates on the (possibly outdated)
 * tally, applies Type I or Type II feedback, re-evaluates, and refreshes tally
 * and previous-output bit.  Multi-class: class y_i is trained towards 1 and
 * one other class, drawn per (epoch, example), towards 0.  The pass is cut into
 * launches (tm_train_chunk); an example whose error e is 0 under the tally as
 * it stands at the start of its launch (gate probability 0) is not visited for
 * feedback in that launch, all others are gated on the tally read at the visit.
 * Advances the handle's epoch counter (part of the random counter) by one. */
int tm_fit_epoch(tm_handle *h, void *stream);

/* Algorithm 1 on one batch: the examples i0 .. i0+cnt-1 of the bound set (the
 * paper's batch size b = cnt), gated on the live tallies like tm_fit_epoch.
 * Uses the current epoch counter without advancing it (tm_set_epoch), so that an
 * epoch can be walked in batches with tm_sync_tallies or other work in between:
 * how often the tallies are recomputed is the caller's choice. */
int tm_fit_batch(tm_handle *h, int64_t i0, int64_t cnt, void *stream);

/* Eq. 3 per class, clamped to [-T, T]: sums device int32 [q][m].
 * X need not be the bound training set.  q may be 0. */
int tm_class_sums(tm_handle *h, const uint32_t *X, int64_t q, int32_t *sums, void *stream);

/* Classification: pred device int32 [q] = lowest class index attaining the
 * largest clamped class sum (two classes in one bank, Eq. 2, generalised to
 * one bank per class).  `sums_scratch` is device int32 [q][m] scratch. */
int tm_predict(tm_handle *h, const uint32_t *X, int64_t q, int32_t *pred, int32_t *sums_scratch,
               void *stream);

/* Size in bytes of the workspace of tm_class_sums_ws / tm_predict_ws for q
 * examples (the literals as bit rows over the examples, and the list of
 * included literals of every clause).  Host-only computation. */
int tm_infer_ws_bytes(const tm_config *cfg, int64_t q, size_t *out);

/* tm_class_sums / tm_predict with a workspace (device, tm_infer_ws_bytes, 256-
 * byte aligned, contents need not be kept between calls).  Same results.  Eq. 1
 * is a conjunction over the INCLUDED literals only, so each clause is evaluated
 * from the list of its included literals instead of from its 2o mask bits; on a
 * trained machine that is a few dozen literals per clause (the lists hold
 * 128 to 1,024 literals depending on o; longer clauses are finished from
 * their masks).  TM_ELIMIT when
 * (2o + 1) * 64 * ceil(q / 2048) * 4 bytes reach 4 GiB: split q. */
int tm_class_sums_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *sums, void *ws, void *stream);
int tm_predict_ws(tm_handle *h, const uint32_t *X, int64_t q, int32_t *pred, int32_t *sums_scratch, void *ws,
                  void *stream);

/* tm_predict_ws for callers that cannot allocate or bring a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the workspace and the sums scratch live in a static device array
 * of TM_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until
 * the process ends.  Same result as tm_predict_ws.  Calls no hipMalloc / hipFree
 * and creates no events or streams; enqueues kernels on `stream` only.
 * TM_ELIMIT when tm_infer_ws_bytes(cfg, q) rounded up to 256 plus q*m*4 bytes
 * exceed TM_STATIC_SCRATCH_BYTES (split q; the literal lists of all clauses
 * alone take C * (128..1024) * 4 bytes, so large machines do not fit at all).
 * All calls on one GPU share that GPU's array: two calls whose kernels can run
 * at the same time (different streams, different handles, different host
 * threads) race on it; calls on one stream are safe.  Nothing needs to be kept
 * in the array between calls. */
#define TM_STATIC_SCRATCH_BYTES (32u << 20)
int tm_predict_static(tm_handle *h, const uint32_t *X, int64_t q, int32_t *pred, void *stream);

/* ---- hooks used by tests, checkpoints and measurements ---------------- */

/* TA states as bytes (Section 2.2: every literal of every clause has an
 * automaton with states 1..2N; Include iff state > N): device uint8 [C][2o],
 * value = state - 1 (0 .. 2N-1), literal k < o is x_k, literal o+k is NOT x_k. */
int tm_get_ta_state(tm_handle *h, uint8_t *out, void *stream);
/* Inverse of tm_get_ta_state; values above 2N-1 are clamped.  Also rebuilds
 * the include masks.  Tallies of bound data become outdated (call
 * tm_sync_tallies). */
int tm_set_ta_state(tm_handle *h, const uint8_t *in, void *stream);

/* Clause outputs (Eq. 1) as a bit matrix: bits device uint32 [C][ceil(q/32)],
 * example i of clause g is bit (i & 31) of bits[g*ceil(q/32) + (i >> 5)];
 * bits beyond q are 0. */
int tm_clause_outputs(tm_handle *h, const uint32_t *X, int64_t q, uint32_t *bits, void *stream);

/* Re-runs the tally pre-calculation (Section 3.1) on the bound data. */
int tm_sync_tallies(tm_handle *h, void *stream);

/* Copies the live voting tallies of Section 3.1 (one per training example and
 * class, the recorded vote sum v_i that Algorithm 1 clips and gates on;
 * unclamped, possibly outdated) to out, device int32 [q][m]. */
int tm_get_tallies(tm_handle *h, int32_t *out, void *stream);

/* Copies the stored previous clause outputs o* of Algorithm 1 to bits, same
 * layout as tm_clause_outputs for the bound q. */
int tm_get_prev_outputs(tm_handle *h, uint32_t *bits, void *stream);

/* Algorithm 1 restricted to examples i0 .. i0+cnt-1 with the gate reading a
 * caller-supplied snapshot (device int32 [q][m]) instead of the live tallies;
 * refreshes still go to the live tallies.  Uses the current epoch counter
 * without advancing it.  Same kernel as tm_fit_epoch; results do not depend
 * on scheduling. */
int tm_feedback_step(tm_handle *h, const int32_t *tally_snapshot, int64_t i0, int64_t cnt,
                     void *stream);

/* tm_fit_epoch cuts the pass of Algorithm 1 over the bound examples into consecutive
 * ranges of this many examples, one launch of the training kernel each, so that a
 * range's slice of the transposed features stays resident in L2 (measurement aid;
 * the cut is also where Section 3.1's recorded tallies are re-read for the gate lists). */
int tm_train_chunk(tm_handle *h, int64_t *examples_per_launch);

/* Schedule knob: every launch of the training kernel is split into `groups`
 * consecutive sub-launches over clause ranges of equal size (1 <= groups <= C;
 * default 1: all clauses at once).  The clauses of a sub-launch gate on the
 * tallies as the sub-launches before it left them, which bounds how outdated a
 * tally can be when thousands of clauses run in step; every such order is a
 * legal schedule of Algorithm 1, and results under a frozen snapshot
 * (tm_feedback_step) do not depend on it. */
int tm_set_clause_groups(tm_handle *h, int32_t groups);

/* How the literal-list evaluation of Eq. 1 / Eq. 3 (tm_class_sums_ws, tm_predict_ws, the tally
 * pre-calculation of Section 3.1) splits the n clauses of a class for q examples: into
 * `shares` workgroups of `clauses_per_share` clauses each (host-only; measurement and test
 * aid).  A wavefront counts the votes of an eighth of a share in 8 bit planes, so
 * clauses_per_share <= 2032 always. */
int tm_eval_shares(const tm_config *cfg, int64_t q, int32_t *shares, int32_t *clauses_per_share);

/* Epoch counter: part of the counter of the random generator behind Algorithm 1's rand()
 * (gate, Type I, negative class), used by the next tm_fit_epoch / tm_fit_batch /
 * tm_feedback_step; tm_fit_epoch advances it by one. */
int tm_set_epoch(tm_handle *h, uint32_t epoch);
int tm_get_epoch(tm_handle *h, uint32_t *epoch);

/* Device-side event counters of the training kernel since the last call of
 * this function (or since tm_bind_train): out is HOST uint64 [10]:
 * [0] visited (clause, example) pairs (every wavefront of the training kernel adds the
 * number of examples of its launch that it walked for its clause), [1] fired gates, [2] Type I feedbacks,
 * [3] tally changes, [4] pairs whose class was trained for the example (gate
 * candidates), [5] Type II feedbacks given to a clause with output 1,
 * [6] blocks of 64 examples that a clause had to evaluate (blocks whose stored
 * outputs are known to be current and in which no gate fires are skipped),
 * [7] gate candidates whose error e was positive both at the start of the
 * launch and at the visit (a random draw was needed),
 * [8] those of the blocks of [6] that were evaluated 32 at a time through the
 * clause's literal list (outdated blocks of a sparse clause in which no gate
 * fired) rather than one by one from its include masks,
 * [9] (clause, launch) pairs for which the clause's automata were fetched and written
 * back (a clause that gets no feedback in a launch only reads its include masks).
 * Synchronises the stream. */
int tm_read_counters(tm_handle *h, uint64_t *out, void *stream);

/* Kernel timing (measurement aid).  `kinds` is a bit mask: while bit 0 is set
 * every launch of the training kernel is bracketed by two events on its stream,
 * with bit 1 every launch of the literal-list evaluation kernel in the tally
 * pre-calculation, with bit 2 every such launch in tm_class_sums_ws /
 * tm_predict_ws; 0 switches timing off, 7 times all three (an event between
 * two kernels costs the stream a few microseconds, so a caller that times a
 * whole step asks only for the kernel it wants).  tm_read_kernel_timing waits
 * for the recorded events and returns, per kind, the summed kernel time in
 * ms[3] and the number of launches in launches[3] (both HOST arrays) since the
 * last read or change of the mask, and forgets them.  Changing the mask forgets
 * what was recorded.  TM_EINVAL for a mask outside 0..7. */
int tm_kernel_timing(tm_handle *h, int kinds);
int tm_read_kernel_timing(tm_handle *h, double *ms, int64_t *launches);

/* Text for an error code; hipError_t of the last failed HIP call on a handle. */
const char *tm_strerror(int code);
int tm_last_hip_error(tm_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* TM_H_ */
