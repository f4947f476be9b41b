"""Pins of the oracle's training loops against an independent restatement.

The classification loops of the oracle (standard synchronous training, sequential
Algorithm 1 in both loop orders and batch by batch, Algorithm 1 under a frozen tally
snapshot) are compared, state by state, with the same procedures written out here in pure
Python on sets of literals, following Section 2.2 (feedback rules), Section 3.1 (standard
training, tallies) and Algorithm 1.  From the oracle only the two feedback tables are taken
(Type I and Type II on one clause, pinned cell by cell against Tables 1 and 2 elsewhere);
clause evaluation, polarity, vote sums, the negative class, the gate, the loop structure and
the tally refresh are restated.  The random draws of the gate, the negative class and the
initial states are rebuilt here from raw Philox words and the written counter layout

    counter = (blk | stream << 28, clause g, example i, epoch),  key = seed,
    streams: 0 initial states, 1 gate, 2 Type I, 3 negative class,

and compared with the oracle draw by draw.  Each restated loop is also run with a planted
mistake (vote sum not recomputed per example, gate counter with clause and example swapped,
refresh left out, stale output fed to the feedback) to show that the comparison would catch it.
"""
import numpy as np
import pytest

from oracle import tm_oracle as O


def key_of(seed):
    return [seed & 0xffffffff, seed >> 32]


def word0(stream, blk, g, i, epoch, seed):
    return O.philox([blk | (stream << 28), g, i & 0xffffffff, epoch | ((i >> 32) << 24)], key_of(seed))[0]


# ---- restated pieces --------------------------------------------------------

def py_gate(t, g, i, epoch, v, target, swap=False):
    """Algorithm 1, lines 3-5: clip, error, fire with probability e / 2T (never at e = 0)."""
    vc = max(-t.T, min(t.T, int(v)))
    e = t.T - vc if target else t.T + vc
    r = word0(O.GATE, 0, i, g, epoch, t.seed) if swap else word0(O.GATE, 0, g, i, epoch, t.seed)
    return r * (2 * t.T) < (e << 32)


def py_neg_class(t, epoch, i, y):
    """The class trained towards 0: uniform over the m - 1 classes other than y."""
    d = (word0(O.NEGCLASS, 0, 0, i, epoch, t.seed) * (t.m - 1)) >> 32
    return d + (1 if d >= y else 0)


def true_literals(x):
    o = len(x)
    return {k for k in range(o) if x[k]} | {o + k for k in range(o) if not x[k]}


def included(t, st):
    return {k for k in range(2 * t.o) if st[k] > t.N}


def out_of(t, st, true_lits):
    """Eq. 1: the conjunction of the included literals (1 for the empty clause)."""
    return 1 if included(t, st) <= true_lits else 0


def sign_of(t, g):
    return 1 if (g % t.n) % 2 == 1 else -1


def vote_sum(t, state, true_lits, c):
    """Eq. 3 for the bank of class c."""
    return sum(sign_of(t, c * t.n + j) * out_of(t, state[c * t.n + j], true_lits) for j in range(t.n))


def give_feedback(t, st, x, g, i, epoch, target, stale_output=None):
    """Algorithm 1, lines 6-10: Type II if y xor polarity, else Type I; both see the clause's
    output on the state before the update."""
    lit = np.concatenate([x, 1 - x]).astype(np.uint8)
    Cout = out_of(t, st, true_literals(x)) if stale_output is None else stale_output
    positive = sign_of(t, g) > 0
    if bool(target) != positive:
        t.type2(st, lit, Cout)
    else:
        t.type1(st, lit, Cout, g, i, epoch)


# ---- restated loops ---------------------------------------------------------

def py_sync_epoch(t, state, X, y, epoch, recompute=True, swap=False):
    """Standard training (Section 3.1, first paragraph): one example at a time; the vote sums of
    the two trained classes are computed from the current clauses, then each of their clauses
    is gated on that sum."""
    first = None
    for i in range(len(y)):
        tl = true_literals(X[i])
        classes = [int(y[i]), py_neg_class(t, epoch, i, int(y[i]))]
        v = [vote_sum(t, state, tl, c) for c in classes]
        if not recompute:       # planted mistake: the sums of the first example are kept
            first = first or v
            v = first
        for r, c in enumerate(classes):
            for j in range(t.n):
                g = c * t.n + j
                if py_gate(t, g, i, epoch, v[r], r == 0, swap):
                    give_feedback(t, state[g], X[i], g, i, epoch, r == 0)


def py_visit(t, state, X, y, g, i, epoch, v_gate, tally, ostar, refresh=True, stale=False):
    """Body of Algorithm 1's loop for clause g and example i."""
    c = g // t.n
    yi = int(y[i])
    if c == yi or c == py_neg_class(t, epoch, i, yi):
        if py_gate(t, g, i, epoch, v_gate, c == yi):
            give_feedback(t, state[g], X[i], g, i, epoch, c == yi, int(ostar[g, i]) if stale else None)
    if refresh:     # lines 12-17, for every visited pair
        o_new = out_of(t, state[g], true_literals(X[i]))
        if o_new != ostar[g, i]:
            tally[i, c] += sign_of(t, g) * (o_new - int(ostar[g, i]))
            ostar[g, i] = o_new


def py_algorithm1(t, state, X, y, epoch, tally, ostar, i0, cnt, example_major, vhat=None, **mistake):
    """Algorithm 1 on the batch i0 .. i0+cnt-1, executed sequentially: clauses outermost or
    examples outermost; gating on the live tallies, or on the snapshot vhat if given."""
    rng_i = range(i0, min(i0 + cnt, len(y)))
    pairs = [(g, i) for i in rng_i for g in range(t.C)] if example_major else \
            [(g, i) for g in range(t.C) for i in rng_i]
    for g, i in pairs:
        c = g // t.n
        v = tally[i, c] if vhat is None else vhat[i, c]
        py_visit(t, state, X, y, g, i, epoch, v, tally, ostar, **mistake)


def py_tallies(t, state, X):
    q = len(X)
    ostar = np.zeros((t.C, q), dtype=np.uint8)
    tally = np.zeros((q, t.m), dtype=np.int32)
    for i in range(q):
        tl = true_literals(X[i])
        for g in range(t.C):
            ostar[g, i] = out_of(t, state[g], tl)
            tally[i, g // t.n] += sign_of(t, g) * int(ostar[g, i])
    return tally, ostar


# ---- the problem ------------------------------------------------------------

M, NCL, OF, NST, TT, SS = 3, 4, 6, 3, 3, 2.5      # 12 clauses, few states: clauses change all the time
Q, EPOCHS = 40, 3


def problem(seed=5):
    rng = np.random.default_rng(seed)
    X = rng.integers(0, 2, size=(Q, OF)).astype(np.uint8)
    y = ((X[:, 0] ^ X[:, 1]) + 2 * (X[:, 2] & X[:, 3])).clip(0, M - 1).astype(np.int32)
    return X, y


def fresh(seed=21):
    return O.Oracle(M, NCL, OF, NST, TT, SS, seed)


# ---- draws rebuilt from Philox words -----------------------------------------

def test_gate_draw_is_word_0_of_the_gate_stream_keyed_by_clause_then_example():
    t = O.Oracle(2, 6, 5, 8, 7, 3.0, (9 << 32) | 12345)
    rng = np.random.default_rng(1)
    differs_when_swapped = 0
    for _ in range(3000):
        g, i, ep = int(rng.integers(0, 12)), int(rng.integers(0, 5000)), int(rng.integers(0, 300))
        v, target = int(rng.integers(-10, 11)), int(rng.integers(0, 2))
        assert bool(t.gate(g, i, ep, v, target)) == py_gate(t, g, i, ep, v, target)
        differs_when_swapped += bool(t.gate(g, i, ep, v, target)) != py_gate(t, g, i, ep, v, target, swap=True)
    assert differs_when_swapped > 300      # the check tells (g, i) from (i, g)


def test_negative_class_draw_is_word_0_of_its_stream_with_clause_0():
    t = O.Oracle(7, 2, 5, 8, 7, 3.0, (3 << 32) | 99)
    rng = np.random.default_rng(2)
    for _ in range(3000):
        i, ep, y = int(rng.integers(0, 100000)), int(rng.integers(0, 300)), int(rng.integers(0, 7))
        assert t.neg_class(ep, i, y) == py_neg_class(t, ep, i, y)


def test_initial_states_are_bit_j_of_word_0_of_block_4lw():
    m, n, o, N, seed = 2, 4, 37, 9, (5 << 32) | 77
    t = O.Oracle(m, n, o, N, 5, 3.0, seed)
    Wf = (o + 31) // 32
    for g in range(m * n):
        for k in range(2 * o):
            h = 1 if k >= o else 0
            f = k - h * o
            lw, j = h * Wf + f // 32, f % 32
            assert t.state[g, k] == N + ((word0(O.INIT, 4 * lw, g, 0, 0, seed) >> j) & 1), (g, k)


# ---- loops --------------------------------------------------------------------

def test_synchronous_epochs_match_the_restated_standard_training():
    X, y = problem()
    t = fresh()
    state = t.state.copy()
    for ep in range(EPOCHS):
        t.sync_epoch(X, y, ep)
        py_sync_epoch(t, state, X, y, ep)
        assert np.array_equal(t.state, state), ep
    assert not np.array_equal(state, fresh().state)      # something was learned at all


@pytest.mark.parametrize("mistake", [dict(recompute=False), dict(swap=True)])
def test_synchronous_comparison_catches_planted_mistakes(mistake):
    X, y = problem()
    t = fresh()
    state = t.state.copy()
    t.sync_epoch(X, y, 0)
    py_sync_epoch(t, state, X, y, 0, **mistake)
    assert not np.array_equal(t.state, state)


def test_pre_calculated_tallies_match_the_restatement():
    X, y = problem()
    t = fresh()
    tally, ostar = t.sync_tallies(X)
    ptally, postar = py_tallies(t, t.state, X)
    assert np.array_equal(tally, ptally) and np.array_equal(ostar, postar)


@pytest.mark.parametrize("example_major", [True, False])
def test_sequential_algorithm1_epochs_match_the_restatement(example_major):
    X, y = problem()
    t = fresh()
    tally, ostar = t.sync_tallies(X)
    state, ptally, postar = t.state.copy(), tally.copy(), ostar.copy()
    changed = 0
    for ep in range(EPOCHS):
        before = tally.copy()
        t.async_epoch(X, y, tally, ostar, ep, example_major)
        py_algorithm1(t, state, X, y, ep, ptally, postar, 0, Q, example_major)
        assert np.array_equal(t.state, state), ep
        assert np.array_equal(tally, ptally) and np.array_equal(ostar, postar), ep
        changed += int((before != tally).sum())
    assert changed > 20      # the tallies really moved, so live gating was exercised


def test_algorithm1_in_batches_matches_the_restatement():
    """Clauses outermost within each batch: the schedule of a machine whose clauses take turns
    batch by batch."""
    X, y = problem()
    t = fresh()
    tally, ostar = t.sync_tallies(X)
    state, ptally, postar = t.state.copy(), tally.copy(), ostar.copy()
    for ep in range(EPOCHS):
        for i0, cnt in [(0, 13), (13, 1), (14, 20), (34, 100)]:
            t.async_range(X, y, tally, ostar, ep, i0, cnt, False)
            py_algorithm1(t, state, X, y, ep, ptally, postar, i0, cnt, False)
            assert np.array_equal(t.state, state), (ep, i0)
            assert np.array_equal(tally, ptally) and np.array_equal(ostar, postar), (ep, i0)
    # one batch that covers everything is the epoch routine
    a, b = fresh(), fresh()
    ta, oa = a.sync_tallies(X)
    tb, ob = b.sync_tallies(X)
    for ep in range(2):
        for major in (True, False):
            a.async_epoch(X, y, ta, oa, ep, major)
            b.async_range(X, y, tb, ob, ep, 0, Q, major)
    assert np.array_equal(a.state, b.state) and np.array_equal(ta, tb) and np.array_equal(oa, ob)


def test_frozen_snapshot_passes_match_the_restatement():
    X, y = problem()
    t = fresh()
    tally, ostar = t.sync_tallies(X)
    state, ptally, postar = t.state.copy(), tally.copy(), ostar.copy()
    rng = np.random.default_rng(4)
    fired = 0
    for ep, (i0, cnt) in enumerate([(0, Q), (5, 17), (0, Q)]):
        vhat = rng.integers(-TT - 1, TT + 2, size=(Q, M)).astype(np.int32) if ep else tally.copy()
        fired += t.feedback_step(X, y, vhat, tally, ostar, ep, i0, cnt)
        py_algorithm1(t, state, X, y, ep, ptally, postar, i0, cnt, False, vhat=vhat)
        assert np.array_equal(t.state, state), ep
        assert np.array_equal(tally, ptally) and np.array_equal(ostar, postar), ep
    assert fired > 50


@pytest.mark.parametrize("mistake", [dict(refresh=False), dict(stale=True)])
def test_algorithm1_comparison_catches_planted_mistakes(mistake):
    X, y = problem()
    t = fresh()
    tally, ostar = t.sync_tallies(X)
    state, ptally, postar = t.state.copy(), tally.copy(), ostar.copy()
    same = True
    for ep in range(EPOCHS):
        t.async_epoch(X, y, tally, ostar, ep, False)
        py_algorithm1(t, state, X, y, ep, ptally, postar, 0, Q, False, **mistake)
        same = same and np.array_equal(t.state, state) and np.array_equal(tally, ptally)
    assert not same
