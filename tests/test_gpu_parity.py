"""GPU parity: the HIP path against the CPU oracle, element by element, through
the C boundary.  Everything here is integer / bit work, so the bar is exact
equality."""
import numpy as np
import pytest
import torch

from oracle import tm_oracle as O
from paper_2009_04861_amd import binding as B
from paper_2009_04861_amd import synth
from tests.helpers import (bits_to_u8, dev_bits, dev_i32, gpu_state_as_oracle, make_pair, push_state,
                           sparse_random_state)

pytestmark = pytest.mark.gpu

# (m, n, o, N, T, s): shapes spanning one and several register slots per lane,
# ragged feature tails, mixed classes inside a 64-clause tile, both saturation paths
SHAPES = [
    (2, 10, 12, 100, 15, 3.9),      # noisy-XOR machine: 2 literal words, classes share a tile
    (3, 6, 37, 20, 4, 3.0),         # ragged tail, 3 classes in one tile
    (10, 20, 784, 128, 16, 10.0),   # image-like feature count, 50 literal words
    (2, 70, 100, 128, 9, 2.0),      # tiles straddle a class boundary; threshold 0x8000
    (4, 4, 1100, 64, 7, 5.0),       # 70 literal words -> 2 register slots
    (2, 4, 2500, 128, 3, 10.0),     # 158 literal words -> 3 slots, 3 mask chunks in evaluation
    (2, 4, 10000, 128, 20, 2.0),    # text-like feature count: 626 literal words -> 10 slots
    (2, 2, 20000, 128, 10, 5.0),    # stress feature count: 1250 literal words -> 20 slots
    (2, 6, 250, 50, 8, 10.0),       # 16 literal words, ragged tail: the widest clause whose Type I blocks are drawn side by side
]


def rand_problem(rng, q, o, m, density=0.3):
    X = (rng.random((q, o)) < density).astype(np.uint8)
    y = rng.integers(0, m, size=q).astype(np.int32)
    return X, y


@pytest.mark.parametrize("shape", SHAPES)
def test_initial_states_match(shape, device):
    m, n, o, N, T, s = shape
    print("init", shape, flush=True)
    ora, gpu = make_pair(m, n, o, N, T, s, 1234)
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)


@pytest.mark.parametrize("shape", SHAPES)
def test_state_roundtrip(shape, device):
    m, n, o, N, T, s = shape
    print("roundtrip", shape, flush=True)
    rng = np.random.default_rng(1)
    ora, gpu = make_pair(m, n, o, N, T, s, 5)
    st = rng.integers(1, 2 * N + 1, size=ora.state.shape).astype(np.int32)
    push_state(gpu, st)
    assert np.array_equal(gpu_state_as_oracle(gpu), st)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("q", [1, 63, 300, 777])
def test_inference_matches(shape, q, device):
    m, n, o, N, T, s = shape
    print("inference", shape, q, flush=True)
    rng = np.random.default_rng(q + o)
    ora, gpu = make_pair(m, n, o, N, T, s, 7)
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, N, 1.5 / o)
    push_state(gpu, ora.state)
    X, _ = rand_problem(rng, q, o, m)
    Xd = dev_bits(gpu, X)
    assert np.array_equal(bits_to_u8(gpu.clause_outputs(Xd), q), ora.clause_outputs(X).T)
    want = ora.class_sums(X)
    assert q < 63 or np.abs(want).max() > 0
    for lists in (True, False):   # literal-list evaluation with a workspace / mask evaluation without
        assert np.array_equal(gpu.class_sums(Xd, lists=lists).cpu().numpy(), want)
        assert np.array_equal(gpu.predict(Xd, lists=lists).cpu().numpy(), ora.predict(X))


@pytest.mark.parametrize("q", [70, 2048, 2049, 4500])
def test_literal_list_lengths_and_dense_clauses(q, device):
    """Clauses with 0 .. 300 included literals that are nevertheless satisfied (the lists
    hold 128 literals; longer clauses are finished from their masks), next to untrained
    clauses that include about half of all literals; ranges of 2048 examples with a tail."""
    m, n, o, N, T = 2, 24, 420, 128, 9
    print("literal lists", q, flush=True)
    rng = np.random.default_rng(q)
    ora, gpu = make_pair(m, n, o, N, T, 4.0, 5)
    X = (rng.random((q, o)) < 0.5).astype(np.uint8)
    X[:, 100:420] = 0                     # features that are always 0: their negated literals always hold
    y = rng.integers(0, m, size=q).astype(np.int32)
    st = np.ones((ora.C, ora.L), dtype=np.int32)
    lengths = [0, 1, 3, 4, 5, 127, 128, 129, 131, 132, 133, 300]
    for g, k in enumerate(lengths):                    # class 0: k always-true literals
        st[g, o + 100:o + 100 + k] = 2 * N
    for g, k in enumerate(lengths):                    # class 1: the same plus one literal that depends on the data
        st[n + g, o + 100:o + 100 + k] = 2 * N
        st[n + g, g if g % 3 else o + g] = 2 * N       # x_g or NOT x_g
    st[12:24] = rng.integers(1, 2 * N + 1, size=(12, ora.L))        # untrained: half of the literals included
    st[n + 12:n + 24] = rng.integers(1, 2 * N + 1, size=(12, ora.L))
    ora.state[:] = st
    push_state(gpu, ora.state)
    Xd = dev_bits(gpu, X)
    want = ora.class_sums(X)
    assert np.abs(want).max() > 0
    for lists in (True, False):
        assert np.array_equal(gpu.class_sums(Xd, lists=lists).cpu().numpy(), want)
        assert np.array_equal(gpu.predict(Xd, lists=lists).cpu().numpy(), ora.predict(X))
    # the tally pre-calculation of bind uses the lists as well
    gpu.bind_train(Xd, dev_i32(gpu, y))
    assert np.array_equal(gpu.tallies().cpu().numpy(), ora.class_sums(X, clamp=False))
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ora.clause_outputs(X).T)


@pytest.mark.parametrize("n", [4080, 4082, 9000])
def test_vote_counters_at_capacity(n, device):
    """Every positive clause of class 0 is satisfied by every example and no negative one is:
    the bit-sliced vote counters of the literal-list kernel hold their largest counts (255
    clauses per wavefront at n = 4080; more clauses split a class over several workgroups)."""
    m, o, N, T, q = 2, 8, 128, 3000, 100
    print("vote counters", n, flush=True)
    rng = np.random.default_rng(n)
    ora, gpu = make_pair(m, n, o, N, T, 4.0, 5)
    st = np.ones((ora.C, ora.L), dtype=np.int32)
    st[0:n:2, 0] = 2 * N          # negative clauses of class 0: x0 AND NOT x0
    st[0:n:2, o] = 2 * N
    st[n + 1:2 * n:4, 1] = 2 * N  # some positive clauses of class 1: x1
    ora.state[:] = st
    push_state(gpu, ora.state)
    X, y = rand_problem(rng, q, o, m)
    Xd = dev_bits(gpu, X)
    want = ora.class_sums(X)
    assert want[:, 0].max() == min(T, n // 2)
    for lists in (True, False):
        assert np.array_equal(gpu.class_sums(Xd, lists=lists).cpu().numpy(), want)
    gpu.bind_train(Xd, dev_i32(gpu, y))
    assert np.array_equal(gpu.tallies().cpu().numpy(), ora.class_sums(X, clamp=False))


@pytest.mark.parametrize("n", [16264, 18288])
def test_vote_counters_when_the_capacity_sets_the_split(n, device):
    """2 classes x 131,067 examples give 128 (class, range) pairs, so the workgroup count alone would
    split a class 8 ways: 2,033 .. 2,040 clauses per share, which the rounding to a multiple of 16
    must not turn into 2,048 (256 same-polarity clauses per wavefront, one more than its 8-plane
    counter holds).  Every positive clause of class 0 is empty (satisfied by every example) and no
    negative one can be satisfied: every example's sum is n/2, in closed form; sampled examples are
    checked against the oracle as well.  n = 18,288 = 9 x 2,032 fills the counters to their bound:
    254 satisfied clauses per wavefront."""
    m, o, N, T, q = 2, 8, 128, 9500, 131067
    print("vote counters, split set by capacity", n, flush=True)
    S, chunk = B.tm_eval_shares(B.make_config(m, n, o, N, T, 4.0, 5), q)
    assert chunk <= 2032 and S * chunk >= n and S == 9 and (n != 18288 or chunk == 2032)
    rng = np.random.default_rng(n)
    ora, gpu = make_pair(m, n, o, N, T, 4.0, 5)
    st = np.ones((ora.C, ora.L), dtype=np.int32)
    st[0:n:2, 0] = 2 * N          # negative clauses of class 0: x0 AND NOT x0
    st[0:n:2, o] = 2 * N
    st[n + 1:2 * n:4, 1] = 2 * N  # some positive clauses of class 1: x1
    st[n:2 * n:2, 2] = 2 * N      # negative clauses of class 1: x2
    ora.state[:] = st
    push_state(gpu, ora.state)
    X, y = rand_problem(rng, q, o, m)
    Xd = dev_bits(gpu, X)
    got = gpu.class_sums(Xd, lists=True).cpu().numpy()
    assert np.all(got[:, 0] == n // 2)
    closed = ((n + 2) // 4) * X[:, 1].astype(np.int64) + ((n // 2 - (n + 2) // 4)) - (n // 2) * X[:, 2].astype(np.int64)
    assert np.array_equal(got[:, 1], closed)
    ex = np.concatenate([[0, 1, 2047, 2048, q - 1], rng.integers(0, q, size=20)])
    assert np.array_equal(got[ex], ora.class_sums(np.ascontiguousarray(X[ex])))
    gpu.bind_train(Xd, dev_i32(gpu, y))
    assert np.array_equal(gpu.tallies().cpu().numpy(), got)     # T is above every sum: nothing is clamped
    gpu.close()


def test_class_sums_are_clamped(device):
    ora, gpu = make_pair(2, 64, 20, 128, 5, 3.0, 3)
    ora.state[:] = 1
    push_state(gpu, ora.state)          # every clause empty -> raw sums 0; silence negatives of class 1
    ora.state[64 + np.arange(0, 64, 2), :] = 256
    push_state(gpu, ora.state)
    X = np.zeros((5, 20), dtype=np.uint8)
    for lists in (True, False):
        got = gpu.class_sums(dev_bits(gpu, X), lists=lists).cpu().numpy()
        assert np.array_equal(got, ora.class_sums(X))
        assert got[0].tolist() == [0, 5]


@pytest.mark.parametrize("shape", SHAPES)
def test_sync_pass_matches(shape, device):
    m, n, o, N, T, s = shape
    print("sync", shape, flush=True)
    rng = np.random.default_rng(11)
    q = 333
    ora, gpu = make_pair(m, n, o, N, T, s, 7)
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, N, 1.5 / o)
    push_state(gpu, ora.state)
    X, y = rand_problem(rng, q, o, m)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar)


@pytest.mark.parametrize("ranges", [24, 27, 31])
def test_sync_pass_with_many_ranges_of_examples(ranges, device):
    """From 24 ranges of 2,048 examples on, the workgroups of the tally pre-calculation are dealt out to the
    eight XCDs range by range (XCD x takes the ranges x, x + 8, ...; the grid is padded to whole rounds of
    eight): every (range, class) must still be evaluated exactly once (24: no range left over after whole
    rounds, 27: three, 31: seven; ragged tail of examples)."""
    m, n, o, N, T, s = 3, 6, 37, 20, 4, 3.0
    q = 2048 * ranges - 5
    print("many ranges", ranges, flush=True)
    rng = np.random.default_rng(ranges)
    ora, gpu = make_pair(m, n, o, N, T, s, 7)
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, N, 1.5 / o)
    push_state(gpu, ora.state)
    X, y = rand_problem(rng, q, o, m)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar)
    assert np.array_equal(gpu.class_sums(dev_bits(gpu, X)).cpu().numpy(), ora.class_sums(X))


def run_frozen(ora, gpu, X, y, epoch, i0, cnt, tally, ostar):
    """One frozen-snapshot step on both sides from the same starting point."""
    snap = tally.copy()
    gpu.feedback_step(dev_i32(gpu, snap), i0, cnt)
    fired = ora.feedback_step(X, y, snap, tally, ostar, epoch, i0, cnt)
    return fired


@pytest.mark.parametrize("shape", SHAPES)
def test_feedback_step_matches_bit_exactly(shape, device):
    m, n, o, N, T, s = shape
    print("feedback", shape, flush=True)
    rng = np.random.default_rng(21)
    q = 200
    ora, gpu = make_pair(m, n, o, N, T, s, 99)
    X, y = rand_problem(rng, q, o, m)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    total_fired = 0
    # ranges that start and end inside 64-example blocks, then whole passes
    for step, (i0, cnt) in enumerate([(0, 1), (1, 70), (71, 57), (128, 72), (0, q), (0, q), (0, q)]):
        B.tm_set_epoch(gpu.h, step)
        total_fired += run_frozen(ora, gpu, X, y, step, i0, cnt, tally, ostar)
        assert np.array_equal(gpu_state_as_oracle(gpu), ora.state), ("state", step)
        assert np.array_equal(gpu.tallies().cpu().numpy(), tally), ("tally", step)
        assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar), ("ostar", step)
    assert total_fired > 0
    c = gpu.counters()
    assert c["fired"] == total_fired


# one feature count per width the training kernel is compiled for (literal words -> register slots per
# lane: 4, 6, 8, 12 and 16; 1, 2, 3, 10 and 20 are among SHAPES), ragged last feature word
@pytest.mark.parametrize("o,N,s,regression", [(4001, 128, 5.0, False), (6003, 64, 3.0, False), (8005, 128, 10.0, False),
                                              (12007, 128, 2.0, False), (16009, 100, 4.0, False), (8005, 128, 1.5, True)])
def test_feedback_step_in_every_kernel_width(o, N, s, regression, device):
    print("feedback, kernel width", o, N, s, regression, flush=True)
    m, n, T, q = (1, 6, 6, 150) if regression else (2, 2, 3, 150)
    rng = np.random.default_rng(o)
    ora = O.Oracle(m, n, o, N, T, s, 17, regression=regression)
    gpu = B.TsetlinMachine(m, n, o, N, T, s, 17, regression=regression)
    X = (rng.random((q, o)) < 0.05).astype(np.uint8)
    y = rng.integers(0, (T + 1) if regression else m, size=q).astype(np.int32)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
    fired = 0
    for step, (i0, cnt) in enumerate([(0, 70), (70, 80), (0, q), (0, q)]):
        B.tm_set_epoch(gpu.h, step)
        fired += run_frozen(ora, gpu, X, y, step, i0, cnt, tally, ostar)
        assert np.array_equal(gpu_state_as_oracle(gpu), ora.state), step
        assert np.array_equal(gpu.tallies().cpu().numpy(), tally), step
        assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar), step
    assert fired > 20
    assert np.array_equal(gpu.class_sums(dev_bits(gpu, X)).cpu().numpy(), ora.class_sums(X))
    gpu.close()


@pytest.mark.parametrize("s", [1.0, 2.0, 4.0, 3.9, 25.0])
@pytest.mark.parametrize("N", [3, 100, 128])
def test_feedback_saturation_and_threshold_paths(s, N, device):
    # small N drives automata into both ends of their range quickly
    print("saturation", s, N, flush=True)
    m, n, o, T = 2, 8, 45, 6
    rng = np.random.default_rng(5)
    q = 150
    ora, gpu = make_pair(m, n, o, N, T, s, 17)
    X, y = rand_problem(rng, q, o, m, density=0.5)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    for ep in range(12):
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, X, y, ep, 0, q, tally, ostar)
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)


@pytest.mark.parametrize("s", [2.0, 3.9])
@pytest.mark.parametrize("N", [3, 100, 128])
def test_feedback_reaches_both_ends_of_the_state_range(s, N, device):
    # plain literals start one below the top, negated ones one above the bottom, and
    # half the examples are all-ones: strong Type I pushes into 2N, weak into 1
    print("ends", s, N, flush=True)
    m, n, o, T = 2, 8, 45, 6
    rng = np.random.default_rng(5)
    q = 150
    ora, gpu = make_pair(m, n, o, N, T, s, 17)
    X, y = rand_problem(rng, q, o, m, density=0.5)
    X[::2] = 1
    ora.state[:, :o] = 2 * N - 1
    ora.state[:, o:] = 2
    push_state(gpu, ora.state)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    for ep in range(6):
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, X, y, ep, 0, q, tally, ostar)
    assert ora.state.min() == 1 and ora.state.max() == 2 * N
    assert (ora.state == 2 * N).sum() > 5 and (ora.state == 1).sum() > 2
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar)


def test_set_state_after_bind_then_step_refreshes_everything(device):
    # the stored previous outputs come from the old clauses; a pass must repair all of them
    m, n, o, N, T, s = 3, 6, 37, 20, 4, 3.0
    rng = np.random.default_rng(77)
    q = 300
    ora, gpu = make_pair(m, n, o, N, T, s, 5)
    X, y = rand_problem(rng, q, o, m)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)                       # tallies / outputs of the initial clauses
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, N, 2.0 / o)
    push_state(gpu, ora.state)                               # new clauses, no re-synchronisation
    for ep, (i0, cnt) in enumerate([(100, 100), (0, q), (0, q)]):
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, X, y, ep, i0, cnt, tally, ostar)
        assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)
        assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
        assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar)


@pytest.mark.parametrize("o", [100, 2500, 5000])
def test_long_runs_of_outdated_blocks_are_swept_through_literal_lists(o, device):
    """Sparse clauses pushed after bind leave every stored output outdated; few gates can open,
    so the passes refresh long runs of blocks, 2048 examples at a time through the clause's
    literal list (clauses of up to 4 register slots per lane and 256 literals; o = 5000 keeps to the block-by-block path).  Ranges start and
    end inside blocks and words; 5,000 examples span two segments of the launch preparation."""
    m, n, N, T, s = 3, 6, 64, 2, 4.0
    print("list sweeps", o, flush=True)
    rng = np.random.default_rng(o)
    q = 5000
    ora, gpu = make_pair(m, n, o, N, T, s, 5)
    X, y = rand_problem(rng, q, o, m)
    X[::7, :300] = 0                                           # every seventh example satisfies the 300-literal clause below
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, N, 2.5 / o)
    ora.state[0, :] = 1                                        # an empty clause
    ora.state[1, :70] = 2 * N                                  # 70 literals: several rounds of the list sweep
    if o >= 300:
        ora.state[2, o:o + 300] = 2 * N                        # 300 negated literals: more than the list in LDS holds
    push_state(gpu, ora.state)
    gpu.counters()
    # snapshot that closes every gate (+T for the label, -T elsewhere) except on 2 % of the examples
    snap = np.full((q, m), -T, dtype=np.int32)
    snap[np.arange(q), y] = T
    snap[rng.random(q) < 0.02] = 0
    fired = 0
    for ep, (i0, cnt) in enumerate([(1234, 3000), (0, q), (4097, 903), (0, q)]):
        B.tm_set_epoch(gpu.h, ep)
        gpu.feedback_step(dev_i32(gpu, snap), i0, cnt)
        fired += ora.feedback_step(X, y, snap, tally, ostar, ep, i0, cnt)
        assert np.array_equal(gpu_state_as_oracle(gpu), ora.state), ep
        assert np.array_equal(gpu.tallies().cpu().numpy(), tally), ep
        assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar), ep
    c = gpu.counters()
    print("fired %d, blocks evaluated %d, of them through lists %d" % (fired, c["blocks_evaluated"], c["blocks_listed"]),
          flush=True)
    assert fired > 20 and c["fired"] == fired
    assert (c["blocks_listed"] > 0) == (o <= 4096)


def test_quiet_epochs_skip_evaluation_but_change_nothing(device):
    # T = 1 closes almost every gate once the sums reach the margin: most blocks are skipped
    m, n, o, N, T, s = 2, 20, 30, 50, 1, 3.0
    rng = np.random.default_rng(78)
    q = 1000
    ora, gpu = make_pair(m, n, o, N, T, s, 6)
    X, y = rand_problem(rng, q, o, m)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    gpu.counters()
    for ep in range(8):
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, X, y, ep, 0, q, tally, ostar)
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar)
    c = gpu.counters()
    blocks = 8 * ora.C * ((q + 63) // 64)
    assert 0 < c["blocks_evaluated"] <= blocks
    print("blocks evaluated: %d of %d" % (c["blocks_evaluated"], blocks), flush=True)


@pytest.mark.parametrize("N", [5, 128])
def test_feedback_with_boosted_true_positives(N, device):
    m, n, o, T, s = 3, 8, 70, 6, 4.0
    rng = np.random.default_rng(91)
    q = 200
    ora, gpu = make_pair(m, n, o, N, T, s, 23, boost=True)
    X, y = rand_problem(rng, q, o, m, density=0.5)
    X[::3] = 1
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, N, 2.0 / o)
    push_state(gpu, ora.state)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    for ep in range(6):
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, X, y, ep, 0, q, tally, ostar)
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar)
    assert ora.state.max() > N


def test_noisy_xor_frozen_epochs_match(device):
    # the small benchmark configuration, whole epochs, snapshot = tallies at epoch start
    Xtr, ytr, Xte, yte = synth.noisy_xor(1000, 500)
    ora, gpu = make_pair(2, 10, 12, 100, 15, 3.9, 1)
    gpu.bind_train(dev_bits(gpu, Xtr), dev_i32(gpu, ytr))
    tally, ostar = ora.sync_tallies(Xtr)
    for ep in range(10):
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, Xtr, ytr, ep, 0, len(ytr), tally, ostar)
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)
    assert np.array_equal(gpu.predict(dev_bits(gpu, Xte)).cpu().numpy(), ora.predict(Xte))


# narrow machines (one launch per epoch) and wide ones: 3 register slots with list sweeps, 10 and 20
# slots with block-by-block sweeps and 3 / 5 launches per epoch (4,000 examples against launches of
# 1,664 and 832)
ASYNC_SHAPES = [(sh, 500) for sh in SHAPES[:4]] + [
    ((2, 6, 2500, 128, 3, 10.0), 4000),
    ((2, 4, 10000, 128, 20, 2.0), 4000),
    ((2, 2, 20000, 128, 10, 5.0), 4000),
]


@pytest.mark.parametrize("shape,q", ASYNC_SHAPES)
def test_async_epoch_invariants(shape, q, device):
    m, n, o, N, T, s = shape
    print("async", shape, q, flush=True)
    rng = np.random.default_rng(31)
    ora, gpu = make_pair(m, n, o, N, T, s, 3)
    X, y = rand_problem(rng, q, o, m)
    Xd = dev_bits(gpu, X)
    gpu.bind_train(Xd, dev_i32(gpu, y))
    launches = -(-q // B.tm_train_chunk(gpu.h))
    assert launches == (1 if o <= 4096 else 3 if o == 10000 else 5)
    sign = np.where(np.arange(ora.C) % n % 2 == 1, 1, -1)
    gpu.counters()
    for ep in range(4):
        gpu.fit_epoch()
        st = gpu.get_ta_state().cpu().numpy()
        assert st.max() <= 2 * N - 1                               # states stay in [1, 2N]
        # atomics lose nothing: the tally is the signed sum of the stored previous outputs
        ostar = bits_to_u8(gpu.prev_outputs(), q).astype(np.int64)
        want = np.stack([(ostar[c * n:(c + 1) * n] * sign[c * n:(c + 1) * n, None]).sum(0) for c in range(m)], 1)
        assert np.array_equal(gpu.tallies().cpu().numpy(), want)
    assert B.tm_get_epoch(gpu.h) == 4
    # eventual consistency: after a pass of pure refreshes the tallies are the exact vote sums
    gpu.sync_tallies()
    ora.state[:] = gpu_state_as_oracle(gpu)
    assert np.array_equal(gpu.tallies().cpu().numpy(), ora.class_sums(X, clamp=False))
    c = gpu.counters()
    # counted on the device: every clause got a wavefront in every launch and walked the launch's examples
    assert c["pairs"] == 4 * q * ora.C and 0 < c["fired"] < c["pairs"]


def test_epochs_walked_in_batches(device):
    """Algorithm 1 batch by batch (tm_fit_batch, b = 250) with the tallies recomputed after every
    batch: the bookkeeping invariants hold after every batch, the epoch counter is the caller's,
    and the noisy-XOR machine learns as it does with whole-epoch passes."""
    hp = synth.WORKLOADS["noisy_xor"]
    Xtr, ytr, Xte, yte = synth.noisy_xor(2000, 2000)
    ora, gpu = make_pair(seed=9, **hp)
    m, n, q, b = hp["m"], hp["n"], len(ytr), 250
    Xd = dev_bits(gpu, Xtr)
    gpu.bind_train(Xd, dev_i32(gpu, ytr))
    Xte_d = dev_bits(gpu, Xte)
    sign = np.where(np.arange(ora.C) % n % 2 == 1, 1, -1)
    gpu.counters()
    accs = []
    for ep in range(40):
        B.tm_set_epoch(gpu.h, ep)
        for i0 in range(0, q, b):
            gpu.fit_batch(i0, b)
            if ep < 3:
                ostar = bits_to_u8(gpu.prev_outputs(), q).astype(np.int64)
                want = np.stack([(ostar[c * n:(c + 1) * n] * sign[c * n:(c + 1) * n, None]).sum(0) for c in range(m)], 1)
                assert np.array_equal(gpu.tallies().cpu().numpy(), want)
            gpu.sync_tallies()
        assert B.tm_get_epoch(gpu.h) == ep
        if ep >= 30:
            accs.append((gpu.predict(Xte_d).cpu().numpy() == yte).mean())
    assert gpu.counters()["pairs"] == 40 * q * ora.C
    print("accuracy with batches of %d: %.4f" % (b, np.mean(accs)), flush=True)
    assert np.mean(accs) > 0.85     # 40 % label noise, 2000 examples: whole-epoch passes reach about 0.93 too
    with pytest.raises(B.TMError) as e:
        gpu.fit_batch(q + 1, 10)
    assert e.value.code == B.TM_EINVAL


@pytest.mark.parametrize("case", range(24))
def test_random_small_configurations(case, device):
    """Random corners of the parameter space (one feature, two clauses, one example, one state
    per action, s = 1, margins beyond the clause count, ...): initial state, pre-calculation, two
    frozen passes, inference, all against the oracle."""
    rng = np.random.default_rng(1000 + case)
    m = int(rng.choice([2, 2, 3, 5, 11]))
    n = int(rng.choice([2, 2, 4, 6, 18, 34]))
    o = int(rng.choice([1, 2, 31, 32, 33, 64, 65, 200]))
    N = int(rng.choice([1, 2, 7, 128]))
    T = int(rng.choice([1, 2, n, 3 * n]))
    s = float(rng.choice([1.0, 1.5, 3.0, 50.0]))
    q = int(rng.choice([1, 2, 63, 64, 65, 129, 400]))
    print("random configuration", case, (m, n, o, N, T, s, q), flush=True)
    ora, gpu = make_pair(m, n, o, N, T, s, 40 + case)
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state)
    X, y = rand_problem(rng, q, o, m, density=float(rng.choice([0.1, 0.5, 0.9])))
    Xd = dev_bits(gpu, X)
    gpu.bind_train(Xd, dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar)
    for ep in range(2):
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, X, y, ep, 0, q, tally, ostar)
        assert np.array_equal(gpu_state_as_oracle(gpu), ora.state), ep
        assert np.array_equal(gpu.tallies().cpu().numpy(), tally), ep
        assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar), ep
    for lists in (True, False):
        assert np.array_equal(gpu.class_sums(Xd, lists=lists).cpu().numpy(), ora.class_sums(X))
        assert np.array_equal(gpu.predict(Xd, lists=lists).cpu().numpy(), ora.predict(X))
    gpu.fit_epoch()
    gpu.sync_tallies()
    ora.state[:] = gpu_state_as_oracle(gpu)
    assert np.array_equal(gpu.tallies().cpu().numpy(), ora.class_sums(X, clamp=False))


def test_clause_groups_are_a_schedule_only(device):
    """Sub-launches over clause ranges (tm_set_clause_groups) must not change the result of a frozen
    pass: group boundaries inside a class, groups of one clause, more examples than one preparation segment."""
    m, n, o, N, T, s = 3, 10, 70, 20, 6, 3.0
    rng = np.random.default_rng(55)
    q = 4500
    ora, gpu = make_pair(m, n, o, N, T, s, 12)
    X, y = rand_problem(rng, q, o, m)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    tally, ostar = ora.sync_tallies(X)
    gpu.counters()
    for ep, groups in enumerate([4, 30, 1, 7]):
        B.tm_set_clause_groups(gpu.h, groups)
        B.tm_set_epoch(gpu.h, ep)
        run_frozen(ora, gpu, X, y, ep, 100 * ep, q, tally, ostar)
        assert np.array_equal(gpu_state_as_oracle(gpu), ora.state), groups
        assert np.array_equal(gpu.tallies().cpu().numpy(), tally), groups
        assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar), groups
    c = gpu.counters()
    visited = sum(q - 100 * ep for ep in range(4))
    assert c["pairs"] == visited * ora.C
    assert c["candidates"] == 2 * n * visited      # every example trains its own class and one other


def test_error_codes(device):
    gpu = B.TsetlinMachine(3, 4, 20, 10, 5, 3.0, 1)
    with pytest.raises(B.TMError) as e:
        gpu.fit_epoch()
    assert e.value.code == B.TM_ESTATE
    X = dev_bits(gpu, np.zeros((10, 20), dtype=np.uint8))
    with pytest.raises(B.TMError) as e:
        gpu.bind_train(X, dev_i32(gpu, np.array([0, 1, 2, 3, 0, 0, 0, 0, 0, 0])))   # label 3 of 3 classes
    assert e.value.code == B.TM_EINVAL
    with pytest.raises(B.TMError) as e:
        gpu.fit_epoch()
    assert e.value.code == B.TM_ESTATE
    gpu.bind_train(X, dev_i32(gpu, np.zeros(10)))
    gpu.fit_epoch()
    # empty inference batch is a no-op
    empty = torch.empty((0, 1), dtype=torch.int32, device=gpu.dev)
    assert gpu.class_sums(empty).shape == (0, 3)
    torch.cuda.synchronize()
