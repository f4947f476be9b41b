"""GPU parity of the training calls the product runs (tm_fit_epoch, tm_fit_batch: Algorithm 1 with
the gate reading the LIVE tallies) against the oracle, bit for bit.

Asynchronous training is not reproducible when clauses run side by side.  With one clause per
sub-launch (tm_set_clause_groups(C)) nothing runs beside a clause, so a tally of example i is only
touched by the clause that visits i, and the training call must reproduce the sequential
Algorithm 1 of the oracle with clauses outermost: every launch of the training kernel covers a
range of examples, within it the clauses take turns, each walking the range in order.  States,
stored previous outputs and tallies are compared after every epoch (every batch), over several
epochs, for narrow and wide clauses, single- and multi-launch epochs, classification and
regression."""
import numpy as np
import pytest

from oracle import tm_oracle as O
from paper_2009_04861_amd import binding as B
from tests.helpers import bits_to_u8, dev_bits, dev_i32, gpu_state_as_oracle

pytestmark = pytest.mark.gpu


def assert_same(gpu, ora, tally, ostar, q, where):
    assert np.array_equal(gpu_state_as_oracle(gpu), ora.state), ("state", where)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs(), q), ostar), ("ostar", where)
    assert np.array_equal(gpu.tallies().cpu().numpy(), tally), ("tally", where)


def oracle_epoch_in_launches(ora, X, y, tally, ostar, epoch, chunk):
    """The schedule of tm_fit_epoch with one clause per sub-launch: launch by launch (ranges of
    `chunk` examples), clause after clause within a launch."""
    for i0 in range(0, len(y), chunk):
        ora.async_range(X, y, tally, ostar, epoch, i0, chunk, example_major=False)


# (m, n, o, N, T, s, q, density): C <= 40; 1, 1, 3, 5 and 10 register slots per lane; the machines of
# more than 4 slots cut an epoch into several launches (tm_train_chunk), q is chosen above that
LIVE_SHAPES = [
    (2, 10, 12, 100, 15, 3.9, 700, 0.5),
    (5, 8, 100, 20, 6, 3.0, 500, 0.3),
    (2, 6, 2500, 128, 4, 10.0, 400, 0.3),
    (5, 2, 4200, 64, 3, 4.0, 4500, 0.2),
    (2, 4, 10000, 128, 3, 2.0, 1800, 0.1),
]


@pytest.mark.parametrize("shape", LIVE_SHAPES)
def test_live_epochs_match_sequential_algorithm1(shape, device):
    m, n, o, N, T, s, q, density = shape
    print("live epochs", shape, flush=True)
    rng = np.random.default_rng(o + q)
    ora = O.Oracle(m, n, o, N, T, s, 77)
    gpu = B.TsetlinMachine(m, n, o, N, T, s, 77)
    X = (rng.random((q, o)) < density).astype(np.uint8)
    y = rng.integers(0, m, size=q).astype(np.int32)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    B.tm_set_clause_groups(gpu.h, ora.C)
    chunk = B.tm_train_chunk(gpu.h)
    launches = (q + chunk - 1) // chunk
    assert launches >= 2 or o <= 4096
    tally, ostar = ora.sync_tallies(X)
    assert_same(gpu, ora, tally, ostar, q, "bind")
    gpu.counters()
    moved = 0
    for ep in range(4):
        before = tally.copy()
        gpu.fit_epoch()
        oracle_epoch_in_launches(ora, X, y, tally, ostar, ep, chunk)
        assert_same(gpu, ora, tally, ostar, q, ep)
        moved += int((before != tally).sum())
    c = gpu.counters()
    print("launches per epoch %d, fired %d, tally entries moved %d" % (launches, c["fired"], moved), flush=True)
    assert B.tm_get_epoch(gpu.h) == 4 and c["fired"] > 50 and moved > 50
    gpu.close()


def test_live_batches_match_sequential_algorithm1(device):
    """tm_fit_batch with ragged batch boundaries (inside blocks of 64 and words of 32 examples)."""
    m, n, o, N, T, s, q = 3, 6, 70, 10, 5, 3.0, 1000
    rng = np.random.default_rng(8)
    ora = O.Oracle(m, n, o, N, T, s, 5)
    gpu = B.TsetlinMachine(m, n, o, N, T, s, 5)
    X = (rng.random((q, o)) < 0.4).astype(np.uint8)
    y = rng.integers(0, m, size=q).astype(np.int32)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    B.tm_set_clause_groups(gpu.h, ora.C)
    tally, ostar = ora.sync_tallies(X)
    for ep in range(3):
        B.tm_set_epoch(gpu.h, ep)
        for i0, cnt in [(0, 1), (1, 99), (100, 333), (433, 64), (497, 5000)]:
            gpu.fit_batch(i0, cnt)
            ora.async_range(X, y, tally, ostar, ep, i0, cnt, example_major=False)
            assert_same(gpu, ora, tally, ostar, q, (ep, i0))
    gpu.close()


@pytest.mark.parametrize("shape", [(24, 40, 20, 24, 1.5, 600), (12, 4200, 128, 12, 2.0, 4300)])
def test_live_regression_epochs_match_sequential_algorithm1(shape, device):
    n, o, N, T, s, q = shape
    print("live regression epochs", shape, flush=True)
    rng = np.random.default_rng(o)
    ora = O.Oracle(1, n, o, N, T, s, 31, regression=True)
    gpu = B.TsetlinMachine(1, n, o, N, T, s, 31, regression=True)
    X = (rng.random((q, o)) < 0.3).astype(np.uint8)
    y = rng.integers(0, T + 1, size=q).astype(np.int32)
    gpu.bind_train(dev_bits(gpu, X), dev_i32(gpu, y))
    B.tm_set_clause_groups(gpu.h, ora.C)
    chunk = B.tm_train_chunk(gpu.h)
    tally, ostar = ora.sync_tallies(X)
    gpu.counters()
    for ep in range(3):
        gpu.fit_epoch()
        oracle_epoch_in_launches(ora, X, y, tally, ostar, ep, chunk)
        assert_same(gpu, ora, tally, ostar, q, ep)
    assert gpu.counters()["fired"] > 50
    gpu.close()
