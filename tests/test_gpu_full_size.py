"""Parity at the benchmark's full size (image-like workload: 60,000 x 784, 10 classes x
2,000 clauses), in the launch configuration bench.py times.  The oracle cannot run the
whole machine in reasonable time, so it follows sampled clauses (whose trajectories are
independent under a frozen tally snapshot) and sampled examples; properties that hold at
any size cover the rest.  No expected value comes from the HIP path: the frozen snapshot
is synthetic."""
import numpy as np
import pytest
import torch

from oracle import tm_oracle as O
from paper_2009_04861_amd import binding as B
from paper_2009_04861_amd import synth
from tests.helpers import bits_to_u8, dev_bits, dev_i32, push_state, sparse_random_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def workload():
    return synth.image_like()


def test_full_size_training_pass_sampled_clauses(workload, device):
    Xtr, ytr, Xte, yte = workload
    hp = synth.WORKLOADS["image_like"]
    m, n, o = hp["m"], hp["n"], hp["o"]
    q = len(ytr)
    print("full size: oracle init", flush=True)
    ora = O.Oracle(seed=3, **hp)
    gpu = B.TsetlinMachine(seed=3, **hp)
    rng = np.random.default_rng(0)
    # sampled clauses: both polarities, first / last class, first / last clause
    ids = np.array([0, 1, n - 1, 3 * n + 500, 3 * n + 501, 7 * n + 1234, m * n - 2, m * n - 1], dtype=np.int32)
    st0 = gpu.get_ta_state().cpu().numpy().astype(np.int32) + 1
    assert np.array_equal(st0[ids], ora.state[ids])
    del st0

    print("full size: bind", flush=True)
    gpu.bind_train(dev_bits(gpu, Xtr), dev_i32(gpu, ytr))
    # tally pre-calculation on sampled examples (exact vote sums of all 20,000 clauses)
    ex = np.concatenate([[0, 1, 63, 64, q - 1], rng.integers(0, q, size=27)])
    want = ora.class_sums(np.ascontiguousarray(Xtr[ex]), clamp=False)
    got = gpu.tallies().cpu().numpy()
    assert np.array_equal(got[ex], want)
    ostar_sub = ora.clause_outputs_subset(Xtr, ids)
    prev = gpu.prev_outputs()
    assert np.array_equal(bits_to_u8(prev[torch.from_numpy(ids).long().to(prev.device)], q), ostar_sub)

    print("full size: frozen pass", flush=True)
    vhat = rng.integers(-hp["T"], hp["T"] + 1, size=(q, m)).astype(np.int32)   # synthetic snapshot
    B.tm_set_epoch(gpu.h, 5)
    gpu.feedback_step(dev_i32(gpu, vhat), 0, q)
    fired = ora.feedback_step_subset(Xtr, ytr, vhat, ostar_sub, 5, 0, q, ids)
    assert fired > 1000
    st1 = gpu.get_ta_state()[torch.from_numpy(ids).long().to(gpu.dev)].cpu().numpy().astype(np.int32) + 1
    assert np.array_equal(st1, ora.state[ids])
    prev = gpu.prev_outputs()
    assert np.array_equal(bits_to_u8(prev[torch.from_numpy(ids).long().to(prev.device)], q), ostar_sub)

    print("full size: tally == signed sum of stored outputs", flush=True)
    tally = gpu.tallies().cpu().numpy()
    sign = np.where(np.arange(n) % 2 == 1, 1, -1).astype(np.int32)
    for c in range(m):
        bits = bits_to_u8(prev[c * n:(c + 1) * n], q)          # [n][q]
        assert np.array_equal(tally[:, c], sign @ bits.astype(np.int32))

    print("full size: asynchronous epoch + refresh pass", flush=True)
    gpu.fit_epoch()
    st = gpu.get_ta_state()
    assert int(st.max()) <= 255
    gpu.sync_tallies()
    ora.state[:] = st.cpu().numpy().astype(np.int32) + 1
    got = gpu.tallies().cpu().numpy()
    assert np.array_equal(got[ex], ora.class_sums(np.ascontiguousarray(Xtr[ex]), clamp=False))
    gpu.close()


def test_full_size_inference_sampled_examples(workload, device):
    Xtr, ytr, Xte, yte = workload
    hp = synth.WORKLOADS["image_like"]
    rng = np.random.default_rng(1)
    ora = O.Oracle(seed=4, init=False, **hp)
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, hp["N"], 3.0 / hp["o"])
    gpu = B.TsetlinMachine(seed=4, **hp)
    push_state(gpu, ora.state)
    Xd = dev_bits(gpu, Xte)
    sums = gpu.class_sums(Xd).cpu().numpy()
    pred = gpu.predict(Xd).cpu().numpy()
    assert np.array_equal(sums, gpu.class_sums(Xd, lists=False).cpu().numpy())   # both evaluation schemes
    assert np.array_equal(pred, gpu.predict(Xd, lists=False).cpu().numpy())
    ex = np.concatenate([[0, 255, 256, len(yte) - 1], rng.integers(0, len(yte), size=44)])
    Xs = np.ascontiguousarray(Xte[ex])
    want = ora.class_sums(Xs)
    assert np.abs(want).max() > 0
    assert np.array_equal(sums[ex], want)
    assert np.array_equal(pred[ex], ora.predict(Xs))
    # properties at any size: clamped range, argmax consistent with the sums
    assert sums.min() >= -hp["T"] and sums.max() <= hp["T"]
    assert np.array_equal(pred, sums.argmax(axis=1))
    gpu.close()


@pytest.mark.parametrize("name,q,n_small", [("text_like", 25000, 64), ("stress", 20000, 32)])
def test_wide_feature_workloads_sampled_clauses(name, q, n_small, device):
    """The text-like (10,000 features, 10 register slots per lane) and stress (20,000 features,
    20 slots) workloads at their real feature width and example counts (stress: a 10 % subsample
    of the examples), with a reduced number of clauses so that the oracle can initialise the
    machine; per-clause work, kernels and launch shapes per clause are those of the full machine."""
    hp = dict(synth.WORKLOADS[name])
    hp["n"] = n_small
    hp["T"] = max(2, int(0.8 * n_small))
    if name == "text_like":
        Xtr, ytr, Xte, yte = synth.text_like(q, 2000)
    else:
        X, y = synth.planted_conjunctions(q + 2000)
        Xtr, ytr, Xte, yte = X[:q], y[:q], X[q:], y[q:]
    m, n = hp["m"], hp["n"]
    rng = np.random.default_rng(2)
    print(name, "oracle init", flush=True)
    ora = O.Oracle(seed=5, **hp)
    gpu = B.TsetlinMachine(seed=5, **hp)
    assert np.array_equal(gpu.get_ta_state().cpu().numpy().astype(np.int32) + 1, ora.state)
    # the second half of the clauses: a trained-looking state (ten negated literals included,
    # everything else excluded), so that clauses are satisfied by most examples of these sparse data
    half = m * n // 2
    ora.state[half:] = rng.integers(1, hp["N"] + 1, size=(m * n - half, ora.L))
    for g in range(half, m * n):
        ora.state[g, hp["o"] + rng.integers(0, hp["o"], size=10)] = rng.integers(hp["N"] + 1, 2 * hp["N"] + 1, size=10)
    push_state(gpu, ora.state)

    print(name, "bind", flush=True)
    gpu.bind_train(dev_bits(gpu, Xtr), dev_i32(gpu, ytr))
    ids = np.array([1, m * n - 2, m * n - 1], dtype=np.int32)   # one young clause, two trained-looking ones
    ostar_sub = ora.clause_outputs_subset(Xtr, ids)
    assert ostar_sub[1:].mean() > 0.3
    prev = gpu.prev_outputs()
    sel = torch.from_numpy(ids).long().to(prev.device)
    assert np.array_equal(bits_to_u8(prev[sel], q), ostar_sub)

    print(name, "frozen pass", flush=True)
    vhat = rng.integers(-hp["T"], hp["T"] + 1, size=(q, m)).astype(np.int32)
    B.tm_set_epoch(gpu.h, 2)
    gpu.feedback_step(dev_i32(gpu, vhat), 0, q)
    fired = ora.feedback_step_subset(Xtr, ytr, vhat, ostar_sub, 2, 0, q, ids)
    assert fired > 100
    st = gpu.get_ta_state()[sel].cpu().numpy().astype(np.int32) + 1
    assert np.array_equal(st, ora.state[ids])
    prev = gpu.prev_outputs()
    assert np.array_equal(bits_to_u8(prev[sel], q), ostar_sub)
    tally = gpu.tallies().cpu().numpy()
    sign = np.where(np.arange(n) % 2 == 1, 1, -1).astype(np.int32)
    for c in range(m):
        bits = bits_to_u8(prev[c * n:(c + 1) * n], q)
        assert np.array_equal(tally[:, c], sign @ bits.astype(np.int32))

    print(name, "inference", flush=True)
    ora.state[:] = gpu.get_ta_state().cpu().numpy().astype(np.int32) + 1
    Xd = dev_bits(gpu, Xte)
    ex = rng.integers(0, len(yte), size=24)
    Xs = np.ascontiguousarray(Xte[ex])
    sums = gpu.class_sums(Xd).cpu().numpy()
    assert np.array_equal(sums[ex], ora.class_sums(Xs))
    assert np.array_equal(sums, gpu.class_sums(Xd, lists=False).cpu().numpy())
    assert np.array_equal(gpu.predict(Xd).cpu().numpy()[ex], ora.predict(Xs))
    gpu.close()


def test_text_like_full_size_sampled_clauses(device):
    """The text-like workload at its full size and in the launch configuration the benchmark times (25,000
    documents x 10,000 features, 2 x 10,000 clauses: 10,000 workgroups per launch, 16 launches per pass).
    The machine's state is synthetic (a tiled pattern: untrained-looking clauses next to trained-looking
    ones), the oracle follows sampled clauses through the pre-calculation and a frozen-snapshot pass."""
    hp = dict(synth.WORKLOADS["text_like"])
    m, n, o, N = hp["m"], hp["n"], hp["o"], hp["N"]
    C, L, q = m * n, 2 * o, 25000
    Xtr, ytr, _, _ = synth.text_like(q, 8)
    rng = np.random.default_rng(3)
    print("text-like full size: state", flush=True)
    pattern = rng.integers(1, N + 1, size=(40, L)).astype(np.int32)            # states 1..2N; excluded everywhere ...
    pattern[:8] = rng.integers(1, 2 * N + 1, size=(8, L))                       # 8 untrained-looking rows
    for r in range(8, 40):                                                      # 32 rows with ten negated literals
        pattern[r, o + rng.integers(0, o, size=10)] = rng.integers(N + 1, 2 * N + 1, size=10)
    gpu = B.TsetlinMachine(seed=6, **hp)
    state_u8 = np.ascontiguousarray(np.tile((pattern - 1).astype(np.uint8), (C // 40, 1)))   # stored value = state - 1
    gpu.set_ta_state(torch.from_numpy(state_u8).to(gpu.dev))
    ids = np.array([3, 9, n - 1, n + 8, C - 2, C - 1], dtype=np.int32)          # both classes, both kinds, both polarities
    ora = O.Oracle(seed=6, init=False, **hp)
    ora.state[ids] = pattern[ids % 40]
    del state_u8

    print("text-like full size: bind", flush=True)
    gpu.bind_train(dev_bits(gpu, Xtr), dev_i32(gpu, ytr))
    assert B.tm_train_chunk(gpu.h) == 1664
    ostar_sub = ora.clause_outputs_subset(Xtr, ids)
    assert 0.05 < ostar_sub[1:].mean() < 0.999
    sel = torch.from_numpy(ids).long().to(gpu.dev)
    assert np.array_equal(bits_to_u8(gpu.prev_outputs()[sel], q), ostar_sub)

    print("text-like full size: frozen pass", flush=True)
    vhat = rng.integers(-hp["T"], hp["T"] + 1, size=(q, m)).astype(np.int32)    # synthetic snapshot
    B.tm_set_epoch(gpu.h, 4)
    gpu.counters()
    gpu.feedback_step(dev_i32(gpu, vhat), 0, q)
    fired = ora.feedback_step_subset(Xtr, ytr, vhat, ostar_sub, 4, 0, q, ids)
    assert fired > 1000
    st = gpu.get_ta_state()[sel].cpu().numpy().astype(np.int32) + 1
    assert np.array_equal(st, ora.state[ids])
    prev = gpu.prev_outputs()
    assert np.array_equal(bits_to_u8(prev[sel], q), ostar_sub)
    c = gpu.counters()
    assert c["pairs"] == q * C                     # counted on the device: 16 launches x 20,000 wavefronts
    # at any size: the tally is the signed sum of the stored outputs (checked on 4,000 examples)
    tally = gpu.tallies().cpu().numpy()
    sign = np.where(np.arange(n) % 2 == 1, 1, -1).astype(np.int32)
    for cls in range(m):
        bits = bits_to_u8(prev[cls * n:(cls + 1) * n, :125], 4000)
        assert np.array_equal(tally[:4000, cls], sign @ bits.astype(np.int32))
    gpu.close()
