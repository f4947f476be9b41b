"""CPU checks of the boundary: the built library loads and exports every
function the header declares; host-only entry points validate configurations."""
import ctypes
import os
import re

import pytest

from paper_2009_04861_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tm_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"tm_create", "tm_fit_epoch", "tm_predict", "tm_class_sums"} <= set(names)
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert set(B.EXPORTS) == set(names)


def test_binding_has_same_names():
    for n in declared_functions():
        if n in ("tm_strerror", "tm_last_hip_error"):
            continue
        assert callable(getattr(B, n)), n


def test_sizes_and_validation_are_host_only():
    cfg = B.make_config(10, 2000, 784, 128, 50, 10.0, 1)
    C, W = 20000, 50
    assert B.tm_state_bytes(cfg) == C * W * 32 + C * W * 4
    ws = B.tm_train_ws_bytes(cfg, 60000)
    qp = 60032
    # tallies + one bit per example per clause + transposed X + bit rows of X + literal lists
    # + gate lists + per-clause freshness ranges + launch order + counters/flag
    qw = ((60000 + 2047) // 2048) * 64

    def list_slots(q):
        # the lists are laid out per (class, share, wavefront of 8) in batches of 8 clauses, 64 clauses of a
        # share per round of batches: shares * 8 * ceil(clauses per share / 64) * 8 slots per class
        S, chunk = B.tm_eval_shares(cfg, q)
        return 10 * S * 8 * ((chunk + 63) // 64) * 8

    slots = list_slots(60000)
    assert C <= slots <= 1.25 * C
    need = (10 * qp * 4 + C * qp // 8 + 25 * qp * 4 + 1569 * qw * 4 + slots * 128 * 4 + slots * 4 + 10 * qp * 4
            + C * 16 + C * 4)
    assert ws >= need
    assert ws < 1.01 * need + 8192
    # inference workspace: literal rows of the examples + literal lists + their lengths
    iw = B.tm_infer_ws_bytes(cfg, 10000)
    slots = list_slots(10000)
    need_i = 1569 * ((10000 + 2047) // 2048) * 64 * 4 + slots * 128 * 4 + slots * 4
    assert need_i <= iw < need_i + 1024
    assert B.tm_infer_ws_bytes(cfg, 0) >= C * 128 * 4
    bad = [dict(m=1), dict(n=3), dict(n=0), dict(o=0), dict(N=0), dict(N=129), dict(T=0), dict(s=0.5)]
    for kw in bad:
        a = dict(m=2, n=4, o=8, N=10, T=5, s=3.0)
        a.update(kw)
        with pytest.raises(B.TMError) as e:
            B.tm_state_bytes(B.make_config(a["m"], a["n"], a["o"], a["N"], a["T"], a["s"], 1))
        assert e.value.code == B.TM_EINVAL
    with pytest.raises(B.TMError) as e:
        B.tm_state_bytes(B.make_config(2, 4, 20481, 10, 5, 3.0, 1))
    assert e.value.code == B.TM_ELIMIT
    assert B.strerror(B.TM_ESTATE).startswith("no training data")


def test_vote_counter_capacity_holds_for_every_split_of_a_class():
    """The literal-list evaluation gives a wavefront an eighth of a share of a class's clauses and
    counts their votes in 8 bit planes (at most 255).  Whatever the number of clauses, classes and
    examples, the split must keep a share at 2,032 clauses or fewer after all rounding, cover all
    clauses and stay a multiple of 16 (polarity alternates with the clause index)."""
    worst = 0
    shapes = [(2, 100), (2, 131067), (2, 200000), (10, 60000), (10, 10000), (5, 26624), (3, 2_100_000)]
    for m, q in shapes:
        ns = set(range(2, 70000, 2)) if (m, q) in ((2, 131067), (10, 60000)) else set()
        for S in range(1, 40):
            ns |= {n for n in range(S * 2030, S * 2050) if n % 2 == 0 and n >= 2}
        for n in sorted(ns):
            S, chunk = B.tm_eval_shares(B.make_config(m, n, 8, 128, 5, 3.0, 1), q)
            assert chunk % 16 == 0 and chunk <= 2032 and S * chunk >= n and (S - 1) * chunk < n, (m, q, n, S, chunk)
            worst = max(worst, chunk)
    assert worst == 2032      # the cap is reached (a share of 2,033 .. 2,040 clauses would round to 2,048)
