"""Asynchronous training on the GPU against the oracle: test accuracy over 5 seeds on three
workloads (mean over the last epochs, because single-epoch accuracy fluctuates).

The oracle gives the two ends of the range of tally staleness a legal asynchronous schedule can
have, both computed in the same run:
  c  standard synchronous training (every clause sees the exact vote sum);
  a  Algorithm 1 run sequentially with tallies as stale as they can get (every clause gates on the
     tallies as they stood at the start of the epoch).
The GPU's schedule lies between the two (how fresh its tallies are depends on the order in which
wavefronts happen to run).  Asserted: the GPU loses at most 1.0 percentage point against
synchronous training (the paper reports that asynchrony costs no noticeable accuracy), and it does
not score more than 1.0 pp above the better of the two oracle schedules.  The two-sided distance
|g - c| to synchronous training alone is printed with every run; on noisy XOR it exceeds 1.0 pp
because the stale schedule itself scores about 2 pp above the synchronous one there (the oracle's
own two figures differ by that much), so it is reported, not asserted.  Full asynchronous training
is not reproducible run to run: this is a statistical check, not a bit-exact one.

Workloads: noisy XOR at its full size; a reduced image-like machine (784 features, 10 x 40 clauses,
2,000 / 1,000 examples, 20 % pixel flips instead of 10 % so that the accuracies stay off the
ceiling); a reduced text-like machine (10,000 features, 2 x 16 clauses, 1,800 / 3,000 documents:
clauses of 10 register slots, two launches of the training kernel per epoch).  The oracle's runs
take most of the time and go to host threads, two per seed."""
import json
import os
import threading

import numpy as np
import pytest

from oracle import tm_oracle as O
from paper_2009_04861_amd import binding as B
from paper_2009_04861_amd import synth
from tests.helpers import dev_bits, dev_i32

pytestmark = pytest.mark.gpu

SEEDS = range(1, 6)


def oracle_accuracy(kind, hp, data, seed, epochs, last, out):
    Xtr, ytr, Xte, yte = data
    ora = O.Oracle(hp["m"], hp["n"], hp["o"], hp["N"], hp["T"], hp["s"], seed)
    if kind == "alg1":
        tally, ostar = ora.sync_tallies(Xtr)
    accs = []
    for ep in range(epochs):
        if kind == "sync":
            ora.sync_epoch(Xtr, ytr, ep)
        else:
            ora.feedback_step(Xtr, ytr, tally.copy(), tally, ostar, ep, 0, len(ytr))
        if ep >= epochs - last:
            accs.append(float((ora.predict(Xte) == yte).mean()))
    out[(kind, seed)] = 100.0 * float(np.mean(accs))


def gpu_accuracy(hp, data, seed, epochs, last):
    Xtr, ytr, Xte, yte = data
    gpu = B.TsetlinMachine(seed=seed, **hp)
    gpu.bind_train(dev_bits(gpu, Xtr), dev_i32(gpu, ytr))
    Xte_d = dev_bits(gpu, Xte)
    accs = []
    for ep in range(epochs):
        gpu.fit_epoch()
        if ep >= epochs - last:
            accs.append(float((gpu.predict(Xte_d).cpu().numpy() == yte).mean()))
    gpu.close()
    return 100.0 * float(np.mean(accs))


def compare(name, hp, data, epochs, last, floor, SEEDS=SEEDS):
    res = {}
    threads = [threading.Thread(target=oracle_accuracy, args=(kind, hp, data, seed, epochs, last, res))
               for seed in SEEDS for kind in ("sync", "alg1")]
    for t in threads:
        t.start()
    gs = []
    for seed in SEEDS:
        print("accuracy", name, "seed", seed, flush=True)
        gs.append(gpu_accuracy(hp, data, seed, epochs, last))
    for t in threads:
        t.join()
    cs = [res[("sync", s)] for s in SEEDS]
    as_ = [res[("alg1", s)] for s in SEEDS]
    for s, g1, c1, a1 in zip(SEEDS, gs, cs, as_):
        print("%s seed %d: gpu async %.2f %%, oracle synchronous %.2f %%, oracle Algorithm 1 (stale) %.2f %%"
              % (name, s, g1, c1, a1), flush=True)
    g, c, a = float(np.mean(gs)), float(np.mean(cs)), float(np.mean(as_))
    print("%s mean of %d seeds: gpu async %.2f %%, oracle synchronous %.2f %%, oracle Algorithm 1 (stale) %.2f %%; "
          "two-sided distance to synchronous training %.2f pp" % (name, len(gs), g, c, a, abs(g - c)), flush=True)
    log = os.environ.get("TM_ACCURACY_LOG")
    if log:
        with open(log, "a") as f:
            f.write(json.dumps({"workload": name, "gpu": gs, "sync": cs, "alg1": as_}) + "\n")
    assert g > floor
    assert g >= c - 1.0, (gs, cs)
    assert g <= max(c, a) + 1.0, (gs, cs, as_)


def test_noisy_xor_accuracy(device):
    compare("noisy_xor", synth.WORKLOADS["noisy_xor"], synth.noisy_xor(), epochs=200, last=50, floor=90.0)


def test_reduced_image_like_accuracy(device):
    hp = dict(m=10, n=40, o=784, N=128, T=10, s=5.0)
    compare("image_like_reduced", hp, synth.image_like(2000, 1000, flip=0.2), epochs=16, last=6, floor=90.0)


def test_reduced_text_like_accuracy(device):
    # T = 6 is below n/2, so the gate can close.  With T = 10 (above n/2, as in the full-size text-like
    # configuration) every asynchronous schedule of this tiny machine - the oracle's own sequential
    # Algorithm 1 included - trails synchronous training by 0.6 to 1.2 pp after 6 epochs (measured: synchronous
    # 93.8 %, tallies frozen per epoch 93.2 %, sequential Algorithm 1 92.9 %, GPU 92.6 %, 8 seeds): that is the
    # method on 16 clauses per class, not the implementation, and too close to the asserted margin to test with.
    hp = dict(m=2, n=16, o=10000, N=128, T=6, s=2.0)
    compare("text_like_reduced", hp, synth.text_like(1800, 3000), epochs=6, last=4, floor=85.0)
