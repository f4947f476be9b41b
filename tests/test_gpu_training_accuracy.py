"""Asynchronous training on the GPU against the oracle, test accuracy on the
noisy-XOR workload over 5 seeds (mean over the last 50 of 200 epochs, because
40 % label noise makes single-epoch accuracy fluctuate).

The oracle gives the two ends of the range of tally staleness a legal
asynchronous schedule can have, both computed in the same run:
  - standard synchronous training (every clause sees the exact vote sum);
  - Algorithm 1 run sequentially with tallies as stale as they can get
    (every clause gates on the tallies as they stood at the start of the epoch).
On this workload the stale end scores about 2 pp ABOVE the synchronous end in
the oracle itself (99.2 % against 97.3 %), so accuracy depends on the schedule
by more than the 1.0 pp the target allows between implementations.  The GPU's
schedule lies between the two ends (how fresh its tallies are depends on the
order in which wavefronts happen to run), so the check is: the GPU loses at most
1.0 pp against synchronous training (the paper reports that asynchrony costs no
noticeable accuracy) and lies within 1.0 pp of the interval spanned by the two
oracle schedules.  Full asynchronous training is not
reproducible run to run, so this is a statistical check, not a bit-exact one."""
import numpy as np
import pytest

from oracle import tm_oracle as O
from paper_2009_04861_amd import binding as B
from paper_2009_04861_amd import synth
from tests.helpers import dev_bits, dev_i32

pytestmark = pytest.mark.gpu

EPOCHS, LAST = 200, 50


def test_noisy_xor_accuracy_within_one_point(device):
    Xtr, ytr, Xte, yte = synth.noisy_xor()
    cfg = synth.WORKLOADS["noisy_xor"]
    acc_gpu, acc_cpu, acc_alg1 = [], [], []
    for seed in range(1, 6):
        print("accuracy seed", seed, flush=True)
        gpu = B.TsetlinMachine(seed=seed, **cfg)
        gpu.bind_train(dev_bits(gpu, Xtr), dev_i32(gpu, ytr))
        Xte_d = dev_bits(gpu, Xte)
        ora = O.Oracle(cfg["m"], cfg["n"], cfg["o"], cfg["N"], cfg["T"], cfg["s"], seed)
        alg1 = O.Oracle(cfg["m"], cfg["n"], cfg["o"], cfg["N"], cfg["T"], cfg["s"], seed)
        tally, ostar = alg1.sync_tallies(Xtr)
        ag, ac, aa = [], [], []
        for ep in range(EPOCHS):
            gpu.fit_epoch()
            ora.sync_epoch(Xtr, ytr, ep)
            alg1.feedback_step(Xtr, ytr, tally.copy(), tally, ostar, ep, 0, len(ytr))
            if ep >= EPOCHS - LAST:
                ag.append((gpu.predict(Xte_d).cpu().numpy() == yte).mean())
                ac.append((ora.predict(Xte) == yte).mean())
                aa.append((alg1.predict(Xte) == yte).mean())
        acc_gpu.append(np.mean(ag))
        acc_cpu.append(np.mean(ac))
        acc_alg1.append(np.mean(aa))
        gpu.close()
    g, c, a = 100 * np.mean(acc_gpu), 100 * np.mean(acc_cpu), 100 * np.mean(acc_alg1)
    print("mean test accuracy: gpu async %.2f %%, oracle synchronous %.2f %%, oracle Algorithm 1 %.2f %%"
          % (g, c, a), flush=True)
    assert g > 90.0
    assert g >= c - 1.0, (acc_gpu, acc_cpu)
    assert min(c, a) - 1.0 <= g <= max(c, a) + 1.0, (acc_gpu, acc_cpu, acc_alg1)
