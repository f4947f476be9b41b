"""Asynchronous training on the GPU against the oracle's synchronous training:
test accuracy on the noisy-XOR workload, 5 seeds, must agree within 1.0
percentage point.  Full asynchronous training is not reproducible run to run,
so this is a statistical check, not a bit-exact one."""
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
    acc_gpu, acc_cpu = [], []
    for seed in range(1, 6):
        print("accuracy seed", seed, flush=True)
        gpu = B.TsetlinMachine(seed=seed, **cfg)
        gpu.bind_train(dev_bits(gpu, Xtr), dev_i32(gpu, ytr))
        Xte_d = dev_bits(gpu, Xte)
        ora = O.Oracle(cfg["m"], cfg["n"], cfg["o"], cfg["N"], cfg["T"], cfg["s"], seed)
        ag, ac = [], []
        for ep in range(EPOCHS):
            gpu.fit_epoch()
            ora.sync_epoch(Xtr, ytr, ep)
            if ep >= EPOCHS - LAST:
                ag.append((gpu.predict(Xte_d).cpu().numpy() == yte).mean())
                ac.append((ora.predict(Xte) == yte).mean())
        acc_gpu.append(np.mean(ag))
        acc_cpu.append(np.mean(ac))
        gpu.close()
    g, c = 100 * np.mean(acc_gpu), 100 * np.mean(acc_cpu)
    print("mean test accuracy: gpu async %.2f %%, oracle sync %.2f %%" % (g, c), flush=True)
    assert g > 90.0
    assert abs(g - c) <= 1.0, (acc_gpu, acc_cpu)
