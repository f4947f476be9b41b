"""tm_predict_static (the entry point for callers that cannot allocate: its workspace is a static
device array inside the library) against tm_predict_ws, through the C boundary, bit for bit: two
calls in a row on the same GPU, the second with a smaller input, so that whatever the first call
left in the shared array must not show in the second."""
import numpy as np
import pytest
import torch

from oracle import tm_oracle as O
from paper_2009_04861_amd import binding as B
from tests.helpers import dev_bits, push_state, sparse_random_state

pytestmark = pytest.mark.gpu


def predict_both(gpu, Xd):
    want = gpu.predict(Xd, lists=True)                    # tm_predict_ws, caller-owned workspace
    got = torch.full((Xd.shape[0],), -7, dtype=torch.int32, device=gpu.dev)
    with torch.cuda.device(gpu.dev):
        B.tm_predict_static(gpu.h, Xd, got)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


@pytest.mark.parametrize("shape", [(10, 200, 784, 128, 50, 10.0, 9000, 2500),     # several workgroups per class
                                   (3, 6, 37, 20, 4, 3.0, 5000, 70),              # one workgroup per class
                                   (2, 40, 4200, 128, 30, 4.0, 3000, 2049)])
def test_static_scratch_prediction_matches_workspace_prediction(shape, device):
    m, n, o, N, T, s, q1, q2 = shape
    print("no-alloc prediction", shape, flush=True)
    rng = np.random.default_rng(o)
    ora = O.Oracle(m, n, o, N, T, s, 3)
    gpu = B.TsetlinMachine(m, n, o, N, T, s, 3)
    ora.state[:] = sparse_random_state(rng, ora.C, ora.L, N, 2.0 / o)
    ora.state[1] = rng.integers(1, 2 * N + 1, size=ora.L)     # an untrained clause among them
    push_state(gpu, ora.state)
    X1 = (rng.random((q1, o)) < 0.4).astype(np.uint8)
    X2 = (rng.random((q2, o)) < 0.4).astype(np.uint8)
    got1, want1 = predict_both(gpu, dev_bits(gpu, X1))
    got2, want2 = predict_both(gpu, dev_bits(gpu, X2))        # smaller input right after the larger one
    assert np.array_equal(got1, want1)
    assert np.array_equal(got2, want2)
    assert len(np.unique(want1)) > 1
    # and both agree with the oracle on a sample
    ex = rng.integers(0, q2, size=40)
    assert np.array_equal(got2[ex], ora.predict(np.ascontiguousarray(X2[ex])))
    gpu.close()


def test_static_scratch_limit_and_empty_input(device):
    gpu = B.TsetlinMachine(10, 2000, 784, 128, 50, 10.0, 1)
    q_fit = 10000                      # the benchmark's test set: 2 MB of literal rows + 10 MB of lists
    X = torch.zeros((q_fit, gpu.Wf), dtype=torch.int32, device=gpu.dev)
    pred = torch.empty(q_fit, dtype=torch.int32, device=gpu.dev)
    B.tm_predict_static(gpu.h, X, pred)
    big = torch.zeros((200000, gpu.Wf), dtype=torch.int32, device=gpu.dev)     # 39 MB of literal rows: over the limit
    with pytest.raises(B.TMError) as e:
        B.tm_predict_static(gpu.h, big, torch.empty(200000, dtype=torch.int32, device=gpu.dev))
    assert e.value.code == B.TM_ELIMIT
    B.tm_predict_static(gpu.h, X[:0], pred[:0])                                # q = 0 is a no-op
    torch.cuda.synchronize()
    gpu.close()
