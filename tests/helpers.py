"""Shared helpers of the GPU parity tests: data conversion between the oracle's
unpacked arrays and the library's packed device tensors."""
import numpy as np
import torch

from oracle import tm_oracle as O
from paper_2009_04861_amd import binding as B
from paper_2009_04861_amd import synth


def make_pair(m, n, o, N, T, s, seed, boost=False):
    """An oracle and a GPU machine with the same configuration."""
    return O.Oracle(m, n, o, N, T, s, seed, boost=boost), B.TsetlinMachine(m, n, o, N, T, s, seed, boost=boost)


def dev_bits(gpu, X_u8):
    return gpu.to_device_bits(synth.pack_features(X_u8))


def dev_i32(gpu, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(gpu.dev)


def gpu_state_as_oracle(gpu):
    """uint8 (state-1) [C][L] -> int32 state 1..2N."""
    return gpu.get_ta_state().cpu().numpy().astype(np.int32) + 1


def push_state(gpu, state):
    gpu.set_ta_state(torch.from_numpy((state - 1).astype(np.uint8)).to(gpu.dev))


def bits_to_u8(bits_i32, q):
    """device int32 [C][ceil(q/32)] -> numpy uint8 [C][q]."""
    w = bits_i32.cpu().numpy().view(np.uint32)
    return synth.unpack_bits(w, q)


def sparse_random_state(rng, C, L, N, p_include):
    """Random TA states with a given fraction of included literals, so that
    clause outputs are a mix of 0 and 1."""
    inc = rng.random((C, L)) < p_include
    lo = rng.integers(1, N + 1, size=(C, L))
    hi = rng.integers(N + 1, 2 * N + 1, size=(C, L))
    return np.where(inc, hi, lo).astype(np.int32)
