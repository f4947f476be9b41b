"""Seeded synthetic workloads and bit packing.

This module holds input generation only: no clause evaluation, no voting, no
feedback.  It is the one module both the CPU oracle's tests and the HIP path's
tests draw their inputs from, so that both sides see identical data.

Every generator is deterministic in its seed (numpy PCG64) and returns
unpacked features X uint8 [q][o] in {0,1} and labels y int32 [q].

The generators stand in for the paper's datasets, which are not reproduced
here: a noisy XOR (the paper's worked learning example, Section 2.2), an
image-like 28x28 task, a sparse bag-of-words task (the paper's text workloads
have thousands of clauses over up to ~100k sparse features, Section 4) and a
large planted-conjunction stress case, and a tabular regression task with
thermometer-coded columns (the paper's regression runs, Section 4.1).
"""
import numpy as np

DATA_SEED_BASE = 20090486


def pack_features(X):
    """uint8 [q][o] -> uint32 [q][ceil(o/32)], feature k at word k>>5, bit k&31
    (least significant bit first); padding bits are 0."""
    X = np.ascontiguousarray(X, dtype=np.uint8)
    q, o = X.shape
    Wf = (o + 31) // 32
    pad = np.zeros((q, Wf * 32), dtype=np.uint8)
    pad[:, :o] = X
    b = np.packbits(pad.reshape(q, Wf, 32), axis=2, bitorder="little")  # [q][Wf][4] bytes
    return np.ascontiguousarray(b).view("<u4").reshape(q, Wf).astype(np.uint32)


def unpack_bits(words, nbits):
    """uint32 [r][w] -> uint8 [r][nbits] (inverse of the packing above)."""
    words = np.ascontiguousarray(words, dtype="<u4")
    r = words.shape[0]
    b = np.unpackbits(words.view(np.uint8).reshape(r, -1), axis=1, bitorder="little")
    return np.ascontiguousarray(b[:, :nbits])


def noisy_xor(q_train=5000, q_test=5000, o=12, noise=0.4, seed=DATA_SEED_BASE + 1):
    """y = x0 XOR x1, remaining features uniform noise; training labels flipped
    with probability `noise`, test labels clean."""
    rng = np.random.default_rng(seed)
    Xtr = rng.integers(0, 2, size=(q_train, o), dtype=np.uint8)
    Xte = rng.integers(0, 2, size=(q_test, o), dtype=np.uint8)
    ytr = (Xtr[:, 0] ^ Xtr[:, 1]).astype(np.int32)
    yte = (Xte[:, 0] ^ Xte[:, 1]).astype(np.int32)
    flip = rng.random(q_train) < noise
    ytr = np.where(flip, 1 - ytr, ytr).astype(np.int32)
    return Xtr, ytr, Xte, yte


def _stroke_prototypes(rng, classes, side):
    protos = np.zeros((classes, side, side), dtype=np.uint8)
    yy, xx = np.mgrid[0:side, 0:side]
    for c in range(classes):
        for _ in range(int(rng.integers(3, 6))):
            x0, y0, x1, y1 = rng.uniform(2, side - 3, size=4)
            thick = rng.uniform(0.9, 1.6)
            dx, dy = x1 - x0, y1 - y0
            ln2 = dx * dx + dy * dy + 1e-9
            t = np.clip(((xx - x0) * dx + (yy - y0) * dy) / ln2, 0.0, 1.0)
            d2 = (xx - (x0 + t * dx)) ** 2 + (yy - (y0 + t * dy)) ** 2
            protos[c] |= (d2 <= thick * thick).astype(np.uint8)
    return protos.reshape(classes, side * side)


def image_like(q_train=60000, q_test=10000, classes=10, side=28, flip=0.10,
               seed=DATA_SEED_BASE + 2):
    """Thresholded side x side images: one random thick-stroke prototype per
    class, every pixel flipped independently with probability `flip`."""
    rng = np.random.default_rng(seed)
    protos = _stroke_prototypes(rng, classes, side)

    def draw(q):
        y = rng.integers(0, classes, size=q).astype(np.int32)
        X = protos[y] ^ (rng.random((q, side * side)) < flip).astype(np.uint8)
        return np.ascontiguousarray(X, dtype=np.uint8), y

    Xtr, ytr = draw(q_train)
    Xte, yte = draw(q_test)
    return Xtr, ytr, Xte, yte


def text_like(q_train=25000, q_test=25000, vocab=10000, classes=2, words_per_doc=150.0,
              zipf=1.1, markers=200, boost=3.0, seed=DATA_SEED_BASE + 3):
    """Sparse bag-of-words: word of rank r present with p_r ~ r^-zipf scaled to
    `words_per_doc` expected words; `markers` words per class get boost*p_r in
    documents of that class."""
    rng = np.random.default_rng(seed)
    ranks = np.arange(1, vocab + 1, dtype=np.float64)
    base = ranks ** (-zipf)
    lo, hi = 0.0, 1e9
    for _ in range(200):  # scale so that sum(min(1, a*base)) = words_per_doc
        a = 0.5 * (lo + hi)
        if np.minimum(1.0, a * base).sum() > words_per_doc:
            hi = a
        else:
            lo = a
    p = np.minimum(1.0, a * base)
    lo_r, hi_r = min(50, vocab // 4), min(5000, vocab)
    pool = rng.permutation(np.arange(lo_r, hi_r))
    per = min(markers, len(pool) // classes)
    pc = np.tile(p, (classes, 1))
    for c in range(classes):
        idx = pool[c * per:(c + 1) * per]
        pc[c, idx] = np.minimum(1.0, boost * p[idx])

    def draw(q):
        y = rng.integers(0, classes, size=q).astype(np.int32)
        X = np.empty((q, vocab), dtype=np.uint8)
        step = 2048
        for a0 in range(0, q, step):
            yy = y[a0:a0 + step]
            X[a0:a0 + step] = rng.random((len(yy), vocab), dtype=np.float32) < pc[yy].astype(np.float32)
        return X, y

    Xtr, ytr = draw(q_train)
    Xte, yte = draw(q_test)
    return Xtr, ytr, Xte, yte


def planted_conjunctions(q=200000, o=20000, density=0.05, planted=64, width=3,
                         seed=DATA_SEED_BASE + 5):
    """Bernoulli(density) features; label = [number of satisfied planted
    `width`-literal conjunctions >= its empirical median] (a fixed majority of
    the planted set would give a constant label at low density)."""
    rng = np.random.default_rng(seed)
    feats = rng.integers(0, o, size=(planted, width))
    pol = rng.integers(0, 2, size=(planted, width)).astype(np.uint8)  # 1: plain, 0: negated
    X = np.empty((q, o), dtype=np.uint8)
    sat = np.zeros(q, dtype=np.int32)
    step = 4096
    for a0 in range(0, q, step):
        blk = (rng.random((min(step, q - a0), o), dtype=np.float32) < density).astype(np.uint8)
        X[a0:a0 + step] = blk
        lit = blk[:, feats] == pol[None, :, :]
        sat[a0:a0 + step] = lit.all(axis=2).sum(axis=1)
    theta = np.median(sat)
    y = (sat > theta).astype(np.int32) if (sat >= theta).mean() > 0.75 else (sat >= theta).astype(np.int32)
    return X, y


def regression_like(q_train=13911, q_test=3478, features=16, thresholds=16, T=1280, noise=0.03,
                    seed=DATA_SEED_BASE + 6):
    """Tabular regression stand-in (the paper's regression runs use a 16-feature table of
    17,389 rows split 80/20, T = n = 1280, s = 1.5): `features` uniform(0,1) columns, each
    thermometer-coded with `thresholds` evenly spaced thresholds (o = features*thresholds
    bits); the continuous target is a fixed smooth non-linear function of six columns plus
    Gaussian noise, clipped to [0,1] and scaled to integers 0..T.  Test targets are noise-free."""
    rng = np.random.default_rng(seed)
    cuts = (np.arange(thresholds, dtype=np.float64) + 0.5) / thresholds

    def draw(q, sigma):
        u = rng.random((q, features))
        f = (0.40 * np.exp(-((u[:, 0] - 0.55) / 0.18) ** 2) + 0.25 * u[:, 1]
             + 0.20 * (u[:, 2] > 0.5) * u[:, 3] + 0.15 * u[:, 4] * u[:, 5])
        f = np.clip(f + sigma * rng.standard_normal(q), 0.0, 1.0)
        X = (u[:, :, None] > cuts[None, None, :]).reshape(q, features * thresholds).astype(np.uint8)
        return np.ascontiguousarray(X), np.rint(f * T).astype(np.int32)

    Xtr, ytr = draw(q_train, noise)
    Xte, yte = draw(q_test, 0.0)
    return Xtr, ytr, Xte, yte


WORKLOADS = {
    # name: model hyper-parameters of the five benchmark configurations
    "noisy_xor": dict(m=2, n=10, o=12, N=100, T=15, s=3.9),
    "image_like": dict(m=10, n=2000, o=784, N=128, T=50, s=10.0),
    "text_like": dict(m=2, n=10000, o=10000, N=128, T=8000, s=2.0),
    "stress": dict(m=2, n=32768, o=20000, N=128, T=20000, s=5.0),
    # regression mode: one bank of clauses, integer targets 0..T
    "regression_like": dict(m=1, n=1280, o=256, N=128, T=1280, s=1.5, regression=True),
}
