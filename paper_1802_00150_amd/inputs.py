"""Seeded synthetic inputs for the five benchmark configurations.

This module serves both the GPU tests / benchmark and the CPU oracle's tests.
It holds none of the method's arithmetic: only random matrices and vectors
with the shapes and value distributions of the paper's language-model
workloads (hidden size 300 with a 10K vocabulary; hidden size 1024, whose
recurrent matrix is 4096 x 1024), which stand in for trained weights and for
the PTB / Text8 data the paper evaluates on.  Everything is float32 numpy on
the host, drawn with numpy's PCG64 from `BASE_SEED + 1000 * config + trial`.
"""
import numpy as np

BASE_SEED = 180200150
STEPS = 35


def rng(config: int, trial: int = 0) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + 1000 * config + trial)


def normal(g: np.random.Generator, shape, std: float) -> np.ndarray:
    return (g.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def lstm_small(trial: int = 0, steps: int = STEPS):
    """Config 1: LSTM, embedding 300, hidden 300, batch 1, token inputs."""
    g = rng(1, trial)
    H = I = 300
    W = normal(g, (4 * H, I + H), 0.05)
    emb = normal(g, (10000, I), 0.1)
    tokens = g.integers(0, 10000, size=steps)
    return dict(I=I, H=H, B=1, k_w=2, k_a=2, T=2, Wx=np.ascontiguousarray(W[:, :I]),
                Wh=np.ascontiguousarray(W[:, I:]), emb=emb, tokens=tokens,
                xs=np.ascontiguousarray(emb[tokens][:, None, :]))


def gemv(trial: int = 0, batch: int = 1, m: int = 4096, n: int = 1024):
    """Config 2: W m x n ~ N(0, 0.02^2), x batch x n ~ N(0, 1)."""
    g = rng(2, trial)
    return dict(m=m, n=n, W=normal(g, (m, n), 0.02), x=normal(g, (batch, n), 1.0))


def lstm_large(trial: int = 0, steps: int = STEPS, B: int = 64, H: int = 1024, I: int = 1024):
    """Config 3: LSTM 1024/1024, batch 64, W3/A3."""
    g = rng(3, trial)
    W = normal(g, (4 * H, I + H), 0.02)
    xs = normal(g, (steps, B, I), 1.0)
    return dict(I=I, H=H, B=B, k_w=3, k_a=3, T=2, Wx=np.ascontiguousarray(W[:, :I]),
                Wh=np.ascontiguousarray(W[:, I:]), xs=xs)


def gru_proj(trial: int = 0, steps: int = STEPS, B: int = 256, H: int = 1024, I: int = 1024,
             V: int = 10000):
    """Config 4: GRU 1024/1024, batch 256, W2/A2, plus a V x H output projection (W2/A3)."""
    g = rng(4, trial)
    W = normal(g, (3 * H, I + H), 0.02)
    Ws = normal(g, (V, H), 0.02)
    xs = normal(g, (steps, B, I), 1.0)
    return dict(I=I, H=H, B=B, V=V, k_w=2, k_a=2, k_proj=3, T=2, Wx=np.ascontiguousarray(W[:, :I]),
                Wh=np.ascontiguousarray(W[:, I:]), Ws=Ws, xs=xs)


def heavy_tailed(trial: int = 0, rows: int = 16384, cols: int = 4096):
    """Config 5: N(0, 0.02^2) with each entry independently scaled x10 with probability 0.01."""
    g = rng(5, trial)
    W = normal(g, (rows, cols), 0.02)
    mask = g.random((rows, cols), dtype=np.float32) < np.float32(0.01)
    W[mask] *= np.float32(10.0)
    return W


def language_model(trial: int = 0, steps: int = STEPS, B: int = 1, H: int = 1024, E: int = 1024,
                   vocab: int = 42000, k: int = 2):
    """Full language-model step at the paper's large shape (hidden 1024, vocabulary 42000, whose
    output layer is 42000 x 1024): embedding table ~ N(0, 0.1^2), LSTM weights and output layer
    ~ N(0, 0.02^2), uniform token ids.  Config index 6 in the seed scheme."""
    g = rng(6, trial)
    W = normal(g, (4 * H, E + H), 0.02)
    emb = normal(g, (vocab, E), 0.1)
    Ws = normal(g, (vocab, H), 0.02)
    bs = normal(g, (vocab,), 0.1)
    ids = g.integers(0, vocab, size=(steps, B)).astype(np.int64)
    return dict(E=E, H=H, B=B, V=vocab, k_w=k, k_a=k, T=2, Wx=np.ascontiguousarray(W[:, :E]),
                Wh=np.ascontiguousarray(W[:, E:]), emb=emb, Ws=Ws, bs=bs, ids=ids)
