"""Seeded activation-frequency traces for the tests of the estimator, balancer and cache manager.
Inputs only: nothing here evaluates the method.

The paper's traces come from real models on public suites; these stand in for them with the two
properties Sec. 3.2 builds on: a skewed (Zipf-like) popularity and its slow evolution over the
verification steps, with a few abrupt shifts."""
import numpy as np


def _popularity(rng, logit, drift, t, shift_every):
    logit += rng.normal(0, drift, size=logit.shape)
    if shift_every and t % shift_every == shift_every - 1:
        logit[...] = np.roll(logit, 3, axis=-1)
    p = np.exp(logit - logit.max(axis=-1, keepdims=True))
    return p / p.sum(axis=-1, keepdims=True)


def sampled_trace(rng, L, N, T, k, steps, drift, shift_every=11):
    """[steps, L, N] histograms of T tokens x k distinct experts drawn from the drifting popularity
    (sampling noise on top of the drift, as a router's picks would have)."""
    out = np.zeros((steps, L, N), dtype=np.int32)
    logit = rng.normal(0, 1.5, size=(L, N))
    for t in range(steps):
        p = _popularity(rng, logit, drift, t, shift_every)
        for l in range(L):
            for _ in range(T):
                out[t, l, rng.choice(N, size=k, replace=False, p=p[l])] += 1
    return out


def smooth_trace(rng, L, N, T, k, steps, drift, shift_every=0):
    """[steps, L, N] expected counts of the same process, rounded with a dither that is fixed per
    expert: a frequency moves only when the popularity does (no sampling noise)."""
    out = np.zeros((steps, L, N), dtype=np.int32)
    logit = rng.normal(0, 1.5, size=(L, N))
    dither = rng.random((L, N))
    for t in range(steps):
        p = _popularity(rng, logit, drift, t, shift_every)
        out[t] = np.minimum(T, np.floor(T * k * p + dither)).astype(np.int32)
    return out
