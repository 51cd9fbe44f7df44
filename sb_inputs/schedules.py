"""Seeded prompts and forced exit / acceptance schedules (inputs, not arithmetic)."""
from typing import Sequence, Tuple

import numpy as np


def make_prompt(vocab: int, n: int, seed: int) -> np.ndarray:
    """n token ids uniform in [0, vocab)."""
    g = np.random.Generator(np.random.Philox(key=[seed, 1]))
    return g.integers(0, vocab, size=n, dtype=np.int32)


def forced_exit_schedule(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """Per draft step: exit layer uniform in [lo, hi]."""
    g = np.random.Generator(np.random.Philox(key=[seed, 2]))
    return g.integers(lo, hi + 1, size=n, dtype=np.int32)


def accept_schedule(seed: int, n_rounds: int, w_max: int) -> np.ndarray:
    """Per round: number of emitted tokens uniform in [1, w_max]."""
    g = np.random.Generator(np.random.Philox(key=[seed, 3]))
    return g.integers(1, w_max + 1, size=n_rounds, dtype=np.int32)


def injection_schedule(greedy: Sequence[int], accepts: Sequence[int], w_max: int,
                       vocab: int) -> Tuple[np.ndarray, int]:
    """Draft-token overrides that make round r emit exactly accepts[r] tokens.

    greedy[0] is the token the prefill produced; greedy[1:] its greedy
    continuation (from a prior plain autoregressive run).  Every round is assumed
    to draft w_max tokens (all exits forced).  In a round that starts after
    greedy[e], drafts 1..a-1 are the true continuation, draft a (if a < w_max) is
    a deliberately wrong id, and later drafts are left to the exit head (-1).
    Returns (forced_draft[len = rounds*w_max], rounds used)."""
    G = np.asarray(greedy, dtype=np.int64)
    out = []
    e = 0
    rounds = 0
    for a in accepts:
        a = int(a)
        if e + a >= len(G):
            break
        row = [-1] * w_max
        for i in range(1, a):
            row[i - 1] = int(G[e + i])
        if a < w_max:
            row[a - 1] = int((G[e + a] + 1) % vocab)
        out += row
        e += a
        rounds += 1
    return np.asarray(out, dtype=np.int32), rounds
