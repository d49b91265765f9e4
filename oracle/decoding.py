"""CPU oracle, part 2: greedy decoding and blockwise parallel decoding.

TEST INFRASTRUCTURE ONLY (see transformer.py).  The algorithms are written over an
abstract scoring function so that they can be driven by the Transformer of
transformer.py or by a scripted lookup table in the tests:

    score(prefix) -> z[k, V]     z[i-1, v] = score of  y_{j+i} = v  under
                                 p_i( . | y_{<=j}, x),  j = len(prefix)

Greedy decoding follows Section 2; predict / verify / accept follow Section 3; the
merged "verify step n + predict step n+1" loop follows Section 4; the relaxed
acceptance tests follow Sections 5.1-5.3.  argmax ties go to the lowest token id
(the paper does not say; numpy's argmax does this).

Bookkeeping the paper leaves to the reader: block row i' (1..k) of a step is the
model evaluated on the prefix  y_{<=j}, P_1..P_{i'};  the proposal P_{i+1} is
checked against head 1 of row i; row k is only needed to supply the proposals of
the next step when the whole block is accepted.

Termination (Section 2): stop after an accepted end-of-sequence token, or after
max_len tokens.  An accepted block is cut at (and including) its first EOS and at
max_len; Section 7.4 shows a final block ending in EOS.

Imposed schedules are not in the paper: they replace the outcome of the verify
test by a given k-hat per step so that throughput can be studied with untrained
heads; the tokens accepted are still P_1..P_k-hat and the next proposals are
still row k-hat of the table.
"""
from __future__ import annotations

import dataclasses
from typing import Callable, List, Optional, Sequence

import numpy as np

ScoreFn = Callable[[Sequence[int]], np.ndarray]


# ----------------------------------------------------------------------------- acceptance tests

def accept_exact(proposal: int, z1: np.ndarray) -> bool:
    """Section 3, Verify: the proposal is the scoring model's own argmax."""
    return proposal == int(np.argmax(z1))


def accept_top_n(n: int):
    """Section 5.1: the proposal lies within the n best-scoring tokens of p_1."""
    def test(proposal: int, z1: np.ndarray) -> bool:
        best = np.argsort(-z1, kind="stable")[:n]
        return proposal in best.tolist()
    return test


def accept_distance(eps: float):
    """Section 5.2 with d(u, v) = |u - v| on intensities."""
    def test(proposal: int, z1: np.ndarray) -> bool:
        return abs(proposal - int(np.argmax(z1))) <= eps
    return test


# ----------------------------------------------------------------------------- results

@dataclasses.dataclass
class Step:
    j: int                  # accepted length before the step
    proposals: List[int]    # P_1..P_k  (candidates for y_{j+1..j+k})
    table: np.ndarray       # A[i'-1, i-1] = argmax of head i at block row i'
    k_verified: int         # longest verified prefix (or the imposed value)
    k_hat: int              # tokens actually appended (after EOS / length cut)


@dataclasses.dataclass
class Decoded:
    tokens: List[int]
    steps: List[Step]
    invocations: int
    ended_by_eos: bool

    @property
    def block_sizes(self) -> List[int]:
        return [s.k_hat for s in self.steps]

    @property
    def mean_block(self) -> float:
        return len(self.tokens) / max(1, len(self.steps))


# ----------------------------------------------------------------------------- Section 2

def greedy_decode(score: ScoreFn, max_len: int, eos_id: int = -1) -> Decoded:
    y: List[int] = []
    calls = 0
    eos = False
    while len(y) < max_len:
        z = score(y)
        calls += 1
        tok = int(np.argmax(z[0]))
        y.append(tok)
        if eos_id >= 0 and tok == eos_id:
            eos = True
            break
    return Decoded(y, [], calls, eos)


# ----------------------------------------------------------------------------- Sections 3-5

def _cut(block: Sequence[int], k_hat: int, j: int, max_len: int, eos_id: int):
    """Cut an accepted block at its first EOS (inclusive) and at max_len."""
    if eos_id >= 0:
        for i in range(k_hat):
            if block[i] == eos_id:
                k_hat = i + 1
                break
    k_hat = min(k_hat, max_len - j)
    eos = eos_id >= 0 and eos_id in list(block[:k_hat])
    return k_hat, eos


def _verify(P, rows_z1, k, accept, min_block):
    """Largest k-hat with every P_{i} (2 <= i <= k-hat) accepted by p_1 at row i-1;
    k-hat >= 1 because P_1 is p_1's own argmax.  Section 5.3 forces k-hat >= min_block."""
    k_hat = 1
    while k_hat < k and accept(P[k_hat], rows_z1(k_hat)):
        k_hat += 1
    return min(k, max(k_hat, min_block))


def blockwise_decode(score: ScoreFn, k: int, max_len: int, eos_id: int = -1,
                     accept=accept_exact, min_block: int = 1,
                     schedule: Optional[Sequence[int]] = None,
                     block_score: Optional[Callable[[Sequence[int], Sequence[int]], np.ndarray]] = None,
                     ) -> Decoded:
    """Combined-model loop of Section 4: one model invocation per step plus one to start.

    ``block_score(prefix, P) -> z[k, k, V]`` may supply all k rows from one pass;
    by default row i' is ``score(prefix + P[:i'])``, one full evaluation per row.
    """
    y: List[int] = []
    j = 0
    steps: List[Step] = []
    z = score(y)                                    # the "+1" invocation: pure Predict
    invocations = 1
    P = [int(np.argmax(z[i])) for i in range(k)]
    eos = False
    while j < max_len and not eos:
        if block_score is not None:
            rows = np.asarray(block_score(y, P))
        else:
            rows = np.stack([score(y + P[:r]) for r in range(1, k + 1)])
        invocations += 1
        A = rows[:, :k, :].argmax(axis=-1)          # A[i'-1, i-1]
        if schedule is not None:
            k_ver = int(schedule[len(steps)])
            if not 1 <= k_ver <= k:
                raise ValueError("imposed accepted length outside 1..k")
        else:
            k_ver = _verify(P, lambda r: rows[r - 1, 0], k, accept, min_block)
        k_hat, eos = _cut(P, k_ver, j, max_len, eos_id)
        steps.append(Step(j, list(P), A.copy(), k_ver, k_hat))
        y.extend(P[:k_hat])                         # Accept
        j += k_hat
        P = [int(t) for t in A[k_hat - 1]]          # next Predict, already computed
    return Decoded(y, steps, invocations, eos)


def blockwise_decode_two_calls(score: ScoreFn, k: int, max_len: int, eos_id: int = -1,
                               accept=accept_exact, min_block: int = 1) -> Decoded:
    """The un-merged algorithm of Section 3: each step invokes the proposal models once
    (Predict) and the scoring model once (Verify)."""
    y: List[int] = []
    j = 0
    steps: List[Step] = []
    invocations = 0
    eos = False
    while j < max_len and not eos:
        z = score(y)                                # Predict with p_1..p_k
        invocations += 1
        P = [int(np.argmax(z[i])) for i in range(k)]
        z1 = [score(y + P[:r])[0] for r in range(1, k)]   # Verify: p_1 at the k-1 later positions
        invocations += 1
        k_ver = _verify(P, lambda r: z1[r - 1], k, accept, min_block)
        k_hat, eos = _cut(P, k_ver, j, max_len, eos_id)
        steps.append(Step(j, list(P), np.zeros((0, 0), dtype=np.int64), k_ver, k_hat))
        y.extend(P[:k_hat])
        j += k_hat
    return Decoded(y, steps, invocations, eos)
