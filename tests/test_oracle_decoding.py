"""Pins for oracle/decoding.py that do not involve any Transformer: a scripted
lookup-table model drives predict / verify / accept (Sections 3-5, Figures 1-2,
Section 7.4) so that a mistake in the bookkeeping (off-by-one row, wrong head,
EOS handling, invocation count) fails here."""
import os

import numpy as np
import pytest

from oracle import (accept_distance, accept_exact, accept_top_n, blockwise_decode,
                    blockwise_decode_two_calls, greedy_decode)

GOLD = os.path.join(os.path.dirname(__file__), "golden")
V = 64
EOS = 2


def onehot(tokens, scores=None):
    z = np.zeros((len(tokens), V))
    for i, t in enumerate(tokens):
        z[i, t] = 1.0 if scores is None else scores[i]
    return z


def scripted(g, correct, k):
    """p_1 continues the fixed sequence g whenever the prefix is a prefix of g; head i
    (i >= 2) proposes the right token g_{j+i} iff i <= correct(j), else a wrong one.
    Prefixes that left g get junk that never equals g."""
    m = len(g)

    def score(prefix):
        j = len(prefix)
        out = []
        on_track = list(prefix) == list(g[:j])
        for i in range(1, k + 1):
            pos = j + i - 1                      # 0-based index into g of token y_{j+i}
            if on_track and pos < m and (i == 1 or i <= correct(j)):
                out.append(g[pos])
            else:
                true = g[pos] if pos < m else 0
                out.append(3 + (true + 7 + i) % (V - 3) if (3 + (true + 7 + i) % (V - 3)) != true
                           else 3 + (true + 8 + i) % (V - 3))
        return onehot(out)
    return score


def read_ints(path, key=None):
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = line.split()
        if key is None:
            return [int(p) for p in parts]
        if parts[0] == key:
            return [int(p) for p in parts[1:]]
    raise KeyError(key)


def test_section_7_4_block_sizes():
    sizes = read_ints(os.path.join(GOLD, "section7_4_block_sizes.txt"))
    assert sizes == [10, 5, 4, 10, 2, 3] and sum(sizes) == 34
    k = 10
    rng = np.random.default_rng(1)
    g = list(rng.integers(3, V, size=33)) + [EOS]
    starts = np.cumsum([0] + sizes[:-1])
    plan = {int(s): c for s, c in zip(starts, sizes)}
    dec = blockwise_decode(scripted(g, lambda j: plan.get(j, 1), k), k, max_len=100, eos_id=EOS)
    assert dec.tokens == g
    assert dec.block_sizes == sizes
    assert len(dec.steps) == 6 and dec.invocations == 7       # steps + 1 (Section 4)
    assert dec.ended_by_eos and dec.tokens[-1] == EOS
    two = blockwise_decode_two_calls(scripted(g, lambda j: plan.get(j, 1), k), k, 100, EOS)
    assert two.tokens == g and two.block_sizes == sizes and two.invocations == 12  # 2 per step


def test_figure_1_and_2_rows():
    f = os.path.join(GOLD, "figure2_rows.txt")
    prefix, P = read_ints(f, "prefix"), read_ints(f, "P")
    rows = [read_ints(f, "row%d" % r) for r in (1, 2, 3)]
    table = {tuple(prefix): P, tuple(prefix + P[:1]): rows[0],
             tuple(prefix + P[:2]): rows[1], tuple(prefix + P[:3]): rows[2]}

    def score(pfx):
        return onehot(table.get(tuple(pfx), [0, 0, 0]))

    # start the loop from the figure's prefix by wrapping the score function
    def shifted(pfx):
        return score(prefix + list(pfx))
    dec = blockwise_decode(shifted, 3, max_len=2, eos_id=-1)
    st = dec.steps[0]
    assert st.proposals == P
    assert st.k_verified == read_ints(f, "khat")[0] == 2
    assert dec.tokens == P[:2]
    assert st.table[1].tolist() == read_ints(f, "next")          # reused as the next Predict
    assert st.table.tolist() == rows


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
def test_all_correct_and_all_wrong(k):
    rng = np.random.default_rng(k)
    m = 23
    g = list(rng.integers(3, V, size=m))
    perfect = blockwise_decode(scripted(g, lambda j: k, k), k, max_len=m)
    assert perfect.tokens == g
    assert len(perfect.steps) == -(-m // k)                     # ceil(m / k) steps
    assert perfect.invocations == -(-m // k) + 1                # m/k + 1 (Section 4)
    worst = blockwise_decode(scripted(g, lambda j: 1, k), k, max_len=m)
    assert worst.tokens == g and len(worst.steps) == m
    assert all(s == 1 for s in worst.block_sizes)
    two = blockwise_decode_two_calls(scripted(g, lambda j: k, k), k, max_len=m)
    assert two.tokens == g and two.invocations == 2 * (-(-m // k))   # 2m/k (Section 4)
    gr = greedy_decode(scripted(g, lambda j: 1, k), max_len=m)
    assert gr.tokens == g and gr.invocations == m


def test_eos_inside_block_and_length_cut():
    k = 6
    g = [5, 6, 7, EOS, 9, 10, 11, 12]
    # every proposal right: the first block would be 6 tokens, but EOS is its 4th
    dec = blockwise_decode(scripted(g, lambda j: k, k), k, max_len=50, eos_id=EOS)
    assert dec.tokens == [5, 6, 7, EOS] and dec.block_sizes == [4] and dec.ended_by_eos
    assert dec.steps[0].k_verified == 6
    # no EOS id: fixed-length decoding (images), cut at max_len
    dec = blockwise_decode(scripted(g, lambda j: k, k), k, max_len=5, eos_id=-1)
    assert dec.tokens == g[:5] and dec.block_sizes == [5] and not dec.ended_by_eos
    # cut by length before the EOS is reached: not an EOS ending
    dec = blockwise_decode(scripted(g, lambda j: k, k), k, max_len=3, eos_id=EOS)
    assert dec.tokens == g[:3] and not dec.ended_by_eos
    assert greedy_decode(scripted(g, lambda j: 1, k), 50, EOS).tokens == [5, 6, 7, EOS]


def test_imposed_schedule():
    k = 4
    g = list(range(3, 3 + 20))
    # heads always wrong; the schedule decides how many proposals are appended
    score = scripted(g, lambda j: 1, k)
    ones = blockwise_decode(score, k, 20, schedule=[1] * 50)
    assert ones.tokens == g                                      # schedule == 1 is greedy
    sched = [2, 4, 1, 3, 4, 4, 2, 1, 1, 1]
    dec = blockwise_decode(score, k, 12, schedule=sched)
    assert dec.block_sizes[:3] == [2, 4, 1]
    assert sum(dec.block_sizes) == 12
    # accepted tokens are the proposals, whatever p_1 thinks of them
    pos = 0
    for st in dec.steps:
        assert dec.tokens[pos:pos + st.k_hat] == st.proposals[:st.k_hat]
        pos += st.k_hat
    # and each step's proposals are the table row of the previous accepted length
    for a, b in zip(dec.steps[:-1], dec.steps[1:]):
        assert b.proposals == a.table[a.k_hat - 1].tolist()
    with pytest.raises(ValueError):
        blockwise_decode(score, k, 12, schedule=[5])


def test_minimum_block_size():
    k = 4
    g = list(range(3, 3 + 16))
    score = scripted(g, lambda j: 1, k)
    fixed = blockwise_decode(score, k, 16, min_block=k)          # l = k: fixed-size blocks
    assert fixed.block_sizes == [4, 4, 4, 4]
    assert fixed.tokens != g and fixed.tokens[0] == g[0]
    assert blockwise_decode(score, k, 16, min_block=1).tokens == g
    two = blockwise_decode(score, k, 16, min_block=2)
    assert all(s >= 2 for s in two.block_sizes[:-1])


def test_top_n_and_distance():
    z1 = np.array([0.1, 0.9, 0.5, 0.5, 0.2])
    assert accept_exact(1, z1) and not accept_exact(2, z1)
    assert accept_top_n(1)(1, z1) and not accept_top_n(1)(2, z1)   # top-1 == exact
    assert accept_top_n(2)(2, z1) and not accept_top_n(2)(3, z1)   # tie: lower id first
    assert accept_top_n(3)(3, z1) and not accept_top_n(3)(4, z1)
    assert accept_distance(0)(1, z1) and not accept_distance(0)(2, z1)  # eps = 0 == exact
    assert accept_distance(2)(3, z1) and not accept_distance(2)(4, z1)
    assert accept_distance(2)(0, z1)

    # decoding with a relaxed test: proposals one intensity off are accepted with eps >= 1
    k = 3
    g = [10, 20, 30, 40, 50, 60]

    def score(prefix):
        j = len(prefix)
        toks = []
        for i in range(1, k + 1):
            pos = j + i - 1
            true = g[pos] if pos < len(g) else 0
            toks.append(true if i == 1 else true + 1)
        return onehot(toks)
    exact = blockwise_decode(score, k, 6)
    assert exact.tokens[0] == 10 and all(s == 1 for s in exact.block_sizes)
    loose = blockwise_decode(score, k, 6, accept=accept_distance(1))
    assert loose.block_sizes[0] == 3 and loose.tokens[:3] == [10, 21, 31]
    assert blockwise_decode(score, k, 6, accept=accept_distance(0)).tokens == exact.tokens
    assert blockwise_decode(score, k, 6, accept=accept_top_n(1)).tokens == exact.tokens


def test_k1_is_greedy_and_bounds():
    rng = np.random.default_rng(7)
    table = {}

    def score(prefix):                                           # arbitrary deterministic model
        key = tuple(prefix)
        if key not in table:
            table[key] = np.random.default_rng(hash(key) % (2 ** 32)).random((5, 6))
        return table[key]
    gr = greedy_decode(score, 12)
    for k in (1, 2, 3, 5):
        dec = blockwise_decode(lambda p: score(p)[:k], k, 12)
        assert dec.tokens == gr.tokens                           # same output as greedy (Section 3)
        assert all(1 <= s <= k for s in dec.block_sizes)
        assert sum(dec.block_sizes) == 12
        if k == 1:
            assert dec.block_sizes == [1] * 12 and dec.invocations == 13
        # k-hat from its definition: k sequential greedy calls, longest common prefix
        for st in dec.steps:
            pfx = gr.tokens[:st.j]
            cont = []
            for _ in range(k):
                cont.append(int(np.argmax(score(pfx + cont)[0])))
            lcp = 0
            while lcp < k and st.proposals[lcp] == cont[lcp]:
                lcp += 1
            assert lcp >= 1 and st.k_verified == lcp
