"""Pins of the fine-tuning-mask oracle (Section 4.4) against the paper and against an
independent construction of the inference-time pattern (Section 4.3.2)."""
import os

import numpy as np
import pytest

from oracle import finetune_mask as F

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden():
    out = {}
    with open(os.path.join(GOLDEN, "alg2_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                out[key] = [int(v) for v in vals]
    return out


def _cases():
    rng = np.random.default_rng(5)
    cases = [(10, [3, 3, 3], [3, 3, 3], 7), (0, [1], [1], 1), (4, [2, 1, 3], [0, 5, 2], 5)]
    for _ in range(6):
        n = int(rng.integers(1, 6))
        kmax = int(rng.integers(1, 7))
        cases.append((int(rng.integers(0, 9)), [int(x) for x in rng.integers(1, 4, n)],
                      [int(x) for x in rng.integers(0, kmax + 1, n)], kmax))
    return cases


def test_positions_match_the_papers_worked_example():
    g = _golden()
    pos = F.finetune_position_ids(g["prompt_len"][0], g["attr_lens"], [g["steps"][0]] * 3, g["k_max"][0])
    kind, attr, k = F.finetune_tokens(g["prompt_len"][0], g["attr_lens"], [g["steps"][0]] * 3)
    for n in range(3):
        a = pos[(kind == F.KIND_ATTR) & (attr == n)]
        assert a[-1] == g["decode_from"][n]
        assert list(pos[(kind == F.KIND_VALUE) & (attr == n)]) == g[f"value_pos_attr{n}"]
    assert list(pos[:10]) == list(range(10))


@pytest.mark.parametrize("case", _cases())
def test_positions_closed_form_and_order(case):
    plen, al, vl, kmax = case
    pos = F.finetune_position_ids(plen, al, vl, kmax)
    kind, attr, k = F.finetune_tokens(plen, al, vl)
    for i in range(len(pos)):
        if kind[i] == F.KIND_PROMPT:
            assert pos[i] == i
        else:
            n = attr[i]
            end = plen + sum(al[:n + 1]) - 1 + n * kmax  # position of the attribute's last token
            if kind[i] == F.KIND_VALUE:
                assert pos[i] == end + k[i]
            else:
                first = i - int(np.sum((kind[:i] == F.KIND_ATTR) & (attr[:i] == n)))
                assert pos[i] == end - (al[n] - 1) + (i - first)
    # the regular training order is the position-ID order: strictly increasing
    assert np.all(np.diff(pos) > 0)


@pytest.mark.parametrize("case", _cases())
def test_mask_set_construction_and_row_sums(case):
    plen, al, vl, kmax = case
    m = F.finetune_mask(plen, al, vl)
    kind, attr, k = F.finetune_tokens(plen, al, vl)
    s = len(kind)
    assert m.shape == (s, s) and np.array_equal(m, np.tril(m))  # never beyond causal
    for qi in range(s):
        if kind[qi] == F.KIND_PROMPT:
            want = set(range(qi + 1))
        elif kind[qi] == F.KIND_ATTR:
            want = {i for i in range(qi + 1) if kind[i] != F.KIND_VALUE}
            assert m[qi].sum() == plen + sum(al[:attr[qi]]) + (qi - np.nonzero((kind == F.KIND_ATTR) & (attr == attr[qi]))[0][0]) + 1
        else:
            n, kk = attr[qi], k[qi]
            want = {i for i in range(s) if kind[i] == F.KIND_PROMPT}
            want |= {i for i in range(s) if kind[i] == F.KIND_ATTR and attr[i] <= n}
            want |= {i for i in range(s) if kind[i] == F.KIND_VALUE and attr[i] < n and k[i] <= kk}
            want |= {i for i in range(s) if kind[i] == F.KIND_VALUE and attr[i] == n and k[i] <= kk}
            assert m[qi].sum() == plen + sum(al[:n + 1]) + sum(min(kk, vl[j]) for j in range(n)) + kk
        assert set(np.nonzero(m[qi])[0]) == want


@pytest.mark.parametrize("case", _cases())
def test_pattern_equals_the_inference_pattern(case):
    """Section 4.4's claim (and the caption of its mask figure): the fine-tuning mask replicates
    what a token can see at inference.  The inference side is built from Section 4.3.2 alone:
    memory order [p, a_1..a_N, values of step 1 (attribute order), values of step 2, ...]; a
    key is visible iff it is in memory no later than the query and its position ID is not
    larger.  Prompt and attribute tokens are queries of the first step only, when no value
    token exists yet."""
    plen, al, vl, kmax = case
    kind, attr, k = F.finetune_tokens(plen, al, vl)
    pos = F.finetune_position_ids(plen, al, vl, kmax)
    s = len(kind)
    # memory index at inference: prefill tokens in skeleton order, then values step by step
    skeleton = [i for i in range(s) if kind[i] != F.KIND_VALUE]
    mem_order = skeleton + sorted((i for i in range(s) if kind[i] == F.KIND_VALUE),
                                  key=lambda i: (k[i], attr[i]))
    mem_index = {tok: j for j, tok in enumerate(mem_order)}
    m_inf = np.zeros((s, s), dtype=np.uint8)
    for qi in range(s):
        for ki in range(s):
            in_memory = mem_index[ki] <= mem_index[qi]
            m_inf[qi, ki] = 1 if (in_memory and pos[ki] <= pos[qi]) else 0
    assert np.array_equal(F.finetune_mask(plen, al, vl), m_inf)


def test_planted_mistakes_break_the_equivalence():
    plen, al, vl, kmax = 3, [2, 1, 2], [3, 2, 3], 4
    good = F.finetune_mask(plen, al, vl)
    kind, attr, k = F.finetune_tokens(plen, al, vl)
    # (a) forgetting the "not generated yet" rule = plain causal; (b) blocking k' >= k
    causal = np.tril(np.ones_like(good))
    assert not np.array_equal(good, causal)
    q = int(np.nonzero((kind == F.KIND_VALUE) & (attr == 1) & (k == 1))[0][0])
    same_k = int(np.nonzero((kind == F.KIND_VALUE) & (attr == 0) & (k == 1))[0][0])
    later_k = int(np.nonzero((kind == F.KIND_VALUE) & (attr == 0) & (k == 2))[0][0])
    assert good[q, same_k] == 1 and good[q, later_k] == 0
    a1 = int(np.nonzero((kind == F.KIND_ATTR) & (attr == 1))[0][0])
    assert good[a1, same_k] == 0  # attribute tokens never see values
