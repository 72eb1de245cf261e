"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each pin is chosen so that a
plausible mistake in the oracle (dropped term, wrong sign or index, transposed
operand, off-by-one in positions or mask) makes at least one of them fail.
"""
import os

import numpy as np
import pytest
import torch

from oracle import brute_force
from oracle import hpd_oracle as O
from paper_2604_26209_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def _values(wl, seed_off, shape):
    return W.normal_values(shape, wl.value_seed * 1000 + seed_off, "cpu", "f32").numpy()


def _run_oracle(wl, dtype=np.float32, pos_mode="contig", attr_len=None, mask_mode="block"):
    """Run all steps; returns (oracle, inputs, per-step result dicts)."""
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len,
                      wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new,
                      pos_mode=pos_mode, attr_len=attr_len, dtype=dtype, mask_mode=mask_mode)
    # (under the literal mask the prefix also holds the skeleton tokens)
    kp = _values(wl, 1, (orc.n_prefix_tokens, wl.n_kv_heads, wl.head_dim))
    vp = _values(wl, 2, (orc.n_prefix_tokens, wl.n_kv_heads, wl.head_dim))
    orc.prefill(kp, vp)
    steps, inputs = [], {"kp": kp, "vp": vp, "q": [], "k": [], "v": []}
    for t in range(wl.max_new):
        n_live = int((wl.branch_len > t).sum())
        q = _values(wl, 10 + 3 * t, (n_live, wl.n_q_heads, wl.head_dim))
        k = _values(wl, 11 + 3 * t, (n_live, wl.n_kv_heads, wl.head_dim))
        v = _values(wl, 12 + 3 * t, (n_live, wl.n_kv_heads, wl.head_dim))
        inputs["q"].append(q), inputs["k"].append(k), inputs["v"].append(v)
        steps.append(orc.step(t, q, k, v))
    return orc, inputs, steps


# ---------------------------------------------------------------------------
# Position IDs
# ---------------------------------------------------------------------------
def test_alg2_worked_example_from_paper():
    g = _read_golden("alg2_worked_example.txt")
    pos_id, end_index = O.alg2_position_ids(g["prompt_len"][0], g["attr_lens"], g["k_max"][0])
    assert [int(pos_id[e]) for e in end_index] == g["decode_from"]
    assert [O.value_position(pos_id, end_index, n, 1) for n in range(3)] == g["first_value_pos"]
    for n in range(3):
        got = [O.value_position(pos_id, end_index, n, k) for k in range(1, g["steps"][0] + 1)]
        assert got == g[f"value_pos_attr{n}"]
    # the prompt itself keeps ordinary positions
    assert list(pos_id[:10]) == list(range(10))


@pytest.mark.parametrize("seed", range(5))
def test_alg2_closed_form_and_no_collisions(seed):
    rng = np.random.default_rng(seed)
    plen = int(rng.integers(0, 30))
    attr = [int(x) for x in rng.integers(1, 6, size=int(rng.integers(1, 7)))]
    kmax = int(rng.integers(1, 9))
    pos_id, end_index = O.alg2_position_ids(plen, attr, kmax)
    used = set(int(x) for x in pos_id)
    assert len(used) == len(pos_id)  # skeleton positions are distinct
    for n in range(len(attr)):
        # closed form: |p| + sum_{m<=n} A_m - 1 + n*K_max  (n 0-based)
        assert int(pos_id[end_index[n]]) == plen + sum(attr[:n + 1]) - 1 + n * kmax
        for k in range(1, kmax + 1):  # a value of <= K_max tokens fits its gap exactly
            p = O.value_position(pos_id, end_index, n, k)
            assert p not in used
            used.add(p)
    # strictly increasing along s: ordering by position ID keeps attribute order
    assert np.all(np.diff(pos_id) > 0)


def test_contig_positions_closed_form():
    wl = W.random_workload(7, t=5, p=4)
    orc, _, steps = _run_oracle(wl)
    doc_of_branch = np.repeat(np.arange(wl.n_docs), np.diff(wl.branch_ptr))
    prompt_of_doc = np.repeat(np.arange(wl.n_prompts), np.diff(wl.doc_ptr))
    for t, res in enumerate(steps):
        live = np.nonzero(wl.branch_len > t)[0]
        d = doc_of_branch[live]
        expect = wl.header_len[prompt_of_doc[d]] + wl.doc_len[d] + t
        assert np.array_equal(res["pos"], expect)
        assert np.array_equal(res["slot"], live * wl.max_new + t)
        assert np.array_equal(orc.positions(t), expect)


def test_paper_gap_positions_match_alg2_per_prompt():
    wl = W.random_workload(3, t=4, p=2, ragged_len=False)
    rng = np.random.default_rng(0)
    attr = rng.integers(1, 5, size=wl.n_branches)
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len,
                      wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new,
                      pos_mode="paper_gap", attr_len=attr)
    for p in range(wl.n_prompts):
        d0, d1 = wl.doc_ptr[p], wl.doc_ptr[p + 1]
        b0, b1 = wl.branch_ptr[d0], wl.branch_ptr[d1]
        plen = int(wl.header_len[p] + wl.doc_len[d0:d1].sum())
        for t in range(wl.max_new):
            for b in range(b0, b1):
                n = b - b0
                expect = plen + int(attr[b0:b + 1].sum()) - 1 + n * wl.max_new + (t + 1)
                assert orc.prompts[p].branch_position(n, t) == expect
        # prefix keeps ordinary increasing positions in this mode
        assert list(orc.prompts[p].prefix_positions()) == list(range(plen))


# ---------------------------------------------------------------------------
# Liveness / slots / memory order
# ---------------------------------------------------------------------------
def test_liveness_and_slots_and_flat_order():
    wl = W.random_workload(11, t=6, p=3)
    orc, _, steps = _run_oracle(wl)
    total = 0
    seen = set()
    for t, res in enumerate(steps):
        live = np.nonzero(wl.branch_len > t)[0]
        assert np.array_equal(orc.live(t), live)
        assert len(res["rows"]) == len(live)
        total += len(live)
        for s in res["slot"]:
            assert s not in seen  # every slot written exactly once
            seen.add(int(s))
            b, tt = divmod(int(s), wl.max_new)
            assert tt < wl.branch_len[b]  # never past the branch's length
    assert total == int(wl.branch_len.sum())
    # flat index: n_prefix + live counts of earlier steps + rank among this step's live
    for p, po in orc.prompts.items():
        b0, b1 = orc.branch_range[p]
        before = po.n_prefix
        for t, res in enumerate(steps):
            live = np.nonzero(wl.branch_len > t)[0]
            sel = np.nonzero((live >= b0) & (live < b1))[0]
            mine = [i for i, r in enumerate(res["rows"]) if r in set(sel)]
            assert np.array_equal(res["flat"][mine], before + np.arange(len(sel)))
            before += len(sel)


# ---------------------------------------------------------------------------
# Mask structure
# ---------------------------------------------------------------------------
def _brute_mask(po):
    """Set construction straight from the block rule, no position IDs."""
    s = len(po.kind)
    m = np.zeros((s, s), dtype=np.uint8)
    hdr = [i for i in range(s) if po.kind[i] == O.KIND_HEADER]
    for qi in range(s):
        if po.kind[qi] == O.KIND_HEADER:
            allowed = [i for i in hdr if i <= qi]
        elif po.kind[qi] == O.KIND_DOC:
            allowed = hdr + [i for i in range(s) if po.kind[i] == O.KIND_DOC
                             and po.doc[i] == po.doc[qi] and i <= qi]
        else:
            allowed = hdr + [i for i in range(s) if po.kind[i] == O.KIND_DOC
                             and po.doc[i] == po.doc[qi]]
            allowed += [i for i in range(s) if po.kind[i] == O.KIND_BRANCH
                        and po.branch[i] == po.branch[qi] and po.step_of[i] <= po.step_of[qi]]
        m[qi, allowed] = 1
    return m


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_mask_equals_block_rule_and_row_sums(seed):
    wl = W.random_workload(seed, t=4, p=2, l_range=(1, 12), h_range=(0, 6))
    orc, _, _ = _run_oracle(wl)
    for po in orc.prompts.values():
        m = po.dense_mask()
        assert np.array_equal(m, _brute_mask(po))
        assert np.array_equal(m, po.mask_rows_fast(list(range(len(po.kind)))))
        for qi in range(len(po.kind)):
            if po.kind[qi] == O.KIND_BRANCH:
                j = po.doc[qi]
                assert m[qi].sum() == po.h + po.doc_lens[j] + po.step_of[qi] + 1
                # nothing outside own block
                for ki in np.nonzero(m[qi])[0]:
                    assert po.kind[ki] == O.KIND_HEADER or po.doc[ki] == j
        # lower-triangular once a block is ordered by position ID
        for b in range(po.n_branches):
            j = po.branch_doc[b]
            idx = [i for i in range(len(po.kind)) if po.kind[i] == O.KIND_HEADER
                   or (po.kind[i] == O.KIND_DOC and po.doc[i] == j)
                   or (po.kind[i] == O.KIND_BRANCH and po.branch[i] == b)]
            idx.sort(key=lambda i: po.pos[i])
            sub = m[np.ix_(idx, idx)]
            assert np.array_equal(sub, np.tril(np.ones_like(sub)))


def test_mask_is_not_triangular_in_memory_order():
    # two branches, two steps: token (b0, t1) sits after (b1, t0) in memory but may not see it,
    # and the mask row of (b0,t1) has a hole -> non-triangular, as the paper states.
    wl = W.make_workload("x", "f32", 2, 2, 8, 10000.0, 2, [2], [1], [3], [2])
    orc, _, _ = _run_oracle(wl)
    po = orc.prompts[0]
    m = po.dense_mask()
    assert m.shape == (9, 9)
    # memory: 0,1 header; 2,3,4 doc; 5=(b0,t0) 6=(b1,t0) 7=(b0,t1) 8=(b1,t1)
    assert list(m[7]) == [1, 1, 1, 1, 1, 1, 0, 1, 0]
    assert list(m[8]) == [1, 1, 1, 1, 1, 0, 1, 0, 1]
    assert list(m[5]) == [1, 1, 1, 1, 1, 1, 0, 0, 0]


# ---------------------------------------------------------------------------
# RoPE identities (independent complex-number formulation)
# ---------------------------------------------------------------------------
def _rope_complex(x, pos, base):
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    z = x[..., :half] + 1j * x[..., half:]
    theta = base ** (-np.arange(half) * 2.0 / d)
    z = z * np.exp(1j * np.asarray(pos, dtype=np.float64)[..., None, None] * theta)
    return np.concatenate([z.real, z.imag], axis=-1)


def test_rope_against_complex_form_and_identities():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 3, 16))
    pos = np.array([0, 1, 7, 100, 4321])
    got = O.rope(x, pos, 500000.0, np.float64)
    assert np.allclose(got, _rope_complex(x, pos, 500000.0), atol=1e-12)
    assert np.array_equal(got[0], x[0])  # position 0 is the identity
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1))
    # <R(a) q, R(b) k> depends on a - b only
    q = rng.standard_normal((1, 1, 16))
    k = rng.standard_normal((1, 1, 16))
    d1 = (O.rope(q, np.array([9]), 1e4, np.float64) * O.rope(k, np.array([4]), 1e4, np.float64)).sum()
    d2 = (O.rope(q, np.array([109]), 1e4, np.float64) * O.rope(k, np.array([104]), 1e4, np.float64)).sum()
    assert abs(d1 - d2) < 1e-10
    # direction of rotation: pair (1, 0) at the first frequency turns counter-clockwise
    e = np.zeros((1, 1, 4)); e[0, 0, 0] = 1.0
    r = O.rope(e, np.array([1]), 1e4, np.float64)[0, 0]
    assert np.allclose(r, [np.cos(1.0), 0.0, np.sin(1.0), 0.0])


# ---------------------------------------------------------------------------
# Softmax / PV special cases
# ---------------------------------------------------------------------------
def test_masked_attention_special_cases():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((3, 4, 8)).astype(np.float32)
    k = rng.standard_normal((6, 2, 8)).astype(np.float32)
    v = rng.standard_normal((6, 2, 8)).astype(np.float32)
    mask = np.ones((3, 6), dtype=np.uint8)
    # all-equal V -> output equals V
    vc = np.broadcast_to(v[:1], v.shape)
    out = O.masked_attention(q, k, vc, mask, 2)
    assert np.allclose(out, np.repeat(vc[0], 2, axis=0)[None].repeat(3, 0), atol=1e-6)
    # exactly one allowed key -> output is its V (and GQA maps heads 0,1->0 ; 2,3->1)
    one = np.zeros((3, 6), dtype=np.uint8)
    one[np.arange(3), [4, 0, 2]] = 1
    out = O.masked_attention(q, k, v, one, 2)
    for r, c in enumerate([4, 0, 2]):
        for h in range(4):
            assert np.allclose(out[r, h], v[c, h // 2], atol=1e-6)
    # library cross-check with an arbitrary mask and GQA
    mask = (rng.random((3, 6)) < 0.6).astype(np.uint8)
    mask[:, 0] = 1
    out = O.masked_attention(q, k, v, mask, 2)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]  # [1, Hq, R, D]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, attn_mask=torch.from_numpy(mask.astype(bool))[None, None])
    assert np.allclose(out, ref[0].permute(1, 0, 2).numpy(), atol=2e-6)


# ---------------------------------------------------------------------------
# The method's main invariant: HPD == ordinary causal attention over the
# contiguous sequence [header, own document, own branch tokens]
# ---------------------------------------------------------------------------
def _causal_reference(wl, inputs, b, t_hi, base):
    """Library routine (torch SDPA, is_causal=True, fp64) over the contiguous
    un-rotated sequence of branch b with positions 0..n-1 and the independent
    complex-number RoPE.  Returns out[t] for t <= t_hi as [Hq, D]."""
    d = int(np.searchsorted(wl.branch_ptr, b, side="right") - 1)
    p = int(np.searchsorted(wl.doc_ptr, d, side="right") - 1)
    tok0 = int(wl.header_len[:p].sum() + wl.doc_len[:wl.doc_ptr[p]].sum())
    h = int(wl.header_len[p])
    doc_off = tok0 + h + int(wl.doc_len[wl.doc_ptr[p]:d].sum())
    l = int(wl.doc_len[d])
    ks = [inputs["kp"][tok0:tok0 + h], inputs["kp"][doc_off:doc_off + l]]
    vs = [inputs["vp"][tok0:tok0 + h], inputs["vp"][doc_off:doc_off + l]]
    qs = [np.zeros((h + l, wl.n_q_heads, wl.head_dim))]
    for t in range(t_hi + 1):
        live = np.nonzero(wl.branch_len > t)[0]
        r = int(np.nonzero(live == b)[0][0])
        ks.append(inputs["k"][t][r:r + 1]); vs.append(inputs["v"][t][r:r + 1])
        qs.append(inputs["q"][t][r:r + 1])
    k = np.concatenate(ks).astype(np.float64)
    v = np.concatenate(vs).astype(np.float64)
    q = np.concatenate(qs).astype(np.float64)
    n = k.shape[0]
    pos = np.arange(n)
    kr = _rope_complex(k, pos, base)
    qr = _rope_complex(q, pos, base)
    g = wl.n_q_heads // wl.n_kv_heads
    tq = torch.from_numpy(qr).permute(1, 0, 2)[None]
    tk = torch.from_numpy(kr).permute(1, 0, 2).repeat_interleave(g, 0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(g, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    return ref[0].permute(1, 0, 2).numpy()[h + l:]  # [t_hi+1, Hq, D]


@pytest.mark.parametrize("seed,dtype,tol", [(21, np.float64, 1e-12), (22, np.float32, 2e-5),
                                            (23, np.float32, 2e-5)])
def test_hpd_equals_contiguous_causal_attention(seed, dtype, tol):
    wl = W.random_workload(seed, t=5, p=3, hq=4, hkv=2, d=16)
    orc, inputs, steps = _run_oracle(wl, dtype=dtype)
    for b in range(wl.n_branches):
        t_hi = int(wl.branch_len[b]) - 1
        ref = _causal_reference(wl, inputs, b, t_hi, wl.rope_base)
        for t in range(t_hi + 1):
            live = np.nonzero(wl.branch_len > t)[0]
            r = int(np.nonzero(live == b)[0][0])
            assert np.array_equal(steps[t]["rows"], np.arange(len(live)))
            err = np.abs(steps[t]["out"][r] - ref[t]).max()
            assert err < tol, (b, t, err)


def test_single_branch_is_standard_causal_decoding():
    # J = 1, N = 1: the layout degenerates to an ordinary sequence
    wl = W.make_workload("single", "f32", 4, 4, 32, 10000.0, 6, [5], [1], [9], [1])
    orc, inputs, steps = _run_oracle(wl, dtype=np.float64)
    ref = _causal_reference(wl, inputs, 0, 5, wl.rope_base)
    po = orc.prompts[0]
    assert np.array_equal(po.dense_mask(), np.tril(np.ones((20, 20), dtype=np.uint8)))
    assert po.pos == list(range(20))
    for t in range(6):
        assert np.abs(steps[t]["out"][0] - ref[t]).max() < 1e-12


def test_fp32_oracle_close_to_fp64_oracle_on_cfg1():
    wl = W.config(1)
    _, _, s32 = _run_oracle(wl, dtype=np.float32)
    _, _, s64 = _run_oracle(wl, dtype=np.float64)
    for a, b in zip(s32, s64):
        assert np.abs(a["out"] - b["out"]).max() < 5e-6


# ---------------------------------------------------------------------------
# Brute force on tiny inputs (different code, fp64 scalar loops)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["general", "h0_l1_t1_n1_gqa"])
def test_oracle_against_scalar_brute_force(case):
    if case == "general":
        wl = W.make_workload("bf", "f32", 4, 2, 8, 10000.0, 3, [3], [2], [4, 2], [2, 1],
                             branch_len=[3, 1, 2])
    else:
        wl = W.make_workload("bf2", "f32", 4, 1, 8, 10000.0, 1, [0], [1], [1], [1])
    orc, inputs, steps = _run_oracle(wl, dtype=np.float64)
    bl = [[int(x) for x in wl.branch_len[wl.branch_ptr[d]:wl.branch_ptr[d + 1]]]
          for d in range(wl.n_docs)]
    ref = brute_force.decode_all_steps(
        int(wl.header_len[0]), [int(x) for x in wl.doc_len], bl, wl.n_q_heads, wl.n_kv_heads,
        wl.head_dim, wl.rope_base, wl.max_new, inputs["kp"].tolist(), inputs["vp"].tolist(),
        [x.tolist() for x in inputs["q"]], [x.tolist() for x in inputs["k"]],
        [x.tolist() for x in inputs["v"]])
    for t in range(wl.max_new):
        if len(ref[t]) == 0:
            assert steps[t]["out"].shape[0] == 0
            continue
        assert np.abs(steps[t]["out"] - np.asarray(ref[t])).max() < 1e-12


# ---------------------------------------------------------------------------
# Properties the method rests on
# ---------------------------------------------------------------------------
def test_branch_independence_bit_identical():
    """Changing another document's KV or another branch's tail leaves a branch's
    output bit-identical (conditional independence, Eq. 3)."""
    wl = W.make_workload("ind", "f32", 2, 2, 16, 10000.0, 3, [4], [2], [6, 5], [2, 2])
    orc, inputs, base_steps = _run_oracle(wl)
    # perturb doc 1's KV and branch 1's inputs, watch branch 0
    kp, vp = inputs["kp"].copy(), inputs["vp"].copy()
    kp[4 + 6:] += 1.0
    vp[4 + 6:] -= 2.0
    orc2 = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len,
                       wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new)
    orc2.prefill(kp, vp)
    for t in range(wl.max_new):
        q, k, v = inputs["q"][t].copy(), inputs["k"][t].copy(), inputs["v"][t].copy()
        q[1:] *= 3.0; k[1:] += 0.5; v[1:] -= 0.5
        res = orc2.step(t, q, k, v)
        assert np.array_equal(res["out"][0], base_steps[t]["out"][0])
        assert not np.array_equal(res["out"][2], base_steps[t]["out"][2])


def test_memory_order_is_irrelevant():
    """Permuting where allowed keys sit in memory (carrying their position IDs)
    does not change the output: order lives in the position IDs only."""
    wl = W.make_workload("perm", "f32", 2, 1, 16, 10000.0, 2, [3], [1], [5], [2])
    orc, inputs, steps = _run_oracle(wl, dtype=np.float64)
    po = orc.prompts[0]
    s = len(po.kind)
    rows = [s - 2, s - 1]  # the two tokens of the last step
    mask = po.mask_rows_fast(rows)
    q = O.rope(inputs["q"][1], np.array([po.pos[r] for r in rows]), wl.rope_base, np.float64)
    ref = O.masked_attention(q, po.k, po.v, mask, 1, np.float64)
    assert np.allclose(ref, steps[1]["out"], atol=1e-13)
    perm = np.random.default_rng(0).permutation(s)
    out = O.masked_attention(q, po.k[perm], po.v[perm], mask[:, perm], 1, np.float64)
    assert np.allclose(out, ref, atol=1e-13)


def test_shifting_all_positions_of_a_prompt_changes_nothing():
    """RoPE is relative: a header-less prompt and the same prompt behind an
    all-zero-attention-free shift give the same result when every position moves
    by a constant (here: compare base positions H+L+t against shifted copies)."""
    wl = W.make_workload("sh", "f32", 2, 2, 16, 10000.0, 2, [0], [1], [6], [2])
    orc, inputs, steps = _run_oracle(wl, dtype=np.float64)
    po = orc.prompts[0]
    shift = 37
    k_shift = O.rope(np.concatenate([inputs["kp"], inputs["k"][0], inputs["k"][1]]),
                     np.asarray(po.pos) + shift, wl.rope_base, np.float64)
    rows = [len(po.kind) - 2, len(po.kind) - 1]
    q = O.rope(inputs["q"][1], np.asarray([po.pos[r] + shift for r in rows]), wl.rope_base, np.float64)
    out = O.masked_attention(q, k_shift, po.v, po.mask_rows_fast(rows), 2, np.float64)
    assert np.allclose(out, steps[1]["out"], atol=1e-11)


# ---------------------------------------------------------------------------
# Planted mistakes: each plausible slip in the oracle must trip the main pin
# ---------------------------------------------------------------------------
def _main_pin_error(wl):
    orc, inputs, steps = _run_oracle(wl, dtype=np.float64)
    worst = 0.0
    for b in range(wl.n_branches):
        t_hi = int(wl.branch_len[b]) - 1
        ref = _causal_reference(wl, inputs, b, t_hi, wl.rope_base)
        for t in range(t_hi + 1):
            live = np.nonzero(wl.branch_len > t)[0]
            r = int(np.nonzero(live == b)[0][0])
            worst = max(worst, float(np.abs(steps[t]["out"][r] - ref[t]).max()))
    return worst


@pytest.mark.parametrize("mistake", ["rope_sign", "no_diagonal", "gqa_interleaved", "no_scale",
                                     "doc_pos_not_restarted", "sees_other_doc", "swap_kv_halves"])
def test_planted_mistakes_are_caught(monkeypatch, mistake):
    wl = W.random_workload(31, t=4, p=2, hq=4, hkv=2, d=16, j_range=(2, 3), n_range=(2, 3),
                           h_range=(2, 6), l_range=(3, 9))
    assert _main_pin_error(wl) < 1e-12
    if mistake == "rope_sign":
        real = O.rope
        monkeypatch.setattr(O, "rope", lambda x, pos, base, dtype=np.float32:
                            real(x, -np.asarray(pos), base, dtype) if np.ndim(pos) and len(pos) % 2
                            else real(x, pos, base, dtype))
    elif mistake == "no_diagonal":
        real = O.PromptOracle.mask_rows_fast
        def bad(self, rows):
            m = real(self, rows)
            m[np.arange(len(rows)), rows] = 0
            return m
        monkeypatch.setattr(O.PromptOracle, "mask_rows_fast", bad)
    elif mistake == "gqa_interleaved":
        real = O.masked_attention
        def bad(q, k, v, mask, n_kv_heads, dtype=np.float32):
            hq = q.shape[1]
            perm = [(h % n_kv_heads) * (hq // n_kv_heads) + h // n_kv_heads for h in range(hq)]
            return real(q[:, perm], k, v, mask, n_kv_heads, dtype)
        monkeypatch.setattr(O, "masked_attention", bad)
    elif mistake == "no_scale":
        real = O.masked_attention
        monkeypatch.setattr(O, "masked_attention", lambda q, k, v, mask, n, dtype=np.float32:
                            real(q * np.sqrt(np.sqrt(q.shape[-1])), k * np.sqrt(np.sqrt(q.shape[-1])),
                                 v, mask, n, dtype))
    elif mistake == "doc_pos_not_restarted":
        real = O.PromptOracle.prefix_positions
        monkeypatch.setattr(O.PromptOracle, "prefix_positions",
                            lambda self: np.arange(self.n_prefix, dtype=np.int64))
    elif mistake == "sees_other_doc":
        real = O.PromptOracle.mask_rows_fast
        def bad(self, rows):
            m = real(self, rows)
            m[:, np.asarray(self.kind) == O.KIND_DOC] = 1
            return m
        monkeypatch.setattr(O.PromptOracle, "mask_rows_fast", bad)
    elif mistake == "swap_kv_halves":
        real = O.rope
        def bad(x, pos, base, dtype=np.float32):
            y = real(x, pos, base, dtype)
            h = y.shape[-1] // 2
            return np.concatenate([y[..., h:], y[..., :h]], axis=-1) if y.shape[1] == 2 else y
        monkeypatch.setattr(O, "rope", bad)
    assert _main_pin_error(wl) > 1e-6


# ---------------------------------------------------------------------------
# The paper-literal mask (Section 4.3.2 over the whole stacked prompt)
# ---------------------------------------------------------------------------
def _paper_case(seed, **kw):
    wl = W.random_workload(seed, **kw)
    attr = np.random.default_rng(1000 + seed).integers(1, 5, size=wl.n_branches)
    return wl, attr


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_paper_mask_set_construction_and_row_sums(seed):
    wl, attr = _paper_case(seed, t=4, p=2, l_range=(1, 9), h_range=(0, 5), j_range=(1, 3), n_range=(1, 4))
    orc, _, _ = _run_oracle(wl, pos_mode="paper_gap", attr_len=attr, mask_mode="paper")
    for po in orc.prompts.values():
        m = po.dense_mask()
        assert np.array_equal(m, po.mask_rows_fast(list(range(len(po.kind)))))
        s = len(po.kind)
        for qi in range(s):
            if po.kind[qi] != O.KIND_BRANCH:
                continue
            b, t = po.branch[qi], po.step_of[qi]
            # written out: header and documents, the attribute names up to the own one, earlier
            # attributes' value tokens up to this step, own tokens
            n_hd = po.h + sum(po.doc_lens)
            want = set(range(n_hd))
            want |= {i for i in range(s) if po.kind[i] == O.KIND_SKELETON and po.branch[i] <= b}
            want |= {i for i in range(s) if po.kind[i] == O.KIND_BRANCH and po.branch[i] <= b
                     and po.step_of[i] <= t}
            assert set(np.nonzero(m[qi])[0]) == want
            assert m[qi].sum() == (n_hd + sum(po.attr_lens[:b + 1])
                                   + sum(min(t + 1, po.branch_len[bb]) for bb in range(b)) + t + 1)
            # nothing with a larger position ID, nothing that was appended later
            assert all(po.pos[i] <= po.pos[qi] and i <= qi for i in np.nonzero(m[qi])[0])
        # ordered by position ID the whole memory is causal: lower triangular, except that a
        # token cannot see what entered memory after it (value tokens of earlier attributes
        # from later steps)
        order = sorted(range(s), key=lambda i: po.pos[i])
        assert len({po.pos[i] for i in order}) == s  # position IDs are distinct
        sub = m[np.ix_(order, order)]
        exists = np.asarray([[ki <= qi for ki in order] for qi in order])
        assert np.array_equal(sub, np.tril(np.ones_like(sub)) * exists)


def test_paper_mask_reduces_to_block_mask_for_one_document_one_attribute():
    wl = W.make_workload("one", "f32", 4, 2, 16, 10000.0, 5, [4], [1], [7], [1])
    attr = np.asarray([3])
    a, _, sa = _run_oracle(wl, dtype=np.float64, pos_mode="paper_gap", attr_len=attr, mask_mode="paper")
    b, _, sb = _run_oracle(wl, dtype=np.float64, pos_mode="paper_gap", attr_len=attr, mask_mode="block")
    # the literal mask adds the attribute's own name tokens (3 of them, in memory after the
    # document); everything else is the block mask
    ma, mb = a.prompts[0].dense_mask(), b.prompts[0].dense_mask()
    n_hd = 4 + 7
    keep = [i for i in range(ma.shape[0]) if not (n_hd <= i < n_hd + 3)]
    assert np.array_equal(ma[np.ix_(keep, keep)], mb)
    rows = [i for i in range(ma.shape[0]) if a.prompts[0].kind[i] == O.KIND_BRANCH]
    assert np.all(ma[np.ix_(rows, list(range(n_hd, n_hd + 3)))] == 1)


def test_paper_mask_sees_more_than_block_mask():
    wl, attr = _paper_case(5, t=3, p=1, j_range=(2, 2), n_range=(2, 2), ragged_len=False)
    a, _, _ = _run_oracle(wl, pos_mode="paper_gap", attr_len=attr, mask_mode="paper")
    b, _, _ = _run_oracle(wl, pos_mode="paper_gap", attr_len=attr, mask_mode="block")
    ma, mb = a.prompts[0].dense_mask(), b.prompts[0].dense_mask()
    po = a.prompts[0]
    rows = [i for i in range(len(po.kind)) if po.kind[i] == O.KIND_BRANCH]
    cols = [i for i in range(len(po.kind)) if po.kind[i] != O.KIND_SKELETON]
    rows_b = [i for i in range(len(b.prompts[0].kind)) if b.prompts[0].kind[i] == O.KIND_BRANCH]
    assert np.all(ma[np.ix_(rows, cols)] >= mb[rows_b])  # the block mask is a subset
    last = rows[-1]  # last attribute of the last document, last step
    assert ma[last].sum() == len(po.kind) and mb[rows_b[-1]].sum() < ma[last].sum()


@pytest.mark.parametrize("seed,dtype,tol", [(41, np.float64, 1e-12), (42, np.float32, 2e-5)])
def test_paper_mask_equals_causal_attention_in_position_order(seed, dtype, tol):
    """Section 4.3.2: appended out of order in memory, the tokens attend as if the sequence
    were laid out by position ID.  Library causal attention (is_causal=True) over everything
    in memory after step t, sorted by position ID, with the independent complex-number RoPE
    at the true position IDs: the rows of the step's queries must equal the oracle's."""
    wl, attr = _paper_case(seed, t=4, p=2, hq=4, hkv=2, d=16, j_range=(1, 3), n_range=(1, 3),
                           h_range=(0, 5), l_range=(1, 8))
    orc, inputs, steps = _run_oracle(wl, dtype=dtype, pos_mode="paper_gap", attr_len=attr, mask_mode="paper")
    g = wl.n_q_heads // wl.n_kv_heads
    for p, po in orc.prompts.items():
        a0, a1 = orc.prefix_range[p]
        b0, b1 = orc.branch_range[p]
        k_all = [inputs["kp"][a0:a1]]
        v_all = [inputs["vp"][a0:a1]]
        q_all = [np.zeros((a1 - a0, wl.n_q_heads, wl.head_dim))]
        # header and documents at 0 .. |p|-1, then the attribute names: Algorithm 2 in closed
        # form (attribute n, 0-based, is shifted by n * K_max)
        plen = a1 - a0 - int(attr[b0:b1].sum())
        skel = [plen + int(attr[b0:b0 + n].sum()) + i + n * wl.max_new
                for n in range(b1 - b0) for i in range(int(attr[b0 + n]))]
        pos_all = [np.concatenate([np.arange(plen), np.asarray(skel, dtype=np.int64)])]
        for t in range(wl.max_new):
            live = np.nonzero(wl.branch_len > t)[0]
            sel = np.nonzero((live >= b0) & (live < b1))[0]
            if len(sel) == 0:
                continue
            k_all.append(inputs["k"][t][sel]); v_all.append(inputs["v"][t][sel]); q_all.append(inputs["q"][t][sel])
            # closed form of Appendix A.1 for the position IDs (not the oracle's own table)
            n_loc = live[sel] - b0
            pos_all.append(np.asarray([plen + int(attr[b0:b0 + n + 1].sum()) - 1 + n * wl.max_new + t + 1
                                       for n in n_loc]))
            k = np.concatenate(k_all).astype(np.float64)
            v = np.concatenate(v_all).astype(np.float64)
            q = np.concatenate(q_all).astype(np.float64)
            pos = np.concatenate(pos_all)
            order = np.argsort(pos, kind="stable")
            kr = _rope_complex(k[order], pos[order], wl.rope_base)
            qr = _rope_complex(q[order], pos[order], wl.rope_base)
            tq = torch.from_numpy(qr).permute(1, 0, 2)[None]
            tk = torch.from_numpy(kr).permute(1, 0, 2).repeat_interleave(g, 0)[None]
            tv = torch.from_numpy(v[order]).permute(1, 0, 2).repeat_interleave(g, 0)[None]
            ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
            ref = ref[0].permute(1, 0, 2).numpy()
            rank = np.empty_like(order)
            rank[order] = np.arange(len(order))
            n_mem = len(pos)
            mine = np.nonzero(np.isin(steps[t]["rows"], sel))[0]
            assert len(mine) == len(sel)
            for i, r in enumerate(mine):
                mem_index = n_mem - len(sel) + i  # this step's tokens are the last ones in memory
                err = np.abs(steps[t]["out"][r] - ref[rank[mem_index]]).max()
                assert err < tol, (p, t, i, err)


def test_paper_mask_against_scalar_brute_force():
    wl = W.make_workload("bfp", "f32", 4, 2, 8, 10000.0, 3, [2], [2], [3, 2], [2, 1], branch_len=[3, 1, 2])
    attr = np.asarray([2, 1, 3])
    orc, inputs, steps = _run_oracle(wl, dtype=np.float64, pos_mode="paper_gap", attr_len=attr,
                                     mask_mode="paper")
    bl = [[int(x) for x in wl.branch_len[wl.branch_ptr[d]:wl.branch_ptr[d + 1]]] for d in range(wl.n_docs)]
    ref = brute_force.decode_all_steps_paper(
        int(wl.header_len[0]), [int(x) for x in wl.doc_len], bl, [int(x) for x in attr], wl.n_q_heads,
        wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new, inputs["kp"].tolist(), inputs["vp"].tolist(),
        [x.tolist() for x in inputs["q"]], [x.tolist() for x in inputs["k"]], [x.tolist() for x in inputs["v"]])
    for t in range(wl.max_new):
        assert np.abs(steps[t]["out"] - np.asarray(ref[t])).max() < 1e-12


@pytest.mark.parametrize("mistake", ["sees_later_attribute", "misses_earlier_attribute", "misses_other_document"])
def test_paper_mask_planted_mistakes_are_caught(monkeypatch, mistake):
    wl = W.make_workload("pl", "f32", 4, 2, 8, 10000.0, 3, [2], [2], [3, 2], [2, 2])
    attr = np.asarray([2, 1, 3, 2])

    def worst():
        orc, inputs, steps = _run_oracle(wl, dtype=np.float64, pos_mode="paper_gap", attr_len=attr,
                                         mask_mode="paper")
        bl = [[3, 3], [3, 3]]
        ref = brute_force.decode_all_steps_paper(
            2, [3, 2], bl, [2, 1, 3, 2], 4, 2, 8, 10000.0, 3, inputs["kp"].tolist(), inputs["vp"].tolist(),
            [x.tolist() for x in inputs["q"]], [x.tolist() for x in inputs["k"]], [x.tolist() for x in inputs["v"]])
        return max(float(np.abs(steps[t]["out"] - np.asarray(ref[t])).max()) for t in range(3))

    assert worst() < 1e-12
    real = O.PromptOracle.mask_rows_fast

    def bad(self, rows):
        m = real(self, rows)
        kind, br, doc = np.asarray(self.kind), np.asarray(self.branch), np.asarray(self.doc)
        for r, qi in enumerate(rows):
            if mistake == "sees_later_attribute":
                m[r, (kind == O.KIND_BRANCH) & (br > br[qi]) & (np.arange(len(kind)) <= qi)] = 1
            elif mistake == "misses_earlier_attribute":
                m[r, (kind == O.KIND_BRANCH) & (br < br[qi])] = 0
            else:
                m[r, (kind == O.KIND_DOC) & (doc != doc[qi])] = 0
        return m

    monkeypatch.setattr(O.PromptOracle, "mask_rows_fast", bad)
    assert worst() > 1e-6


# ---------------------------------------------------------------------------
# The first inference step: attention of the prefix tokens themselves
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed,dtype,tol", [(51, np.float64, 1e-12), (52, np.float32, 2e-5)])
def test_prefill_attention_equals_causal_attention_per_document(seed, dtype, tol):
    """Under the block mask a document token sees the header and its own document up to
    itself: ordinary causal attention (library routine, independent complex-number RoPE) over
    the contiguous sequence [header, document] with positions 0..n-1; the header rows are the
    first H rows of any of them."""
    wl = W.random_workload(seed, t=2, p=2, hq=4, hkv=2, d=16, j_range=(1, 3), h_range=(0, 6), l_range=(1, 9))
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len,
                      wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new, dtype=dtype)
    kp = _values(wl, 1, (wl.n_prefix_tokens, wl.n_kv_heads, wl.head_dim))
    vp = _values(wl, 2, (wl.n_prefix_tokens, wl.n_kv_heads, wl.head_dim))
    qp = _values(wl, 3, (wl.n_prefix_tokens, wl.n_q_heads, wl.head_dim))
    orc.prefill(kp, vp)
    got = orc.prefill_attention(qp)
    g = wl.n_q_heads // wl.n_kv_heads
    for p in range(wl.n_prompts):
        a0, _ = orc.prefix_range[p]
        h = int(wl.header_len[p])
        off = a0 + h
        for d in range(wl.doc_ptr[p], wl.doc_ptr[p + 1]):
            l = int(wl.doc_len[d])
            idx = np.concatenate([np.arange(a0, a0 + h), np.arange(off, off + l)])
            n = len(idx)
            kr = _rope_complex(kp[idx].astype(np.float64), np.arange(n), wl.rope_base)
            qr = _rope_complex(qp[idx].astype(np.float64), np.arange(n), wl.rope_base)
            tq = torch.from_numpy(qr).permute(1, 0, 2)[None]
            tk = torch.from_numpy(kr).permute(1, 0, 2).repeat_interleave(g, 0)[None]
            tv = torch.from_numpy(vp[idx].astype(np.float64)).permute(1, 0, 2).repeat_interleave(g, 0)[None]
            ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
            ref = ref[0].permute(1, 0, 2).numpy()
            assert np.abs(got[p][idx - a0] - ref).max() < tol, (p, d)
            off += l


def test_prefill_attention_planted_mistake_is_caught(monkeypatch):
    wl = W.random_workload(53, t=2, p=1, hq=2, hkv=1, d=8, j_range=(2, 2), h_range=(2, 4), l_range=(3, 6))
    kp = _values(wl, 1, (wl.n_prefix_tokens, 1, 8)); vp = _values(wl, 2, (wl.n_prefix_tokens, 1, 8))
    qp = _values(wl, 3, (wl.n_prefix_tokens, 2, 8))

    def run():
        orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len, 2, 1, 8,
                          wl.rope_base, wl.max_new, dtype=np.float64)
        orc.prefill(kp, vp)
        return orc.prefill_attention(qp)[0]

    good = run()
    real = O.PromptOracle.mask_rows_fast
    monkeypatch.setattr(O.PromptOracle, "mask_rows_fast",
                        lambda self, rows: np.tril(np.ones((len(rows), len(self.kind)), dtype=np.uint8)))
    bad = run()  # plain causal over the stacked memory: the second document sees the first
    h, l0 = int(wl.header_len[0]), int(wl.doc_len[0])
    assert np.abs(good[:h + l0] - bad[:h + l0]).max() < 1e-12  # header and first document unchanged
    assert np.abs(good[h + l0:] - bad[h + l0:]).max() > 1e-6


@pytest.mark.parametrize("seed,dtype,tol", [(61, np.float64, 1e-12), (62, np.float32, 2e-5)])
def test_prefill_attention_under_the_literal_mask_is_plain_causal_attention(seed, dtype, tol):
    """First inference step, Section 4.3.2 taken literally: header, stacked documents and the
    attribute names are one sequence and the mask is the standard causal one.  Library causal
    attention over each prompt's prefix in memory order, with the independent complex-number
    RoPE at positions 0 .. |p|-1 for header and documents and Algorithm 2's closed form for the
    names (attribute n shifted by n * K_max): every row must equal the oracle's, the names'
    rows - the ones whose outputs start the branches - included."""
    wl, attr = _paper_case(seed, t=3, p=2, hq=4, hkv=2, d=16, j_range=(1, 3), n_range=(1, 3),
                           h_range=(0, 5), l_range=(1, 8))
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len,
                      wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new,
                      pos_mode="paper_gap", attr_len=attr, dtype=dtype, mask_mode="paper")
    n_tok = orc.n_prefix_tokens
    assert n_tok == wl.n_prefix_tokens + int(attr.sum())
    kp = _values(wl, 1, (n_tok, wl.n_kv_heads, wl.head_dim))
    vp = _values(wl, 2, (n_tok, wl.n_kv_heads, wl.head_dim))
    qp = _values(wl, 3, (n_tok, wl.n_q_heads, wl.head_dim))
    orc.prefill(kp, vp)
    got = orc.prefill_attention(qp)
    g = wl.n_q_heads // wl.n_kv_heads
    for p in range(wl.n_prompts):
        a0, a1 = orc.prefix_range[p]
        b0, b1 = orc.branch_range[p]
        plen = a1 - a0 - int(attr[b0:b1].sum())
        skel = [plen + int(attr[b0:b0 + n].sum()) + i + n * wl.max_new
                for n in range(b1 - b0) for i in range(int(attr[b0 + n]))]
        pos = np.concatenate([np.arange(plen), np.asarray(skel, dtype=np.int64)])
        assert len(pos) == a1 - a0 and np.all(np.diff(pos) > 0)  # memory order is position order
        kr = _rope_complex(kp[a0:a1].astype(np.float64), pos, wl.rope_base)
        qr = _rope_complex(qp[a0:a1].astype(np.float64), pos, wl.rope_base)
        tq = torch.from_numpy(qr).permute(1, 0, 2)[None]
        tk = torch.from_numpy(kr).permute(1, 0, 2).repeat_interleave(g, 0)[None]
        tv = torch.from_numpy(vp[a0:a1].astype(np.float64)).permute(1, 0, 2).repeat_interleave(g, 0)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
        assert np.abs(got[p] - ref).max() < tol, p


def test_prefill_attention_literal_and_block_masks_differ_only_behind_the_first_document():
    """Same prompt under both masks: header and first-document rows are identical (they see the
    same keys at the same positions); a later document's rows are not."""
    wl = W.random_workload(63, t=2, p=1, hq=2, hkv=1, d=8, j_range=(2, 2), n_range=(1, 2), h_range=(2, 4), l_range=(3, 6))
    attr = np.ones(wl.n_branches, dtype=np.int64)
    outs = {}
    for mode, pos_mode in (("block", "paper_gap"), ("paper", "paper_gap")):
        orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len, 2, 1, 8,
                          wl.rope_base, wl.max_new, pos_mode=pos_mode, attr_len=attr, dtype=np.float64,
                          mask_mode=mode)
        n_tok = orc.n_prefix_tokens
        kp = _values(wl, 1, (n_tok, 1, 8)); vp = _values(wl, 2, (n_tok, 1, 8)); qp = _values(wl, 3, (n_tok, 2, 8))
        orc.prefill(kp, vp)
        outs[mode] = orc.prefill_attention(qp)[0]
    h, l0 = int(wl.header_len[0]), int(wl.doc_len[0])
    n = wl.n_prefix_tokens
    assert np.abs(outs["block"][:h + l0] - outs["paper"][:h + l0]).max() < 1e-12
    assert np.abs(outs["block"][h + l0:n] - outs["paper"][h + l0:n]).max() > 1e-6


# ---------------------------------------------------------------------------
# Algorithm 2 by a walk along s, independent of the oracle's closed form
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(6))
def test_alg2_equals_a_walk_that_reserves_k_max_ids_behind_every_attribute(seed):
    """Appendix A.1 in words: positions run on along s, and behind every attribute K_max IDs
    are left free for its value.  Walk s token by token with a counter."""
    rng = np.random.default_rng(100 + seed)
    plen = int(rng.integers(0, 40))
    attr = [int(x) for x in rng.integers(1, 7, size=int(rng.integers(1, 9)))]
    kmax = int(rng.integers(1, 33))
    want, ends, counter = [], [], 0
    for _ in range(plen):
        want.append(counter)
        counter += 1
    for a in attr:
        for _ in range(a):
            want.append(counter)
            counter += 1
        ends.append(len(want) - 1)
        counter += kmax  # the IDs of the value tokens to come
    pos_id, end_index = O.alg2_position_ids(plen, attr, kmax)
    assert [int(x) for x in pos_id] == want
    assert [int(x) for x in end_index] == ends


# ---------------------------------------------------------------------------
# The bf16 key cache (Appendix B: bf16 inference): rounding and where it is applied
# ---------------------------------------------------------------------------
def _bf16_via_torch(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).float().numpy()


def test_round_to_bf16_equals_the_library_conversion_over_the_whole_exponent_range():
    rng = np.random.default_rng(5)
    # every exponent (subnormals, normals, the largest finite ones), random mantissas and signs
    bits = rng.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x)]
    got, want = O.round_to_bf16(x), _bf16_via_torch(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # N(0,1) magnitudes, the values the parity tests feed
    y = rng.standard_normal(1 << 18).astype(np.float32)
    assert np.array_equal(O.round_to_bf16(y).view(np.uint32), _bf16_via_torch(y).view(np.uint32))
    # the low 16 bits are gone and the value moved by at most half a bf16 ulp
    assert not np.any(O.round_to_bf16(y).view(np.uint32) & 0xFFFF)
    ulp = np.float32(2.0) ** (np.floor(np.log2(np.abs(y))) - 7)
    assert np.all(np.abs(O.round_to_bf16(y) - y) <= ulp / 2)


def test_round_to_bf16_hand_computed_cases():
    f = lambda bits: np.asarray([bits], dtype=np.uint32).view(np.float32)
    r = lambda bits: int(O.round_to_bf16(f(bits)).view(np.uint32)[0])
    # ties go to the even neighbour, in both directions
    assert r(0x3F808000) == 0x3F800000   # 1 + 2^-8: halfway between 1.0 (even) and 1 + 2^-7
    assert r(0x3F818000) == 0x3F820000   # 1 + 3*2^-8: halfway, the odd one below goes up
    assert r(0x3F808001) == 0x3F810000   # just above the tie: up
    assert r(0x3F807FFF) == 0x3F800000   # just below: down
    assert r(0xBF808000) == 0xBF800000 and r(0xBF818000) == 0xBF820000  # sign carried along
    # zeros, infinities, representable values stay
    for bits in (0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x3F800000, 0x40490000, 0x00010000):
        assert r(bits) == bits
    # a carry out of the mantissa raises the exponent; the largest finite fp32 overflows to inf
    assert r(0x3FFFFFFF) == 0x40000000
    assert r(0x7F7FFFFF) == 0x7F800000
    # subnormals: the smallest fp32 subnormal rounds to zero, half the smallest bf16 one ties to zero
    assert r(0x00000001) == 0x00000000 and r(0x00008000) == 0x00000000 and r(0x00008001) == 0x00010000
    # exact small numbers: 0.1f = 0x3DCCCCCD -> 0x3DCD0000
    assert r(0x3DCCCCCD) == 0x3DCD0000


def test_bf16_cache_changes_the_stored_key_and_nothing_else():
    """cache_dtype="bf16" = the unrounded oracle whose rotated keys are rounded on entry: same
    values, positions, masks; outputs equal the plain definition fed with pre-rounded keys."""
    wl = W.random_workload(21, t=4, p=2)
    kw = dict(pos_mode="contig")
    plain = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len, wl.n_q_heads,
                        wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new, **kw)
    cached = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len, wl.n_q_heads,
                         wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new, cache_dtype="bf16", **kw)
    kp = _values(wl, 1, (plain.n_prefix_tokens, wl.n_kv_heads, wl.head_dim))
    vp = _values(wl, 2, (plain.n_prefix_tokens, wl.n_kv_heads, wl.head_dim))
    plain.prefill(kp, vp), cached.prefill(kp, vp)
    differs = False
    for t in range(wl.max_new):
        n_live = int((wl.branch_len > t).sum())
        q = _values(wl, 10 + 3 * t, (n_live, wl.n_q_heads, wl.head_dim))
        k = _values(wl, 11 + 3 * t, (n_live, wl.n_kv_heads, wl.head_dim))
        v = _values(wl, 12 + 3 * t, (n_live, wl.n_kv_heads, wl.head_dim))
        a, b = plain.step(t, q, k, v), cached.step(t, q, k, v)
        for key in ("rows", "pos", "slot", "flat"):
            assert np.array_equal(a[key], b[key])
        for p in plain.prompts:
            pa, pb = plain.prompts[p], cached.prompts[p]
            # the cache: keys are the library's bf16 conversion of the unrounded ones, values untouched
            assert np.array_equal(pb.k.view(np.uint32), _bf16_via_torch(pa.k).view(np.uint32))
            assert np.array_equal(pb.v, pa.v)
            assert pa.pos == pb.pos and pa.kind == pb.kind
            assert np.array_equal(pa.mask_rows_fast(list(range(len(pa.kind)))),
                                  pb.mask_rows_fast(list(range(len(pb.kind)))))
            # outputs: the plain definition over the rounded keys, with the query rotated in fp32
            live = [x for x in pa.live(t)]
            b0, _ = plain.branch_range[p]
            sel = np.nonzero(np.isin(a["rows"], np.nonzero(np.isin(plain.live(t), np.asarray(live) + b0))[0]))[0]
            rows = list(range(len(pa.kind) - len(live), len(pa.kind)))
            qr = O.rope(q[a["rows"][sel]], a["pos"][sel], wl.rope_base)
            want = O.masked_attention(qr, _bf16_via_torch(pa.k), pa.v, pa.mask_rows(rows), wl.n_kv_heads)
            assert np.array_equal(b["out"][sel], want)
        differs |= not np.array_equal(a["out"], b["out"])
        # ... and the rounding of the keys moves the outputs by little (2^-9 relative per key)
        rms = float(np.sqrt(np.mean(a["out"].astype(np.float64) ** 2)))
        assert np.abs(a["out"] - b["out"]).max() <= 5e-2 * rms
    assert differs  # the mode is not a no-op
