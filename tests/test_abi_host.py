"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its
host-side layout logic (no GPU call) agrees bit-for-bit with the oracle's integers."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import hpd_oracle as O
from paper_2604_26209_amd import binding as B
from paper_2604_26209_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "hpd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(hpd_[a-z_]+)\s*\(", text))
    assert {"hpd_build_layout", "hpd_rope_positions", "hpd_decode_attention", "hpd_kv_append"} <= declared
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)
    # the benchmark's reference kernels have a header of their own
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "hpd_peaks.h")).read(), flags=re.S)
    peaks = set(re.findall(r"\b(hpd_[a-z_]+)\s*\(", text))
    assert peaks == set(B.PEAK_EXPORTS)
    for name in peaks:
        assert hasattr(lib, name), name
    assert sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h")) == ["hpd.h", "hpd_peaks.h"]


def _host_layout(wl, pos_mode=B.HPD_POS_CONTIG, attr_len=None):
    return B.layout_from_workload(wl, pos_mode=pos_mode, attr_len=attr_len, flags=B.HPD_FLAG_HOST_ONLY)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_host_tables_match_oracle_on_configs(k):
    wl = W.config(k)
    lay = _host_layout(wl)
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len,
                      wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new)
    n_live = lay.n_live()
    live = B.hpd_layout_query(lay, B.HPD_Q_LIVE_BRANCH)
    base = B.hpd_layout_query(lay, B.HPD_Q_BRANCH_BASE_POS)
    off = 0
    for t in range(wl.max_new):
        want = orc.live(t)
        assert n_live[t] == len(want)
        assert np.array_equal(live[off:off + n_live[t]], want)
        assert np.array_equal(base[want].astype(np.int64) + 1 + t, orc.positions(t))
        off += n_live[t]
    c = lay.counts()
    assert c[B.HPD_C_TOTAL_LIVE] == wl.branch_len.sum() == off
    assert c[B.HPD_C_N_PREFIX_TOKENS] == wl.n_prefix_tokens
    assert c[B.HPD_C_N_TAIL_SLOTS] == wl.n_branches * wl.max_new
    # segments: aligned, disjoint, inside the pool
    seg_off = B.hpd_layout_query(lay, B.HPD_Q_SEG_OFF).astype(np.int64)
    seg_len = B.hpd_layout_query(lay, B.HPD_Q_SEG_LEN).astype(np.int64)
    assert np.all(seg_off % B.HPD_KEY_BLOCK == 0)
    order = np.argsort(seg_off, kind="stable")
    ends = seg_off[order] + seg_len[order]
    assert np.all(ends[:-1] <= seg_off[order][1:])
    assert ends.max() <= c[B.HPD_C_N_PREFIX_SLOTS]
    assert np.array_equal(seg_len[:wl.n_prompts], wl.header_len)
    assert np.array_equal(seg_len[wl.n_prompts:], wl.doc_len)
    # positions of segment starts: header 0, document right after its header
    pos0 = B.hpd_layout_query(lay, B.HPD_Q_SEG_POS0)
    prompt_of_doc = np.repeat(np.arange(wl.n_prompts), np.diff(wl.doc_ptr))
    assert np.all(pos0[:wl.n_prompts] == 0)
    assert np.array_equal(pos0[wl.n_prompts:], wl.header_len[prompt_of_doc])
    # raw token order = prompts in order, header then documents
    raw = B.hpd_layout_query(lay, B.HPD_Q_SEG_RAW_OFF)
    for p in range(wl.n_prompts):
        a, _ = orc.prefix_range[p]
        assert raw[p] == a
        run = a + wl.header_len[p]
        for d in range(wl.doc_ptr[p], wl.doc_ptr[p + 1]):
            assert raw[wl.n_prompts + d] == run
            run += wl.doc_len[d]
    pool = B.hpd_layout_query(lay, B.HPD_Q_POOL_BYTES)
    eb = 4 if wl.dtype == "f32" else 2
    assert pool[2] == wl.n_branches * wl.max_new * wl.n_kv_heads * wl.head_dim * eb
    units = B.hpd_layout_query(lay, B.HPD_Q_N_UNITS)
    for t in range(wl.max_new):
        alive_docs = len(set(np.searchsorted(wl.branch_ptr, orc.live(t), side="right") - 1))
        assert units[t] == alive_docs


def test_paper_gap_mode_matches_oracle_and_worked_example():
    # the worked example of Section 4.3.2: 10-token prompt, three 3-token attributes, K_max 7
    wl = W.make_workload("fig2", "f32", 2, 2, 16, 10000.0, 7, [4], [1], [6], [3], branch_len=[3, 3, 3])
    lay = _host_layout(wl, B.HPD_POS_PAPER_GAP, attr_len=[3, 3, 3])
    base = B.hpd_layout_query(lay, B.HPD_Q_BRANCH_BASE_POS)
    assert list(base) == [12, 22, 32]
    assert list(base + 1) == [13, 23, 33]
    # random ragged batch against the oracle's Algorithm 2
    wl = W.random_workload(5, t=6, p=4)
    attr = np.random.default_rng(1).integers(1, 6, size=wl.n_branches)
    lay = _host_layout(wl, B.HPD_POS_PAPER_GAP, attr_len=attr)
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len,
                      wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new,
                      pos_mode="paper_gap", attr_len=attr)
    base = B.hpd_layout_query(lay, B.HPD_Q_BRANCH_BASE_POS).astype(np.int64)
    for t in range(wl.max_new):
        live = orc.live(t)
        assert np.array_equal(base[live] + 1 + t, orc.positions(t))
    pos0 = B.hpd_layout_query(lay, B.HPD_Q_SEG_POS0)
    for p, po in orc.prompts.items():
        for j, d in enumerate(range(wl.doc_ptr[p], wl.doc_ptr[p + 1])):
            assert pos0[wl.n_prompts + d] == po.doc_pos0[j]


def test_invalid_inputs_return_error_codes():
    wl = W.config(1)
    cfg = B.config_from_workload(wl, flags=B.HPD_FLAG_HOST_ONLY)

    def build(**kw):
        args = dict(header_len=wl.header_len, doc_ptr=wl.doc_ptr, doc_len=wl.doc_len,
                    branch_ptr=wl.branch_ptr, branch_len=wl.branch_len)
        args.update(kw)
        return B.hpd_build_layout(cfg, **args)

    with pytest.raises(B.HpdError) as e:
        build(branch_len=[9, 1, 1, 1])  # longer than K_max = 8
    assert e.value.status == B.HPD_E_INVALID
    with pytest.raises(B.HpdError):
        build(branch_len=[0, 1, 1, 1])
    with pytest.raises(B.HpdError):
        build(doc_ptr=[0, -1])  # non-monotone CSR
    with pytest.raises(B.HpdError):
        build(doc_len=[0])
    with pytest.raises(B.HpdError):
        build(header_len=[-1])
    with pytest.raises(B.HpdError):
        build(branch_ptr=[0, -1])
    bad = B.config_from_workload(wl, flags=B.HPD_FLAG_HOST_ONLY)
    bad.head_dim = 63
    with pytest.raises(B.HpdError):
        B.hpd_build_layout(bad, wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr)
    bad = B.config_from_workload(wl, flags=B.HPD_FLAG_HOST_ONLY)
    bad.n_kv_heads = 3
    with pytest.raises(B.HpdError):
        B.hpd_build_layout(bad, wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr)
    bad = B.config_from_workload(wl, pos_mode=B.HPD_POS_PAPER_GAP, flags=B.HPD_FLAG_HOST_ONLY)
    with pytest.raises(B.HpdError):  # gap mode needs attribute lengths
        B.hpd_build_layout(bad, wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr)
    # a host-only layout refuses device calls instead of crashing
    lay = build()
    with pytest.raises(B.HpdError):
        B.hpd_rope_positions(lay, 0, 0)
    # so do the device-side pruning calls; the state does not exist before hpd_dynamic_begin
    with pytest.raises(B.HpdError) as e:
        B.hpd_dynamic_begin(lay)
    assert e.value.status == B.HPD_E_INVALID
    with pytest.raises(B.HpdError):
        B.hpd_dynamic_state(lay)
    with pytest.raises(B.HpdError):
        B.hpd_dynamic_read(lay, 4)
    assert B.hpd_status_string(B.HPD_E_INVALID) == "invalid argument"


def test_finetune_mask_host_checks():
    """No GPU call: sizes and argument checks of hpd_finetune_mask (outputs NULL)."""
    assert B.hpd_finetune_mask(10, [3, 3, 3], [3, 3, 3], 7) == 28
    assert B.hpd_finetune_mask(0, [], [], 4) == 0
    for bad in [dict(prompt_len=-1, attr_len=[1], value_len=[1], k_max=2),
                dict(prompt_len=1, attr_len=[0], value_len=[1], k_max=2),
                dict(prompt_len=1, attr_len=[1], value_len=[3], k_max=2),
                dict(prompt_len=1, attr_len=[1], value_len=[1], k_max=0)]:
        with pytest.raises(B.HpdError):
            B.hpd_finetune_mask(**bad)
    with pytest.raises(B.HpdError):
        B.hpd_finetune_mask(46000, [1], [1], 2)  # S beyond the limit


def test_host_tables_under_the_literal_mask():
    """HPD_MASK_PAPER, host only: one skeleton segment per prompt after its documents, sized
    by the attribute lengths; token counts and input order agree with the oracle's."""
    wl = W.random_workload(17, t=4, p=3, j_range=(1, 3), n_range=(1, 4))
    attr = np.random.default_rng(17).integers(1, 5, size=wl.n_branches).astype(np.int32)
    lay = B.layout_from_workload(wl, pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr, mask_mode=B.HPD_MASK_PAPER,
                                 flags=B.HPD_FLAG_HOST_ONLY)
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len, wl.n_q_heads,
                      wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new, pos_mode="paper_gap",
                      attr_len=attr, mask_mode="paper")
    c = lay.counts()
    assert int(c[B.HPD_C_N_PREFIX_TOKENS]) == orc.n_prefix_tokens == wl.n_prefix_tokens + int(attr.sum())
    seg_len = B.hpd_layout_query(lay, B.HPD_Q_SEG_LEN)
    seg_off = B.hpd_layout_query(lay, B.HPD_Q_SEG_OFF)
    raw_off = B.hpd_layout_query(lay, B.HPD_Q_SEG_RAW_OFF)
    P, nd = wl.n_prompts, wl.n_docs
    assert len(seg_len) == 2 * P + nd
    for p in range(P):
        b0, b1 = wl.branch_ptr[wl.doc_ptr[p]], wl.branch_ptr[wl.doc_ptr[p + 1]]
        assert seg_len[P + nd + p] == attr[b0:b1].sum()
        assert seg_off[P + nd + p] % B.HPD_KEY_BLOCK == 0
        a0, a1 = orc.prefix_range[p]
        assert raw_off[p] == a0  # header first
        assert raw_off[P + nd + p] + seg_len[P + nd + p] == a1  # the names last
    # decode positions still follow Algorithm 2
    base = B.hpd_layout_query(lay, B.HPD_Q_BRANCH_BASE_POS)
    for p, po in orc.prompts.items():
        b0, b1 = orc.branch_range[p]
        assert list(base[b0:b1]) == po.base_pos
        assert po.skeleton_pos[-1] == po.base_pos[-1]


def test_rope_table_covers_the_step_budget_not_only_the_announced_lengths():
    """The device-side pruning calls ignore branch_len and may decode any branch up to step
    T - 1, so the (cos, sin) table must reach base_pos + T for every branch."""
    T = 8
    # the branch with the largest base position announces a single step
    wl = W.make_workload("short_len", "bf16", 4, 2, 128, 500000.0, T, [5], [2], [10, 40], [2, 3],
                         branch_len=[T, T, 1, 1, 1])
    lay = _host_layout(wl)
    base = B.hpd_layout_query(lay, B.HPD_Q_BRANCH_BASE_POS).astype(np.int64)
    assert int(lay.counts()[B.HPD_C_MAX_POS]) == int(base.max()) + T == 5 + 40 - 1 + T
    attr = np.asarray([2, 1, 3, 1, 2], dtype=np.int32)
    lay = _host_layout(wl, B.HPD_POS_PAPER_GAP, attr_len=attr)
    base = B.hpd_layout_query(lay, B.HPD_Q_BRANCH_BASE_POS).astype(np.int64)
    assert int(lay.counts()[B.HPD_C_MAX_POS]) == int(base.max()) + T
