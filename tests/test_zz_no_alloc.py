"""hpd_dynamic_begin_static - the allocation-free variant of hpd_dynamic_begin (state in a
file-scope device array) - against hpd_dynamic_begin through the C ABI: same live lists, same
counts, same output bits at every step, on two passes in a row over the shared array, the second
with a smaller batch; a layout beyond the array's size is refused."""
import numpy as np
import pytest
import torch

from paper_2604_26209_amd import workloads as W

import hpd_harness as H

pytestmark = pytest.mark.gpu


def _dynamic_pass(B, wl, lay, inputs, begin):
    """One decode pass with device-side lists; returns per step (n_live, live list, outputs)."""
    kp, vp, kt, vt = B.alloc_pools(lay)
    for x in (kp, vp, kt, vt):
        x.fill_(float("nan"))
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    begin(lay)
    res = []
    for t in range(wl.max_new):
        n, live = B.hpd_dynamic_read(lay, wl.n_branches)
        out = torch.full((max(n, 1), wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        if n:
            B.hpd_dynamic_step(lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, out)
        res.append((n, live.copy(), out[:n].clone()))
        if t + 1 < wl.max_new:
            fin = (wl.branch_len[live] == t + 1).astype(np.uint8) if n else np.zeros(1, np.uint8)
            B.hpd_dynamic_prune(lay, torch.from_numpy(fin).cuda())
    torch.cuda.synchronize()
    return res


@pytest.mark.parametrize("literal", [False, True])
def test_static_state_equals_allocated_state_on_two_passes_in_a_row(literal):
    from paper_2604_26209_amd import binding as B
    big = W.random_workload(140, dtype="bf16", d=128, base=500000.0, t=9, hq=8, hkv=2, p=4,
                            j_range=(1, 4), n_range=(1, 24), l_range=(1, 260), h_range=(0, 70))
    small = W.random_workload(141, dtype="bf16", d=128, base=500000.0, t=5, hq=8, hkv=2, p=2,
                              j_range=(1, 2), n_range=(1, 6), l_range=(1, 90), h_range=(0, 40))
    assert small.n_branches < big.n_branches and small.n_docs < big.n_docs
    for wl in (big, small):  # the second pass finds the first one's state in the shared array
        attr = np.random.default_rng(7).integers(1, 5, size=wl.n_branches).astype(np.int32)
        kw = dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr, mask_mode=B.HPD_MASK_PAPER) if literal else {}
        print(f"static pruning state: {wl.n_branches} branches, {wl.n_docs} documents, literal mask {literal}", flush=True)
        lay_a = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32, **kw)
        lay_s = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32, **kw)
        inputs = H.Inputs(wl, lay_a.n_live(), "cuda", lay_a.counts()[B.HPD_C_N_PREFIX_TOKENS])
        want = _dynamic_pass(B, wl, lay_a, inputs, B.hpd_dynamic_begin)
        got = _dynamic_pass(B, wl, lay_s, inputs, B.hpd_dynamic_begin_static)
        n_live = lay_a.n_live()
        for t, ((n0, live0, out0), (n1, live1, out1)) in enumerate(zip(want, got)):
            assert n0 == n1 == int(n_live[t]), f"step {t}: n_live {n1} != {n0}"
            assert np.array_equal(live0, live1), f"step {t}: live lists differ"
            assert bool(torch.isfinite(out1).all())
            assert torch.equal(out0, out1), f"step {t}: outputs differ"
        # the state the caller may read is the array's: the same address for every layout
        live_ptr, n_ptr = B.hpd_dynamic_state(lay_s)
        assert live_ptr != 0 and n_ptr != 0 and live_ptr != B.hpd_dynamic_state(lay_a)[0]
        # a layout goes back to a state of its own with hpd_dynamic_begin
        again = _dynamic_pass(B, wl, lay_s, inputs, B.hpd_dynamic_begin)
        assert all(torch.equal(a[2], b[2]) for a, b in zip(want, again))


def test_static_state_refuses_a_layout_beyond_its_size():
    from paper_2604_26209_amd import binding as B
    n_docs = B.HPD_DYNAMIC_STATIC_MAX_BYTES // 32 + 8  # 8 words of descriptor per document alone exceed the array
    wl = W.make_workload("many_docs", "bf16", 8, 2, 128, 500000.0, 2, [4], [n_docs], [1] * n_docs, [1] * n_docs)
    lay = B.layout_from_workload(wl)
    with pytest.raises(B.HpdError) as e:
        B.hpd_dynamic_begin_static(lay)
    assert e.value.status == B.HPD_E_CAPACITY
    assert "scratch" in str(e.value)
    with pytest.raises(B.HpdError):  # no state was bound
        B.hpd_dynamic_state(lay)
    B.hpd_dynamic_begin(lay)  # the allocating call takes it
    n, live = B.hpd_dynamic_read(lay, wl.n_branches)
    assert n == n_docs and np.array_equal(live, np.arange(n_docs))
