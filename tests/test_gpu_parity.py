"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integers (positions, slots, masks) bit-exact; outputs within 1e-4 max-abs
(fp32) or 2e-2 x RMS (bf16)."""
import numpy as np
import pytest
import torch

from paper_2604_26209_amd import workloads as W

import hpd_harness as H

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def test_cfg1_fp32_all_steps_two_call_and_fused():
    wl = W.config(1)
    _say("cfg1 two-call")
    hip = H.run_hip(wl)
    err = H.check_all(wl, hip, label="cfg1")
    _say(f"cfg1 max-abs {err:.2e}")
    _say("cfg1 fused")
    hip2 = H.run_hip(wl, inputs=hip["inputs"], fused=True)
    for a, b in zip(hip["out"], hip2["out"]):
        assert torch.equal(a, b)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_ragged_fp32(seed):
    _say(f"random fp32 seed {seed}")
    wl = W.random_workload(seed, dtype="f32", hq=4, hkv=2, d=64, t=6, p=3)
    hip = H.run_hip(wl)
    H.check_all(wl, hip, label=f"rand_f32_{seed}")


def test_fp32_other_head_dims_and_empty_header():
    for d, hq, hkv in [(32, 2, 1), (128, 4, 4), (96, 3, 1)]:
        _say(f"fp32 D={d}")
        wl = W.random_workload(40 + d, dtype="f32", hq=hq, hkv=hkv, d=d, t=3, p=2, h_range=(0, 0),
                               l_range=(1, 40))
        H.check_all(wl, H.run_hip(wl), label=f"f32_D{d}")


@pytest.mark.parametrize("mode", [1, 2, 3, 4])
@pytest.mark.parametrize("seed", [11, 12])
def test_random_ragged_bf16_both_kernels(seed, mode):
    """mode 1 = generic wave-reduction kernel, 2 = LDS-streaming MFMA kernel (the default for
    this shape), 3 / 4 = the same with the wide / narrow workgroup shape forced."""
    _say(f"random bf16 seed {seed} mode {mode}")
    wl = W.random_workload(seed, dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=5, p=3,
                           h_range=(0, 70), l_range=(1, 150), n_range=(1, 12))
    hip = H.run_hip(wl, kernel_mode=mode)
    rel = H.check_all(wl, hip, label=f"rand_bf16_{seed}_m{mode}")
    _say(f"  worst err/rms {rel:.2e}")


@pytest.mark.parametrize("mode", [3, 4])
@pytest.mark.parametrize("g", [1, 2, 4, 8])
def test_stream_kernel_fused_step_equals_two_calls(g, mode):
    """hpd_decode_step (one launch, append inside the attention kernel) against
    hpd_kv_append + hpd_decode_attention: same tail pools, same outputs, bit for bit."""
    _say(f"stream fused vs two-call G={g} mode {mode}")
    wl = W.random_workload(60 + g, dtype="bf16", hq=8, hkv=8 // g, d=128, base=500000.0, t=6, p=3,
                           h_range=(0, 90), l_range=(1, 300), n_range=(1, 14))
    a = H.run_hip(wl, kernel_mode=mode, fused=False, poison_pools="zero")
    b = H.run_hip(wl, inputs=a["inputs"], kernel_mode=mode, fused=True, poison_pools="zero")
    for x, y in zip(a["out"], b["out"]):
        assert torch.equal(x, y)
    for x, y in zip(a["pools"][2:], b["pools"][2:]):
        assert torch.equal(x, y)
    rel = H.check_all(wl, b, label=f"stream_fused_g{g}")
    _say(f"  worst err/rms {rel:.2e}")


@pytest.mark.parametrize("seed", range(100, 108))
def test_random_layout_sweep_stream_kernel(seed):
    """Random small batches through the step call: group size, head count, number of steps
    (up to four chunks of tail positions), ragged lengths, document and branch counts all
    drawn from the seed; all workgroup shapes."""
    rng = np.random.default_rng(seed)
    g = int(rng.choice([1, 2, 4, 8]))
    hkv = int(rng.choice([1, 2, 4]))
    t = int(rng.integers(1, 27))
    wl = W.random_workload(seed, dtype="bf16", hq=hkv * g, hkv=hkv, d=128, base=500000.0, t=t,
                           p=int(rng.integers(1, 4)), j_range=(1, 3), n_range=(1, int(rng.integers(2, 40))),
                           h_range=(0, int(rng.integers(1, 100))), l_range=(1, int(rng.integers(2, 400))))
    for mode in (3, 4):
        _say(f"sweep seed {seed}: G={g} Hkv={hkv} T={t} branches={wl.n_branches} mode {mode}")
        hip = H.run_hip(wl, kernel_mode=mode, fused=True)
        H.check_all(wl, hip, label=f"sweep_{seed}_m{mode}")


@pytest.mark.parametrize("mode", [3, 4])
@pytest.mark.parametrize("case", ["tiny_prefix", "many_branches", "no_header_one_key"])
def test_tail_tile_formats_of_the_newest_chunk(case, mode):
    """The newest chunk of tail positions is cut into tiles of 1 x 32, 2 x 16, 4 x 8 or 8 x 4
    (positions x branches) depending on how many positions it holds: every step 0..11 goes through
    each format at least once, with full chunks behind it from step 8 on.  Cases: prefixes so short
    that a tile of the newest chunk is among the first requests (its row table is then written
    before the loaders start); documents with more branches than one tile or one row block holds
    (tiles that span row blocks, ragged last tile); no header and a one-token document.  Every
    group size; fused = two-call bit for bit; against the oracle."""
    kw = dict(tiny_prefix=dict(p=3, j_range=(1, 3), n_range=(1, 40), h_range=(0, 20), l_range=(1, 40)),
              many_branches=dict(p=2, j_range=(1, 2), n_range=(30, 70), h_range=(0, 70), l_range=(1, 300)),
              no_header_one_key=dict(p=2, j_range=(1, 3), n_range=(1, 35), h_range=(0, 0), l_range=(1, 1)))[case]
    for g in (1, 2, 4, 8):
        _say(f"tile formats: {case} G={g} mode {mode}")
        wl = W.random_workload(300 + g, dtype="bf16", hq=8, hkv=8 // g, d=128, base=500000.0, t=12, **kw)
        a = H.run_hip(wl, kernel_mode=mode, fused=True)
        rel = H.check_all(wl, a, label=f"fmt_{case}_g{g}_m{mode}")
        b = H.run_hip(wl, inputs=a["inputs"], kernel_mode=mode, fused=False)
        for x, y in zip(a["out"], b["out"]):
            assert torch.equal(x, y)
        _say(f"  worst err/rms {rel:.2e}")


@pytest.mark.parametrize("mode", [1, 3, 4])
@pytest.mark.parametrize("case", ["peaked_x4", "argmax_x16", "flat_div16", "common_offset", "rising"])
def test_score_ranges_of_the_online_softmax(case, mode):
    """Inputs other than N(0,1): scores 4 and 16 times as wide (rows that one or two keys
    dominate, up to an argmax), 16 times as narrow (a flat average), with a large common
    component in queries and keys (every score near +16 in log2 units: the reference point of
    the exponentials must follow), and with keys that grow along the document and the steps (the
    maximum of a row keeps rising, block after block: the accumulators are rescaled again and
    again).  Same tolerance as everywhere; generic kernel (mode 1) and all workgroup shapes."""
    wl = W.random_workload(400, dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=11, p=2,
                           j_range=(1, 3), n_range=(1, 20), h_range=(0, 70), l_range=(40, 400))
    from paper_2604_26209_amd import binding as B
    lay = B.layout_from_workload(wl)
    inp = H.Inputs(wl, lay.n_live(), "cuda", lay.counts()[B.HPD_C_N_PREFIX_TOKENS])
    bf = lambda x: x.float().to(torch.bfloat16)
    if case in ("peaked_x4", "argmax_x16", "flat_div16"):
        f = dict(peaked_x4=4.0, argmax_x16=16.0, flat_div16=1.0 / 16)[case]
        inp.q = [bf(x.float() * f) for x in inp.q]
    elif case == "common_offset":
        inp.q = [bf(x.float() + 1.0) for x in inp.q]
        inp.k_raw = bf(inp.k_raw.float() + 1.0)
        inp.k_new = [bf(x.float() + 1.0) for x in inp.k_new]
    else:
        # a component along which all queries point and the keys grow with their index
        n = inp.k_raw.shape[0]
        ramp = torch.arange(n, device="cuda", dtype=torch.float32)[:, None, None] * (4.0 / max(n, 1))
        inp.k_raw = bf(inp.k_raw.float() + ramp)
        inp.k_new = [bf(x.float() + 4.0 + 0.3 * t) for t, x in enumerate(inp.k_new)]
        inp.q = [bf(x.float() * 0.5 + 1.0) for x in inp.q]
    _say(f"score ranges: {case} mode {mode}")
    a = H.run_hip(wl, inputs=inp, kernel_mode=mode, fused=mode != 1)
    rel = H.check_all(wl, a, label=f"{case}_m{mode}")
    _say(f"  worst err/rms {rel:.2e}")


def test_values_beyond_the_half_range_saturate():
    """The pools hold their bf16 values in half format, which ends at 65504: keys and values of
    larger magnitude (bf16 can carry them) are stored as +-65504.  Nothing overflows - every output
    stays finite, also in the rows that attend to such elements -, and the prompts without such
    elements are unaffected (same tolerance against the oracle as ever)."""
    wl = W.random_workload(410, dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=6, p=3,
                           j_range=(1, 3), n_range=(2, 12), h_range=(10, 70), l_range=(40, 200))
    from paper_2604_26209_amd import binding as B
    lay = B.layout_from_workload(wl)
    inp = H.Inputs(wl, lay.n_live(), "cuda", lay.counts()[B.HPD_C_N_PREFIX_TOKENS])
    # prompt 0 only: a few huge elements in its header, its first document and its new rows
    h0 = int(wl.header_len[0])
    big = torch.tensor(1.0e5, dtype=torch.bfloat16, device="cuda")
    inp.k_raw[1, 0, 5] = big
    inp.k_raw[h0 + 3, 1, 70] = -big
    inp.v_raw[2, 0, 9] = big
    inp.v_raw[h0 + 4, 1, 100] = -big
    inp.k_new[0][0, 0, 17] = big
    inp.v_new[1][0, 1, 3] = big
    for mode in (3, 4):
        _say(f"saturation mode {mode}")
        a = H.run_hip(wl, inputs=inp, kernel_mode=mode, fused=True)
        for o in a["out"]:
            assert bool(torch.isfinite(o.float()).all())
        H.check_all(wl, a, prompts=[1, 2], label=f"saturate_m{mode}")


@pytest.mark.parametrize("g", [3, 5, 6, 7])
def test_stream_kernel_group_sizes_that_are_not_powers_of_two(g):
    """Group sizes such as 40 query heads over 8 kv heads (5) run on the streaming kernel with
    the rows of a branch padded to the next power of two; padding rows are neither loaded nor
    stored.  Decode (both masks, fused = two-call) and prefill, all workgroup shapes."""
    rng = np.random.default_rng(190 + g)
    hkv = int(rng.choice([1, 2]))
    wl = W.random_workload(190 + g, dtype="bf16", hq=hkv * g, hkv=hkv, d=128, base=500000.0,
                           t=int(rng.integers(2, 20)), p=3, j_range=(1, 3), n_range=(1, 30),
                           h_range=(0, 100), l_range=(1, 300))
    attr = rng.integers(1, 5, size=wl.n_branches).astype(np.int32)
    from paper_2604_26209_amd import binding as B
    for paper in (False, True):
        kw = dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr, mask_mode=B.HPD_MASK_PAPER) if paper else {}
        okw = dict(pos_mode="paper_gap", attr_len=attr, mask_mode="paper") if paper else {}
        for mode in (3, 4):
            _say(f"G={g} Hkv={hkv} T={wl.max_new} branches={wl.n_branches} literal={paper} mode {mode}")
            a = H.run_hip(wl, kernel_mode=mode, fused=True, **kw)
            H.check_all(wl, a, label=f"g{g}_m{mode}", **okw)
            b = H.run_hip(wl, inputs=a["inputs"], kernel_mode=mode, fused=False, **kw)
            for x, y in zip(a["out"], b["out"]):
                assert torch.equal(x, y)
            _check_prefill(wl, mode, f"g{g}_prefill_m{mode}", attr_len=attr if paper else None)
        _check_prefill(wl, 0, f"g{g}_prefill_m0", attr_len=attr if paper else None)


@pytest.mark.parametrize("seed,kw", [(120, dict(hq=8, hkv=2, p=3, j_range=(1, 4), n_range=(1, 14), l_range=(1, 200))),
                                     (121, dict(hq=8, hkv=8, p=2, j_range=(2, 3), n_range=(3, 40), l_range=(1, 90))),
                                     (122, dict(hq=16, hkv=2, p=2, j_range=(1, 2), n_range=(1, 30), l_range=(30, 300)))])
def test_device_side_pruning_equals_host_lists(seed, kw):
    """hpd_dynamic_*: the live list is built on the GPU from per-row "finished" flags (here: a
    branch is flagged in the step that exhausts its length).  The device-side live list and
    count must equal the layout's host-built lists of every step, and hpd_dynamic_step must
    write the very bits hpd_decode_step writes."""
    from paper_2604_26209_amd import binding as B
    wl = W.random_workload(seed, dtype="bf16", d=128, base=500000.0, t=10, h_range=(0, 70), **kw)
    ref = H.run_hip(wl, fused=True)
    lay = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32)
    inputs = ref["inputs"]
    kp, vp, kt, vt = B.alloc_pools(lay)
    for x in (kp, vp, kt, vt):
        x.fill_(float("nan"))
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    B.hpd_dynamic_begin(lay)
    live_ptr, n_ptr = B.hpd_dynamic_state(lay)
    assert live_ptr != 0 and n_ptr != 0
    n_live = lay.n_live()
    live_flat = B.hpd_layout_query(lay, B.HPD_Q_LIVE_BRANCH)
    off = 0
    for t in range(wl.max_new):
        n = int(n_live[t])
        want_live = live_flat[off:off + n]
        off += n
        got_n, got_live = B.hpd_dynamic_read(lay, wl.n_branches)
        assert got_n == n, f"step {t}: n_live {got_n} != {n}"
        assert np.array_equal(got_live, want_live), f"step {t}: live list differs"
        out = torch.full((max(n, 1), wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        if n:
            B.hpd_dynamic_step(lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, out)
            assert torch.equal(out[:n], ref["out"][t]), f"step {t}: outputs differ from hpd_decode_step"
        if t + 1 < wl.max_new:
            fin = torch.from_numpy((wl.branch_len[want_live] == t + 1).astype(np.uint8)).cuda() if n else \
                torch.zeros(1, dtype=torch.uint8, device="cuda")
            B.hpd_dynamic_prune(lay, fin)
    with pytest.raises(B.HpdError):
        B.hpd_dynamic_step(lay, 0, inputs.q[0], inputs.k_new[0], inputs.v_new[0], kp, vp, kt, vt, out)  # wrong step


@pytest.mark.parametrize("literal", [False, True])
@pytest.mark.parametrize("seed", [130, 131])
def test_device_side_pruning_with_lengths_unknown_to_the_layout(seed, literal):
    """The use the entry points exist for: the layout is built with every branch at the full
    step budget (nobody knows yet where a branch ends), and branches leave when the caller
    flags them (the stop condition of Section 4.3.4).  With flags taken from a hidden
    length per branch, every step must match the oracle run on the workload that has those
    lengths.  Under the literal mask a branch that has left stays visible to the later ones
    as far as it got: the device keeps the number of tokens it reached."""
    import dataclasses
    from paper_2604_26209_amd import binding as B
    wl = W.random_workload(seed, dtype="bf16", d=128, base=500000.0, t=9, hq=8, hkv=2, p=3,
                           j_range=(1, 3), n_range=(1, 20), l_range=(1, 260), h_range=(0, 50))
    cap = dataclasses.replace(wl, branch_len=np.full(wl.n_branches, wl.max_new, dtype=np.int32))
    attr = np.random.default_rng(seed).integers(1, 5, size=wl.n_branches).astype(np.int32)
    kw = dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr, mask_mode=B.HPD_MASK_PAPER) if literal else {}
    okw = dict(pos_mode="paper_gap", attr_len=attr, mask_mode="paper") if literal else {}
    ref = H.run_hip(wl, fused=True, **kw)  # for the inputs, positions and slots of the hidden lengths
    inputs = ref["inputs"]
    lay = B.layout_from_workload(cap, out_dtype=B.HPD_OUT_F32, **kw)
    kp, vp, kt, vt = B.alloc_pools(lay)
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    B.hpd_dynamic_begin(lay)
    outs = []
    for t in range(wl.max_new):
        live = np.nonzero(wl.branch_len > t)[0]
        got_n, got_live = B.hpd_dynamic_read(lay, wl.n_branches)
        assert got_n == len(live) and np.array_equal(got_live, live), f"step {t}: live list differs"
        out = torch.full((max(len(live), 1), wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32,
                         device="cuda")
        if len(live):
            B.hpd_dynamic_step(lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, out)
        outs.append(out[:len(live)])
        if t + 1 < wl.max_new:
            fin = (wl.branch_len[live] == t + 1).astype(np.uint8) if len(live) else np.zeros(1, np.uint8)
            B.hpd_dynamic_prune(lay, torch.from_numpy(fin).cuda())
    hip = dict(ref)
    hip["out"] = outs
    H.check_all(wl, hip, label=f"dynamic_{seed}", **okw)


class _PageAllocator:
    """Host-side page allocator of the paged-tail tests: pages come from a shuffled free list,
    a branch takes one when it reaches a page boundary and gives all of them back when it
    ends, so pages are reused and hold stale rows of other branches."""

    def __init__(self, wl, page_size, seed):
        self.wl, self.ps = wl, page_size
        self.ppb = -(-wl.max_new // page_size)
        need, held = 0, 0
        for t in range(wl.max_new):  # pages in use at the same time
            if t % page_size == 0:
                held += int((wl.branch_len > t).sum())
            need = max(need, held)
            held -= int(((wl.branch_len == t + 1) * (-(-(t + 1) // page_size))).sum())
        self.n_pages = max(need, 1)
        self.free = list(np.random.default_rng(seed).permutation(self.n_pages))
        self.table = np.full((wl.n_branches, self.ppb), -7, dtype=np.int32)  # -7: never assigned

    def before_step(self, t):
        if t % self.ps == 0:
            for b in np.nonzero(self.wl.branch_len > t)[0]:
                self.table[b, t // self.ps] = self.free.pop()

    def after_step(self, t):
        for b in np.nonzero(self.wl.branch_len == t + 1)[0]:
            for i in range(self.ppb):
                if self.table[b, i] >= 0:
                    self.free.append(int(self.table[b, i]))
                    self.table[b, i] = -7

    def slots(self, live, t):
        return self.table[live, t // self.ps].astype(np.int64) * self.ps + t % self.ps


@pytest.mark.parametrize("case", ["stream_fused", "stream_two_call", "generic_f32", "dynamic"])
def test_paged_tails(case):
    """hpd_set_tail_pages: tail pools of n_pages pages (fewer than B * T slots; pages of ended
    branches are reused) against the contiguous pools: same outputs bit for bit, slots as the
    page table says, and within tolerance of the oracle."""
    from paper_2604_26209_amd import binding as B
    _say(f"paged tails: {case}")
    f32 = case == "generic_f32"
    if f32:
        wl = W.random_workload(140, dtype="f32", hq=4, hkv=2, d=64, t=19, p=2, n_range=(1, 9))
    else:
        wl = W.random_workload(141, dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=21, p=3,
                               j_range=(1, 3), n_range=(1, 14), h_range=(0, 80), l_range=(1, 200))
    ps = 8
    ref = H.run_hip(wl, fused=(case != "stream_two_call"))
    inputs = ref["inputs"]
    lay = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_SAME if f32 else B.HPD_OUT_F32)
    alloc = _PageAllocator(wl, ps, seed=7)
    assert alloc.n_pages * ps < wl.n_branches * wl.max_new, "the case must save memory"
    table = torch.from_numpy(alloc.table).cuda()
    full = B.hpd_layout_query(lay, B.HPD_Q_POOL_BYTES)
    B.hpd_set_tail_pages(lay, ps, alloc.n_pages, table)
    paged = B.hpd_layout_query(lay, B.HPD_Q_POOL_BYTES)
    assert paged[2] * wl.n_branches * wl.max_new == full[2] * alloc.n_pages * ps and paged[0] == full[0]
    kp, vp, kt, vt = B.alloc_pools(lay)
    for x in (kp, vp, kt, vt):
        x.fill_(float("nan"))
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    if case == "dynamic":
        B.hpd_dynamic_begin(lay)
    outs = []
    for t in range(wl.max_new):
        live = np.nonzero(wl.branch_len > t)[0]
        n = len(live)
        alloc.before_step(t)
        table.copy_(torch.from_numpy(alloc.table))
        out = torch.full((n, wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        slot = torch.full((max(n, 1),), -1, dtype=torch.int64, device="cuda")
        if n:
            a = (lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, out)
            if case == "dynamic":
                B.hpd_dynamic_step(*a)
            elif case == "stream_two_call":
                B.hpd_kv_append(lay, t, inputs.k_new[t], inputs.v_new[t], kt, vt, slot)
                B.hpd_decode_attention(lay, t, inputs.q[t], kp, vp, kt, vt, out)
                assert np.array_equal(slot[:n].cpu().numpy(), alloc.slots(live, t)), f"step {t}: slots"
            else:
                B.hpd_decode_step(*a)
            assert torch.equal(out, ref["out"][t]), f"step {t}: paged and contiguous outputs differ"
        outs.append(out)
        if case == "dynamic" and t + 1 < wl.max_new:
            fin = (wl.branch_len[live] == t + 1).astype(np.uint8) if n else np.zeros(1, np.uint8)
            B.hpd_dynamic_prune(lay, torch.from_numpy(fin).cuda())
        torch.cuda.synchronize()  # the table is rewritten on the host for the next step
        alloc.after_step(t)
    hip = dict(ref)
    hip["out"] = outs
    H.check_all(wl, hip, label=f"paged_{case}")
    # switching paging off restores the contiguous sizes; bad arguments are refused
    B.hpd_set_tail_pages(lay, 0)
    assert np.array_equal(B.hpd_layout_query(lay, B.HPD_Q_POOL_BYTES), full)
    for bad in (4, 12, -8):
        with pytest.raises(B.HpdError):
            B.hpd_set_tail_pages(lay, bad, 4, table)
    with pytest.raises(B.HpdError):
        B.hpd_set_tail_pages(lay, 8, 0, table)
    with pytest.raises(B.HpdError):
        B.hpd_set_tail_pages(lay, 8, 4, None)


@pytest.mark.parametrize("seed", range(150, 158))
def test_paged_tails_random_sweep(seed):
    """Page size, group size, workgroup shape, step budget and batch drawn from the seed: the
    paged step call against the contiguous one, bit for bit.  Odd seeds use the device-side
    lists, whose launches split a document's rows by its full branch count (the host does not
    know the live count), so sums may be grouped differently than in hpd_decode_step: those
    are checked against the oracle."""
    from paper_2604_26209_amd import binding as B
    rng = np.random.default_rng(seed)
    g = (1, 2, 4, 8)[seed % 4]
    hkv = int(rng.choice([1, 2]))
    ps = (8, 16, 32)[seed % 3]
    t_max = int(rng.integers(2, 41))
    mode = 3 + (seed // 2) % 2
    wl = W.random_workload(seed, dtype="bf16", hq=hkv * g, hkv=hkv, d=128, base=500000.0, t=t_max,
                           p=int(rng.integers(1, 4)), j_range=(1, 3), n_range=(1, int(rng.integers(2, 30))),
                           h_range=(0, 60), l_range=(1, int(rng.integers(2, 300))))
    _say(f"paged sweep seed {seed}: G={g} Hkv={hkv} T={t_max} page {ps} mode {mode} branches {wl.n_branches}")
    ref = H.run_hip(wl, kernel_mode=mode, fused=True)
    inputs = ref["inputs"]
    lay = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32)
    B.hpd_set_kernel_mode(lay, mode)
    alloc = _PageAllocator(wl, ps, seed=seed)
    table = torch.from_numpy(alloc.table).cuda()
    B.hpd_set_tail_pages(lay, ps, alloc.n_pages, table)
    kp, vp, kt, vt = B.alloc_pools(lay)
    for x in (kp, vp, kt, vt):
        x.fill_(float("nan"))
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    dynamic = seed % 2 == 1
    if dynamic:
        B.hpd_dynamic_begin(lay)
    outs = []
    for t in range(wl.max_new):
        live = np.nonzero(wl.branch_len > t)[0]
        if len(live) == 0:
            break
        alloc.before_step(t)
        table.copy_(torch.from_numpy(alloc.table))
        out = torch.full((len(live), wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        a = (lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, out)
        (B.hpd_dynamic_step if dynamic else B.hpd_decode_step)(*a)
        if not dynamic:
            assert torch.equal(out, ref["out"][t]), f"seed {seed} step {t}: paged and contiguous outputs differ"
        outs.append(out)
        if dynamic and t + 1 < wl.max_new:
            B.hpd_dynamic_prune(lay, torch.from_numpy((wl.branch_len[live] == t + 1).astype(np.uint8)).cuda())
        torch.cuda.synchronize()
        alloc.after_step(t)
    while len(outs) < wl.max_new:
        outs.append(torch.zeros((0, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device="cuda"))
    hip = dict(ref)
    hip["out"] = outs
    H.check_all(wl, hip, label=f"paged_sweep_{seed}")


@pytest.mark.parametrize("dynamic", [False, True])
def test_decode_pass_replayed_from_a_hip_graph(dynamic):
    """The step calls only enqueue kernels (no allocation, no synchronisation, no memset), so a
    whole decode pass can be captured in a HIP graph.  The graph is replayed three times, with
    eager work and synchronisations in between (tails cleared, outputs poisoned), and every
    replay must reproduce the eager pass bit for bit."""
    from paper_2604_26209_amd import binding as B
    wl = W.random_workload(180, dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=9, p=3,
                           j_range=(1, 3), n_range=(1, 10), h_range=(0, 60), l_range=(1, 150))
    ref = H.run_hip(wl, fused=True)
    inputs = ref["inputs"]
    lay = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32)
    kp, vp, kt, vt = B.alloc_pools(lay)
    kp.zero_(), vp.zero_()
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    n_live = lay.n_live()
    outs = [torch.zeros((int(n_live[t]), wl.n_q_heads, wl.head_dim), dtype=torch.float32, device="cuda")
            for t in range(wl.max_new)]
    fins = [torch.from_numpy((wl.branch_len[np.nonzero(wl.branch_len > t)[0]] == t + 1).astype(np.uint8)).cuda()
            for t in range(wl.max_new)]

    def one_pass():
        if dynamic:
            B.hpd_dynamic_begin(lay)
        for t in range(wl.max_new):
            if int(n_live[t]) == 0:
                break
            a = (lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, outs[t])
            (B.hpd_dynamic_step if dynamic else B.hpd_decode_step)(*a)
            if dynamic and t + 1 < wl.max_new and int(n_live[t + 1]) > 0:
                B.hpd_dynamic_prune(lay, fins[t])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_pass()  # also the first hpd_dynamic_begin, which allocates and synchronises
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one_pass()
    for rep in range(3):
        kt.fill_(float("nan")), vt.fill_(float("nan"))
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for t in range(wl.max_new):
            assert torch.equal(outs[t], ref["out"][t]), f"replay {rep} step {t}: differs from the eager pass"


@pytest.mark.parametrize("dynamic", [False, True])
def test_paged_tails_under_the_literal_mask(dynamic):
    """Under HPD_MASK_PAPER a branch that has left is still read by the later branches of its
    prompt, so its pages stay; the pools still hold only the pages that were ever reached.
    Paged step calls (host lists / device-side lists) against the contiguous ones."""
    from paper_2604_26209_amd import binding as B
    wl = W.random_workload(143 + int(dynamic), dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=20, p=3,
                           j_range=(1, 3), n_range=(1, 12), h_range=(0, 60), l_range=(1, 150))
    attr = np.random.default_rng(143).integers(1, 5, size=wl.n_branches).astype(np.int32)
    kw = dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr, mask_mode=B.HPD_MASK_PAPER)
    ref = H.run_hip(wl, fused=True, **kw)
    inputs = ref["inputs"]
    lay = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32, **kw)
    ps = 8
    ppb = -(-wl.max_new // ps)
    need = int(np.sum(-(-wl.branch_len // ps)))  # pages ever reached
    assert need < wl.n_branches * ppb
    order = list(np.random.default_rng(5).permutation(need))
    table_h = np.full((wl.n_branches, ppb), -7, dtype=np.int32)
    table = torch.from_numpy(table_h).cuda()
    B.hpd_set_tail_pages(lay, ps, need, table)
    kp, vp, kt, vt = B.alloc_pools(lay)
    for x in (kp, vp, kt, vt):
        x.fill_(float("nan"))
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    if dynamic:
        B.hpd_dynamic_begin(lay)
    outs = []
    for t in range(wl.max_new):
        live = np.nonzero(wl.branch_len > t)[0]
        if t % ps == 0:
            for b in live:
                table_h[b, t // ps] = order.pop()
            table.copy_(torch.from_numpy(table_h))
        out = torch.full((len(live), wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        if len(live):
            a = (lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, out)
            (B.hpd_dynamic_step if dynamic else B.hpd_decode_step)(*a)
            if not dynamic:
                assert torch.equal(out, ref["out"][t]), f"step {t}: paged and contiguous outputs differ"
        outs.append(out)
        if dynamic and t + 1 < wl.max_new:
            fin = (wl.branch_len[live] == t + 1).astype(np.uint8) if len(live) else np.zeros(1, np.uint8)
            B.hpd_dynamic_prune(lay, torch.from_numpy(fin).cuda())
        torch.cuda.synchronize()
    assert not order
    hip = dict(ref)
    hip["out"] = outs
    H.check_all(wl, hip, label="paged_literal", pos_mode="paper_gap", attr_len=attr, mask_mode="paper")


def test_bf16_output_is_the_fp32_output_rounded_once():
    """out_dtype = SAME writes RNE(bf16) of exactly the values out_dtype = F32 writes."""
    _say("bf16 out == rne(fp32 out)")
    wl = W.config(2, n_prompts=3)
    for mode in (1, 3, 4):
        a = H.run_hip(wl, kernel_mode=mode, out_f32=True)
        b = H.run_hip(wl, inputs=a["inputs"], kernel_mode=mode, out_f32=False)
        for x, y in zip(a["out"], b["out"]):
            assert y.dtype == torch.bfloat16 and torch.equal(x.to(torch.bfloat16), y)


def test_mfma_edge_shapes():
    cases = {
        "single_branch_h0_l1": W.make_workload("e1", "bf16", 4, 1, 128, 500000.0, 3, [0], [1], [1], [1]),
        "mha_g1": W.make_workload("e2", "bf16", 2, 2, 128, 500000.0, 2, [5], [1], [33], [3]),
        "many_rows_two_row_groups": W.make_workload("e3", "bf16", 16, 2, 128, 500000.0, 2, [40], [1],
                                                    [100], [40]),  # 8*40 = 320 rows -> 10 blocks
        "exact_blocks": W.make_workload("e4", "bf16", 8, 2, 128, 500000.0, 4, [64], [2], [128, 96], [8, 16]),
        "t1": W.make_workload("e5", "bf16", 8, 8, 128, 500000.0, 1, [7], [1], [9], [5]),
        "long_tail": W.make_workload("e6", "bf16", 8, 2, 128, 500000.0, 40, [33], [1], [70], [9]),
        "nine_row_blocks": W.make_workload("e7", "bf16", 8, 1, 128, 500000.0, 2, [10], [2], [50, 45], [35, 3]),
    }
    for name, wl in cases.items():
        for mode in (3, 4):
            for fused in (False, True):
                _say(f"mfma edge {name} mode {mode} fused {fused}")
                hip = H.run_hip(wl, kernel_mode=mode, fused=fused)
                H.check_all(wl, hip, label=name)


def test_paper_gap_positions_mode():
    _say("paper-gap mode")
    wl = W.random_workload(21, dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=4, p=2)
    attr = np.random.default_rng(3).integers(1, 6, size=wl.n_branches).astype(np.int32)
    for mode, fused in ((3, False), (3, True), (4, False), (4, True)):  # wide / narrow workgroup shape
        hip = H.run_hip(wl, pos_mode=1, attr_len=attr, kernel_mode=mode, fused=fused)
        H.check_all(wl, hip, pos_mode="paper_gap", attr_len=attr, label=f"gap_m{mode}")
    wl = W.random_workload(22, dtype="f32", t=4, p=2)
    attr = np.random.default_rng(4).integers(1, 6, size=wl.n_branches).astype(np.int32)
    hip = H.run_hip(wl, pos_mode=1, attr_len=attr)
    H.check_all(wl, hip, pos_mode="paper_gap", attr_len=attr, label="gap_f32")


def test_paper_literal_mask_mode():
    """HPD_MASK_PAPER: one causal order by position ID over the whole stacked prompt (all
    documents, the tokens of every earlier branch up to the current step, finished ones
    included).  Outputs against the oracle's dense mask, and the exported mask bit-exact."""
    from paper_2604_26209_amd import binding as B
    cases = [("f32", dict(hq=4, hkv=2, d=64, t=5, p=2, j_range=(1, 3), n_range=(1, 5), l_range=(1, 40)), (1,)),
             ("bf16", dict(hq=8, hkv=2, d=128, base=500000.0, t=6, p=3, j_range=(1, 4), n_range=(1, 9),
                           h_range=(0, 70), l_range=(1, 150)), (1, 3, 4))]
    for i, (dt, kw, modes) in enumerate(cases):
        wl = W.random_workload(70 + i, dtype=dt, **kw)
        attr = np.random.default_rng(70 + i).integers(1, 6, size=wl.n_branches).astype(np.int32)
        for mode in modes:
            for fused in (False, True):
                _say(f"paper mask {dt} mode {mode} fused {fused}")
                hip = H.run_hip(wl, pos_mode=1, attr_len=attr, mask_mode=B.HPD_MASK_PAPER, fused=fused,
                                kernel_mode=mode)
                H.check_all(wl, hip, pos_mode="paper_gap", attr_len=attr, mask_mode="paper",
                            label=f"paper_{dt}_m{mode}")
        orc, _ = H.run_oracle(wl, hip["inputs"], pos_mode="paper_gap", attr_len=attr, mask_mode="paper")
        for p, po in orc.prompts.items():
            s = B.hpd_expand_mask(hip["layout"], p, wl.max_new - 1)
            m = torch.full((s, s), 7, dtype=torch.uint8, device="cuda")
            B.hpd_expand_mask(hip["layout"], p, wl.max_new - 1, m)
            assert np.array_equal(m.cpu().numpy(), po.dense_mask())
    # the literal mask orders a prompt by position ID: positions that restart per document do not
    with pytest.raises(B.HpdError):
        B.layout_from_workload(wl, pos_mode=0, mask_mode=B.HPD_MASK_PAPER)


@pytest.mark.parametrize("g", [1, 2, 4, 8])
def test_paper_literal_mask_stream_kernel_shapes(g):
    """The streaming kernel under HPD_MASK_PAPER: every group size, all workgroup shapes,
    prompts with more rows than one workgroup takes (several row groups, each appending the
    earlier groups' newest tokens itself in the step call), finished branches as keys, a tail
    of more than one chunk of 8 positions; the step call equals the two-call sequence bit for
    bit."""
    from paper_2604_26209_amd import binding as B
    wl = W.random_workload(80 + g, dtype="bf16", hq=8, hkv=8 // g, d=128, base=500000.0, t=11, p=2,
                           j_range=(2, 4), n_range=(3, 30 if g < 4 else 20), h_range=(0, 90), l_range=(1, 200))
    attr = np.random.default_rng(80 + g).integers(1, 4, size=wl.n_branches).astype(np.int32)
    for mode in (3, 4):
        _say(f"paper mask stream G={g} mode {mode}: {wl.n_branches} branches")
        a = H.run_hip(wl, pos_mode=1, attr_len=attr, mask_mode=B.HPD_MASK_PAPER, kernel_mode=mode,
                      fused=False, poison_pools=True)
        rel = H.check_all(wl, a, pos_mode="paper_gap", attr_len=attr, mask_mode="paper", label=f"paper_g{g}_m{mode}")
        _say(f"  worst err/rms {rel:.2e}")
        b = H.run_hip(wl, inputs=a["inputs"], pos_mode=1, attr_len=attr, mask_mode=B.HPD_MASK_PAPER,
                      kernel_mode=mode, fused=True, poison_pools=True)
        for x, y in zip(a["out"], b["out"]):
            assert torch.equal(x, y)


def _check_prefill(wl, mode, label, out_f32=None, attr_len=None):
    """hpd_prefill_attention against the oracle's prefill_attention, all prompts.  With
    `attr_len`: the literal mask (gap positions), whose prefix also holds the attribute names."""
    from paper_2604_26209_amd import binding as B
    if out_f32 is None:
        out_f32 = wl.dtype == "bf16"
    paper = attr_len is not None
    layout = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32 if out_f32 else B.HPD_OUT_SAME,
                                    **(dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr_len,
                                            mask_mode=B.HPD_MASK_PAPER) if paper else {}))
    if mode:
        B.hpd_set_kernel_mode(layout, mode)
    n_tok = int(layout.counts()[B.HPD_C_N_PREFIX_TOKENS])
    assert n_tok == wl.n_prefix_tokens + (int(np.sum(attr_len)) if paper else 0)
    inputs = H.Inputs(wl, layout.n_live(), "cuda", n_tok)
    q = W.normal_values((n_tok, wl.n_q_heads, wl.head_dim), wl.value_seed * 1000 + 3, "cuda", wl.dtype)
    kp, vp, kt, vt = B.alloc_pools(layout)
    for x in (kp, vp):
        x.fill_(float("nan"))
    B.hpd_prefix_fill(layout, inputs.k_raw, inputs.v_raw, kp, vp)
    out = torch.full((n_tok, wl.n_q_heads, wl.head_dim), float("nan"),
                     dtype=torch.float32 if out_f32 else H.torch_dtype(wl), device="cuda")
    B.hpd_prefill_attention(layout, q, kp, vp, out)
    torch.cuda.synchronize()
    orc, _ = H.run_oracle(wl, inputs, steps=[], **(dict(pos_mode="paper_gap", attr_len=attr_len,
                                                        mask_mode="paper") if paper else {}))
    ref = orc.prefill_attention(q.float().cpu().numpy())
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all(), f"{label}: non-finite output"
    worst = 0.0
    for p, want in ref.items():
        a0, a1 = orc.prefix_range[p]
        err = float(np.abs(got[a0:a1] - want).max())
        if wl.dtype == "f32":
            assert err <= H.F32_TOL, f"{label} prompt {p}: max-abs {err:.3e}"
            worst = max(worst, err)
        else:
            # The RMS of a token's outputs falls from |v| (a token that sees one key) to
            # |v| / sqrt(keys): the bound is taken per token, relative to that token's own
            # RMS over its Hq x D outputs.
            diff = np.abs(got[a0:a1] - want).reshape(a1 - a0, -1).max(axis=1)
            rms = np.sqrt(np.mean(want.astype(np.float64).reshape(a1 - a0, -1) ** 2, axis=1))
            bad = np.nonzero(diff > H.BF16_TOL * rms)[0]
            assert bad.size == 0, (f"{label} prompt {p}: token {bad[0]} max-abs {diff[bad[0]]:.3e} > "
                                   f"{H.BF16_TOL} * rms {rms[bad[0]]:.3e}")
            worst = max(worst, float((diff / rms).max()))
    return worst


def test_prefill_attention_fp32_generic():
    for seed, kw in [(90, dict(hq=4, hkv=2, d=64, t=2, p=3, j_range=(1, 3), h_range=(0, 20), l_range=(1, 70))),
                     (91, dict(hq=2, hkv=2, d=32, t=1, p=2, h_range=(0, 0), l_range=(1, 5)))]:
        wl = W.random_workload(seed, dtype="f32", **kw)
        _say(f"prefill f32 seed {seed}: {wl.n_prefix_tokens} tokens")
        _check_prefill(wl, 0, f"prefill_f32_{seed}")


@pytest.mark.parametrize("g", [1, 2, 4, 8])
def test_prefill_attention_bf16_all_kernels(g):
    """Generic kernel and all shapes of the streaming kernel: segments shorter than a row
    block, segments of many row groups, empty headers, ragged ends."""
    wl = W.random_workload(92 + g, dtype="bf16", hq=8, hkv=8 // g, d=128, base=500000.0, t=2, p=3,
                           j_range=(1, 3), h_range=(0, 90), l_range=(1, 260 if g > 1 else 700))
    for mode in (0, 1, 3, 4):  # 0: the default, the dense shape
        _say(f"prefill bf16 G={g} mode {mode}: {wl.n_prefix_tokens} tokens")
        rel = _check_prefill(wl, mode, f"prefill_bf16_g{g}_m{mode}")
        _say(f"  worst err/rms {rel:.2e}")


def test_prefill_attention_literal_mask_fp32_generic():
    """First inference step under HPD_MASK_PAPER: header, stacked documents and attribute names
    as one causal sequence; the names' rows are the ones whose outputs start the branches."""
    for seed, kw in [(95, dict(hq=4, hkv=2, d=64, t=3, p=3, j_range=(1, 3), h_range=(0, 20), l_range=(1, 70))),
                     (96, dict(hq=2, hkv=2, d=32, t=2, p=2, h_range=(0, 0), l_range=(1, 5)))]:
        wl = W.random_workload(seed, dtype="f32", **kw)
        attr = np.random.default_rng(seed).integers(1, 5, size=wl.n_branches).astype(np.int32)
        _say(f"prefill literal f32 seed {seed}: {wl.n_prefix_tokens} + {int(attr.sum())} tokens")
        _check_prefill(wl, 0, f"prefill_literal_f32_{seed}", attr_len=attr)


@pytest.mark.parametrize("g", [1, 2, 4, 8])
def test_prefill_attention_literal_mask_bf16_all_kernels(g):
    wl = W.random_workload(97 + g, dtype="bf16", hq=8, hkv=8 // g, d=128, base=500000.0, t=2, p=3,
                           j_range=(1, 4), n_range=(1, 30), h_range=(0, 90), l_range=(1, 200 if g > 1 else 500))
    attr = np.random.default_rng(97 + g).integers(1, 5, size=wl.n_branches).astype(np.int32)
    for mode in (0, 1, 3, 4):
        _say(f"prefill literal bf16 G={g} mode {mode}: {wl.n_prefix_tokens} + {int(attr.sum())} tokens")
        rel = _check_prefill(wl, mode, f"prefill_literal_bf16_g{g}_m{mode}", attr_len=attr)
        _say(f"  worst err/rms {rel:.2e}")


@pytest.mark.parametrize("literal", [False, True])
def test_prefix_fill_fast_kernel_equals_general_kernel(literal):
    """hpd_prefix_fill for bf16 / 128 channels (16-byte moves, V interleave through LDS, V padding
    zeroed in the same pass) against the element-wise kernel (kernel_mode 1): the same bits in
    every slot of both pools, ragged segments, empty headers, attribute-name segments."""
    from paper_2604_26209_amd import binding as B
    wl = W.random_workload(170 + int(literal), dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=3, p=4,
                           j_range=(1, 4), n_range=(1, 12), h_range=(0, 70), l_range=(1, 150))
    attr = np.random.default_rng(170).integers(1, 5, size=wl.n_branches).astype(np.int32)
    kw = dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr, mask_mode=B.HPD_MASK_PAPER) if literal else {}
    pools = []
    for mode in (0, 1):
        lay = B.layout_from_workload(wl, **kw)
        if mode:
            B.hpd_set_kernel_mode(lay, mode)
        n_tok = int(lay.counts()[B.HPD_C_N_PREFIX_TOKENS])
        k_raw = W.normal_values((n_tok, wl.n_kv_heads, wl.head_dim), 1, "cuda", wl.dtype)
        v_raw = W.normal_values((n_tok, wl.n_kv_heads, wl.head_dim), 2, "cuda", wl.dtype)
        kp, vp, _, _ = B.alloc_pools(lay)
        kp.fill_(3.0), vp.fill_(3.0)  # K padding is left alone by both kernels
        B.hpd_prefix_fill(lay, k_raw, v_raw, kp, vp)
        pools.append((kp, vp))
    torch.cuda.synchronize()
    _say(f"prefix fill, literal {literal}: {n_tok} tokens, {pools[0][0].numel()} pool elements")
    assert torch.equal(pools[0][0].view(torch.int16), pools[1][0].view(torch.int16))
    assert torch.equal(pools[0][1].view(torch.int16), pools[1][1].view(torch.int16))
    assert bool((pools[0][0] != 3.0).any())


def test_finetune_mask_and_positions_bit_exact():
    """hpd_finetune_mask (Section 4.4) against the loop oracle: mask and position IDs."""
    from oracle import finetune_mask as F
    from paper_2604_26209_amd import binding as B
    rng = np.random.default_rng(9)
    cases = [(10, [3, 3, 3], [3, 3, 3], 7), (0, [1], [1], 1), (4, [2, 1, 3], [0, 5, 2], 5)]
    for _ in range(4):
        n = int(rng.integers(1, 20))
        kmax = int(rng.integers(1, 31))
        cases.append((int(rng.integers(0, 100)), [int(x) for x in rng.integers(1, 6, n)],
                      [int(x) for x in rng.integers(0, kmax + 1, n)], kmax))
    for plen, al, vl, kmax in cases:
        _say(f"finetune mask: prompt {plen}, {len(al)} attributes, K_max {kmax}")
        s = B.hpd_finetune_mask(plen, al, vl, kmax)
        assert s == plen + sum(al) + sum(vl)
        pos = torch.full((s,), -7, dtype=torch.int32, device="cuda")
        m = torch.full((s, s), 7, dtype=torch.uint8, device="cuda")
        B.hpd_finetune_mask(plen, al, vl, kmax, pos, m)
        assert np.array_equal(pos.cpu().numpy(), F.finetune_position_ids(plen, al, vl, kmax))
        assert np.array_equal(m.cpu().numpy(), F.finetune_mask(plen, al, vl))


def test_mask_export_bit_exact():
    from paper_2604_26209_amd import binding as B
    _say("mask export")
    wl = W.random_workload(31, dtype="f32", t=4, p=3, l_range=(1, 30), h_range=(0, 12))
    hip = H.run_hip(wl)
    orc, _ = H.run_oracle(wl, hip["inputs"])
    for p, po in orc.prompts.items():
        s = B.hpd_expand_mask(hip["layout"], p, wl.max_new - 1)
        assert s == len(po.kind)
        m = torch.full((s, s), 7, dtype=torch.uint8, device="cuda")
        B.hpd_expand_mask(hip["layout"], p, wl.max_new - 1, m)
        assert np.array_equal(m.cpu().numpy(), po.dense_mask())


def test_kv_pools_hold_rotated_keys_at_reported_slots():
    """K tail and prefix pools against the oracle's cache (rotated K), through the
    documented pool layouts."""
    from paper_2604_26209_amd import binding as B
    _say("pool contents")
    wl = W.random_workload(51, dtype="f32", hq=4, hkv=2, d=64, t=4, p=2)
    hip = H.run_hip(wl, poison_pools="zero")
    orc, res = H.run_oracle(wl, hip["inputs"])
    kp, vp, kt, vt = [x.cpu().numpy() for x in hip["pools"]]
    lay = hip["layout"]
    c = lay.counts()
    NP, T, Hkv, D = int(c[B.HPD_C_N_PREFIX_SLOTS]), wl.max_new, wl.n_kv_heads, wl.head_dim
    kp = kp.reshape(Hkv, NP, D)
    vp = vp.reshape(Hkv, NP // 8, D, 8)
    kt = kt.reshape(wl.n_branches, Hkv, T, D)
    vt = vt.reshape(wl.n_branches, Hkv, T, D)
    seg_off = B.hpd_layout_query(lay, B.HPD_Q_SEG_OFF)
    for p, po in orc.prompts.items():
        segs = [(p, 0, po.h)]
        run = po.h
        for j, d in enumerate(range(wl.doc_ptr[p], wl.doc_ptr[p + 1])):
            segs.append((wl.n_prompts + d, run, po.doc_lens[j]))
            run += po.doc_lens[j]
        for sid, first, n in segs:
            for i in range(n):
                slot = seg_off[sid] + i
                assert np.abs(kp[:, slot, :] - po.k[first + i]).max() < 1e-5
                assert np.array_equal(vp[:, slot // 8, :, slot % 8], po.v[first + i])
        b0, _ = orc.branch_range[p]
        for idx in range(po.n_prefix, len(po.kind)):
            b, t = b0 + po.branch[idx], po.step_of[idx]
            assert np.abs(kt[b, :, t, :] - po.k[idx]).max() < 1e-5
            assert np.array_equal(vt[b, :, t, :], po.v[idx])


@pytest.mark.parametrize("kernel_mode,fused", [(0, False), (0, True), (1, False)])
def test_bf16_kv_pools_hold_the_rounded_rotated_keys(kernel_mode, fused):
    """The bf16 pools themselves (not only the attention outputs computed from them): prefix and
    tail keys must be the bf16 rounding of the oracle's fp32-rotated keys - the same value, held
    in IEEE half format, which represents every bf16 value of the normal half range exactly -
    except where the kernels' fused multiply-add lands on the other side of a rounding tie: such
    elements may differ by one bf16 ulp and must be rare -, values must be the input values in
    the same format, through the 8-key interleave of the prefix pool.  Covers the 128-channel fill kernel and
    the fused append of the streaming kernel (mode 0), the two-call append kernel, and the
    element-wise fill kernel (mode 1)."""
    from paper_2604_26209_amd import binding as B
    _say(f"bf16 pool contents mode {kernel_mode} fused {fused}")
    wl = W.random_workload(52, dtype="bf16", hq=8, hkv=2, d=128, base=500000.0, t=10, p=3,
                           j_range=(1, 3), n_range=(1, 9), l_range=(1, 150), h_range=(0, 70))
    hip = H.run_hip(wl, poison_pools="zero", kernel_mode=kernel_mode, fused=fused)
    orc, res = H.run_oracle(wl, hip["inputs"])  # bf16 key cache
    bits = lambda x: x.view(torch.int16).cpu().numpy().view(np.uint16)
    kp, vp, kt, vt = [bits(x) for x in hip["pools"]]
    lay = hip["layout"]
    c = lay.counts()
    NP, T, Hkv, D = int(c[B.HPD_C_N_PREFIX_SLOTS]), wl.max_new, wl.n_kv_heads, wl.head_dim
    kp = kp.reshape(Hkv, NP, D)
    vp = vp.reshape(Hkv, NP // 8, D, 8)
    kt = kt.reshape(wl.n_branches, Hkv, T, D)
    vt = vt.reshape(wl.n_branches, Hkv, T, D)
    as_bits = lambda a: (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    seg_off = B.hpd_layout_query(lay, B.HPD_Q_SEG_OFF)
    n_keys = n_off = 0

    def check_k(got_half, want_f32):
        # a key element is the bf16-rounded rotated key in IEEE half format: exact where the
        # value is a normal half (|k| >= 2^-14), within 2^-24 below that
        nonlocal n_keys, n_off
        want_f32 = np.ascontiguousarray(want_f32, dtype=np.float32)
        assert not np.any(want_f32.view(np.uint32) & 0xFFFF)
        got_f32 = np.ascontiguousarray(got_half).view(np.float16).astype(np.float32)
        normal = np.abs(want_f32) >= 2.0 ** -13
        assert not np.any(got_f32[normal].view(np.uint32) & 0xFFFF), "a stored key is not a bf16 value"
        diff = np.abs(as_bits(got_f32[normal]).astype(np.int32) - as_bits(want_f32[normal]).astype(np.int32))
        if diff.size:
            assert diff.max() <= 1, "a stored key is more than one bf16 ulp from the rounded oracle key"
        small = ~normal
        assert np.all(np.abs(got_f32[small] - want_f32[small]) <= 2.0 ** -24 + np.abs(want_f32[small]) * 2.0 ** -7)
        n_keys += diff.size
        n_off += int((diff != 0).sum())

    def check_v(got_half, want_f32):
        # a value element is the caller's bf16 value in half format: the same value wherever it
        # is a normal half, within 2^-24 below
        want_f32 = np.ascontiguousarray(want_f32, dtype=np.float32)
        got_f32 = np.ascontiguousarray(got_half).view(np.float16).astype(np.float32)
        normal = np.abs(want_f32) >= 2.0 ** -13
        assert np.array_equal(got_f32[normal], want_f32[normal])
        assert np.all(np.abs(got_f32[~normal] - want_f32[~normal]) <= 2.0 ** -24)

    for p, po in orc.prompts.items():
        segs = [(p, 0, po.h)]
        run = po.h
        for j, d in enumerate(range(wl.doc_ptr[p], wl.doc_ptr[p + 1])):
            segs.append((wl.n_prompts + d, run, po.doc_lens[j]))
            run += po.doc_lens[j]
        for sid, first, n in segs:
            for i in range(n):
                slot = seg_off[sid] + i
                check_k(kp[:, slot, :], po.k[first + i])
                check_v(vp[:, slot // 8, :, slot % 8], po.v[first + i])
            # the V padding behind the segment is zero (masked keys must contribute 0 * V = 0)
            for slot in range(seg_off[sid] + n, -(-(seg_off[sid] + n) // 32) * 32):
                assert not vp[:, slot // 8, :, slot % 8].any()
        b0, _ = orc.branch_range[p]
        for idx in range(po.n_prefix, len(po.kind)):
            b, t = b0 + po.branch[idx], po.step_of[idx]
            check_k(kt[b, :, t, :], po.k[idx])
            check_v(vt[b, :, t, :], po.v[idx])
    print(f"bf16 pools: {n_off} of {n_keys} stored key elements one ulp from the rounded oracle key "
          f"({n_off / n_keys:.2e})")
    assert n_off <= 2e-3 * n_keys


def test_error_paths_on_device_layout():
    from paper_2604_26209_amd import binding as B
    wl = W.config(1)
    lay = B.layout_from_workload(wl)
    with pytest.raises(B.HpdError):
        B.hpd_rope_positions(lay, wl.max_new, torch.zeros(4, dtype=torch.int32, device="cuda"))
    with pytest.raises(B.HpdError):
        B.hpd_rope_positions(lay, -1, torch.zeros(4, dtype=torch.int32, device="cuda"))
    with pytest.raises(B.HpdError):
        B.hpd_kv_append(lay, 0, None, None, None, None)
    with pytest.raises(B.HpdError):
        B.hpd_set_kernel_mode(lay, 2)  # fp32 / D=64 has no MFMA path
    x = torch.zeros(8, device="cuda")
    with pytest.raises(B.HpdError):
        B.hpd_prefill_attention(lay, None, x, x, x)
