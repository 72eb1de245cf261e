"""Parity at the benchmark configurations' full sizes, launched as bench.py launches them
(automatic kernel choice, fused step call), on sampled prompts the oracle can afford: every
integer output of the whole batch bit-exact, fp32 outputs of the sampled prompts within
2e-2 x RMS(step) for every step, and the bf16 outputs that bench.py times equal to the fp32
outputs rounded once (RNE), bit for bit, for every row of the whole batch."""
import numpy as np
import pytest
import torch

from paper_2604_26209_amd import workloads as W

import hpd_harness as H

pytestmark = pytest.mark.gpu


def _integers_whole_batch(wl, hip):
    """positions and slots of every live branch of every step against closed forms the oracle
    tests pin (H + L + t ; b*T + t) - cheap enough for the whole batch."""
    doc_of_branch = np.repeat(np.arange(wl.n_docs), np.diff(wl.branch_ptr))
    prompt_of_doc = np.repeat(np.arange(wl.n_prompts), np.diff(wl.doc_ptr))
    for t in range(wl.max_new):
        live = np.nonzero(wl.branch_len > t)[0]
        d = doc_of_branch[live]
        assert np.array_equal(hip["pos"][t].cpu().numpy(), wl.header_len[prompt_of_doc[d]] + wl.doc_len[d] + t)
        assert np.array_equal(hip["slot"][t].cpu().numpy(), live.astype(np.int64) * wl.max_new + t)


@pytest.mark.parametrize("k,prompts", [(2, [0, 31]), (3, [5, 63]), (4, [15]), (5, None)])
def test_full_size_config(k, prompts):
    wl = W.config(k)
    print(f"full-size cfg{k}: {wl.n_prompts} prompts, {wl.n_docs} docs, {wl.n_branches} branches", flush=True)
    hip = H.run_hip(wl, fused=True, poison_pools=True)
    _integers_whole_batch(wl, hip)
    # whole batch, every step: the pools were poisoned with NaN, so a single read of a padding
    # slot or of an unwritten tail slot would show; and an output is a convex combination of
    # value rows, so no element can exceed the largest |v| of the inputs
    vmax = max(float(hip["inputs"].v_raw.abs().max()), max(float(x.abs().max()) for x in hip["inputs"].v_new))
    for t, o in enumerate(hip["out"]):
        assert bool(torch.isfinite(o).all()), f"cfg{k} step {t}: non-finite output"
        assert float(o.abs().max()) <= vmax * (1 + 1e-2), f"cfg{k} step {t}: output outside the hull of V"
    if prompts is None:
        # ragged config: a prompt with one document, one with the most documents, the prompt
        # holding the longest and the one holding the shortest document
        nd = np.diff(wl.doc_ptr)
        prompt_of_doc = np.repeat(np.arange(wl.n_prompts), nd)
        prompts = sorted({int(np.argmin(nd)), int(np.argmax(nd)),
                          int(prompt_of_doc[np.argmax(wl.doc_len)]),
                          int(prompt_of_doc[np.argmin(wl.doc_len)])})
    print(f"  oracle on prompts {prompts}", flush=True)
    worst = H.check_all(wl, hip, prompts=prompts, label=f"cfg{k}")
    print(f"  worst max-abs / RMS(step) = {worst:.4f}", flush=True)
    # the price of the bf16 key cache, made visible: the same outputs against the oracle whose
    # cache keeps the rotated keys in fp32 (first two steps of one sampled prompt)
    far = H.distance_to_unrounded_oracle(wl, hip, prompts[:1], min(2, wl.max_new), label=f"cfg{k}")
    print(f"  against the oracle with an unrounded (fp32) key cache: worst max-abs / RMS(step) = {far:.4f} "
          f"(bound {H.BF16_TOL_UNROUNDED_CACHE})", flush=True)
    # the launch configuration bench.py times: outputs in the K/V element type
    print("  bf16 outputs == RNE(fp32 outputs), whole batch", flush=True)
    hip16 = H.run_hip(wl, inputs=hip["inputs"], fused=True, poison_pools=True, out_f32=False)
    for t, (x, y) in enumerate(zip(hip["out"], hip16["out"])):
        assert y.dtype == torch.bfloat16
        assert torch.equal(x.to(torch.bfloat16), y), f"cfg{k} step {t}: bf16 output is not RNE(fp32 output)"


@pytest.mark.parametrize("k,prompts", [(3, [7]), (5, None)])
def test_full_size_config_paper_literal_mask(k, prompts):
    """The literal mask over the whole stacked prompt at full size, launched as
    `bench.py --mask paper` launches it (automatic kernel choice, fused step call, the bench's
    seeded skeleton lengths): integers of the whole batch, sampled prompts against the oracle.
    Config 5 has finished branches whose tokens stay visible to the later branches."""
    from paper_2604_26209_amd import binding as B
    wl = W.config(k)
    attr = np.random.default_rng(26209100 + k).integers(1, 5, size=wl.n_branches).astype(np.int32)
    print(f"full-size cfg{k}, paper-literal mask", flush=True)
    hip = H.run_hip(wl, fused=True, poison_pools=True, pos_mode=1, attr_len=attr, mask_mode=B.HPD_MASK_PAPER)
    for t in range(wl.max_new):
        live = np.nonzero(wl.branch_len > t)[0]
        assert np.array_equal(hip["slot"][t].cpu().numpy(), live.astype(np.int64) * wl.max_new + t)
    vmax = max(float(hip["inputs"].v_raw.abs().max()), max(float(x.abs().max()) for x in hip["inputs"].v_new))
    for t, o in enumerate(hip["out"]):
        assert bool(torch.isfinite(o).all()), f"cfg{k} step {t}: non-finite output"
        assert float(o.abs().max()) <= vmax * (1 + 1e-2), f"cfg{k} step {t}: output outside the hull of V"
    if prompts is None:
        nd = np.diff(wl.doc_ptr)
        prompts = sorted({int(np.argmin(nd)), int(np.argmax(nd))})
    print(f"  oracle on prompts {prompts}", flush=True)
    worst = H.check_all(wl, hip, prompts=prompts, pos_mode="paper_gap", attr_len=attr, mask_mode="paper",
                        label=f"cfg{k}_paper")
    print(f"  worst max-abs / RMS(step) = {worst:.4f}", flush=True)


@pytest.mark.parametrize("k,prompts,literal", [(2, [0, 31], False), (3, [11], False), (3, [20], True), (5, None, True)])
def test_full_size_prefill_attention(k, prompts, literal):
    """hpd_prefill_attention at full size, launched as `bench.py --phase prefill` (and
    `--mask paper`) launches it: sampled prompts against the oracle (per-token RMS bound),
    every output finite and inside the hull of V."""
    from paper_2604_26209_amd import binding as B
    wl = W.config(k)
    attr = np.random.default_rng(26209100 + k).integers(1, 5, size=wl.n_branches).astype(np.int32) if literal else None
    layout = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32,
                                    **(dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr,
                                            mask_mode=B.HPD_MASK_PAPER) if literal else {}))
    n_tok = int(layout.counts()[B.HPD_C_N_PREFIX_TOKENS])
    print(f"full-size cfg{k}, prefill attention over {n_tok} tokens, literal mask: {literal}", flush=True)
    if prompts is None:  # ragged config: the prompts with the fewest and the most documents
        nd = np.diff(wl.doc_ptr)
        prompts = sorted({int(np.argmin(nd)), int(np.argmax(nd))})
    base = wl.value_seed * 1000
    shp = (n_tok, wl.n_kv_heads, wl.head_dim)
    k_raw = W.normal_values(shp, base + 1, "cuda", wl.dtype)
    v_raw = W.normal_values(shp, base + 2, "cuda", wl.dtype)
    q = W.normal_values((n_tok, wl.n_q_heads, wl.head_dim), base + 3, "cuda", wl.dtype)
    kp, vp, kt, vt = B.alloc_pools(layout)
    kp.fill_(float("nan")); vp.fill_(float("nan"))
    B.hpd_prefix_fill(layout, k_raw, v_raw, kp, vp)
    out = torch.full((n_tok, wl.n_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    B.hpd_prefill_attention(layout, q, kp, vp, out)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    assert float(out.abs().max()) <= float(v_raw.abs().max()) * (1 + 1e-2)
    from oracle import hpd_oracle as O
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len, wl.n_q_heads,
                      wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new, prompts=prompts, cache_dtype="bf16",
                      **(dict(pos_mode="paper_gap", attr_len=attr, mask_mode="paper") if literal else {}))
    kd, vd, qd = {}, {}, {}
    for p in prompts:
        a, b = orc.prefix_range[p]
        kd[p], vd[p], qd[p] = (x[a:b].float().cpu().numpy() for x in (k_raw, v_raw, q))
    orc.prefill(kd, vd)
    ref = orc.prefill_attention(qd)
    for p in prompts:
        a, b = orc.prefix_range[p]
        got = out[a:b].cpu().numpy()
        diff = np.abs(got - ref[p]).reshape(b - a, -1).max(axis=1)
        rms = np.sqrt(np.mean(ref[p].astype(np.float64).reshape(b - a, -1) ** 2, axis=1))
        assert np.all(diff <= H.BF16_TOL * rms), f"cfg{k} prompt {p}: worst {float((diff / rms).max()):.3e}"
        print(f"  prompt {p}: worst max-abs / RMS(token) = {float((diff / rms).max()):.4f}", flush=True)


@pytest.mark.parametrize("k", [2, 5])
def test_full_size_device_lists_and_paged_tails_equal_decode_step(k):
    """The two variants of the step call at a benchmark configuration's full size: live lists
    kept on the GPU (flags in) and tail pools behind a page table (pages in a seeded random
    order, as bench.py --page-size sets them up), both at once, must write the very bits
    hpd_decode_step writes with host-built lists and contiguous tails - whole batch, every step."""
    from paper_2604_26209_amd import binding as B
    wl = W.config(k)
    print(f"full-size cfg{k}: device-side lists + paged tails", flush=True)
    ref = H.run_hip(wl, fused=True, poison_pools=True, out_f32=False)
    inputs = ref["inputs"]
    lay = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_SAME)
    ps = 8
    ppb = -(-wl.max_new // ps)
    table = torch.from_numpy(np.random.default_rng(k).permutation(wl.n_branches * ppb).astype(np.int32)
                             .reshape(wl.n_branches, ppb)).cuda()
    B.hpd_set_tail_pages(lay, ps, wl.n_branches * ppb, table)
    kp, vp, kt, vt = B.alloc_pools(lay)
    for x in (kp, vp, kt, vt):
        x.fill_(float("nan"))
    B.hpd_prefix_fill(lay, inputs.k_raw, inputs.v_raw, kp, vp)
    B.hpd_dynamic_begin(lay)
    for t in range(wl.max_new):
        live = np.nonzero(wl.branch_len > t)[0]
        if len(live) == 0:
            break
        got_n, got_live = B.hpd_dynamic_read(lay, wl.n_branches)
        assert got_n == len(live) and np.array_equal(got_live, live), f"cfg{k} step {t}: live list"
        out = torch.full_like(ref["out"][t], float("nan"))
        B.hpd_dynamic_step(lay, t, inputs.q[t], inputs.k_new[t], inputs.v_new[t], kp, vp, kt, vt, out)
        assert torch.equal(out, ref["out"][t]), f"cfg{k} step {t}: outputs differ"
        if t + 1 < wl.max_new:
            B.hpd_dynamic_prune(lay, torch.from_numpy((wl.branch_len[live] == t + 1).astype(np.uint8)).cuda())


@pytest.mark.parametrize("k,prompt,literal", [(2, 31, False), (3, 40, False), (3, 9, True), (5, None, False)])
def test_full_size_mask_export_bit_exact(k, prompt, literal):
    """The exported dense mask of one prompt of a benchmark configuration after its last decode
    step (every token the prompt ever holds) against the oracle's mask, bit for bit; for the
    ragged configuration the prompt with the most documents."""
    from oracle import hpd_oracle as O
    from paper_2604_26209_amd import binding as B
    wl = W.config(k)
    if prompt is None:
        prompt = int(np.argmax(np.diff(wl.doc_ptr)))
    attr = np.random.default_rng(26209100 + k).integers(1, 5, size=wl.n_branches).astype(np.int32) if literal else None
    kw = dict(pos_mode="paper_gap", attr_len=attr, mask_mode="paper") if literal else {}
    orc = O.HPDOracle(wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr, wl.branch_len, 1, 1, 2,
                      wl.rope_base, wl.max_new, prompts=[prompt], **kw)  # one head of two channels: only the mask matters
    a0, a1 = orc.prefix_range[prompt]
    z = np.zeros((a1 - a0, 1, 2), dtype=np.float32)
    orc.prefill({prompt: z}, {prompt: z})
    for t in range(wl.max_new):
        n = int((wl.branch_len > t).sum())
        x = np.zeros((n, 1, 2), dtype=np.float32)
        orc.step(t, x, x, x)
    po = orc.prompts[prompt]
    want = po.mask_rows_fast(list(range(len(po.kind))))
    layout = B.layout_from_workload(wl, **(dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr,
                                                mask_mode=B.HPD_MASK_PAPER) if literal else {}))
    s = B.hpd_expand_mask(layout, prompt, wl.max_new - 1)
    print(f"full-size cfg{k} prompt {prompt}: mask of {s} tokens, literal: {literal}", flush=True)
    assert s == len(po.kind)
    m = torch.full((s, s), 7, dtype=torch.uint8, device="cuda")
    B.hpd_expand_mask(layout, prompt, wl.max_new - 1, m)
    assert np.array_equal(m.cpu().numpy(), want)
