#!/usr/bin/env python3
"""Benchmark of HPD masked decode attention on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input: for every
decode step t = 0..T-1 of the workload, RoPE(K) + KV append and RoPE(Q) + masked attention
(shared header + own document + own tail) + output, for one attention layer.  Inputs and KV
pools are resident in HBM before the timed region.  Metric: branch-tokens/s =
sum_t n_live(t) / time.

Cold-cache protocol: R independent replicas of the KV pools ("layers", R x footprint >= ~2 GB,
far above the 256 MB Infinity Cache) are decoded interleaved - decode step t of layer 0, of
layer 1, ... of layer R-1, then step t+1 of layer 0, ... - as the layers of a real model
would be, so that every launch finds its KV evicted.  (Running all T steps of one replica
back to back would serve steps 1..T-1 out of the Infinity Cache.)

Prints ONE JSON line.  Without --config the headline (value, ms_per_step, roofline,
cpu_baseline) is the largest single-GPU configuration (configs[4], the ragged mixed batch: the
only one with every feature of the path in it - stacked documents of different lengths, ragged
branch counts, early stopping) timed over exactly --steps passes, and `per_config` carries the
same measurement for all five configurations (each timed for at least MIN_TIMED_S), the 70B-like
one against both roofs.  With --config k the line is that configuration's alone (used for the
profiler runs and for side measurements).  `roofline.achieved` = algorithmic bytes of the timed
launches / their GPU time, taken live with one pair of HIP events around the timed region (on
the stream the kernels are launched on); `roofline.traffic` is NOT measured by this run: it is
read from the rocprofv3 counter summary under profiles/ that `traffic_source` names.
`measured_peaks` are three reference kernels of the library (plain read, plain copy, independent
MFMAs) timed in this run.  `cpu_baseline` times the CPU oracle on a bounded sample of the
headline workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16

MIN_WARMUP_S = 0.2   # warm-up lasts at least this long (clocks, caches, code objects)
MIN_TIMED_S = 0.3    # per_config entries other than the headline are timed at least this long

# rocprofv3 counter summaries (FETCH_SIZE / WRITE_SIZE, scaled by a 1 GiB copy) of
# `bench.py --config k`: the line "total traffic X MB per launch" is what roofline.traffic quotes
PROFILE_OF_CONFIG = {2: "profiles/attn_stream_cfg2_llama3_8b.txt", 3: "profiles/attn_stream_cfg3_stacked.txt",
                     4: "profiles/attn_stream_cfg4_long_70b.txt", 5: "profiles/attn_stream_cfg5_ragged.txt"}


def profiled_traffic(k):
    """(HBM bytes per launch, file) from the committed profiler summary of configuration k, or
    (None, None)."""
    import re
    rel = PROFILE_OF_CONFIG.get(k)
    try:
        m = re.search(r"total traffic ([0-9.]+) MB per launch", open(os.path.join(ROOT, rel)).read())
        return (float(m.group(1)) * 1e6, rel) if m else (None, None)
    except (OSError, TypeError):
        return None, None


def algorithmic_bytes(wl, n_live_lists, eb, paper=False, attr_len=None):
    """Bytes the method has to move per decode step: each shared prefix K/V once per
    (prompt | document, kv head), each tail once per (branch, kv head), Q in, O out, new K/V
    in and out.  Returns (attention_bytes[t], append_bytes[t], flops[t]).
    paper = the literal mask over the whole prompt: the same prefix bytes (every document of a
    live prompt once), the tails of all branches of a live prompt up to its last live one
    (finished ones as far as they got) once, and every row multiplies with all of them."""
    import numpy as np

    tok_b = 2 * wl.n_kv_heads * wl.head_dim * eb
    doc_of_branch = np.repeat(np.arange(wl.n_docs), np.diff(wl.branch_ptr))
    prompt_of_doc = np.repeat(np.arange(wl.n_prompts), np.diff(wl.doc_ptr))
    attn, app, flops = [], [], []
    for t, live in enumerate(n_live_lists):
        docs = np.unique(doc_of_branch[live])
        prompts = np.unique(prompt_of_doc[docs])
        prefix = int(wl.header_len[prompts].sum() + wl.doc_len[docs].sum()) * tok_b
        n = len(live)
        tail = n * (t + 1) * tok_b
        qo = n * 2 * wl.n_q_heads * wl.head_dim * eb
        attn.append(prefix + tail + qo)
        app.append(n * 2 * tok_b)
        keys = wl.header_len[prompt_of_doc[doc_of_branch[live]]] + wl.doc_len[doc_of_branch[live]] + t + 1
        if paper:
            in_mem = np.minimum(wl.branch_len, t + 1)
            csum = np.concatenate([[0], np.cumsum(in_mem)])
            p_of_b = prompt_of_doc[doc_of_branch]
            first_b = wl.branch_ptr[wl.doc_ptr[:-1]]
            prefix, tail = 0, 0
            for pr in prompts:
                d0, d1 = wl.doc_ptr[pr], wl.doc_ptr[pr + 1]
                last = live[p_of_b[live] == pr].max()
                prefix += int(wl.header_len[pr] + wl.doc_len[d0:d1].sum()) * tok_b
                prefix += int(attr_len[first_b[pr]:last + 1].sum()) * tok_b  # attribute names up to the last live branch
                tail += int(csum[last + 1] - csum[first_b[pr]]) * tok_b
            attn[-1] = prefix + tail + qo
            plen = np.asarray([wl.header_len[pr] + wl.doc_len[wl.doc_ptr[pr]:wl.doc_ptr[pr + 1]].sum()
                               for pr in range(wl.n_prompts)])
            acum = np.concatenate([[0], np.cumsum(attr_len)])
            keys = (plen[p_of_b[live]] + (csum[live + 1] - csum[first_b[p_of_b[live]]])
                    + (acum[live + 1] - acum[first_b[p_of_b[live]]]))
        flops.append(int(4 * wl.head_dim * wl.n_q_heads * keys.sum()))
    return attn, app, flops


def cpu_baseline(wl, budget_s=15.0, paper=False, attr_len=None):
    """Times the dense CPU oracle on as many prompts of the workload as fit the budget."""
    import numpy as np
    import torch

    from oracle import hpd_oracle as O
    from paper_2604_26209_amd import workloads as W

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    cores = len(os.sched_getaffinity(0))
    done_tokens, spent, used = 0, 0.0, []
    p = 0
    while p < 64 * wl.n_prompts and (spent < budget_s or not used):
        pid, p = p, p % wl.n_prompts  # small workloads are repeated until the budget is used
        d0, d1 = int(wl.doc_ptr[p]), int(wl.doc_ptr[p + 1])
        b0, b1 = int(wl.branch_ptr[d0]), int(wl.branch_ptr[d1])
        n_tok = int(wl.header_len[p] + wl.doc_len[d0:d1].sum())
        if paper:  # the attribute names are fed with the prompt
            n_tok += int(attr_len[b0:b1].sum())
        g = np.random.default_rng(1000 + p)
        kr = g.standard_normal((n_tok, wl.n_kv_heads, wl.head_dim), dtype=np.float32)
        vr = g.standard_normal((n_tok, wl.n_kv_heads, wl.head_dim), dtype=np.float32)
        bl = wl.branch_len[b0:b1]
        ins = []
        for t in range(wl.max_new):
            n = int((bl > t).sum())
            ins.append((g.standard_normal((n, wl.n_q_heads, wl.head_dim), dtype=np.float32),
                        g.standard_normal((n, wl.n_kv_heads, wl.head_dim), dtype=np.float32),
                        g.standard_normal((n, wl.n_kv_heads, wl.head_dim), dtype=np.float32)))
        t0 = time.perf_counter()
        po = O.PromptOracle(int(wl.header_len[p]), wl.doc_len[d0:d1],
                            [[int(x) for x in wl.branch_len[int(wl.branch_ptr[d]):int(wl.branch_ptr[d + 1])]]
                             for d in range(d0, d1)],
                            wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.rope_base, wl.max_new,
                            cache_dtype="bf16" if wl.dtype == "bf16" else None,
                            **(dict(pos_mode="paper_gap", mask_mode="paper",
                                    attr_lens=[int(x) for x in attr_len[b0:b1]]) if paper else {}))
        po.prefill(kr, vr)
        for t in range(wl.max_new):
            po.step(t, *ins[t])
        spent += time.perf_counter() - t0
        done_tokens += int(bl.sum())
        used.append(pid)
        p = pid + 1
    return {"value": done_tokens / spent, "unit": "branch-tokens/s", "cores": int(min(threads, cores)),
            "kind": "oracle",
            "sample": f"{len(used)} prompt decodes (prompts 0..{min(used[-1], wl.n_prompts - 1)} of "
                      f"{wl.n_prompts}, repeated if needed), all {wl.max_new} steps incl. prefix RoPE, "
                      f"{done_tokens} branch-tokens in {spent:.1f} s; host affinity {cores} cores"}


def bench_prefill(args, wl, layout, B, W, torch, np, out_f32, attr_len=None):
    """hpd_prefill_attention on the workload's header and document tokens: every prefix token a
    query over header + own document up to itself.  With `attr_len` (the literal mask): header,
    documents and attribute names of a prompt as one causal sequence.  A step = one call over
    the whole batch."""
    dev = "cuda"
    eb = 4 if wl.dtype == "f32" else 2
    base = wl.value_seed * 1000
    n_tok = int(B.hpd_layout_query(layout, B.HPD_Q_COUNTS)[B.HPD_C_N_PREFIX_TOKENS])
    shp = (n_tok, wl.n_kv_heads, wl.head_dim)
    k_raw = W.normal_values(shp, base + 1, dev, wl.dtype)
    v_raw = W.normal_values(shp, base + 2, dev, wl.dtype)
    q = W.normal_values((n_tok, wl.n_q_heads, wl.head_dim), base + 3, dev, wl.dtype)
    tdt = torch.float32 if (out_f32 or wl.dtype == "f32") else torch.bfloat16
    out = torch.empty((n_tok, wl.n_q_heads, wl.head_dim), dtype=tdt, device=dev)
    kp, vp, kt, vt = B.alloc_pools(layout, dev)
    B.hpd_prefix_fill(layout, k_raw, v_raw, kp, vp)
    torch.cuda.synchronize()
    # multiply-adds: a header token i sees i + 1 keys, token i of a document H + i + 1
    keys = 0
    for p in range(wl.n_prompts):
        h = int(wl.header_len[p])
        keys += h * (h + 1) // 2
        for d in range(wl.doc_ptr[p], wl.doc_ptr[p + 1]):
            l = int(wl.doc_len[d])
            keys += l * h + l * (l + 1) // 2
        if attr_len is not None:  # one causal sequence: header, documents, names
            n = h + int(wl.doc_len[wl.doc_ptr[p]:wl.doc_ptr[p + 1]].sum()) + \
                int(attr_len[wl.branch_ptr[wl.doc_ptr[p]]:wl.branch_ptr[wl.doc_ptr[p + 1]]].sum())
            keys += n * (n + 1) // 2 - (h * (h + 1) // 2 + sum(
                int(l) * h + int(l) * (int(l) + 1) // 2 for l in wl.doc_len[wl.doc_ptr[p]:wl.doc_ptr[p + 1]]))
    flops = 4 * wl.head_dim * wl.n_q_heads * keys
    tok_b = 2 * wl.n_kv_heads * wl.head_dim * eb
    alg_bytes = n_tok * (tok_b + 2 * wl.n_q_heads * wl.head_dim * eb)  # K/V once, Q in, O out
    steps, warmup = max(1, args.steps // 4), max(1, args.warmup // 4)
    for _ in range(warmup):
        B.hpd_prefill_attention(layout, q, kp, vp, out)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        B.hpd_prefill_attention(layout, q, kp, vp, out)
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dur_s = ev0.elapsed_time(ev1) * 1e-3
    tf = flops * steps / dur_s / 1e12
    rec = {"metric": "prefix tokens/s of HPD prefill attention (side measurement)",
           "value": round(n_tok * steps / elapsed, 1), "unit": "prefix-tokens/s", "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed * 1e3 / steps, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype,
           "data": "synthetic",
           "config": {"workload": f"configs[{args.config - 1}] {wl.name}: {wl.note}; prefill attention"
                                  + ("; paper-literal mask, attribute names included" if attr_len is not None else ""),
                      "prefix_tokens": n_tok, "heads": f"{wl.n_q_heads}/{wl.n_kv_heads}x{wl.head_dim}",
                      "out_dtype": "f32" if tdt == torch.float32 else wl.dtype, "call": "hpd_prefill_attention"},
           "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                        "kernel": "attn_stream_kernel (prefill instantiation)", "launches": steps,
                        "avg_launch_us": round(dur_s / steps * 1e6, 2), "flops_per_launch": int(flops),
                        "algorithmic_bytes_per_launch": int(alg_bytes)}}
    print(json.dumps(rec))


def measured_peaks(B, torch):
    """Three reference kernels of the library, timed with HIP events on the current stream: what a
    plain read, a plain copy and a loop of independent bf16 MFMAs reach on this GPU."""
    dev = "cuda"
    n = 1 << 30  # bytes per buffer: four times the 256 MB Infinity Cache
    a = torch.empty(n // 4, dtype=torch.float32, device=dev).normal_()
    b = torch.empty(n // 4, dtype=torch.float32, device=dev).normal_()
    c = torch.empty(n // 4, dtype=torch.float32, device=dev)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)

    def timed(fn, reps):
        fn(), fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def read2():  # alternating buffers: every launch finds its input evicted
        B.hpd_peak_read(a, n, sink)
        B.hpd_peak_read(b, n, sink)

    t_read = timed(read2, 10) / 2
    t_copy = timed(lambda: (B.hpd_peak_copy(c, a, n), B.hpd_peak_copy(c, b, n)), 10) / 2
    flops = []
    t_mfma = timed(lambda: flops.append(B.hpd_peak_mfma(sink, 4000)), 5)
    return {"hbm_read_gbs": round(n / t_read / 1e9, 1), "hbm_copy_gbs_read_plus_write": round(2 * n / t_copy / 1e9, 1),
            "mfma_bf16_tflops": round(flops[-1] / t_mfma / 1e12, 1),
            "kernels": "hpd_peak_read / hpd_peak_copy over 1 GiB buffers (alternating), hpd_peak_mfma "
                       "(4 independent v_mfma_f32_32x32x16_bf16 chains per wave, 8 waves per CU)",
            "published": {"hbm_gbs": HBM_PEAK_GBS, "mfma_bf16_tflops": MFMA_BF16_PEAK_TFLOPS}}


def measure_decode(args, k, steps, warmup, B, W, torch, np, min_timed_s=0.0):
    """Times `steps` passes (at least min_timed_s seconds' worth) of configuration k's decode and
    returns the record of that configuration (no cpu_baseline)."""
    dev = "cuda"
    wl = W.config(k)
    eb = 4 if wl.dtype == "f32" else 2
    out_f32 = args.out == "f32" or wl.dtype == "f32"
    paper = args.mask == "paper"
    # skeleton (attribute-name) lengths for the gap positions: 1..4 tokens, seeded
    attr_len = np.random.default_rng(26209100 + k).integers(1, 5, size=wl.n_branches).astype(np.int32)
    layout = B.layout_from_workload(wl, out_dtype=B.HPD_OUT_F32 if out_f32 else B.HPD_OUT_SAME,
                                    **(dict(pos_mode=B.HPD_POS_PAPER_GAP, attr_len=attr_len,
                                            mask_mode=B.HPD_MASK_PAPER) if paper else {}))
    if args.kernel_mode:
        B.hpd_set_kernel_mode(layout, args.kernel_mode)
    if args.page_size and not paper:
        ppb = -(-wl.max_new // args.page_size)
        page_table = torch.from_numpy(np.random.default_rng(26209200).permutation(wl.n_branches * ppb)
                                      .astype(np.int32).reshape(wl.n_branches, ppb)).cuda()
        B.hpd_set_tail_pages(layout, args.page_size, wl.n_branches * ppb, page_table)
    n_live = layout.n_live()
    live_flat = B.hpd_layout_query(layout, B.HPD_Q_LIVE_BRANCH)
    live_lists, off = [], 0
    for t in range(wl.max_new):
        live_lists.append(live_flat[off:off + n_live[t]])
        off += n_live[t]
    total_tokens = int(sum(n_live))
    attn_b, app_b, flops = algorithmic_bytes(wl, live_lists, eb, paper, attr_len)

    if args.phase == "prefill":
        bench_prefill(args, wl, layout, B, W, torch, np, out_f32, attr_len if paper else None)
        return None

    pool_bytes = B.hpd_layout_query(layout, B.HPD_Q_POOL_BYTES)
    footprint = int(pool_bytes.sum())
    R = args.replicas or max(2, -(-(2 << 30) // footprint))
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    stream_kernel = wl.dtype == "bf16" and wl.head_dim == 128 and args.kernel_mode != 1

    # ---- inputs (seeded), resident in HBM
    base = wl.value_seed * 1000
    # (the layout's count: under the literal mask the attribute-name tokens are fed as well)
    n_prefix = int(B.hpd_layout_query(layout, B.HPD_Q_COUNTS)[B.HPD_C_N_PREFIX_TOKENS])
    k_raw = W.normal_values((n_prefix, wl.n_kv_heads, wl.head_dim), base + 1, dev, wl.dtype)
    v_raw = W.normal_values((n_prefix, wl.n_kv_heads, wl.head_dim), base + 2, dev, wl.dtype)
    q, kn, vn, outs = [], [], [], []
    for t in range(wl.max_new):
        n = int(n_live[t])
        q.append(W.normal_values((n, wl.n_q_heads, wl.head_dim), base + 10 + 3 * t, dev, wl.dtype))
        kn.append(W.normal_values((n, wl.n_kv_heads, wl.head_dim), base + 11 + 3 * t, dev, wl.dtype))
        vn.append(W.normal_values((n, wl.n_kv_heads, wl.head_dim), base + 12 + 3 * t, dev, wl.dtype))
        outs.append(torch.empty((n, wl.n_q_heads, wl.head_dim), dtype=torch.float32 if out_f32 else tdt, device=dev))
    pools = []
    for _ in range(R):
        ps = B.alloc_pools(layout, dev)
        B.hpd_prefix_fill(layout, k_raw, v_raw, ps[0], ps[1])
        ps[2].zero_(), ps[3].zero_()
        pools.append(ps)
    del k_raw, v_raw
    torch.cuda.synchronize()

    def sweep(first, n_layers, events=None):
        """n_layers passes (all decode steps of the workload, one KV replica each), interleaved
        step by step.  With `events`, every launch of the dominant kernel is bracketed by a
        pair of events on the same stream."""
        for t in range(wl.max_new):
            if int(n_live[t]) == 0:
                continue
            for j in range(n_layers):
                kp, vp, kt, vt = pools[(first + j) % R]
                if args.two_call:
                    B.hpd_kv_append(layout, t, kn[t], vn[t], kt, vt)
                if events is not None:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                if args.two_call:
                    B.hpd_decode_attention(layout, t, q[t], kp, vp, kt, vt, outs[t])
                else:
                    B.hpd_decode_step(layout, t, q[t], kn[t], vn[t], kp, vp, kt, vt, outs[t])
                if events is not None:
                    e1.record()
                    events.append((t, e0, e1))

    def run(n_passes, events=None, marks=None):
        """`marks`: a list that receives one event per group of up to R passes (recorded after
        the group, on the same stream), for the spread of the GPU time over the run."""
        done = 0
        while done < n_passes:
            n = min(R, n_passes - done)
            sweep(done, n, events)
            done += n
            if marks is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record()
                marks.append((n, ev))

    live_steps = [t for t in range(wl.max_new) if int(n_live[t]) > 0]
    # warm-up: at least `warmup` passes and at least MIN_WARMUP_S of GPU work
    t_w = time.perf_counter()
    run(max(1, warmup))
    torch.cuda.synchronize()
    warm_passes = max(1, warmup)
    while time.perf_counter() - t_w < MIN_WARMUP_S:
        run(R)
        torch.cuda.synchronize()
        warm_passes += R
    pass_s = (time.perf_counter() - t_w) / warm_passes
    # passes of the timed region: `steps`, more if that would be shorter than min_timed_s, and
    # never fewer than five groups of R passes (for the spread)
    if min_timed_s > 0:
        steps = max(steps, 5 * R, min(int(min_timed_s / pass_s) + 1, 4000))
    # The timed region.  In the fused call it holds launches of the dominant kernel only, back
    # to back on one stream, so one pair of events around it gives that kernel's average launch
    # duration (an event pair around every launch would add about 2 us of dispatch gap to each).
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    marks = []
    run(steps, marks=marks)
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # GPU milliseconds per pass of every group of passes (R replicas, interleaved step by step)
    group_ms, prev = [], ev0
    for n, ev in marks:
        group_ms.append(prev.elapsed_time(ev) / n)
        prev = ev
    ms_per_step = elapsed * 1e3 / steps
    value = total_tokens * steps / elapsed

    # ---- roofline of the dominant kernel (attention), live
    if args.two_call:
        # the append kernel sits between the attention launches: bracket each attention launch
        events = []
        run(steps, events)
        torch.cuda.synchronize()
        dur_s = sum(e0.elapsed_time(e1) for _, e0, e1 in events) * 1e-3
        launched = [t for t, _, _ in events]
    else:
        dur_s = ev0.elapsed_time(ev1) * 1e-3
        launched = live_steps * steps
    # the fused step kernel also does the append (new K/V in, rotated K/V out)
    alg = sum(attn_b[t] + (0 if args.two_call else app_b[t]) for t in launched)
    achieved = alg / dur_s / 1e9
    mfma_tflops = sum(flops[t] for t in launched) / dur_s / 1e12
    traffic, traffic_src = (None, None) if (args.two_call or out_f32 or paper or args.page_size or args.kernel_mode) \
        else profiled_traffic(k)
    # arithmetic intensity decides the binding roof: above the ridge of the published peaks
    # (2500 TFLOP/s / 8 TB/s = 312 flop/byte) or within reach of it the matrix pipes bind first
    intensity = sum(flops[t] for t in launched) / alg
    bound = "mfma" if intensity > 150 else "hbm"
    roofline = {"bound": bound,
                "achieved": round(mfma_tflops if bound == "mfma" else achieved, 1),
                "peak": MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else HBM_PEAK_GBS,
                "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
                "frac": round(mfma_tflops / MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic,
                "traffic_source": (f"{traffic_src}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of `bench.py --config {k}`, "
                                   "not measured by this run") if traffic_src else None,
                "kernel": ("attn_stream_kernel" if stream_kernel else
                           "append_kernel + attention_generic_kernel (two launches per step)"),
                "launches": len(launched), "avg_launch_us": round(dur_s / len(launched) * 1e6, 2),
                "algorithmic_bytes_per_launch": int(alg / len(launched)),
                "hbm_gbs": round(achieved, 1), "frac_of_hbm_peak": round(achieved / HBM_PEAK_GBS, 4),
                "useful_tflops": round(mfma_tflops, 1),
                "useful_tflops_frac_of_mfma_peak": round(mfma_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                "flop_per_byte": round(intensity, 1)}

    rec = {
        "metric": "branch tokens/s of HPD masked decode attention; achieved HBM GB/s vs peak",
        "value": round(value, 1), "unit": "branch-tokens/s", "n_gpus": 1, "steps": steps,
        "warmup": warm_passes, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{k - 1}] {wl.name}: {wl.note}"
                               + ("; paper-literal mask over the whole prompt, gap positions" if paper else ""),
                   "prompts": wl.n_prompts, "documents": wl.n_docs, "branches": wl.n_branches,
                   "decode_steps_per_pass": wl.max_new, "branch_tokens_per_pass": total_tokens,
                   "heads": f"{wl.n_q_heads}/{wl.n_kv_heads}x{wl.head_dim}", "kv_replicas": R,
                   "kv_footprint_mb": round(footprint / 1e6, 1), "out_dtype": "f32" if out_f32 else wl.dtype,
                   **({"tail_page_size": args.page_size} if args.page_size and not paper else {}),
                   "call": "hpd_kv_append+hpd_decode_attention" if args.two_call else "hpd_decode_step",
                   **({"arithmetic": "inputs, cache values and outputs bf16; the pools hold the bf16 values in "
                                     "IEEE half format and both products run on v_mfma_f32_32x32x16_f16 "
                                     "(same dense peak as bf16), fp32 accumulation and softmax"}
                      if stream_kernel else {}),
                   "parity_checked_on": ("fp32 outputs against the CPU oracle (tests/test_gpu_full_size.py, this "
                                         "configuration's full size and launch shape), and bf16 outputs == "
                                         "RNE(fp32 outputs) bit for bit for every row" if wl.dtype == "bf16" else
                                         "fp32 outputs against the CPU oracle, every row")},
        "roofline": roofline,
        "gpu_ms_per_step": {"median": round(float(np.median(group_ms)), 4), "min": round(float(min(group_ms)), 4),
                            "max": round(float(max(group_ms)), 4), "groups": len(group_ms)},
    }
    if args.per_step and not args.two_call:
        reps = max(1, steps // R)
        pairs = []
        for t in live_steps:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                for kp, vp, kt, vt in pools:
                    B.hpd_decode_step(layout, t, q[t], kn[t], vn[t], kp, vp, kt, vt, outs[t])
            e1.record()
            pairs.append((t, e0, e1))
        torch.cuda.synchronize()
        us = [e0.elapsed_time(e1) * 1e3 / (reps * R) for _, e0, e1 in pairs]
        rec["per_step"] = {"steps": live_steps, "launches_per_step": reps * R,
                           "us": [round(x, 2) for x in us],
                           "gbs": [round((attn_b[t] + app_b[t]) / (x * 1e-6) / 1e9, 1)
                                   for (t, _, _), x in zip(pairs, us)]}
    if args.dynamic and not (args.two_call or paper):
        # side measurement: the same passes with the live list kept on the GPU (flags in, no
        # host-built lists), one pass after the other, against hpd_decode_step in that order
        fins = [torch.from_numpy((wl.branch_len[live_lists[t]] == t + 1).astype(np.uint8)).to(dev)
                if len(live_lists[t]) else torch.zeros(1, dtype=torch.uint8, device=dev) for t in range(wl.max_new)]

        def one_pass(p, dyn):
            kp, vp, kt, vt = pools[p % R]
            if dyn:
                B.hpd_dynamic_begin(layout)
            for t in live_steps:
                if dyn:
                    B.hpd_dynamic_step(layout, t, q[t], kn[t], vn[t], kp, vp, kt, vt, outs[t])
                    if t + 1 < wl.max_new:
                        B.hpd_dynamic_prune(layout, fins[t])
                else:
                    B.hpd_decode_step(layout, t, q[t], kn[t], vn[t], kp, vp, kt, vt, outs[t])

        res = {}
        for dyn in (True, False, True, False):
            for p in range(min(warmup, R)):
                one_pass(p, dyn)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for p in range(steps):
                one_pass(p, dyn)
            e1.record()
            torch.cuda.synchronize()
            res.setdefault(dyn, []).append(e0.elapsed_time(e1) / steps)
        rec["dynamic"] = {"gpu_ms_per_pass_device_lists": round(min(res[True]), 4),
                          "gpu_ms_per_pass_host_lists": round(min(res[False]), 4),
                          "call": "hpd_dynamic_begin + (hpd_dynamic_step, hpd_dynamic_prune) per step"}
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(args.copy_calibration):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    rec["_workload"] = (wl, paper, attr_len)
    del pools, q, kn, vn, outs
    torch.cuda.empty_cache()
    return rec


HEADLINE_CONFIG = 5


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=0,
                    help="0 (default): headline on configs[4] plus per_config for all five; 1..5: that "
                         "configuration alone")
    ap.add_argument("--replicas", type=int, default=0, help="KV replicas (0 = enough for 2 GB)")
    ap.add_argument("--out", default="same", choices=["f32", "same"],
                    help="output element type: the K/V element type (default) or fp32")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measured_peaks reference kernels")
    ap.add_argument("--two-call", action="store_true", help="hpd_kv_append + hpd_decode_attention")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="after the timed regions, run this many 1 GiB device copies (reference "
                         "dispatches for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--mask", default="block", choices=["block", "paper"],
                    help="block: header + own document + own branch (the benchmark's metric); paper: "
                         "the literal mask over the whole stacked prompt, with the paper's gap positions")
    ap.add_argument("--phase", default="decode", choices=["decode", "prefill"],
                    help="decode: the benchmark's metric; prefill: hpd_prefill_attention (the attention of "
                         "the header and document tokens themselves, first inference step), a side measurement")
    ap.add_argument("--kernel-mode", type=int, default=0,
                    help="hpd_set_kernel_mode: 0 automatic (default), 1 generic kernel, 3 / 4 streaming "
                         "kernel with the wide / narrow workgroup shape")
    ap.add_argument("--page-size", type=int, default=0,
                    help="side measurement: tail pools paged (hpd_set_tail_pages) with this page size, "
                         "pages in a seeded random order")
    ap.add_argument("--dynamic", action="store_true",
                    help="also time the passes with the live list kept on the GPU (hpd_dynamic_*)")
    ap.add_argument("--per-step", action="store_true",
                    help="second run: one event pair per decode step (all replicas of that step back "
                         "to back), adds per_step {us, gbs} to the record")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2604_26209_amd import binding as B
    from paper_2604_26209_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)

    if args.config:  # one configuration, exactly --steps passes
        rec = measure_decode(args, args.config, args.steps, args.warmup, B, W, torch, np)
        if rec is None:
            return
        wl, paper, attr_len = rec.pop("_workload")
        if not args.no_cpu_baseline:
            rec["cpu_baseline"] = cpu_baseline(wl, paper=paper, attr_len=attr_len)
        print(json.dumps(rec))
        return

    # ---- the full record: headline on the largest configuration, every configuration in per_config
    if args.phase != "decode":
        print("bench.py: --phase prefill needs --config k", file=sys.stderr)
        sys.exit(2)
    per_config, head = {}, None
    for k in (1, 2, 3, 4, 5):
        print(f"bench: configuration {k}", file=sys.stderr, flush=True)
        if k == HEADLINE_CONFIG:
            r = measure_decode(args, k, args.steps, args.warmup, B, W, torch, np)  # exactly --steps passes
            head = r
        else:
            r = measure_decode(args, k, args.steps, args.warmup, B, W, torch, np, min_timed_s=MIN_TIMED_S)
        rf = r["roofline"]
        per_config[str(k)] = {
            "workload": r["config"]["workload"], "value": r["value"], "unit": r["unit"],
            "passes_timed": r["steps"], "ms_per_pass": r["ms_per_step"],
            "gpu_ms_per_pass": r["gpu_ms_per_step"], "kernel": rf["kernel"],
            "avg_launch_us": rf["avg_launch_us"], "launches": rf["launches"],
            "algorithmic_bytes_per_launch": rf["algorithmic_bytes_per_launch"],
            "hbm_gbs": rf["hbm_gbs"], "frac": rf["frac_of_hbm_peak"],
            "useful_tflops": rf["useful_tflops"], "frac_of_mfma_peak": rf["useful_tflops_frac_of_mfma_peak"],
            "flop_per_byte": rf["flop_per_byte"], "bound": rf["bound"],
            "traffic": rf["traffic"], "traffic_source": rf["traffic_source"]}
        if k == 1:
            per_config["1"]["note"] = ("the correctness configuration: 0.2 MB per step, bound by launch latency "
                                       "(generic fp32 kernels, two launches per step)")
    wl, paper, attr_len = head.pop("_workload")
    head["config"]["headline"] = ("configs[4] is the largest single-GPU configuration (2.6 GB of algorithmic bytes "
                                  "per launch) and the only one with every part of the path in it: stacked documents "
                                  "of ragged lengths, ragged branch counts, early stopping")
    head["per_config"] = per_config
    if not args.no_peaks:
        head["measured_peaks"] = measured_peaks(B, torch)
    if not args.no_cpu_baseline:
        head["cpu_baseline"] = cpu_baseline(wl, paper=paper, attr_len=attr_len)
    print(json.dumps(head))


if __name__ == "__main__":
    main()
