"""fp64 pure-loop brute force for tiny HPD inputs.  TEST INFRASTRUCTURE ONLY.

Shares nothing with ``hpd_oracle`` (no mask, no flat cache): for every live
branch it writes out, token by token, the set of keys the method lets the
branch see (Section 4.3.2 restricted to header + own document + own branch)
and evaluates softmax attention with scalar loops and ``math`` functions.
Used as one of the pins of the dense oracle; far too slow for anything but a
few dozen tokens.  ``decode_all_steps_paper`` does the same for the section's
rule taken literally over the whole prompt (every stacked document, and the
value tokens of all earlier attributes up to the current step), with the
position IDs of Appendix A.1 written out as a closed form.
"""
from __future__ import annotations

import math


def _rope_scalar(vec, pos, base):
    d = len(vec)
    half = d // 2
    out = [0.0] * d
    for i in range(half):
        ang = pos * (base ** (-2.0 * i / d))
        c, s = math.cos(ang), math.sin(ang)
        a, b = vec[i], vec[i + half]
        out[i] = a * c - b * s
        out[i + half] = b * c + a * s
    return out


def decode_all_steps(header_len, doc_lens, branch_lens, hq, hkv, d, base, t_max,
                     k_prefix, v_prefix, q_steps, k_steps, v_steps):
    """One prompt, contiguous-position mode.

    k_prefix / v_prefix : [n_prefix][hkv][d] nested lists, order header, doc0, doc1, ...
    q_steps[t]          : [n_live(t)][hq][d];  k_steps[t], v_steps[t] : [n_live(t)][hkv][d]
    branch_lens         : per document list of branch lengths.
    Returns out[t][r][h][d] as nested lists of Python floats.
    """
    group = hq // hkv
    branch_doc = [j for j, bl in enumerate(branch_lens) for _ in bl]
    blen = [x for bl in branch_lens for x in bl]
    doc_start = []
    acc = header_len
    for l in doc_lens:
        doc_start.append(acc)
        acc += l
    # tails[b] = list of (rotated k [hkv][d], v [hkv][d])
    tails = [[] for _ in blen]
    outs = []
    for t in range(t_max):
        live = [b for b in range(len(blen)) if blen[b] > t]
        # append first: a query sees its own token
        for r, b in enumerate(live):
            j = branch_doc[b]
            pos = header_len + doc_lens[j] + t
            kr = [_rope_scalar(k_steps[t][r][hk], pos, base) for hk in range(hkv)]
            tails[b].append((kr, v_steps[t][r]))
        step_out = []
        for r, b in enumerate(live):
            j = branch_doc[b]
            qpos = header_len + doc_lens[j] + t
            row_out = []
            for h in range(hq):
                hk = h // group
                qr = _rope_scalar(q_steps[t][r][h], qpos, base)
                keys, vals = [], []
                for i in range(header_len):  # header at positions 0..H-1
                    keys.append(_rope_scalar(k_prefix[i][hk], i, base))
                    vals.append(v_prefix[i][hk])
                for i in range(doc_lens[j]):  # own document restarts at H
                    tok = doc_start[j] + i
                    keys.append(_rope_scalar(k_prefix[tok][hk], header_len + i, base))
                    vals.append(v_prefix[tok][hk])
                for (kr, vv) in tails[b]:  # own earlier tokens and itself
                    keys.append(kr[hk])
                    vals.append(vv[hk])
                scores = [sum(qr[x] * kk[x] for x in range(d)) / math.sqrt(d) for kk in keys]
                m = max(scores)
                w = [math.exp(s - m) for s in scores]
                z = sum(w)
                row_out.append([sum(w[n] * vals[n][x] for n in range(len(keys))) / z
                                for x in range(d)])
            step_out.append(row_out)
        outs.append(step_out)
    return outs


def decode_all_steps_paper(header_len, doc_lens, branch_lens, attr_lens, hq, hkv, d, base, t_max,
                           k_prefix, v_prefix, q_steps, k_steps, v_steps):
    """One prompt, the paper's own positions and its literal mask.

    Header and document token i sits at position i.  The name tokens of attribute n (0-based
    over all branches of the prompt, in (document, attribute) order) follow in memory, attribute
    by attribute, and end at position |p| + A_0 + .. + A_n - 1 + n * K_max; value token k
    (1-based) of the attribute sits k slots after that.  Branch b at step t sees: header and
    documents, the name tokens of attributes 0..b, tokens 0..min(t, len-1) of every earlier
    branch, and its own tokens 0..t.  k_prefix / v_prefix hold header, documents and then the
    name tokens; other arguments and the result as in ``decode_all_steps``; ``attr_lens`` is
    the flat list A_n.
    """
    group = hq // hkv
    blen = [x for bl in branch_lens for x in bl]
    n_prefix = header_len + sum(doc_lens)
    base_pos, run = [], n_prefix
    name_tok = []  # (index in k_prefix, position, attribute) of every name token
    for n, a in enumerate(attr_lens):
        for i in range(a):
            name_tok.append((run + i, run + i + n * t_max, n))
        run += a
        base_pos.append(run - 1 + n * t_max)
    tails = [[] for _ in blen]
    outs = []
    for t in range(t_max):
        live = [b for b in range(len(blen)) if blen[b] > t]
        for r, b in enumerate(live):
            pos = base_pos[b] + 1 + t
            kr = [_rope_scalar(k_steps[t][r][hk], pos, base) for hk in range(hkv)]
            tails[b].append((kr, v_steps[t][r]))
        step_out = []
        for r, b in enumerate(live):
            qpos = base_pos[b] + 1 + t
            row_out = []
            for h in range(hq):
                hk = h // group
                qr = _rope_scalar(q_steps[t][r][h], qpos, base)
                keys, vals = [], []
                for i in range(n_prefix):
                    keys.append(_rope_scalar(k_prefix[i][hk], i, base))
                    vals.append(v_prefix[i][hk])
                for (idx, npos, n) in name_tok:  # attribute names up to the own one
                    if n <= b:
                        keys.append(_rope_scalar(k_prefix[idx][hk], npos, base))
                        vals.append(v_prefix[idx][hk])
                for bb in range(b + 1):  # earlier attributes and itself, whatever is in memory
                    for (kr, vv) in tails[bb][:t + 1]:
                        keys.append(kr[hk])
                        vals.append(vv[hk])
                scores = [sum(qr[x] * kk[x] for x in range(d)) / math.sqrt(d) for kk in keys]
                m = max(scores)
                w = [math.exp(s_ - m) for s_ in scores]
                z = sum(w)
                row_out.append([sum(w[n] * vals[n][x] for n in range(len(keys))) / z
                                for x in range(d)])
            step_out.append(row_out)
        outs.append(step_out)
    return outs
