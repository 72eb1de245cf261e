"""CPU oracle for the fine-tuning mask of Hyper-Parallel Decoding.  TEST INFRASTRUCTURE ONLY.

Section 4.4 ("Fine-tuning and Distillation"): a training sequence holds the prompt and, in the
regular token order, every attribute followed by its ground-truth value,

    s_train = cat(p, a_1, v_1, a_2, v_2, ..., a_N, v_N),

with (a) the position IDs of inference - Appendix A.1: the attributes keep the positions of
Algorithm 2 (a gap of K_max after every attribute) and value token k (1-based) of attribute
n sits at pos_id[end(a_n)] + k - and (b) the causal mask with two additions:

  * value token v_{n,k} may not attend to v_{n',k'} with n' < n and k' > k (those would not
    have been generated yet when v_{n,k} is decoded in parallel), and
  * no attribute token attends to any value token (none exists at the first inference step).

Plain loops over token pairs; nothing is shared with the product code.

Pins (tests/test_oracle_finetune_mask.py): the position IDs against the worked example the
paper prints (golden file) and the closed form; the mask against an explicit set construction
and closed-form row sums; and the section's own claim that the pattern equals the one seen
at inference - the inference pattern being built independently from Section 4.3.2's rule
(a key is visible iff it is already in memory and not later in position-ID order) over the
inference memory order [p, a_1..a_N, step-1 values, step-2 values, ...].
"""
from __future__ import annotations

import numpy as np

KIND_PROMPT, KIND_ATTR, KIND_VALUE = 0, 1, 2


def finetune_tokens(prompt_len, attr_lens, value_lens):
    """Token table of s_train in sequence order: arrays kind[S], attr[S] (attribute index n,
    -1 for the prompt), k[S] (1-based index of a value token inside its value, 0 otherwise)."""
    kind, attr, k = [], [], []
    kind += [KIND_PROMPT] * int(prompt_len)
    attr += [-1] * int(prompt_len)
    k += [0] * int(prompt_len)
    for n, (a, kn) in enumerate(zip(attr_lens, value_lens)):
        kind += [KIND_ATTR] * int(a)
        attr += [n] * int(a)
        k += [0] * int(a)
        kind += [KIND_VALUE] * int(kn)
        attr += [n] * int(kn)
        k += list(range(1, int(kn) + 1))
    return np.asarray(kind), np.asarray(attr), np.asarray(k)


def finetune_position_ids(prompt_len, attr_lens, value_lens, k_max):
    """Position IDs of s_train: Algorithm 2 for prompt and attributes, pos_id[end(a_n)] + k for
    the value tokens."""
    pos = list(range(int(prompt_len)))
    nxt = int(prompt_len)  # ordinary position of the next skeleton token
    offset = 0
    for a, kn in zip(attr_lens, value_lens):
        assert 0 <= kn <= k_max, "a value longer than K_max does not fit its gap"
        for _ in range(int(a)):
            pos.append(nxt + offset)
            nxt += 1
        end_pos = pos[-1]
        pos.extend(end_pos + kk for kk in range(1, int(kn) + 1))
        offset += int(k_max)
    return np.asarray(pos, dtype=np.int64)


def finetune_mask(prompt_len, attr_lens, value_lens):
    """Dense 0/1 mask [S, S] (query row, key column) over s_train."""
    kind, attr, k = finetune_tokens(prompt_len, attr_lens, value_lens)
    s = len(kind)
    m = np.zeros((s, s), dtype=np.uint8)
    for qi in range(s):
        for ki in range(qi + 1):  # standard causal mask
            ok = True
            if kind[ki] == KIND_VALUE:
                if kind[qi] == KIND_ATTR:
                    ok = False  # attribute tokens never see value tokens
                elif kind[qi] == KIND_VALUE and attr[ki] < attr[qi] and k[ki] > k[qi]:
                    ok = False  # not generated yet when (n, k) is decoded in parallel
            m[qi, ki] = 1 if ok else 0
    return m
