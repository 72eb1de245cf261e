"""CPU oracle for Hyper-Parallel Decoding (HPD) masked decode attention.

TEST INFRASTRUCTURE ONLY.  This is the plain, slow, dense formulation the paper
itself runs (Section 4.3.2: scaled dot-product attention with an explicit,
non-triangular mask; Limitations, "Compatibility"): an explicit position-ID
vector, an explicit dense 0/1 mask over a flat append-at-end KV cache, RoPE,
masked softmax attention.  No tiling, no fusion, no sharing of prefix work.
Only tests, the smoke check and the benchmark's CPU-baseline leg may use it;
the product path never imports it, and it imports nothing from the product.

Arithmetic is NumPy in ``dtype`` (fp32 by default, fp64 on request); RoPE
angles are always formed in fp64 and then cast.  Nothing is rounded in between,
with one optional exception: ``cache_dtype="bf16"`` stores the rotated key in
the cache rounded (to nearest even) to bfloat16, the storage type of the KV
cache in the paper's bf16 inference (Appendix B, "Fine-tuning and Inference
Details").  A cache entry is a quantised code; when the compared implementation
keeps a bf16 cache, both sides have to take that rounding in the same precision
or the comparison measures the cache format instead of the implementation.

What each piece follows
-----------------------
* ``alg2_position_ids``  - Appendix A.1, Algorithm 2 (gaps of K_max between
  attributes) and the rule "value token k of attribute n gets
  pos_id[end(a_n)] + k" (first paragraph of Appendix A.1).
* memory order          - Section 4.3.2 / Figure 2 caption: new tokens are
  always appended at the end of the cache, step after step.
* mask                  - Section 4.3.2: causal in *position-ID order*, not in
  memory order.  ``mask_mode="block"`` restricts it to the blocks a token may
  see (shared header, own document, own branch), which makes Eq. 3's
  independence exact.  ``mask_mode="paper"`` is the section's rule taken
  literally over the whole stacked prompt: a token sees every token of its
  prompt that is already in memory and has a position ID not larger than its
  own - all stacked documents and the value tokens of the earlier attributes
  up to its own step (Section 4.4 states the same for fine-tuning: v_{n,k} may not
  see v_{n',k'} with n' < n and k' > k, so k' <= k it does see).  It needs the
  paper's own position IDs (``pos_mode="paper_gap"``): with positions that
  restart per document "position order" would mix the documents.  Under this
  mask the skeleton (attribute-name) tokens a_1..a_N are cache entries as in the
  paper's input s = cat(p, a_1:N): they are fed with the prompt (memory order
  [header | documents | a_1 .. a_N]) at Algorithm 2's positions, so a value token
  also sees the attribute names up to its own.  Under the block mask they only
  shape the position IDs.
* first inference step  - Section 4.3.2 ("First Inference Step"): the whole input is fed
  once; ``prefill_attention`` is the attention of that pass for the header and
  document tokens (every token a query, causal in position order inside the blocks
  it may see).
* decode step           - Section 4.3.3: only the new tokens are fed, positions
  are the previous ones plus one.
* pruning               - Section 4.3.4: a finished value is fed no more.
* stacking / batching   - Sections 4.3.5 and 4.3.6.
* slot b*K_max + t      - Algorithm 1's ``values = empty(J, N, K_max)`` and its
  ``d[jN+i]`` branch order.

Pins (tests/test_oracle_*.py): the worked position example of Section 4.3.2 /
Figure 2 (golden file), closed forms for positions / mask row sums / slots,
equality with ordinary causal attention over the contiguous sequence
[header, own document, own branch] computed by a library routine with an
independently written complex-number RoPE, single-branch reduction to standard
causal decoding, RoPE identities, memory-order permutation invariance, branch
independence, and an fp64 triple-loop brute force on tiny inputs.  The
paper-literal mask is pinned by: equality with ordinary causal attention (library
routine) over all tokens in memory *sorted by position ID*, the closed-form row
sums, an explicit set construction, reduction to the block mask for one document
with one attribute, and its own scalar brute force.
The bf16 key cache is pinned by: ``round_to_bf16`` against the library's float32 ->
bfloat16 conversion bit for bit over every exponent, hand-computed ties, carries,
subnormals and infinities; and the cached oracle against the unrounded one (only
the stored keys differ, by exactly that conversion; outputs equal the plain
definition over the converted keys).  Algorithm 2 is also pinned by a token-by-token
walk along s that reserves K_max IDs behind every attribute.
The paper-gap position mode with several stacked documents is a reading of
this build (the paper writes Algorithm 2 for one document only); it is pinned
by closed form only.
"""
from __future__ import annotations

import numpy as np

KIND_HEADER, KIND_DOC, KIND_BRANCH, KIND_SKELETON = 0, 1, 2, 3


# ----------------------------------------------------------------------------
# Position IDs
# ----------------------------------------------------------------------------
def alg2_position_ids(prompt_len: int, attr_lens, k_max: int):
    """Position IDs of s = cat(p, a_1..a_N) with room for K_max value tokens behind
    every attribute (Appendix A.1, Algorithm 2), in closed form: the prompt keeps
    0 .. |p|-1, and token i (0-based) of attribute n (0-based) - whose index in s is
    |p| + A_0 + .. + A_{n-1} + i - sits n * K_max further on, one gap for every
    attribute in front of it.  Returns (pos_id[|s|], end_index[N]) where end_index[n]
    is the index in s of the last token of attribute n."""
    a = np.asarray([int(x) for x in attr_lens], dtype=np.int64)
    first = int(prompt_len) + np.concatenate([[0], np.cumsum(a)[:-1]]).astype(np.int64)  # index in s
    gaps_before = np.repeat(np.arange(len(a), dtype=np.int64), a)  # attribute of every skeleton token
    pos_id = np.concatenate([np.arange(int(prompt_len), dtype=np.int64),
                             int(prompt_len) + np.arange(int(a.sum()), dtype=np.int64) + gaps_before * int(k_max)])
    end_index = (first + a - 1).astype(np.int64)
    return pos_id, end_index


def value_position(pos_id, end_index, n: int, k: int) -> int:
    """Position ID of the k-th (1-based) value token of attribute n (0-based)."""
    return int(pos_id[end_index[n]]) + int(k)


# ----------------------------------------------------------------------------
# RoPE (rotate-half pairing, no frequency scaling)
# ----------------------------------------------------------------------------
def rope(x: np.ndarray, pos, base: float, dtype=np.float32) -> np.ndarray:
    """Rotate x[..., D] at integer position(s) ``pos`` (broadcast over leading
    axes: pos has shape x.shape[:-2] + (1,) or is scalar / [n] for x[n, heads, D])."""
    x = np.asarray(x, dtype=dtype)
    d = x.shape[-1]
    half = d // 2
    i = np.arange(half, dtype=np.float64)
    theta = np.float64(base) ** (-2.0 * i / d)
    pos = np.asarray(pos, dtype=np.float64)
    ang = pos[..., None] * theta  # [..., half]
    if x.ndim == 3 and ang.ndim == 2:  # x [n, heads, D], pos [n]
        ang = ang[:, None, :]
    c = np.cos(ang).astype(dtype)
    s = np.sin(ang).astype(dtype)
    x1 = x[..., :half]
    x2 = x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = x1 * c - x2 * s
    out[..., half:] = x2 * c + x1 * s
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest-even bfloat16, returned as fp32 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


# ----------------------------------------------------------------------------
# Dense masked attention (the plain definition)
# ----------------------------------------------------------------------------
def masked_attention(q, k, v, mask, n_kv_heads: int, dtype=np.float32):
    """q [R, Hq, D] (already rotated), k/v [S, Hkv, D] (k rotated),
    mask [R, S] of 0/1.  Returns softmax(q k^T / sqrt(D) masked) v  as [R, Hq, D].
    Query head h uses kv head h // (Hq / Hkv)."""
    q = np.asarray(q, dtype=dtype)
    k = np.asarray(k, dtype=dtype)
    v = np.asarray(v, dtype=dtype)
    r, hq, d = q.shape
    group = hq // n_kv_heads
    allowed = np.asarray(mask).astype(bool)
    out = np.zeros((r, hq, d), dtype=dtype)
    scale = dtype(1.0) / np.sqrt(dtype(d))
    for h in range(hq):
        hk = h // group
        s = (q[:, h, :] @ k[:, hk, :].T) * scale  # [R, S]
        s = np.where(allowed, s, dtype(-np.inf))
        m = s.max(axis=1, keepdims=True)
        p = np.exp(s - m)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, hk, :]
    return out


# ----------------------------------------------------------------------------
# One prompt
# ----------------------------------------------------------------------------
class PromptOracle:
    """Flat append-at-end KV cache of one prompt with explicit position IDs and
    an explicit dense mask."""

    def __init__(self, header_len, doc_lens, branch_lens, n_q_heads, n_kv_heads, head_dim,
                 rope_base, max_new, pos_mode="contig", attr_lens=None, dtype=np.float32,
                 cache_dtype=None, mask_mode="block"):
        self.cache_dtype = cache_dtype
        assert cache_dtype in (None, "bf16")
        assert mask_mode in ("block", "paper")
        assert mask_mode == "block" or pos_mode == "paper_gap", "the literal mask needs the paper's positions"
        self.mask_mode = mask_mode
        self.h = int(header_len)
        self.doc_lens = [int(x) for x in doc_lens]
        self.branch_lens = [[int(x) for x in bl] for bl in branch_lens]  # per doc
        assert len(self.branch_lens) == len(self.doc_lens)
        self.hq, self.hkv, self.d = int(n_q_heads), int(n_kv_heads), int(head_dim)
        self.attr_lens, self.skeleton_pos = [], []  # skeleton tokens in memory (literal mask only)
        self.base = float(rope_base)
        self.t_max = int(max_new)
        self.pos_mode = pos_mode
        self.dtype = dtype
        # local branch list in (doc, n) order  == the paper's d[jN+i] order
        self.branch_doc = [j for j, bl in enumerate(self.branch_lens) for _ in bl]
        self.branch_len = [x for bl in self.branch_lens for x in bl]
        for x in self.branch_len:
            assert 1 <= x <= self.t_max
        self.n_branches = len(self.branch_len)
        # ---- position IDs of the prefix and the base position of every branch
        if pos_mode == "contig":
            # every document restarts right after the header; a branch continues
            # from the end of its own document
            self.doc_pos0 = [self.h for _ in self.doc_lens]
            self.base_pos = [self.h + self.doc_lens[j] - 1 for j in self.branch_doc]
        elif pos_mode == "paper_gap":
            # the paper's own sequence: header and documents with ordinary
            # increasing positions, then the skeleton attributes with gaps
            assert attr_lens is not None and len(attr_lens) == self.n_branches
            self.doc_pos0 = []
            acc = self.h
            for l in self.doc_lens:
                self.doc_pos0.append(acc)
                acc += l
            pos_id, end_index = alg2_position_ids(acc, attr_lens, self.t_max)
            self.base_pos = [int(pos_id[e]) for e in end_index]
            if mask_mode == "paper":  # the skeleton is part of the input: s = cat(p, a_1..a_N)
                self.attr_lens = [int(a) for a in attr_lens]
                self.skeleton_pos = [int(x) for x in pos_id[acc:]]
        else:
            raise ValueError(pos_mode)
        # ---- flat memory (grows): per-token bookkeeping + KV
        self.kind, self.doc, self.branch, self.step_of, self.pos = [], [], [], [], []
        self.k = np.zeros((0, self.hkv, self.d), dtype=dtype)
        self.v = np.zeros((0, self.hkv, self.d), dtype=dtype)
        self.steps_done = 0

    # -- prefix ---------------------------------------------------------------
    @property
    def n_prefix(self):
        return self.h + sum(self.doc_lens) + len(self.skeleton_pos)

    def prefix_positions(self):
        pos = list(range(self.h))
        for j, l in enumerate(self.doc_lens):
            pos.extend(self.doc_pos0[j] + i for i in range(l))
        pos.extend(self.skeleton_pos)
        return np.asarray(pos, dtype=np.int64)

    def prefill(self, k_raw, v_raw):
        """k_raw, v_raw [n_prefix, Hkv, D] un-rotated, memory order
        [header | doc_0 | doc_1 | ...] (literal mask: followed by the skeleton tokens
        a_1 .. a_N of all attributes in (document, attribute) order)."""
        assert len(self.kind) == 0
        assert k_raw.shape == (self.n_prefix, self.hkv, self.d)
        self.kind = [KIND_HEADER] * self.h
        self.doc = [-1] * self.h
        for j, l in enumerate(self.doc_lens):
            self.kind.extend([KIND_DOC] * l)
            self.doc.extend([j] * l)
        self.branch = [-1] * (self.h + sum(self.doc_lens))
        for n, a in enumerate(self.attr_lens):
            self.kind.extend([KIND_SKELETON] * a)
            self.doc.extend([self.branch_doc[n]] * a)
            self.branch.extend([n] * a)
        self.step_of = [-1] * self.n_prefix
        pos = self.prefix_positions()
        self.pos = [int(x) for x in pos]
        self.k = self._to_cache(rope(k_raw, pos, self.base, self.dtype))
        self.v = np.asarray(v_raw, dtype=self.dtype).copy()

    def prefill_attention(self, q_raw):
        """Attention outputs of the prefix tokens themselves (the first inference step):
        q_raw [n_prefix, Hq, D] un-rotated, memory order as in ``prefill``.  Every prefix
        token is a query at its own position ID over the mask rows of the prefix.  Call
        after ``prefill`` and before the first decode step.  Returns [n_prefix, Hq, D]."""
        assert len(self.kind) == self.n_prefix and self.steps_done == 0
        assert q_raw.shape == (self.n_prefix, self.hq, self.d)
        rows = list(range(self.n_prefix))
        mask = self.mask_rows_fast(rows)
        qr = rope(q_raw, np.asarray(self.pos, dtype=np.int64), self.base, self.dtype)
        return masked_attention(qr, self.k, self.v, mask, self.hkv, self.dtype)

    def _to_cache(self, k_rot):
        if self.cache_dtype == "bf16":
            return round_to_bf16(k_rot).astype(self.dtype)
        return k_rot

    # -- liveness ---------------------------------------------------------------
    def live(self, t):
        """Local ids of the branches still being decoded at 0-based step t."""
        return [b for b in range(self.n_branches) if self.branch_len[b] > t]

    def branch_position(self, b, t):
        return self.base_pos[b] + 1 + t

    # -- mask -------------------------------------------------------------------
    def _visible_block(self, qi, ki):
        """May token qi ever look into the block token ki belongs to?"""
        if self.mask_mode == "paper":
            return True  # one causal order over the whole prompt: position IDs decide alone
        kk = self.kind[ki]
        if kk == KIND_HEADER:
            return True  # the header is shared by everything in the prompt
        qk = self.kind[qi]
        if kk == KIND_SKELETON:
            return False  # only the literal mask keeps skeleton tokens in memory
        if kk == KIND_DOC:
            return qk != KIND_HEADER and self.doc[qi] == self.doc[ki]
        # ki is a branch token: only its own branch sees it
        return qk == KIND_BRANCH and self.branch[qi] == self.branch[ki]

    def mask_rows(self, rows):
        """Dense 0/1 mask [len(rows), S] over the current memory.
        allowed  <=>  block visible  and  key already in memory  and
        pos[key] <= pos[query]   (causality in position-ID order)."""
        s = len(self.kind)
        m = np.zeros((len(rows), s), dtype=np.uint8)
        for r, qi in enumerate(rows):
            for ki in range(s):
                if ki <= qi and self._visible_block(qi, ki) and self.pos[ki] <= self.pos[qi]:
                    m[r, ki] = 1
        return m

    def dense_mask(self):
        """Full [S, S] mask of everything currently in memory."""
        return self.mask_rows(list(range(len(self.kind))))

    # -- one decode step ----------------------------------------------------------
    def step(self, t, q, k_new, v_new):
        """Decode step t for this prompt's live branches (ascending local id).
        q [n_live, Hq, D], k_new / v_new [n_live, Hkv, D], all un-rotated.
        Appends K (rotated) and V, then attends.  Returns
        (out [n_live, Hq, D], pos [n_live], flat_index [n_live])."""
        assert t == self.steps_done, "steps must be taken in order"
        live = self.live(t)
        n_live = len(live)
        assert q.shape == (n_live, self.hq, self.d)
        assert k_new.shape == (n_live, self.hkv, self.d) and v_new.shape == k_new.shape
        pos = np.asarray([self.branch_position(b, t) for b in live], dtype=np.int64)
        first = len(self.kind)
        if n_live:
            self.k = np.concatenate(
                [self.k, self._to_cache(rope(k_new, pos, self.base, self.dtype))], axis=0)
            self.v = np.concatenate([self.v, np.asarray(v_new, dtype=self.dtype)], axis=0)
        for r, b in enumerate(live):
            self.kind.append(KIND_BRANCH)
            self.doc.append(self.branch_doc[b])
            self.branch.append(b)
            self.step_of.append(t)
            self.pos.append(int(pos[r]))
        rows = list(range(first, first + n_live))
        self.steps_done += 1
        if n_live == 0:
            return (np.zeros((0, self.hq, self.d), dtype=self.dtype), pos,
                    np.zeros(0, dtype=np.int64))
        mask = self.mask_rows_fast(rows)
        qr = rope(q, pos, self.base, self.dtype)
        out = masked_attention(qr, self.k, self.v, mask, self.hkv, self.dtype)
        return out, pos, np.asarray(rows, dtype=np.int64)

    def mask_rows_fast(self, rows):
        """Same mask as ``mask_rows`` built with array comparisons (the per-element
        loop above is the definition; tests check the two agree)."""
        kind = np.asarray(self.kind)
        doc = np.asarray(self.doc)
        branch = np.asarray(self.branch)
        pos = np.asarray(self.pos)
        idx = np.arange(len(kind))
        rows = np.asarray(rows, dtype=np.int64)
        qk, qd, qb, qp = kind[rows, None], doc[rows, None], branch[rows, None], pos[rows, None]
        vis = (kind[None, :] == KIND_HEADER)
        vis = vis | ((kind[None, :] == KIND_DOC) & (qk != KIND_HEADER) & (qd == doc[None, :]))
        vis = vis | ((kind[None, :] == KIND_BRANCH) & (qk == KIND_BRANCH) & (qb == branch[None, :]))
        if self.mask_mode == "paper":
            vis = np.ones_like(vis)
        m = vis & (idx[None, :] <= rows[:, None]) & (pos[None, :] <= qp)
        return m.astype(np.uint8)


# ----------------------------------------------------------------------------
# A batch of prompts
# ----------------------------------------------------------------------------
class HPDOracle:
    """Batch wrapper: prompts are independent (Section 4.3.6); global branch ids
    run over (prompt, document, attribute)."""

    def __init__(self, header_len, doc_ptr, doc_len, branch_ptr, branch_len, n_q_heads,
                 n_kv_heads, head_dim, rope_base, max_new, pos_mode="contig", attr_len=None,
                 dtype=np.float32, prompts=None, cache_dtype=None, mask_mode="block"):
        """``prompts``: optional subset of prompt ids to instantiate (others are
        skipped entirely; global ids keep their full-batch values)."""
        header_len = np.asarray(header_len)
        doc_ptr = np.asarray(doc_ptr)
        doc_len = np.asarray(doc_len)
        branch_ptr = np.asarray(branch_ptr)
        n_br = int(branch_ptr[-1])
        if branch_len is None:
            branch_len = np.full(n_br, max_new, dtype=np.int64)
        branch_len = np.asarray(branch_len)
        self.t_max = int(max_new)
        self.hq, self.hkv, self.d = int(n_q_heads), int(n_kv_heads), int(head_dim)
        self.dtype = dtype
        self.n_prompts = int(header_len.shape[0])
        self.n_branches = n_br
        self.branch_len = branch_len.astype(np.int64)
        self.prompt_ids = list(range(self.n_prompts)) if prompts is None else sorted(prompts)
        self.prompts = {}
        self.prefix_range = {}  # prompt -> (first, last+1) global prefix token
        self.branch_range = {}  # prompt -> (first, last+1) global branch id
        tok = 0
        for p in range(self.n_prompts):
            d0, d1 = int(doc_ptr[p]), int(doc_ptr[p + 1])
            b0, b1 = int(branch_ptr[d0]), int(branch_ptr[d1])
            n_tok = int(header_len[p]) + int(doc_len[d0:d1].sum())
            if mask_mode == "paper":
                n_tok += int(np.asarray(attr_len)[b0:b1].sum())
            self.prefix_range[p] = (tok, tok + n_tok)
            self.branch_range[p] = (b0, b1)
            tok += n_tok
            if p in self.prompt_ids:
                bl = [[int(x) for x in branch_len[int(branch_ptr[d]):int(branch_ptr[d + 1])]]
                      for d in range(d0, d1)]
                al = None if attr_len is None else [int(x) for x in np.asarray(attr_len)[b0:b1]]
                self.prompts[p] = PromptOracle(int(header_len[p]), doc_len[d0:d1], bl, n_q_heads,
                                               n_kv_heads, head_dim, rope_base, max_new,
                                               pos_mode, al, dtype, cache_dtype, mask_mode)
        self.n_prefix_tokens = tok

    def live(self, t):
        """Global ids of all live branches at step t, ascending."""
        return np.nonzero(self.branch_len > t)[0]

    def prefill(self, k_raw, v_raw):
        """k_raw, v_raw: [n_prefix_tokens, Hkv, D] for the whole batch (global
        prefix-token order), or a dict prompt -> per-prompt arrays."""
        for p, po in self.prompts.items():
            if isinstance(k_raw, dict):
                po.prefill(np.asarray(k_raw[p]), np.asarray(v_raw[p]))
            else:
                a, b = self.prefix_range[p]
                po.prefill(np.asarray(k_raw[a:b]), np.asarray(v_raw[a:b]))

    def prefill_attention(self, q_raw):
        """q_raw [n_prefix_tokens, Hq, D] for the whole batch (or a dict prompt -> array):
        attention outputs of the prefix tokens of the instantiated prompts, as a dict
        prompt -> [n_prefix(prompt), Hq, D]."""
        out = {}
        for p, po in self.prompts.items():
            if isinstance(q_raw, dict):
                out[p] = po.prefill_attention(np.asarray(q_raw[p]))
            else:
                a, b = self.prefix_range[p]
                out[p] = po.prefill_attention(np.asarray(q_raw[a:b]))
        return out

    def step(self, t, q, k_new, v_new):
        """q [n_live, Hq, D], k_new / v_new [n_live, Hkv, D] for ALL live branches
        of the batch in ascending global id.  Only instantiated prompts are
        computed.  Returns dict with
          rows  : indices into the live list that were computed
          out   : [len(rows), Hq, D]
          pos   : [len(rows)] position IDs
          slot  : [len(rows)] per-branch tail slot  b*K_max + t
          flat  : [len(rows)] column in the owning prompt's flat cache."""
        live = self.live(t)
        rows, outs, poss, slots, flats = [], [], [], [], []
        for p, po in self.prompts.items():
            b0, b1 = self.branch_range[p]
            sel = np.nonzero((live >= b0) & (live < b1))[0]
            out, pos, flat = po.step(t, np.asarray(q[sel]), np.asarray(k_new[sel]),
                                     np.asarray(v_new[sel]))
            rows.append(sel)
            outs.append(out)
            poss.append(pos)
            flats.append(flat)
            slots.append(live[sel].astype(np.int64) * self.t_max + t)
        return {
            "rows": np.concatenate(rows) if rows else np.zeros(0, np.int64),
            "out": np.concatenate(outs, axis=0) if outs else np.zeros((0, self.hq, self.d), self.dtype),
            "pos": np.concatenate(poss) if poss else np.zeros(0, np.int64),
            "slot": np.concatenate(slots) if slots else np.zeros(0, np.int64),
            "flat": np.concatenate(flats) if flats else np.zeros(0, np.int64),
        }

    def positions(self, t):
        """Position IDs of all live branches at step t (instantiated prompts only
        return values; needs every prompt instantiated for a full vector)."""
        live = self.live(t)
        out = np.zeros(live.shape[0], dtype=np.int64)
        for p, po in self.prompts.items():
            b0, b1 = self.branch_range[p]
            for r in np.nonzero((live >= b0) & (live < b1))[0]:
                out[r] = po.branch_position(int(live[r]) - b0, t)
        return out
