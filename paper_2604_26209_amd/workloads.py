"""Seeded synthetic inputs for HPD masked decode attention.

This module only draws shapes and random values.  It contains none of the
method's arithmetic (no positions, masks, live lists, RoPE or attention), so
both the CPU oracle's tests and the HIP path can be fed from it without
sharing any logic.

The structures stand in for the paper's attribute-value-extraction prompts
(Section 4.3.5, Appendix B): a shared instruction/attribute header, J stacked
documents, N attribute branches per document, and a maximum value length
K_max.  Datasets and model weights are not available, and attention cost only
depends on shapes, so Q/K/V are i.i.d. N(0,1) draws.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

STRUCT_SEED = 26209000  # structure RNG seed base; config k uses STRUCT_SEED + k


@dataclass
class Workload:
    """Shape of one batch of HPD prompts (CSR over prompts -> docs -> branches)."""

    name: str
    dtype: str  # "f32" or "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    max_new: int  # K_max: number of decode steps / tail capacity per branch
    header_len: np.ndarray  # int32 [P]
    doc_ptr: np.ndarray  # int32 [P+1]
    doc_len: np.ndarray  # int32 [n_docs]
    branch_ptr: np.ndarray  # int32 [n_docs+1]
    branch_len: np.ndarray  # int32 [n_branches], each in [1, max_new]
    value_seed: int = 1
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n_prompts(self) -> int:
        return int(self.header_len.shape[0])

    @property
    def n_docs(self) -> int:
        return int(self.doc_len.shape[0])

    @property
    def n_branches(self) -> int:
        return int(self.branch_len.shape[0])

    @property
    def n_prefix_tokens(self) -> int:
        """Header and document tokens of all prompts, in prompt order."""
        return int(self.header_len.sum() + self.doc_len.sum())


def make_workload(
    name,
    dtype,
    n_q_heads,
    n_kv_heads,
    head_dim,
    rope_base,
    max_new,
    header_len,
    docs_per_prompt,
    doc_len,
    branches_per_doc,
    branch_len=None,
    value_seed=1,
    note="",
) -> Workload:
    """Assemble CSR arrays from per-prompt / per-document lists."""
    header_len = np.asarray(header_len, dtype=np.int32)
    docs_per_prompt = np.asarray(docs_per_prompt, dtype=np.int64)
    doc_len = np.asarray(doc_len, dtype=np.int32)
    branches_per_doc = np.asarray(branches_per_doc, dtype=np.int64)
    assert docs_per_prompt.shape[0] == header_len.shape[0]
    assert doc_len.shape[0] == docs_per_prompt.sum()
    assert branches_per_doc.shape[0] == doc_len.shape[0]
    doc_ptr = np.zeros(header_len.shape[0] + 1, dtype=np.int32)
    doc_ptr[1:] = np.cumsum(docs_per_prompt)
    branch_ptr = np.zeros(doc_len.shape[0] + 1, dtype=np.int32)
    branch_ptr[1:] = np.cumsum(branches_per_doc)
    n_br = int(branch_ptr[-1])
    if branch_len is None:
        branch_len = np.full(n_br, max_new, dtype=np.int32)
    branch_len = np.asarray(branch_len, dtype=np.int32)
    assert branch_len.shape[0] == n_br
    return Workload(
        name=name,
        dtype=dtype,
        n_q_heads=n_q_heads,
        n_kv_heads=n_kv_heads,
        head_dim=head_dim,
        rope_base=float(rope_base),
        max_new=int(max_new),
        header_len=header_len,
        doc_ptr=doc_ptr,
        doc_len=doc_len,
        branch_ptr=branch_ptr,
        branch_len=branch_len,
        value_seed=value_seed,
        note=note,
    )


def uniform_workload(name, dtype, hq, hkv, d, base, t, p, h, j, l, n, value_seed=1, note=""):
    """P identical prompts: header h, j documents of l tokens, n branches each, all of length t."""
    return make_workload(
        name, dtype, hq, hkv, d, base, t,
        header_len=[h] * p,
        docs_per_prompt=[j] * p,
        doc_len=[l] * (p * j),
        branches_per_doc=[n] * (p * j),
        value_seed=value_seed,
        note=note,
    )


def config(k: int, n_prompts: int | None = None) -> Workload:
    """The k-th benchmark configuration (1-based).  ``n_prompts`` overrides the
    prompt count (used by tests that want the same shape on fewer prompts)."""
    if k == 1:
        p = n_prompts or 1
        return uniform_workload("cfg1_tiny_f32", "f32", 4, 4, 64, 10000.0, 8, p, 16, 1, 48, 4,
                                value_seed=101, note="tiny fp32 MHA layer")
    if k == 2:
        p = n_prompts or 32
        return uniform_workload("cfg2_llama3_8b", "bf16", 32, 8, 128, 500000.0, 16, p, 64, 1, 512, 16,
                                value_seed=102, note="Llama-3-8B-like GQA 32/8 x 128")
    if k == 3:
        p = n_prompts or 64
        return uniform_workload("cfg3_stacked", "bf16", 32, 8, 128, 500000.0, 12, p, 64, 4, 384, 24,
                                value_seed=103, note="4 stacked documents, 96 branches per prompt")
    if k == 4:
        p = n_prompts or 16
        return uniform_workload("cfg4_long_70b", "bf16", 64, 8, 128, 500000.0, 32, p, 128, 2, 2048, 48,
                                value_seed=104, note="70B-like GQA 64/8 x 128, long documents")
    if k == 5:
        p = n_prompts or 128
        t = 32
        rng = np.random.default_rng(STRUCT_SEED + 5)
        docs_per_prompt, doc_len, branches_per_doc, branch_len = [], [], [], []
        for _ in range(p):
            j = int(rng.integers(1, 9))  # 1..8 stacked documents
            docs_per_prompt.append(j)
            for _ in range(j):
                l = int(rng.integers(64, 2049))  # document length 64..2048
                n = int(rng.integers(4, 25))  # 4..24 branches
                doc_len.append(l)
                branches_per_doc.append(n)
                branch_len.extend(int(x) for x in rng.integers(1, t + 1, size=n))  # early EOS
        return make_workload("cfg5_ragged", "bf16", 32, 8, 128, 500000.0, t,
                             header_len=[64] * p, docs_per_prompt=docs_per_prompt, doc_len=doc_len,
                             branches_per_doc=branches_per_doc, branch_len=branch_len,
                             value_seed=105, note="ragged mixed batch with early EOS")
    raise ValueError(f"unknown config {k}")


def random_workload(seed, dtype="f32", hq=4, hkv=2, d=64, base=10000.0, t=6, p=3,
                    h_range=(0, 40), j_range=(1, 4), l_range=(1, 80), n_range=(1, 6),
                    ragged_len=True) -> Workload:
    """Small random ragged batch for parity and property tests."""
    rng = np.random.default_rng(seed)
    header_len, docs_per_prompt, doc_len, branches_per_doc, branch_len = [], [], [], [], []
    for _ in range(p):
        header_len.append(int(rng.integers(h_range[0], h_range[1] + 1)))
        j = int(rng.integers(j_range[0], j_range[1] + 1))
        docs_per_prompt.append(j)
        for _ in range(j):
            doc_len.append(int(rng.integers(l_range[0], l_range[1] + 1)))
            n = int(rng.integers(n_range[0], n_range[1] + 1))
            branches_per_doc.append(n)
            if ragged_len:
                branch_len.extend(int(x) for x in rng.integers(1, t + 1, size=n))
            else:
                branch_len.extend([t] * n)
    return make_workload(f"random_{seed}", dtype, hq, hkv, d, base, t, header_len, docs_per_prompt,
                         doc_len, branches_per_doc, branch_len, value_seed=seed)


def normal_values(shape, seed, device="cpu", dtype="f32"):
    """N(0,1) draws as a torch tensor on ``device``; bf16 draws are the bf16
    roundings of fp32 N(0,1) draws.  The stream depends on (seed, device type)."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    x = torch.randn(tuple(int(s) for s in shape), generator=gen, device=device, dtype=torch.float32)
    if dtype == "bf16":
        return x.to(torch.bfloat16)
    if dtype == "f32":
        return x
    raise ValueError(dtype)
