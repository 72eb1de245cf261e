"""Thin ctypes binding of libhpd.so: same names as include/hpd.h, argument
marshalling only.  Device buffers are passed as torch tensors (their
``data_ptr()``) or raw integer addresses; streams as ``torch.cuda.Stream``,
raw ``hipStream_t`` integers or None (= torch's current stream).

There is no fallback: if the library has not been built, importing this module
raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhpd.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first with `python -m paper_2604_26209_amd.build` "
        "(or __graft_entry__.build()); there is no CPU fallback")


def _load():
    # PyTorch owns the device memory and the streams handed to the library, so both must
    # talk to the same HIP runtime: bind to the libamdhip64 that torch ships (same SONAME
    # as the one the library was linked against) before the library itself is loaded.
    import torch

    hip = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(hip):
        ctypes.CDLL(hip, mode=ctypes.RTLD_GLOBAL)
    return ctypes.CDLL(LIB_PATH)


_lib = _load()

HPD_OK, HPD_E_INVALID, HPD_E_OVERFLOW, HPD_E_UNSUPPORTED, HPD_E_HIP, HPD_E_NOMEM, HPD_E_CAPACITY = 0, -1, -2, -3, -4, -5, -6
HPD_DYNAMIC_STATIC_MAX_BYTES = 1 << 20
HPD_F32, HPD_BF16 = 0, 1
HPD_POS_CONTIG, HPD_POS_PAPER_GAP = 0, 1
HPD_MASK_BLOCK = 0
HPD_MASK_PAPER = 1
HPD_FLAG_HOST_ONLY = 1
HPD_OUT_SAME, HPD_OUT_F32 = 0, 1
HPD_KEY_BLOCK = 32
(HPD_Q_COUNTS, HPD_Q_POOL_BYTES, HPD_Q_N_LIVE, HPD_Q_LIVE_BRANCH, HPD_Q_BRANCH_BASE_POS,
 HPD_Q_BRANCH_DOC, HPD_Q_SEG_OFF, HPD_Q_SEG_LEN, HPD_Q_SEG_POS0, HPD_Q_SEG_RAW_OFF,
 HPD_Q_N_UNITS) = range(11)
(HPD_C_N_PROMPTS, HPD_C_N_DOCS, HPD_C_N_BRANCHES, HPD_C_N_PREFIX_TOKENS, HPD_C_N_PREFIX_SLOTS,
 HPD_C_N_TAIL_SLOTS, HPD_C_MAX_POS, HPD_C_TOTAL_LIVE, HPD_N_COUNTS) = range(9)

EXPORTS = ["hpd_build_layout", "hpd_layout_free", "hpd_layout_query", "hpd_prefix_fill",
           "hpd_rope_positions", "hpd_kv_append", "hpd_decode_attention", "hpd_decode_step",
           "hpd_expand_mask", "hpd_set_kernel_mode", "hpd_status_string", "hpd_finetune_mask",
           "hpd_prefill_attention", "hpd_dynamic_begin", "hpd_dynamic_prune", "hpd_dynamic_step",
           "hpd_dynamic_state", "hpd_dynamic_read", "hpd_set_tail_pages", "hpd_dynamic_begin_static"]
# include/hpd_peaks.h: reference kernels for the benchmark's measured peaks
PEAK_EXPORTS = ["hpd_peak_read", "hpd_peak_copy", "hpd_peak_mfma"]


class hpd_config(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("rope_base", ctypes.c_double), ("max_new", ctypes.c_int32),
                ("pos_mode", ctypes.c_int32), ("mask_mode", ctypes.c_int32),
                ("flags", ctypes.c_int32), ("out_dtype", ctypes.c_int32)]


_vp, _i32, _i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_lib.hpd_build_layout.argtypes = [ctypes.POINTER(hpd_config), _i32, _i32p, _i32p, _i32p, _i32p,
                                  _i32p, _i32p, _vp, ctypes.POINTER(_vp)]
_lib.hpd_layout_free.argtypes = [_vp]
_lib.hpd_layout_free.restype = None
_lib.hpd_layout_query.argtypes = [_vp, _i32, _vp, ctypes.c_size_t]
_lib.hpd_prefix_fill.argtypes = [_vp] * 6
_lib.hpd_rope_positions.argtypes = [_vp, _i32, _vp, _i32p, _vp]
_lib.hpd_kv_append.argtypes = [_vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.hpd_decode_attention.argtypes = [_vp, _i32] + [_vp] * 7
_lib.hpd_decode_step.argtypes = [_vp, _i32] + [_vp] * 9
_lib.hpd_expand_mask.argtypes = [_vp, _i32, _i32, _vp, _i32p, _vp]
_lib.hpd_set_kernel_mode.argtypes = [_vp, _i32]
_lib.hpd_prefill_attention.argtypes = [_vp] * 6
_lib.hpd_dynamic_begin.argtypes = [_vp, _vp]
_lib.hpd_dynamic_begin_static.argtypes = [_vp, _vp]
_lib.hpd_dynamic_prune.argtypes = [_vp, _vp, _vp]
_lib.hpd_dynamic_step.argtypes = [_vp, _i32] + [_vp] * 9
_lib.hpd_dynamic_state.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp)]
_lib.hpd_dynamic_read.argtypes = [_vp, _i32p, _i32, _i32p, _vp]
_lib.hpd_set_tail_pages.argtypes = [_vp, _i32, _i32, _vp]
_lib.hpd_finetune_mask.argtypes = [_i32, _i32, _i32p, _i32p, _i32, _vp, _vp, ctypes.POINTER(ctypes.c_int64), _vp]
_lib.hpd_peak_read.argtypes = [_vp, ctypes.c_size_t, _vp, _vp]
_lib.hpd_peak_copy.argtypes = [_vp, _vp, ctypes.c_size_t, _vp]
_lib.hpd_peak_mfma.argtypes = [_vp, _i32, ctypes.POINTER(ctypes.c_double), _vp]
for _name in PEAK_EXPORTS:
    getattr(_lib, _name).restype = ctypes.c_int
_lib.hpd_status_string.argtypes = [ctypes.c_int]
_lib.hpd_status_string.restype = ctypes.c_char_p
for _name in EXPORTS:
    if _name not in ("hpd_layout_free", "hpd_status_string"):
        getattr(_lib, _name).restype = ctypes.c_int


class HpdError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {hpd_status_string(status)} ({status})")


def hpd_status_string(status: int) -> str:
    return _lib.hpd_status_string(int(status)).decode()


def _check(status, where):
    if status != HPD_OK:
        raise HpdError(status, where)


def _ptr(x):
    """Device or host address of a tensor / integer / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(s):
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def _host_i32(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(np.asarray(a), dtype=np.int32)
    return arr, arr.ctypes.data_as(_i32p)


class hpd_layout:
    """Owner of an opaque ``hpd_layout*``."""

    def __init__(self, handle, cfg):
        self.handle = handle
        self.cfg = cfg

    def free(self):
        if self.handle:
            _lib.hpd_layout_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    # convenience accessors built on hpd_layout_query
    def counts(self):
        return hpd_layout_query(self, HPD_Q_COUNTS)

    def n_live(self):
        return hpd_layout_query(self, HPD_Q_N_LIVE)


def hpd_build_layout(cfg: hpd_config, header_len, doc_ptr, doc_len, branch_ptr, branch_len=None,
                     attr_len=None, stream=None) -> hpd_layout:
    keep = []
    args = []
    for a in (header_len, doc_ptr, doc_len, branch_ptr, branch_len, attr_len):
        arr, p = _host_i32(a)
        keep.append(arr)
        args.append(p)
    n_prompts = int(np.asarray(header_len).shape[0])
    out = _vp()
    st = None if (cfg.flags & HPD_FLAG_HOST_ONLY) else _stream(stream)
    rc = _lib.hpd_build_layout(ctypes.byref(cfg), n_prompts, *args, st, ctypes.byref(out))
    _check(rc, "hpd_build_layout")
    return hpd_layout(out.value, cfg)


def hpd_layout_free(layout: hpd_layout):
    layout.free()


def hpd_layout_query(layout: hpd_layout, what: int):
    """Returns the selected table as a NumPy array."""
    h = layout.handle
    if what == HPD_Q_COUNTS:
        out = np.zeros(HPD_N_COUNTS, dtype=np.int64)
    elif what == HPD_Q_POOL_BYTES:
        out = np.zeros(4, dtype=np.int64)
    else:
        c = np.zeros(HPD_N_COUNTS, dtype=np.int64)
        _check(_lib.hpd_layout_query(h, HPD_Q_COUNTS, c.ctypes.data, c.nbytes), "hpd_layout_query")
        n_seg = int(c[HPD_C_N_PROMPTS] + c[HPD_C_N_DOCS])
        if layout.cfg.mask_mode == HPD_MASK_PAPER:  # plus one skeleton segment per prompt
            n_seg += int(c[HPD_C_N_PROMPTS])
        size = {HPD_Q_N_LIVE: layout.cfg.max_new, HPD_Q_N_UNITS: layout.cfg.max_new,
                HPD_Q_LIVE_BRANCH: int(c[HPD_C_TOTAL_LIVE]),
                HPD_Q_BRANCH_BASE_POS: int(c[HPD_C_N_BRANCHES]),
                HPD_Q_BRANCH_DOC: int(c[HPD_C_N_BRANCHES]), HPD_Q_SEG_OFF: n_seg,
                HPD_Q_SEG_LEN: n_seg, HPD_Q_SEG_POS0: n_seg, HPD_Q_SEG_RAW_OFF: n_seg}[what]
        out = np.zeros(max(size, 1), dtype=np.int32)[:size]
        if size == 0:
            return out
    _check(_lib.hpd_layout_query(h, int(what), out.ctypes.data, out.nbytes), "hpd_layout_query")
    return out


def hpd_prefix_fill(layout, k_raw, v_raw, k_prefix, v_prefix, stream=None):
    _check(_lib.hpd_prefix_fill(layout.handle, _ptr(k_raw), _ptr(v_raw), _ptr(k_prefix),
                                _ptr(v_prefix), _stream(stream)), "hpd_prefix_fill")


def hpd_rope_positions(layout, step, pos_out, stream=None) -> int:
    n = ctypes.c_int32(0)
    _check(_lib.hpd_rope_positions(layout.handle, int(step), _ptr(pos_out), ctypes.byref(n),
                                   _stream(stream)), "hpd_rope_positions")
    return int(n.value)


def hpd_kv_append(layout, step, k_new, v_new, k_tail, v_tail, slot_out=None, stream=None):
    _check(_lib.hpd_kv_append(layout.handle, int(step), _ptr(k_new), _ptr(v_new), _ptr(k_tail),
                              _ptr(v_tail), _ptr(slot_out), _stream(stream)), "hpd_kv_append")


def hpd_decode_attention(layout, step, q, k_prefix, v_prefix, k_tail, v_tail, out, stream=None):
    _check(_lib.hpd_decode_attention(layout.handle, int(step), _ptr(q), _ptr(k_prefix),
                                     _ptr(v_prefix), _ptr(k_tail), _ptr(v_tail), _ptr(out),
                                     _stream(stream)), "hpd_decode_attention")


def hpd_decode_step(layout, step, q, k_new, v_new, k_prefix, v_prefix, k_tail, v_tail, out,
                    stream=None):
    _check(_lib.hpd_decode_step(layout.handle, int(step), _ptr(q), _ptr(k_new), _ptr(v_new),
                                _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tail), _ptr(v_tail),
                                _ptr(out), _stream(stream)), "hpd_decode_step")


def hpd_prefill_attention(layout, q, k_prefix, v_prefix, out, stream=None):
    _check(_lib.hpd_prefill_attention(layout.handle, _ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(out),
                                      _stream(stream)), "hpd_prefill_attention")


def hpd_dynamic_begin(layout, stream=None):
    _check(_lib.hpd_dynamic_begin(layout.handle, _stream(stream)), "hpd_dynamic_begin")


def hpd_dynamic_begin_static(layout, stream=None):
    _check(_lib.hpd_dynamic_begin_static(layout.handle, _stream(stream)), "hpd_dynamic_begin_static")


def hpd_dynamic_prune(layout, finished, stream=None):
    _check(_lib.hpd_dynamic_prune(layout.handle, _ptr(finished), _stream(stream)), "hpd_dynamic_prune")


def hpd_dynamic_step(layout, step, q, k_new, v_new, k_prefix, v_prefix, k_tail, v_tail, out, stream=None):
    _check(_lib.hpd_dynamic_step(layout.handle, int(step), _ptr(q), _ptr(k_new), _ptr(v_new),
                                 _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tail), _ptr(v_tail),
                                 _ptr(out), _stream(stream)), "hpd_dynamic_step")


def hpd_dynamic_state(layout):
    """Device addresses (ints) of the live list (int32 [B]) and of n_live (int32 [1])."""
    live, n = _vp(), _vp()
    _check(_lib.hpd_dynamic_state(layout.handle, ctypes.byref(live), ctypes.byref(n)), "hpd_dynamic_state")
    return int(live.value), int(n.value)


def hpd_set_tail_pages(layout, page_size, n_pages=0, page_table=None) -> None:
    """page_table: int32 device tensor [B][ceil(T / page_size)] that the caller keeps alive and
    updates; page_size = 0 switches paging off."""
    if page_table is not None and not isinstance(page_table, int):
        import torch
        if page_table.dtype != torch.int32 or not page_table.is_cuda or not page_table.is_contiguous():
            raise TypeError("page_table: a contiguous int32 device tensor")
    _check(_lib.hpd_set_tail_pages(layout.handle, int(page_size), int(n_pages), _ptr(page_table)),
           "hpd_set_tail_pages")


def hpd_dynamic_read(layout, capacity, stream=None):
    """(n_live, live list as a NumPy array) of the device-side state; synchronises."""
    live = np.zeros(max(int(capacity), 1), dtype=np.int32)
    n = ctypes.c_int32(0)
    _check(_lib.hpd_dynamic_read(layout.handle, live.ctypes.data_as(_i32p), int(capacity), ctypes.byref(n),
                                 _stream(stream)), "hpd_dynamic_read")
    return int(n.value), live[:min(int(n.value), int(capacity))]


def hpd_expand_mask(layout, prompt, step_hi, mask_out=None, stream=None) -> int:
    s = ctypes.c_int32(0)
    _check(_lib.hpd_expand_mask(layout.handle, int(prompt), int(step_hi), _ptr(mask_out),
                                ctypes.byref(s), _stream(stream)), "hpd_expand_mask")
    return int(s.value)


def hpd_finetune_mask(prompt_len, attr_len, value_len, k_max, pos_out=None, mask_out=None, stream=None) -> int:
    """Returns S; fills the device tensors pos_out (int32 [S]) / mask_out (uint8 [S][S]) if given."""
    a = np.ascontiguousarray(attr_len, dtype=np.int32)
    v = np.ascontiguousarray(value_len, dtype=np.int32)
    s = ctypes.c_int64(0)
    _check(_lib.hpd_finetune_mask(int(prompt_len), int(a.shape[0]), a.ctypes.data_as(_i32p),
                                  v.ctypes.data_as(_i32p), int(k_max), _ptr(pos_out), _ptr(mask_out),
                                  ctypes.byref(s), _stream(stream)), "hpd_finetune_mask")
    return int(s.value)


def hpd_peak_read(src, nbytes, sink, stream=None):
    _check(_lib.hpd_peak_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)), "hpd_peak_read")


def hpd_peak_copy(dst, src, nbytes, stream=None):
    _check(_lib.hpd_peak_copy(_ptr(dst), _ptr(src), int(nbytes), _stream(stream)), "hpd_peak_copy")


def hpd_peak_mfma(sink, iters, stream=None) -> float:
    """Enqueues the MFMA loop; returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(_lib.hpd_peak_mfma(_ptr(sink), int(iters), ctypes.byref(flops), _stream(stream)), "hpd_peak_mfma")
    return float(flops.value)


def hpd_set_kernel_mode(layout, mode: int):
    _check(_lib.hpd_set_kernel_mode(layout.handle, int(mode)), "hpd_set_kernel_mode")



# ---------------------------------------------------------------------------
# marshalling helpers (no arithmetic of the method)
# ---------------------------------------------------------------------------
def config_from_workload(wl, pos_mode=HPD_POS_CONTIG, flags=0, out_dtype=HPD_OUT_SAME,
                         mask_mode=HPD_MASK_BLOCK) -> hpd_config:
    return hpd_config(wl.n_q_heads, wl.n_kv_heads, wl.head_dim,
                      HPD_F32 if wl.dtype == "f32" else HPD_BF16, float(wl.rope_base),
                      wl.max_new, pos_mode, mask_mode, flags, out_dtype)


def layout_from_workload(wl, pos_mode=HPD_POS_CONTIG, attr_len=None, flags=0, stream=None,
                         out_dtype=HPD_OUT_SAME, mask_mode=HPD_MASK_BLOCK):
    cfg = config_from_workload(wl, pos_mode, flags, out_dtype, mask_mode)
    return hpd_build_layout(cfg, wl.header_len, wl.doc_ptr, wl.doc_len, wl.branch_ptr,
                            wl.branch_len, attr_len, stream)


def alloc_pools(layout, device="cuda"):
    """Allocates the four KV pools as flat torch tensors of the layout's dtype."""
    import torch
    sizes = hpd_layout_query(layout, HPD_Q_POOL_BYTES)
    dt = torch.float32 if layout.cfg.dtype == HPD_F32 else torch.bfloat16
    eb = 4 if layout.cfg.dtype == HPD_F32 else 2
    return [torch.empty(int(s) // eb, dtype=dt, device=device) for s in sizes]
