"""ctypes binding of libsp.so: same entry-point names as include/sp.h, argument marshalling only.

Device tensors are torch CUDA tensors (PyTorch is used for device memory and streams only);
host tables are numpy arrays.  No computation happens here.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

SP_F32, SP_BF16 = 0, 1
SALIENCY_SUM, SALIENCY_MEAN = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def lib_path() -> str:
    return os.path.join(_HERE, "libsp.so")


class SpError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("sp status %d: %s" % (status, msg))
        self.status = status


class _SegTable(C.Structure):
    _fields_ = [("n_prompts", C.c_int32), ("n_segments", C.c_int32), ("n_tokens", C.c_int32),
                ("prompt_seg_off", C.c_void_p), ("seg_tok_start", C.c_void_p), ("seg_tok_len", C.c_void_p),
                ("seg_parent", C.c_void_p), ("seg_path", C.c_void_p), ("tok_pos", C.c_void_p),
                ("alibi_slopes", C.c_void_p), ("seg_cached", C.c_void_p)]


def lib() -> C.CDLL:
    """Load libsp.so (built in-tree by paper_2404_06910_amd.build).  Raises if it is missing:
    there is no fallback path."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("libsp.so not found at %s: run `python -m paper_2404_06910_amd.build` "
                          "(or __graft_entry__.build()) first; there is no CPU fallback" % path)
    L = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    sig = {
        "sp_create": (C.c_int, [C.POINTER(vp), C.c_int, vp]),
        "sp_destroy": (None, [vp]),
        "sp_set_stream": (C.c_int, [vp, vp]),
        "sp_last_error": (C.c_char_p, [vp]),
        "sp_version": (C.c_char_p, []),
        "sp_plan_create": (C.c_int, [vp, C.POINTER(_SegTable), i32, i32, i32, C.c_int, C.POINTER(vp)]),
        "sp_plan_destroy": (None, [vp]),
        "sp_plan_update": (C.c_int, [vp, C.POINTER(_SegTable)]),
        "sp_plan_info": (C.c_int, [vp, C.POINTER(i64)]),
        "sp_plan_visible_pairs": (i64, [vp]),
        "sp_plan_work_items": (i64, [vp, vp, i64, vp, i64]),
        "sp_plan_work_slots": (i64, [vp]),
        "sp_plan_key_ranges": (i64, [vp, vp, i64]),
        "sp_plan_path_offsets": (C.c_int, [vp, vp]),
        "sp_plan_path_offsets_device": (vp, [vp]),
        "sp_plan_visible_keys": (i64, [vp, i32, vp, i64]),
        "sp_plan_joined_keys": (i64, [vp, i32, vp, i32, vp, i64]),
        "sp_forkjoin_prefill": (C.c_int, [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, f32]),
        "sp_path_saliency": (C.c_int, [vp, vp, C.c_int, i64, i64, i64, vp, vp, vp, i32, C.c_int, vp]),
        "sp_path_saliency_static": (C.c_int, [vp, vp, C.c_int, i64, i64, i64, vp, vp, vp, i32, C.c_int, vp]),
        "sp_prune_topk": (C.c_int, [vp, vp, vp, i32, i32, i32, vp]),
        "sp_pruned_decode": (C.c_int, [vp, vp, vp, i32, vp, vp, i64, i64, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp,
                                       vp, f32]),
        "sp_equilibrium_positions": (C.c_int, [C.POINTER(_SegTable), vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _LIB = L
    return L


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _make_table(prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path, n_tokens, tok_pos=None,
                alibi_slopes=None, seg_cached=None, n_q_heads=None):
    keep = [_i32(prompt_seg_off), _i32(seg_tok_start), _i32(seg_tok_len), _i32(seg_parent), _i32(seg_path)]
    pos = None if tok_pos is None else np.ascontiguousarray(np.asarray(tok_pos, dtype=np.float32))
    slopes = None if alibi_slopes is None else np.ascontiguousarray(np.asarray(alibi_slopes, dtype=np.float32))
    cached = None if seg_cached is None else np.ascontiguousarray(np.asarray(seg_cached, dtype=np.uint8))
    # the C ABI takes plain pointers and cannot see how long the arrays are: check that here
    n_seg = len(keep[1])
    for name, a, n in (("seg_tok_len", keep[2], n_seg), ("seg_parent", keep[3], n_seg), ("seg_path", keep[4], n_seg),
                       ("tok_pos", pos, int(n_tokens)), ("seg_cached", cached, n_seg),
                       ("alibi_slopes", slopes, n_q_heads)):
        if a is not None and n is not None and a.size != n:
            raise ValueError("%s has %d entries, expected %d" % (name, a.size, n))
    t = _SegTable(len(keep[0]) - 1, len(keep[1]), int(n_tokens), _np_ptr(keep[0]), _np_ptr(keep[1]),
                  _np_ptr(keep[2]), _np_ptr(keep[3]), _np_ptr(keep[4]), _np_ptr(pos), _np_ptr(slopes),
                  _np_ptr(cached))
    return t, keep + [pos, slopes, cached]


def _dev(t, what: str) -> int:
    """Device pointer of a torch CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must be a CUDA tensor" % what)
    return t.data_ptr()


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return SP_F32
    if t.dtype == torch.bfloat16:
        return SP_BF16
    raise ValueError("unsupported tensor dtype %s" % t.dtype)


class Context:
    """sp_ctx: device + HIP stream (defaults to torch's current stream on that device)."""

    def __init__(self, device: int = 0, stream: Optional[int] = None):
        import torch
        self._h = C.c_void_p()
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        st = lib().sp_create(C.byref(self._h), device, C.c_void_p(stream))
        if st != 0:
            raise SpError(st, lib().sp_last_error(None).decode())
        self.device = device

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().sp_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != 0:
            raise SpError(st, lib().sp_last_error(self._h).decode())

    def sp_set_stream(self, stream: int):
        self._check(lib().sp_set_stream(self._h, C.c_void_p(stream)))

    # -- a1 ------------------------------------------------------------------------------
    def sp_forkjoin_prefill(self, plan: "Plan", Q, K, V, O, softmax_scale: float):
        if not (Q.stride(-1) == K.stride(-1) == V.stride(-1) == O.stride(-1) == 1):
            raise ValueError("innermost stride must be 1")
        if O.stride(0) != Q.stride(0) or O.stride(1) != Q.stride(1) or K.stride() != V.stride():
            raise ValueError("O must share Q's strides and V must share K's strides")
        if _dtype_code(Q) != plan.dtype:
            raise ValueError("tensor dtype does not match the plan")
        self._check(lib().sp_forkjoin_prefill(self._h, plan._h, _dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"),
                                              _dev(O, "O"), Q.stride(0), Q.stride(1), K.stride(0), K.stride(1),
                                              float(softmax_scale)))
        return O

    # -- a2 ------------------------------------------------------------------------------
    def sp_path_saliency(self, logits, target, row_path, n_path_slots: int, score, prior=None,
                         mode: int = SALIENCY_SUM, _entry: str = "sp_path_saliency"):
        if logits.dim() != 2 or logits.stride(1) != 1:
            raise ValueError("logits must be [rows, vocab] with unit inner stride")
        self._check(getattr(lib(), _entry)(self._h, _dev(logits, "logits"), _dtype_code(logits), logits.shape[0],
                                           logits.shape[1], logits.stride(0), _dev(target, "target"),
                                           _dev(row_path, "row_path"), _dev(prior, "prior"), int(n_path_slots),
                                           int(mode), _dev(score, "score")))
        return score

    def sp_path_saliency_static(self, logits, target, row_path, n_path_slots: int, score, prior=None,
                                mode: int = SALIENCY_SUM):
        return self.sp_path_saliency(logits, target, row_path, n_path_slots, score, prior, mode,
                                     _entry="sp_path_saliency_static")

    # -- a3 ------------------------------------------------------------------------------
    def sp_prune_topk(self, score, path_off, n_prompts: int, n_paths_max: int, k: int, kept):
        po = path_off if isinstance(path_off, int) else _dev(path_off, "path_off")
        self._check(lib().sp_prune_topk(self._h, _dev(score, "score"), po, int(n_prompts), int(n_paths_max), int(k),
                                        _dev(kept, "kept")))
        return kept

    # -- a4 ------------------------------------------------------------------------------
    def sp_pruned_decode(self, plan: "Plan", kept, k: int, K_prefill, V_prefill, K_resp, V_resp, resp_capacity: int,
                         q_new, k_new, v_new, o_out, softmax_scale: float, resp_len=None, resp_len_add: int = 0,
                         pos_resp=None, new_pos=None):
        if K_prefill.stride() != V_prefill.stride() or K_prefill.stride(-1) != 1:
            raise ValueError("K_prefill and V_prefill must share strides, inner stride 1")
        for t, n in ((K_resp, "K_resp"), (V_resp, "V_resp"), (q_new, "q_new"), (k_new, "k_new"), (v_new, "v_new"),
                     (o_out, "o_out")):
            if not t.is_contiguous():
                raise ValueError("%s must be contiguous" % n)
        self._check(lib().sp_pruned_decode(self._h, plan._h, _dev(kept, "kept"), int(k), _dev(K_prefill, "K_prefill"),
                                           _dev(V_prefill, "V_prefill"), K_prefill.stride(0), K_prefill.stride(1),
                                           _dev(K_resp, "K_resp"), _dev(V_resp, "V_resp"), _dev(pos_resp, "pos_resp"),
                                           int(resp_capacity), _dev(resp_len, "resp_len"), int(resp_len_add),
                                           _dev(new_pos, "new_pos"), _dev(q_new, "q_new"), _dev(k_new, "k_new"),
                                           _dev(v_new, "v_new"), _dev(o_out, "o_out"), float(softmax_scale)))
        return o_out


class Plan:
    """sp_plan.  ctx=None builds a host-only plan (inspection only, no GPU needed)."""

    def __init__(self, ctx: Optional[Context], prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path,
                 n_tokens: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, tok_pos=None,
                 alibi_slopes=None, seg_cached=None):
        t, keep = _make_table(prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path, n_tokens, tok_pos,
                              alibi_slopes, seg_cached, n_q_heads)
        self._h = C.c_void_p()
        self.ctx = ctx
        self.dtype = dtype
        self.n_q_heads = n_q_heads
        st = lib().sp_plan_create(ctx._h if ctx else None, C.byref(t), n_q_heads, n_kv_heads, head_dim, dtype,
                                  C.byref(self._h))
        del keep
        if st != 0:
            raise SpError(st, lib().sp_last_error(ctx._h if ctx else None).decode())
        self.n_prompts = t.n_prompts

    def update(self, prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path, n_tokens: int, tok_pos=None,
               alibi_slopes=None, seg_cached=None):
        """sp_plan_update: rebuild this plan in place for another segment table."""
        t, keep = _make_table(prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path, n_tokens, tok_pos,
                              alibi_slopes, seg_cached, self.n_q_heads)
        st = lib().sp_plan_update(self._h, C.byref(t))
        del keep
        if st != 0:
            raise SpError(st, lib().sp_last_error(self.ctx._h if self.ctx else None).decode())
        self.n_prompts = t.n_prompts

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            lib().sp_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def info(self) -> dict:
        a = (C.c_int64 * 8)()
        lib().sp_plan_info(self._h, a)
        names = ["n_prompts", "n_segments", "n_tokens", "n_path_slots", "n_row_groups", "n_tiles", "n_work_items",
                 "max_ranges"]
        return dict(zip(names, [int(x) for x in a]))

    def work_items(self):
        """sp_plan_work_items: (items [n, 8] int32, slot_begin [n_slots + 1] int32)."""
        n = int(lib().sp_plan_work_items(self._h, None, 0, None, 0))
        ns = int(lib().sp_plan_work_slots(self._h))
        items = np.zeros((max(n, 1), 8), dtype=np.int32)
        begin = np.zeros(ns + 1, dtype=np.int32)
        lib().sp_plan_work_items(self._h, _np_ptr(items), n, _np_ptr(begin), ns + 1)
        return items[:n], begin

    def key_ranges(self) -> np.ndarray:
        """sp_plan_key_ranges: [n, 2] int32 (first token, length)."""
        n = int(lib().sp_plan_key_ranges(self._h, None, 0))
        out = np.zeros((max(n, 1), 2), dtype=np.int32)
        lib().sp_plan_key_ranges(self._h, _np_ptr(out), n)
        return out[:n]

    def visible_pairs(self) -> int:
        return int(lib().sp_plan_visible_pairs(self._h))

    def path_offsets(self) -> np.ndarray:
        out = np.zeros(self.n_prompts + 1, dtype=np.int32)
        lib().sp_plan_path_offsets(self._h, _np_ptr(out))
        return out

    def path_offsets_device(self) -> int:
        return int(lib().sp_plan_path_offsets_device(self._h) or 0)

    def visible_keys(self, token: int) -> np.ndarray:
        n = lib().sp_plan_visible_keys(self._h, int(token), None, 0)
        if n < 0:
            raise SpError(int(n), "sp_plan_visible_keys")
        out = np.zeros(max(int(n), 1), dtype=np.int32)
        lib().sp_plan_visible_keys(self._h, int(token), _np_ptr(out), int(n))
        return out[:n]

    def joined_keys(self, prompt: int, kept: Sequence[int]) -> np.ndarray:
        kk = _i32(list(kept))
        n = lib().sp_plan_joined_keys(self._h, int(prompt), _np_ptr(kk), len(kk), None, 0)
        if n < 0:
            raise SpError(int(n), "sp_plan_joined_keys")
        out = np.zeros(max(int(n), 1), dtype=np.int32)
        lib().sp_plan_joined_keys(self._h, int(prompt), _np_ptr(kk), len(kk), _np_ptr(out), int(n))
        return out[:n]


def equilibrium_positions(prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path, n_tokens) -> np.ndarray:
    """sp_equilibrium_positions: host helper, returns fp32 [n_tokens]."""
    t, keep = _make_table(prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, seg_path, n_tokens)
    out = np.zeros(int(n_tokens), dtype=np.float32)
    st = lib().sp_equilibrium_positions(C.byref(t), _np_ptr(out))
    del keep
    if st != 0:
        raise SpError(st, lib().sp_last_error(None).decode())
    return out
