"""ctypes front end of the CPU oracle (oracle/gr_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg.  The product package never imports this module, and this module never imports
the product package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gr_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall"]
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", *CFLAGS, _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_check_table.restype = ctypes.c_int64
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a, dtype):
    assert a is None or (a.dtype == dtype and a.flags["C_CONTIGUOUS"]), (None if a is None else (a.dtype, dtype))
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def attn_unified(q, k_shared, v_shared, cu_seqlens, k_unshared, v_unshared, u, sm_scale, triples=None):
    """Unified-cache attention.  bf16 tensors are uint16 bit patterns.

    q [B,W,Hq,d]; k_shared/v_shared [total_L,Hkv,d]; k_unshared/v_unshared [B,W,ND,Hkv,d].
    triples: int32 [n,3] rows (b, w, hq) to evaluate, default all in (b, w, hq) order.
    Returns (out fp64 [n,d], lse fp64 [n]).
    """
    lib = _load()
    B, W, Hq, d = q.shape
    Hkv = k_shared.shape[1]
    ND = k_unshared.shape[2]
    if triples is None:
        bb, ww, hh = np.meshgrid(np.arange(B), np.arange(W), np.arange(Hq), indexing="ij")
        triples = np.stack([bb.ravel(), ww.ravel(), hh.ravel()], axis=1)
    triples = np.ascontiguousarray(triples, dtype=np.int32)
    n = triples.shape[0]
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty(n, dtype=np.float64)
    rc = lib.oracle_attn_unified(
        ctypes.c_int(B), ctypes.c_int(W), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(ND),
        ctypes.c_int(int(u)), ctypes.c_float(float(sm_scale)),
        _p(q, np.uint16), _p(k_shared, np.uint16), _p(v_shared, np.uint16), _p(cu_seqlens, np.int32),
        _p(k_unshared, np.uint16), _p(v_unshared, np.uint16), _p(triples, np.int32), ctypes.c_int64(n),
        _p(out, np.float64), _p(lse, np.float64))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_unified failed: {rc}")
    return out, lse


def attn_unified_f32kv(q, k_shared_f32, v_shared_f32, cu_seqlens, k_unshared, v_unshared, u, sm_scale, triples=None):
    """Unified-cache attention with the prompt K/V given as fp32 values (a narrower storage format, already widened).

    q, k_unshared, v_unshared: bf16 bit patterns as in attn_unified; k_shared_f32 / v_shared_f32: float32 [total_L,Hkv,d].
    Returns (out fp64 [n,d], lse fp64 [n]).
    """
    lib = _load()
    B, W, Hq, d = q.shape
    Hkv = k_shared_f32.shape[1]
    ND = k_unshared.shape[2]
    if triples is None:
        bb, ww, hh = np.meshgrid(np.arange(B), np.arange(W), np.arange(Hq), indexing="ij")
        triples = np.stack([bb.ravel(), ww.ravel(), hh.ravel()], axis=1)
    triples = np.ascontiguousarray(triples, dtype=np.int32)
    n = triples.shape[0]
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty(n, dtype=np.float64)
    rc = lib.oracle_attn_unified_f32kv(
        ctypes.c_int(B), ctypes.c_int(W), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(ND),
        ctypes.c_int(int(u)), ctypes.c_float(float(sm_scale)),
        _p(q, np.uint16), _p(k_shared_f32, np.float32), _p(v_shared_f32, np.float32), _p(cu_seqlens, np.int32),
        _p(k_unshared, np.uint16), _p(v_unshared, np.uint16), _p(triples, np.int32), ctypes.c_int64(n),
        _p(out, np.float64), _p(lse, np.float64))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_unified_f32kv failed: {rc}")
    return out, lse


def prefill_attn_causal(q, k, v, cu_seqlens, sm_scale, triples=None):
    """Causal self-attention over packed prompts.  bf16 tensors are uint16 bit patterns.

    q [total_L,Hq,d]; k, v [total_L,Hkv,d]; cu_seqlens int32 [B+1].
    triples: int32 [n,3] rows (b, i, hq) to evaluate (i = token index inside request b), default all.
    Returns (out fp64 [n,d], lse fp64 [n]).
    """
    lib = _load()
    total_L, Hq, d = q.shape
    Hkv = k.shape[1]
    cu_seqlens = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    B = len(cu_seqlens) - 1
    if triples is None:
        rows = [(b, i, h) for b in range(B) for i in range(int(cu_seqlens[b + 1] - cu_seqlens[b])) for h in range(Hq)]
        triples = np.array(rows, dtype=np.int32).reshape(-1, 3)
    triples = np.ascontiguousarray(triples, dtype=np.int32)
    n = triples.shape[0]
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty(n, dtype=np.float64)
    rc = lib.oracle_prefill_attn_causal(
        ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_float(float(sm_scale)),
        _p(q, np.uint16), _p(k, np.uint16), _p(v, np.uint16), _p(cu_seqlens, np.int32), _p(triples, np.int32),
        ctypes.c_int64(n), _p(out, np.float64), _p(lse, np.float64))
    if rc != 0:
        raise RuntimeError(f"oracle_prefill_attn_causal failed: {rc}")
    return out, lse


def check_table(items, V) -> int:
    items = np.ascontiguousarray(items, dtype=np.int32)
    return int(_load().oracle_check_table(_p(items, np.int32), ctypes.c_int64(items.shape[0]),
                                          ctypes.c_int(items.shape[1]), ctypes.c_int(V)))


def mask_row(items, V, prefix):
    """Dense additive mask row (0 / -inf) for the tokens that may follow `prefix`."""
    items = np.ascontiguousarray(items, dtype=np.int32)
    prefix = np.ascontiguousarray(prefix, dtype=np.int32)
    a = np.empty(V, dtype=np.float32)
    rc = _load().oracle_mask_row(_p(items, np.int32), ctypes.c_int64(items.shape[0]), ctypes.c_int(items.shape[1]),
                                 ctypes.c_int(V), _p(prefix, np.int32), ctypes.c_int(prefix.shape[0]), _p(a, np.float32))
    if rc != 0:
        raise RuntimeError(f"oracle_mask_row failed: {rc}")
    return a


def _select(fn_name, items, logits, scores_in, prefix_in, step, use_mask, want_visited):
    lib = _load()
    B, W, V = logits.shape
    depth = prefix_in.shape[2]
    if items is None:
        items_arr = np.zeros((0, depth), dtype=np.int32)
        use_mask = False
    else:
        items_arr = np.ascontiguousarray(items, dtype=np.int32)
    parent = np.empty((B, W), dtype=np.int32)
    token = np.empty((B, W), dtype=np.int32)
    scores = np.empty((B, W), dtype=np.float32)
    prefix = np.empty((B, W, depth), dtype=np.int32)
    rng = np.empty((B, W, 2), dtype=np.int32)
    item_index = np.empty((B, W), dtype=np.int32)
    args = [ctypes.c_int(B), ctypes.c_int(W), ctypes.c_int(V), ctypes.c_int(depth), ctypes.c_int(int(step)),
            _p(items_arr, np.int32), ctypes.c_int64(items_arr.shape[0]), ctypes.c_int(1 if use_mask else 0),
            _p(logits, np.float32), _p(scores_in, np.float32), _p(prefix_in, np.int32),
            _p(parent, np.int32), _p(token, np.int32), _p(scores, np.float32), _p(prefix, np.int32),
            _p(rng, np.int32), _p(item_index, np.int32)]
    visited = None
    if want_visited:
        visited = np.zeros(B, dtype=np.int64)
        args.append(_p(visited, np.int64))
    rc = getattr(lib, fn_name)(*args)
    if rc != 0:
        raise RuntimeError(f"{fn_name} failed: {rc}")
    res = dict(parent=parent, token=token, scores=scores, prefix=prefix, range=rng, item_index=item_index)
    if want_visited:
        res["visited"] = visited
    return res


def beam_select(items, logits, scores_in, prefix_in, step, use_mask=True):
    """Mask + log-softmax + score accumulation + full sort.  items=None means unconstrained."""
    return _select("oracle_beam_select", items, logits, scores_in, prefix_in, step, use_mask, False)


def beam_select_heap(items, logits, scores_in, prefix_in, step, use_mask=True):
    """Same result through per-beam sorted lists and a size-W min-heap with early termination."""
    return _select("oracle_beam_select_heap", items, logits, scores_in, prefix_in, step, use_mask, True)


def unshared_reorder(kv, parent):
    """kv uint16 [B,W,ND,Hkv,d] reordered in place along W by parent [B,W]."""
    B, W = parent.shape
    row = int(np.prod(kv.shape[2:]))
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    rc = _load().oracle_unshared_reorder(ctypes.c_int(B), ctypes.c_int(W), ctypes.c_int64(row),
                                         _p(parent, np.int32), _p(kv, np.uint16))
    if rc != 0:
        raise RuntimeError(f"oracle_unshared_reorder failed: {rc}")
    return kv


def unshared_reorder_two_sweeps(kv, parent):
    """The paper's own in-place procedure (direction index per row, upward writes walking down, then the rest
    walking up).  Needs live rows first with non-decreasing parents; raises ValueError otherwise.
    Returns (kv, direction int32 [B,W])."""
    B, W = parent.shape
    row = int(np.prod(kv.shape[2:]))
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    direction = np.zeros((B, W), dtype=np.int32)
    rc = _load().oracle_unshared_reorder_two_sweeps(ctypes.c_int(B), ctypes.c_int(W), ctypes.c_int64(row),
                                                    _p(parent, np.int32), _p(kv, np.uint16), _p(direction, np.int32))
    if rc == -1:
        raise ValueError("two-sweep reorder needs live rows first and non-decreasing parents")
    if rc != 0:
        raise RuntimeError(f"oracle_unshared_reorder_two_sweeps failed: {rc}")
    return kv, direction
