"""MI355X (gfx950) hot path of a generative-recommendation decode step: thin binding over libgr.so.

The calls have the names and meaning of the C ABI in include/gr.h:

    gr_beam_attn         shared-prefix beam attention over a separated KV cache
    gr_item_mask_build   valid-item mask blob from the sorted item table (load time)
    gr_beam_select       masked log-softmax + beam score accumulation + top-W selection
    gr_beam_reorder      in-place move of the surviving beams' own KV cache to their new slots

This module only marshals arguments (torch CUDA tensors -> device pointers, current stream ->
hipStream_t).  Every step of the path runs in the HIP kernels; there is no CPU or PyTorch fallback,
and loading fails loudly when the library has not been built.
"""
import ctypes
import os

from . import build as _build

__all__ = ["load_library", "gr_beam_attn", "gr_beam_attn_fp8kv", "gr_prefill_attn", "gr_item_mask_build", "gr_beam_select", "gr_beam_select_noalloc", "gr_beam_reorder",
           "gr_status_string",
           "attn_workspace_bytes", "select_workspace_bytes", "GrError", "GR_SELECT_FORCE_DENSE", "LIB_PATH",
           "gr_diag_stream_read", "gr_diag_mfma_loop", "gr_diag_attn_plan", "gr_diag_issue_loop", "gr_diag_issue_loop_lds", "gr_beam_attn_slots", "gr_beam_slot_update"]

LIB_PATH = _build.LIB_PATH
GR_SELECT_FORCE_DENSE = 1
_lib = None


class GrError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {gr_status_string(status)} ({int(status)})")


class _AttnParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("W", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("ND", ctypes.c_int32), ("u", ctypes.c_int32), ("max_L", ctypes.c_int32),
                ("total_L", ctypes.c_int64), ("sm_scale", ctypes.c_float),
                ("q", ctypes.c_void_p), ("k_shared", ctypes.c_void_p), ("v_shared", ctypes.c_void_p),
                ("cu_seqlens", ctypes.c_void_p), ("k_unshared", ctypes.c_void_p), ("v_unshared", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("lse_out", ctypes.c_void_p)]


class _AttnFp8Params(ctypes.Structure):
    _fields_ = [("attn", _AttnParams), ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float)]


class _PrefillParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
                ("max_L", ctypes.c_int32), ("total_L", ctypes.c_int64), ("sm_scale", ctypes.c_float),
                ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("cu_seqlens", ctypes.c_void_p),
                ("out", ctypes.c_void_p), ("lse_out", ctypes.c_void_p)]


class _SelectParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("W", ctypes.c_int32), ("V", ctypes.c_int32), ("depth", ctypes.c_int32),
                ("step", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("mask", ctypes.c_void_p), ("logits", ctypes.c_void_p), ("scores_in", ctypes.c_void_p),
                ("prefix_in", ctypes.c_void_p), ("range_in", ctypes.c_void_p), ("parent_out", ctypes.c_void_p),
                ("token_out", ctypes.c_void_p), ("scores_out", ctypes.c_void_p), ("prefix_out", ctypes.c_void_p),
                ("range_out", ctypes.c_void_p), ("item_index_out", ctypes.c_void_p)]


def load_library(path: str = None):
    """dlopen libgr.so and declare the C signatures.  Raises if the library is not built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(path)
    lib.gr_status_string.restype = ctypes.c_char_p
    lib.gr_status_string.argtypes = [ctypes.c_int32]
    lib.gr_beam_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.gr_beam_attn_workspace_bytes.argtypes = [ctypes.POINTER(_AttnParams)]
    lib.gr_beam_attn.restype = ctypes.c_int32
    lib.gr_beam_attn.argtypes = [ctypes.POINTER(_AttnParams), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.gr_item_mask_bytes.restype = ctypes.c_size_t
    lib.gr_item_mask_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
    lib.gr_item_mask_build_workspace_bytes.restype = ctypes.c_size_t
    lib.gr_item_mask_build_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
    lib.gr_item_mask_build.restype = ctypes.c_int32
    lib.gr_item_mask_build.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                       ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.gr_beam_select_workspace_bytes.restype = ctypes.c_size_t
    lib.gr_beam_select_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
    lib.gr_beam_select.restype = ctypes.c_int32
    lib.gr_beam_select.argtypes = [ctypes.POINTER(_SelectParams), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.gr_beam_select_noalloc.restype = ctypes.c_int32
    lib.gr_beam_select_noalloc.argtypes = [ctypes.POINTER(_SelectParams), ctypes.c_void_p]
    lib.gr_beam_select_noalloc_max_workspace_bytes.restype = ctypes.c_size_t
    lib.gr_beam_select_noalloc_max_workspace_bytes.argtypes = []
    lib.gr_diag_stream_read.restype = ctypes.c_int32
    lib.gr_diag_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    lib.gr_diag_mfma_loop.restype = ctypes.c_int32
    lib.gr_diag_mfma_loop.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    lib.gr_beam_attn_fp8kv.restype = ctypes.c_int32
    lib.gr_beam_attn_fp8kv.argtypes = [ctypes.POINTER(_AttnFp8Params), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.gr_prefill_attn.restype = ctypes.c_int32
    lib.gr_prefill_attn.argtypes = [ctypes.POINTER(_PrefillParams), ctypes.c_void_p]
    lib.gr_diag_issue_loop.restype = ctypes.c_int32
    lib.gr_diag_issue_loop.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p] * 2
    lib.gr_beam_attn_slots.restype = ctypes.c_int32
    lib.gr_beam_attn_slots.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.gr_beam_slot_update.restype = ctypes.c_int32
    lib.gr_beam_slot_update.argtypes = [ctypes.c_int32] * 4 + [ctypes.c_void_p] * 4
    lib.gr_diag_issue_loop_lds.restype = ctypes.c_int32
    lib.gr_diag_issue_loop_lds.argtypes = [ctypes.c_void_p] + [ctypes.c_int32] * 5 + [ctypes.c_void_p] * 2
    lib.gr_diag_attn_plan.restype = ctypes.c_int32
    lib.gr_diag_attn_plan.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.gr_diag_mfma_flops.restype = ctypes.c_double
    lib.gr_diag_mfma_flops.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.gr_beam_reorder.restype = ctypes.c_int32
    lib.gr_beam_reorder.argtypes = [ctypes.c_int32] * 6 + [ctypes.c_void_p] * 4
    _lib = lib
    return lib


def gr_status_string(status) -> str:
    return load_library().gr_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _check(t, dtype, shape, name):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous CUDA tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")


def _attn_params(q, k_shared, v_shared, cu_seqlens, k_unshared, v_unshared, u, sm_scale, max_L, total_L, out, lse_out):
    B, W, Hq, d = q.shape
    Hkv = k_shared.shape[1]
    ND = k_unshared.shape[2]
    p = _AttnParams()
    p.B, p.W, p.Hq, p.Hkv, p.d, p.ND, p.u = B, W, Hq, Hkv, d, ND, int(u)
    p.max_L, p.total_L, p.sm_scale = int(max_L), int(total_L), float(sm_scale)
    p.q, p.k_shared, p.v_shared = q.data_ptr(), k_shared.data_ptr(), v_shared.data_ptr()
    p.cu_seqlens, p.k_unshared, p.v_unshared = cu_seqlens.data_ptr(), k_unshared.data_ptr(), v_unshared.data_ptr()
    p.out = out.data_ptr() if out is not None else None
    p.lse_out = lse_out.data_ptr() if lse_out is not None else None
    return p


def attn_workspace_bytes(B, W, Hq, Hkv, d, max_L, total_L=None) -> int:
    """Workspace bytes of gr_beam_attn.  Without total_L the batch is taken as ragged (the larger answer)."""
    p = _AttnParams()
    p.B, p.W, p.Hq, p.Hkv, p.d, p.max_L = B, W, Hq, Hkv, d, int(max_L)
    p.total_L = int(total_L) if total_L is not None else max(0, B * int(max_L) - 1)
    return int(load_library().gr_beam_attn_workspace_bytes(ctypes.byref(p)))


def gr_beam_attn(q, k_shared, v_shared, cu_seqlens, k_unshared, v_unshared, u, sm_scale, max_L, total_L,
                 out=None, lse_out=None, workspace=None, stream=None, slot=None):
    """Shared-prefix beam attention.  bf16 CUDA tensors: q [B,W,Hq,d], k/v_shared [total_L,Hkv,d],
    k/v_unshared [B,W,ND,Hkv,d]; cu_seqlens int32 [B+1].  max_L / total_L are host integers.
    `slot` (int32 [B,W,ND], optional) routes the call to gr_beam_attn_slots: the own-token rows are read through it.
    Returns (out bf16 [B,W,Hq,d], lse fp32 [B,W,Hq] or None).  Enqueues on `stream` (default: current)."""
    import torch
    lib = load_library()
    B, W, Hq, d = q.shape
    _check(q, torch.bfloat16, None, "q")
    _check(k_shared, torch.bfloat16, (k_shared.shape[0], k_shared.shape[1], d), "k_shared")
    _check(v_shared, torch.bfloat16, tuple(k_shared.shape), "v_shared")
    _check(cu_seqlens, torch.int32, (B + 1,), "cu_seqlens")
    _check(k_unshared, torch.bfloat16, (B, W, k_unshared.shape[2], k_shared.shape[1], d), "k_unshared")
    _check(v_unshared, torch.bfloat16, tuple(k_unshared.shape), "v_unshared")
    if k_shared.shape[0] < int(total_L):
        raise ValueError("k_shared has fewer rows than total_L")
    if out is None:
        out = torch.empty_like(q)
    _check(out, torch.bfloat16, tuple(q.shape), "out")
    if lse_out is not None:
        _check(lse_out, torch.float32, (B, W, Hq), "lse_out")
    p = _attn_params(q, k_shared, v_shared, cu_seqlens, k_unshared, v_unshared, u, sm_scale, max_L, total_L, out, lse_out)
    need = int(lib.gr_beam_attn_workspace_bytes(ctypes.byref(p)))
    if workspace is None and need > 0:
        workspace = _scratch(need, q.device, stream)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if slot is not None:
        _check(slot, torch.int32, (B, W, k_unshared.shape[2]), "slot")
        rc = lib.gr_beam_attn_slots(ctypes.byref(p), _ptr(slot), _ptr(workspace), ws_bytes, _stream(stream))
    else:
        rc = lib.gr_beam_attn(ctypes.byref(p), _ptr(workspace), ws_bytes, _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_beam_attn_slots" if slot is not None else "gr_beam_attn")
    return out, lse_out


def gr_beam_attn_slots(q, k_shared, v_shared, cu_seqlens, k_unshared, v_unshared, slot, u, sm_scale, max_L, total_L,
                       out=None, lse_out=None, workspace=None, stream=None):
    """gr_beam_attn with the own-token caches read through the slot table `slot` (int32 [B,W,ND]; see gr_beam_slot_update)."""
    if slot is None:
        raise ValueError("slot is required")
    return gr_beam_attn(q, k_shared, v_shared, cu_seqlens, k_unshared, v_unshared, u, sm_scale, max_L, total_L,
                        out=out, lse_out=lse_out, workspace=workspace, stream=stream, slot=slot)


def gr_beam_attn_fp8kv(q, k_shared_fp8, v_shared_fp8, k_scale, v_scale, cu_seqlens, k_unshared, v_unshared, u, sm_scale, max_L, total_L,
                       out=None, lse_out=None, workspace=None, stream=None):
    """gr_beam_attn over a prompt cache stored as FP8 E4M3 codes: k/v_shared_fp8 uint8 CUDA tensors [total_L,Hkv,d],
    value = code * scale.  Everything else as for gr_beam_attn."""
    import torch
    lib = load_library()
    B, W, Hq, d = q.shape
    _check(q, torch.bfloat16, None, "q")
    _check(k_shared_fp8, torch.uint8, (k_shared_fp8.shape[0], k_shared_fp8.shape[1], d), "k_shared_fp8")
    _check(v_shared_fp8, torch.uint8, tuple(k_shared_fp8.shape), "v_shared_fp8")
    _check(cu_seqlens, torch.int32, (B + 1,), "cu_seqlens")
    _check(k_unshared, torch.bfloat16, (B, W, k_unshared.shape[2], k_shared_fp8.shape[1], d), "k_unshared")
    _check(v_unshared, torch.bfloat16, tuple(k_unshared.shape), "v_unshared")
    if k_shared_fp8.shape[0] < int(total_L):
        raise ValueError("k_shared_fp8 has fewer rows than total_L")
    if out is None:
        out = torch.empty_like(q)
    _check(out, torch.bfloat16, tuple(q.shape), "out")
    if lse_out is not None:
        _check(lse_out, torch.float32, (B, W, Hq), "lse_out")
    p = _AttnFp8Params(_attn_params(q, k_shared_fp8, v_shared_fp8, cu_seqlens, k_unshared, v_unshared, u, sm_scale, max_L, total_L, out, lse_out),
                       float(k_scale), float(v_scale))
    need = int(lib.gr_beam_attn_workspace_bytes(ctypes.byref(p.attn)))
    if workspace is None and need > 0:
        workspace = _scratch(need, q.device, stream)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib.gr_beam_attn_fp8kv(ctypes.byref(p), _ptr(workspace), ws_bytes, _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_beam_attn_fp8kv")
    return out, lse_out


def gr_prefill_attn(q, k, v, cu_seqlens, sm_scale, max_L, total_L, out=None, lse_out=None, stream=None):
    """Causal self-attention over packed prompts.  bf16 CUDA tensors: q [total_L,Hq,d], k/v [total_L,Hkv,d];
    cu_seqlens int32 [B+1].  max_L / total_L are host integers.  Returns (out bf16 [total_L,Hq,d], lse or None)."""
    import torch
    lib = load_library()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    B = cu_seqlens.shape[0] - 1
    _check(q, torch.bfloat16, None, "q")
    _check(k, torch.bfloat16, (T, Hkv, d), "k")
    _check(v, torch.bfloat16, (T, Hkv, d), "v")
    _check(cu_seqlens, torch.int32, (B + 1,), "cu_seqlens")
    if T < int(total_L):
        raise ValueError("q has fewer rows than total_L")
    if out is None:
        out = torch.empty_like(q)
    _check(out, torch.bfloat16, tuple(q.shape), "out")
    if lse_out is not None:
        _check(lse_out, torch.float32, (T, Hq), "lse_out")
    p = _PrefillParams(B, Hq, Hkv, d, int(max_L), int(total_L), float(sm_scale), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                       cu_seqlens.data_ptr(), out.data_ptr(), lse_out.data_ptr() if lse_out is not None else None)
    rc = lib.gr_prefill_attn(ctypes.byref(p), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_prefill_attn")
    return out, lse_out


def gr_item_mask_build(items_sorted, V, stream=None):
    """Build the mask blob from a sorted, distinct int32 CUDA table [N, 3].  Returns a uint8 CUDA tensor."""
    import torch
    lib = load_library()
    _check(items_sorted, torch.int32, None, "items_sorted")
    N, depth = items_sorted.shape
    nbytes = int(lib.gr_item_mask_bytes(N, depth, int(V)))
    if nbytes == 0:
        raise GrError(-2, "gr_item_mask_bytes")
    blob = torch.empty(nbytes, dtype=torch.uint8, device=items_sorted.device)
    ws = torch.empty(int(lib.gr_item_mask_build_workspace_bytes(N, depth, int(V))), dtype=torch.uint8, device=items_sorted.device)
    rc = lib.gr_item_mask_build(_ptr(items_sorted), N, depth, int(V), _ptr(blob), nbytes, _ptr(ws), ws.numel(), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_item_mask_build")
    return blob


def select_workspace_bytes(B, W, V, depth) -> int:
    return int(load_library().gr_beam_select_workspace_bytes(B, W, V, depth))


def _scratch(nbytes, device, stream):
    """A workspace the wrapper allocates itself belongs to the stream the kernels run on: allocated under another
    stream, the caching allocator could hand the block out again while they still use it."""
    import torch
    if stream is None:
        return torch.empty(nbytes, dtype=torch.uint8, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _select_call(mask, logits, scores_in, prefix_in, range_in, step, flags, out, allocate_outputs):
    import torch
    B, W, V = logits.shape
    depth = prefix_in.shape[2]
    _check(logits, torch.float32, None, "logits")
    _check(scores_in, torch.float32, (B, W), "scores_in")
    _check(prefix_in, torch.int32, (B, W, depth), "prefix_in")
    _check(range_in, torch.int32, (B, W, 2), "range_in")
    dev = logits.device
    if out is None:
        out = {}
    spec = dict(parent=((B, W), torch.int32), token=((B, W), torch.int32), scores=((B, W), torch.float32),
                prefix=((B, W, depth), torch.int32), range=((B, W, 2), torch.int32), item_index=((B, W), torch.int32))
    for k, (shape, dt) in spec.items():
        if k not in out or out[k] is None:
            if not allocate_outputs:
                raise ValueError(f"out[{k!r}] must be preallocated for a call that allocates nothing")
            out[k] = torch.empty(shape, dtype=dt, device=dev)
        _check(out[k], dt, shape, k)
    p = _SelectParams()
    p.B, p.W, p.V, p.depth, p.step, p.flags = B, W, V, depth, int(step), int(flags)
    p.mask = mask.data_ptr() if mask is not None else None
    p.logits, p.scores_in = logits.data_ptr(), scores_in.data_ptr()
    p.prefix_in, p.range_in = prefix_in.data_ptr(), range_in.data_ptr()
    p.parent_out, p.token_out, p.scores_out = out["parent"].data_ptr(), out["token"].data_ptr(), out["scores"].data_ptr()
    p.prefix_out, p.range_out, p.item_index_out = out["prefix"].data_ptr(), out["range"].data_ptr(), out["item_index"].data_ptr()
    return p, out


def gr_beam_select(mask, logits, scores_in, prefix_in, range_in, step, flags=0, out=None, workspace=None, stream=None):
    """Beam item step.  logits fp32 [B,W,V]; scores_in fp32 [B,W]; prefix_in int32 [B,W,depth]; range_in int32
    [B,W,2]; mask = blob from gr_item_mask_build or None.  `out` may hold preallocated tensors under the keys
    parent, token, scores, prefix, range, item_index.  Returns that dict.  Enqueues on `stream`."""
    lib = load_library()
    p, out = _select_call(mask, logits, scores_in, prefix_in, range_in, step, flags, out, True)
    if workspace is None:
        workspace = _scratch(int(lib.gr_beam_select_workspace_bytes(p.B, p.W, p.V, p.depth)), logits.device, stream)
    rc = lib.gr_beam_select(ctypes.byref(p), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_beam_select")
    return out


def gr_beam_select_noalloc(mask, logits, scores_in, prefix_in, range_in, step, out, flags=0, stream=None):
    """The same item step through the entry point that allocates nothing: the workspace is a static device array inside
    the library and every output tensor must be passed in `out`.  Calls that overlap on one GPU race."""
    lib = load_library()
    p, out = _select_call(mask, logits, scores_in, prefix_in, range_in, step, flags, out, False)
    rc = lib.gr_beam_select_noalloc(ctypes.byref(p), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_beam_select_noalloc")
    return out


def gr_beam_reorder(parent, k_unshared, v_unshared, u, stream=None):
    """Move every surviving beam's own KV cache to its new slot, in place.  parent int32 [B,W] (from
    gr_beam_select); k/v_unshared bf16 [B,W,ND,Hkv,d]; token slots [0,u) move.  Enqueues on `stream`."""
    import torch
    lib = load_library()
    B, W, ND, Hkv, d = k_unshared.shape
    _check(parent, torch.int32, (B, W), "parent")
    _check(k_unshared, torch.bfloat16, None, "k_unshared")
    _check(v_unshared, torch.bfloat16, tuple(k_unshared.shape), "v_unshared")
    rc = lib.gr_beam_reorder(B, W, ND, Hkv, d, int(u), _ptr(parent), _ptr(k_unshared), _ptr(v_unshared), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_beam_reorder")


def gr_beam_slot_update(parent, slot_in, u, ND, out=None, stream=None):
    """The slot table after a beam step (nothing in the caches moves): out[b,j,t] = slot_in[b,parent[b,j],t] for t < u,
    j*ND + t otherwise.  parent int32 [B,W]; slot_in int32 [B,W,ND] or None (identity).  Returns out int32 [B,W,ND]."""
    import torch
    lib = load_library()
    B, W = parent.shape
    _check(parent, torch.int32, (B, W), "parent")
    if slot_in is not None:
        _check(slot_in, torch.int32, (B, W, int(ND)), "slot_in")
    if out is None:
        out = _scratch(B * W * int(ND) * 4, parent.device, stream).view(torch.int32).view(B, W, int(ND))
    _check(out, torch.int32, (B, W, int(ND)), "out")
    rc = lib.gr_beam_slot_update(B, W, int(ND), int(u), _ptr(parent), _ptr(slot_in), _ptr(out), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_beam_slot_update")
    return out


def gr_diag_attn_plan(rows_per_workgroup=0, l_segments=0):
    """Force the attention launch plan (rows per workgroup 128/256, prompt segments 1..16) for later calls; (0, 0) = built-in rule."""
    rc = load_library().gr_diag_attn_plan(int(rows_per_workgroup), int(l_segments))
    if rc != 0:
        raise GrError(rc, "gr_diag_attn_plan")


def gr_diag_issue_loop(operands, workgroups, iters, n_fma, n_exp, with_mfma, sink, stream=None):
    """Enqueue the MFMA / VALU issue test (see gr.h).  `operands`: 16 KiB CUDA tensor."""
    if operands.numel() * operands.element_size() < 16384:
        raise ValueError("operands must hold 16 KiB")
    rc = load_library().gr_diag_issue_loop(_ptr(operands), int(workgroups), int(iters), int(n_fma), int(n_exp), int(bool(with_mfma)),
                                           _ptr(sink), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_diag_issue_loop")


def gr_diag_issue_loop_lds(operands, workgroups, rounds, n_fma, n_exp, lds_every, sink, stream=None):
    """Enqueue the issue test with the MFMA's first operand read from LDS every `lds_every`-th slot (see gr.h)."""
    if operands.numel() * operands.element_size() < 16384:
        raise ValueError("operands must hold 16 KiB")
    rc = load_library().gr_diag_issue_loop_lds(_ptr(operands), int(workgroups), int(rounds), int(n_fma), int(n_exp), int(lds_every),
                                               _ptr(sink), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_diag_issue_loop_lds")


def gr_diag_stream_read(src, sink, stream=None):
    """Enqueue a plain streaming read of the CUDA tensor `src` (measured HBM read rate).  `sink`: any 4-byte CUDA tensor."""
    rc = load_library().gr_diag_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_diag_stream_read")


def gr_diag_mfma_loop(operands, workgroups, iters, sink, stream=None):
    """Enqueue a loop of back-to-back bf16 MFMAs on `operands` (16 KiB CUDA tensor).  Returns the launch's FLOP count."""
    lib = load_library()
    if operands.numel() * operands.element_size() < 16384:
        raise ValueError("operands must hold 16 KiB")
    rc = lib.gr_diag_mfma_loop(_ptr(operands), int(workgroups), int(iters), _ptr(sink), _stream(stream))
    if rc != 0:
        raise GrError(rc, "gr_diag_mfma_loop")
    return float(lib.gr_diag_mfma_flops(int(workgroups), int(iters)))

