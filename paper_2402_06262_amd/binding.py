"""ctypes binding of libroco.so: same names as include/roco.h, argument marshalling only.

PyTorch supplies device memory (`tensor.data_ptr()`) and the HIP stream
(`torch.cuda.current_stream().cuda_stream`); no arithmetic of the method happens here.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

ROCO_F32 = 0
ROCO_BF16 = 1
ROCO_IMPORTANCE_MAS, ROCO_IMPORTANCE_AAS, ROCO_IMPORTANCE_OLDEST, ROCO_IMPORTANCE_LAST = 0, 1, 2, 3
ROCO_IMPORTANCE_COUNT = 4
ROCO_SCOPE_STD, ROCO_SCOPE_WINDOW, ROCO_SCOPE_ALL = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libroco.so"
_lib: Optional[ctypes.CDLL] = None


class RocoError(RuntimeError):
    """A roco_* call returned a negative code."""

    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {roco_strerror(code)} (code {code})")


class RocoParams(ctypes.Structure):
    """Mirror of `roco_params` (include/roco.h)."""

    _fields_ = [
        ("units", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("budget", ctypes.c_int32),
        ("scope", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("recency_window", ctypes.c_int32),
        ("recency_bias", ctypes.c_float),
        ("importance", ctypes.c_int32),
        ("scope_kind", ctypes.c_int32),
        ("sinks", ctypes.c_int32),
    ]

    def __init__(self, units, head_dim, budget, scope, dtype, scale=0.0, recency_window=0, recency_bias=0.0,
                 importance=0, scope_kind=0, sinks=0):
        super().__init__(int(units), int(head_dim), int(budget), int(scope), int(dtype), float(scale),
                         int(recency_window), float(recency_bias), int(importance), int(scope_kind), int(sinks))


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library() -> ctypes.CDLL:
    """Load the built HIP library; raises if it is missing (there is no other implementation)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built; run `python -m paper_2402_06262_amd.build` "
                           "(hipcc, gfx950) first -- the RoCo path has no CPU fallback")
    lib = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    pp = ctypes.POINTER(RocoParams)
    lib.roco_prefill_workspace_bytes.restype = sz
    lib.roco_prefill_workspace_bytes.argtypes = [pp, i32]
    lib.roco_prefill_gqa_workspace_bytes.restype = sz
    lib.roco_prefill_gqa_workspace_bytes.argtypes = [pp, i32, i32]
    lib.roco_prefill_compress_gqa.restype = ctypes.c_int
    lib.roco_prefill_compress_gqa.argtypes = [pp, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_prefill_compress_lse.restype = ctypes.c_int
    lib.roco_prefill_compress_lse.argtypes = [pp, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_decode_workspace_bytes.restype = sz
    lib.roco_decode_workspace_bytes.argtypes = [pp]
    lib.roco_decode_step_launches.restype = ctypes.c_int
    lib.roco_decode_step_launches.argtypes = [pp]
    lib.roco_prefill_compress.restype = ctypes.c_int
    lib.roco_prefill_compress.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_decode_step.restype = ctypes.c_int
    lib.roco_decode_step.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_decode_step_static.restype = ctypes.c_int
    lib.roco_decode_step_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.roco_probe_cache_read.restype = ctypes.c_int
    lib.roco_probe_cache_read.argtypes = [pp, vp, vp, vp, sz, vp]
    lib.roco_probe_mfma.restype = ctypes.c_int
    lib.roco_probe_mfma.argtypes = [i32, i32, i32, vp, sz, vp]
    lib.roco_block_workspace_bytes.restype = sz
    lib.roco_block_workspace_bytes.argtypes = [pp, i32]
    lib.roco_encode_block.restype = ctypes.c_int
    lib.roco_encode_block.argtypes = [pp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_encode_block_gqa.restype = ctypes.c_int
    lib.roco_encode_block_gqa.argtypes = [pp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_decode_step_gqa.restype = ctypes.c_int
    lib.roco_decode_step_gqa.argtypes = [pp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_select_victims.restype = ctypes.c_int
    lib.roco_select_victims.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_select_retained.restype = ctypes.c_int
    lib.roco_select_retained.argtypes = [pp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.roco_set_overlap.restype = ctypes.c_int
    lib.roco_set_overlap.argtypes = [i32, i32, vp, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp]
    lib.roco_strerror.restype = ctypes.c_char_p
    lib.roco_strerror.argtypes = [ctypes.c_int]
    lib.roco_version.restype = ctypes.c_int
    lib.roco_version.argtypes = []
    lib.roco_profile_kernel.restype = ctypes.c_int
    lib.roco_profile_kernel.argtypes = [ctypes.c_int]
    lib.roco_profile_sampling.restype = ctypes.c_int
    lib.roco_profile_sampling.argtypes = [ctypes.c_int]
    lib.roco_profile_read.restype = ctypes.c_int
    lib.roco_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    _lib = lib
    return lib


def roco_strerror(code: int) -> str:
    return load_library().roco_strerror(int(code)).decode()


def roco_version() -> int:
    return int(load_library().roco_version())


def prefill_workspace_bytes(params: RocoParams, L_max: int) -> int:
    return int(load_library().roco_prefill_workspace_bytes(ctypes.byref(params), int(L_max)))


def decode_workspace_bytes(params: RocoParams) -> int:
    return int(load_library().roco_decode_workspace_bytes(ctypes.byref(params)))


PROF_KERNELS = {"decode_select": 0, "decode_attend": 1, "decode_finish": 2, "prefill_rows": 3,
                "prefill_columns": 4, "prefill_select": 5, "prefill_gather": 6, "read_probe": 7,
                "block_prepare": 8, "block_attend": 9, "block_finish": 10, "mfma_probe": 11}


def roco_profile_kernel(which: int) -> None:
    rc = load_library().roco_profile_kernel(int(which))
    if rc != 0:
        raise RocoError(rc, "roco_profile_kernel")


def roco_profile_sampling(every: int) -> None:
    rc = load_library().roco_profile_sampling(int(every))
    if rc != 0:
        raise RocoError(rc, "roco_profile_sampling")


def roco_profile_read():
    """(total milliseconds, launches) of the profiled kernel since the last read."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    rc = load_library().roco_profile_read(ctypes.byref(ms), ctypes.byref(n))
    if rc != 0:
        raise RocoError(rc, "roco_profile_read")
    return ms.value, n.value


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None stays NULL); host ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("roco: tensors must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def roco_prefill_compress(params: RocoParams, Q, K, V, length, L_max: int, K_cache, V_cache, stats, pos,
                          n_used, next_slot, O, workspace, workspace_bytes: Optional[int] = None, stream=None) -> None:
    """See include/roco.h.  Tensors are device tensors; `O` may be None."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_prefill_compress(
        ctypes.byref(params), _ptr(Q), _ptr(K), _ptr(V), _ptr(length), int(L_max), _ptr(K_cache),
        _ptr(V_cache), _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(O), _ptr(workspace),
        int(workspace_bytes),
        _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_prefill_compress")


def roco_decode_step(params: RocoParams, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used, next_slot,
                     out, evicted_slot, evicted_pos, workspace, workspace_bytes: Optional[int] = None,
                     stream=None) -> None:
    """See include/roco.h.  `evicted_slot` / `evicted_pos` may be None."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_decode_step(
        ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(qpos), _ptr(K_cache), _ptr(V_cache),
        _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(out), _ptr(evicted_slot), _ptr(evicted_pos),
        _ptr(workspace), int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_decode_step")


def roco_decode_step_static(params: RocoParams, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used,
                            next_slot, out, evicted_slot, evicted_pos, stream=None) -> None:
    """See include/roco.h: the decode step on the library's own static scratch (no workspace, no allocation)."""
    rc = load_library().roco_decode_step_static(
        ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(qpos), _ptr(K_cache), _ptr(V_cache),
        _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(out), _ptr(evicted_slot), _ptr(evicted_pos),
        _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_decode_step_static")


def prefill_gqa_workspace_bytes(params: RocoParams, group: int, L_max: int) -> int:
    return int(load_library().roco_prefill_gqa_workspace_bytes(ctypes.byref(params), int(group), int(L_max)))


def roco_prefill_compress_gqa(params: RocoParams, group: int, Q, K, V, lens, L_max: int, K_cache, V_cache, stats, pos,
                              n_used, next_slot, O, workspace, workspace_bytes: Optional[int] = None,
                              stream=None) -> None:
    """See include/roco.h: prefill with one-step eviction for key/value heads shared by `group` query heads."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_prefill_compress_gqa(
        ctypes.byref(params), int(group), _ptr(Q), _ptr(K), _ptr(V), _ptr(lens), int(L_max), _ptr(K_cache),
        _ptr(V_cache), _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(O), _ptr(workspace),
        int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_prefill_compress_gqa")


def roco_prefill_compress_lse(params: RocoParams, group: int, Q, K, V, lens, L_max: int, lse, K_cache, V_cache, stats,
                              pos, n_used, next_slot, workspace, workspace_bytes: Optional[int] = None,
                              stream=None) -> None:
    """See include/roco.h: prefill-compress from row normalisers the caller's attention kernel already produced."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_prefill_compress_lse(
        ctypes.byref(params), int(group), _ptr(Q), _ptr(K), _ptr(V), _ptr(lens), int(L_max), _ptr(lse), _ptr(K_cache),
        _ptr(V_cache), _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(workspace), int(workspace_bytes),
        _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_prefill_compress_lse")


def decode_step_launches(params: RocoParams) -> int:
    """1 if a decode step of these params is one fused kernel, 2 if it is the split pair (see include/roco.h)."""
    rc = int(load_library().roco_decode_step_launches(ctypes.byref(params)))
    if rc < 0:
        raise RocoError(rc, "roco_decode_step_launches")
    return rc


def block_workspace_bytes(params: RocoParams, block: int) -> int:
    return int(load_library().roco_block_workspace_bytes(ctypes.byref(params), int(block)))


def roco_encode_block(params: RocoParams, block: int, q, k_new, v_new, qpos0, K_cache, V_cache, stats, pos, n_used,
                      next_slot, out, evicted_slot, evicted_pos, workspace, workspace_bytes: Optional[int] = None,
                      stream=None) -> None:
    """See include/roco.h: free and encode `block` tokens within one eviction step."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_encode_block(
        ctypes.byref(params), int(block), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(qpos0), _ptr(K_cache),
        _ptr(V_cache), _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(out), _ptr(evicted_slot),
        _ptr(evicted_pos), _ptr(workspace), int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_encode_block")


def roco_encode_block_gqa(params: RocoParams, block: int, group: int, q, k_new, v_new, qpos0, K_cache, V_cache, stats,
                          pos, n_used, next_slot, out, evicted_slot, evicted_pos, workspace,
                          workspace_bytes: Optional[int] = None, stream=None) -> None:
    """See include/roco.h: block-wise step of key/value heads shared by `group` query heads each."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_encode_block_gqa(
        ctypes.byref(params), int(block), int(group), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(qpos0), _ptr(K_cache),
        _ptr(V_cache), _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(out), _ptr(evicted_slot),
        _ptr(evicted_pos), _ptr(workspace), int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_encode_block_gqa")


def roco_decode_step_gqa(params: RocoParams, group: int, q, k_new, v_new, qpos, K_cache, V_cache, stats, pos, n_used,
                         next_slot, out, evicted_slot, evicted_pos, workspace, workspace_bytes: Optional[int] = None,
                         stream=None) -> None:
    """See include/roco.h: one decode step of key/value heads shared by `group` query heads each."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_decode_step_gqa(
        ctypes.byref(params), int(group), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(qpos), _ptr(K_cache),
        _ptr(V_cache), _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot), _ptr(out), _ptr(evicted_slot),
        _ptr(evicted_pos), _ptr(workspace), int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_decode_step_gqa")


def roco_probe_cache_read(params: RocoParams, K_cache, V_cache, workspace, workspace_bytes: Optional[int] = None,
                          stream=None) -> None:
    """See include/roco.h: the loads of the decode attention kernel, and nothing else (benchmark aid)."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_probe_cache_read(ctypes.byref(params), _ptr(K_cache), _ptr(V_cache), _ptr(workspace),
                                              int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_probe_cache_read")


def roco_probe_mfma(workgroups: int, iters: int, sink, stream=None, random_operands: bool = False, mix: int = 0) -> int:
    """See include/roco.h: a loop of the prefill passes' matrix instruction, or (mix = 1 row pass, 2 column pass) the
    steady state of a pass's instruction mix (benchmark aid).  Returns the flops of the call."""
    mode = (1 + int(mix)) if mix else (1 if random_operands else 0)
    rc = load_library().roco_probe_mfma(int(workgroups), int(iters), mode, _ptr(sink),
                                        sink.numel() * sink.element_size(), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_probe_mfma")
    return int(workgroups) * 4 * int(iters) * (32 if mix else 8) * 32768


def roco_set_overlap(pos_a, mask_a, n_used_a, pos_b, mask_b, n_used_b, max_pos: int, inter, uni, stream=None) -> None:
    """See include/roco.h: |A and B| and |A or B| per unit of two sets of cached positions (masks may be None)."""
    rc = load_library().roco_set_overlap(int(pos_a.shape[0]), int(pos_a.shape[1]), _ptr(pos_a), _ptr(mask_a), _ptr(n_used_a),
                                         int(pos_b.shape[1]), _ptr(pos_b), _ptr(mask_b), _ptr(n_used_b), int(max_pos),
                                         _ptr(inter), _ptr(uni), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_set_overlap")


def roco_select_victims(params: RocoParams, stats, pos, n_used, next_slot, workspace,
                        workspace_bytes: Optional[int] = None, stream=None) -> None:
    """See include/roco.h: recompute next_slot from stats / pos / n_used."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_select_victims(ctypes.byref(params), _ptr(stats), _ptr(pos), _ptr(n_used), _ptr(next_slot),
                                            _ptr(workspace), int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_select_victims")


def roco_select_retained(params: RocoParams, keep: int, stats, pos, n_used, mask, workspace,
                         workspace_bytes: Optional[int] = None, stream=None) -> None:
    """See include/roco.h: mask of the tokens that survive a shrink of every unit to `keep` tokens."""
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    rc = load_library().roco_select_retained(ctypes.byref(params), int(keep), _ptr(stats), _ptr(pos), _ptr(n_used),
                                             _ptr(mask), _ptr(workspace), int(workspace_bytes), _stream(stream))
    if rc != 0:
        raise RocoError(rc, "roco_select_retained")


@dataclass
class RocoCache:
    """Caller-owned device buffers of the budgeted cache (plain torch tensors, nothing else)."""

    K: "object"  # [units, B, d]
    V: "object"
    stats: "object"  # [units, 3, B] fp32: Acc, Acc2, Count
    pos: "object"  # [units, B] int32
    n_used: "object"  # [units] int32
    next_slot: "object"  # [units] int32: victim already chosen for the next step (library-maintained)


def alloc_cache(params: RocoParams, device="cuda") -> RocoCache:
    import torch
    dt = torch.bfloat16 if params.dtype == ROCO_BF16 else torch.float32
    U, B, d = params.units, params.budget, params.head_dim
    return RocoCache(
        torch.zeros((U, B, d), dtype=dt, device=device),
        torch.zeros((U, B, d), dtype=dt, device=device),
        torch.zeros((U, 3, B), dtype=torch.float32, device=device),
        torch.full((U, B), -1, dtype=torch.int32, device=device),
        torch.zeros((U,), dtype=torch.int32, device=device),
        torch.full((U,), -1, dtype=torch.int32, device=device),
    )
