"""ctypes binding of libmoe_hip.so: same names and argument order as include/moe.h.

Argument marshalling only.  Tensors must live on the GPU, be contiguous and have the dtype the
C interface states; outputs are allocated with torch when not passed in.  Work is enqueued on
torch's current stream.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

SYMBOLS = ["moe_status_string", "moe_build_id", "moe_route", "moe_route_segments", "moe_permute", "moe_permute_static", "moe_expert_group_forward",
           "moe_expert_group_forward_ex", "moe_expert_group_forward_gather", "moe_expert_list_forward",
           "moe_shared_forward", "moe_shared_forward_ex", "moe_combine", "moe_combine_parts",
           "moe_fused_shared_sets", "moe_fused_workspace_bytes", "moe_expert_group_forward_fused",
           "moe_permute_workspace_bytes", "moe_expert_workspace_bytes", "moe_shared_workspace_bytes",
           "moe_workspace_bytes", "moe_residual_norm", "moe_probe_mfma", "moe_tile_clock_buffer"]


class MoeError(RuntimeError):
    pass


def lib_path() -> str:
    return os.path.join(_HERE, "libmoe_hip.so")


def load() -> ctypes.CDLL:
    """Load the built library (building it first only if it does not exist).  A library that was built
    from other sources than the ones beside it is refused: its results and timings would be
    attributed to kernels that are not the ones running."""
    global _LIB
    if _LIB is not None:
        return _LIB
    from . import build as _build
    if not os.path.exists(lib_path()):
        _build.build()
    lib = ctypes.CDLL(lib_path())
    c_int, c_vp, c_sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.moe_build_id.restype = ctypes.c_char_p
    lib.moe_build_id.argtypes = []
    built, here = lib.moe_build_id().decode(), _build.source_id()
    if built != here:
        raise MoeError(f"{lib_path()} was built from other sources (library {built[:12]}, sources {here[:12]}): "
                       "rebuild it with `python -m paper_2604_26881_amd.build`")
    lib.moe_status_string.restype = ctypes.c_char_p
    lib.moe_status_string.argtypes = [c_int]
    lib.moe_route.restype = c_int
    lib.moe_route.argtypes = [c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp]
    lib.moe_route_segments.restype = c_int
    lib.moe_route_segments.argtypes = [c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp,
                                       c_vp]
    lib.moe_permute.restype = c_int
    lib.moe_permute.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.moe_permute_static.restype = c_int
    lib.moe_permute_static.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp]
    lib.moe_expert_group_forward.restype = c_int
    lib.moe_expert_group_forward.argtypes = [c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int,
                                             c_vp, c_vp, c_sz, c_vp]
    lib.moe_expert_group_forward_ex.restype = c_int
    lib.moe_expert_group_forward_ex.argtypes = [c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int,
                                                c_int, c_vp, c_vp, c_sz, c_int, c_vp]
    lib.moe_expert_group_forward_gather.restype = c_int
    lib.moe_expert_group_forward_gather.argtypes = [c_int, c_int, c_vp, c_vp, c_int, c_vp, c_vp, c_vp, c_vp, c_int,
                                                    c_int, c_int, c_int, c_vp, c_vp, c_sz, c_int, c_vp]
    lib.moe_expert_list_forward.restype = c_int
    lib.moe_expert_list_forward.argtypes = [c_vp, c_int, c_vp, c_vp, c_int, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int,
                                            c_int, c_vp, c_vp, c_sz, c_int, c_vp]
    lib.moe_shared_forward.restype = c_int
    lib.moe_shared_forward.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.moe_shared_forward_ex.restype = c_int
    lib.moe_shared_forward_ex.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_sz,
                                          c_int, c_vp]
    lib.moe_combine.restype = c_int
    lib.moe_combine.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_int, c_vp, c_vp]
    lib.moe_combine_parts.restype = c_int
    lib.moe_combine_parts.argtypes = [c_vp, c_vp, c_vp, c_vp, c_int, c_vp, c_int, c_int, c_int, c_vp, c_vp]
    lib.moe_fused_shared_sets.restype = c_int
    lib.moe_fused_shared_sets.argtypes = [c_int] * 6
    lib.moe_fused_workspace_bytes.restype = c_sz
    lib.moe_fused_workspace_bytes.argtypes = [c_int] * 4
    lib.moe_expert_group_forward_fused.restype = c_int
    lib.moe_expert_group_forward_fused.argtypes = [c_int, c_int, c_vp, c_vp, c_int, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp,
                                                   c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp,
                                                   c_sz, c_int, c_vp]
    for n in ("moe_permute_workspace_bytes", "moe_expert_workspace_bytes", "moe_shared_workspace_bytes"):
        getattr(lib, n).restype = c_sz
    lib.moe_permute_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.moe_expert_workspace_bytes.argtypes = [c_int, c_int]
    lib.moe_shared_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.moe_residual_norm.restype = c_int
    lib.moe_residual_norm.argtypes = [c_vp, c_vp, c_int, c_int, ctypes.c_float, c_vp, c_vp]
    lib.moe_tile_clock_buffer.restype = c_int
    lib.moe_tile_clock_buffer.argtypes = [c_vp, c_int]
    lib.moe_probe_mfma.restype = c_int
    lib.moe_probe_mfma.argtypes = [c_vp, c_sz, c_int, c_int, c_vp, c_vp]
    lib.moe_workspace_bytes.restype = c_sz
    lib.moe_workspace_bytes.argtypes = [c_int] * 6
    _LIB = lib
    return lib


def moe_tile_clock_buffer(clocks):
    """Switch the clock record of the tile kernels on (clocks = int64 GPU tensor of 4 * n entries, n workgroups
    recorded) or off (None) for launches made by this host thread."""
    if clocks is None:
        _check(load().moe_tile_clock_buffer(None, 0), "moe_tile_clock_buffer")
        return
    _check(load().moe_tile_clock_buffer(_ptr(clocks, torch.int64, "clocks"), clocks.numel() // 4), "moe_tile_clock_buffer")


def moe_probe_mfma(operands, iters: int, workgroups: int, clocks):
    """One launch of the MFMA rate probe: operands = at least 32768 bytes of bf16 on the GPU, clocks = int64 GPU
    tensor of 2 * workgroups entries (shader clock ticks, 100 MHz ticks per workgroup).  The caller times it."""
    if clocks.numel() < 2 * workgroups:
        raise MoeError("moe_probe_mfma: clocks needs 2 * workgroups entries")
    rc = load().moe_probe_mfma(_ptr(operands, torch.bfloat16, "operands"), operands.numel() * operands.element_size(),
                               int(iters), int(workgroups), _ptr(clocks, torch.int64, "clocks"), _stream())
    _check(rc, "moe_probe_mfma")
    return clocks


def build_id() -> str:
    """Id of the sources the loaded library was built from (see build.source_id)."""
    return load().moe_build_id().decode()


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise MoeError(f"{what}: {load().moe_status_string(rc).decode()} (status {rc})")


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype], name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise MoeError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise MoeError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise MoeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def moe_workspace_bytes(T: int, H: int, E: int, K: int, I: int, Is: int) -> int:
    return int(load().moe_workspace_bytes(T, H, E, K, I, Is))


def moe_route(x, Wr, bias, K: int, renorm: bool, topk_ids=None, topk_w=None):
    T, H = x.shape
    E = Wr.shape[0]
    if topk_ids is None:
        topk_ids = torch.empty((T, K), dtype=torch.int32, device=x.device)
    if topk_w is None:
        topk_w = torch.empty((T, K), dtype=torch.float32, device=x.device)
    rc = load().moe_route(_ptr(x, torch.bfloat16, "x"), _ptr(Wr, torch.bfloat16, "Wr"),
                          _ptr(bias, torch.float32, "bias"), T, H, E, K, int(bool(renorm)),
                          _ptr(topk_ids, torch.int32, "topk_ids"), _ptr(topk_w, torch.float32, "topk_w"), _stream())
    _check(rc, "moe_route")
    return topk_ids, topk_w


def moe_route_segments(x, Wr, bias_rows, seg_offsets, K: int, renorm: bool, topk_ids=None, topk_w=None):
    """bias_rows [n_seg, E] fp32, seg_offsets [n_seg + 1] int32, both on the device: token t of
    segment s is routed with bias_rows[s] (one launch for a batch assembled from several tenants)."""
    T, H = x.shape
    E = Wr.shape[0]
    n_seg = bias_rows.shape[0]
    if bias_rows.shape != (n_seg, E) or seg_offsets.numel() != n_seg + 1:
        raise MoeError("moe_route_segments: bias_rows must be [n_seg, E] and seg_offsets [n_seg + 1]")
    if topk_ids is None:
        topk_ids = torch.empty((T, K), dtype=torch.int32, device=x.device)
    if topk_w is None:
        topk_w = torch.empty((T, K), dtype=torch.float32, device=x.device)
    rc = load().moe_route_segments(_ptr(x, torch.bfloat16, "x"), _ptr(Wr, torch.bfloat16, "Wr"),
                                   _ptr(bias_rows, torch.float32, "bias_rows"),
                                   _ptr(seg_offsets, torch.int32, "seg_offsets"), n_seg, T, H, E, K,
                                   int(bool(renorm)), _ptr(topk_ids, torch.int32, "topk_ids"),
                                   _ptr(topk_w, torch.float32, "topk_w"), _stream())
    _check(rc, "moe_route_segments")
    return topk_ids, topk_w


def segment_offsets(tenant_rows, T: int, device):
    """Device array of segment bounds for moe_route_segments, or None when the tenants' row ranges
    are not the consecutive slices [0, a1), [a1, a2), ... [.., T) of the batch."""
    bounds = [0]
    for a, b in tenant_rows:
        if a != bounds[-1] or b < a:
            return None
        bounds.append(b)
    if bounds[-1] != T:
        return None
    return torch.tensor(bounds, dtype=torch.int32, device=device)


def moe_permute(topk_ids, x, E: int, expert_offsets=None, src_of_row=None, row_of_pair=None, Xp=None,
                workspace=None, materialize: bool = True):
    """materialize=False: only the index arrays are built (Xp is returned as None); the block calls
    then take x and src_of_row (moe_expert_group_forward_gather)."""
    T, K = topk_ids.shape
    H = x.shape[1]
    dev = x.device
    if expert_offsets is None:
        expert_offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
    if src_of_row is None:
        src_of_row = torch.empty(T * K, dtype=torch.int32, device=dev)
    if row_of_pair is None:
        row_of_pair = torch.empty(T * K, dtype=torch.int32, device=dev)
    if not materialize:
        Xp = None
    elif Xp is None:
        Xp = torch.empty((T * K, H), dtype=torch.bfloat16, device=dev)
    if workspace is None:
        workspace = torch.empty(max(int(load().moe_permute_workspace_bytes(T, K, E)), 256), dtype=torch.uint8,
                                device=dev)
    rc = load().moe_permute(_ptr(topk_ids, torch.int32, "topk_ids"), _ptr(x, torch.bfloat16, "x"), T, H, E, K,
                            _ptr(expert_offsets, torch.int32, "expert_offsets"),
                            _ptr(src_of_row, torch.int32, "src_of_row"),
                            _ptr(row_of_pair, torch.int32, "row_of_pair"), _ptr(Xp, torch.bfloat16, "Xp"),
                            _ptr(workspace, None, "workspace"), workspace.numel() * workspace.element_size(),
                            _stream())
    _check(rc, "moe_permute")
    return expert_offsets, src_of_row, row_of_pair, Xp


def moe_permute_static(topk_ids, x, E: int, expert_offsets, src_of_row, row_of_pair, Xp=None):
    """moe_permute without a workspace and without any allocation: every output tensor is the caller's
    (Xp None: index arrays only); the sort's table lives in a buffer inside the library."""
    T, K = topk_ids.shape
    H = x.shape[1]
    rc = load().moe_permute_static(_ptr(topk_ids, torch.int32, "topk_ids"), _ptr(x, torch.bfloat16, "x"), T, H, E, K,
                                   _ptr(expert_offsets, torch.int32, "expert_offsets"),
                                   _ptr(src_of_row, torch.int32, "src_of_row"),
                                   _ptr(row_of_pair, torch.int32, "row_of_pair"), _ptr(Xp, torch.bfloat16, "Xp"),
                                   _stream())
    _check(rc, "moe_permute_static")
    return expert_offsets, src_of_row, row_of_pair, Xp


def moe_expert_group_forward(group_lo: int, group_hi: int, Xp, expert_offsets, Wg, Wu, Wd, Yp, workspace,
                             policy: int = 0):
    """policy 0 (default) is the plain call; any other value goes to moe_expert_group_forward_ex."""
    P, H = Xp.shape
    E, I, _ = Wg.shape
    args = (int(group_lo), int(group_hi), _ptr(Xp, torch.bfloat16, "Xp"),
            _ptr(expert_offsets, torch.int32, "expert_offsets"), _ptr(Wg, torch.bfloat16, "Wg"),
            _ptr(Wu, torch.bfloat16, "Wu"), _ptr(Wd, torch.bfloat16, "Wd"), P, H, E, I, _ptr(Yp, torch.bfloat16, "Yp"),
            _ptr(workspace, None, "workspace"), 0 if workspace is None else workspace.numel() * workspace.element_size())
    if int(policy) == 0:
        rc = load().moe_expert_group_forward(*args, _stream())
    else:
        rc = load().moe_expert_group_forward_ex(*args, int(policy), _stream())
    _check(rc, "moe_expert_group_forward")
    return Yp


def moe_expert_group_forward_gather(group_lo: int, group_hi: int, x, src_of_row, K: int, expert_offsets, Wg, Wu, Wd,
                                    Yp, workspace, policy: int = 0):
    """The block invocation reading its rows as x[src_of_row[r] // K] (no permuted copy)."""
    P = src_of_row.shape[0]
    H = x.shape[1]
    E, I, _ = Wg.shape
    if x.shape[0] * K != P:
        raise MoeError("moe_expert_group_forward_gather: x must have P / K rows")
    rc = load().moe_expert_group_forward_gather(int(group_lo), int(group_hi), _ptr(x, torch.bfloat16, "x"),
                                                _ptr(src_of_row, torch.int32, "src_of_row"), int(K),
                                                _ptr(expert_offsets, torch.int32, "expert_offsets"),
                                                _ptr(Wg, torch.bfloat16, "Wg"), _ptr(Wu, torch.bfloat16, "Wu"),
                                                _ptr(Wd, torch.bfloat16, "Wd"), P, H, E, I,
                                                _ptr(Yp, torch.bfloat16, "Yp"), _ptr(workspace, None, "workspace"),
                                                0 if workspace is None else workspace.numel() * workspace.element_size(),
                                                int(policy), _stream())
    _check(rc, "moe_expert_group_forward_gather")
    return Yp


def moe_expert_list_forward(expert_ids, tokens, src_of_row, K: int, expert_offsets, Wg, Wu, Wd, Yp, workspace,
                            policy: int = 0):
    """Block invocation for the experts listed in expert_ids (int32 GPU tensor).  tokens is Xp when
    src_of_row is None, else x (rows read through src_of_row)."""
    E, I, H = Wg.shape
    P = Yp.shape[0]
    rc = load().moe_expert_list_forward(_ptr(expert_ids, torch.int32, "expert_ids"), int(expert_ids.numel()),
                                        _ptr(tokens, torch.bfloat16, "tokens"),
                                        _ptr(src_of_row, torch.int32, "src_of_row"), int(K),
                                        _ptr(expert_offsets, torch.int32, "expert_offsets"),
                                        _ptr(Wg, torch.bfloat16, "Wg"), _ptr(Wu, torch.bfloat16, "Wu"),
                                        _ptr(Wd, torch.bfloat16, "Wd"), P, H, E, I,
                                        _ptr(Yp, torch.bfloat16, "Yp"), _ptr(workspace, None, "workspace"),
                                        0 if workspace is None else workspace.numel() * workspace.element_size(),
                                        int(policy), _stream())
    _check(rc, "moe_expert_list_forward")
    return Yp


def balanced_blocks(rows_per_expert: Sequence[int], n_blocks: int) -> List[List[int]]:
    """Hot-expert-aware block formation on the host: experts sorted by observed load (rows in a
    previous batch) are dealt, heaviest first, to the block with the fewest rows so far.  Returns
    n_blocks lists of expert ids (each ascending); every expert appears exactly once."""
    n_blocks = max(1, min(int(n_blocks), len(rows_per_expert)))
    order = sorted(range(len(rows_per_expert)), key=lambda e: (-int(rows_per_expert[e]), e))
    blocks: List[List[int]] = [[] for _ in range(n_blocks)]
    load_ = [0] * n_blocks
    for e in order:
        b = min(range(n_blocks), key=lambda i: (load_[i], len(blocks[i]), i))
        blocks[b].append(e)
        load_[b] += int(rows_per_expert[e])
    return [sorted(b) for b in blocks]


def moe_shared_forward(x, Wsg, Wsu, Wsd, wgate, S, sg, workspace, policy: int = 0):
    """policy 0 (default) is the plain call; any other value goes to moe_shared_forward_ex."""
    T, H = x.shape
    Is = Wsg.shape[0]
    args = (_ptr(x, torch.bfloat16, "x"), _ptr(Wsg, torch.bfloat16, "Wsg"), _ptr(Wsu, torch.bfloat16, "Wsu"),
            _ptr(Wsd, torch.bfloat16, "Wsd"), _ptr(wgate, torch.bfloat16, "wgate"), T, H, Is, _ptr(S, torch.bfloat16, "S"),
            _ptr(sg, torch.float32, "sg"), _ptr(workspace, None, "workspace"),
            0 if workspace is None else workspace.numel() * workspace.element_size())
    if int(policy) == 0:
        rc = load().moe_shared_forward(*args, _stream())
    else:
        rc = load().moe_shared_forward_ex(*args, int(policy), _stream())
    _check(rc, "moe_shared_forward")
    return S, sg


def moe_combine(Yp, row_of_pair, topk_w, S, sg, out=None):
    T, K = topk_w.shape
    H = Yp.shape[1]
    if out is None:
        out = torch.empty((T, H), dtype=torch.bfloat16, device=Yp.device)
    rc = load().moe_combine(_ptr(Yp, torch.bfloat16, "Yp"), _ptr(row_of_pair, torch.int32, "row_of_pair"),
                            _ptr(topk_w, torch.float32, "topk_w"), _ptr(S, torch.bfloat16, "S"),
                            _ptr(sg, torch.float32, "sg"), T, H, K, _ptr(out, torch.bfloat16, "out"), _stream())
    _check(rc, "moe_combine")
    return out


def moe_fused_shared_sets(T: int, H: int, E: int, K: int, I: int, Is: int) -> int:
    """Number of shared-expert sets the fused block call would run for these sizes, 0 when it does not apply."""
    return int(load().moe_fused_shared_sets(T, H, E, K, I, Is))


def moe_expert_group_forward_fused(group_lo: int, group_hi: int, x, src_of_row, K: int, expert_offsets, Wg, Wu, Wd,
                                   Wsg, Wsu, Wsd, wgate, Yp, S_parts, sg, workspace, policy: int = 0):
    """The block invocation for experts [group_lo, group_hi) that also runs the shared experts (as Is / I
    experts of size I on every token) in the same two launches; S_parts [Is / I, T, H]."""
    T, H = x.shape
    E, I, _ = Wg.shape
    Is = Wsg.shape[0]
    rc = load().moe_expert_group_forward_fused(int(group_lo), int(group_hi), _ptr(x, torch.bfloat16, "x"),
                                               _ptr(src_of_row, torch.int32, "src_of_row"), int(K),
                                               _ptr(expert_offsets, torch.int32, "expert_offsets"),
                                               _ptr(Wg, torch.bfloat16, "Wg"), _ptr(Wu, torch.bfloat16, "Wu"),
                                               _ptr(Wd, torch.bfloat16, "Wd"), _ptr(Wsg, torch.bfloat16, "Wsg"),
                                               _ptr(Wsu, torch.bfloat16, "Wsu"), _ptr(Wsd, torch.bfloat16, "Wsd"),
                                               _ptr(wgate, torch.bfloat16, "wgate"), T, H, E, I, Is,
                                               _ptr(Yp, torch.bfloat16, "Yp"), _ptr(S_parts, torch.bfloat16, "S_parts"),
                                               _ptr(sg, torch.float32, "sg"), _ptr(workspace, None, "workspace"),
                                               0 if workspace is None else workspace.numel() * workspace.element_size(),
                                               int(policy), _stream())
    _check(rc, "moe_expert_group_forward_fused")
    return Yp, S_parts, sg


def moe_combine_parts(Yp, row_of_pair, topk_w, S_parts, sg, out=None):
    T, K = topk_w.shape
    H = Yp.shape[1]
    if out is None:
        out = torch.empty((T, H), dtype=torch.bfloat16, device=Yp.device)
    rc = load().moe_combine_parts(_ptr(Yp, torch.bfloat16, "Yp"), _ptr(row_of_pair, torch.int32, "row_of_pair"),
                                  _ptr(topk_w, torch.float32, "topk_w"), _ptr(S_parts, torch.bfloat16, "S_parts"),
                                  int(S_parts.shape[0]), _ptr(sg, torch.float32, "sg"), T, H, K,
                                  _ptr(out, torch.bfloat16, "out"), _stream())
    _check(rc, "moe_combine_parts")
    return out


def moe_residual_norm(x, y, out=None, eps: float = 1e-6):
    T, H = x.shape
    if out is None:
        out = torch.empty_like(x)
    rc = load().moe_residual_norm(_ptr(x, torch.bfloat16, "x"), _ptr(y, torch.bfloat16, "y"), T, H, float(eps),
                                  _ptr(out, torch.bfloat16, "out"), _stream())
    _check(rc, "moe_residual_norm")
    return out


@dataclass
class LayerBuffers:
    """Every output and scratch tensor of one layer forward, allocated once and reused."""
    topk_ids: torch.Tensor
    topk_w: torch.Tensor
    expert_offsets: torch.Tensor
    src_of_row: torch.Tensor
    row_of_pair: torch.Tensor
    Xp: torch.Tensor
    Yp: torch.Tensor
    S: Optional[torch.Tensor]
    sg: Optional[torch.Tensor]
    out: torch.Tensor
    workspace: torch.Tensor
    workspace_shared: Optional[torch.Tensor]
    workspace_permute: Optional[torch.Tensor] = None
    S_parts: Optional[torch.Tensor] = None          # [Is / I, T, H]: outputs of the shared experts of the fused block call
    workspace_fused: Optional[torch.Tensor] = None

    @staticmethod
    def allocate(T: int, H: int, E: int, K: int, I: int, Is: int, device="cuda") -> "LayerBuffers":
        lib = load()
        P = T * K
        i32 = dict(dtype=torch.int32, device=device)
        bf = dict(dtype=torch.bfloat16, device=device)
        ws = max(int(lib.moe_expert_workspace_bytes(P, I)), 256)
        wss = int(lib.moe_shared_workspace_bytes(T, H, Is))
        ns = int(lib.moe_fused_shared_sets(T, H, E, K, I, Is)) if Is > 0 else 0
        fused = {}
        if ns > 0:     # the fused call's h holds the routed rows and then the rows of every shared set
            fused = dict(S_parts=torch.empty((ns, T, H), **bf),
                         workspace_fused=torch.empty(int(lib.moe_fused_workspace_bytes(T, K, I, Is)), dtype=torch.uint8,
                                                     device=device))
        return LayerBuffers(**fused,
            topk_ids=torch.empty((T, K), **i32), topk_w=torch.empty((T, K), dtype=torch.float32, device=device),
            expert_offsets=torch.empty(E + 1, **i32), src_of_row=torch.empty(P, **i32),
            row_of_pair=torch.empty(P, **i32), Xp=torch.empty((P, H), **bf), Yp=torch.empty((P, H), **bf),
            S=torch.empty((T, H), **bf) if Is > 0 else None,
            sg=torch.empty(T, dtype=torch.float32, device=device) if Is > 0 else None,
            out=torch.empty((T, H), **bf), workspace=torch.empty(ws, dtype=torch.uint8, device=device),
            workspace_shared=torch.empty(max(wss, 256), dtype=torch.uint8, device=device) if Is > 0 else None,
            workspace_permute=torch.empty(max(int(lib.moe_permute_workspace_bytes(T, K, E)), 256), dtype=torch.uint8,
                                          device=device))


def moe_layer_forward(x, Wr, bias, Wg, Wu, Wd, shared, K: int, renorm: bool,
                      groups: Optional[Sequence[Tuple[int, int]]] = None, buf: Optional[LayerBuffers] = None,
                      tenant_rows: Optional[List[Tuple[int, int]]] = None, policy: int = 0,
                      shared_policy: int = 0, shared_stream: Optional[torch.cuda.Stream] = None,
                      fused_gather: bool = False, seg_offsets: Optional[torch.Tensor] = None,
                      fused_shared: bool = False) -> LayerBuffers:
    """One MoE layer in the paper's order: gating, micro-batch construction, one call per expert
    block, shared expert, aggregation.  Sequencing only; every step is a library call.

    shared: (Wsg, Wsu, Wsd, wgate) or None.  groups: expert blocks (lo, hi), default one block.
    tenant_rows with a [n_tenants, E] bias: one gating launch over the whole batch with one bias row
    per tenant slice (seg_offsets: the slice bounds on the device, built here when not given; pass
    it when the call is captured into a graph); slices that are not consecutive are gated one by one.
    shared_stream: run the shared expert on this stream, concurrently with gating, permutation and
    the routed blocks (it depends on x only); the aggregation waits for it.
    fused_gather: no permuted copy Xp; the block calls read x through src_of_row.
    fused_shared: the first block call also runs the shared experts (moe_expert_group_forward_fused, which
    reads x through src_of_row) and the aggregation takes their outputs as separate parts; sizes the fused
    call does not serve fall back to the separate calls."""
    T, H = x.shape
    E, I, _ = Wg.shape
    Is = 0 if shared is None else shared[0].shape[0]
    if buf is None:
        buf = LayerBuffers.allocate(T, H, E, K, I, Is, x.device)
    main = torch.cuda.current_stream()
    fork = None
    fused_shared = bool(fused_shared and shared is not None and buf.S_parts is not None)
    if fused_shared:
        fused_gather, shared_stream = True, None
    if shared is not None and shared_stream is not None:
        fork = torch.cuda.Event()     # the shared expert needs x only: its branch forks off here
        fork.record(main)
    if (tenant_rows is not None and bias is not None and seg_offsets is None and len(tenant_rows) > 1
            and not torch.cuda.is_current_stream_capturing()):   # (a capture cannot take the host-to-device copy)
        seg_offsets = segment_offsets(tenant_rows, T, x.device)
    if tenant_rows is not None and bias is not None and seg_offsets is not None:
        moe_route_segments(x, Wr, bias, seg_offsets, K, renorm, buf.topk_ids, buf.topk_w)
    elif tenant_rows is not None:
        for i, (a, b) in enumerate(tenant_rows):
            moe_route(x[a:b], Wr, None if bias is None else bias[i], K, renorm, buf.topk_ids[a:b], buf.topk_w[a:b])
    else:
        moe_route(x, Wr, bias, K, renorm, buf.topk_ids, buf.topk_w)
    moe_permute(buf.topk_ids, x, E, buf.expert_offsets, buf.src_of_row, buf.row_of_pair, buf.Xp,
                buf.workspace_permute, materialize=not fused_gather)
    for i, (lo, hi) in enumerate(groups or [(0, E)]):
        if fused_shared and i == 0:
            moe_expert_group_forward_fused(lo, hi, x, buf.src_of_row, K, buf.expert_offsets, Wg, Wu, Wd, shared[0],
                                           shared[1], shared[2], shared[3], buf.Yp, buf.S_parts, buf.sg,
                                           buf.workspace_fused, policy)
        elif fused_gather:
            moe_expert_group_forward_gather(lo, hi, x, buf.src_of_row, K, buf.expert_offsets, Wg, Wu, Wd, buf.Yp,
                                            buf.workspace, policy)
        else:
            moe_expert_group_forward(lo, hi, buf.Xp, buf.expert_offsets, Wg, Wu, Wd, buf.Yp, buf.workspace, policy)
    if fused_shared:
        moe_combine_parts(buf.Yp, buf.row_of_pair, buf.topk_w, buf.S_parts, buf.sg, buf.out)
        return buf
    if shared is not None and shared_stream is None:
        moe_shared_forward(x, shared[0], shared[1], shared[2], shared[3], buf.S, buf.sg, buf.workspace_shared,
                           shared_policy)
    if shared is not None and shared_stream is not None:
        # enqueued after the routed path, so that in a captured graph the routed path shares its
        # hardware queue with the aggregation and the step's critical path crosses no queue boundary
        shared_stream.wait_event(fork)
        with torch.cuda.stream(shared_stream):
            # 0x400: leave room on the CUs for the small kernels of the routed path running beside it
            moe_shared_forward(x, shared[0], shared[1], shared[2], shared[3], buf.S, buf.sg, buf.workspace_shared,
                               shared_policy | 0x400)
        main.wait_stream(shared_stream)
    moe_combine(buf.Yp, buf.row_of_pair, buf.topk_w, buf.S, buf.sg, buf.out)
    return buf


def moe_stack_forward(x, layers, K: int, renorm: bool, buf: Optional[LayerBuffers] = None, x_out=None,
                      eps: float = 1e-6):
    """A stack of MoE layers without attention: x <- residual_norm(x, MoE_l(x)) for each layer.

    layers: sequence of dicts with Wr, Wg, Wu, Wd and optionally Wsg, Wsu, Wsd, wgate, bias.
    Everything is enqueued on the current stream; nothing synchronises.  Returns the final
    activations (x_out if given; x itself is not modified)."""
    T, H = x.shape
    first = layers[0]
    E, I, _ = first["Wg"].shape
    Is = 0 if first.get("Wsg") is None else first["Wsg"].shape[0]
    if buf is None:
        buf = LayerBuffers.allocate(T, H, E, K, I, Is, x.device)
    cur = x
    if x_out is None:
        x_out = torch.empty_like(x)
    for w in layers:
        shared = None if w.get("Wsg") is None else (w["Wsg"], w["Wsu"], w["Wsd"], w["wgate"])
        moe_layer_forward(cur, w["Wr"], w.get("bias"), w["Wg"], w["Wu"], w["Wd"], shared, K, renorm, buf=buf)
        moe_residual_norm(cur, buf.out, x_out, eps)
        cur = x_out
    return x_out
