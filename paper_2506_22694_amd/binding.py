"""Thin Python binding over the C ABI of libvocabtrim.so (include/vocabtrim.h).

Argument marshalling only: torch tensors supply device memory and the current
HIP stream; every step of the path runs in the library's kernels.  There is no
fallback: if the library is missing, or a call returns an error status, a
RuntimeError is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libvocabtrim.so")

VT_F32, VT_BF16 = 0, 1
VT_I32, VT_I64 = 0, 1
VT_MAX_TOP_M = 64

EXPORTS = (
    "vt_status_string", "vt_last_device_error",
    "vt_count_tokens", "vt_count_tokens_ws_bytes",
    "vt_build_trimmed_head", "vt_build_trimmed_head_ws_bytes", "vt_build_trimmed_head_by_rank",
    "vt_choose_k", "vt_choose_k_ws_bytes",
    "vt_draft_head_step", "vt_draft_head_step_ws_bytes", "vt_draft_head_step_ws_init",
    "vt_draft_head_step_static", "vt_draft_head_step_plan", "vt_draft_head_step_multi_plan",
    "vt_tree_expand", "vt_tree_rerank", "vt_draft_tree_level", "vt_stream_read_reference",
    "vt_build_trimmed_heads", "vt_draft_head_step_multi", "vt_draft_head_step_multi_ws_bytes",
)
VT_MAX_HEADS, VT_MULTI_MAX_ROWS = 16, 256
VT_TREE_MAX_CANDIDATES, VT_TREE_MAX_KEEP = 16384, 1024

_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen libvocabtrim.so and declare its prototypes.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(hipcc, gfx950). There is no CPU fallback.")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz, ci = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
    L.vt_status_string.argtypes = [ci]
    L.vt_status_string.restype = ctypes.c_char_p
    L.vt_last_device_error.argtypes = []
    L.vt_last_device_error.restype = ctypes.c_char_p
    L.vt_count_tokens.argtypes = [vp, ci, i64, i32, vp, vp, vp, sz, vp]
    L.vt_count_tokens.restype = ci
    L.vt_count_tokens_ws_bytes.argtypes = [i32, i64]
    L.vt_count_tokens_ws_bytes.restype = sz
    L.vt_build_trimmed_head.argtypes = [vp, i32, vp, ci, i32, i32, vp, vp, vp, sz, vp]
    L.vt_build_trimmed_head.restype = ci
    L.vt_build_trimmed_head_ws_bytes.argtypes = [i32, i32, i32]
    L.vt_build_trimmed_head_ws_bytes.restype = sz
    L.vt_build_trimmed_head_by_rank.argtypes = [vp, i32, vp, ci, i32, i32, vp, vp, vp, sz, vp]
    L.vt_build_trimmed_head_by_rank.restype = ci
    L.vt_choose_k.argtypes = [vp, i32, ci, ctypes.c_double, i64, vp, vp, sz, vp]
    L.vt_choose_k.restype = ci
    L.vt_choose_k_ws_bytes.argtypes = [i32]
    L.vt_choose_k_ws_bytes.restype = sz
    L.vt_draft_head_step.argtypes = [vp, ci, i32, vp, ci, i32, i32, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    L.vt_draft_head_step.restype = ci
    L.vt_draft_head_step_static.argtypes = [vp, ci, i32, vp, ci, i32, i32, vp, i32, vp, vp, vp, vp, vp]
    L.vt_draft_head_step_static.restype = ci
    L.vt_draft_head_step_plan.argtypes = [i32, i32, i32, i32, ci, ctypes.c_char_p, sz]
    L.vt_draft_head_step_plan.restype = ci
    L.vt_draft_head_step_multi_plan.argtypes = [i32, i32, vp, i32, vp, i32, ci, ctypes.c_char_p, sz]
    L.vt_draft_head_step_multi_plan.restype = ci
    L.vt_draft_head_step_ws_bytes.argtypes = [i32, i32, i32, i32]
    L.vt_draft_head_step_ws_bytes.restype = sz
    L.vt_draft_head_step_ws_init.argtypes = [vp, sz, vp]
    L.vt_draft_head_step_ws_init.restype = ci
    L.vt_tree_expand.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
    L.vt_tree_expand.restype = ci
    L.vt_tree_rerank.argtypes = [vp, i32, i32, vp, vp]
    L.vt_tree_rerank.restype = ci
    L.vt_draft_tree_level.argtypes = [vp, ci, i32, vp, ci, i32, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    L.vt_draft_tree_level.restype = ci
    L.vt_stream_read_reference.argtypes = [vp, sz, vp, vp]
    L.vt_stream_read_reference.restype = ci
    L.vt_build_trimmed_heads.argtypes = [vp, i32, i32, vp, ci, i32, vp, vp, vp, vp, sz, vp]
    L.vt_build_trimmed_heads.restype = ci
    L.vt_draft_head_step_multi.argtypes = [vp, ci, i32, i32, vp, ci, vp, vp, i32, vp, i32, vp, vp, vp, vp, sz, vp]
    L.vt_draft_head_step_multi.restype = ci
    L.vt_draft_head_step_multi_ws_bytes.argtypes = [i32, i32, vp, i32, i32]
    L.vt_draft_head_step_multi_ws_bytes.restype = sz
    _lib = L
    return L


class VocabTrimError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        L = load_library()
        msg = L.vt_status_string(status).decode()
        if status == 6:
            msg += " (" + L.vt_last_device_error().decode() + ")"
        super().__init__(msg)


def _check(status: int) -> None:
    if status != 0:
        raise VocabTrimError(status)


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return VT_BF16
    if t.dtype == torch.float32:
        return VT_F32
    raise TypeError(f"unsupported element type {t.dtype}")


def _require_cuda(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def _scratch(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# --------------------------------------------------------------------------- Alg. 1
def count_tokens(ids: torch.Tensor, V: int, counts: torch.Tensor | None = None,
                 n_invalid: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> torch.Tensor:
    """counts[t] += 1 for every id in `ids` (int32/int64 device tensor).  Returns counts (int64 [V])."""
    L = load_library()
    _require_cuda(ids, counts, n_invalid, ws)
    if ids.dtype == torch.int32:
        it = VT_I32
    elif ids.dtype == torch.int64:
        it = VT_I64
    else:
        raise TypeError("ids must be int32 or int64")
    dev = ids.device
    if counts is None:
        counts = torch.zeros(V, dtype=torch.int64, device=dev)
    n = ids.numel()
    need = L.vt_count_tokens_ws_bytes(V, n)
    if ws is None:
        ws = _scratch(need, dev)
    _check(L.vt_count_tokens(_ptr(ids) if n else None, it, n, V, _ptr(counts), _ptr(n_invalid), _ptr(ws),
                             ws.numel(), _stream(dev)))
    return counts


# --------------------------------------------------------------------------- Eq. 1
def build_trimmed_head(counts: torch.Tensor, W: torch.Tensor | None, k: int, ws: torch.Tensor | None = None,
                       out_map: torch.Tensor | None = None, out_W: torch.Tensor | None = None, order: str = "id"):
    """Top-k ids by count (ties -> lower id) and the gathered head rows.

    order="id": ascending target id; order="rank": (count descending, id ascending), every prefix being
    the build for a smaller k.  Returns (map int32 [k], W_trim [k,d] or None); `out_map` / `out_W` supply
    the result tensors.
    """
    if order not in ("id", "rank"):
        raise ValueError("order must be 'id' or 'rank'")
    L = load_library()
    _require_cuda(counts, W, ws)
    if counts.dtype != torch.int64:
        raise TypeError("counts must be int64")
    dev = counts.device
    V = counts.numel()
    _require_cuda(out_map, out_W)
    if out_map is not None and (out_map.dtype != torch.int32 or out_map.numel() != k):
        raise ValueError("out_map must be int32 [k]")
    map_ = out_map if out_map is not None else torch.empty(k, dtype=torch.int32, device=dev)
    if W is not None:
        d = W.shape[1]
        if out_W is not None and (out_W.dtype != W.dtype or tuple(out_W.shape) != (k, d)):
            raise ValueError("out_W must be [k, d] of W's element type")
        W_trim = out_W if out_W is not None else torch.empty((k, d), dtype=W.dtype, device=dev)
        wt = _dtype_code(W)
    else:
        d, W_trim, wt = 8, None, VT_BF16
    if ws is None:
        ws = _scratch(L.vt_build_trimmed_head_ws_bytes(V, d, k), dev)
    fn = L.vt_build_trimmed_head if order == "id" else L.vt_build_trimmed_head_by_rank
    _check(fn(_ptr(counts), V, _ptr(W), wt, d, k, _ptr(map_), _ptr(W_trim), _ptr(ws), ws.numel(), _stream(dev)))
    return map_, W_trim


VT_K_TOP_P, VT_K_MIN_COUNT = 0, 1


def choose_k(counts: torch.Tensor, top_p: float | None = None, min_count: int | None = None,
             ws: torch.Tensor | None = None):
    """k from the counts (Top-P mass or minimum count).  Returns host ints (k, covered, total); synchronises."""
    L = load_library()
    _require_cuda(counts, ws)
    if counts.dtype != torch.int64:
        raise TypeError("counts must be int64")
    if (top_p is None) == (min_count is None):
        raise ValueError("give exactly one of top_p and min_count")
    dev = counts.device
    V = counts.numel()
    if ws is None:
        ws = _scratch(L.vt_choose_k_ws_bytes(V), dev)
    out = torch.empty(3, dtype=torch.int64, device=dev)
    mode = VT_K_TOP_P if top_p is not None else VT_K_MIN_COUNT
    _check(L.vt_choose_k(_ptr(counts), V, mode, float(top_p or 0.0), int(min_count or 0), _ptr(out), _ptr(ws),
                         ws.numel(), _stream(dev)))
    k, cov, tot = (int(x) for x in out.cpu().tolist())
    return k, cov, tot


# --------------------------------------------------------------------------- Alg. 2, drafting lines
class StepWorkspace:
    """Device scratch of the draft step: allocated once (no initialisation needed), reused by every step."""

    def __init__(self, n: int, k: int, d: int, m: int, device):
        L = load_library()
        nbytes = L.vt_draft_head_step_ws_bytes(n, k, d, m)
        if nbytes == 0:
            raise VocabTrimError(2)
        self.buf = _scratch(nbytes, device)

    @property
    def nbytes(self) -> int:
        return self.buf.numel()


def draft_head_step(h: torch.Tensor, W_trim: torch.Tensor, map_: torch.Tensor, m: int,
                    ws: StepWorkspace | None = None, return_lse: bool = False, return_full: bool = False,
                    out_ids: torch.Tensor | None = None, out_logp: torch.Tensor | None = None):
    """One draft step: (ids int32 [n,m] in target vocabulary, logp fp32 [n,m]) [+ lse [n]] [+ logp_full [n,k]]."""
    L = load_library()
    _require_cuda(h, W_trim, map_)
    n, d = h.shape
    k = W_trim.shape[0]
    if W_trim.shape[1] != d or map_.numel() != k or map_.dtype != torch.int32:
        raise ValueError("shape / dtype mismatch between h, W_trim and map")
    dev = h.device
    if ws is None:
        ws = StepWorkspace(n, k, d, m, dev)
    if out_ids is None:
        out_ids = torch.empty((n, m), dtype=torch.int32, device=dev)
    if out_logp is None:
        out_logp = torch.empty((n, m), dtype=torch.float32, device=dev)
    lse = torch.empty(n, dtype=torch.float32, device=dev) if return_lse else None
    full = torch.empty((n, k), dtype=torch.float32, device=dev) if return_full else None
    _check(L.vt_draft_head_step(_ptr(h), _dtype_code(h), n, _ptr(W_trim), _dtype_code(W_trim), k, d, _ptr(map_), m,
                                _ptr(out_ids), _ptr(out_logp), _ptr(lse), _ptr(full), _ptr(ws.buf), ws.nbytes,
                                _stream(dev)))
    res = [out_ids, out_logp]
    if return_lse:
        res.append(lse)
    if return_full:
        res.append(full)
    return tuple(res)


def draft_head_step_plan(n: int, k: int, d: int, m: int, dtype=torch.bfloat16) -> str:
    """The kernels the library launches for a draft step of this shape (host-only query)."""
    L = load_library()
    buf = ctypes.create_string_buffer(256)
    _check(L.vt_draft_head_step_plan(n, k, d, m, VT_BF16 if dtype == torch.bfloat16 else VT_F32, buf, 256))
    return buf.value.decode()


VT_STATIC_WS_BYTES = 4 << 20


def draft_head_step_static(h: torch.Tensor, W_trim: torch.Tensor, map_: torch.Tensor, m: int,
                           out_ids: torch.Tensor, out_logp: torch.Tensor, out_lse: torch.Tensor | None = None,
                           out_logp_full: torch.Tensor | None = None):
    """The draft step on the library's own per-GPU scratch array: no workspace, nothing allocated here either
    (the caller supplies every result tensor).  Returns (out_ids, out_logp)."""
    L = load_library()
    _require_cuda(h, W_trim, map_, out_ids, out_logp, out_lse, out_logp_full)
    n, d = h.shape
    k = W_trim.shape[0]
    if W_trim.shape[1] != d or map_.numel() != k or map_.dtype != torch.int32:
        raise ValueError("shape / dtype mismatch between h, W_trim and map")
    if out_ids.dtype != torch.int32 or out_logp.dtype != torch.float32 or out_ids.numel() != n * m or \
            out_logp.numel() != n * m:
        raise ValueError("out_ids / out_logp must be int32 / float32 [n, m]")
    if out_lse is not None and (out_lse.dtype != torch.float32 or out_lse.numel() != n):
        raise ValueError("out_lse must be float32 [n]")
    if out_logp_full is not None and (out_logp_full.dtype != torch.float32 or out_logp_full.numel() != n * k):
        raise ValueError("out_logp_full must be float32 [n, k]")
    _check(L.vt_draft_head_step_static(_ptr(h), _dtype_code(h), n, _ptr(W_trim), _dtype_code(W_trim), k, d,
                                       _ptr(map_), m, _ptr(out_ids), _ptr(out_logp), _ptr(out_lse),
                                       _ptr(out_logp_full), _stream(h.device)))
    return out_ids, out_logp


# --------------------------------------------------------------------------- several task heads (Sec. 4.1)
def _host_i32(values):
    arr = (ctypes.c_int32 * len(values))(*[int(v) for v in values])
    return arr


def _host_ptrs(tensors):
    arr = (ctypes.c_void_p * len(tensors))(*[_ptr(t) for t in tensors])
    return arr


def build_trimmed_heads(counts: torch.Tensor, W: torch.Tensor | None, ks, ws: torch.Tensor | None = None):
    """Eq. 1 for several count vectors (counts int64 [n_heads, V]) over one W: [(map_i, W_trim_i or None)]."""
    L = load_library()
    _require_cuda(counts, W, ws)
    if counts.dtype != torch.int64 or counts.dim() != 2 or not counts.is_contiguous():
        raise TypeError("counts must be a contiguous int64 [n_heads, V] tensor")
    H, V = counts.shape
    ks = [int(k) for k in ks]
    if len(ks) != H:
        raise ValueError("one k per row of counts")
    dev = counts.device
    maps = [torch.empty(max(k, 1), dtype=torch.int32, device=dev) for k in ks]
    if W is not None:
        d, wt = W.shape[1], _dtype_code(W)
        Ws = [torch.empty((max(k, 1), d), dtype=W.dtype, device=dev) for k in ks]
    else:
        d, wt, Ws = 8, VT_BF16, None
    if ws is None:
        ws = _scratch(L.vt_build_trimmed_head_ws_bytes(V, d, max(max(ks), 1)), dev)
    _check(L.vt_build_trimmed_heads(_ptr(counts), V, H, _ptr(W), wt, d, _host_i32(ks), _host_ptrs(maps),
                                    _host_ptrs(Ws) if Ws is not None else None, _ptr(ws), ws.numel(), _stream(dev)))
    return [(maps[i], Ws[i] if Ws is not None else None) for i in range(H)]


def draft_head_step_multi_plan(n: int, d: int, ks, head_of_row, m: int, dtype=torch.bfloat16) -> str:
    """How draft_head_step_multi would run these rows (pure host): one launch over several heads' tiles, or head by head."""
    L = load_library()
    buf = ctypes.create_string_buffer(256)
    ks = [int(k) for k in ks]
    hor = [int(x) for x in head_of_row]
    _check(L.vt_draft_head_step_multi_plan(n, d, _host_i32(ks), len(ks), _host_i32(hor), m,
                                           VT_BF16 if dtype == torch.bfloat16 else VT_F32, buf, 256))
    return buf.value.decode()


class MultiStepWorkspace:
    """Device scratch of a multi-head draft step of up to n rows over heads of the given sizes."""

    def __init__(self, n: int, d: int, ks, m: int, device):
        L = load_library()
        ks = [int(k) for k in ks]
        nbytes = L.vt_draft_head_step_multi_ws_bytes(n, d, _host_i32(ks), len(ks), m)
        if nbytes == 0:
            raise VocabTrimError(2)
        self.buf = _scratch(nbytes, device)

    @property
    def nbytes(self) -> int:
        return self.buf.numel()


def draft_head_step_multi(h: torch.Tensor, heads, head_of_row, m: int, ws: MultiStepWorkspace | None = None,
                          return_lse: bool = False, out_ids: torch.Tensor | None = None,
                          out_logp: torch.Tensor | None = None):
    """One draft step in which hidden row i uses heads[head_of_row[i]]; heads = [(W_trim, map), ...].

    head_of_row is a host sequence of ints.  Returns (ids [n,m], logp [n,m]) [+ lse [n]]."""
    L = load_library()
    Wts = [hd[0] for hd in heads]
    maps = [hd[1] for hd in heads]
    _require_cuda(h, *Wts, *maps)
    n, d = h.shape
    for Wt, mp in heads:
        if Wt.shape[1] != d or mp.numel() != Wt.shape[0] or mp.dtype != torch.int32 or Wt.dtype != h.dtype:
            raise ValueError("shape / dtype mismatch between h and a head")
    ks = [int(Wt.shape[0]) for Wt in Wts]
    hor = [int(x) for x in head_of_row]
    if len(hor) != n:
        raise ValueError("head_of_row must name a head for every row of h")
    dev = h.device
    if ws is None:
        ws = MultiStepWorkspace(n, d, ks, m, dev)
    if out_ids is None:
        out_ids = torch.empty((n, m), dtype=torch.int32, device=dev)
    if out_logp is None:
        out_logp = torch.empty((n, m), dtype=torch.float32, device=dev)
    lse = torch.empty(n, dtype=torch.float32, device=dev) if return_lse else None
    _check(L.vt_draft_head_step_multi(_ptr(h), _dtype_code(h), n, d, _host_ptrs(Wts), _dtype_code(h), _host_i32(ks),
                                      _host_ptrs(maps), len(heads), _host_i32(hor), m, _ptr(out_ids), _ptr(out_logp),
                                      _ptr(lse), _ptr(ws.buf), ws.nbytes, _stream(dev)))
    return (out_ids, out_logp, lse) if return_lse else (out_ids, out_logp)


# --------------------------------------------------------------------------- draft-tree selection (Sec. 4.1)
def tree_expand(parent_cum: torch.Tensor, step_logp: torch.Tensor, step_ids: torch.Tensor, K: int, out=None):
    """Next frontier of the draft tree: (parent int32 [K], token int32 [K], cum fp32 [K]), best first.

    `out` = (parent, token, cum) supplies the result tensors."""
    L = load_library()
    _require_cuda(parent_cum, step_logp, step_ids)
    if parent_cum.dtype != torch.float32 or step_logp.dtype != torch.float32 or step_ids.dtype != torch.int32:
        raise TypeError("parent_cum / step_logp must be float32 and step_ids int32")
    n, m = step_logp.shape
    if tuple(step_ids.shape) != (n, m) or parent_cum.numel() != n:
        raise ValueError("shape mismatch between parent_cum, step_logp and step_ids")
    dev = step_logp.device
    if out is not None:
        parent, token, cum = out
        _require_cuda(parent, token, cum)
        if (parent.dtype, token.dtype, cum.dtype) != (torch.int32, torch.int32, torch.float32) or \
                min(parent.numel(), token.numel(), cum.numel()) < K:
            raise ValueError("out must be (int32 [K], int32 [K], float32 [K])")
    else:
        parent = torch.empty(K, dtype=torch.int32, device=dev)
        token = torch.empty(K, dtype=torch.int32, device=dev)
        cum = torch.empty(K, dtype=torch.float32, device=dev)
    _check(L.vt_tree_expand(_ptr(parent_cum), _ptr(step_logp), _ptr(step_ids), n, m, K, _ptr(parent), _ptr(token),
                            _ptr(cum), _stream(dev)))
    return parent, token, cum


def tree_rerank(cum: torch.Tensor, T: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Indices (int32 [T], ascending) of the T best cumulative scores."""
    L = load_library()
    _require_cuda(cum)
    if cum.dtype != torch.float32 or cum.dim() != 1:
        raise TypeError("cum must be a float32 vector")
    if out is None:
        out = torch.empty(T, dtype=torch.int32, device=cum.device)
    elif not out.is_cuda or out.dtype != torch.int32 or out.numel() < T:
        raise ValueError("out must be a device int32 tensor of at least T elements")
    _check(L.vt_tree_rerank(_ptr(cum), cum.numel(), T, _ptr(out), _stream(cum.device)))
    return out


def draft_tree_level(h: torch.Tensor, W_trim: torch.Tensor, map_: torch.Tensor, m: int, parent_cum: torch.Tensor,
                     K: int, ws: StepWorkspace | None = None, out=None, out_ids: torch.Tensor | None = None,
                     out_logp: torch.Tensor | None = None):
    """Draft step for the frontier rows + the tree expansion on its result, in one call.

    Returns (parent int32 [K], token int32 [K], cum fp32 [K], ids int32 [n,m], logp fp32 [n,m])."""
    L = load_library()
    _require_cuda(h, W_trim, map_, parent_cum)
    n, d = h.shape
    k = W_trim.shape[0]
    if W_trim.shape[1] != d or map_.numel() != k or map_.dtype != torch.int32:
        raise ValueError("shape / dtype mismatch between h, W_trim and map")
    if parent_cum.dtype != torch.float32 or parent_cum.numel() != n:
        raise ValueError("parent_cum must be float32 [n]")
    dev = h.device
    if ws is None:
        ws = StepWorkspace(n, k, d, m, dev)
    if out_ids is None:
        out_ids = torch.empty((n, m), dtype=torch.int32, device=dev)
    if out_logp is None:
        out_logp = torch.empty((n, m), dtype=torch.float32, device=dev)
    if out is not None:
        parent, token, cum = out
    else:
        parent = torch.empty(K, dtype=torch.int32, device=dev)
        token = torch.empty(K, dtype=torch.int32, device=dev)
        cum = torch.empty(K, dtype=torch.float32, device=dev)
    _check(L.vt_draft_tree_level(_ptr(h), _dtype_code(h), n, _ptr(W_trim), _dtype_code(W_trim), k, d, _ptr(map_), m,
                                 _ptr(parent_cum), K, _ptr(parent), _ptr(token), _ptr(cum), _ptr(out_ids),
                                 _ptr(out_logp), _ptr(ws.buf), ws.nbytes, _stream(dev)))
    return parent, token, cum, out_ids, out_logp


# --------------------------------------------------------------------------- measurement reference
def stream_read_reference(t: torch.Tensor, sink: torch.Tensor) -> None:
    """Reads every byte of `t` once on the device (plain streaming read; timing reference only)."""
    L = load_library()
    _require_cuda(t, sink)
    _check(L.vt_stream_read_reference(_ptr(t), t.numel() * t.element_size(), _ptr(sink), _stream(t.device)))
