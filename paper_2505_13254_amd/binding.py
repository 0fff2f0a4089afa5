"""ctypes binding of libheterospec.so: argument marshalling only.

Every function has the name and the arguments of the C entry point it calls (see
include/heterospec.h); tensors are torch tensors on the GPU, used purely as device memory.
There is no CPU path: if the library is not built, importing this module's functions raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libheterospec.so")

HS_F32, HS_BF16 = 0, 1
HS_ACCEPT_GREEDY, HS_ACCEPT_STOCHASTIC, HS_ACCEPT_STOCHASTIC_POINTMASS = 0, 1, 2
HS_PSTAR_CUMULATIVE, HS_PSTAR_LOCAL = 0, 1
HS_MAX_TOPK = 64

_c = ctypes
_vp, _i32, _i64, _f32, _sz = _c.c_void_p, _c.c_int32, _c.c_int64, _c.c_float, _c.c_size_t

_SIGNATURES = {
    "hs_status_string": (_c.c_char_p, [_c.c_int]),
    "hs_last_error": (_c.c_char_p, []),
    "hs_version": (_c.c_char_p, []),
    "hs_draft_entropy_topk_workspace": (_sz, [_i32, _i32, _i32]),
    "hs_draft_entropy_topk": (_c.c_int, [_vp, _i64, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "hs_draft_entropy_topk_rows": (_c.c_int, [_vp, _i64, _vp, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                              _vp]),
    "hs_draft_entropy_topk_fused": (_c.c_int, [_vp, _i64, _vp, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                               _vp]),
    "hs_workspace_prepare": (_c.c_int, [_vp, _sz, _vp]),
    "hs_tree_prune_workspace": (_sz, [_i32, _i32]),
    "hs_tree_prune": (_c.c_int, [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "hs_tree_prune_static": (_c.c_int, [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "hs_tree_prune_counted": (_c.c_int, [_vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                         _sz, _vp]),
    "hs_tree_expand": (_c.c_int, [_vp] * 15 + [_i32] * 5 + [_vp]),
    "hs_adaptive_control": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _i32, _vp, _i32, _i32, _i32, _i32,
                                       _c.c_int, _vp, _vp, _vp, _vp, _vp, _vp]),
    "hs_adaptive_policy": (_c.c_int, [_i32, _vp, _i32, _i32, _i32, _i32, _vp, _vp]),
    "hs_tree_attention_workspace": (_sz, [_i32, _i32, _i64, _i32, _i32, _i32, _c.c_int]),
    "hs_tree_attention": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32,
                                     _c.c_int, _f32, _vp, _vp, _vp, _sz, _vp]),
    "hs_tree_attention_shared_tree": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32,
                                                 _i32, _c.c_int, _f32, _vp, _vp, _vp, _sz, _vp]),
    "hs_tree_attention_lens": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32,
                                          _i32, _c.c_int, _f32, _vp, _vp, _vp, _sz, _vp]),
    "hs_tree_attention_paged": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _i32, _i32,
                                           _i32, _i32, _c.c_int, _f32, _vp, _vp, _vp, _sz, _vp]),
    "hs_kv_commit_paged": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _i32, _i32, _vp, _i32, _i32, _i32,
                                      _c.c_int, _vp]),
    "hs_kv_commit": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _c.c_int, _vp]),
    "hs_tree_validate": (_c.c_int, [_vp, _vp, _vp, _i32, _i32, _vp, _vp]),
    "hs_time_next_attention": (_c.c_int, [_vp, _vp]),
    "hs_tree_attention_last_kernel": (_c.c_int32, []),
    "hs_tree_attention_plan": (_c.c_int, [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _c.c_int, _vp, _vp]),
    "hs_verify_accept_workspace": (_sz, [_i32, _i32, _i32]),
    "hs_verify_accept_workspace_mode": (_sz, [_i32, _i32, _i32, _c.c_int]),
    "hs_verify_accept": (_c.c_int, [_vp, _vp, _i64, _vp, _vp, _vp, _i32, _i32, _i32, _c.c_int, _f32, _vp, _i32,
                                    _vp, _vp, _vp, _vp, _sz, _vp]),
}

_lib_handle = None


class HsError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__("%s failed with status %d: %s" % (where, status, detail))
        self.status = status


def lib():
    """The loaded library; raises if it has not been built (there is no fallback)."""
    global _lib_handle
    if _lib_handle is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libheterospec.so is not built: run `python -m paper_2505_13254_amd.build` "
                               "(or __graft_entry__.build()) first")
        h = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(h, name)
            fn.restype, fn.argtypes = res, args
        _lib_handle = h
    return _lib_handle


def exported_symbols():
    return sorted(_SIGNATURES)


def _check(status: int, where: str):
    if status != 0:
        raise HsError(status, where, lib().hs_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else _vp(t.data_ptr())


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError("%s must be a contiguous %s tensor on the GPU" % (name, dtype))
    return t


def _stream(stream) -> _vp:
    s = torch.cuda.current_stream() if stream is None else stream
    return _vp(s.cuda_stream)


def workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    """A 256-byte aligned scratch buffer (torch's allocator aligns to at least 512 bytes)."""
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def hs_workspace_prepare(ws: Optional[torch.Tensor], stream=None) -> None:
    """Clears a workspace tensor on the GPU (what hs_draft_entropy_topk_fused asks of its workspace)."""
    if ws is None:
        return
    _check(lib().hs_workspace_prepare(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "hs_workspace_prepare")


def hs_draft_entropy_topk(logits: torch.Tensor, K: int, temperature: float = 1.0, *, want_full: bool = True,
                          out: Optional[Dict[str, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None,
                          row_index: Optional[torch.Tensor] = None, fused: bool = False,
                          stream=None) -> Dict[str, torch.Tensor]:
    """logits float32 [N, V] (row stride may exceed V).  Returns topk_idx, topk_logp, ent_topk, ent_full, lse
    for its N rows, or, with row_index int32 [R] (GPU), for the R rows that row_index names
    (hs_draft_entropy_topk_rows; a negative entry leaves that result row untouched).
    fused: hs_draft_entropy_topk_fused (one launch); `ws` must then be given and PREPARED
    (hs_workspace_prepare, and only completed fused calls on it since)."""
    if logits.dim() != 2 or logits.dtype != torch.float32 or not logits.is_cuda or logits.stride(1) != 1:
        raise ValueError("logits must be a float32 [R, V] GPU tensor with unit inner stride")
    N, V = logits.shape
    R = N
    if row_index is not None:
        _dev(row_index, torch.int32, "row_index")
        R = row_index.numel()
    dev = logits.device
    if out is None:
        out = dict(topk_idx=torch.empty((R, K), dtype=torch.int32, device=dev),
                   topk_logp=torch.empty((R, K), dtype=torch.float32, device=dev),
                   ent_topk=torch.empty(R, dtype=torch.float32, device=dev))
        if want_full:
            out["ent_full"] = torch.empty(R, dtype=torch.float32, device=dev)
            out["lse"] = torch.empty(R, dtype=torch.float32, device=dev)
    need = lib().hs_draft_entropy_topk_workspace(R, V, K)
    if ws is None and not fused:
        ws = workspace(need, dev)
    stride = logits.stride(0) if N > 1 else max(V, logits.stride(0))
    tail = (_ptr(out["topk_idx"]), _ptr(out["topk_logp"]), _ptr(out["ent_topk"]), _ptr(out.get("ent_full")),
            _ptr(out.get("lse")), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    if fused:
        if ws is None or ws.numel() < need:
            raise ValueError("the fused call needs a prepared workspace of at least %d bytes" % need)
        st = lib().hs_draft_entropy_topk_fused(_ptr(logits), stride, _ptr(row_index), R, V, K, float(temperature), *tail)
    elif row_index is None:
        st = lib().hs_draft_entropy_topk(_ptr(logits), stride, R, V, K, float(temperature), *tail)
    else:
        st = lib().hs_draft_entropy_topk_rows(_ptr(logits), stride, _ptr(row_index), R, V, K, float(temperature), *tail)
    _check(st, "hs_draft_entropy_topk")
    return out


def hs_tree_prune(parent: torch.Tensor, logc: torch.Tensor, node_offsets: torch.Tensor, d_max: torch.Tensor,
                  theta: torch.Tensor, max_nodes: torch.Tensor, *, node_counts: Optional[torch.Tensor] = None,
                  out: Optional[Dict[str, torch.Tensor]] = None,
                  ws: Optional[torch.Tensor] = None, stream=None) -> Dict[str, torch.Tensor]:
    """All arguments are GPU tensors: parent int32 [NN], logc float32 [NN], node_offsets int32 [B+1],
    d_max int32 [B], theta float32 [B], max_nodes int32 [B].  Returns depth, cumlogp, keep, out_offsets,
    out_src, out_parent (the last two sized NN; the first out_offsets[B] entries are valid).
    With node_counts int32 [B] the call is hs_tree_prune_counted (trees stored with spare capacity)."""
    if node_counts is not None:
        _dev(node_counts, torch.int32, "node_counts")
    _dev(parent, torch.int32, "parent"); _dev(logc, torch.float32, "logc")
    _dev(node_offsets, torch.int32, "node_offsets"); _dev(d_max, torch.int32, "d_max")
    _dev(theta, torch.float32, "theta"); _dev(max_nodes, torch.int32, "max_nodes")
    NN, B = parent.numel(), node_offsets.numel() - 1
    dev = parent.device
    if out is None:
        out = dict(depth=torch.empty(NN, dtype=torch.int32, device=dev),
                   cumlogp=torch.empty(NN, dtype=torch.float32, device=dev),
                   keep=torch.empty(NN, dtype=torch.uint8, device=dev),
                   out_offsets=torch.empty(B + 1, dtype=torch.int32, device=dev),
                   out_src=torch.empty(max(NN, 1), dtype=torch.int32, device=dev),
                   out_parent=torch.empty(max(NN, 1), dtype=torch.int32, device=dev))
    need = lib().hs_tree_prune_workspace(B, NN)
    if ws is None:
        ws = workspace(need, dev)
    tail = (_ptr(d_max), _ptr(theta), _ptr(max_nodes), _ptr(out["depth"]), _ptr(out["cumlogp"]), _ptr(out["keep"]),
            _ptr(out["out_offsets"]), _ptr(out["out_src"]), _ptr(out["out_parent"]),
            _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    if node_counts is None:
        st = lib().hs_tree_prune(_ptr(parent), _ptr(logc), _ptr(node_offsets), B, NN, *tail)
    else:
        st = lib().hs_tree_prune_counted(_ptr(parent), _ptr(logc), _ptr(node_offsets), _ptr(node_counts), B, NN, *tail)
    _check(st, "hs_tree_prune")
    return out


def hs_tree_prune_static(parent: torch.Tensor, logc: torch.Tensor, node_offsets: torch.Tensor, d_max: torch.Tensor,
                         theta: torch.Tensor, max_nodes: torch.Tensor, *, out: Dict[str, torch.Tensor],
                         stream=None) -> Dict[str, torch.Tensor]:
    """hs_tree_prune on the library's own static scratch: no workspace, and `out` (depth, cumlogp, keep,
    out_offsets, out_src, out_parent as hs_tree_prune returns them) must be given, so the call allocates
    nothing."""
    _dev(parent, torch.int32, "parent"); _dev(logc, torch.float32, "logc")
    _dev(node_offsets, torch.int32, "node_offsets"); _dev(d_max, torch.int32, "d_max")
    _dev(theta, torch.float32, "theta"); _dev(max_nodes, torch.int32, "max_nodes")
    NN, B = parent.numel(), node_offsets.numel() - 1
    st = lib().hs_tree_prune_static(_ptr(parent), _ptr(logc), _ptr(node_offsets), B, NN, _ptr(d_max), _ptr(theta),
                                    _ptr(max_nodes), _ptr(out["depth"]), _ptr(out["cumlogp"]), _ptr(out["keep"]),
                                    _ptr(out["out_offsets"]), _ptr(out["out_src"]), _ptr(out["out_parent"]),
                                    _stream(stream))
    _check(st, "hs_tree_prune_static")
    return out


def new_tree_state(B: int, cap: int, F: int, device) -> Dict[str, torch.Tensor]:
    """Device arrays of hs_tree_expand's draft-tree state (uninitialised: the first call initialises them)."""
    i32 = dict(dtype=torch.int32, device=device)
    f32 = dict(dtype=torch.float32, device=device)
    return dict(parent=torch.empty(B * cap, **i32), token=torch.empty(B * cap, **i32), depth=torch.empty(B * cap, **i32),
                logc=torch.empty(B * cap, **f32), cumlogp=torch.empty(B * cap, **f32), ent=torch.empty(B * cap, **f32),
                n_nodes=torch.empty(B, **i32), level=torch.empty(B, **i32), frontier=torch.empty(B * F, **i32),
                n_frontier=torch.empty(B, **i32), frontier_rows=torch.empty(B * F, **i32),
                node_offsets=(torch.arange(B + 1, dtype=torch.int64) * cap).to(torch.int32).to(device))


def hs_tree_expand(state: Dict[str, torch.Tensor], topk_idx, topk_logp, ent_topk, d_limit, B: int, cap: int, F: int,
                   K: int, first: bool, *, stream=None) -> Dict[str, torch.Tensor]:
    """state: the tensors of new_tree_state(); topk_idx int32 [B*F, K], topk_logp float32 [B*F, K], ent_topk
    float32 [B*F] (hs_draft_entropy_topk's results for the frontier slots); d_limit int32 [B] or None."""
    _dev(topk_idx, torch.int32, "topk_idx"); _dev(topk_logp, torch.float32, "topk_logp")
    _dev(ent_topk, torch.float32, "ent_topk")
    if topk_idx.numel() < B * F * K or ent_topk.numel() < B * F:
        raise ValueError("Top-K results must cover B * F frontier slots")
    if d_limit is not None:
        _dev(d_limit, torch.int32, "d_limit")
    for k in ("parent", "token", "depth", "n_nodes", "level", "frontier", "n_frontier", "frontier_rows"):
        _dev(state[k], torch.int32, k)
    for k in ("logc", "cumlogp", "ent"):
        _dev(state[k], torch.float32, k)
    if state["parent"].numel() < B * cap or state["frontier"].numel() < B * F:
        raise ValueError("state arrays are smaller than B * cap / B * F")
    st = lib().hs_tree_expand(_ptr(state["parent"]), _ptr(state["token"]), _ptr(state["logc"]), _ptr(state["cumlogp"]),
                              _ptr(state["depth"]), _ptr(state["ent"]), _ptr(state["n_nodes"]), _ptr(state["level"]),
                              _ptr(state["frontier"]), _ptr(state["n_frontier"]), _ptr(state["frontier_rows"]),
                              _ptr(topk_idx), _ptr(topk_logp), _ptr(ent_topk), _ptr(d_limit), B, cap, F, K,
                              1 if first else 0, _stream(stream))
    _check(st, "hs_tree_expand")
    return state


def hs_adaptive_control(parent, logc, ent, node_offsets, node_counts, bin_edges, gamma, alpha: int, d_base: int,
                        n_default: int, mode: int = 0, *, out: Optional[Dict[str, torch.Tensor]] = None,
                        stream=None) -> Dict[str, torch.Tensor]:
    """parent int32 [NN], logc / ent float32 [NN], node_offsets int32 [B+1], node_counts int32 [B] or None (GPU);
    bin_edges (ascending, n_bins - 1 values) and gamma are host sequences of floats.
    Returns phi float32 [B] and pstar, bin, d_prime, n_prime int32 [B]."""
    _dev(parent, torch.int32, "parent"); _dev(logc, torch.float32, "logc"); _dev(ent, torch.float32, "ent")
    _dev(node_offsets, torch.int32, "node_offsets")
    if node_counts is not None:
        _dev(node_counts, torch.int32, "node_counts")
    B, NN = node_offsets.numel() - 1, parent.numel()
    dev = parent.device
    edges = (_f32 * max(1, len(bin_edges)))(*[float(x) for x in bin_edges])
    gam = (_f32 * max(1, len(gamma)))(*[float(x) for x in gamma])
    if out is None:
        out = dict(phi=torch.empty(B, dtype=torch.float32, device=dev))
        for k in ("pstar", "bin", "d_prime", "n_prime"):
            out[k] = torch.empty(B, dtype=torch.int32, device=dev)
    st = lib().hs_adaptive_control(_ptr(parent), _ptr(logc), _ptr(ent), _ptr(node_offsets), _ptr(node_counts), B, NN,
                                   _c.cast(edges, _vp), len(bin_edges) + 1, _c.cast(gam, _vp), len(gamma), int(alpha),
                                   int(d_base), int(n_default), int(mode), _ptr(out["phi"]), _ptr(out["pstar"]),
                                   _ptr(out["bin"]), _ptr(out["d_prime"]), _ptr(out["n_prime"]), _stream(stream))
    _check(st, "hs_adaptive_control")
    return out


def hs_adaptive_policy(bin: int, gamma, alpha: int, d_base: int, n_default: int):
    """(d_prime, n_prime) of entropy bin `bin`, from the library's own formula (host arithmetic only)."""
    gam = (_f32 * max(1, len(gamma)))(*[float(x) for x in gamma])
    dp, np_ = _i32(0), _i32(0)
    st = lib().hs_adaptive_policy(int(bin), _c.cast(gam, _vp), len(gamma), int(alpha), int(d_base), int(n_default),
                                  _c.byref(dp), _c.byref(np_))
    _check(st, "hs_adaptive_policy")
    return int(dp.value), int(np_.value)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return HS_F32
    if t.dtype == torch.bfloat16:
        return HS_BF16
    raise ValueError("q/k/v must be float32 or bfloat16")


def hs_tree_attention(q, k_prefix, v_prefix, k_tree, v_tree, parent, node_offsets, prefix_offsets,
                      host_node_offsets, host_prefix_offsets, scale: float, *, want_lse: bool = False,
                      out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                      ws: Optional[torch.Tensor] = None, stream=None,
                      prefix_lens: Optional[torch.Tensor] = None, host_prefix_lens: Optional[torch.Tensor] = None,
                      shared_tree: bool = False):
    """q [NN,Hq,D]; k_prefix, v_prefix [total_prefix,Hkv,D]; k_tree, v_tree [NN,Hkv,D] (float32 or bfloat16, GPU);
    parent int32 [NN], node_offsets int32 [B+1], prefix_offsets int64 [B+1] on the GPU and the same two offset
    arrays on the host (CPU tensors).  Returns (o [NN,Hq,D], lse [NN,Hq] or None).
    With prefix_lens (int64 [B], GPU) and host_prefix_lens (the same on the CPU) the call is
    hs_tree_attention_lens: prefix_offsets then delimit cache regions with spare capacity.
    shared_tree: the call is hs_tree_attention_shared_tree: parent int32 [M] is one tree that all B entries
    (of M rows each) use."""
    dt = _dtype_code(q)
    for name, t in (("q", q), ("k_prefix", k_prefix), ("v_prefix", v_prefix), ("k_tree", k_tree), ("v_tree", v_tree)):
        _dev(t, q.dtype, name)
    _dev(parent, torch.int32, "parent"); _dev(node_offsets, torch.int32, "node_offsets")
    _dev(prefix_offsets, torch.int64, "prefix_offsets")
    hno = host_node_offsets.to(dtype=torch.int32, device="cpu").contiguous()
    hpo = host_prefix_offsets.to(dtype=torch.int64, device="cpu").contiguous()
    NN, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    B = hno.numel() - 1
    dev = q.device
    if out is None:
        out = torch.empty_like(q)
    if want_lse and lse is None:
        lse = torch.empty((NN, Hq), dtype=torch.float32, device=dev)
    need = lib().hs_tree_attention_workspace(B, NN, int(hpo[-1]), Hq, Hkv, D, dt)
    if ws is None:
        ws = workspace(need, dev)
    head = (_ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree), _ptr(parent),
            _ptr(node_offsets), _ptr(prefix_offsets), _vp(hno.data_ptr()), _vp(hpo.data_ptr()))
    tail = (B, Hq, Hkv, D, dt, float(scale), _ptr(out), _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel(),
            _stream(stream))
    if shared_tree:
        if prefix_lens is not None:
            raise ValueError("shared_tree and prefix_lens cannot be combined")
        st = lib().hs_tree_attention_shared_tree(*head, *tail)
    elif prefix_lens is None:
        st = lib().hs_tree_attention(*head, *tail)
    else:
        _dev(prefix_lens, torch.int64, "prefix_lens")
        hl = host_prefix_lens.to(dtype=torch.int64, device="cpu").contiguous()
        st = lib().hs_tree_attention_lens(*head, _ptr(prefix_lens), _vp(hl.data_ptr()), *tail)
    _check(st, "hs_tree_attention")
    return out, lse


def hs_tree_attention_paged(q, k_pages, v_pages, k_tree, v_tree, parent, node_offsets, host_node_offsets, block_table,
                            prefix_lens, host_prefix_lens, scale: float, *, want_lse: bool = False,
                            out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                            ws: Optional[torch.Tensor] = None, stream=None):
    """q [NN,Hq,D]; k_pages, v_pages [n_pages, page_tokens, Hkv, D]; k_tree, v_tree [NN,Hkv,D]; parent int32 [NN],
    node_offsets int32 [B+1], block_table int32 [B, max_blocks], prefix_lens int64 [B] on the GPU;
    host_node_offsets and host_prefix_lens the same on the CPU.  Returns (o, lse or None)."""
    dt = _dtype_code(q)
    for name, t in (("q", q), ("k_pages", k_pages), ("v_pages", v_pages), ("k_tree", k_tree), ("v_tree", v_tree)):
        _dev(t, q.dtype, name)
    _dev(parent, torch.int32, "parent"); _dev(node_offsets, torch.int32, "node_offsets")
    _dev(block_table, torch.int32, "block_table"); _dev(prefix_lens, torch.int64, "prefix_lens")
    hno = host_node_offsets.to(dtype=torch.int32, device="cpu").contiguous()
    hl = host_prefix_lens.to(dtype=torch.int64, device="cpu").contiguous()
    NN, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    B = hno.numel() - 1
    if block_table.dim() != 2 or block_table.shape[0] != B or k_pages.dim() != 4:
        raise ValueError("block_table must be [B, max_blocks] and the pools [n_pages, page_tokens, Hkv, D]")
    dev = q.device
    if out is None:
        out = torch.empty_like(q)
    if want_lse and lse is None:
        lse = torch.empty((NN, Hq), dtype=torch.float32, device=dev)
    need = lib().hs_tree_attention_workspace(B, NN, int(hl.sum()), Hq, Hkv, D, dt)
    if ws is None:
        ws = workspace(need, dev)
    st = lib().hs_tree_attention_paged(_ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(k_tree), _ptr(v_tree), _ptr(parent),
                                       _ptr(node_offsets), _vp(hno.data_ptr()), _ptr(block_table), block_table.shape[1],
                                       k_pages.shape[1], _ptr(prefix_lens), _vp(hl.data_ptr()), B, Hq, Hkv, D, dt,
                                       float(scale), _ptr(out), _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel(),
                                       _stream(stream))
    _check(st, "hs_tree_attention_paged")
    return out, lse


def hs_kv_commit_paged(k_tree, v_tree, node_offsets, accept_path, accept_len, k_pages, v_pages, block_table, cache_lens,
                       *, stream=None):
    """As hs_kv_commit, into pools k_pages, v_pages [n_pages, page_tokens, Hkv, D] through block_table int32
    [B, max_blocks]; cache_lens int64 [B] is updated in place."""
    dt = _dtype_code(k_tree)
    for name, t in (("k_tree", k_tree), ("v_tree", v_tree), ("k_pages", k_pages), ("v_pages", v_pages)):
        _dev(t, k_tree.dtype, name)
    _dev(node_offsets, torch.int32, "node_offsets"); _dev(accept_path, torch.int32, "accept_path")
    _dev(accept_len, torch.int32, "accept_len"); _dev(block_table, torch.int32, "block_table")
    _dev(cache_lens, torch.int64, "cache_lens")
    B = node_offsets.numel() - 1
    Hkv, D = k_tree.shape[1], k_tree.shape[2]
    st = lib().hs_kv_commit_paged(_ptr(k_tree), _ptr(v_tree), _ptr(node_offsets), _ptr(accept_path), _ptr(accept_len),
                                  accept_path.shape[1], _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                  block_table.shape[1], k_pages.shape[1], _ptr(cache_lens), B, Hkv, D, dt, _stream(stream))
    _check(st, "hs_kv_commit_paged")
    return cache_lens


def hs_kv_commit(k_tree, v_tree, node_offsets, accept_path, accept_len, k_cache, v_cache, cache_offsets, cache_lens,
                 *, stream=None):
    """k_tree, v_tree [NN,Hkv,D] and k_cache, v_cache [capacity,Hkv,D] of one element type; node_offsets int32
    [B+1], accept_path int32 [B,max_depth], accept_len int32 [B], cache_offsets int64 [B+1], cache_lens int64
    [B] (updated in place); all on the GPU."""
    dt = _dtype_code(k_tree)
    for name, t in (("k_tree", k_tree), ("v_tree", v_tree), ("k_cache", k_cache), ("v_cache", v_cache)):
        _dev(t, k_tree.dtype, name)
    _dev(node_offsets, torch.int32, "node_offsets"); _dev(accept_path, torch.int32, "accept_path")
    _dev(accept_len, torch.int32, "accept_len"); _dev(cache_offsets, torch.int64, "cache_offsets")
    _dev(cache_lens, torch.int64, "cache_lens")
    B = node_offsets.numel() - 1
    if accept_path.dim() != 2 or accept_path.shape[0] != B or accept_len.numel() != B or cache_lens.numel() != B:
        raise ValueError("accept_path must be [B, max_depth]; accept_len and cache_lens [B]")
    Hkv, D = k_tree.shape[1], k_tree.shape[2]
    st = lib().hs_kv_commit(_ptr(k_tree), _ptr(v_tree), _ptr(node_offsets), _ptr(accept_path), _ptr(accept_len),
                            accept_path.shape[1], _ptr(k_cache), _ptr(v_cache), _ptr(cache_offsets), _ptr(cache_lens),
                            B, Hkv, D, dt, _stream(stream))
    _check(st, "hs_kv_commit")
    return cache_lens


def hs_verify_accept(target_logits, draft_logits, token, parent, node_offsets, mode: int, temperature: float,
                     uniforms, max_depth: int, *, out: Optional[Dict[str, torch.Tensor]] = None,
                     ws: Optional[torch.Tensor] = None, stream=None) -> Dict[str, torch.Tensor]:
    """target_logits / draft_logits float32 [NN, V] (draft and uniforms may be None when greedy; rows may be
    padded: unit stride along the vocabulary, the same row stride in both), token and parent int32 [NN],
    node_offsets int32 [B+1], uniforms float32 [NN + B].  Returns accept_len [B], accept_path [B, max_depth],
    bonus_token [B]."""
    def rows(t, name):
        if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("%s must be a float32 [NN, V] GPU tensor with unit stride along V" % name)
        return t.stride(0) if t.shape[0] > 1 else t.shape[1]
    row_stride = rows(target_logits, "target_logits")
    NN, V = target_logits.shape
    B = node_offsets.numel() - 1
    dev = target_logits.device
    if draft_logits is not None:
        if draft_logits.shape != target_logits.shape or rows(draft_logits, "draft_logits") != row_stride:
            raise ValueError("draft_logits must have the shape and row stride of target_logits")
    if uniforms is not None:
        _dev(uniforms, torch.float32, "uniforms")
        if uniforms.numel() != NN + B:
            raise ValueError("uniforms must hold NN + B values")
    _dev(token, torch.int32, "token"); _dev(parent, torch.int32, "parent")
    _dev(node_offsets, torch.int32, "node_offsets")
    if out is None:
        out = dict(accept_len=torch.empty(B, dtype=torch.int32, device=dev),
                   accept_path=torch.empty((B, max_depth), dtype=torch.int32, device=dev),
                   bonus_token=torch.empty(B, dtype=torch.int32, device=dev))
    need = lib().hs_verify_accept_workspace_mode(B, NN, V, int(mode))
    if ws is None:
        ws = workspace(need, dev)
    st = lib().hs_verify_accept(_ptr(target_logits), _ptr(draft_logits), row_stride, _ptr(token), _ptr(parent),
                                _ptr(node_offsets), B, NN, V, int(mode), float(temperature), _ptr(uniforms),
                                int(max_depth), _ptr(out["accept_len"]), _ptr(out["accept_path"]),
                                _ptr(out["bonus_token"]), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "hs_verify_accept")
    return out


def hs_time_next_attention(start_event, stop_event) -> None:
    """start_event, stop_event: torch.cuda.Event(enable_timing=True) that have been recorded at least once
    (torch creates the HIP event at the first record), or both None.  The next tree-attention call of this
    thread attaches them to its attention kernel; start_event.elapsed_time(stop_event) is then the
    kernel's own duration."""
    if start_event is None and stop_event is None:
        _check(lib().hs_time_next_attention(None, None), "hs_time_next_attention")
        return
    h0, h1 = start_event.cuda_event, stop_event.cuda_event
    if not h0 or not h1:
        raise ValueError("hs_time_next_attention: record each event once before handing it over")
    _check(lib().hs_time_next_attention(_c.c_void_p(h0), _c.c_void_p(h1)), "hs_time_next_attention")


def hs_tree_attention_plan(host_node_offsets, host_prefix_offsets, Hq, Hkv, D, dtype, *, host_prefix_lens=None,
                           paged=False, max_blocks=0):
    """Host only.  host_node_offsets int32 [B+1], host_prefix_offsets int64 [B+1] (None when paged),
    host_prefix_lens int64 [B] or None: CPU tensors.  Returns (totals int64 [6], per_seq int32 [B,4]) as the
    header describes them."""
    B = host_node_offsets.numel() - 1
    totals = torch.zeros(6, dtype=torch.int64)
    per_seq = torch.zeros(max(B, 1), 4, dtype=torch.int32)
    hp = None if host_prefix_offsets is None else host_prefix_offsets.data_ptr()
    hl = None if host_prefix_lens is None else host_prefix_lens.data_ptr()
    _check(lib().hs_tree_attention_plan(host_node_offsets.data_ptr(), hp, hl, 1 if paged else 0, int(max_blocks), B,
                                        int(Hq), int(Hkv), int(D), int(dtype), totals.data_ptr(), per_seq.data_ptr()),
           "hs_tree_attention_plan")
    return totals, per_seq[:B]


def hs_tree_attention_last_kernel() -> int:
    """1: this thread's last tree-attention call ran on the matrix cores, 2: on the vector ALUs, 0: it launched nothing."""
    return int(lib().hs_tree_attention_last_kernel())


def hs_tree_validate(parent, token, node_offsets, *, stream=None) -> torch.Tensor:
    """parent int32 [NN], token int32 [NN] or None, node_offsets int32 [B+1] (GPU).  Returns the device
    report int32 [2]: number of offending rows, global index of the first (-1 if none)."""
    _dev(parent, torch.int32, "parent"); _dev(node_offsets, torch.int32, "node_offsets")
    if token is not None:
        _dev(token, torch.int32, "token")
    report = torch.empty(2, dtype=torch.int32, device=parent.device)
    st = lib().hs_tree_validate(_ptr(parent), _ptr(token), _ptr(node_offsets), node_offsets.numel() - 1,
                                parent.numel(), _ptr(report), _stream(stream))
    _check(st, "hs_tree_validate")
    return report
