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
HS_MAX_TOPK = 64

_c = ctypes
_vp, _i32, _i64, _f32, _sz = _c.c_void_p, _c.c_int32, _c.c_int64, _c.c_float, _c.c_size_t

_SIGNATURES = {
    "hs_status_string": (_c.c_char_p, [_c.c_int]),
    "hs_last_error": (_c.c_char_p, []),
    "hs_version": (_c.c_char_p, []),
    "hs_draft_entropy_topk_workspace": (_sz, [_i32, _i32, _i32]),
    "hs_draft_entropy_topk": (_c.c_int, [_vp, _i64, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "hs_tree_prune_workspace": (_sz, [_i32, _i32]),
    "hs_tree_prune": (_c.c_int, [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "hs_tree_attention_workspace": (_sz, [_i32, _i32, _i64, _i32, _i32, _i32, _c.c_int]),
    "hs_tree_attention": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32,
                                     _c.c_int, _f32, _vp, _vp, _vp, _sz, _vp]),
    "hs_verify_accept_workspace": (_sz, [_i32, _i32, _i32]),
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


def hs_draft_entropy_topk(logits: torch.Tensor, K: int, temperature: float = 1.0, *, want_full: bool = True,
                          out: Optional[Dict[str, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None,
                          stream=None) -> Dict[str, torch.Tensor]:
    """logits float32 [R, V] (row stride may exceed V).  Returns topk_idx, topk_logp, ent_topk, ent_full, lse."""
    if logits.dim() != 2 or logits.dtype != torch.float32 or not logits.is_cuda or logits.stride(1) != 1:
        raise ValueError("logits must be a float32 [R, V] GPU tensor with unit inner stride")
    R, V = logits.shape
    dev = logits.device
    if out is None:
        out = dict(topk_idx=torch.empty((R, K), dtype=torch.int32, device=dev),
                   topk_logp=torch.empty((R, K), dtype=torch.float32, device=dev),
                   ent_topk=torch.empty(R, dtype=torch.float32, device=dev))
        if want_full:
            out["ent_full"] = torch.empty(R, dtype=torch.float32, device=dev)
            out["lse"] = torch.empty(R, dtype=torch.float32, device=dev)
    need = lib().hs_draft_entropy_topk_workspace(R, V, K)
    if ws is None:
        ws = workspace(need, dev)
    st = lib().hs_draft_entropy_topk(_ptr(logits), logits.stride(0) if R > 1 else max(V, logits.stride(0)), R, V, K,
                                     float(temperature), _ptr(out["topk_idx"]), _ptr(out["topk_logp"]),
                                     _ptr(out["ent_topk"]), _ptr(out.get("ent_full")), _ptr(out.get("lse")),
                                     _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "hs_draft_entropy_topk")
    return out


def hs_tree_prune(parent: torch.Tensor, logc: torch.Tensor, node_offsets: torch.Tensor, d_max: torch.Tensor,
                  theta: torch.Tensor, max_nodes: torch.Tensor, *, out: Optional[Dict[str, torch.Tensor]] = None,
                  ws: Optional[torch.Tensor] = None, stream=None) -> Dict[str, torch.Tensor]:
    """All arguments are GPU tensors: parent int32 [NN], logc float32 [NN], node_offsets int32 [B+1],
    d_max int32 [B], theta float32 [B], max_nodes int32 [B].  Returns depth, cumlogp, keep, out_offsets,
    out_src, out_parent (the last two sized NN; the first out_offsets[B] entries are valid)."""
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
    st = lib().hs_tree_prune(_ptr(parent), _ptr(logc), _ptr(node_offsets), B, NN, _ptr(d_max), _ptr(theta),
                             _ptr(max_nodes), _ptr(out["depth"]), _ptr(out["cumlogp"]), _ptr(out["keep"]),
                             _ptr(out["out_offsets"]), _ptr(out["out_src"]), _ptr(out["out_parent"]),
                             _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "hs_tree_prune")
    return out


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return HS_F32
    if t.dtype == torch.bfloat16:
        return HS_BF16
    raise ValueError("q/k/v must be float32 or bfloat16")


def hs_tree_attention(q, k_prefix, v_prefix, k_tree, v_tree, parent, node_offsets, prefix_offsets,
                      host_node_offsets, host_prefix_offsets, scale: float, *, want_lse: bool = False,
                      out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                      ws: Optional[torch.Tensor] = None, stream=None):
    """q [NN,Hq,D]; k_prefix, v_prefix [total_prefix,Hkv,D]; k_tree, v_tree [NN,Hkv,D] (float32 or bfloat16, GPU);
    parent int32 [NN], node_offsets int32 [B+1], prefix_offsets int64 [B+1] on the GPU and the same two offset
    arrays on the host (CPU tensors).  Returns (o [NN,Hq,D], lse [NN,Hq] or None)."""
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
    st = lib().hs_tree_attention(_ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree), _ptr(parent),
                                 _ptr(node_offsets), _ptr(prefix_offsets), _vp(hno.data_ptr()), _vp(hpo.data_ptr()),
                                 B, Hq, Hkv, D, dt, float(scale), _ptr(out), _ptr(lse), _ptr(ws),
                                 0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "hs_tree_attention")
    return out, lse


def hs_verify_accept(target_logits, draft_logits, token, parent, node_offsets, mode: int, temperature: float,
                     uniforms, max_depth: int, *, out: Optional[Dict[str, torch.Tensor]] = None,
                     ws: Optional[torch.Tensor] = None, stream=None) -> Dict[str, torch.Tensor]:
    """target_logits / draft_logits float32 [NN, V] (draft and uniforms may be None when greedy), token and
    parent int32 [NN], node_offsets int32 [B+1], uniforms float32 [NN + B].  Returns accept_len [B],
    accept_path [B, max_depth], bonus_token [B]."""
    _dev(target_logits, torch.float32, "target_logits")
    NN, V = target_logits.shape
    B = node_offsets.numel() - 1
    dev = target_logits.device
    if draft_logits is not None:
        _dev(draft_logits, torch.float32, "draft_logits")
        if draft_logits.shape != target_logits.shape:
            raise ValueError("draft_logits must have the shape of target_logits")
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
    need = lib().hs_verify_accept_workspace(B, NN, V)
    if ws is None:
        ws = workspace(need, dev)
    st = lib().hs_verify_accept(_ptr(target_logits), _ptr(draft_logits), V, _ptr(token), _ptr(parent),
                                _ptr(node_offsets), B, NN, V, int(mode), float(temperature), _ptr(uniforms),
                                int(max_depth), _ptr(out["accept_len"]), _ptr(out["accept_path"]),
                                _ptr(out["bonus_token"]), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "hs_verify_accept")
    return out
