"""ctypes binding of liblpp.so: argument marshalling only.

Function names and argument order follow include/lpp.h.  Device buffers are
torch tensors on the current HIP device (PyTorch is used for device memory and
streams only); every step of the path runs in the library's kernels.  There is
no fallback: a missing library raises at import of this module's loader.
"""
import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblpp.so")

LPP_OK, LPP_EINVAL, LPP_EUNSUPPORTED, LPP_ENOWORKSPACE, LPP_EHIP = range(5)
LPP_F32, LPP_BF16 = 0, 1


class LppError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().lpp_strerror(status).decode()} (status {status})")


class VerifyOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("accept_len", "path", "final_token", "decision", "ratio", "mass", "n_agg",
                 "q_tok", "p_tok", "final_tok_all")]


_lib = None


def lib() -> C.CDLL:
    """Load liblpp.so (built in-tree by ``python -m paper_2502_06352_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run __graft_entry__.build() "
                          "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
    L.lpp_strerror.restype = C.c_char_p; L.lpp_strerror.argtypes = [i32]
    L.lpp_version.restype = C.c_char_p; L.lpp_version.argtypes = []
    L.lpp_tree_create.restype = i32; L.lpp_tree_create.argtypes = [vp, i32, C.POINTER(vp)]
    L.lpp_tree_destroy.restype = i32; L.lpp_tree_destroy.argtypes = [vp]
    L.lpp_tree_info.restype = i32; L.lpp_tree_info.argtypes = [vp] + [C.POINTER(i32)] * 4
    L.lpp_tree_walk_status.restype = i32; L.lpp_tree_walk_status.argtypes = [vp, C.POINTER(i32)]
    L.lpp_tree_walk_reset.restype = i32; L.lpp_tree_walk_reset.argtypes = [vp, vp]
    L.lpp_tree_set_walk_patience.restype = i32; L.lpp_tree_set_walk_patience.argtypes = [vp, i32]
    L.lpp_build_neighbours_workspace.restype = sz
    L.lpp_build_neighbours_workspace.argtypes = [i32, i32, i32]
    L.lpp_build_neighbours.restype = i32
    L.lpp_build_neighbours.argtypes = [vp, i32, i32, i32, vp, vp, sz, vp]
    L.lpp_tree_attention_workspace.restype = sz
    L.lpp_tree_attention_workspace.argtypes = [vp, i32, i32, i32, i32]
    L.lpp_tree_attention.restype = i32
    L.lpp_tree_attention.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, vp, vp, sz, vp]
    L.lpp_tree_attention_gqa.restype = i32
    L.lpp_tree_attention_gqa.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp, vp, sz, vp]
    L.lpp_tree_attention_layers_workspace.restype = sz
    L.lpp_tree_attention_layers_workspace.argtypes = [vp, i32, i32, i32, i32, i32]
    L.lpp_tree_attention_layers.restype = i32
    L.lpp_tree_attention_layers.argtypes = [vp, i32, i32, vp, i32, vp, i32, i32, i32, i32, i32, f32, vp, sz, vp]
    L.lpp_relaxed_verify_workspace.restype = sz
    L.lpp_relaxed_verify_workspace.argtypes = [vp, i32, i32, i32]
    L.lpp_relaxed_verify.restype = i32
    L.lpp_relaxed_verify.argtypes = [vp, vp, vp, i64, i32, i32, i32, vp, vp, i32, i32, f32, vp, vp,
                                     C.POINTER(VerifyOut), vp, sz, vp]
    L.lpp_relaxed_verify_static.restype = i32
    L.lpp_relaxed_verify_static.argtypes = [vp, vp, vp, i64, i32, i32, i32, vp, vp, i32, i32, f32, vp, vp,
                                            C.POINTER(VerifyOut), vp]
    L.lpp_relaxed_verify_additive.restype = i32
    L.lpp_relaxed_verify_additive.argtypes = L.lpp_relaxed_verify.argtypes
    L.lpp_relaxed_verify_sampled.restype = i32
    L.lpp_relaxed_verify_sampled.argtypes = [vp, vp, vp, f32, i32, vp, i64, i32, i32, i32, vp, vp, i32, i32, f32, vp, vp,
                                             C.POINTER(VerifyOut), vp, sz, vp]
    L.lpp_relaxed_verify_opts.restype = i32
    L.lpp_relaxed_verify_opts.argtypes = [vp, vp, vp, i64, i32, i32, i32, vp, vp, i32, i32, vp, vp, vp,
                                          C.POINTER(VerifyOut), vp, sz, vp]
    L.lpp_commit_kv.restype = i32
    L.lpp_commit_kv.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
    L.lpp_probe_stream_read.restype = i32
    L.lpp_probe_stream_read.argtypes = [vp, sz, vp, i32, vp]
    _lib = L
    return L


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    s = int(getattr(stream, "cuda_stream", stream))
    return s or None


def _check(status: int, where: str) -> None:
    if status != LPP_OK:
        raise LppError(status, where)


class Tree:
    """Owner of an ``lpp_tree*`` (lpp_tree_create / lpp_tree_destroy)."""

    def __init__(self, parent):
        parent = np.ascontiguousarray(parent, dtype=np.int32)
        self.parent = parent
        self.handle = C.c_void_p()
        _check(lib().lpp_tree_create(parent.ctypes.data, len(parent), C.byref(self.handle)), "lpp_tree_create")
        v = [C.c_int32() for _ in range(4)]
        _check(lib().lpp_tree_info(self.handle, *[C.byref(x) for x in v]), "lpp_tree_info")
        self.M, self.depth, self.n_parents, self.max_children = [x.value for x in v]

    def walk_gave_up(self) -> int:
        """Number of walks that gave up since the handle was made or last reset."""
        v = C.c_int32()
        _check(lib().lpp_tree_walk_status(self.handle, C.byref(v)), "lpp_tree_walk_status")
        return int(v.value)

    def walk_reset(self, stream=None) -> None:
        _check(lib().lpp_tree_walk_reset(self.handle, _stream(stream)), "lpp_tree_walk_reset")

    def set_walk_patience(self, rounds: int) -> None:
        _check(lib().lpp_tree_set_walk_patience(self.handle, rounds), "lpp_tree_set_walk_patience")

    def close(self):
        if getattr(self, "handle", None):
            lib().lpp_tree_destroy(self.handle)
            self.handle = None

    __del__ = close


def lpp_build_neighbours_workspace(V: int, D: int, k: int) -> int:
    return int(lib().lpp_build_neighbours_workspace(V, D, k))


def lpp_build_neighbours(E, k: int, neigh, ws, stream=None) -> None:
    V, D = E.shape
    _check(lib().lpp_build_neighbours(_ptr(E), V, D, k, _ptr(neigh), _ptr(ws),
                                      0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "lpp_build_neighbours")


def lpp_tree_attention_workspace(tree: Tree, B: int, H: int, S: int, Dh: int) -> int:
    return int(lib().lpp_tree_attention_workspace(tree.handle, B, H, S, Dh))


def lpp_tree_attention(tree: Tree, dtype: int, q, k_cache, v_cache, k_tree, v_tree, seq_len,
                       B: int, H: int, S: int, Dh: int, scale: float, out, ws, stream=None) -> None:
    _check(lib().lpp_tree_attention(tree.handle, dtype, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree),
                                    _ptr(v_tree), _ptr(seq_len), B, H, S, Dh, scale, _ptr(out), _ptr(ws),
                                    0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "lpp_tree_attention")


def lpp_tree_attention_gqa(tree: Tree, dtype: int, out_dtype: int, q, k_cache, v_cache, k_tree, v_tree, seq_len,
                           B: int, H: int, Hkv: int, S: int, Dh: int, scale: float, out, ws, stream=None) -> None:
    _check(lib().lpp_tree_attention_gqa(tree.handle, dtype, out_dtype, _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                        _ptr(k_tree), _ptr(v_tree), _ptr(seq_len), B, H, Hkv, S, Dh, scale,
                                        _ptr(out), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                        _stream(stream)), "lpp_tree_attention_gqa")


class AttentionLayer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("q", "k_cache", "v_cache", "k_tree", "v_tree", "out")]


def lpp_tree_attention_layers_workspace(tree: Tree, L: int, B: int, H: int, S: int, Dh: int) -> int:
    return int(lib().lpp_tree_attention_layers_workspace(tree.handle, L, B, H, S, Dh))


def lpp_tree_attention_layers(tree: Tree, dtype: int, out_dtype: int, layers, seq_len, B: int, H: int, Hkv: int,
                              S: int, Dh: int, scale: float, ws, stream=None) -> None:
    """``layers``: a sequence of dicts with the tensors q, k_cache, v_cache, k_tree, v_tree, out of one layer each."""
    arr = (AttentionLayer * len(layers))(*[AttentionLayer(**{n: _ptr(y.get(n)) for n, _ in AttentionLayer._fields_})
                                           for y in layers])
    _check(lib().lpp_tree_attention_layers(tree.handle, dtype, out_dtype, arr, len(layers), _ptr(seq_len), B, H, Hkv,
                                           S, Dh, scale, _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                           _stream(stream)), "lpp_tree_attention_layers")


def lpp_relaxed_verify_workspace(tree: Tree, B: int, V: int, k: int) -> int:
    return int(lib().lpp_relaxed_verify_workspace(tree.handle, B, V, k))


def lpp_relaxed_verify(tree: Tree, target_logits, drafter_logits, ldv: int, vocab_offset: int, V: int,
                       B: int, tokens, neigh, kstride: int, k: int, lam: float, u_accept, u_final,
                       out: dict, ws, stream=None) -> None:
    """``out`` maps lpp_verify_out field names to tensors (missing / None = not wanted)."""
    vo = VerifyOut(**{n: _ptr(out.get(n)) for n, _ in VerifyOut._fields_})
    _check(lib().lpp_relaxed_verify(tree.handle, _ptr(target_logits), _ptr(drafter_logits), ldv, vocab_offset,
                                    V, B, _ptr(tokens), _ptr(neigh), kstride, k, lam, _ptr(u_accept),
                                    _ptr(u_final), C.byref(vo), _ptr(ws),
                                    0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "lpp_relaxed_verify")


def lpp_relaxed_verify_static(tree: Tree, target_logits, drafter_logits, ldv: int, vocab_offset: int, V: int,
                              B: int, tokens, neigh, kstride: int, k: int, lam: float, u_accept, u_final,
                              out: dict, stream=None) -> None:
    """As lpp_relaxed_verify, without a workspace: the library's static device array holds the walk words."""
    vo = VerifyOut(**{n: _ptr(out.get(n)) for n, _ in VerifyOut._fields_})
    _check(lib().lpp_relaxed_verify_static(tree.handle, _ptr(target_logits), _ptr(drafter_logits), ldv, vocab_offset,
                                           V, B, _ptr(tokens), _ptr(neigh), kstride, k, lam, _ptr(u_accept),
                                           _ptr(u_final), C.byref(vo), _stream(stream)),
           "lpp_relaxed_verify_static")


def lpp_relaxed_verify_additive(tree: Tree, target_logits, drafter_logits, ldv: int, vocab_offset: int, V: int,
                                B: int, tokens, neigh, kstride: int, k: int, delta: float, u_accept, u_final,
                                out: dict, ws, stream=None) -> None:
    """As lpp_relaxed_verify, under the additive bound ``sum_A r < delta``."""
    vo = VerifyOut(**{n: _ptr(out.get(n)) for n, _ in VerifyOut._fields_})
    _check(lib().lpp_relaxed_verify_additive(tree.handle, _ptr(target_logits), _ptr(drafter_logits), ldv,
                                             vocab_offset, V, B, _ptr(tokens), _ptr(neigh), kstride, k, delta,
                                             _ptr(u_accept), _ptr(u_final), C.byref(vo), _ptr(ws),
                                             0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "lpp_relaxed_verify_additive")


class VerifyOptions(C.Structure):
    _fields_ = [("bound", C.c_int32), ("bound_value", C.c_float), ("rule", C.c_int32), ("siblings", C.c_int32),
                ("uncond_logits", C.c_void_p), ("cfg_scale", C.c_float), ("top_k", C.c_int32)]


LPP_BOUND_MULTIPLICATIVE, LPP_BOUND_ADDITIVE = 0, 1
LPP_RULE_PREFIX, LPP_RULE_SKIP = 0, 1
LPP_SIBLINGS_IID, LPP_SIBLINGS_DISTINCT = 0, 1


def lpp_relaxed_verify_opts(tree: Tree, target_logits, drafter_logits, ldv: int, vocab_offset: int, V: int,
                            B: int, tokens, neigh, kstride: int, k: int, u_accept, u_final, out: dict, ws,
                            stream=None, *, bound: int = 0, bound_value: float = 0.0, rule: int = 0,
                            siblings: int = 0, uncond_logits=None, cfg_scale: float = 0.0, top_k: int = 0) -> None:
    """lpp_relaxed_verify with the bound, the choice of A, the sibling scheme and the front end as options."""
    vo = VerifyOut(**{n: _ptr(out.get(n)) for n, _ in VerifyOut._fields_})
    opts = VerifyOptions(bound, bound_value, rule, siblings, _ptr(uncond_logits), cfg_scale, top_k)
    _check(lib().lpp_relaxed_verify_opts(tree.handle, _ptr(target_logits), _ptr(drafter_logits), ldv, vocab_offset,
                                         V, B, _ptr(tokens), _ptr(neigh), kstride, k, C.byref(opts),
                                         _ptr(u_accept), _ptr(u_final), C.byref(vo), _ptr(ws),
                                         0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "lpp_relaxed_verify_opts")


def lpp_commit_kv(tree: Tree, dtype: int, k_tree, v_tree, path, accept_len, seq_len, B: int, H: int, S: int,
                  Dh: int, k_cache, v_cache, new_len, stream=None) -> None:
    _check(lib().lpp_commit_kv(tree.handle, dtype, _ptr(k_tree), _ptr(v_tree), _ptr(path), _ptr(accept_len),
                               _ptr(seq_len), B, H, S, Dh, _ptr(k_cache), _ptr(v_cache), _ptr(new_len),
                               _stream(stream)), "lpp_commit_kv")


def lpp_relaxed_verify_sampled(tree: Tree, cond_logits, uncond_logits, cfg_scale: float, top_k: int,
                               drafter_logits, ldv: int, vocab_offset: int, V: int, B: int, tokens, neigh,
                               kstride: int, k: int, lam: float, u_accept, u_final, out: dict, ws,
                               stream=None) -> None:
    """As lpp_relaxed_verify, with guidance and top-k applied to the target rows inside the kernel."""
    vo = VerifyOut(**{n: _ptr(out.get(n)) for n, _ in VerifyOut._fields_})
    _check(lib().lpp_relaxed_verify_sampled(tree.handle, _ptr(cond_logits), _ptr(uncond_logits), cfg_scale, top_k,
                                            _ptr(drafter_logits), ldv, vocab_offset, V, B, _ptr(tokens),
                                            _ptr(neigh), kstride, k, lam, _ptr(u_accept), _ptr(u_final),
                                            C.byref(vo), _ptr(ws),
                                            0 if ws is None else ws.numel() * ws.element_size(), _stream(stream)),
           "lpp_relaxed_verify_sampled")


def lpp_probe_stream_read(src, blocks: int, sink=None, stream=None) -> None:
    """Measurement aid: one streaming read of ``src`` (nothing is written)."""
    _check(lib().lpp_probe_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), blocks,
                                       _stream(stream)), "lpp_probe_stream_read")
