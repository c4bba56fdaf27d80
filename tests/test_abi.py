"""Host-only checks of the C ABI: the library loads, exports every function include/lpp.h
declares, and validates its arguments before anything is enqueued (no kernel runs here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2502_06352_amd as lpp
from paper_2502_06352_amd.binding import VerifyOut

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000          # a non-null pointer value that validation never dereferences


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(lpp.LIB_PATH):
        from paper_2502_06352_amd.build import build_library
        build_library(verbose=False)
    return lpp.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lpp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lpp_[a-z_]+)\s*\(", text)))


def test_every_declared_function_is_exported(L):
    names = declared_functions()
    assert {"lpp_build_neighbours", "lpp_tree_attention", "lpp_relaxed_verify", "lpp_tree_create",
            "lpp_tree_destroy", "lpp_tree_info", "lpp_strerror", "lpp_version",
            "lpp_build_neighbours_workspace", "lpp_tree_attention_workspace",
            "lpp_relaxed_verify_workspace"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"{n} is declared in lpp.h but not exported by liblpp.so"
    assert L.lpp_version().decode().startswith("lpp")
    assert [L.lpp_strerror(i).decode() for i in range(5)] == [
        "ok", "invalid argument", "unsupported size or type", "workspace missing or too small",
        "HIP runtime error (or no device)"]
    assert L.lpp_strerror(99).decode() == "unknown status"


def test_walk_state_calls_validate(L):
    t = lpp.Tree([-1, 0, 0, 1])
    v = C.c_int32(7)
    assert L.lpp_tree_walk_status(None, C.byref(v)) == lpp.LPP_EINVAL
    assert L.lpp_tree_walk_status(t.handle, None) == lpp.LPP_EINVAL
    assert L.lpp_tree_walk_reset(None, None) == lpp.LPP_EINVAL
    assert L.lpp_tree_set_walk_patience(None, 5) == lpp.LPP_EINVAL
    assert L.lpp_tree_set_walk_patience(t.handle, -2) == lpp.LPP_EINVAL
    assert L.lpp_tree_set_walk_patience(t.handle, 1 << 30) == lpp.LPP_OK      # (capped)
    import torch
    if not torch.cuda.is_available():                                          # host-only handle
        assert L.lpp_tree_walk_status(t.handle, C.byref(v)) == lpp.LPP_EHIP and v.value == 0
        assert L.lpp_tree_walk_reset(t.handle, None) == lpp.LPP_EHIP


def _create(L, parent):
    parent = np.asarray(parent, dtype=np.int32)
    h = C.c_void_p()
    st = L.lpp_tree_create(parent.ctypes.data if len(parent) else None, len(parent), C.byref(h))
    return st, h


def test_tree_validation_and_info(L):
    for bad in ([], [0], [-1, 1], [-1, 0, 2], [-1, -1]):
        st, h = _create(L, bad)
        assert st == lpp.LPP_EINVAL and not h.value, bad
    st, h = _create(L, [-1] + [0] * 256)                       # M = 257 > LPP_MAX_ROWS
    assert st == lpp.LPP_EINVAL
    assert L.lpp_tree_create(None, 3, C.byref(C.c_void_p())) == lpp.LPP_EINVAL
    t = lpp.Tree([-1, 0, 0, 1, 1, 1, 2])
    assert (t.M, t.depth, t.n_parents, t.max_children) == (7, 2, 3, 3)
    assert L.lpp_tree_info(None, None, None, None, None) == lpp.LPP_EINVAL
    assert L.lpp_tree_destroy(None) == lpp.LPP_OK


def test_workspace_queries(L):
    t = lpp.Tree([-1, 0, 0, 1])
    assert lpp.lpp_relaxed_verify_workspace(t, 4, 1024, 16) >= 2 * 4 * 4 * 4
    assert L.lpp_relaxed_verify_workspace(None, 4, 1024, 16) == 0
    assert lpp.lpp_tree_attention_workspace(t, 2, 4, 1024, 64) > 0
    assert lpp.lpp_tree_attention_workspace(t, 2, 4, 1024, 96) == 0      # unsupported head dim
    assert lpp.lpp_build_neighbours_workspace(1024, 8, 16) > 1024 * 16 * 4
    for V, D, k in ((0, 8, 1), (16, 0, 1), (16, 8, 0), (16, 8, 17), (16, 300, 4), (1 << 17, 8, 4), (8192, 8, 5000)):
        assert lpp.lpp_build_neighbours_workspace(V, D, k) == 0


def test_verify_argument_validation_without_a_kernel(L):
    t = lpp.Tree([-1, 0, 0, 1])
    out = VerifyOut(accept_len=FAKE, path=FAKE, final_token=FAKE)
    big = 1 << 20

    def call(target=FAKE, drafter=FAKE, ldv=1024, off=0, V=1024, B=1, tokens=FAKE, neigh=FAKE, kstride=16, k=16,
             lam=2.0, ua=FAKE, uf=FAKE, o=out, ws=FAKE, wsb=big, tree=t):
        return L.lpp_relaxed_verify(tree.handle if tree else None, target, drafter, ldv, off, V, B, tokens, neigh,
                                    kstride, k, lam, ua, uf, C.byref(o) if o is not None else None, ws, wsb, None)

    assert call(tree=None) == lpp.LPP_EINVAL
    for kw in (dict(target=None), dict(drafter=None), dict(tokens=None), dict(neigh=None), dict(ua=None),
               dict(uf=None), dict(o=None), dict(B=0), dict(V=0), dict(k=0), dict(k=17), dict(k=2000, kstride=2000),
               dict(off=-1), dict(off=1), dict(lam=float("nan")), dict(o=VerifyOut(path=FAKE, final_token=FAKE))):
        assert call(**kw) == lpp.LPP_EINVAL, kw
    assert call(V=40000, ldv=40000) == lpp.LPP_EUNSUPPORTED
    assert call(ws=None) == lpp.LPP_ENOWORKSPACE
    assert call(wsb=8) == lpp.LPP_ENOWORKSPACE
    # everything valid: the only thing missing is a device (or, on a GPU machine, this would enqueue work
    # on fake pointers -- so the call is only made where there is no device)
    import torch
    if not torch.cuda.is_available():
        assert call() == lpp.LPP_EHIP


def test_attention_and_neighbour_argument_validation(L):
    t = lpp.Tree([-1, 0, 0, 1])
    big = 1 << 26

    def attn(tree=t, dtype=lpp.LPP_BF16, q=FAKE, kc=FAKE, vc=FAKE, kt=FAKE, vt=FAKE, B=1, H=2, S=64, Dh=64,
             scale=0.0, out=FAKE, ws=FAKE, wsb=big):
        return L.lpp_tree_attention(tree.handle if tree else None, dtype, q, kc, vc, kt, vt, None, B, H, S, Dh,
                                    scale, out, ws, wsb, None)

    for kw in (dict(tree=None), dict(q=None), dict(kt=None), dict(vt=None), dict(out=None), dict(kc=None),
               dict(vc=None), dict(B=0), dict(H=0), dict(S=-1), dict(Dh=0), dict(scale=float("nan")),
               dict(scale=-1.0), dict(scale=float("inf"))):
        assert attn(**kw) == lpp.LPP_EINVAL, kw
    assert attn(Dh=96) == lpp.LPP_EUNSUPPORTED
    assert attn(dtype=7) == lpp.LPP_EUNSUPPORTED
    assert attn(ws=None) == lpp.LPP_ENOWORKSPACE
    assert attn(wsb=16) == lpp.LPP_ENOWORKSPACE

    def knn(E=FAKE, V=64, D=8, k=4, neigh=FAKE, ws=FAKE, wsb=big):
        return L.lpp_build_neighbours(E, V, D, k, neigh, ws, wsb, None)

    for kw in (dict(E=None), dict(neigh=None), dict(V=0), dict(D=0), dict(k=0), dict(k=65)):
        assert knn(**kw) == lpp.LPP_EINVAL, kw
    for kw in (dict(D=300), dict(V=1 << 17), dict(V=8192, k=5000)):
        assert knn(**kw) == lpp.LPP_EUNSUPPORTED, kw
    assert knn(ws=None) == lpp.LPP_ENOWORKSPACE
    assert knn(wsb=16) == lpp.LPP_ENOWORKSPACE
    import torch
    if not torch.cuda.is_available():
        assert attn() == lpp.LPP_EHIP
        assert knn() == lpp.LPP_EHIP


def test_variant_entry_points_validate_like_the_plain_ones(L):
    from paper_2502_06352_amd.binding import VerifyOptions
    t = lpp.Tree([-1, 0, 0, 1])
    out = VerifyOut(accept_len=FAKE, path=FAKE, final_token=FAKE)
    big = 1 << 20

    def opts_call(opts, k=16, V=1024):
        return L.lpp_relaxed_verify_opts(t.handle, FAKE, FAKE, 8192, 0, V, 1, FAKE, FAKE, 8192, k,
                                         C.byref(opts) if opts is not None else None, FAKE, FAKE, C.byref(out),
                                         FAKE, big, None)

    good = dict(bound=0, bound_value=2.0, rule=0, siblings=0, uncond_logits=None, cfg_scale=0.0, top_k=0)
    assert opts_call(None) == lpp.LPP_EINVAL
    for bad in (dict(bound=2), dict(rule=-1), dict(rule=2), dict(siblings=3), dict(top_k=-1),
                dict(cfg_scale=float("nan")), dict(bound_value=float("nan"))):
        assert opts_call(VerifyOptions(**{**good, **bad})) == lpp.LPP_EINVAL, bad
    assert opts_call(VerifyOptions(**good), k=1025) == lpp.LPP_EINVAL            # k > V
    assert opts_call(VerifyOptions(**good), k=4097, V=8192) == lpp.LPP_EUNSUPPORTED   # k > LPP_MAX_K

    def static_call(tree=t, target=FAKE, B=1, k=16, lam=2.0, o=out):
        return L.lpp_relaxed_verify_static(tree.handle if tree else None, target, FAKE, 1024, 0, 1024, B, FAKE, FAKE,
                                           16, k, lam, FAKE, FAKE, C.byref(o) if o is not None else None, None)

    for kw in (dict(tree=None), dict(target=None), dict(B=0), dict(k=17), dict(lam=float("nan")), dict(o=None)):
        assert static_call(**kw) == lpp.LPP_EINVAL, kw
    assert static_call(B=65536 // 4 + 1) == lpp.LPP_EUNSUPPORTED       # B * M beyond the static array
    import torch
    if not torch.cuda.is_available():
        assert static_call() == lpp.LPP_EHIP

    def gqa(H=4, Hkv=2, out_dtype=lpp.LPP_F32, dtype=lpp.LPP_BF16):
        return L.lpp_tree_attention_gqa(t.handle, dtype, out_dtype, FAKE, FAKE, FAKE, FAKE, FAKE, None, 1, H, Hkv,
                                        64, 64, 0.0, FAKE, FAKE, 1 << 26, None)

    for kw in (dict(Hkv=0), dict(Hkv=3), dict(Hkv=8)):
        assert gqa(**kw) == lpp.LPP_EINVAL, kw
    assert gqa(out_dtype=5) == lpp.LPP_EUNSUPPORTED

    assert L.lpp_commit_kv(t.handle, lpp.LPP_BF16, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 64, 64, FAKE, FAKE, FAKE,
                           None) == lpp.LPP_EINVAL                     # new_len must not be seq_len itself
    assert L.lpp_commit_kv(t.handle, 9, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 64, 64, FAKE, FAKE, None,
                           None) == lpp.LPP_EUNSUPPORTED
    assert L.lpp_commit_kv(None, lpp.LPP_BF16, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 2, 64, 64, FAKE, FAKE, None,
                           None) == lpp.LPP_EINVAL
