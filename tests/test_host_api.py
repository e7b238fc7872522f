"""Host-side checks that need no GPU: the C-ABI library loads, exports what the header
declares, and rejects bad arguments before launching anything; the input generator is pinned."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2204_00595_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2204_00595_amd import build
        build.build()
    return b


def test_library_exports_every_declared_symbol(binding):
    header = open(os.path.join(ROOT, "include", "monarch.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(monarch_[a-z_0-9]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_status_strings(binding):
    assert binding.monarch_version() >= 100
    seen = set()
    for code in (0, -1, -2, -3, -4):
        sname = binding.monarch_status_string(code)
        assert sname and sname != "unknown status"
        seen.add(sname)
    assert len(seen) == 5
    assert binding.monarch_status_string(-99) == "unknown status"


def test_forward_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    ok_ptr = 4096  # never dereferenced: validation fails first or batch == 0 returns early
    args = dict(batch=0, n_in=768, k=4, q=192, s=192, dtype=1)

    def call(x=ok_ptr, R=ok_ptr, Lp=ok_ptr, y=ok_ptr, flags=0, **kw):
        a = dict(args, **kw)
        return L.monarch_fwd_ex(x, R, Lp, y, a["batch"], a["n_in"], a["k"], a["q"], a["s"], a["dtype"], None, flags)

    assert call() == binding.MONARCH_OK                      # empty batch: no-op
    assert call(x=None, y=None) == binding.MONARCH_OK        # ... and then x, y may be NULL
    assert call(x=None, batch=1) == binding.MONARCH_ERR_INVALID
    assert call(R=None) == binding.MONARCH_ERR_INVALID
    assert call(Lp=None) == binding.MONARCH_ERR_INVALID
    assert call(y=None, batch=1) == binding.MONARCH_ERR_INVALID
    assert call(x=4098) == binding.MONARCH_ERR_INVALID       # misaligned
    assert call(batch=-1) == binding.MONARCH_ERR_INVALID
    assert call(n_in=770) == binding.MONARCH_ERR_INVALID     # n_in % k != 0
    for key in ("n_in", "k", "q", "s"):
        assert call(**{key: 0}) == binding.MONARCH_ERR_INVALID
        assert call(**{key: -3}) == binding.MONARCH_ERR_INVALID
    assert call(dtype=7) == binding.MONARCH_ERR_INVALID
    assert call(flags=64) == binding.MONARCH_ERR_INVALID
    assert call(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID
    assert call(flags=binding.MONARCH_FLAG_WS_PACKED) == binding.MONARCH_ERR_INVALID   # no workspace to reuse
    # a row far too wide for any kernel of this build
    assert call(n_in=4 * 2000000, q=2000000, s=4) == binding.MONARCH_ERR_UNSUPPORTED
    assert L.monarch_fwd(ok_ptr, ok_ptr, ok_ptr, ok_ptr, 0, 768, 4, 192, 192, 1, None) == binding.MONARCH_OK


def test_forward_with_workspace_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced
    need = binding.monarch_fwd_workspace_bytes(0, 768, 4, 192, 192, 1)
    assert need == 2 * 2 * 4 * 192 * 192                       # packed copies of R and L
    assert binding.monarch_fwd_workspace_bytes(0, 4096, 64, 64, 64, 1) == 2 * 2 * 64 ** 3   # m = 64: packed R and L
    assert binding.monarch_fwd_workspace_bytes(0, 6, 2, 4, 2, 0) == 0        # shape without a packed-weight kernel
    assert binding.monarch_fwd_workspace_bytes(0, 768, 4, 192, 192, 1, binding.MONARCH_FLAG_GENERIC) == 0
    assert binding.monarch_fwd_workspace_bytes(0, 770, 4, 192, 192, 1) == 0  # invalid arguments

    def call(x=p, R=p, Lp=p, y=p, ws=p, ws_bytes=need, flags=0, batch=0, n_in=768, k=4, q=192, s=192, dtype=1):
        return L.monarch_fwd_ws(x, R, Lp, y, batch, n_in, k, q, s, dtype, None, ws, ws_bytes, flags)

    assert call() == binding.MONARCH_OK
    assert call(ws=None) == binding.MONARCH_ERR_WORKSPACE
    assert call(ws_bytes=need - 1) == binding.MONARCH_ERR_WORKSPACE
    assert call(ws=p + 16) == binding.MONARCH_ERR_WORKSPACE     # not 256-byte aligned
    assert call(R=None) == binding.MONARCH_ERR_INVALID
    assert call(x=None, batch=1) == binding.MONARCH_ERR_INVALID
    assert call(n_in=770) == binding.MONARCH_ERR_INVALID
    assert call(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID
    assert call(flags=binding.MONARCH_FLAG_WS_PACKED) == binding.MONARCH_OK
    assert call(flags=binding.MONARCH_FLAG_WS_PACKED, ws=None) == binding.MONARCH_ERR_WORKSPACE
    # fp32 layers with square blocks of 32 / 64: the vector between the factors goes through the workspace, in whole 32-row tiles
    fneed = binding.monarch_fwd_workspace_bytes(33, 3 * 64, 3, 64, 64, 0)
    assert fneed == 2 * 32 * 3 * 64 * 4
    assert binding.monarch_fwd_t_workspace_bytes(33, 3 * 64, 3, 64, 64, 0, 0) == fneed
    assert binding.monarch_bwd_workspace_bytes(33, 3 * 64, 3, 64, 64, 0, 0) >= 3 * fneed
    assert binding.monarch_fwd_workspace_bytes(33, 3 * 64, 3, 64, 64, 0, binding.MONARCH_FLAG_GENERIC) == 0
    assert call(ws_bytes=fneed - 1, batch=33, n_in=192, k=3, q=64, s=64, dtype=0) == binding.MONARCH_ERR_WORKSPACE
    assert call(ws=None, ws_bytes=0, batch=33, n_in=192, k=3, q=64, s=64, dtype=0) == binding.MONARCH_ERR_WORKSPACE
    assert call(ws_bytes=fneed, batch=0, n_in=192, k=3, q=64, s=64, dtype=0) == binding.MONARCH_OK
    # shapes without a packed-weight kernel behave as monarch_fwd_ex and need no workspace
    assert call(ws=None, ws_bytes=0, n_in=6, k=2, q=4, s=2, dtype=0) == binding.MONARCH_OK
    assert call(ws=None, ws_bytes=0, flags=binding.MONARCH_FLAG_GENERIC) == binding.MONARCH_OK


def test_dense_form_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced: every case below is refused before any launch

    def call(R=p, Lp=p, M=p, n_in=768, k=4, q=192, s=192, dtype=1, flags=0):
        return L.monarch_to_dense(R, Lp, M, n_in, k, q, s, dtype, None, flags)

    assert call(R=None) == binding.MONARCH_ERR_INVALID
    assert call(Lp=None) == binding.MONARCH_ERR_INVALID
    assert call(M=None) == binding.MONARCH_ERR_INVALID
    assert call(M=p + 8) == binding.MONARCH_ERR_INVALID          # not 16-byte aligned
    assert call(n_in=770) == binding.MONARCH_ERR_INVALID         # k does not divide n_in
    assert call(q=0) == binding.MONARCH_ERR_INVALID
    assert call(dtype=2) == binding.MONARCH_ERR_INVALID
    for f in (binding.MONARCH_FLAG_WGRAD_F32, binding.MONARCH_FLAG_GENERIC, binding.MONARCH_FLAG_WS_PACKED, 1024):
        assert call(flags=f) == binding.MONARCH_ERR_INVALID
    assert call(k=1 << 13, n_in=1 << 13, q=1 << 12, s=1) == binding.MONARCH_ERR_UNSUPPORTED


def test_backward_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096

    def call(ptrs=(p,) * 7, batch=1, n_in=768, k=4, q=192, s=192, dtype=1, ws=None, ws_bytes=0, flags=0):
        return L.monarch_bwd(*ptrs, batch, n_in, k, q, s, dtype, None, ws, ws_bytes, flags)

    for bad in range(7):
        ptrs = [p] * 7
        ptrs[bad] = None
        assert call(tuple(ptrs)) == binding.MONARCH_ERR_INVALID
    assert call(n_in=769) == binding.MONARCH_ERR_INVALID
    assert call(flags=1024) == binding.MONARCH_ERR_INVALID
    need = binding.monarch_bwd_workspace_bytes(1, 768, 4, 192, 192, 1, binding.MONARCH_FLAG_GENERIC)
    assert need > 0
    g = binding.MONARCH_FLAG_GENERIC
    assert call(flags=g) == binding.MONARCH_ERR_WORKSPACE                          # none given
    assert call(ws=4096, ws_bytes=need - 1, flags=g) == binding.MONARCH_ERR_WORKSPACE  # too small
    assert call(ws=4096 + 16, ws_bytes=need, flags=g) == binding.MONARCH_ERR_WORKSPACE  # misaligned
    assert binding.monarch_bwd_workspace_bytes(1, 769, 4, 192, 192, 1, 0) == 0


def test_affine_layer_calls_reject_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced
    need = binding.monarch_fwd_workspace_bytes(0, 768, 4, 192, 192, 1)

    def fwd(x=p, R=p, Lp=p, bias=p, y=p, ws=p, ws_bytes=need, flags=0, batch=0, n_in=768, k=4, q=192, s=192, dtype=1):
        return L.monarch_fwd_bias(x, R, Lp, bias, y, batch, n_in, k, q, s, dtype, None, ws, ws_bytes, flags)

    assert fwd() == binding.MONARCH_OK
    assert fwd(bias=None) == binding.MONARCH_OK                      # the plain forward with workspace
    assert fwd(bias=p + 8) == binding.MONARCH_ERR_INVALID            # not 16-byte aligned
    assert fwd(R=None) == binding.MONARCH_ERR_INVALID
    assert fwd(y=None, batch=3) == binding.MONARCH_ERR_INVALID
    assert fwd(n_in=770) == binding.MONARCH_ERR_INVALID
    assert fwd(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID
    assert fwd(ws=None) == binding.MONARCH_ERR_WORKSPACE
    assert fwd(ws_bytes=need - 1) == binding.MONARCH_ERR_WORKSPACE
    assert fwd(ws=None, ws_bytes=0, flags=binding.MONARCH_FLAG_GENERIC) == binding.MONARCH_OK
    assert fwd(ws=None, ws_bytes=0, n_in=6, k=2, q=4, s=2, dtype=0) == binding.MONARCH_OK

    bneed = binding.monarch_bwd_workspace_bytes(1, 768, 4, 192, 192, 1, 0)

    def bwd(ptrs=(p,) * 8, batch=1, ws=p, ws_bytes=bneed, flags=0, n_in=768):
        return L.monarch_bwd_bias(*ptrs, batch, n_in, 4, 192, 192, 1, None, ws, ws_bytes, flags)

    for bad in range(7):  # dbias (index 7) may be NULL, the others may not
        ptrs = [p] * 8
        ptrs[bad] = None
        assert bwd(tuple(ptrs)) == binding.MONARCH_ERR_INVALID
    assert bwd((p,) * 7 + (p + 4,)) == binding.MONARCH_ERR_INVALID   # dbias not 16-byte aligned
    assert bwd(ws=None) == binding.MONARCH_ERR_WORKSPACE
    assert bwd(ws_bytes=bneed - 1) == binding.MONARCH_ERR_WORKSPACE
    assert bwd(n_in=770) == binding.MONARCH_ERR_INVALID
    assert bwd(flags=binding.MONARCH_FLAG_WS_PACKED) == binding.MONARCH_ERR_INVALID
    # the bias gradient's partial rows are part of the backward workspace: it grows with the batch up to 128 chunks
    small = binding.monarch_bwd_workspace_bytes(64, 768, 4, 192, 192, 1, binding.MONARCH_FLAG_GENERIC)
    big = binding.monarch_bwd_workspace_bytes(64 * 128, 768, 4, 192, 192, 1, binding.MONARCH_FLAG_GENERIC)
    assert big - small >= 127 * 768 * 4


def test_layer_with_nonlinearity_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced
    need = binding.monarch_fwd_workspace_bytes(0, 768, 4, 192, 192, 1)

    def fwd(x=p, R=p, Lp=p, bias=p, y_pre=p + 64, y=p, ws=p, ws_bytes=need, flags=0, batch=0, n_in=768, k=4, q=192,
            s=192, dtype=1):
        return L.monarch_fwd_bias_gelu(x, R, Lp, bias, y_pre, y, batch, n_in, k, q, s, dtype, None, ws, ws_bytes, flags)

    assert fwd() == binding.MONARCH_OK
    assert fwd(bias=None) == binding.MONARCH_OK                      # no bias
    assert fwd(y_pre=None) == binding.MONARCH_OK                     # pre-activation not wanted
    assert fwd(y_pre=p) == binding.MONARCH_ERR_INVALID               # the two outputs may not be one buffer
    assert fwd(y_pre=p + 8) == binding.MONARCH_ERR_INVALID           # not 16-byte aligned
    assert fwd(bias=p + 8) == binding.MONARCH_ERR_INVALID
    assert fwd(Lp=None) == binding.MONARCH_ERR_INVALID
    assert fwd(y=None, batch=3) == binding.MONARCH_ERR_INVALID
    assert fwd(n_in=770) == binding.MONARCH_ERR_INVALID
    assert fwd(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID
    assert fwd(ws=None) == binding.MONARCH_ERR_WORKSPACE
    assert fwd(ws_bytes=need - 1) == binding.MONARCH_ERR_WORKSPACE
    assert fwd(ws=None, ws_bytes=0, flags=binding.MONARCH_FLAG_GENERIC) == binding.MONARCH_OK
    assert fwd(ws=None, ws_bytes=0, n_in=6, k=2, q=4, s=2, dtype=0) == binding.MONARCH_OK

    bneed = binding.monarch_bwd_workspace_bytes(1, 768, 4, 192, 192, 1, 0)

    def bwd(ptrs=(p,) * 9, batch=1, ws=p, ws_bytes=bneed, flags=0, n_in=768):
        return L.monarch_bwd_bias_gelu_in(*ptrs, batch, n_in, 4, 192, 192, 1, None, ws, ws_bytes, flags)

    for bad in range(8):  # dy, x, x_pre, R, L, dx_pre, dR, dL; dbias (index 8) may be NULL
        ptrs = [p] * 9
        ptrs[5] = p + 64  # dx_pre is a buffer of its own
        ptrs[bad] = None
        assert bwd(tuple(ptrs)) == binding.MONARCH_ERR_INVALID, bad
    assert bwd((p, p, p, p, p, p, p, p, p)) == binding.MONARCH_ERR_INVALID        # dx_pre over x_pre
    assert bwd((p, p, p + 8, p, p, p + 64, p, p, p)) == binding.MONARCH_ERR_INVALID   # x_pre not 16-byte aligned
    ok = (p, p, p, p, p, p + 64, p, p, None)
    assert bwd(ok, ws=None) == binding.MONARCH_ERR_WORKSPACE
    assert bwd(ok, ws_bytes=bneed - 1) == binding.MONARCH_ERR_WORKSPACE
    assert bwd(ok, n_in=770) == binding.MONARCH_ERR_INVALID
    assert bwd(ok, flags=binding.MONARCH_FLAG_WS_PACKED) == binding.MONARCH_ERR_INVALID


def test_projection_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced

    def call(A=p, R=p, Lp=p, n=256, m=16, dtype=0, flags=0):
        return L.monarch_project(A, R, Lp, n, m, dtype, None, flags)

    assert call(A=None) == binding.MONARCH_ERR_INVALID
    assert call(R=None) == binding.MONARCH_ERR_INVALID
    assert call(Lp=None) == binding.MONARCH_ERR_INVALID
    assert call(A=p + 4) == binding.MONARCH_ERR_INVALID
    assert call(n=255) == binding.MONARCH_ERR_INVALID            # n is not m * m
    assert call(n=0, m=0) == binding.MONARCH_ERR_INVALID
    assert call(dtype=3) == binding.MONARCH_ERR_INVALID
    assert call(flags=binding.MONARCH_FLAG_PERM_B) == binding.MONARCH_ERR_INVALID
    assert call(n=65 * 65, m=65) == binding.MONARCH_ERR_UNSUPPORTED


def test_transposed_multiply_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced
    need = binding.monarch_fwd_t_workspace_bytes(0, 768, 4, 192, 192, 1)
    assert need == 3 * 2 * 4 * 192 * 192                                    # three operand orders of the weights
    assert binding.monarch_fwd_t_workspace_bytes(100, 4096, 64, 64, 64, 1) == 100 * 4096 * 2 + 2 * 2 * 64 ** 3
    assert binding.monarch_fwd_t_workspace_bytes(0, 256, 16, 16, 16, 0) == 0
    assert binding.monarch_fwd_t_workspace_bytes(0, 6, 2, 4, 2, 0) == 0
    assert binding.monarch_fwd_t_workspace_bytes(0, 768, 4, 192, 192, 1, binding.MONARCH_FLAG_GENERIC) == 0

    def call(x=p, R=p, Lp=p, y=p, ws=p, ws_bytes=need, flags=0, batch=0, n_in=768, k=4, q=192, s=192, dtype=1):
        return L.monarch_fwd_t(x, R, Lp, y, batch, n_in, k, q, s, dtype, None, ws, ws_bytes, flags)

    assert call() == binding.MONARCH_OK
    assert call(ws=None) == binding.MONARCH_ERR_WORKSPACE
    assert call(ws_bytes=need - 1) == binding.MONARCH_ERR_WORKSPACE
    assert call(ws=p + 16) == binding.MONARCH_ERR_WORKSPACE
    assert call(R=None) == binding.MONARCH_ERR_INVALID
    assert call(x=None, batch=2) == binding.MONARCH_ERR_INVALID
    assert call(n_in=770) == binding.MONARCH_ERR_INVALID
    assert call(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID
    assert call(flags=binding.MONARCH_FLAG_WS_PACKED) == binding.MONARCH_ERR_INVALID
    assert call(ws=None, ws_bytes=0, flags=binding.MONARCH_FLAG_GENERIC) == binding.MONARCH_OK
    assert call(ws=None, ws_bytes=0, n_in=6, k=2, q=4, s=2, dtype=0) == binding.MONARCH_OK


def test_saved_intermediate_calls_reject_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced
    need = binding.monarch_saved_bytes(1000, 768, 4, 192, 192, 1)
    assert need == 1000 * 768 * 2                                   # B x k*q bf16
    assert binding.monarch_saved_bytes(1000, 4096, 64, 64, 64, 1) == 0   # kernels that recompute
    assert binding.monarch_saved_bytes(1000, 256, 16, 16, 16, 0) == 0
    assert binding.monarch_saved_bytes(1000, 768, 4, 192, 192, 1, binding.MONARCH_FLAG_GENERIC) == 0
    assert binding.monarch_saved_bytes(1000, 770, 4, 192, 192, 1) == 0

    def fwd(x=p, R=p, Lp=p, y=p, sv=p, sv_bytes=need, batch=1000, n_in=768, k=4, q=192, s=192, dtype=1, flags=0):
        return L.monarch_fwd_save(x, R, Lp, y, sv, sv_bytes, batch, n_in, k, q, s, dtype, None, flags)

    assert fwd(sv=None) == binding.MONARCH_ERR_WORKSPACE
    assert fwd(sv_bytes=need - 1) == binding.MONARCH_ERR_WORKSPACE
    assert fwd(sv=p + 8) == binding.MONARCH_ERR_WORKSPACE
    assert fwd(R=None) == binding.MONARCH_ERR_INVALID
    assert fwd(y=None) == binding.MONARCH_ERR_INVALID
    assert fwd(n_in=770) == binding.MONARCH_ERR_INVALID
    assert fwd(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID
    assert fwd(batch=0, sv_bytes=binding.monarch_saved_bytes(0, 768, 4, 192, 192, 1)) == binding.MONARCH_OK
    # shapes without the path: the plain forward, no buffer needed
    assert fwd(sv=None, sv_bytes=0, batch=0, n_in=6, k=2, q=4, s=2, dtype=0) == binding.MONARCH_OK

    bneed = binding.monarch_bwd_workspace_bytes(1000, 768, 4, 192, 192, 1, 0)

    def bwd(sv=p, sv_bytes=need, ws=p, ws_bytes=bneed, flags=0, dbias=None):
        return L.monarch_bwd_saved(p, p, sv, sv_bytes, p, p, p, p, p, dbias, 1000, 768, 4, 192, 192, 1, None, ws, ws_bytes, flags)

    assert bwd(sv_bytes=need - 1) == binding.MONARCH_ERR_WORKSPACE
    assert bwd(sv=p + 8) == binding.MONARCH_ERR_WORKSPACE
    assert bwd(ws=None) == binding.MONARCH_ERR_WORKSPACE
    assert bwd(flags=binding.MONARCH_FLAG_WS_PACKED) == binding.MONARCH_ERR_INVALID


def test_complex_calls_reject_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    p = 4096  # never dereferenced

    def fwd(x=p, R=p, Lp=p, y=p, batch=0, n_in=16, k=4, q=4, s=4, flags=0):
        return L.monarch_fwd_c64(x, R, Lp, y, batch, n_in, k, q, s, None, flags)

    assert fwd() == binding.MONARCH_OK
    assert fwd(R=None) == binding.MONARCH_ERR_INVALID
    assert fwd(y=None, batch=1) == binding.MONARCH_ERR_INVALID
    assert fwd(x=p + 8) == binding.MONARCH_ERR_INVALID
    assert fwd(n_in=18) == binding.MONARCH_ERR_INVALID
    assert fwd(flags=binding.MONARCH_FLAG_GENERIC) == binding.MONARCH_ERR_INVALID
    assert fwd(n_in=4 * 40000, q=40000) == binding.MONARCH_ERR_UNSUPPORTED     # one row does not fit the LDS

    def fwd_h(x=p, R=p, Lp=p, y=p, batch=0, n_in=16, k=4, q=4, s=4, flags=0):
        return L.monarch_fwd_h_c64(x, R, Lp, y, batch, n_in, k, q, s, None, flags)

    assert fwd_h() == binding.MONARCH_OK
    assert fwd_h(Lp=None) == binding.MONARCH_ERR_INVALID
    assert fwd_h(x=None, batch=1) == binding.MONARCH_ERR_INVALID
    assert fwd_h(y=p + 8) == binding.MONARCH_ERR_INVALID
    assert fwd_h(n_in=18) == binding.MONARCH_ERR_INVALID
    assert fwd_h(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID
    assert fwd_h(n_in=4 * 4, s=40000, q=40000) == binding.MONARCH_ERR_UNSUPPORTED     # one row does not fit the LDS

    def bwd(ptrs=(p,) * 7, batch=1, n_in=16, flags=0):
        return L.monarch_bwd_c64(*ptrs, batch, n_in, 4, 4, 4, None, flags)

    for bad in range(7):
        ptrs = [p] * 7
        ptrs[bad] = None
        assert bwd(tuple(ptrs)) == binding.MONARCH_ERR_INVALID
    assert bwd(n_in=18) == binding.MONARCH_ERR_INVALID
    assert bwd(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID

    cneed = binding.monarch_c64_workspace_bytes(binding.C64_BWD, 5, 16, 4, 4, 4, 0)
    assert cneed >= 5 * (2 * 16 + 16) * 8
    assert binding.monarch_c64_workspace_bytes(binding.C64_BWD, 5, 18, 4, 4, 4, 0) == 0          # n_in not k*p
    assert binding.monarch_c64_workspace_bytes(binding.C64_BWD, 5, 16, 4, 4, 4, binding.MONARCH_FLAG_GENERIC) == 0
    assert binding.monarch_c64_workspace_bytes(3, 5, 16, 4, 4, 4, 0) == 0                        # no such pass
    assert binding.monarch_c64_workspace_bytes(binding.C64_FWD, 5, 16, 4, 4, 4, 0) == 0          # shape-generic forward: none
    # square blocks of 16 / 32 / 64: the tiled intermediate, whole 32-row tiles
    mneed = binding.monarch_c64_workspace_bytes(binding.C64_FWD, 33, 4 * 16, 4, 16, 16, 0)
    assert mneed == 2 * 32 * 4 * 16 * 8
    assert binding.monarch_c64_workspace_bytes(binding.C64_FWD_H, 33, 4 * 16, 4, 16, 16, 0) == mneed
    assert binding.monarch_c64_workspace_bytes(binding.C64_BWD, 33, 4 * 16, 4, 16, 16, 0) >= 2 * mneed

    def fwd_ws(fn, ptrs=(p,) * 4, ws=p, ws_bytes=mneed, flags=0, n_in=64):
        return fn(*ptrs, 33, n_in, 4, 16, 16, None, ws, ws_bytes, flags)

    for fn in (L.monarch_fwd_c64_ws, L.monarch_fwd_h_c64_ws):
        for bad in range(4):
            ptrs = [p] * 4
            ptrs[bad] = None
            assert fwd_ws(fn, tuple(ptrs)) == binding.MONARCH_ERR_INVALID
        assert fwd_ws(fn, ws_bytes=mneed - 1) == binding.MONARCH_ERR_WORKSPACE
        assert fwd_ws(fn, ws=p + 16) == binding.MONARCH_ERR_WORKSPACE
        assert fwd_ws(fn, n_in=66) == binding.MONARCH_ERR_INVALID
        assert fwd_ws(fn, flags=binding.MONARCH_FLAG_GENERIC) == binding.MONARCH_ERR_INVALID

    def bwd_ws(ptrs=(p,) * 7, batch=5, n_in=16, ws=p, ws_bytes=cneed, flags=0):
        return L.monarch_bwd_c64_ws(*ptrs, batch, n_in, 4, 4, 4, None, ws, ws_bytes, flags)

    for bad in range(7):
        ptrs = [p] * 7
        ptrs[bad] = None
        assert bwd_ws(tuple(ptrs)) == binding.MONARCH_ERR_INVALID
    assert bwd_ws(ws_bytes=cneed - 1) == binding.MONARCH_ERR_WORKSPACE
    assert bwd_ws(ws=p + 16) == binding.MONARCH_ERR_WORKSPACE                                   # not 256-byte aligned
    assert bwd_ws(n_in=18) == binding.MONARCH_ERR_INVALID
    assert bwd_ws(flags=binding.MONARCH_FLAG_WGRAD_F32) == binding.MONARCH_ERR_INVALID

    assert L.monarch_dft_factors(None, p, 4, 0, None) == binding.MONARCH_ERR_INVALID
    assert L.monarch_dft_factors(p, p, 0, 0, None) == binding.MONARCH_ERR_INVALID
    assert L.monarch_dft_factors(p, p + 8, 4, 0, None) == binding.MONARCH_ERR_INVALID
    assert L.monarch_dft_factors(p, p, 2000, 0, None) == binding.MONARCH_ERR_UNSUPPORTED


def test_stream_copy_rejects_bad_arguments_without_a_gpu(binding):
    L = binding.lib()
    assert L.monarch_stream_copy(None, None, 0, None) == binding.MONARCH_OK          # empty copy: no-op
    assert L.monarch_stream_copy(None, 4096, 64, None) == binding.MONARCH_ERR_INVALID
    assert L.monarch_stream_copy(4096, 8192, 24, None) == binding.MONARCH_ERR_INVALID   # not a multiple of 16
    assert L.monarch_stream_copy(4100, 8192, 64, None) == binding.MONARCH_ERR_INVALID   # misaligned
    assert L.monarch_stream_copy(4096, 4128, 64, None) == binding.MONARCH_ERR_INVALID   # overlap


def test_kernel_name_reports_dispatch(binding):
    assert binding.monarch_kernel_name(0, 770, 4, 192, 192, 1) == "invalid"
    assert binding.monarch_kernel_name(4, 768, 4, 192, 192, 1) == "invalid"
    assert binding.monarch_kernel_name(3, 768, 4, 192, 192, 1) == "mfma_fwd_t_wide_bf16"
    assert binding.monarch_kernel_name(3, 4096, 64, 64, 64, 1) == "mfma_fwd_t_sq64_bf16"
    assert binding.monarch_kernel_name(3, 256, 16, 16, 16, 0) == "mfma_fwd_t_sq16_f32"
    assert binding.monarch_kernel_name(3, 6, 2, 4, 2, 0) == "generic_fwd_t"
    assert binding.monarch_kernel_name(2, 768, 4, 192, 192, 1) == "mfma_fwd_frag_bf16"
    assert binding.monarch_kernel_name(2, 4096, 64, 64, 64, 1) == "mfma_fwd_sq64_packed_bf16"
    assert [binding.monarch_kernel_name(ps, 5 * 32, 5, 32, 32, 0, binding.MONARCH_FLAG_PERM_B) for ps in (0, 1, 2, 3)] == \
        ["generic_fwd", "mfma_bwd_stages_f32", "mfma_fwd_stages_f32", "mfma_fwd_t_stages_f32"]
    assert binding.monarch_kernel_name(2, 6, 2, 4, 2, 0) == "generic_fwd"   # no packed-weight kernel: same as pass 0
    assert binding.monarch_kernel_name(0, 6, 2, 4, 2, 0) == "generic_fwd"
    assert binding.monarch_kernel_name(1, 6, 2, 4, 2, 0) == "generic_bwd"
    assert binding.monarch_kernel_name(0, 768, 4, 192, 192, 1, binding.MONARCH_FLAG_GENERIC) == "generic_fwd"
    assert binding.monarch_kernel_name(0, 4 * 2000000, 4, 2000000, 4, 1) == "unsupported"
    # every four-block layer shape of ViT-B, GPT-2 small and GPT-2 medium has matrix-core kernels
    for n_in, q, s in ((768, 192, 192), (768, 192, 576), (768, 192, 768), (3072, 192, 192),
                       (1024, 256, 256), (1024, 256, 768), (1024, 256, 1024), (4096, 256, 256),
                       (512, 128, 128), (512, 128, 512), (2048, 128, 128)):
        assert [binding.monarch_kernel_name(ps, n_in, 4, q, s, 1) for ps in (0, 1, 2)] == \
            ["mfma_fwd_wide_bf16", "mfma_bwd_wide_bf16", "mfma_fwd_frag_bf16"], (n_in, q, s)


def test_python_binding_fails_loudly_without_the_library(binding, monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.lib()


def test_product_package_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2204_00595_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                for needle in ("import oracle", "from oracle", "monarch_oracle", "oracle/", "oracle."):
                    assert needle not in text, (os.path.join(dirpath, fn), needle)


# ------------------------------------------------------------ input generator ----

def test_generator_is_counter_based_and_normal():
    from paper_2204_00595_amd import synth
    a = synth.normal(42, (200000,))
    assert np.array_equal(a[:1000], synth.normal(42, (1000,)))          # prefix property
    assert np.array_equal(a.reshape(400, 500), synth.normal(42, (400, 500)))
    assert not np.array_equal(a[:1000], synth.normal(43, (1000,)))
    assert abs(float(a.mean())) < 0.01 and abs(float(a.std()) - 1.0) < 0.01
    assert abs(float(np.mean(a.astype(np.float64) ** 4)) - 3.0) < 0.1    # kurtosis of a normal
    b = synth.normal(42, (200000,), std=0.25)
    assert abs(float(b.std()) - 0.25) < 0.005


def test_bf16_rounding_is_nearest_even_and_widening_is_exact():
    from paper_2204_00595_amd import synth
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins (1.0);
    # 1 + 3*2^-8 is a tie between 1 + 2^-7 and 1 + 2^-6: even wins (1 + 2^-6).
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0, 3.0e38],
                    dtype=np.float32)
    got = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(vals))
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 0.0, 2.9907e38], dtype=np.float32)
    assert np.allclose(got[:6], want[:6], rtol=0, atol=0)
    assert abs(float(got[6]) / 3.0e38 - 1) < 2.0 ** -8 and np.isfinite(got[6])
    torch = pytest.importorskip("torch")
    a = synth.normal(1, (50000,))
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(synth.f32_to_bf16_bits(a), ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(synth.quantize(a, "bf16"), ref.float().numpy())
    assert np.array_equal(synth.quantize(a, "f32"), a)


def test_workload_table_matches_the_stated_shapes():
    from paper_2204_00595_amd import synth
    w = synth.WORKLOADS
    assert (w["sq256_f32"].n_in, w["sq256_f32"].n_out, w["sq256_f32"].B) == (256, 256, 64)
    assert (w["vitb_proj"].n_in, w["vitb_proj"].n_out, w["vitb_proj"].B) == (768, 768, 12608)
    assert (w["gpt2s_fc1"].n_in, w["gpt2s_fc1"].n_out, w["gpt2s_fc1"].B) == (768, 3072, 8192)
    assert (w["sq4096"].n_in, w["sq4096"].n_out, w["sq4096"].B) == (4096, 4096, 16384)
    assert (w["gpt2m_fc1"].n_in, w["gpt2m_fc1"].n_out) == (1024, 4096)
    assert (w["gpt2m_fc2"].n_in, w["gpt2m_fc2"].n_out) == (4096, 1024)
    # square Monarch: 2 n sqrt(n) parameters, O(n sqrt n) work (Section 3.2.2)
    sq = w["sq4096"]
    assert sq.k * sq.q * (sq.p + sq.s) == 2 * 4096 * 64
    assert sq.fwd_flops() == 2 * (2 * 4096 * 64) * sq.B
    x, R, L, dy = synth.make_inputs(w["vitb_proj"], rows=8)
    assert x.shape == (8, 768) and R.shape == (4, 192, 192) and L.shape == (4, 192, 192) and dy.shape == (8, 768)
    assert abs(float(R.std()) - 192 ** -0.5) < 0.002
