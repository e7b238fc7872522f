"""monarch_fwd_static (the forward whose scratch memory is an array inside the library, for callers that
cannot allocate) against monarch_fwd_ws through the C ABI: same kernels, so the results must agree bit for
bit, on two calls in a row that share the array, the second one smaller and of another shape; and against
the oracle to the multiply's tolerance."""
import ctypes

import numpy as np
import pytest

import oracle
import parity_util
from paper_2204_00595_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
CASES = [
    # first call: large packed copies; second call: fewer rows and a smaller shape in the same array
    (("static_gpt2m_fc1", "bf16", 330, 4, 256, 256, 1024), ("static_k4_64", "bf16", 70, 4, 64, 64, 64)),
    (("static_sq_m64", "bf16", 100, 64, 64, 64, 64), ("static_k4_192", "bf16", 37, 4, 192, 192, 192)),
    # shapes without a packed-weight kernel run without any workspace
    (("static_sq_m16", "f32", 131, 16, 16, 16, 16), ("static_rect", "f32", 19, 3, 2, 6, 5)),
]


def _dev(a, dtype):
    dt = torch.float32 if dtype == "f32" else torch.bfloat16
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(dt).contiguous()


@pytest.mark.parametrize("pair", CASES, ids=lambda p: p[0][0])
def test_static_workspace_forward_matches_the_workspace_forward(pair):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2204_00595_amd import binding
    lib = binding.lib()
    vp = ctypes.c_void_p
    for case in pair:  # two calls in a row on the same GPU: the second finds the first one's packed weights in the array
        name, dtype, Bn, k, p, q, s = case
        sh = synth.Shape(name, dtype, Bn, k, p, q, s, config=90 + parity_util.stable_seed(name))
        x, R, L, _ = synth.make_inputs(sh)
        xd, Rd, Ld = _dev(x, dtype), _dev(R, dtype), _dev(L, dtype)
        code = 0 if dtype == "f32" else 1
        y_static = torch.full((Bn, sh.n_out), float("nan"), dtype=xd.dtype, device="cuda")
        y_ws = torch.full_like(y_static, float("nan"))
        need = binding.monarch_fwd_workspace_bytes(Bn, sh.n_in, k, q, s, code, 0)
        assert need <= binding.MONARCH_STATIC_WORKSPACE_BYTES
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        st = vp(int(torch.cuda.current_stream().cuda_stream))
        rc = lib.monarch_fwd_static(vp(xd.data_ptr()), vp(Rd.data_ptr()), vp(Ld.data_ptr()), vp(y_static.data_ptr()),
                                    Bn, sh.n_in, k, q, s, code, st, 0)
        assert rc == 0, binding.monarch_status_string(rc)
        rc = lib.monarch_fwd_ws(vp(xd.data_ptr()), vp(Rd.data_ptr()), vp(Ld.data_ptr()), vp(y_ws.data_ptr()),
                                Bn, sh.n_in, k, q, s, code, st, vp(ws.data_ptr()), ws.numel(), 0)
        assert rc == 0, binding.monarch_status_string(rc)
        torch.cuda.synchronize()
        assert torch.equal(y_static, y_ws), name
        parity_util.check(name + ".y", y_static.float().cpu().numpy(), oracle.fwd(x, R, L), TOL[dtype])


def test_static_workspace_forward_rejects_what_it_cannot_serve():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2204_00595_amd import binding
    x = torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda")
    R = torch.zeros((4, 64, 64), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.MonarchError) as e:
        binding.monarch_fwd_static(x, R, R, y, flags=binding.MONARCH_FLAG_WS_PACKED)
    assert e.value.status == binding.MONARCH_ERR_INVALID
