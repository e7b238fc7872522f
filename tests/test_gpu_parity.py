"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element on
the same seeded inputs.  Tolerance = max relative Frobenius error over the tensors of a call:
<= 1e-5 for fp32, <= 2e-2 for bf16 storage with fp32 accumulation."""
import numpy as np
import pytest

import oracle
import parity_util
from paper_2204_00595_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
GUARD = 256  # elements of NaN canary either side of every output


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2204_00595_amd import binding
    binding.lib()  # fails loudly if libmonarch.so is missing
    return binding


def tdtype(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(tdtype(dtype)).contiguous()


def guarded(shape, dt):
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * GUARD,), float("nan"), dtype=dt, device="cuda")
    return buf, buf[GUARD:GUARD + n].view(*shape)


def check_guard(buf, name):
    assert bool(torch.isnan(buf[:GUARD]).all()) and bool(torch.isnan(buf[-GUARD:]).all()), name + ": wrote out of bounds"


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def run_fwd(B, sh, x, R, L, flags=0, ws=False):
    """monarch_fwd / monarch_fwd_ex, or (ws=True) monarch_fwd_ws with a guarded workspace."""
    ybuf, y = guarded((x.shape[0], sh.n_out), tdtype(sh.dtype))
    if ws:
        code = 0 if sh.dtype == "f32" else 1
        need = B.monarch_fwd_workspace_bytes(x.shape[0], sh.n_in, sh.k, sh.q, sh.s, code, flags)
        wbuf = torch.full((need + 512 + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
        off = (-(wbuf.data_ptr() + GUARD)) % 256 + GUARD  # 256-byte aligned start inside the canary
        B.monarch_fwd_ws(dev(x, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype), y, workspace=wbuf[off:off + need], flags=flags)
        torch.cuda.synchronize()
        assert bool((wbuf[:off] == 0x5A).all()) and bool((wbuf[off + need:] == 0x5A).all()), "workspace: wrote out of bounds"
    else:
        B.monarch_fwd(dev(x, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype), y, flags=flags)
        torch.cuda.synchronize()
    check_guard(ybuf, "y")
    out = host(y)
    assert np.isfinite(out).all(), "y has unwritten or non-finite entries"
    return out


def run_bwd(B, sh, dy, x, R, L, flags=0):
    dt = tdtype(sh.dtype)
    gdt = torch.float32 if (flags & B.MONARCH_FLAG_WGRAD_F32) else dt
    bx, dx = guarded((x.shape[0], sh.n_in), dt)
    bR, dR = guarded(R.shape, gdt)
    bL, dL = guarded(L.shape, gdt)
    B.monarch_bwd(dev(dy, sh.dtype), dev(x, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype), dx, dR, dL, flags=flags)
    torch.cuda.synchronize()
    for buf, name in ((bx, "dx"), (bR, "dR"), (bL, "dL")):
        check_guard(buf, name)
    outs = [host(t) for t in (dx, dR, dL)]
    for o, name in zip(outs, ("dx", "dR", "dL")):
        assert np.isfinite(o).all(), name + " has unwritten or non-finite entries"
    return outs


def compare(sh, got, want, names):
    """Global relative Frobenius error <= the tolerance, and every row (activations) / block (weight
    gradients) within 4x of it: see parity_util.check."""
    errs = {n: oracle.rel_fro(g, w) for n, g, w in zip(names, got, want)}
    print("  %s %s" % (sh.name, " ".join("%s=%.2e" % kv for kv in errs.items())), flush=True)
    for n, g, w in zip(names, got, want):
        parity_util.check("%s.%s" % (sh.name, n), g, w, TOL[sh.dtype])
    return errs


SMALL = [
    # name, dtype, B, k, p, q, s  -- several row tiles plus a ragged tail; k | q and k !| q
    ("sq_m2", "f32", 5, 2, 2, 2, 2),
    ("sq_m16", "f32", 64, 16, 16, 16, 16),
    ("sq_m16_tail", "f32", 131, 16, 16, 16, 16),
    # the backward takes one workgroup per 16-row tile up to 1024 tiles and persistent workgroups beyond
    ("sq_m16_1024_tiles", "f32", 16384 - 5, 16, 16, 16, 16),
    ("sq_m16_1025_tiles", "f32", 16384 + 3, 16, 16, 16, 16),
    # ... and the forward up to 2048 tiles
    ("sq_m16_2048_tiles", "f32", 32768 - 7, 16, 16, 16, 16),
    ("sq_m16_2049_tiles", "f32", 32768 + 5, 16, 16, 16, 16),
    ("rect_2_3_4_2", "f32", 37, 2, 3, 4, 2),
    ("rect_3_2_6_5", "f32", 19, 3, 2, 6, 5),
    ("rect_4_3_8_2", "f32", 70, 4, 3, 8, 2),
    ("rect_3_4_5_2", "f32", 33, 3, 4, 5, 2),
    ("one_block", "f32", 21, 1, 5, 3, 4),
    ("one_row", "f32", 1, 4, 8, 8, 8),
    ("sq_m16_bf16", "bf16", 77, 16, 16, 16, 16),
    ("k4_64_bf16", "bf16", 150, 4, 64, 64, 64),
    ("k4_64_128_bf16", "bf16", 97, 4, 64, 64, 128),
    ("k4_128_64_64_bf16", "bf16", 65, 4, 128, 64, 64),
    ("sq_m32_bf16", "bf16", 45, 32, 32, 32, 32),
    ("rect_bf16_odd", "bf16", 29, 3, 10, 6, 14),
    ("k4_192_bf16", "bf16", 200, 4, 192, 192, 192),
    ("sq_m64_bf16", "bf16", 40, 64, 64, 64, 64),
]


def small_shape(case):
    name, dtype, Bn, k, p, q, s = case
    return synth.Shape(name, dtype, Bn, k, p, q, s, config=90 + parity_util.stable_seed(name))


@pytest.mark.parametrize("generic", [False, True], ids=["dispatch", "generic"])
@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_shapes_fwd_bwd(B, case, generic):
    sh = small_shape(case)
    flags = B.MONARCH_FLAG_GENERIC if generic else 0
    print("\n  kernels: %s / %s" % (B.monarch_kernel_name(0, sh.n_in, sh.k, sh.q, sh.s, 0 if sh.dtype == "f32" else 1, flags),
                                    B.monarch_kernel_name(1, sh.n_in, sh.k, sh.q, sh.s, 0 if sh.dtype == "f32" else 1, flags)), flush=True)
    x, R, L, dy = synth.make_inputs(sh)
    y = run_fwd(B, sh, x, R, L, flags)
    compare(sh, [y], [oracle.fwd(x, R, L)], ["y"])
    yw = run_fwd(B, sh, x, R, L, flags, ws=True)
    compare(sh, [yw], [oracle.fwd(x, R, L)], ["y_ws"])
    got = run_bwd(B, sh, dy, x, R, L, flags)
    compare(sh, got, oracle.bwd(dy, x, R, L), ["dx", "dR", "dL"])
    got32 = run_bwd(B, sh, dy, x, R, L, flags | B.MONARCH_FLAG_WGRAD_F32)
    compare(sh, got32, oracle.bwd(dy, x, R, L), ["dx", "dR32", "dL32"])


# The other Monarch layer shapes of the paper's ViT-B / GPT-2 small / GPT-2 medium models (four blocks):
# attention output projection, fused q,k,v projection and the second MLP layer, and the layers of a
# width-512 model (MLP-Mixer-S channel mixing), at a batch of several 64-row tiles plus a ragged tail.  All of them must be served by the matrix-core kernels.
MODEL_LAYERS = [
    ("gpt2m_proj_1024_1024", "bf16", 1100, 4, 256, 256, 256),
    ("qkv_768_2304", "bf16", 1100, 4, 192, 192, 576),
    ("gpt2m_qkv_1024_3072", "bf16", 1100, 4, 256, 256, 768),
    ("gpt2s_fc2_3072_768", "bf16", 1100, 4, 768, 192, 192),
    ("gpt2m_fc2_4096_1024", "bf16", 333, 4, 1024, 256, 256),   # ragged against the 256-row tiles of the step-1 GEMM
    ("w512_proj_512_512", "bf16", 1100, 4, 128, 128, 128),
    ("w512_fc1_512_2048", "bf16", 1100, 4, 128, 128, 512),
    ("w512_fc2_2048_512", "bf16", 1100, 4, 512, 128, 128),
]


@pytest.mark.parametrize("case", MODEL_LAYERS, ids=lambda c: c[0])
def test_model_layer_shapes_on_matrix_cores(B, case):
    sh = small_shape(case)
    names = [B.monarch_kernel_name(ps, sh.n_in, sh.k, sh.q, sh.s, 1) for ps in (0, 1, 2)]
    assert names == ["mfma_fwd_wide_bf16", "mfma_bwd_wide_bf16", "mfma_fwd_frag_bf16"], names
    x, R, L, dy = synth.make_inputs(sh)
    yo = oracle.fwd(x, R, L)
    compare(sh, [run_fwd(B, sh, x, R, L), run_fwd(B, sh, x, R, L, ws=True)], [yo, yo], ["y", "y_ws"])
    bias = make_bias(sh)
    compare(sh, [run_fwd_bias(B, sh, x, R, L, bias)], [oracle.fwd_bias(x, R, L, bias)], ["y_bias"])
    compare(sh, run_bwd_bias(B, sh, dy, x, R, L), oracle.bwd_bias(dy, x, R, L), ["dx", "dR", "dL", "dbias"])
    compare(sh, run_bwd(B, sh, dy, x, R, L, B.MONARCH_FLAG_WGRAD_F32), oracle.bwd(dy, x, R, L), ["dx", "dR32", "dL32"])


# Shapes without a tuned kernel that the shape-generic matrix-core kernels must serve: block sizes that are
# multiples of 16 (forward; a size that is 16 mod 32 ends on a half-empty K-step) or of 32 (backward; any k:
# the weight-gradient GEMM takes four blocks per workgroup and masks the ones past the last).  name, dtype, B, k, p, q, s, backward on matrix cores too
TILED = [
    ("vits_proj_384_384", "bf16", 300, 4, 96, 96, 96, True),
    ("vits_fc1_384_1536", "bf16", 203, 4, 96, 96, 384, True),
    ("vits_fc2_1536_384", "bf16", 140, 4, 384, 96, 96, True),
    ("vits_few_rows", "bf16", 5, 4, 96, 96, 96, True),
    ("k8_64_32_96", "bf16", 131, 8, 64, 32, 96, True),
    ("k12_32_64_32", "bf16", 77, 12, 32, 64, 32, True),
    ("k16_wide_mid", "bf16", 50, 16, 32, 192, 32, True),
    ("k2_64_32_96", "bf16", 150, 2, 64, 32, 96, True),
    ("k6_32_64_32", "bf16", 101, 6, 32, 64, 32, True),
    ("k1_dense_pair_32", "bf16", 70, 1, 64, 96, 32, True),
    ("k2_tail_48_80_48", "bf16", 90, 2, 48, 80, 48, False),
    ("k3_32_48_16", "bf16", 67, 3, 32, 48, 16, False),
    ("k1_dense_pair", "bf16", 33, 1, 64, 48, 80, False),
]


@pytest.mark.parametrize("reading", ["A", "B"])
@pytest.mark.parametrize("case", TILED, ids=lambda c: c[0])
def test_shape_generic_matrix_core_kernels(B, case, reading):
    sh = small_shape(case[:7])
    flags = B.MONARCH_FLAG_PERM_B if reading == "B" else 0
    rd = oracle.READING_B if reading == "B" else oracle.READING_A
    names = [B.monarch_kernel_name(ps, sh.n_in, sh.k, sh.q, sh.s, 1, flags) for ps in (0, 1)]
    assert names == ["mfma_fwd_tiled_bf16", "mfma_bwd_tiled_bf16" if case[7] else "generic_bwd"], names
    x, R, L, dy = synth.make_inputs(sh)
    compare(sh, [run_fwd(B, sh, x, R, L, flags)], [oracle.fwd(x, R, L, rd)], ["y"])
    bias = make_bias(sh)
    compare(sh, [run_fwd_bias(B, sh, x, R, L, bias, flags)], [oracle.fwd_bias(x, R, L, bias, rd)], ["y_bias"])
    compare(sh, run_bwd(B, sh, dy, x, R, L, flags), oracle.bwd(dy, x, R, L, rd), ["dx", "dR", "dL"])
    compare(sh, run_bwd_bias(B, sh, dy, x, R, L, flags | B.MONARCH_FLAG_WGRAD_F32), oracle.bwd_bias(dy, x, R, L, rd),
            ["dx", "dR32", "dL32", "dbias32"])


# fp32 layers with square blocks of 32 or 64: every call that takes a workspace runs on the fp32 matrix-core stage
# kernels (any block count, both readings); batches long enough that a workgroup takes several 32-row tiles, the last
# one ragged.  name, B, k, m
F32_STAGE_CASES = [("f32_m32", 100, 32, 32), ("f32_k3_m64", 67, 3, 64), ("f32_k5_m32", 333, 5, 32), ("f32_m64", 40, 64, 64),
                   ("f32_k8_m32_long", 8219, 8, 32), ("f32_k2_m64_long", 16421, 2, 64)]


@pytest.mark.parametrize("reading", ["A", "B"])
@pytest.mark.parametrize("case", F32_STAGE_CASES, ids=lambda c: c[0])
def test_fp32_square_blocks_on_matrix_cores(B, case, reading):
    name, Bn, k, m = case
    sh = synth.Shape(name, "f32", Bn, k, m, m, m, config=300 + parity_util.stable_seed(name))
    flags = B.MONARCH_FLAG_PERM_B if reading == "B" else 0
    rd = oracle.READING_B if reading == "B" else oracle.READING_A
    names = [B.monarch_kernel_name(ps, sh.n_in, k, m, m, 0, flags) for ps in (1, 2, 3)]
    assert names == ["mfma_bwd_stages_f32", "mfma_fwd_stages_f32", "mfma_fwd_t_stages_f32"], names
    x, R, L, dy = synth.make_inputs(sh)
    compare(sh, [run_fwd(B, sh, x, R, L, flags, ws=True)], [oracle.fwd(x, R, L, rd)], ["y_ws"])
    compare(sh, run_bwd(B, sh, dy, x, R, L, flags), oracle.bwd(dy, x, R, L, rd), ["dx", "dR", "dL"])
    compare(sh, [run_fwd_t(B, sh, dy, R, L, flags)], [oracle.fwd_t(dy, R, L, rd)], ["xM"])
    compare(sh, run_bwd_bias(B, sh, dy, x, R, L, flags), oracle.bwd_bias(dy, x, R, L, rd), ["dx", "dR", "dL", "dbias"])
    bias = make_bias(sh)   # the layer calls around the multiply: bias and nonlinearity as passes of their own
    compare(sh, [run_fwd_bias(B, sh, x, R, L, bias, flags)], [oracle.fwd_bias(x, R, L, bias, rd)], ["y_bias"])
    if reading == "A" and Bn < 1000:
        gelu_layer_case(B, sh, flags)
    for u, v in zip(run_bwd(B, sh, dy, x, R, L, flags), run_bwd(B, sh, dy, x, R, L, flags)):   # fixed summation order
        assert np.array_equal(u, v)
    # empty batch: zero gradients
    e = run_bwd(B, sh, dy[:0], x[:0], R, L, flags)
    assert e[0].shape == (0, sh.n_in) and not e[1].any() and not e[2].any()


def test_shape_generic_kernels_on_random_shapes(B):
    """Seeded random shapes with blocks that are multiples of 32 and any block count (odd ones too): forward,
    backward and transposed multiply must run on the shape-generic matrix-core kernels and match the oracle."""
    rng = np.random.default_rng(20220400595)
    done = 0
    while done < 10:
        k = int(rng.integers(1, 10))
        p, q, s = (int(32 * rng.integers(1, 6)) for _ in range(3))
        Bn = int(rng.integers(1, 200))
        reading = int(rng.integers(0, 2))
        flags = B.MONARCH_FLAG_PERM_B if reading else 0
        names = [B.monarch_kernel_name(ps, k * p, k, q, s, 1, flags) for ps in (0, 1, 3)]
        if names != ["mfma_fwd_tiled_bf16", "mfma_bwd_tiled_bf16", "mfma_fwd_t_tiled_bf16"]:
            continue  # a shape with a tuned kernel
        done += 1
        sh = synth.Shape("rand%d_k%d_%d_%d_%d_B%d_r%d" % (done, k, p, q, s, Bn, reading), "bf16", Bn, k, p, q, s, config=200 + done)
        rd = oracle.READING_B if reading else oracle.READING_A
        x, R, L, dy = synth.make_inputs(sh)
        compare(sh, [run_fwd(B, sh, x, R, L, flags)], [oracle.fwd(x, R, L, rd)], ["y"])
        compare(sh, run_bwd(B, sh, dy, x, R, L, flags), oracle.bwd(dy, x, R, L, rd), ["dx", "dR", "dL"])
        compare(sh, [run_fwd_t(B, sh, dy, R, L, flags)], [oracle.fwd_t(dy, R, L, rd)], ["xM"])


@pytest.mark.parametrize("case", [c for c in SMALL if c[3] != c[5]][:5], ids=lambda c: c[0])
def test_alternative_mid_permutation(B, case):
    sh = small_shape(case)
    x, R, L, dy = synth.make_inputs(sh)
    f = B.MONARCH_FLAG_PERM_B
    y = run_fwd(B, sh, x, R, L, f)
    compare(sh, [y], [oracle.fwd(x, R, L, oracle.READING_B)], ["y"])
    got = run_bwd(B, sh, dy, x, R, L, f)
    compare(sh, got, oracle.bwd(dy, x, R, L, oracle.READING_B), ["dx", "dR", "dL"])


@pytest.mark.parametrize("m", [16])
def test_hadamard_is_bit_exact(B, m):
    """All blocks = Sylvester H_m gives M = H_n; with x in {-1,0,1} every value is an integer
    of magnitude <= n = 256, exact in fp32 and in bf16: the GPU must match bit for bit."""
    import scipy.linalg
    H = scipy.linalg.hadamard(m).astype(np.float32)
    R = np.broadcast_to(H, (m, m, m)).copy()
    rng = np.random.default_rng(1)
    x = rng.integers(-1, 2, size=(70, m * m)).astype(np.float32)
    want = oracle.fwd(x, R, R)
    for dtype in ("f32", "bf16"):
        sh = synth.Shape("hadamard", dtype, 70, m, m, m, m)
        for flags in (0, B.MONARCH_FLAG_GENERIC):
            assert np.array_equal(run_fwd(B, sh, x, R, R, flags), want)


def test_identity_blocks_and_empty_batch(B):
    m = 16
    eye = np.broadcast_to(np.eye(m, dtype=np.float32), (m, m, m)).copy()
    sh = synth.Shape("eye", "bf16", 9, m, m, m, m)
    x = synth.quantize(synth.normal(5, (9, m * m)), "bf16")
    assert np.array_equal(run_fwd(B, sh, x, eye, eye), x.astype(np.float64))
    # empty batch: forward is a no-op, backward zero-fills the weight gradients
    sh0 = synth.Shape("empty", "f32", 0, 4, 8, 8, 8)
    x0, R0, L0, dy0 = synth.make_inputs(sh0)
    assert run_fwd(B, sh0, x0, R0, L0).shape == (0, 32)
    dx, dR, dL = run_bwd(B, sh0, dy0, x0, R0, L0)
    assert dx.shape == (0, 32) and not dR.any() and not dL.any()


def test_backward_identities_on_gpu_outputs(B):
    """<dy, y> = <dx, x> = <dR, R> = <dL, L> must hold for the GPU results themselves."""
    sh = synth.Shape("euler", "f32", 300, 4, 32, 32, 48, config=77)
    x, R, L, dy = synth.make_inputs(sh)
    y = run_fwd(B, sh, x, R, L)
    dx, dR, dL = run_bwd(B, sh, dy, x, R, L)
    ref = np.sum(dy * y)
    for v in (np.sum(dx * x), np.sum(dR * R), np.sum(dL * L)):
        assert abs(v - ref) < 1e-4 * abs(ref)


@pytest.mark.parametrize("case", [("k4_192", "bf16", 1000, 4, 192, 192, 192), ("k4_fc1", "bf16", 700, 4, 64, 64, 128),
                                  ("sq_m64", "bf16", 300, 64, 64, 64, 64), ("sq_m16", "f32", 5000, 16, 16, 16, 16)],
                         ids=lambda c: c[0])
def test_matrix_core_backward_is_bit_reproducible(B, case):
    """The matrix-core backward sums its per-chunk partial gradients in a fixed order: two calls on the
    same inputs must agree bit for bit (dx, dR and dL), and so must two forward calls."""
    sh = small_shape(case)
    x, R, L, dy = synth.make_inputs(sh)
    a = run_bwd(B, sh, dy, x, R, L)
    b = run_bwd(B, sh, dy, x, R, L)
    for u, v, name in zip(a, b, ("dx", "dR", "dL")):
        assert np.array_equal(u, v), name
    assert np.array_equal(run_fwd(B, sh, x, R, L), run_fwd(B, sh, x, R, L))
    assert np.array_equal(run_fwd(B, sh, x, R, L, ws=True), run_fwd(B, sh, x, R, L, ws=True))


@pytest.mark.parametrize("case", [("k4_192", "bf16", 200, 4, 192, 192, 192), ("k4_fc1", "bf16", 130, 4, 64, 64, 128),
                                  ("sq_m64", "bf16", 70, 64, 64, 64, 64)], ids=lambda c: c[0])
def test_forward_reuses_packed_weights(B, case):
    """monarch_fwd_ws packs R and L into the workspace; a second call with MONARCH_FLAG_WS_PACKED on other
    rows must use those copies (R and L are passed as NaN to prove that they are not read)."""
    sh = small_shape(case)
    x, R, L, _ = synth.make_inputs(sh)
    x2 = synth.quantize(synth.normal(4242, x.shape), sh.dtype)
    code = 1
    need = B.monarch_fwd_workspace_bytes(x.shape[0], sh.n_in, sh.k, sh.q, sh.s, code, 0)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    Rd, Ld = dev(R, sh.dtype), dev(L, sh.dtype)
    y1 = B.monarch_fwd_ws(dev(x, sh.dtype), Rd, Ld, workspace=ws)
    nanR, nanL = torch.full_like(Rd, float("nan")), torch.full_like(Ld, float("nan"))
    y2 = B.monarch_fwd_ws(dev(x2, sh.dtype), nanR, nanL, workspace=ws, flags=B.MONARCH_FLAG_WS_PACKED)
    torch.cuda.synchronize()
    compare(sh, [host(y1), host(y2)], [oracle.fwd(x, R, L), oracle.fwd(x2, R, L)], ["y", "y_packed"])


FULL = ["sq256_f32", "vitb_proj", "gpt2s_fc1", "sq4096", "gpt2m_fc1", "gpt2m_fc2"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_workloads(B, name):
    """The five stated workloads at full size, in the launch configuration the benchmark times."""
    sh = synth.WORKLOADS[name]
    x, R, L, dy = synth.make_inputs(sh)
    code = 0 if sh.dtype == "f32" else 1
    print("\n  kernels: %s / %s" % (B.monarch_kernel_name(0, sh.n_in, sh.k, sh.q, sh.s, code),
                                    B.monarch_kernel_name(1, sh.n_in, sh.k, sh.q, sh.s, code)), flush=True)
    y = run_fwd(B, sh, x, R, L)
    yo = oracle.fwd(x, R, L)
    compare(sh, [y], [yo], ["y"])
    print("  forward with workspace: %s" % B.monarch_kernel_name(2, sh.n_in, sh.k, sh.q, sh.s, code), flush=True)
    compare(sh, [run_fwd(B, sh, x, R, L, ws=True)], [yo], ["y_ws"])
    got = run_bwd(B, sh, dy, x, R, L)
    want = oracle.bwd(dy, x, R, L)
    compare(sh, got, want, ["dx", "dR", "dL"])
    # properties that hold at any size, on the GPU outputs
    ref = np.sum(dy * y)
    assert abs(np.sum(got[0] * x) - ref) < 2e-2 * abs(ref) + 1e-2 * np.sqrt(x.size)


def test_mlp_pair_end_to_end(B):
    """GPT-2-medium-style pair 1024 -> 4096 -> 1024 (no nonlinearity between the two multiplies):
    GPU chain (hidden activation stored in bf16) against the oracle chain in fp64."""
    s1, s2 = synth.WORKLOADS["gpt2m_fc1"], synth.WORKLOADS["gpt2m_fc2"]
    rows = 2048
    x, R1, L1, _ = synth.make_inputs(s1, rows=rows)
    _, R2, L2, dy = synth.make_inputs(s2, rows=rows)
    dt = torch.bfloat16
    xd, R1d, L1d, R2d, L2d, dyd = (dev(a, "bf16") for a in (x, R1, L1, R2, L2, dy))
    h = B.monarch_fwd(xd, R1d, L1d)
    y = B.monarch_fwd(h, R2d, L2d)
    dh, dR2, dL2 = B.monarch_bwd(dyd, h, R2d, L2d)
    dx, dR1, dL1 = B.monarch_bwd(dh, xd, R1d, L1d)
    torch.cuda.synchronize()
    assert h.dtype == dt
    ho = oracle.fwd(x, R1, L1)
    yo = oracle.fwd(ho, R2, L2)
    dho, dR2o, dL2o = oracle.bwd(dy, ho, R2, L2)
    dxo, dR1o, dL1o = oracle.bwd(dho, x, R1, L1)
    sh = synth.Shape("mlp_pair", "bf16", rows, 4, 256, 256, 1024)
    compare(sh, [host(t) for t in (h, y, dh, dR2, dL2, dx, dR1, dL1)],
            [ho, yo, dho, dR2o, dL2o, dxo, dR1o, dL1o],
            ["h", "y", "dh", "dR2", "dL2", "dx", "dR1", "dL1"])


# ---------------------------------------------------------------- affine layer ----

def run_fwd_bias(B, sh, x, R, L, bias, flags=0):
    ybuf, y = guarded((x.shape[0], sh.n_out), tdtype(sh.dtype))
    code = 0 if sh.dtype == "f32" else 1
    need = B.monarch_fwd_workspace_bytes(x.shape[0], sh.n_in, sh.k, sh.q, sh.s, code, flags)
    wbuf = torch.full((need + 512 + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    off = (-(wbuf.data_ptr() + GUARD)) % 256 + GUARD
    B.monarch_fwd_bias(dev(x, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype), dev(bias, sh.dtype), y,
                       workspace=wbuf[off:off + need] if need else None, flags=flags)
    torch.cuda.synchronize()
    assert bool((wbuf[:off] == 0x5A).all()) and bool((wbuf[off + need:] == 0x5A).all()), "workspace: wrote out of bounds"
    check_guard(ybuf, "y")
    out = host(y)
    assert np.isfinite(out).all(), "y has unwritten or non-finite entries"
    return out


def run_bwd_bias(B, sh, dy, x, R, L, flags=0):
    dt = tdtype(sh.dtype)
    gdt = torch.float32 if (flags & B.MONARCH_FLAG_WGRAD_F32) else dt
    bx, dx = guarded((x.shape[0], sh.n_in), dt)
    bR, dR = guarded(R.shape, gdt)
    bL, dL = guarded(L.shape, gdt)
    bb, db = guarded((sh.n_out,), gdt)
    B.monarch_bwd_bias(dev(dy, sh.dtype), dev(x, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype), dx, dR, dL, db, flags=flags)
    torch.cuda.synchronize()
    for buf, name in ((bx, "dx"), (bR, "dR"), (bL, "dL"), (bb, "dbias")):
        check_guard(buf, name)
    outs = [host(t) for t in (dx, dR, dL, db)]
    for o, name in zip(outs, ("dx", "dR", "dL", "dbias")):
        assert np.isfinite(o).all(), name + " has unwritten or non-finite entries"
    return outs


def make_bias(sh):
    return synth.quantize(synth.normal(synth.tensor_seed(sh.config, "x") + 991, (sh.n_out,)), sh.dtype)


@pytest.mark.parametrize("generic", [False, True], ids=["dispatch", "generic"])
@pytest.mark.parametrize("case", SMALL + [("odd_n_out", "f32", 300, 3, 4, 5, 7), ("odd_n_out_bf16", "bf16", 130, 3, 4, 5, 7)],
                         ids=lambda c: c[0])
def test_affine_layer_small_shapes(B, case, generic):
    """monarch_fwd_bias / monarch_bwd_bias against the oracle's affine layer (bias of unit variance)."""
    sh = small_shape(case)
    flags = B.MONARCH_FLAG_GENERIC if generic else 0
    x, R, L, dy = synth.make_inputs(sh)
    bias = make_bias(sh)
    y = run_fwd_bias(B, sh, x, R, L, bias, flags)
    compare(sh, [y], [oracle.fwd_bias(x, R, L, bias)], ["y"])
    want = oracle.bwd_bias(dy, x, R, L)
    compare(sh, run_bwd_bias(B, sh, dy, x, R, L, flags), want, ["dx", "dR", "dL", "dbias"])
    got32 = run_bwd_bias(B, sh, dy, x, R, L, flags | B.MONARCH_FLAG_WGRAD_F32)
    compare(sh, got32, want, ["dx", "dR32", "dL32", "dbias32"])
    # fp32 bias gradient: a sum of B exactly representable values in fp32, error far below the storage rounding
    assert oracle.rel_fro(got32[3], want[3]) <= 1e-5


def test_affine_layer_edge_cases(B):
    # x = 0: every output row is the bias, bit for bit (0 + bias is exact)
    for case in (("k4_192", "bf16", 70, 4, 192, 192, 192), ("sq_m16", "f32", 33, 16, 16, 16, 16), ("rect", "f32", 5, 3, 2, 6, 5),
                 ("sq_m64", "bf16", 33, 64, 64, 64, 64)):
        sh = small_shape(case)
        x, R, L, dy = synth.make_inputs(sh)
        bias = make_bias(sh)
        y = run_fwd_bias(B, sh, np.zeros_like(x), R, L, bias)
        assert np.array_equal(y, np.tile(bias.astype(np.float64), (sh.B, 1))), sh.name
        # all-ones upstream gradient: the bias gradient counts the rows
        db = run_bwd_bias(B, sh, np.ones_like(dy), x, R, L, B.MONARCH_FLAG_WGRAD_F32)[3]
        assert np.array_equal(db, np.full(sh.n_out, float(sh.B))), sh.name
    # empty batch: the bias gradient is zero-filled like the weight gradients
    sh0 = synth.Shape("empty", "f32", 0, 4, 8, 8, 8)
    x0, R0, L0, dy0 = synth.make_inputs(sh0)
    assert run_fwd_bias(B, sh0, x0, R0, L0, make_bias(sh0)).shape == (0, 32)
    dx, dR, dL, db = run_bwd_bias(B, sh0, dy0, x0, R0, L0)
    assert not dR.any() and not dL.any() and not db.any()
    # packed weights left in the workspace are reused with a different bias
    sh = small_shape(("k4_192", "bf16", 200, 4, 192, 192, 192))
    x, R, L, _ = synth.make_inputs(sh)
    need = B.monarch_fwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, 1)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    b1, b2 = make_bias(sh), -make_bias(sh)
    y1 = B.monarch_fwd_bias(dev(x, "bf16"), dev(R, "bf16"), dev(L, "bf16"), dev(b1, "bf16"), workspace=ws)
    nanw = torch.full(R.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    y2 = B.monarch_fwd_bias(dev(x, "bf16"), nanw, nanw.clone(), dev(b2, "bf16"), workspace=ws, flags=B.MONARCH_FLAG_WS_PACKED)
    torch.cuda.synchronize()
    compare(sh, [host(y1), host(y2)], [oracle.fwd_bias(x, R, L, b1), oracle.fwd_bias(x, R, L, b2)], ["y1", "y2"])


@pytest.mark.parametrize("name", FULL)
def test_affine_layer_full_size(B, name):
    sh = synth.WORKLOADS[name]
    x, R, L, dy = synth.make_inputs(sh)
    bias = make_bias(sh)
    y = run_fwd_bias(B, sh, x, R, L, bias)
    compare(sh, [y], [oracle.fwd_bias(x, R, L, bias)], ["y"])
    got = run_bwd_bias(B, sh, dy, x, R, L)
    compare(sh, got, oracle.bwd_bias(dy, x, R, L), ["dx", "dR", "dL", "dbias"])


# ---------------------------------------------------------------- layer with the block's nonlinearity ----

def run_fwd_gelu(B, sh, x, R, L, bias, flags=0, want_pre=True):
    """monarch_fwd_bias_gelu with guarded outputs and workspace: (y_pre or None, y) on the host."""
    dt = tdtype(sh.dtype)
    ybuf, y = guarded((x.shape[0], sh.n_out), dt)
    pbuf, y_pre = guarded((x.shape[0], sh.n_out), dt) if want_pre else (None, None)
    code = 0 if sh.dtype == "f32" else 1
    need = B.monarch_fwd_workspace_bytes(x.shape[0], sh.n_in, sh.k, sh.q, sh.s, code, flags)
    wbuf = torch.full((need + 512 + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    off = (-(wbuf.data_ptr() + GUARD)) % 256 + GUARD
    B.monarch_fwd_bias_gelu(dev(x, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype),
                            dev(bias, sh.dtype) if bias is not None else None, y_pre, y, want_pre=want_pre,
                            workspace=wbuf[off:off + need] if need else None, flags=flags)
    torch.cuda.synchronize()
    assert bool((wbuf[:off] == 0x5A).all()) and bool((wbuf[off + need:] == 0x5A).all()), "workspace: wrote out of bounds"
    check_guard(ybuf, "y")
    outs = [host(y)]
    if want_pre:
        check_guard(pbuf, "y_pre")
        outs.insert(0, host(y_pre))
    for o in outs:
        assert np.isfinite(o).all(), "an output has unwritten or non-finite entries"
    return outs if want_pre else [None] + outs


def run_bwd_gelu_in(B, sh, dy, x, x_pre, R, L, flags=0):
    dt = tdtype(sh.dtype)
    gdt = torch.float32 if (flags & B.MONARCH_FLAG_WGRAD_F32) else dt
    bx, dx = guarded((x.shape[0], sh.n_in), dt)
    bR, dR = guarded(R.shape, gdt)
    bL, dL = guarded(L.shape, gdt)
    bb, db = guarded((sh.n_out,), gdt)
    B.monarch_bwd_bias_gelu_in(dev(dy, sh.dtype), dev(x, sh.dtype), dev(x_pre, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype),
                               dx, dR, dL, db, flags=flags)
    torch.cuda.synchronize()
    for buf, name in ((bx, "dx_pre"), (bR, "dR"), (bL, "dL"), (bb, "dbias")):
        check_guard(buf, name)
    outs = [host(t) for t in (dx, dR, dL, db)]
    for o, name in zip(outs, ("dx_pre", "dR", "dL", "dbias")):
        assert np.isfinite(o).all(), name + " has unwritten or non-finite entries"
    return outs


def gelu_layer_case(B, sh, flags=0):
    """Both calls of one shape against the oracle: the layer as a block's first layer (forward) and as its
    second (backward, its input being gelu of a stored pre-activation)."""
    from oracle import activation
    x, R, L, dy = synth.make_inputs(sh)
    bias = make_bias(sh)
    want_pre, want_y = activation.fwd_bias_gelu(x, R, L, bias)
    compare(sh, run_fwd_gelu(B, sh, x, R, L, bias, flags), [want_pre, want_y], ["y_pre", "y"])
    # the layer's input as a first layer would have stored it: pre-activation x, activation gelu(x), both rounded
    xin = synth.quantize(activation.gelu(x), sh.dtype)
    want = activation.bwd_bias_gelu_in(dy, x, R, L, x=xin)
    compare(sh, run_bwd_gelu_in(B, sh, dy, xin, x, R, L, flags), want, ["dx_pre", "dR", "dL", "dbias"])


@pytest.mark.parametrize("generic", [False, True], ids=["dispatch", "generic"])
@pytest.mark.parametrize("case", SMALL + [("odd_n_out", "f32", 300, 3, 4, 5, 7), ("odd_n_out_bf16", "bf16", 130, 3, 4, 5, 7)],
                         ids=lambda c: c[0])
def test_layer_with_nonlinearity_small_shapes(B, case, generic):
    """monarch_fwd_bias_gelu / monarch_bwd_bias_gelu_in against oracle.activation: the fused epilogues (bf16, k = 4)
    and the separate elementwise passes (every other shape, and everything under MONARCH_FLAG_GENERIC)."""
    gelu_layer_case(B, small_shape(case), B.MONARCH_FLAG_GENERIC if generic else 0)


@pytest.mark.parametrize("case", MODEL_LAYERS, ids=lambda c: c[0])
def test_layer_with_nonlinearity_model_layer_shapes(B, case):
    name, dtype, Bn, k, p, q, s = case[:7]
    gelu_layer_case(B, synth.Shape(name, dtype, min(Bn, 333), k, p, q, s, config=70 + parity_util.stable_seed(name)))


def test_layer_with_nonlinearity_edge_cases(B):
    from oracle import activation
    for case in (("k4_192", "bf16", 70, 4, 192, 192, 192), ("sq_m16", "f32", 33, 16, 16, 16, 16), ("rect", "f32", 5, 3, 2, 6, 5)):
        sh = small_shape(case)
        x, R, L, dy = synth.make_inputs(sh)
        bias = make_bias(sh)
        # no bias; and no pre-activation output: the same y bit for bit
        want_pre, want_y = activation.fwd_bias_gelu(x, R, L, np.zeros(sh.n_out))
        pre, y = run_fwd_gelu(B, sh, x, R, L, None)
        compare(sh, [pre, y], [want_pre, want_y], ["y_pre_nobias", "y_nobias"])
        _, y2 = run_fwd_gelu(B, sh, x, R, L, None, want_pre=False)
        assert np.array_equal(y, y2), sh.name
        # x = 0: every row is gelu(bias); a large negative bias gives exact zeros, a large positive one the bias itself
        big = np.where(np.arange(sh.n_out) % 2 == 0, 40.0, -40.0)
        pre, y = run_fwd_gelu(B, sh, np.zeros_like(x), R, L, big)
        assert np.array_equal(pre, np.tile(big, (sh.B, 1))) and np.array_equal(y, np.tile(np.maximum(big, 0.0), (sh.B, 1))), sh.name
        # backward at x_pre = 0: gelu'(0) = 1/2 exactly, so dx_pre is half the plain dx (a power of two: same rounding)
        zeros = np.zeros_like(x)
        dxh = run_bwd_gelu_in(B, sh, dy, zeros, zeros, R, L)[0]
        dx = run_bwd_bias(B, sh, dy, zeros, R, L)[0]
        assert np.array_equal(dxh, 0.5 * dx), sh.name
    sh0 = synth.Shape("empty", "bf16", 0, 4, 64, 64, 64)
    x0, R0, L0, dy0 = synth.make_inputs(sh0)
    assert run_fwd_gelu(B, sh0, x0, R0, L0, make_bias(sh0))[1].shape == (0, 256)
    dx, dR, dL, db = run_bwd_gelu_in(B, sh0, dy0, x0, x0, R0, L0)
    assert dx.shape == (0, 256) and not dR.any() and not dL.any() and not db.any()


@pytest.mark.parametrize("name", ["sq256_f32", "vitb_proj", "sq4096", "gpt2m_fc1", "gpt2m_fc2"])
def test_layer_with_nonlinearity_full_size(B, name):
    gelu_layer_case(B, synth.WORKLOADS[name])


def test_feed_forward_block_end_to_end(B):
    """GPT-2-medium-style block 1024 -> 4096 -> gelu -> 1024 with biases, forward and backward through the four
    layer calls, against the oracle's chain in fp64 (2048 rows)."""
    from oracle import activation
    s1, s2 = synth.WORKLOADS["gpt2m_fc1"], synth.WORKLOADS["gpt2m_fc2"]
    rows = 2048
    x, R1, L1, _ = synth.make_inputs(s1, rows=rows)
    _, R2, L2, dy = synth.make_inputs(s2, rows=rows)
    b1, b2 = make_bias(s1), make_bias(s2)
    xd, R1d, L1d, R2d, L2d, dyd, b1d, b2d = (dev(a, "bf16") for a in (x, R1, L1, R2, L2, dy, b1, b2))
    h, g = B.monarch_fwd_bias_gelu(xd, R1d, L1d, b1d)
    y = B.monarch_fwd_bias(g, R2d, L2d, b2d)
    dh, dR2, dL2, db2 = B.monarch_bwd_bias_gelu_in(dyd, g, h, R2d, L2d)
    dx, dR1, dL1, db1 = B.monarch_bwd_bias(dh, xd, R1d, L1d)
    torch.cuda.synchronize()
    ho, go = activation.fwd_bias_gelu(x, R1, L1, b1)
    yo = oracle.fwd_bias(go, R2, L2, b2)
    dho, dR2o, dL2o, db2o = activation.bwd_bias_gelu_in(dy, ho, R2, L2)
    dxo, dR1o, dL1o, db1o = oracle.bwd_bias(dho, x, R1, L1)
    sh = synth.Shape("ffn_block", "bf16", rows, 4, 256, 256, 1024)
    compare(sh, [host(t) for t in (h, g, y, dh, dR2, dL2, db2, dx, dR1, dL1, db1)],
            [ho, go, yo, dho, dR2o, dL2o, db2o, dxo, dR1o, dL1o, db1o],
            ["h", "g", "y", "dh", "dR2", "dL2", "db2", "dx", "dR1", "dL1", "db1"])


# Dense form of M: every entry is one fp32 sum of at most q products, rounded once to the storage type
# (relative 2^-24 / 2^-9 per entry), so the bound is much tighter than for the multiply.
DENSE_TOL = {"f32": 1e-6, "bf16": 3e-3}
DENSE_EXTRA = [
    ("k_gt_q", "f32", 9, 5, 3, 2, 3),          # k > q: some (kk, c) pairs have no term at all
    ("ragged_cols", "f32", 9, 3, 100, 7, 5),   # n_in = 300: a partial tile of columns, s not a multiple of 4
    ("ragged_cols_bf16", "bf16", 9, 6, 50, 4, 9),
    ("long_sums_odd_p", "f32", 9, 2, 5, 40, 3),  # q/k = 20 terms split over the waves of a workgroup, p % 4 != 0
]


def run_dense(B, sh, R, L, flags=0):
    buf, M = guarded((sh.n_out, sh.n_in), tdtype(sh.dtype))
    B.monarch_to_dense(dev(R, sh.dtype), dev(L, sh.dtype), M, flags=flags)
    torch.cuda.synchronize()
    check_guard(buf, "M")
    out = host(M)
    assert np.isfinite(out).all(), "M has unwritten or non-finite entries"
    return out


@pytest.mark.parametrize("reading", [0, 1], ids=["reading_a", "reading_b"])
@pytest.mark.parametrize("case", [c for c in SMALL if c[0] != "sq_m64_bf16"] + DENSE_EXTRA, ids=lambda c: c[0])
def test_dense_form_small_shapes(B, case, reading):
    """monarch_to_dense against the literal product of the four dense matrices of Definition 3.1."""
    from oracle import dense
    sh = small_shape(case)
    x, R, L, _ = synth.make_inputs(sh)
    got = run_dense(B, sh, R, L, B.MONARCH_FLAG_PERM_B if reading else 0)
    want = dense.monarch_dense(R, L, reading)
    err = oracle.rel_fro(got, want)
    print("\n  %s M=%.2e" % (sh.name, err), flush=True)
    assert err <= DENSE_TOL[sh.dtype]
    assert np.all(got[want == 0] == 0), "an entry outside the sparsity pattern of M is not zero"
    # and it is the matrix the step-by-step multiply applies: y = x M^T
    assert oracle.rel_fro(x.astype(np.float64) @ got.T, oracle.fwd(x, R, L, reading)) <= TOL[sh.dtype]


@pytest.mark.parametrize("name", FULL)
def test_dense_form_full_size(B, name):
    """Full-size factors: row col of M^T is the oracle's forward applied to the unit vector e_col."""
    sh = synth.WORKLOADS[name]
    _, R, L, _ = synth.make_inputs(sh, rows=1)
    got = run_dense(B, sh, R, L)
    want = oracle.fwd(np.eye(sh.n_in, dtype=np.float32), R, L).T
    err = oracle.rel_fro(got, want)
    print("\n  %s M=%.2e" % (sh.name, err), flush=True)
    assert err <= DENSE_TOL[sh.dtype]
    assert np.all(got[want == 0] == 0)
    if sh.k == sh.q == sh.s == sh.p:  # Equation (1), sampled entries
        m = sh.k
        rng = np.random.default_rng(5)
        for l, j, kk, i in rng.integers(0, m, size=(200, 4)):
            ref = np.float64(L[j, l, kk]) * np.float64(R[kk, j, i])
            assert abs(got[l * m + j, kk * m + i] - ref) <= 2.0 ** -8 * abs(ref) + 1e-30


def test_random_small_shapes_every_entry_point(B):
    """Seeded sweep over shapes nobody tuned for (k, p, q, s in 1..12, odd sizes, both readings, both
    storage types): every entry point against the oracle."""
    from oracle import dense
    rng = np.random.default_rng(20240595)
    for it in range(24):
        k, p, q, s = (int(v) for v in rng.integers(1, 13, size=4))
        rows = int(rng.integers(1, 150))
        dtype = "bf16" if it % 2 else "f32"
        reading = int(rng.integers(0, 2))
        flags = B.MONARCH_FLAG_PERM_B if reading else 0
        sh = synth.Shape("sweep%d_k%d_p%d_q%d_s%d_%s_r%d" % (it, k, p, q, s, dtype, reading), dtype, rows, k, p, q, s, config=40 + it)
        print("\n  " + sh.name, flush=True)
        x, R, L, dy = synth.make_inputs(sh)
        bias = make_bias(sh)
        compare(sh, [run_fwd(B, sh, x, R, L, flags), run_fwd_bias(B, sh, x, R, L, bias, flags)],
                [oracle.fwd(x, R, L, reading), oracle.fwd_bias(x, R, L, bias, reading)], ["y", "y_bias"])
        compare(sh, run_bwd_bias(B, sh, dy, x, R, L, flags), oracle.bwd_bias(dy, x, R, L, reading), ["dx", "dR", "dL", "dbias"])
        M = run_dense(B, sh, R, L, flags)
        assert oracle.rel_fro(M, dense.monarch_dense(R, L, reading)) <= DENSE_TOL[dtype]


def test_rows_beyond_two_to_the_31_elements(B):
    """Maximum size: a batch whose activations hold more than 2^31 elements (fp32 m = 16 kernels,
    B = 2^23 + 21 rows of 256).  Sampled rows, including the last ones, against the oracle; the
    weight gradients through the identity <dR, R> = <dL, L> = <dy, y>, which holds at any size."""
    sh = synth.Shape("huge", "f32", (1 << 23) + 21, 16, 16, 16, 16, config=1)
    blk = 1 << 16
    xb, R, L, dyb = synth.make_inputs(sh, rows=blk)
    reps = -(-sh.B // blk)
    ramp = (torch.arange(sh.B, device="cuda", dtype=torch.float32) % 1009.0).mul_(1.0 / 1024).unsqueeze(1)
    x = torch.from_numpy(xb).cuda().repeat(reps, 1)[:sh.B].contiguous().add_(ramp)    # every row differs from its
    dy = torch.from_numpy(dyb).cuda().repeat(reps, 1)[:sh.B].contiguous().sub_(ramp)  # copies 65536 rows away
    del ramp
    Rd, Ld = dev(R, "f32"), dev(L, "f32")
    assert x.numel() > 2 ** 31
    y = B.monarch_fwd(x, Rd, Ld)
    dx, dR, dL = B.monarch_bwd(dy, x, Rd, Ld)
    torch.cuda.synchronize()
    rows = torch.tensor([0, 1, 17, blk - 1, blk, 3 * blk + 5, (1 << 23) - 1, 1 << 23, sh.B - 2, sh.B - 1], device="cuda")
    xs, dys = x[rows].cpu().numpy(), dy[rows].cpu().numpy()
    compare(sh, [host(y[rows]), host(dx[rows])], [oracle.fwd(xs, R, L), oracle.bwd(dys, xs, R, L)[0]], ["y_rows", "dx_rows"])
    ref = float((dy.double() * y.double()).sum())
    for name, g, w in (("dR", dR, Rd), ("dL", dL, Ld)):
        v = float((g.double() * w.double()).sum())
        print("  <%s, weight> = %.6e, <dy, y> = %.6e" % (name, v, ref), flush=True)
        assert abs(v - ref) <= 1e-4 * abs(ref), name


# --------------------------------------------- forward that saves, backward that reuses ----

@pytest.mark.parametrize("case", [("k4_192", "bf16", 200, 4, 192, 192, 192), ("k4_64_128", "bf16", 97, 4, 64, 64, 128),
                                  ("k4_128_64", "bf16", 65, 4, 128, 64, 64)] + MODEL_LAYERS +
                         [("sq_m64", "bf16", 40, 64, 64, 64, 64), ("sq_m16", "f32", 70, 16, 16, 16, 16), ("rect", "f32", 19, 3, 2, 6, 5)],
                         ids=lambda c: c[0])
def test_saved_intermediate_forward_and_backward(B, case):
    """monarch_fwd_save gives the same y as monarch_fwd; monarch_bwd_saved, fed its buffer, gives the
    gradients of the recomputing backward (against the oracle; dx and dR even bit for bit: their path
    does not change).  Shapes without the path fall back to the plain calls."""
    sh = small_shape(case)
    code = 0 if sh.dtype == "f32" else 1
    x, R, L, dy = synth.make_inputs(sh)
    xd, Rd, Ld, dyd = (dev(a, sh.dtype) for a in (x, R, L, dy))
    need = B.monarch_saved_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code)
    assert (need > 0) == (sh.k == 4 and sh.dtype == "bf16")
    sbuf = torch.full((need + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    saved = sbuf[GUARD:GUARD + need] if need else None
    ybuf, y = guarded((sh.B, sh.n_out), tdtype(sh.dtype))
    B.monarch_fwd_save(xd, Rd, Ld, y, saved)
    torch.cuda.synchronize()
    check_guard(ybuf, "y")
    assert bool((sbuf[:GUARD] == 0x5A).all()) and bool((sbuf[GUARD + need:] == 0x5A).all()), "saved: wrote out of bounds"
    assert torch.equal(y, B.monarch_fwd(xd, Rd, Ld))
    compare(sh, [host(y)], [oracle.fwd(x, R, L)], ["y"])
    want = oracle.bwd_bias(dy, x, R, L)
    plain = B.monarch_bwd_bias(dyd, xd, Rd, Ld)
    got = B.monarch_bwd_saved(dyd, xd, saved, Rd, Ld, want_dbias=True)
    torch.cuda.synchronize()
    compare(sh, [host(t) for t in got], want, ["dx", "dR", "dL", "dbias"])
    if need:
        assert torch.equal(got[0], plain[0]) and torch.equal(got[1], plain[1]) and torch.equal(got[3], plain[3])
        # a NULL buffer means "recompute"
        again = B.monarch_bwd_saved(dyd, xd, None, Rd, Ld)
        assert all(torch.equal(a, b) for a, b in zip(again[:3], plain[:3]))
    got32 = B.monarch_bwd_saved(dyd, xd, saved, Rd, Ld, flags=B.MONARCH_FLAG_WGRAD_F32)
    compare(sh, [host(t) for t in got32[:3]], want[:3], ["dx", "dR32", "dL32"])


@pytest.mark.parametrize("name", ["vitb_proj", "gpt2s_fc1", "gpt2m_fc1", "gpt2m_fc2"])
def test_saved_intermediate_full_size(B, name):
    sh = synth.WORKLOADS[name]
    x, R, L, dy = synth.make_inputs(sh)
    xd, Rd, Ld, dyd = (dev(a, sh.dtype) for a in (x, R, L, dy))
    y, saved = B.monarch_fwd_save(xd, Rd, Ld)
    got = B.monarch_bwd_saved(dyd, xd, saved, Rd, Ld)
    torch.cuda.synchronize()
    compare(sh, [host(y)] + [host(t) for t in got[:3]], [oracle.fwd(x, R, L)] + list(oracle.bwd(dy, x, R, L)), ["y", "dx", "dR", "dL"])


# ------------------------------------------------------ transposed multiply (M*) ----

def run_fwd_t(B, sh, xin, R, L, flags=0):
    """monarch_fwd_t with guarded output and a guarded, 256-byte aligned workspace."""
    ybuf, y = guarded((xin.shape[0], sh.n_in), tdtype(sh.dtype))
    code = 0 if sh.dtype == "f32" else 1
    need = B.monarch_fwd_t_workspace_bytes(xin.shape[0], sh.n_in, sh.k, sh.q, sh.s, code, flags)
    wbuf = torch.full((need + 512 + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    off = (-(wbuf.data_ptr() + GUARD)) % 256 + GUARD
    B.monarch_fwd_t(dev(xin, sh.dtype), dev(R, sh.dtype), dev(L, sh.dtype), y, workspace=wbuf[off:off + need] if need else None, flags=flags)
    torch.cuda.synchronize()
    assert bool((wbuf[:off] == 0x5A).all()) and bool((wbuf[off + need:] == 0x5A).all()), "workspace: wrote out of bounds"
    check_guard(ybuf, "y")
    out = host(y)
    assert np.isfinite(out).all(), "y has unwritten or non-finite entries"
    return out


@pytest.mark.parametrize("generic", [False, True], ids=["dispatch", "generic"])
@pytest.mark.parametrize("case", SMALL + MODEL_LAYERS + [c[:7] for c in TILED], ids=lambda c: c[0])
def test_transposed_multiply_small_shapes(B, case, generic):
    sh = small_shape(case)
    if case[0] in [c[0] for c in TILED] and not generic:
        assert B.monarch_kernel_name(3, sh.n_in, sh.k, sh.q, sh.s, 1, 0) == "mfma_fwd_t_tiled_bf16"
    flags = B.MONARCH_FLAG_GENERIC if generic else 0
    _, R, L, xin = synth.make_inputs(sh)  # the upstream-gradient tensor has the input shape of x M
    print("\n  kernel: %s" % B.monarch_kernel_name(3, sh.n_in, sh.k, sh.q, sh.s, 0 if sh.dtype == "f32" else 1, flags), flush=True)
    compare(sh, [run_fwd_t(B, sh, xin, R, L, flags)], [oracle.fwd_t(xin, R, L)], ["xM"])
    if sh.k != sh.q:
        f = flags | B.MONARCH_FLAG_PERM_B
        compare(sh, [run_fwd_t(B, sh, xin, R, L, f)], [oracle.fwd_t(xin, R, L, oracle.READING_B)], ["xM_reading_b"])
    sh0 = synth.Shape("empty", sh.dtype, 0, sh.k, sh.p, sh.q, sh.s)
    assert run_fwd_t(B, sh0, xin[:0], R, L, flags).shape == (0, sh.n_in)


@pytest.mark.parametrize("name", FULL)
def test_transposed_multiply_full_size(B, name):
    sh = synth.WORKLOADS[name]
    z, R, L, xin = synth.make_inputs(sh)
    got = run_fwd_t(B, sh, xin, R, L)
    compare(sh, [got], [oracle.fwd_t(xin, R, L)], ["xM"])
    # adjoint of the multiply, on GPU outputs: <x M, z> = <x, z M^T>
    y = run_fwd(B, sh, z, R, L)
    lhs, rhs = np.sum(got * z), np.sum(xin * y)
    assert abs(lhs - rhs) < 2e-2 * abs(rhs) + 1e-2 * np.sqrt(z.size)


def test_hadamard_monarch_times_its_transpose_is_n_times_identity_on_gpu(B):
    """M = H_256 (all blocks Sylvester H_16): M* then M multiplies small-integer vectors by 256 exactly
    (the Hadamard transform is in MM*, Proposition 3.2)."""
    import scipy.linalg
    m = 16
    H = scipy.linalg.hadamard(m).astype(np.float32)
    blocks = np.broadcast_to(H, (m, m, m)).copy()
    sh = synth.Shape("hadamard_mm", "f32", 70, m, m, m, m)
    x = np.random.default_rng(3).integers(-3, 4, size=(70, m * m)).astype(np.float32)
    z = run_fwd_t(B, sh, x, blocks, blocks)
    assert np.array_equal(z, x.astype(np.float64) @ scipy.linalg.hadamard(m * m).astype(np.float64))
    assert np.array_equal(run_fwd(B, sh, z.astype(np.float32), blocks, blocks), 256.0 * x)


# ------------------------------------------------------------- complex-valued ----

def cdev(a):
    return torch.from_numpy(np.ascontiguousarray(a.astype(np.complex64))).cuda()


def cnormal(seed, shape, std=1.0):
    """Complex Gaussian with fp32-representable parts (both sides consume the same complex64 values)."""
    return (synth.normal(seed, shape, std) + 1j * synth.normal(seed + 1, shape, std)).astype(np.complex64)


COMPLEX_CASES = [("c_sq4", 9, 4, 4, 4, 4), ("c_sq16", 70, 16, 16, 16, 16), ("c_rect", 33, 3, 4, 5, 2), ("c_k4", 130, 4, 32, 32, 48),
                 ("c_one_row", 1, 2, 3, 4, 2), ("c_wide", 77, 2, 70, 130, 66), ("c_sq64", 21, 64, 64, 64, 64),
                 # square blocks of 16 / 32 / 64 with a block count that is not the block size, and batches long enough
                 # that a workgroup of the matrix-core kernels takes several row tiles (the last one ragged)
                 ("c_m32", 100, 32, 32, 32, 32), ("c_k3_m64", 67, 3, 64, 64, 64), ("c_k5_m16", 200, 5, 16, 16, 16),
                 ("c_m32_long", 8219, 8, 32, 32, 32), ("c_m64_long", 16421, 2, 64, 64, 64), ("c_m16_long", 33003, 4, 16, 16, 16)]


def guarded_workspace(need):
    """(buffer, view): `need` bytes, 256-byte aligned, between two runs of canary bytes."""
    wbuf = torch.full((need + 512 + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    off = (-(wbuf.data_ptr() + GUARD)) % 256 + GUARD
    return wbuf, off, wbuf[off:off + need]


def workspace_untouched_outside(wbuf, off, need):
    return bool((wbuf[:off] == 0x5A).all()) and bool((wbuf[off + need:] == 0x5A).all())


@pytest.mark.parametrize("reading", [0, 1], ids=["reading_a", "reading_b"])
@pytest.mark.parametrize("case", COMPLEX_CASES, ids=lambda c: c[0])
def test_complex_forward_and_backward(B, case, reading):
    from oracle import complex_ref
    name, rows, k, p, q, s = case
    x, R, L, dy = (cnormal(8000 + 10 * i, shp, std) for i, (shp, std) in enumerate(
        (((rows, k * p), 1.0), ((k, q, p), p ** -0.5), ((k, s, q), q ** -0.5), ((rows, k * s), 1.0))))
    flags = B.MONARCH_FLAG_PERM_B if reading else 0
    xd, Rd, Ld, dyd = cdev(x), cdev(R), cdev(L), cdev(dy)
    y = B.monarch_fwd_c64(xd, Rd, Ld, flags=flags)
    dx, dR, dL = B.monarch_bwd_c64(dyd, xd, Rd, Ld, flags=flags)
    torch.cuda.synchronize()
    yh = B.monarch_fwd_h_c64(dyd, Rd, Ld, flags=flags)   # conjugate transpose applied to the rows of dy
    # the same three calls with a (guarded) workspace: matrix-core kernels for the square blocks of 16 / 32 / 64,
    # elsewhere the same data kernels and the weight gradients by a batch-contracted GEMM
    outs_ws = []
    for pass_, call in ((B.C64_FWD, lambda w: (B.monarch_fwd_c64_ws(xd, Rd, Ld, workspace=w, flags=flags),)),
                        (B.C64_BWD, lambda w: B.monarch_bwd_c64_ws(dyd, xd, Rd, Ld, workspace=w, flags=flags)),
                        (B.C64_FWD_H, lambda w: (B.monarch_fwd_h_c64_ws(dyd, Rd, Ld, workspace=w, flags=flags),))):
        need = B.monarch_c64_workspace_bytes(pass_, rows, k * p, k, q, s, flags)
        wbuf, off, view = guarded_workspace(need)
        print("\n  %s pass %d workspace %d bytes" % (name, pass_, need), flush=True)
        outs_ws += list(call(view))
        torch.cuda.synchronize()
        assert workspace_untouched_outside(wbuf, off, need), "workspace: wrote out of bounds (pass %d)" % pass_
    on_matrix_cores = p == q == s and p in (16, 32, 64)
    if not on_matrix_cores:
        assert torch.equal(outs_ws[0], y) and torch.equal(outs_ws[1], dx) and torch.equal(outs_ws[4], yh), \
            "the data path is the same kernel code with or without the workspace"
    ref = list(complex_ref.bwd(dy, x, R, L, reading))
    y_ref, yh_ref = complex_ref.fwd(x, R, L, reading), complex_ref.fwd_h(dy, R, L, reading)
    want = [y_ref] + ref + [yh_ref] + [y_ref] + ref + [yh_ref]
    names = ("y", "dx", "dR", "dL", "xMh", "y_ws", "dx_ws", "dR_ws", "dL_ws", "xMh_ws")
    errs = {}
    for nm, got, w in zip(names, [y, dx, dR, dL, yh] + outs_ws, want):
        g = got.cpu().numpy().astype(np.complex128)
        errs[nm] = float(np.linalg.norm((g - w).ravel()) / np.linalg.norm(w.ravel()))
        if nm in ("y_ws", "dx_ws", "xMh_ws"):   # no batch row may be wrong as a whole either
            rel = np.linalg.norm(g - w, axis=1) / np.linalg.norm(w, axis=1)
            assert float(rel.max()) <= 4 * TOL["f32"], (nm, int(rel.argmax()), float(rel.max()))
        if nm in ("dR_ws", "dL_ws"):             # ... and no block of a weight gradient
            rel = np.linalg.norm((g - w).reshape(k, -1), axis=1) / np.linalg.norm(w.reshape(k, -1), axis=1)
            assert float(rel.max()) <= 4 * TOL["f32"], (nm, int(rel.argmax()), float(rel.max()))
    print("  %s %s" % (name, " ".join("%s=%.2e" % kv for kv in errs.items())), flush=True)
    assert max(errs.values()) <= TOL["f32"], errs
    if on_matrix_cores:   # fixed summation order: the same bits on a second call
        again = B.monarch_bwd_c64_ws(dyd, xd, Rd, Ld, flags=flags)
        assert all(torch.equal(u, v) for u, v in zip(again, outs_ws[1:4]))
    # empty batch: no-op forward, zero gradients
    e = B.monarch_bwd_c64(dyd[:0], xd[:0], Rd, Ld, flags=flags)
    assert e[0].shape == (0, k * p) and not bool(e[1].any()) and not bool(e[2].any())
    e = B.monarch_bwd_c64_ws(dyd[:0], xd[:0], Rd, Ld, flags=flags)
    assert e[0].shape == (0, k * p) and not bool(e[1].any()) and not bool(e[2].any())
    assert B.monarch_fwd_h_c64(dyd[:0], Rd, Ld, flags=flags).shape == (0, k * p)
    assert B.monarch_fwd_c64_ws(xd[:0], Rd, Ld, flags=flags).shape == (0, k * s)
    assert B.monarch_fwd_h_c64_ws(dyd[:0], Rd, Ld, flags=flags).shape == (0, k * p)


def test_stage_kernels_on_random_block_counts(B):
    """Seeded random block counts (multiples of 8 and not), batches and readings through the matrix-core stage kernels:
    the complex calls with a workspace for blocks of 16 / 32 / 64 and the fp32 layer calls for blocks of 32 / 64."""
    from oracle import complex_ref
    rng = np.random.default_rng(2204005950)
    for it in range(10):
        m = int(rng.choice([16, 32, 64]))
        k = int(rng.integers(1, 41))
        rows = int(rng.integers(1, 1200))
        reading = int(rng.integers(0, 2))
        flags = B.MONARCH_FLAG_PERM_B if reading else 0
        x, R, L, dy = (cnormal(8600 + 10 * it + 2 * i, shp, std) for i, (shp, std) in enumerate(
            (((rows, k * m), 1.0), ((k, m, m), m ** -0.5), ((k, m, m), m ** -0.5), ((rows, k * m), 1.0))))
        xd, Rd, Ld, dyd = cdev(x), cdev(R), cdev(L), cdev(dy)
        got = [B.monarch_fwd_c64_ws(xd, Rd, Ld, flags=flags), B.monarch_fwd_h_c64_ws(dyd, Rd, Ld, flags=flags)]
        got += list(B.monarch_bwd_c64_ws(dyd, xd, Rd, Ld, flags=flags))
        want = [complex_ref.fwd(x, R, L, reading), complex_ref.fwd_h(dy, R, L, reading)] + list(complex_ref.bwd(dy, x, R, L, reading))
        errs = [float(np.linalg.norm(g.cpu().numpy().astype(np.complex128) - w) / np.linalg.norm(w)) for g, w in zip(got, want)]
        print("\n  c64 m=%d k=%d rows=%d reading=%d: %s" % (m, k, rows, reading, " ".join("%.1e" % e for e in errs)), flush=True)
        assert max(errs) <= TOL["f32"], (m, k, rows, reading, errs)
        if m == 16:
            continue
        sh = synth.Shape("stage_rand%d_k%d_m%d_B%d_r%d" % (it, k, m, rows, reading), "f32", rows, k, m, m, m, config=400 + it)
        rd = oracle.READING_B if reading else oracle.READING_A
        xr, Rr, Lr, dyr = synth.make_inputs(sh)
        compare(sh, [run_fwd(B, sh, xr, Rr, Lr, flags, ws=True)], [oracle.fwd(xr, Rr, Lr, rd)], ["y_ws"])
        compare(sh, run_bwd(B, sh, dyr, xr, Rr, Lr, flags), oracle.bwd(dyr, xr, Rr, Lr, rd), ["dx", "dR", "dL"])
        compare(sh, [run_fwd_t(B, sh, dyr, Rr, Lr, flags)], [oracle.fwd_t(dyr, Rr, Lr, rd)], ["xM"])


@pytest.mark.parametrize("m", [4, 16, 64])
def test_dft_monarch_times_its_conjugate_transpose_is_n(B, m):
    """F F* = n I on the GPU: monarch_fwd_c64 with the DFT factors, then monarch_fwd_h_c64 with the same factors,
    returns n x (the product M M* of Section 3.1 with M1 = M2 = the DFT Monarch matrix, applied right to left)."""
    n = m * m
    x = cnormal(8200 + m, (13, n))
    R, L = B.monarch_dft_factors(m, False)
    back = B.monarch_fwd_h_c64(B.monarch_fwd_c64(cdev(x), R, L), R, L).cpu().numpy().astype(np.complex128)
    err = float(np.linalg.norm(back - n * x) / np.linalg.norm(n * x))
    print("\n  m=%d: %.2e" % (m, err), flush=True)
    assert err <= TOL["f32"]


@pytest.mark.parametrize("m", [2, 3, 8, 16, 64])
def test_dft_factors_make_the_monarch_matrix_a_fourier_transform(B, m):
    """monarch_dft_factors + monarch_fwd_c64 against the library FFT of the grid-transposed input (the
    4-step splitting), forward and inverse; the inverse factors undo the forward ones."""
    from oracle import complex_ref
    n = m * m
    x = cnormal(8100 + m, (11, n))
    xt = x.astype(np.complex128).reshape(11, m, m).transpose(0, 2, 1).reshape(11, n)
    for inverse in (False, True):
        R, L = B.monarch_dft_factors(m, inverse)
        Ro, Lo = complex_ref.dft_factors(m, inverse)
        assert np.abs(R.cpu().numpy() - Ro).max() <= 2e-7 and np.abs(L.cpu().numpy() - Lo).max() <= 2e-7 / (n if inverse else 1) + 1e-12
        y = B.monarch_fwd_c64(cdev(x), R, L).cpu().numpy().astype(np.complex128)
        want = np.fft.ifft(xt, axis=1) if inverse else np.fft.fft(xt, axis=1)
        err = float(np.linalg.norm(y - want) / np.linalg.norm(want))
        print("\n  m=%d inverse=%s: %.2e" % (m, inverse, err), flush=True)
        assert err <= TOL["f32"]
    # F^-1 P applied to (F P x) un-transposed: P (F P)^-1 ... simply: ifft-Monarch of the transposed fft-Monarch output returns x
    R, L = B.monarch_dft_factors(m, False)
    Ri, Li = B.monarch_dft_factors(m, True)
    y = B.monarch_fwd_c64(cdev(x), R, L)                                   # F P x
    yt = y.reshape(11, m, m).transpose(1, 2).contiguous().reshape(11, n)   # P (F P x)
    back = B.monarch_fwd_c64(yt, Ri, Li).cpu().numpy()                     # F^-1 P P F P x = P x
    assert np.linalg.norm(back - xt) / np.linalg.norm(xt) <= TOL["f32"]


# ------------------------------------------------------ projection (Algorithm 1) ----
# Only the products L[j][l][k] * R[k][j][i] are determined (sign and scaling of a singular pair are
# free), so the Monarch matrix is compared, not the factors.  fp32 Jacobi against the fp64 SVD: the
# leading singular pair of a slice is conditioned by its relative gap (about 1e-2 for 64 x 64 Gaussian
# slices), hence 1e-4; the objective itself is insensitive to that and is held to 1e-5.
PROJ_TOL = {"f32": 1e-4, "bf16": 2e-2}


def run_project(B, A, dtype):
    from oracle import project
    n = A.shape[0]
    m = int(round(n ** 0.5))
    bR, R = guarded((m, m, m), tdtype(dtype))
    bL, L = guarded((m, m, m), tdtype(dtype))
    B.monarch_project(dev(A, dtype), R, L)
    torch.cuda.synchronize()
    check_guard(bR, "R")
    check_guard(bL, "L")
    Lh, Rh = host(L), host(R)
    assert np.isfinite(Lh).all() and np.isfinite(Rh).all()
    return Lh, Rh, project.monarch_square(Lh, Rh)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m", [1, 2, 3, 5, 8, 16, 33, 64])
def test_projection_of_dense_matrices(B, m, dtype):
    from oracle import project
    n = m * m
    A = synth.quantize(synth.normal(7100 + m, (n, n)), dtype)
    _, _, M = run_project(B, A, dtype)
    Lo, Ro = project.project_square(A)
    Mo = project.monarch_square(Lo, Ro)
    err = oracle.rel_fro(M, Mo)
    obj, obj_o = float(np.sum((A - M) ** 2)), float(np.sum((A - Mo) ** 2))
    print("\n  m=%d %s: M err %.2e, objective %.8e (optimal %.8e)" % (m, dtype, err, obj, obj_o), flush=True)
    assert err <= PROJ_TOL[dtype]
    # distance to A: optimal up to 1e-5 relative, plus the rounding of the factors themselves
    slack = (1e-6 if dtype == "f32" else 2.0 ** -7) * float(np.linalg.norm(Mo))
    assert np.sqrt(obj) <= np.sqrt(obj_o) * (1 + 1e-5) + slack


@pytest.mark.parametrize("m", [4, 16, 64])
def test_projection_recovers_monarch_matrices_and_handles_zero_slices(B, m):
    """A in M is a fixed point (remark after Theorem 1), through monarch_to_dense as well; slices that
    are entirely zero give zero factors, not NaN."""
    from oracle import project
    sh = synth.Shape("proj%d" % m, "f32", 1, m, m, m, m, config=60)
    _, R0, L0, _ = synth.make_inputs(sh)
    L0[1, :, 2] = 0.0  # slice (j = 1, k = 2) of the Monarch matrix becomes zero
    A = project.monarch_square(L0, R0)
    L, R, M = run_project(B, A, "f32")
    assert oracle.rel_fro(M, A) <= 1e-5
    assert not L[1, :, 2].any() or not R[2, 1, :].any()
    Md = run_dense(B, sh, R.astype(np.float32), L.astype(np.float32))
    assert oracle.rel_fro(Md, A) <= 1e-5
    Lz, Rz, Mz = run_project(B, np.zeros((m * m, m * m), dtype=np.float32), "f32")
    assert not Lz.any() and not Rz.any()


@pytest.mark.parametrize("case", [("k4_192", "bf16", 1000, 4, 192, 192, 192), ("sq_m64", "bf16", 300, 64, 64, 64, 64),
                                  ("sq_m16", "f32", 64, 16, 16, 16, 16), ("rect_generic", "f32", 50, 3, 4, 5, 7),
                                  ("f32_stage_k8_m32", "f32", 300, 8, 32, 32, 32)],
                         ids=lambda c: c[0])
def test_calls_can_be_captured_in_a_graph(B, case):
    """The library allocates nothing, clears memory with kernels only and enqueues everything on the
    caller's stream, so a forward + backward (with bias gradient) can be captured in a HIP graph.
    Four replays, with eager work and synchronisations between them, each against the eager result:
    bit for bit on the matrix-core kernels, to fp32 summation order on the shape-generic backward
    (its weight gradients are fp32 atomics)."""
    sh = small_shape(case)
    x, R, L, dy = synth.make_inputs(sh)
    xd, Rd, Ld, dyd, bd = (dev(a, sh.dtype) for a in (x, R, L, dy, make_bias(sh)))
    code = 0 if sh.dtype == "f32" else 1
    outs = [torch.empty((sh.B, sh.n_out), dtype=xd.dtype, device="cuda"), torch.empty_like(xd), torch.empty_like(Rd),
            torch.empty_like(Ld), torch.empty((sh.n_out,), dtype=xd.dtype, device="cuda")]
    fneed = B.monarch_fwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code)
    fws = torch.empty(max(fneed, 256), dtype=torch.uint8, device="cuda")
    ws = torch.empty(B.monarch_bwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, code), dtype=torch.uint8, device="cuda")

    def step():
        B.monarch_fwd_bias(xd, Rd, Ld, bd, outs[0], workspace=fws if fneed else None)
        B.monarch_bwd_bias(dyd, xd, Rd, Ld, outs[1], outs[2], outs[3], outs[4], workspace=ws)

    step()  # eager: reference values, and every kernel is loaded before the capture
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    generic = B.monarch_kernel_name(1, sh.n_in, sh.k, sh.q, sh.s, code) == "generic_bwd"
    for rep in range(4):
        for t in outs:
            t.fill_(float("nan"))  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, want) in enumerate(zip(outs, ref)):
            if generic and i in (2, 3):
                assert oracle.rel_fro(host(got), host(want)) <= 1e-6, (rep, i)
            else:
                assert torch.equal(got, want), (rep, i)
    compare(sh, [host(outs[0]), host(outs[4])], [oracle.fwd_bias(x, R, L, host(bd)), oracle.bwd_bias(dy, x, R, L)[3]], ["y", "dbias"])


def test_complex_calls_with_workspace_can_be_captured_in_a_graph(B):
    """The complex calls with a workspace only enqueue kernels (no clearing by memset, no allocation): forward,
    conjugate-transpose forward and backward captured in one HIP graph, four replays bit for bit against eager."""
    rows, k, m = 200, 16, 32
    x, R, L, dy = (cdev(cnormal(8800 + 2 * i, shp, std)) for i, (shp, std) in enumerate(
        (((rows, k * m), 1.0), ((k, m, m), m ** -0.5), ((k, m, m), m ** -0.5), ((rows, k * m), 1.0))))
    ws = torch.empty(B.monarch_c64_workspace_bytes(B.C64_BWD, rows, k * m, k, m, m), dtype=torch.uint8, device="cuda")
    outs = [torch.empty_like(x), torch.empty_like(x), torch.empty_like(x), torch.empty_like(R), torch.empty_like(L)]

    def step():
        B.monarch_fwd_c64_ws(x, R, L, outs[0], workspace=ws)
        B.monarch_fwd_h_c64_ws(dy, R, L, outs[1], workspace=ws)
        B.monarch_bwd_c64_ws(dy, x, R, L, outs[2], outs[3], outs[4], workspace=ws)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, want) in enumerate(zip(outs, ref)):
            assert torch.equal(got, want), (rep, i)


@pytest.mark.parametrize("bias", [False, True], ids=["no_bias", "bias"])
@pytest.mark.parametrize("case", [("k4_192", "bf16", 3 * 50, 4, 192, 192, 192), ("sq_m16", "f32", 3 * 7, 16, 16, 16, 16),
                                  ("rect", "f32", 3 * 5, 3, 4, 5, 2)], ids=lambda c: c[0])
def test_autograd_glue_matches_the_oracle(B, case, bias):
    """torch.autograd through the library (no arithmetic in Python): a 3-D input, loss = <dy, y>, the
    gradients torch hands back against the oracle's."""
    from paper_2204_00595_amd import autograd as mag
    sh = small_shape(case)
    x, R, L, dy = synth.make_inputs(sh)
    b = make_bias(sh) if bias else None
    xd = dev(x, sh.dtype).reshape(3, sh.B // 3, sh.n_in).requires_grad_(True)
    Rd, Ld = dev(R, sh.dtype).requires_grad_(True), dev(L, sh.dtype).requires_grad_(True)
    bd = dev(b, sh.dtype).requires_grad_(True) if bias else None
    y = mag.monarch_linear(xd, Rd, Ld, bd)
    assert y.shape == (3, sh.B // 3, sh.n_out)
    y.backward(dev(dy, sh.dtype).reshape(3, sh.B // 3, sh.n_out))
    torch.cuda.synchronize()
    want_y = oracle.fwd_bias(x, R, L, b) if bias else oracle.fwd(x, R, L)
    want = oracle.bwd_bias(dy, x, R, L)
    got = [host(y.detach().reshape(sh.B, -1)), host(xd.grad.reshape(sh.B, -1)), host(Rd.grad), host(Ld.grad)]
    names = ["y", "dx", "dR", "dL"]
    if bias:
        got.append(host(bd.grad))
        names.append("dbias")
    compare(sh, got, [want_y] + list(want[:len(got) - 1]), names)
    layer = mag.MonarchLinear(sh.n_in, sh.n_out, nblocks=sh.k, bias=bias, q=sh.q, device="cuda", dtype=tdtype(sh.dtype))
    with torch.no_grad():
        out = layer(xd.detach())
        M = layer.to_dense()
        ref = xd.detach().reshape(sh.B, -1).double() @ M.double().T + (layer.bias.double() if bias else 0.0)
        assert float((out.reshape(sh.B, -1).double() - ref).norm() / ref.norm()) <= TOL[sh.dtype]


def test_calls_run_on_the_stream_they_are_given(B):
    """Everything is enqueued on the caller's stream: on a side stream, behind a long-running copy on that
    same stream, the results are those of the default stream; operands at 16-byte (not 256-byte) offsets."""
    sh = small_shape(("k4_192", "bf16", 200, 4, 192, 192, 192))
    x, R, L, dy = synth.make_inputs(sh)

    def offset(a):  # a tensor that starts 16 bytes into its allocation
        t = dev(a, sh.dtype)
        buf = torch.empty(t.numel() + 8, dtype=t.dtype, device="cuda")
        v = buf[8:8 + t.numel()].view(t.shape)
        v.copy_(t)
        assert v.data_ptr() % 256 == 16
        return v

    xd, Rd, Ld, dyd = offset(x), offset(R), offset(L), offset(dy)
    y0 = B.monarch_fwd(xd, Rd, Ld)
    g0 = B.monarch_bwd_bias(dyd, xd, Rd, Ld)
    t0 = B.monarch_fwd_t(dyd, Rd, Ld)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    big = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    with torch.cuda.stream(side):
        big2 = big.clone()  # keeps the side stream busy while the calls are enqueued behind it
        y1 = B.monarch_fwd(xd, Rd, Ld, stream=side)
        g1 = B.monarch_bwd_bias(dyd, xd, Rd, Ld, stream=side)
        t1 = B.monarch_fwd_t(dyd, Rd, Ld, stream=side)
    side.synchronize()
    assert torch.equal(y0, y1) and torch.equal(t0, t1) and all(torch.equal(a, b) for a, b in zip(g0, g1))
    compare(sh, [host(y1), host(t1)] + [host(t) for t in g1], [oracle.fwd(x, R, L), oracle.fwd_t(dy, R, L)] + list(oracle.bwd_bias(dy, x, R, L)),
            ["y", "xM", "dx", "dR", "dL", "dbias"])
    del big2
    # the same with `stream=side` only (the side stream is NOT torch's current stream): the binding's own
    # temporary workspaces must belong to the side stream, or the default stream's next allocations --
    # made and overwritten here while the side stream is still busy -- would land in them
    ev = torch.cuda.Event()
    ev.record()
    side.wait_event(ev)
    with torch.cuda.stream(side):
        big3 = big.clone()
    outs = [torch.empty_like(y0), torch.empty_like(t0)] + [torch.empty_like(t) for t in g0]
    B.monarch_fwd(xd, Rd, Ld, outs[0], stream=side)
    B.monarch_bwd_bias(dyd, xd, Rd, Ld, outs[2], outs[3], outs[4], outs[5], stream=side)
    B.monarch_fwd_t(dyd, Rd, Ld, outs[1], stream=side)
    need = B.monarch_bwd_workspace_bytes(sh.B, sh.n_in, sh.k, sh.q, sh.s, 1, 0)
    junk = [torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda") for _ in range(3)]  # default stream, runs at once
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(y0, outs[0]) and torch.equal(t0, outs[1]) and all(torch.equal(a, b) for a, b in zip(g0, outs[2:]))
    del big3, junk


def test_stream_copy_is_bit_exact(B):
    n = (1 << 20) + 48  # bytes: several grid strides plus a ragged tail of three 16-byte pieces
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    buf = torch.full((n + 2 * GUARD,), 7, dtype=torch.uint8, device="cuda")
    B.monarch_stream_copy(buf[GUARD:GUARD + n], src)
    torch.cuda.synchronize()
    assert bool((buf[GUARD:GUARD + n] == src).all())
    assert bool((buf[:GUARD] == 7).all()) and bool((buf[-GUARD:] == 7).all())
