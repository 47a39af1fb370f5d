"""Per-operator parity on the GPU, through the C ABI: each kernel family against the matching step
of the oracle on the same seeded inputs."""
import numpy as np
import pytest

from oracle import encoder_oracle as O
from paper_2412_11272_amd import binding as wf

pytestmark = pytest.mark.gpu


def _bf16_round(a: np.ndarray):
    import torch
    return torch.from_numpy(a.astype(np.float32)).bfloat16()


def _rel(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())


# M spans: one partial small tile, several small tiles + ragged tail, enough rows for the large tile, and
# (the last two) the row count of a 64-stream prompt prefill, where the small tile has to fill the chip
LINEAR_SHAPES = [(75, 384, 384), (300, 1152, 384), (1000, 128, 1536), (257, 256, 64),
                 (12500, 3840, 1280), (12345, 1280, 5120), (12301, 5120, 1280),
                 (6401, 1280, 1280), (6400, 1280, 5120), (10001, 2560, 640),
                 # at most one 128 x 128 tile per CU: the four-stage operand ring, incl. its shortest K (4 and 5 steps)
                 (2600, 1024, 4096), (4951, 768, 256), (1500, 2048, 320)]


def test_linear_shapes_reach_every_tile_family():
    """Small-batch kernel, 128 x 128, 256 x 256 and 320 x 256 tiles (the last both with streaming stores, result
    >= 64 MB, and with plain ones) all occur among the shapes of test_linear_bf16."""
    picks = {(M, N): wf.gemm_tile_choice(M, N) for M, N, _ in LINEAR_SHAPES}
    assert set(picks.values()) == {(0, 0), (128, 128), (256, 256), (320, 256)}
    assert picks[(12500, 3840)] == (320, 256) and picks[(10001, 2560)] == (320, 256) and picks[(12301, 5120)] == (256, 256)


@pytest.mark.parametrize("M,N,K", LINEAR_SHAPES)
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_linear_bf16(M, N, K, epi):
    import torch
    rng = np.random.default_rng(M + N + K + epi)
    a = _bf16_round(rng.standard_normal((M, K)))
    w = _bf16_round(rng.standard_normal((N, K)) * 0.05)
    bias = rng.standard_normal(N).astype(np.float32)
    a64, w64 = a.float().numpy().astype(np.float64), w.float().numpy().astype(np.float64)
    ref = O.linear(a64, w64, bias.astype(np.float64))
    ad, wd, bd = a.cuda(), w.cuda(), torch.from_numpy(bias).cuda()
    if epi == 2:
        x0 = rng.standard_normal((M, N)).astype(np.float32)
        out = torch.from_numpy(x0).cuda()
        ref = x0.astype(np.float64) + ref
    else:
        out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        if epi == 1:
            ref = O.gelu(ref)
    wf.op_linear(wf.WF_PRECISION_BF16, ad, wd, bd, out, epi)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.all(np.isfinite(got))
    # inputs are exactly representable, accumulation is fp32: only the output rounding (2^-9) remains
    tol = 5e-3 if epi != 2 else 2e-5
    assert _rel(got, ref) < tol


def _linear_case(M, N, K, epi, seed):
    import torch
    rng = np.random.default_rng(seed)
    a = _bf16_round(rng.standard_normal((M, K)))
    w = _bf16_round(rng.standard_normal((N, K)) * 0.05)
    bias = rng.standard_normal(N).astype(np.float32)
    ref = O.linear(a.float().numpy().astype(np.float64), w.float().numpy().astype(np.float64), bias.astype(np.float64))
    if epi == 2:
        x0 = rng.standard_normal((M, N)).astype(np.float32)
        out = torch.from_numpy(x0).cuda()
        ref = x0.astype(np.float64) + ref
    else:
        out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        if epi == 1:
            ref = O.gelu(ref)
    wf.op_linear(wf.WF_PRECISION_BF16, a.cuda(), w.cuda(), torch.from_numpy(bias).cuda(), out, epi)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.all(np.isfinite(got)), (M, N, K, epi)
    assert _rel(got, ref) < (5e-3 if epi != 2 else 2e-5), (M, N, K, epi, wf.gemm_tile_choice(M, N))


def test_linear_bf16_at_the_edges_of_every_kernel_choice():
    """Row counts on both sides of each switch of the launcher: small-batch kernel / 128 x 128 tile (1024 rows), one
    tile per CU with four operand stages / two per CU (256 tiles of 128 x 128), 128 x 128 / large tile (160 tiles of
    256 x 256), 256 / 320 rows; K loops of 1 to 5 steps; every epilogue."""
    cases = [(1024, 256, 192), (1025, 256, 192), (1025, 128, 64), (4096, 1024, 256), (4097, 1024, 320),
             (3840, 2560, 128), (4096, 2560, 128), (4097, 2560, 64), (5100, 2560, 256), (5121, 2560, 192),
             (8191, 1280, 320), (8193, 1280, 64), (6400, 2560, 128), (6657, 2560, 192)]
    picks = set()
    for i, (M, N, K) in enumerate(cases):
        picks.add(wf.gemm_tile_choice(M, N))
        for epi in (0, 1, 2):
            _linear_case(M, N, K, epi, 1000 + 3 * i + epi)
    assert picks == {(0, 0), (128, 128), (256, 256), (320, 256)}


def test_linear_bf16_random_shapes():
    """Seeded random shapes across all kernel choices (row counts 1 .. 9000, widths and depths in the kernels' units)."""
    rng = np.random.default_rng(77)
    for i in range(24):
        M = int(rng.integers(1, 9001))
        N = 128 * int(rng.integers(1, 21))
        K = 64 * int(rng.integers(1, 17))
        _linear_case(M, N, K, int(rng.integers(0, 3)), 2000 + i)


@pytest.mark.parametrize("M,N,K", [(75, 384, 384), (300, 1152, 240), (1000, 128, 1536)])
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_linear_f32(M, N, K, epi):
    import torch
    if K % 64:
        K = 256
    rng = np.random.default_rng(M + N + K + epi)
    a = rng.standard_normal((M, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    ref = O.linear(a.astype(np.float64), w.astype(np.float64), bias.astype(np.float64))
    x0 = rng.standard_normal((M, N)).astype(np.float32)
    out = torch.from_numpy(x0.copy()).cuda()
    if epi == 1:
        ref = O.gelu(ref)
    if epi == 2:
        ref = x0 + ref
    wf.op_linear(wf.WF_PRECISION_F32, torch.from_numpy(a).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(bias).cuda(),
                 out, epi)
    torch.cuda.synchronize()
    assert _rel(out.cpu().numpy(), ref) < 2e-6


@pytest.mark.parametrize("M,d", [(1, 128), (75, 384), (333, 512), (1001, 768), (50, 1024), (4097, 1280), (3, 2048)])
def test_layernorm(M, d):
    import torch
    rng = np.random.default_rng(M * d)
    x = (rng.standard_normal((M, d)) * 3 + 0.7).astype(np.float32)
    x[0] = 2.5                                               # constant row -> exactly the shift
    g = rng.standard_normal(d).astype(np.float32)
    b = rng.standard_normal(d).astype(np.float32)
    ref = O.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    xd, gd, bd = (torch.from_numpy(t).cuda() for t in (x, g, b))
    out = torch.empty((M, d), dtype=torch.float32, device="cuda")
    wf.op_layernorm(xd, gd, bd, out)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), ref, atol=2e-5)
    outb = torch.empty((M, d), dtype=torch.bfloat16, device="cuda")
    wf.op_layernorm(xd, gd, bd, outb)
    torch.cuda.synchronize()
    assert _rel(outb.float().cpu().numpy(), ref) < 5e-3


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (75, 1152, 384), (425, 2048, 512), (33, 256, 2048), (1024, 384, 1280)])
@pytest.mark.parametrize("epi", [0, 1])
def test_layernorm_fused_into_the_small_batch_product(M, N, K, epi):
    """QKV / fc1 of a single stream's buffer: the product normalises its fp32 operand itself.  Against LayerNorm
    followed by the product in the oracle, with the normalised rows rounded to bf16 as the kernel stores them; rows
    with a mean far from zero, an outlier in first place (the kernel shifts its sums by that element) and a
    constant row are in the batch."""
    import torch
    rng = np.random.default_rng(M + N + K + epi)
    x = (rng.standard_normal((M, K)) * 1.5 + 0.3).astype(np.float32)
    x[0] = 7.25                                              # constant row -> exactly the shift
    if M > 4:
        x[1] += 300.0                                        # mean 200 standard deviations away from zero
        x[2, 0] = 500.0                                      # the pivot of the shifted sums is an outlier
        x[3] *= 1e-3
    g = (1.0 + 0.2 * rng.standard_normal(K)).astype(np.float32)
    b = (0.1 * rng.standard_normal(K)).astype(np.float32)
    w = _bf16_round(rng.standard_normal((N, K)) * 0.05)
    bias = rng.standard_normal(N).astype(np.float32)
    u = O.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    u16 = _bf16_round(u).float().numpy().astype(np.float64)                  # what reaches the matrix pipe
    ref = O.linear(u16, w.float().numpy().astype(np.float64), bias.astype(np.float64))
    if epi == 1:
        ref = O.gelu(ref)
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    wf.op_ln_linear(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), w.cuda(),
                    torch.from_numpy(bias).cuda(), out, epi)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.all(np.isfinite(got))
    # bf16 rounding of u flips where the kernel's fp32 statistics differ from the oracle's in the last bit: a few
    # elements of u move by one bf16 step (2^-8 relative), which the 5e-3 on the result covers
    assert _rel(got, ref) < 6e-3


LENS = [[1], [75], [64, 65, 63], [128, 129, 1, 2, 300], [1525, 75, 700]]
# (lens, heads): few queries -> the kernel that splits the key loop over the waves (one stream's buffer: at most 256
# workgroups of 32 queries); [1525, 75, 700] x 3 heads and the last case are beyond that and run with 128-query work items
CASES = [(l, 3) for l in LENS] + [([1525, 700, 300, 129, 128, 75, 64, 1], 20)]


@pytest.mark.parametrize("lens,n_heads", CASES)
@pytest.mark.parametrize("sharp", [1.0, 6.0])
@pytest.mark.parametrize("precision", [wf.WF_PRECISION_BF16, wf.WF_PRECISION_F32])
def test_attention(lens, n_heads, sharp, precision):
    import torch
    d = 64 * n_heads
    M = sum(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rng = np.random.default_rng(M + int(sharp))
    qkv = rng.standard_normal((M, 3 * d)).astype(np.float32)
    qkv[:, :2 * d] *= np.sqrt(sharp)                         # logits std ~ sharp
    if precision == wf.WF_PRECISION_BF16:
        t = torch.from_numpy(qkv).bfloat16()
        qkv64 = t.float().numpy().astype(np.float64)
        out = torch.full((M, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    else:
        t = torch.from_numpy(qkv)
        qkv64 = qkv.astype(np.float64)
        out = torch.full((M, d), float("nan"), dtype=torch.float32, device="cuda")
    ref = np.concatenate([O.multi_head_attention(qkv64[a:b, :d], qkv64[a:b, d:2 * d], qkv64[a:b, 2 * d:], n_heads)
                          for a, b in zip(cu[:-1], cu[1:])])
    wf.op_attention(precision, t.cuda(), out, cu, n_heads)
    got = out.float().cpu().numpy()
    assert np.all(np.isfinite(got))
    # bf16: P is rounded to bf16 before the P.V product and the output is bf16
    assert _rel(got, ref) < (1e-2 if precision == wf.WF_PRECISION_BF16 else 1e-5)
