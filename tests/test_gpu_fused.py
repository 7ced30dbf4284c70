"""GPU parity of iflow_qgemv_fused: rms normalization or the silu-gated input in front of the product and a residual
behind it, in one launch, against the plain definitions in oracle/decode_ops.py (the 3.5-bit format at many shapes,
every other format at ragged ones)."""
import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_parity import NAMES, TOL, gpu, gpu_quantize, say  # noqa: F401

pytestmark = pytest.mark.gpu


def dev16(torch, bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.float16)


def bits_of(t):
    return t.cpu().numpy().view(np.uint16)


def err(y_bits, yref):
    y = y_bits.view(np.float16).astype(np.float64)
    rms = np.sqrt(np.mean(yref ** 2))
    return float(np.max(np.abs(y - yref) / np.maximum(np.abs(yref), max(rms, 1e-30))))


def make(torch, iflow, orc, rows, cols, seed, sigma=0.02, name="Q3H_B64"):
    w = synth.weights(rows, cols, sigma, seed)
    packed, _ = gpu_quantize(torch, iflow, iflow.FORMATS[name], w)
    q, s, o = orc.quantize(orc.FORMATS[name], w)
    return packed, orc.dequant(orc.FORMATS[name], q, s, o)


@pytest.mark.parametrize("rows,cols", [(300, 1024), (1000, 4096 + 64), (37, 64), (40, 18 * 4096 + 64)])
@pytest.mark.parametrize("with_residual", [False, True])
def test_rms_gain_in_front_of_the_product(gpu, orc, rows, cols, with_residual):
    torch, iflow = gpu
    from oracle import decode_ops as ops
    say(f"[case] fused rms gain rows={rows} cols={cols} residual={with_residual}")
    packed, wdeq = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 1100 + rows)
    x = synth.activations(1, cols, synth.BASE_SEED + 1101)[0].view(np.uint16)
    g = (1.0 + 0.2 * np.random.default_rng(synth.BASE_SEED + 1102).standard_normal(cols)).astype(np.float16).view(np.uint16)
    r = synth.activations(1, rows, synth.BASE_SEED + 1103)[0].view(np.uint16) if with_residual else None
    eps = 1e-5
    y = torch.full((rows,), float("nan"), dtype=torch.float16, device="cuda")
    iflow.qgemv_fused(iflow.Q3H_B64, [packed], [rows], cols, dev16(torch, x), [y], iflow.X_RMS_GAIN, dev16(torch, g), eps,
                      [dev16(torch, r)] if with_residual else None)
    torch.cuda.synchronize()
    e = err(bits_of(y), ops.rms_linear(wdeq, x, g, eps, r))                  # the definition: no rounding between norm and product
    e_split = err(bits_of(y), ops.fused_gemv(wdeq, ops.gain(x, g), ops.rms_scale(x, eps), r))
    say(f"        max rel err {e:.3e} against the definition, {e_split:.3e} against the evaluation order with fp16(x g)")
    assert np.isfinite(y.cpu().numpy().astype(np.float32)).all() and e <= TOL and e_split <= TOL


@pytest.mark.parametrize("rows,cols", [(300, 1024), (520, 11008)])
def test_silu_gated_input_and_in_place_residual(gpu, orc, rows, cols):
    torch, iflow = gpu
    from oracle import decode_ops as ops
    say(f"[case] fused silu*mul rows={rows} cols={cols}, residual in place")
    packed, wdeq = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 1200 + rows)
    a = (synth.activations(1, cols, synth.BASE_SEED + 1201)[0].astype(np.float32) * 2.5).astype(np.float16).view(np.uint16)
    b = synth.activations(1, cols, synth.BASE_SEED + 1202)[0].view(np.uint16)
    h = synth.activations(1, rows, synth.BASE_SEED + 1203)[0].view(np.uint16)
    hidden = dev16(torch, h).clone()                           # updated in place: residual and output are the same buffer
    iflow.qgemv_fused(iflow.Q3H_B64, [packed], [rows], cols, dev16(torch, a), [hidden], iflow.X_SILU_MUL, dev16(torch, b), 0.0, [hidden])
    torch.cuda.synchronize()
    e = err(bits_of(hidden), ops.silu_linear(wdeq, a, b, h))
    e_split = err(bits_of(hidden), ops.fused_gemv(wdeq, ops.silu_mul(a, b), 1.0, h))
    say(f"        max rel err {e:.3e} against the definition, {e_split:.3e} against the evaluation order with fp16(silu(a) b)")
    assert e <= TOL and e_split <= TOL


def test_two_matrices_share_the_normalized_input_and_plain_with_residual(gpu, orc):
    torch, iflow = gpu
    from oracle import decode_ops as ops
    rows = [700, 333]
    cols = 2048
    say("[case] fused: two matrices behind one rms gain; plain product with residual")
    mats = [make(torch, iflow, orc, r, cols, synth.BASE_SEED + 1300 + r) for r in rows]
    x = synth.activations(1, cols, synth.BASE_SEED + 1301)[0].view(np.uint16)
    g = (0.5 + np.random.default_rng(synth.BASE_SEED + 1302).random(cols)).astype(np.float16).view(np.uint16)
    res1 = synth.activations(1, rows[1], synth.BASE_SEED + 1303)[0].view(np.uint16)
    ys = [torch.full((r,), float("nan"), dtype=torch.float16, device="cuda") for r in rows]
    iflow.qgemv_fused(iflow.Q3H_B64, [m[0] for m in mats], rows, cols, dev16(torch, x), ys, iflow.X_RMS_GAIN, dev16(torch, g), 1e-6,
                      [None, dev16(torch, res1)])
    torch.cuda.synchronize()
    assert err(bits_of(ys[0]), ops.rms_linear(mats[0][1], x, g, 1e-6)) <= TOL
    assert err(bits_of(ys[1]), ops.rms_linear(mats[1][1], x, g, 1e-6, res1)) <= TOL
    # no operation on x: equals iflow_qgemv when there is no residual, bit for bit
    y0 = torch.empty((rows[0],), dtype=torch.float16, device="cuda")
    y1 = torch.empty((rows[0],), dtype=torch.float16, device="cuda")
    iflow.qgemv_fused(iflow.Q3H_B64, [mats[0][0]], [rows[0]], cols, dev16(torch, x), [y0])
    iflow.qgemv(iflow.Q3H_B64, mats[0][0], rows[0], cols, dev16(torch, x), y1)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(y0), bits_of(y1))
    res0 = synth.activations(1, rows[0], synth.BASE_SEED + 1304)[0].view(np.uint16)
    iflow.qgemv_fused(iflow.Q3H_B64, [mats[0][0]], [rows[0]], cols, dev16(torch, x), [y0], residual_list=[dev16(torch, res0)])
    torch.cuda.synchronize()
    assert err(bits_of(y0), ops.fused_gemv(mats[0][1], x, 1.0, res0)) <= TOL


def test_feed_forward_block_at_7b_size(gpu, orc):
    """h -> rms gain -> gate, up (one launch) -> silu(gate) * up -> down + h (one launch): two launches, no other kernel.
    Weights drawn on the device; sampled rows of each stage against the oracle, given the stage's actual inputs."""
    torch, iflow = gpu
    from oracle import decode_ops as ops
    fmt, ofmt = iflow.Q3H_B64, orc.Q3H_B64
    hidden, ffn = 4096, 11008
    say("[case] fused feed-forward block 4096 -> 2 x 11008 -> 4096")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 1400)
    mats = []
    for i, (rows, cols) in enumerate([(ffn, hidden), (ffn, hidden), (hidden, ffn)]):
        wd = torch.randn((rows, cols), generator=gen, device="cuda", dtype=torch.float32) * 0.02
        n = iflow.packed_bytes(fmt, rows, cols)
        packed = torch.empty(n, dtype=torch.uint8, device="cuda")
        iflow.quantize(fmt, wd, rows, cols, packed, n)
        idx = synth.sample_rows(rows, 40, synth.BASE_SEED + 1401 + i)
        q, s, o = orc.quantize(ofmt, wd[torch.from_numpy(idx).cuda()].cpu().numpy())
        mats.append((packed, rows, cols, idx, orc.dequant(ofmt, q, s, o)))
        del wd
    h = synth.activations(1, hidden, synth.BASE_SEED + 1405)[0].view(np.uint16)
    g = (1.0 + 0.1 * np.random.default_rng(synth.BASE_SEED + 1406).standard_normal(hidden)).astype(np.float16).view(np.uint16)
    hd, gd = dev16(torch, h), dev16(torch, g)
    gate = torch.empty((ffn,), dtype=torch.float16, device="cuda")
    up = torch.empty((ffn,), dtype=torch.float16, device="cuda")
    out = torch.empty((hidden,), dtype=torch.float16, device="cuda")
    iflow.qgemv_fused(fmt, [mats[0][0], mats[1][0]], [ffn, ffn], hidden, hd, [gate, up], iflow.X_RMS_GAIN, gd, 1e-5)
    iflow.qgemv_fused(fmt, [mats[2][0]], [hidden], ffn, gate, [out], iflow.X_SILU_MUL, up, 0.0, [hd])
    torch.cuda.synchronize()
    for t, m in ((gate, mats[0]), (up, mats[1])):
        full = t.cpu().numpy().astype(np.float64)
        want = ops.rms_linear(m[4], h, g, 1e-5)
        assert np.max(np.abs(full[m[3]] - want) / np.maximum(np.abs(want), np.sqrt(np.mean(full ** 2)))) <= TOL
    m = mats[2]
    full = out.cpu().numpy().astype(np.float64)
    want = ops.silu_linear(m[4], bits_of(gate), bits_of(up), h[m[3]])
    e = float(np.max(np.abs(full[m[3]] - want) / np.maximum(np.abs(want), np.sqrt(np.mean(full ** 2)))))
    say(f"        down + residual: max rel err on sampled rows {e:.3e}")
    assert np.isfinite(full).all() and e <= TOL


OTHER_FORMATS = [n for n in NAMES if n != "Q3H_B64"]


@pytest.mark.parametrize("name", OTHER_FORMATS)
def test_other_formats_rms_gain_two_matrices_and_residual(gpu, orc, name):
    """Ragged in every direction: a last strip of two blocks, row counts that fill neither a group nor a workgroup."""
    torch, iflow = gpu
    from oracle import decode_ops as ops
    fmt = iflow.FORMATS[name]
    rows, cols = [301, 77], 4096 + 128
    say(f"[case] fused rms gain {name} rows={rows} cols={cols}")
    mats = [make(torch, iflow, orc, r, cols, synth.BASE_SEED + 1500 + r, name=name) for r in rows]
    x = synth.activations(1, cols, synth.BASE_SEED + 1501)[0].view(np.uint16)
    g = (1.0 + 0.2 * np.random.default_rng(synth.BASE_SEED + 1502).standard_normal(cols)).astype(np.float16).view(np.uint16)
    res1 = synth.activations(1, rows[1], synth.BASE_SEED + 1503)[0].view(np.uint16)
    ys = [torch.full((r,), float("nan"), dtype=torch.float16, device="cuda") for r in rows]
    iflow.qgemv_fused(fmt, [m[0] for m in mats], rows, cols, dev16(torch, x), ys, iflow.X_RMS_GAIN, dev16(torch, g), 1e-5,
                      [None, dev16(torch, res1)])
    torch.cuda.synchronize()
    e0 = err(bits_of(ys[0]), ops.rms_linear(mats[0][1], x, g, 1e-5))
    e1 = err(bits_of(ys[1]), ops.rms_linear(mats[1][1], x, g, 1e-5, res1))
    say(f"        max rel err {e0:.3e} {e1:.3e}")
    assert e0 <= TOL and e1 <= TOL
    # one matrix per launch gives the same bits
    y_alone = torch.full((rows[1],), float("nan"), dtype=torch.float16, device="cuda")
    iflow.qgemv_fused(fmt, [mats[1][0]], [rows[1]], cols, dev16(torch, x), [y_alone], iflow.X_RMS_GAIN, dev16(torch, g), 1e-5,
                      [dev16(torch, res1)])
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(y_alone), bits_of(ys[1]))


@pytest.mark.parametrize("name", OTHER_FORMATS)
def test_other_formats_silu_gate_in_place_residual_and_plain(gpu, orc, name):
    torch, iflow = gpu
    from oracle import decode_ops as ops
    fmt = iflow.FORMATS[name]
    rows, cols = 520, 11008
    say(f"[case] fused silu*mul {name} rows={rows} cols={cols}, residual in place; plain")
    packed, wdeq = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 1600, name=name)
    a = (synth.activations(1, cols, synth.BASE_SEED + 1601)[0].astype(np.float32) * 2.5).astype(np.float16).view(np.uint16)
    b = synth.activations(1, cols, synth.BASE_SEED + 1602)[0].view(np.uint16)
    h = synth.activations(1, rows, synth.BASE_SEED + 1603)[0].view(np.uint16)
    hidden = dev16(torch, h).clone()
    iflow.qgemv_fused(fmt, [packed], [rows], cols, dev16(torch, a), [hidden], iflow.X_SILU_MUL, dev16(torch, b), 0.0, [hidden])
    torch.cuda.synchronize()
    e = err(bits_of(hidden), ops.silu_linear(wdeq, a, b, h))
    say(f"        max rel err {e:.3e}")
    assert e <= TOL
    # no operation and no residual: iflow_qgemv's bits; with a residual: the definition
    y0 = torch.empty((rows,), dtype=torch.float16, device="cuda")
    y1 = torch.empty((rows,), dtype=torch.float16, device="cuda")
    iflow.qgemv_fused(fmt, [packed], [rows], cols, dev16(torch, b), [y0])
    iflow.qgemv(fmt, packed, rows, cols, dev16(torch, b), y1)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(y0), bits_of(y1))
    iflow.qgemv_fused(fmt, [packed], [rows], cols, dev16(torch, b), [y0], residual_list=[dev16(torch, h)])
    torch.cuda.synchronize()
    assert err(bits_of(y0), ops.fused_gemv(wdeq, b, 1.0, h)) <= TOL


def test_other_formats_rows_too_long_for_the_staged_activations_are_refused(gpu):
    """Beyond what fits in LDS the fused call of the other formats returns a shape error before any launch."""
    torch, iflow = gpu
    fmt = iflow.FORMATS["Q4_B64"]
    rows, cols = 8, 65536
    n = iflow.packed_bytes(fmt, rows, cols)
    packed = torch.zeros(n, dtype=torch.uint8, device="cuda")
    x = torch.zeros(cols, dtype=torch.float16, device="cuda")
    y = torch.zeros(rows, dtype=torch.float16, device="cuda")
    with pytest.raises(iflow.IflowError) as info:
        iflow.qgemv_fused(fmt, [packed], [rows], cols, x, [y], residual_list=[y])
    assert info.value.status == iflow.ERR_SHAPE


def gated_excess(y_bits, w_gate, w_up, x_bits, g_bits=None, eps=0.0):
    """The reference is the definition silu(W_gate n) (W_up n) with n = rms_norm(x; g, eps) (n = x without gains), no
    rounding in between.  Largest |y - silu(g) u| as a multiple of what the product tolerance allows for a product of two row sums: each
    factor may be off by TOL relative to max(|factor|, rms of its vector) (the bar every plain product is held to), which
    first-order propagation through silu(g) u turns into TOL (|silu'(g)| max(|g|, rms g) |u| + |silu(g)| max(|u|, rms u)),
    plus half an fp16 ulp of the result for the one rounding at the store."""
    from oracle import decode_ops as ops
    if g_bits is None:
        g, u = ops.fused_gemv(w_gate, x_bits), ops.fused_gemv(w_up, x_bits)
    else:
        g, u = ops.rms_linear(w_gate, x_bits, g_bits, eps), ops.rms_linear(w_up, x_bits, g_bits, eps)
    sig = 1.0 / (1.0 + np.exp(-g))
    dsilu = sig * (1.0 + g * (1.0 - sig))
    yref = ops.gated_rms(w_gate, w_up, x_bits, g_bits, eps)
    assert np.max(np.abs(yref - ops.silu(g) * u)) <= 1e-12
    allowed = TOL * (np.abs(dsilu) * np.maximum(np.abs(g), np.sqrt(np.mean(g * g))) * np.abs(u)
                     + np.abs(ops.silu(g)) * np.maximum(np.abs(u), np.sqrt(np.mean(u * u)))) + 2.0 ** -11 * np.abs(yref) + 2.0 ** -25
    y = y_bits.view(np.float16).astype(np.float64)
    return float(np.max(np.abs(y - yref) / allowed))


@pytest.mark.parametrize("name", NAMES)
@pytest.mark.parametrize("rows,cols,normalized", [(301, 4096 + 128, True), (5200, 256, False), (77, 11008, True), (1, 64, True),
                                                  (3, 192, False)])
def test_gated_pair_of_projections(gpu, orc, name, rows, cols, normalized):
    """iflow_qgemv_gated: silu(gate) * up from the two products in one launch; ragged strips and rows, several row groups
    per wavefront (5200 rows), three strips (11008 columns)."""
    torch, iflow = gpu
    from oracle import decode_ops as ops
    fmt = iflow.FORMATS[name]
    say(f"[case] gated pair {name} rows={rows} cols={cols} rms={normalized}")
    # gate sums of a few units, so that silu is neither the identity nor zero
    gate = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 1700 + rows, sigma=2.0 / np.sqrt(cols), name=name)
    up = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 1701 + rows, name=name)
    x = synth.activations(1, cols, synth.BASE_SEED + 1702)[0].view(np.uint16)
    y = torch.full((rows,), float("nan"), dtype=torch.float16, device="cuda")
    if normalized:
        g = (1.0 + 0.2 * np.random.default_rng(synth.BASE_SEED + 1703).standard_normal(cols)).astype(np.float16).view(np.uint16)
        iflow.qgemv_gated(fmt, gate[0], up[0], rows, cols, dev16(torch, x), y, iflow.X_RMS_GAIN, dev16(torch, g), 1e-5)
    else:
        g = None
        iflow.qgemv_gated(fmt, gate[0], up[0], rows, cols, dev16(torch, x), y)
    torch.cuda.synchronize()
    e = gated_excess(bits_of(y), gate[1], up[1], x, g, 1e-5)
    say(f"        largest error / allowed error {e:.3f}")
    assert np.isfinite(y.cpu().numpy().astype(np.float32)).all() and e <= 1.0
    # swapping the two matrices is a different function (the gate acts on the first)
    if not normalized:
        y2 = torch.empty_like(y)
        iflow.qgemv_gated(fmt, up[0], gate[0], rows, cols, dev16(torch, x), y2)
        torch.cuda.synchronize()
        assert gated_excess(bits_of(y2), up[1], gate[1], x) <= 1.0
        assert not np.array_equal(bits_of(y), bits_of(y2))


@pytest.mark.parametrize("name", NAMES)
def test_fused_smallest_shapes(gpu, orc, name):
    """One row of one or two blocks: every lane but the first few is past the end of the strip."""
    torch, iflow = gpu
    from oracle import decode_ops as ops
    fmt = iflow.FORMATS[name]
    for rows, cols in ((1, 64), (2, 128)):
        say(f"[case] fused smallest {name} rows={rows} cols={cols}")
        packed, wdeq = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 1900 + cols, sigma=0.1, name=name)
        x = synth.activations(1, cols, synth.BASE_SEED + 1901)[0].view(np.uint16)
        g = (1.0 + 0.2 * np.random.default_rng(synth.BASE_SEED + 1902).standard_normal(cols)).astype(np.float16).view(np.uint16)
        r = synth.activations(1, rows, synth.BASE_SEED + 1903)[0].view(np.uint16)
        y = torch.full((rows,), float("nan"), dtype=torch.float16, device="cuda")
        iflow.qgemv_fused(fmt, [packed], [rows], cols, dev16(torch, x), [y], iflow.X_RMS_GAIN, dev16(torch, g), 1e-5, [dev16(torch, r)])
        torch.cuda.synchronize()
        assert err(bits_of(y), ops.rms_linear(wdeq, x, g, 1e-5, r)) <= TOL
        iflow.qgemv_fused(fmt, [packed], [rows], cols, dev16(torch, x), [y], iflow.X_SILU_MUL, dev16(torch, g), 0.0)
        torch.cuda.synchronize()
        assert err(bits_of(y), ops.silu_linear(wdeq, x, g)) <= TOL


def test_gated_pair_rows_longer_than_one_staging_pass(gpu, orc):
    """73 792 columns: the 3.5-bit kernel stages them in two passes and carries the partial sums; the other formats'
    kernel has no second pass and the call is refused before any launch."""
    torch, iflow = gpu
    from oracle import decode_ops as ops
    rows, cols = 40, 18 * 4096 + 64
    say(f"[case] gated pair Q3H_B64 rows={rows} cols={cols} (two staging passes)")
    gate = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 2000, sigma=2.0 / np.sqrt(cols))
    up = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 2001)
    x = synth.activations(1, cols, synth.BASE_SEED + 2002)[0].view(np.uint16)
    g = (1.0 + 0.2 * np.random.default_rng(synth.BASE_SEED + 2003).standard_normal(cols)).astype(np.float16).view(np.uint16)
    y = torch.full((rows,), float("nan"), dtype=torch.float16, device="cuda")
    iflow.qgemv_gated(iflow.Q3H_B64, gate[0], up[0], rows, cols, dev16(torch, x), y, iflow.X_RMS_GAIN, dev16(torch, g), 1e-5)
    torch.cuda.synchronize()
    e = gated_excess(bits_of(y), gate[1], up[1], x, g, 1e-5)
    say(f"        largest error / allowed error {e:.3f}")
    assert e <= 1.0
    fmt = iflow.FORMATS["Q4_B64"]
    n = iflow.packed_bytes(fmt, rows, cols)
    packed = torch.zeros(n, dtype=torch.uint8, device="cuda")
    with pytest.raises(iflow.IflowError) as info:
        iflow.qgemv_gated(fmt, packed, packed, rows, cols, dev16(torch, x), y)
    assert info.value.status == iflow.ERR_SHAPE
