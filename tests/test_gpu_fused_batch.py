"""GPU parity of iflow_qgemm_fused: the modules around the product for a small batch of activation vectors (every vector is
normalized, gated and carried on by itself), all nine formats, against the unsplit definitions in oracle/decode_ops.py
evaluated vector by vector."""
import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_fused import bits_of, dev16, err, make
from test_gpu_parity import NAMES, TOL, gpu, say  # noqa: F401

pytestmark = pytest.mark.gpu
EPS = 1e-5


def vectors(batch, n, seed, scale=1.0):
    """fp16 bit patterns [batch][n]; the vectors differ in size so that their normalization scalars differ"""
    x = synth.activations(batch, n, seed).astype(np.float32) * (scale * (1.0 + 0.5 * np.arange(batch)[:, None]))
    return x.astype(np.float16).view(np.uint16)


@pytest.mark.parametrize("name", NAMES)
@pytest.mark.parametrize("rows,cols,batch", [(100, 1408, 2), (37, 4096 + 64, 5), (520, 11008, 16)])
def test_batch_rms_gain_and_residual(gpu, orc, name, rows, cols, batch):
    """rms normalization per vector (one ragged strip; a second strip of one block; three strips at the full sixteen vectors)
    with a residual per vector."""
    torch, iflow = gpu
    from oracle import decode_ops as ops
    say(f"[case] batch fused rms gain {name} rows={rows} cols={cols} batch={batch}")
    packed, wdeq = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 5100 + rows, name=name)
    X = vectors(batch, cols, synth.BASE_SEED + 5101)
    g = (1.0 + 0.2 * np.random.default_rng(synth.BASE_SEED + 5102).standard_normal(cols)).astype(np.float16).view(np.uint16)
    R = vectors(batch, rows, synth.BASE_SEED + 5103, 0.5)
    Y = torch.full((batch, rows), float("nan"), dtype=torch.float16, device="cuda")
    iflow.qgemm_fused(iflow.FORMATS[name], packed, rows, cols, dev16(torch, X), batch, Y, iflow.X_RMS_GAIN, dev16(torch, g), EPS, dev16(torch, R))
    torch.cuda.synchronize()
    got = bits_of(Y)
    worst = max(err(got[b], ops.rms_linear(wdeq, X[b], g, EPS, R[b])) for b in range(batch))
    say(f"        max rel err {worst:.3e}")
    assert np.isfinite(Y.cpu().numpy().astype(np.float32)).all() and worst <= TOL


@pytest.mark.parametrize("name", NAMES)
def test_batch_silu_gate_in_place_residual_and_plain(gpu, orc, name):
    """The silu-gated input with the residual updated in place (the hidden states of seven queries), then the plain product
    with and without a residual; without any module the outputs are iflow_qgemm's."""
    torch, iflow = gpu
    from oracle import decode_ops as ops
    rows, cols, batch = 264, 2112, 7
    say(f"[case] batch fused silu gate / plain {name} rows={rows} cols={cols} batch={batch}")
    fmt = iflow.FORMATS[name]
    packed, wdeq = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 5200, name=name)
    A = vectors(batch, cols, synth.BASE_SEED + 5201)
    B = vectors(batch, cols, synth.BASE_SEED + 5202, 0.7)
    H = vectors(batch, rows, synth.BASE_SEED + 5203, 0.5)
    hidden = dev16(torch, H).clone()
    iflow.qgemm_fused(fmt, packed, rows, cols, dev16(torch, A), batch, hidden, iflow.X_SILU_MUL, dev16(torch, B), 0.0, hidden)
    torch.cuda.synchronize()
    got = bits_of(hidden)
    worst = max(err(got[b], ops.silu_linear(wdeq, A[b], B[b], H[b])) for b in range(batch))
    assert np.isfinite(hidden.cpu().numpy().astype(np.float32)).all() and worst <= TOL, f"silu gate: {worst}"
    Y = torch.full((batch, rows), float("nan"), dtype=torch.float16, device="cuda")
    iflow.qgemm_fused(fmt, packed, rows, cols, dev16(torch, A), batch, Y, iflow.X_PLAIN, None, 0.0, dev16(torch, H))
    torch.cuda.synchronize()
    got = bits_of(Y)
    worst_p = max(err(got[b], ops.fused_gemv(wdeq, A[b], 1.0, H[b])) for b in range(batch))
    assert worst_p <= TOL, f"plain + residual: {worst_p}"
    Y2 = torch.full((batch, rows), float("nan"), dtype=torch.float16, device="cuda")
    Y3 = torch.full((batch, rows), float("nan"), dtype=torch.float16, device="cuda")
    iflow.qgemm_fused(fmt, packed, rows, cols, dev16(torch, A), batch, Y2)
    iflow.qgemm(fmt, packed, rows, cols, dev16(torch, A), batch, Y3)
    torch.cuda.synchronize()
    e23 = max(err(bits_of(Y2)[b], bits_of(Y3)[b].view(np.float16).astype(np.float64)) for b in range(batch))
    assert e23 <= TOL
    say(f"        max rel err {worst:.3e} (silu gate), {worst_p:.3e} (plain + residual), {e23:.3e} against iflow_qgemm")


def test_batch_of_one_is_the_vector_entry_point(gpu, orc):
    torch, iflow = gpu
    from oracle import decode_ops as ops
    rows, cols = 300, 1024
    packed, wdeq = make(torch, iflow, orc, rows, cols, synth.BASE_SEED + 5300)
    X = vectors(1, cols, synth.BASE_SEED + 5301)
    g = (1.0 + 0.2 * np.random.default_rng(synth.BASE_SEED + 5302).standard_normal(cols)).astype(np.float16).view(np.uint16)
    Y = torch.full((1, rows), float("nan"), dtype=torch.float16, device="cuda")
    y1 = torch.full((rows,), float("nan"), dtype=torch.float16, device="cuda")
    iflow.qgemm_fused(iflow.Q3H_B64, packed, rows, cols, dev16(torch, X), 1, Y, iflow.X_RMS_GAIN, dev16(torch, g), EPS)
    iflow.qgemv_fused(iflow.Q3H_B64, [packed], [rows], cols, dev16(torch, X[0]), [y1], iflow.X_RMS_GAIN, dev16(torch, g), EPS)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(Y)[0], bits_of(y1))
    assert err(bits_of(Y)[0], ops.rms_linear(wdeq, X[0], g, EPS)) <= TOL
    with pytest.raises(iflow.IflowError) as ei:                 # more than sixteen vectors
        iflow.qgemm_fused(iflow.Q3H_B64, packed, rows, cols, dev16(torch, vectors(17, cols, 1)), 17,
                          torch.empty((17, rows), dtype=torch.float16, device="cuda"))
    assert ei.value.status == iflow.ERR_SHAPE
