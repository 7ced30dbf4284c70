"""GPU parity of the chained launch with the modules of a decoder layer inside it (iflow_qgemv_chain_plan_fused): rms
normalization in front of a phase, the gate of a gated feed-forward where its two projections are summed, residuals at the
store.  Every phase's output is compared with the oracle's unsplit definition (oracle/decode_ops.py), evaluated on the
inputs the GPU actually used (read back from the device)."""
import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_chain import Arena
from test_gpu_fused import gated_excess
from test_gpu_parity import TOL, gpu, gpu_quantize, say  # noqa: F401

pytestmark = pytest.mark.gpu
EPS = 1e-5


def dev16(torch, bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.float16)


def bits_of(t):
    return t.cpu().numpy().view(np.uint16)


def err(y_bits, yref):
    y = y_bits.view(np.float16).astype(np.float64)
    rms = np.sqrt(np.mean(yref ** 2))
    return float(np.max(np.abs(y - yref) / np.maximum(np.abs(yref), max(rms, 1e-30))))


def quantized(torch, iflow, orc, rows, cols, seed, sigma, fmt_name="Q3H_B64"):
    w = synth.weights(rows, cols, sigma, seed)
    packed, _ = gpu_quantize(torch, iflow, iflow.FORMATS[fmt_name], w)
    q, s, o = orc.quantize(orc.FORMATS[fmt_name], w)
    return packed, orc.dequant(orc.FORMATS[fmt_name], q, s, o)


def layers_chain(torch, iflow, orc, hidden, ffn, nlayers, seed, fmt_name="Q3H_B64"):
    """nlayers decoder layers as four phases each: norm -> q,k,v | o + residual | norm -> silu(gate) * up | down + residual
    (q's output stands in for the attention output).  Returns the phases, a description of what each phase computes, and
    the hidden-state input of the launch."""
    arena = Arena(torch, 2 * nlayers * (8 * (hidden + 128) + 2 * (ffn + 128)))
    rng = np.random.default_rng(seed)
    h_in = dev16(torch, synth.activations(1, hidden, seed + 1)[0].view(np.uint16))
    phases, what = [], []
    h = h_in
    for layer in range(nlayers):
        s0 = seed + 100 * layer
        g1 = dev16(torch, (1.0 + 0.2 * rng.standard_normal(hidden)).astype(np.float16).view(np.uint16))
        g2 = dev16(torch, (1.0 + 0.2 * rng.standard_normal(hidden)).astype(np.float16).view(np.uint16))
        wq, wk, wv = [quantized(torch, iflow, orc, hidden, hidden, s0 + i, 1.0 / np.sqrt(hidden), fmt_name) for i in range(3)]
        wo = quantized(torch, iflow, orc, hidden, hidden, s0 + 3, 0.5 / np.sqrt(hidden), fmt_name)
        wg = quantized(torch, iflow, orc, ffn, hidden, s0 + 4, 2.0 / np.sqrt(hidden), fmt_name)
        wu = quantized(torch, iflow, orc, ffn, hidden, s0 + 5, 1.0 / np.sqrt(hidden), fmt_name)
        wd = quantized(torch, iflow, orc, hidden, ffn, s0 + 6, 0.5 / np.sqrt(ffn), fmt_name)
        q, k, v = arena.take(hidden), arena.take(hidden), arena.take(hidden)
        h1, a, h2 = arena.take(hidden), arena.take(ffn), arena.take(hidden)
        phases.append((hidden, h, [(wq[0], hidden, q), (wk[0], hidden, k), (wv[0], hidden, v)], {"x_op": iflow.X_RMS_GAIN, "aux": g1, "eps": EPS}))
        what.append(("norm_linear", h, g1, [(wq[1], q), (wk[1], k), (wv[1], v)]))
        phases.append((hidden, q, [(wo[0], hidden, h1, h)], {}))
        what.append(("linear_residual", q, h, [(wo[1], h1)]))
        phases.append((hidden, h1, [(wg[0], ffn, a), (wu[0], ffn, None)], {"x_op": iflow.X_RMS_GAIN, "aux": g2, "eps": EPS, "gated": True}))
        what.append(("norm_gated", h1, g2, [(wg[1], wu[1], a)]))
        phases.append((ffn, a, [(wd[0], hidden, h2, h1)], {}))
        what.append(("linear_residual", a, h1, [(wd[1], h2)]))
        h = h2
    return phases, what, h_in


def plan_fused(torch, iflow, phases, fmt_name="Q3H_B64"):
    rows_all = [m[1] for ph in phases for m in ph[2]]
    ws_bytes = iflow.qgemv_chain_workspace_bytes(rows_all)
    plan_bytes = iflow.qgemv_chain_plan_bytes(phases)
    ws = torch.full((ws_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    plan = torch.full((plan_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    return iflow.qgemv_chain_plan_fused(iflow.FORMATS[fmt_name], phases, plan, plan_bytes, ws, ws_bytes), (plan, ws)


def check(what, label):
    from oracle import decode_ops as ops
    worst = 0.0
    for p, item in enumerate(what):
        if item[0] == "norm_linear":
            _, x, g, outs = item
            for wdeq, y in outs:
                e = err(bits_of(y), ops.rms_linear(wdeq, bits_of(x), bits_of(g), EPS))
                assert np.isfinite(y.cpu().numpy().astype(np.float32)).all() and e <= TOL, f"{label}: phase {p} rel err {e}"
                worst = max(worst, e)
        elif item[0] == "linear_residual":
            _, x, r, outs = item
            for wdeq, y in outs:
                e = err(bits_of(y), ops.fused_gemv(wdeq, bits_of(x), 1.0, bits_of(r)))
                assert e <= TOL, f"{label}: phase {p} rel err {e}"
                worst = max(worst, e)
        else:
            _, x, g, outs = item
            for wg, wu, y in outs:
                e = gated_excess(bits_of(y), wg, wu, bits_of(x), bits_of(g), EPS)
                assert np.isfinite(y.cpu().numpy().astype(np.float32)).all() and e <= 1.0, f"{label}: phase {p} gated excess {e}"
    return worst


@pytest.mark.parametrize("hidden,ffn,nlayers", [(1088, 4160, 2), (256, 704, 3), (4096, 11008, 1)])
def test_fused_layers_in_one_launch(gpu, orc, hidden, ffn, nlayers):
    """Decoder layers (four dependent phases each, every module in use: two normalizations, a gated pair, residuals from a
    launch input and from earlier phases) in one launch; ragged strips (17 and 65 blocks), a tiny case, and 7B shapes."""
    torch, iflow = gpu
    say(f"[case] fused chain: {nlayers} layer(s), hidden={hidden} ffn={ffn}")
    phases, what, h_in = layers_chain(torch, iflow, orc, hidden, ffn, nlayers, synth.BASE_SEED + 4000 + hidden)
    chain, keep = plan_fused(torch, iflow, phases)
    assert chain.fused == 1
    for it in range(3):
        if it:                                                  # a new hidden state, outputs poisoned: nothing left over from the last launch
            h_in.copy_(dev16(torch, synth.activations(1, hidden, synth.BASE_SEED + 4100 + it)[0].view(np.uint16)))
            for _, _, mats, _ in phases:
                for m in mats:
                    if m[2] is not None:
                        m[2].fill_(float("nan"))
        iflow.qgemv_chain_launch(chain)
        iflow.qgemv_chain_check(chain)
        worst = check(what, f"launch {it}")
        say(f"        launch {it}: largest rel err of the linear phases {worst:.3e}")


@pytest.mark.parametrize("fmt_name,hidden,ffn,nlayers", [("Q4_B64", 1088, 4160, 2), ("Q8_B64", 1088, 4160, 2), ("Q4_B32", 256, 704, 3),
                                                         ("Q8_B32", 2112, 1088, 1), ("Q4_B64", 4096, 11008, 1),
                                                         ("Q6_B64", 1088, 4160, 2), ("Q5_B64", 256, 704, 3), ("Q3_B32", 2112, 1088, 1),
                                                         ("Q2_B32", 1088, 4160, 2)])
def test_fused_layers_in_one_launch_other_formats(gpu, orc, fmt_name, hidden, ffn, nlayers):
    """The same decoder layers through the chained launch of the 4- and 8-bit formats (every module in use)."""
    torch, iflow = gpu
    say(f"[case] fused chain, {fmt_name}: {nlayers} layer(s), hidden={hidden} ffn={ffn}")
    phases, what, h_in = layers_chain(torch, iflow, orc, hidden, ffn, nlayers, synth.BASE_SEED + 4500 + hidden, fmt_name)
    chain, keep = plan_fused(torch, iflow, phases, fmt_name)
    assert chain.fused == 1 and chain.format == iflow.FORMATS[fmt_name]
    for it in range(2):
        if it:
            h_in.copy_(dev16(torch, synth.activations(1, hidden, synth.BASE_SEED + 4600 + it)[0].view(np.uint16)))
            for _, _, mats, _ in phases:
                for m in mats:
                    if m[2] is not None:
                        m[2].fill_(float("nan"))
        iflow.qgemv_chain_launch(chain)
        iflow.qgemv_chain_check(chain)
        worst = check(what, f"{fmt_name} launch {it}")
        say(f"        launch {it}: largest rel err of the linear phases {worst:.3e}")


def test_fused_chain_graph_replay_and_plain_plan_unchanged(gpu, orc):
    """A fused chain captured in a HIP graph replays to the eager result; a plan without modules made through the fused
    entry point is the plain plan (same outputs, bit for bit, as iflow_qgemv)."""
    torch, iflow = gpu
    say("[case] fused chain: graph replay; plain plan through the fused entry point")
    phases, what, h_in = layers_chain(torch, iflow, orc, 512, 1408, 1, synth.BASE_SEED + 4200)
    chain, keep = plan_fused(torch, iflow, phases)
    iflow.qgemv_chain_launch(chain)
    torch.cuda.synchronize()
    eager = [bits_of(m[2]).copy() for _, _, mats, _ in phases for m in mats if m[2] is not None]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            iflow.qgemv_chain_launch(chain, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for _, _, mats, _ in phases:
            for m in mats:
                if m[2] is not None:
                    m[2].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        iflow.qgemv_chain_check(chain)
        got = [bits_of(m[2]) for _, _, mats, _ in phases for m in mats if m[2] is not None]
        assert all(np.array_equal(a, b) for a, b in zip(got, eager)), f"replay {rep}"
    # no module anywhere: the plain kernel runs, outputs equal iflow_qgemv's
    packed, _ = quantized(torch, iflow, orc, 300, 1024, synth.BASE_SEED + 4300, 0.02)
    x = dev16(torch, synth.activations(1, 1024, synth.BASE_SEED + 4301)[0].view(np.uint16))
    y = torch.full((300,), float("nan"), dtype=torch.float16, device="cuda")
    plain, keep2 = plan_fused(torch, iflow, [(1024, x, [(packed, 300, y)], {})])
    assert plain.fused == 0
    iflow.qgemv_chain_launch(plain)
    single = torch.empty((300,), dtype=torch.float16, device="cuda")
    iflow.qgemv(iflow.Q3H_B64, packed, 300, 1024, x, single)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(y), bits_of(single))
