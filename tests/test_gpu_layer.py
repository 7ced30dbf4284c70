"""GPU parity of a whole decoder layer of the decode step, the six launches a caller would issue per layer:

  rms norm -> q, k, v | rotary embedding + cache append | grouped-query attention | o + residual |
  rms norm -> silu(gate) * up | down + residual

Every launch is checked against the oracle's definition of that stage applied to the launch's ACTUAL inputs (read back
from the device), so each stage is held to its own bar and errors do not accumulate across stages; then the same six
launches are captured in a HIP graph and every replay must reproduce the eager results bit for bit.
"""
import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_fused import bits_of, dev16, err, gated_excess, make
from test_gpu_parity import TOL, gpu, say  # noqa: F401
from test_gpu_rope import close_bits

pytestmark = pytest.mark.gpu

N_HEADS, N_KV, D, FFN, MAX_SEQ, BASE, EPS = 4, 2, 128, 1408, 64, 10000.0, 1e-5
HIDDEN = N_HEADS * D


class Layer:
    def __init__(self, torch, iflow, orc, name, seed):
        self.torch, self.iflow, self.fmt = torch, iflow, iflow.FORMATS[name]
        shapes = {"q": (HIDDEN, HIDDEN), "k": (N_KV * D, HIDDEN), "v": (N_KV * D, HIDDEN), "o": (HIDDEN, HIDDEN),
                  "gate": (FFN, HIDDEN), "up": (FFN, HIDDEN), "down": (HIDDEN, FFN)}
        self.shape = shapes
        self.w = {k: make(torch, iflow, orc, r, c, seed + i, sigma=(0.08 if k == "gate" else 0.03), name=name)
                  for i, (k, (r, c)) in enumerate(shapes.items())}
        rng = np.random.default_rng(seed + 50)
        self.g1 = (1.0 + 0.1 * rng.standard_normal(HIDDEN)).astype(np.float16).view(np.uint16)
        self.g2 = (1.0 + 0.1 * rng.standard_normal(HIDDEN)).astype(np.float16).view(np.uint16)
        self.g1d, self.g2d = dev16(torch, self.g1), dev16(torch, self.g2)
        f16 = dict(dtype=torch.float16, device="cuda")
        self.q, self.k, self.v = (torch.empty((n,), **f16) for n in (HIDDEN, N_KV * D, N_KV * D))
        self.ao, self.hv = torch.empty((HIDDEN,), **f16), torch.empty((FFN,), **f16)
        self.ws_bytes = iflow.attn_decode_workspace_bytes(N_HEADS)
        self.ws = torch.empty((self.ws_bytes,), dtype=torch.uint8, device="cuda")

    def launches(self, h, kc, vc, position, stream=None):
        """The layer as a list of closures, one per launch, in order."""
        f, fmt, w, s = self.iflow, self.fmt, self.w, self.shape
        return [
            lambda: f.qgemv_fused(fmt, [w["q"][0], w["k"][0], w["v"][0]], [s["q"][0], s["k"][0], s["v"][0]], HIDDEN, h,
                                  [self.q, self.k, self.v], f.X_RMS_GAIN, self.g1d, EPS, stream=stream),
            lambda: f.rope_append(self.q, self.k, self.v, N_HEADS, N_KV, D, position, MAX_SEQ, BASE, f.ROPE_HALVES, kc, vc, stream=stream),
            lambda: f.attn_decode(self.q, kc, vc, N_HEADS, N_KV, D, position + 1, MAX_SEQ, D ** -0.5, self.ao, self.ws, self.ws_bytes,
                                  stream=stream),
            lambda: f.qgemv_fused(fmt, [w["o"][0]], [HIDDEN], HIDDEN, self.ao, [h], residual_list=[h], stream=stream),
            lambda: f.qgemv_gated(fmt, w["gate"][0], w["up"][0], FFN, HIDDEN, h, self.hv, f.X_RMS_GAIN, self.g2d, EPS, stream=stream),
            lambda: f.qgemv_fused(fmt, [w["down"][0]], [HIDDEN], FFN, self.hv, [h], residual_list=[h], stream=stream),
        ]


def start_state(torch, seed, filled):
    rng = np.random.default_rng(seed)
    h = rng.standard_normal(HIDDEN).astype(np.float16)
    kc = np.zeros((N_KV, MAX_SEQ, D), np.float16)
    vc = np.zeros((N_KV, MAX_SEQ, D), np.float16)
    kc[:, :filled] = rng.standard_normal((N_KV, filled, D)).astype(np.float16)
    vc[:, :filled] = rng.standard_normal((N_KV, filled, D)).astype(np.float16)
    to = lambda a: torch.from_numpy(a.copy()).cuda()
    return to(h), to(kc), to(vc)


@pytest.mark.parametrize("name", ["Q3H_B64", "Q4_B64", "Q8_B32", "Q5_B64"])
def test_three_decode_steps_stage_by_stage(gpu, orc, name):
    torch, iflow = gpu
    from oracle import attention as att
    from oracle import decode_ops as ops
    from oracle import rope as R
    layer = Layer(torch, iflow, orc, name, synth.BASE_SEED + 2100)
    filled = 21
    h, kc, vc = start_state(torch, synth.BASE_SEED + 2150, filled)
    sync = torch.cuda.synchronize
    for position in range(filled, filled + 3):
        say(f"[case] decoder layer {name}, position {position}: six launches, each against the oracle on its actual inputs")
        run = layer.launches(h, kc, vc, position)
        h0 = bits_of(h).copy()
        run[0](); sync()
        q0, k0, v0 = bits_of(layer.q).copy(), bits_of(layer.k).copy(), bits_of(layer.v).copy()
        for got, key in ((q0, "q"), (k0, "k"), (v0, "v")):
            assert err(got, ops.rms_linear(layer.w[key][1], h0, layer.g1, EPS)) <= TOL, key
        okc, ovc = bits_of(kc).copy(), bits_of(vc).copy()
        run[1](); sync()
        q_rot = R.rope_append(q0.reshape(N_HEADS, D), k0.reshape(N_KV, D), v0.reshape(N_KV, D), position, BASE, iflow.ROPE_HALVES, okc, ovc)
        assert close_bits(bits_of(layer.q), q_rot) and close_bits(bits_of(kc), okc) and np.array_equal(bits_of(vc), ovc)
        run[2](); sync()
        ref = att.gqa_decode(bits_of(layer.q).reshape(N_HEADS, D), bits_of(kc), bits_of(vc), position + 1, D ** -0.5)
        assert err(bits_of(layer.ao), ref.reshape(-1)) <= TOL
        ao = bits_of(layer.ao).copy()
        run[3](); sync()
        assert err(bits_of(h), ops.fused_gemv(layer.w["o"][1], ao, 1.0, h0)) <= TOL
        h1 = bits_of(h).copy()
        run[4](); sync()
        assert gated_excess(bits_of(layer.hv), layer.w["gate"][1], layer.w["up"][1], h1, layer.g2, EPS) <= 1.0
        hv = bits_of(layer.hv).copy()
        run[5](); sync()
        assert err(bits_of(h), ops.fused_gemv(layer.w["down"][1], hv, 1.0, h1)) <= TOL
        assert np.isfinite(h.cpu().numpy().astype(np.float32)).all()


def test_layer_graph_replays_equal_eager(gpu, orc):
    """The six launches captured once and replayed three times (the hidden state evolves, the cache row is rewritten),
    with eager work and synchronizations in between: every replay's results equal the eager sequence's, bit for bit."""
    torch, iflow = gpu
    layer = Layer(torch, iflow, orc, "Q3H_B64", synth.BASE_SEED + 2200)
    filled, position = 30, 30
    say("[case] decoder layer as a HIP graph: three replays against three eager passes")
    h, kc, vc = start_state(torch, synth.BASE_SEED + 2250, filled)
    eager = []
    for _ in range(3):
        for launch in layer.launches(h, kc, vc, position):
            launch()
        torch.cuda.synchronize()
        eager.append((bits_of(h).copy(), bits_of(layer.hv).copy(), bits_of(layer.ao).copy(), bits_of(kc).copy()))
    h2, kc2, vc2 = start_state(torch, synth.BASE_SEED + 2250, filled)
    stream = torch.cuda.Stream()
    raw = stream.cuda_stream
    graph = torch.cuda.CUDAGraph()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=stream):
        for launch in layer.launches(h2, kc2, vc2, position, stream=raw):
            launch()
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(h2), bits_of(start_state(torch, synth.BASE_SEED + 2250, filled)[0]))   # capturing ran nothing
    for i in range(3):
        graph.replay()
        torch.cuda.synchronize()
        got = (bits_of(h2), bits_of(layer.hv), bits_of(layer.ao), bits_of(kc2))
        for a, b in zip(got, eager[i]):
            assert np.array_equal(a, b), i
        _ = (torch.ones(1000, device="cuda") * 2).sum().item()                # eager work between the replays
