"""GPU parity of a whole decode step of a decoder stack in one launch (iflow_decode_stack_plan / _launch): per layer the
rms-normalized q, k, v products, the rotary embedding with the cache append, grouped-query attention, the output projection
with its residual, the gated feed-forward and the down projection with its residual.  The launch leaves every intermediate
vector in its scratch buffer, so every stage is compared with the oracle's definition of that stage (oracle/decode_ops.py,
oracle/rope.py, oracle/attention.py) evaluated on the inputs the GPU actually used, as in test_gpu_layer.py, and the cache
rows are compared with what iflow_rope_append writes for the same inputs."""
import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_fused import bits_of, dev16, err, gated_excess, make
from test_gpu_parity import TOL, gpu, say  # noqa: F401
from test_gpu_rope import close_bits

pytestmark = pytest.mark.gpu
D, BASE, EPS = 128, 10000.0, 1e-5


def r128(n):
    return (n + 127) // 128 * 128


class Stack:
    """A stack of random layers with its device buffers, planned once."""

    def __init__(self, torch, iflow, orc, name, n_layers, n_heads, n_kv, ffn, max_seq, pairing, seed, filled):
        self.torch, self.iflow, self.name = torch, iflow, name
        self.n_layers, self.n_heads, self.n_kv, self.ffn, self.max_seq, self.pairing = n_layers, n_heads, n_kv, ffn, max_seq, pairing
        self.hidden = hidden = n_heads * D
        kvd = n_kv * D
        rng = np.random.default_rng(seed)
        self.layers = []
        for l in range(n_layers):
            s0 = seed + 100 * l
            shapes = {"wq": (hidden, hidden, 1.0), "wk": (kvd, hidden, 1.0), "wv": (kvd, hidden, 1.0), "wo": (hidden, hidden, 0.5),
                      "w_gate": (ffn, hidden, 2.0), "w_up": (ffn, hidden, 1.0), "w_down": (hidden, ffn, 0.5)}
            ly = {"w16": {}}
            for i, (key, (r, c, gain)) in enumerate(shapes.items()):
                ly[key], ly["w16"][key] = make(torch, iflow, orc, r, c, s0 + i, sigma=gain / np.sqrt(c), name=name)
            for key in ("norm1", "norm2"):
                ly[key + "_bits"] = (1.0 + 0.2 * rng.standard_normal(hidden)).astype(np.float16).view(np.uint16)
                ly[key] = dev16(torch, ly[key + "_bits"])
            kc = np.zeros((n_kv, max_seq, D), np.float16)
            vc = np.zeros((n_kv, max_seq, D), np.float16)
            kc[:, :filled] = rng.standard_normal((n_kv, filled, D)).astype(np.float16)
            vc[:, :filled] = rng.standard_normal((n_kv, filled, D)).astype(np.float16)
            ly["k_cache"], ly["v_cache"] = torch.from_numpy(kc).cuda(), torch.from_numpy(vc).cuda()
            self.layers.append(ly)
        f16 = dict(dtype=torch.float16, device="cuda")
        self.h_in = dev16(torch, synth.activations(1, hidden, seed + 7)[0].view(np.uint16))
        self.h_out = torch.zeros((hidden,), **f16)
        self.off = {}
        o = 0
        for key, n in (("q", hidden), ("k", kvd), ("v", kvd), ("t", hidden), ("h1", hidden), ("a", ffn), ("h2", hidden)):
            self.off[key] = (o, n)
            o += r128(n)
        self.per_layer = o
        fmt = iflow.FORMATS[name]
        sizes = iflow.decode_stack_sizes(iflow.decode_stack(fmt, hidden, ffn, n_heads, n_kv, max_seq, EPS, BASE, pairing, n_layers=n_layers))
        assert sizes[0] == n_layers * self.per_layer * 2
        self.scratch = torch.zeros((sizes[0] // 2,), **f16)
        self.plan = torch.empty((sizes[1],), dtype=torch.uint8, device="cuda")
        self.ws = torch.empty((sizes[2],), dtype=torch.uint8, device="cuda")
        self.desc = iflow.decode_stack(fmt, hidden, ffn, n_heads, n_kv, max_seq, EPS, BASE, pairing, layers=self.layers, h_in=self.h_in,
                                       h_out=self.h_out, scratch=self.scratch)
        self.chain = iflow.decode_stack_plan(self.desc, self.plan, sizes[1], self.ws, sizes[2])

    def vec(self, scratch_bits, layer, key):
        o, n = self.off[key]
        return scratch_bits[layer * self.per_layer + o: layer * self.per_layer + o + n]

    def step_and_check(self, position):
        """One launch at `position`, then every stage of every layer against the oracle on the stage's actual inputs."""
        from oracle import attention as att
        from oracle import decode_ops as ops
        from oracle import rope as R
        torch, iflow = self.torch, self.iflow
        before = [(bits_of(ly["k_cache"]).copy(), bits_of(ly["v_cache"]).copy()) for ly in self.layers]
        iflow.decode_stack_launch(self.chain, position)
        iflow.qgemv_chain_check(self.chain)
        s = bits_of(self.scratch)
        h = bits_of(self.h_in)
        for l, ly in enumerate(self.layers):
            w = ly["w16"]
            q, k, v = (self.vec(s, l, key) for key in ("q", "k", "v"))
            for got, key in ((q, "wq"), (k, "wk"), (v, "wv")):
                assert err(got, ops.rms_linear(w[key], h, ly["norm1_bits"], EPS)) <= TOL, (l, key)
            # the caches: row `position` holds the rotated key and the value, every other row is untouched
            okc, ovc = before[l][0].copy(), before[l][1].copy()
            q_rot = R.rope_append(q.reshape(self.n_heads, D), k.reshape(self.n_kv, D), v.reshape(self.n_kv, D), position, BASE, self.pairing,
                                  okc, ovc)
            kc, vc = bits_of(ly["k_cache"]), bits_of(ly["v_cache"])
            assert close_bits(kc, okc) and np.array_equal(vc, ovc), l
            # ... and is what the stand-alone launch writes for the same inputs, bit for bit
            kc2, vc2 = torch.from_numpy(before[l][0].view(np.int16)).cuda(), torch.from_numpy(before[l][1].view(np.int16)).cuda()
            q2 = dev16(torch, q.copy())
            iflow.rope_append(q2, dev16(torch, k.copy()), dev16(torch, v.copy()), self.n_heads, self.n_kv, D, position, self.max_seq, BASE,
                              self.pairing, kc2, vc2)
            assert np.array_equal(bits_of(kc2), kc) and np.array_equal(bits_of(vc2), vc), l
            t = self.vec(s, l, "t")
            ref = att.gqa_decode(bits_of(q2).reshape(self.n_heads, D), kc, vc, position + 1, D ** -0.5)
            assert err(t, ref.reshape(-1)) <= TOL, l
            ref = att.gqa_decode(q_rot.reshape(self.n_heads, D), kc, vc, position + 1, D ** -0.5)
            assert err(t, ref.reshape(-1)) <= 2 * TOL, l       # (the oracle's own rotation of q: an fp16 step apart here and there)
            h1 = self.vec(s, l, "h1")
            assert err(h1, ops.fused_gemv(w["wo"], t, 1.0, h)) <= TOL, l
            a = self.vec(s, l, "a")
            assert gated_excess(a, w["w_gate"], w["w_up"], h1, ly["norm2_bits"], EPS) <= 1.0, l
            h2 = bits_of(self.h_out) if l == self.n_layers - 1 else self.vec(s, l, "h2")
            assert err(h2, ops.fused_gemv(w["w_down"], a, 1.0, h1)) <= TOL, l
            h = h2
        assert np.isfinite(self.h_out.cpu().numpy().astype(np.float32)).all()


@pytest.mark.parametrize("name,n_heads,n_kv,ffn,pairing", [
    ("Q3H_B64", 4, 2, 1408, 1),       # two query heads per key/value head
    ("Q3H_B64", 4, 4, 704, 0),        # one: multi-head attention; adjacent pairs
    ("Q3H_B64", 8, 2, 1408, 1),       # four: two passes over the range
    ("Q4_B64", 4, 2, 1408, 0),
    ("Q8_B32", 4, 2, 1408, 1),
    ("Q6_B64", 4, 2, 1408, 1),        # a bit-plane format
    ("Q3_B32", 4, 4, 704, 0),
])
def test_decode_steps_of_a_small_stack_stage_by_stage(gpu, orc, name, n_heads, n_kv, ffn, pairing):
    torch, iflow = gpu
    filled = 21
    say(f"[case] decode stack {name}, {n_heads} heads / {n_kv} kv heads, ffn {ffn}, pairing {pairing}: 2 layers, positions {filled}..{filled + 2}")
    st = Stack(torch, iflow, orc, name, 2, n_heads, n_kv, ffn, 64, pairing, synth.BASE_SEED + 3100 + n_heads + n_kv, filled)
    for position in range(filled, filled + 3):
        st.step_and_check(position)


def test_decode_stack_from_an_empty_cache(gpu, orc):
    """Positions 0, 1, 2 of a fresh sequence: the first step attends to its own key alone."""
    torch, iflow = gpu
    say("[case] decode stack Q3H_B64 from an empty cache: positions 0, 1, 2")
    st = Stack(torch, iflow, orc, "Q3H_B64", 2, 4, 2, 704, 16, 1, synth.BASE_SEED + 3200, 0)
    for position in range(3):
        st.step_and_check(position)
        if position == 0:                                      # softmax over one position: the attention output is the value itself
            s = bits_of(st.scratch)
            v, t = st.vec(s, 0, "v").reshape(2, D), st.vec(s, 0, "t").reshape(4, D)
            assert np.array_equal(t[0], v[0]) and np.array_equal(t[1], v[0]) and np.array_equal(t[2], v[1]) and np.array_equal(t[3], v[1])


@pytest.mark.parametrize("position", [1500, 2047])
def test_decode_stack_long_context_many_ranges(gpu, orc, position):
    """A context long enough that every key/value head's positions are split over many workgroups, each with several blocks
    (and, at the last row of the cache, the step's own position in the last range)."""
    torch, iflow = gpu
    say(f"[case] decode stack Q3H_B64, 8 heads / 4 kv heads, context {position}, cache of 2048 rows")
    st = Stack(torch, iflow, orc, "Q3H_B64", 1, 8, 4, 1408, 2048, 1, synth.BASE_SEED + 3300, position)
    st.step_and_check(position)


def test_decode_stack_at_7b_shape(gpu, orc):
    """Two layers of the 7B shape (32 heads, hidden 4096, feed-forward 11008) at position 700 of a 1024-row cache."""
    torch, iflow = gpu
    say("[case] decode stack Q3H_B64 at the 7B layer shape: 2 layers, position 700")
    st = Stack(torch, iflow, orc, "Q3H_B64", 2, 32, 32, 11008, 1024, 1, synth.BASE_SEED + 3400, 700)
    st.step_and_check(700)
    st.step_and_check(701)


def test_decode_stack_graph_replays_equal_eager(gpu, orc):
    """The launch captured once in a HIP graph and replayed three times, with eager work and synchronizations in between:
    every replay gives the eager launch's results bit for bit (same position: the cache row is rewritten with the same values)."""
    torch, iflow = gpu
    say("[case] decode stack Q3H_B64 as a HIP graph: three replays against the eager launch")
    st = Stack(torch, iflow, orc, "Q3H_B64", 2, 8, 4, 1408, 64, 1, synth.BASE_SEED + 3600, 33)
    st.step_and_check(33)
    want = (bits_of(st.h_out).copy(), bits_of(st.scratch).copy(), [bits_of(ly["k_cache"]).copy() for ly in st.layers])
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=stream):
        iflow.decode_stack_launch(st.chain, 33, stream=stream.cuda_stream)
    torch.cuda.synchronize()
    for i in range(3):
        st.h_out.zero_(); st.scratch.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        iflow.qgemv_chain_check(st.chain)
        assert np.array_equal(bits_of(st.h_out), want[0]) and np.array_equal(bits_of(st.scratch), want[1]), i
        for ly, kc in zip(st.layers, want[2]):
            assert np.array_equal(bits_of(ly["k_cache"]), kc), i
        _ = (torch.ones(1000, device="cuda") * 2).sum().item()                # eager work between the replays


def test_decode_stack_launch_and_plan_refuse_what_they_cannot_run(gpu, orc):
    torch, iflow = gpu
    say("[case] decode stack: refused positions, shapes and launches")
    st = Stack(torch, iflow, orc, "Q3H_B64", 1, 4, 2, 704, 16, 1, synth.BASE_SEED + 3500, 3)
    for position in (-1, 16, 1 << 40):
        with pytest.raises(iflow.IflowError) as info:
            iflow.decode_stack_launch(st.chain, position)
        assert info.value.status == iflow.ERR_SHAPE
    with pytest.raises(iflow.IflowError) as info:                 # a stack's plan needs a position
        iflow.qgemv_chain_launch(st.chain)
    assert info.value.status == iflow.ERR_SHAPE
    fmt = iflow.FORMATS["Q3H_B64"]
    bad = [dict(n_heads=6, n_kv_heads=2),                        # three query heads per key/value head
           dict(hidden=640),                                     # not n_heads * 128
           dict(head_dim=64), dict(ffn=100), dict(max_seq=0), dict(n_layers=0), dict(rope_pairing=2)]
    for change in bad:
        args = dict(fmt=fmt, hidden=512, ffn=704, n_heads=4, n_kv_heads=2, max_seq=16, eps=EPS, rope_base=BASE, rope_pairing=1, n_layers=1)
        args.update(change)
        with pytest.raises(iflow.IflowError) as info:
            iflow.decode_stack_sizes(iflow.decode_stack(**args))
        assert info.value.status == iflow.ERR_SHAPE, change
    with pytest.raises(iflow.IflowError) as info:
        iflow.decode_stack_sizes(iflow.decode_stack(99, 512, 704, 4, 2, 16, EPS, BASE, 1, n_layers=1))
    assert info.value.status == iflow.ERR_FORMAT
    st.step_and_check(3)                                         # the refused calls left the chain usable
