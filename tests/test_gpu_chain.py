"""GPU parity of the chained launch (iflow_qgemv_chain_plan / _launch): every phase against the CPU oracle and against the
single-product kernel on the same inputs; repeated launches, HIP-graph replays, decoder-layer shapes."""
import sys

import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_parity import TOL, gpu, gpu_quantize, rel_err, say  # noqa: F401

pytestmark = pytest.mark.gpu


class Arena:
    """All outputs of a chain as views of one allocation (also makes sure that views, not only whole tensors, work)."""

    def __init__(self, torch, nbytes):
        self.torch = torch
        self.buf = torch.empty((nbytes // 2,), dtype=torch.float16, device="cuda")
        self.used = 0

    def take(self, rows):
        n = (rows + 127) // 128 * 128
        assert self.used + n <= self.buf.numel()
        v = self.buf[self.used:self.used + rows]
        self.used += n
        v.fill_(float("nan"))
        return v


def plan_chain(torch, iflow, phases, stream=None, fmt_name="Q3H_B64"):
    """Workspace and plan buffers (filled with 0xFF first: the plan call has to zero what it needs) and the compiled chain."""
    rows_all = [m[1] for ph in phases for m in ph[2]]
    ws_bytes = iflow.qgemv_chain_workspace_bytes(rows_all)
    plan_bytes = iflow.qgemv_chain_plan_bytes(phases)
    ws = torch.full((ws_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    plan = torch.full((plan_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    chain = iflow.qgemv_chain_plan(iflow.FORMATS[fmt_name], phases, plan, plan_bytes, ws, ws_bytes, stream=stream)
    return chain, (plan, ws)


def build_chain(torch, iflow, spec, seed, sigma=0.02, fmt_name="Q3H_B64"):
    """spec: list of phases (cols, src, [rows...]) with src None (fresh input) or (phase, matrix) of an earlier
    phase.  Returns device phases for iflow.qgemv_chain_plan, host copies of the weights, the compiled chain and its
    buffers."""
    fmt = iflow.FORMATS[fmt_name]
    arena = Arena(torch, 2 * sum((r + 127) // 128 * 128 for _, _, rl in spec for r in rl) + 4096)
    phases, host = [], []
    for p, (cols, src, row_list) in enumerate(spec):
        mats, hw = [], []
        for j, rows in enumerate(row_list):
            w = synth.weights(rows, cols, sigma, seed + 100 * p + j)
            packed, _ = gpu_quantize(torch, iflow, fmt, w)
            mats.append((packed, rows, arena.take(rows)))
            hw.append(w)
        if src is None:
            x = torch.from_numpy(synth.activations(1, cols, seed + 7 + p)[0].view(np.int16)).cuda().view(torch.float16)
        else:
            x = phases[src[0]][2][src[1]][2]
            assert x.numel() == cols
        phases.append((cols, x, mats))
        host.append(hw)
    chain, keep = plan_chain(torch, iflow, phases, fmt_name=fmt_name)
    return phases, host, chain, keep


def same_as_single_product(got16, ref16, fmt_name="Q3H_B64"):
    """3.5-bit format: the chain runs the single-product kernel's loads, decode and sums in the same order - equal bit for
    bit.  The 4- and 8-bit formats' single-product kernel groups its rows differently, so its fp32 sums (of biased levels:
    large terms that cancel, which is where the 8-bit format spends most of its error budget) are added in another order: the
    two agree to within the product tolerance."""
    if fmt_name == "Q3H_B64":
        return bool(np.array_equal(got16, ref16))
    g = got16.view(np.float16).astype(np.float64)
    r = ref16.view(np.float16).astype(np.float64)
    return rel_err(g[None, :], r[None, :]) <= TOL


def check_phases(torch, iflow, orc, phases, host, what, fmt_name="Q3H_B64"):
    """Every output against the oracle (given the activations the GPU actually used) and against iflow_qgemv."""
    fmt, ofmt = iflow.FORMATS[fmt_name], orc.FORMATS[fmt_name]
    for p, (cols, x, mats) in enumerate(phases):
        xh = x.cpu().numpy().view(np.uint16)[None, :]
        for j, (packed, rows, y) in enumerate(mats):
            got = y.cpu().numpy()
            assert np.isfinite(got).all(), f"{what}: phase {p} matrix {j} has non-finite outputs"
            q, s, o = orc.quantize(ofmt, host[p][j])
            ref = orc.gemm(orc.dequant(ofmt, q, s, o), xh)[0]
            e = rel_err(got.astype(np.float64)[None, :], ref[None, :])
            assert e <= TOL, f"{what}: phase {p} matrix {j} rel err {e}"
            single = torch.empty((rows,), dtype=torch.float16, device="cuda")
            iflow.qgemv(fmt, packed, rows, cols, x, single)
            torch.cuda.synchronize()
            assert same_as_single_product(got.view(np.uint16), single.cpu().numpy().view(np.uint16), fmt_name), f"{what}: phase {p} matrix {j}"


SPEC_RAGGED = [
    (1408, None, [1024, 37, 2048]),        # 22 blocks: one ragged strip; an odd matrix in the middle
    (1024, (0, 0), [4160]),                # consumes the first output
    (4160, (1, 0), [100, 64]),             # 65 blocks: a second strip of one block
    (2048, (0, 2), [77]),                  # consumes an output from three phases back
    (128, None, [5]),                      # a fresh input in the middle of the chain; most workgroups have no rows
]


def test_chain_ragged_phases_and_relaunch(gpu, orc):
    torch, iflow = gpu
    say("[case] chain ragged spec, three launches with new inputs")
    phases, host, chain, keep = build_chain(torch, iflow, SPEC_RAGGED, synth.BASE_SEED + 500, sigma=0.03)
    for it in range(3):
        if it:
            for p, (cols, x, _) in enumerate(phases):
                if SPEC_RAGGED[p][1] is None:
                    x.copy_(torch.from_numpy(synth.activations(1, cols, synth.BASE_SEED + 600 + 10 * it + p)[0].view(np.int16)).cuda().view(torch.float16))
            for _, _, mats in phases:
                for m in mats:
                    m[2].fill_(float("nan"))
        iflow.qgemv_chain_launch(chain)
        iflow.qgemv_chain_check(chain)
        check_phases(torch, iflow, orc, phases, host, f"launch {it}")


# A wavefront's steps of all phases form one sequence over its register sets (no padding per phase in the 3.5-bit format): the
# phases below give the wavefronts 1, 2 or 4, 3, 3 and 2 or 4 steps (row pairs x strips), so that phases start at every set and
# end in the middle of a round, some wavefronts of a workgroup with more steps than others, one phase with rows for a few
# workgroups only.
SPEC_STEP_COUNTS = [
    (1408, None, [6144]),                  # one pair of rows per wavefront, one strip
    (6144, (0, 0), [6400]),                # two strips; the first wavefronts of a workgroup have two pairs, the others one
    (1408, None, [18432]),                 # three pairs, one strip
    (8256, None, [6144]),                  # one pair, three strips (the last one a single block)
    (6144, (3, 0), [6200, 37]),            # two strips again, an odd matrix behind
    (128, None, [5]),
    (1408, None, [6144]),                  # and a phase behind the nearly empty one
]


def test_chain_phases_of_every_step_count(gpu, orc):
    torch, iflow = gpu
    say("[case] chain whose phases give the wavefronts 1 to 4 steps each, two launches")
    phases, host, chain, keep = build_chain(torch, iflow, SPEC_STEP_COUNTS, synth.BASE_SEED + 520)
    for it in range(2):
        if it:
            for _, _, mats in phases:
                for m in mats:
                    m[2].fill_(float("nan"))
        iflow.qgemv_chain_launch(chain)
        iflow.qgemv_chain_check(chain)
        check_phases(torch, iflow, orc, phases, host, f"launch {it}")
    # the launch's clock stamps (a diagnostic of the workspace header): a plausible shader clock
    ws = keep[1]
    w = [int(v) & 0xFFFFFFFF for v in ws.view(torch.int32)[iflow.CHAIN_WS_CLOCKS:iflow.CHAIN_WS_CLOCKS + 4].cpu().tolist()]
    cycles, ticks = (w[2] - w[0]) & 0xFFFFFFFF, (w[3] - w[1]) & 0xFFFFFFFF
    assert ticks > 0 and 300.0 < 100.0 * cycles / ticks < 3500.0, (w, cycles, ticks)


@pytest.mark.parametrize("fmt_name", ["Q4_B64", "Q8_B64", "Q4_B32", "Q8_B32", "Q6_B64", "Q5_B64", "Q3_B32", "Q2_B32"])
def test_chain_other_formats_ragged_phases_and_relaunch(gpu, orc, fmt_name):
    """The 4- and 8-bit formats of Table 3 through the same chained launch (strips of 2048 and 1024 columns, block headers
    behind the codes): ragged strips, odd matrices, hand-overs across several phases, three launches."""
    torch, iflow = gpu
    say(f"[case] chain ragged spec, {fmt_name}, three launches with new inputs")
    phases, host, chain, keep = build_chain(torch, iflow, SPEC_RAGGED, synth.BASE_SEED + 540, sigma=0.03, fmt_name=fmt_name)
    assert chain.format == iflow.FORMATS[fmt_name]
    for it in range(3):
        if it:
            for p, (cols, x, _) in enumerate(phases):
                if SPEC_RAGGED[p][1] is None:
                    x.copy_(torch.from_numpy(synth.activations(1, cols, synth.BASE_SEED + 640 + 10 * it + p)[0].view(np.int16)).cuda().view(torch.float16))
            for _, _, mats in phases:
                for m in mats:
                    m[2].fill_(float("nan"))
        iflow.qgemv_chain_launch(chain)
        iflow.qgemv_chain_check(chain)
        check_phases(torch, iflow, orc, phases, host, f"{fmt_name} launch {it}", fmt_name=fmt_name)


@pytest.mark.parametrize("fmt_name", ["Q4_B64", "Q8_B64", "Q6_B64", "Q3_B32"])
def test_chain_other_formats_two_7b_layers(gpu, orc, fmt_name):
    """Config 3's formats at the 7B layer shapes: two decoder layers (eight dependent phases) in one launch; all rows against
    the single-product kernel, sampled rows of every output against the oracle."""
    torch, iflow = gpu
    say(f"[case] chain of two 7B-shaped layers, {fmt_name}")
    hidden, ffn = 4096, 11008
    fmt, ofmt = iflow.FORMATS[fmt_name], orc.FORMATS[fmt_name]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 560)
    arena = Arena(torch, 2 * 2 * (5 * hidden + 2 * ffn + 7 * 128) + 4096)
    x0 = (torch.randn((hidden,), generator=gen, device="cuda") * 2.0 ** -6).to(torch.float16)
    phases, keepw = [], []
    last = x0
    for layer in range(2):
        for rows_list, cols in (([hidden] * 3, hidden), ([hidden], hidden), ([ffn] * 2, hidden), ([hidden], ffn)):
            mats = []
            for rows in rows_list:
                w = torch.randn((rows, cols), generator=gen, device="cuda", dtype=torch.float32) * 0.02
                nb = iflow.packed_bytes(fmt, rows, cols)
                pk = torch.empty(nb, dtype=torch.uint8, device="cuda")
                iflow.quantize(fmt, w, rows, cols, pk, nb)
                keepw.append(w)
                mats.append((pk, rows, arena.take(rows)))
            phases.append((cols, last, mats))
            last = mats[0][2]
    chain, keep = plan_chain(torch, iflow, phases, fmt_name=fmt_name)
    for it in range(2):
        iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)
    rng = np.random.default_rng(synth.BASE_SEED + 561)
    wi = 0
    for p, (cols, x, mats) in enumerate(phases):
        xh = x.cpu().numpy().view(np.uint16)[None, :]
        for j, (pk, rows, y) in enumerate(mats):
            got = y.cpu().numpy()
            assert np.isfinite(got).all(), f"phase {p} matrix {j}"
            single = torch.empty((rows,), dtype=torch.float16, device="cuda")
            iflow.qgemv(fmt, pk, rows, cols, x, single)
            torch.cuda.synchronize()
            assert same_as_single_product(got.view(np.uint16), single.cpu().numpy().view(np.uint16), fmt_name), f"phase {p} matrix {j}: differs from iflow_qgemv"
            pick = np.unique(np.concatenate([[0, 1, rows - 2, rows - 1], rng.integers(0, rows, 28)]))
            wsel = keepw[wi][torch.from_numpy(pick).cuda()].cpu().numpy()
            q, s_, o_ = orc.quantize(ofmt, wsel)
            ref = orc.gemm(orc.dequant(ofmt, q, s_, o_), xh)[0]
            e = rel_err(got.astype(np.float64)[pick][None, :], ref[None, :])
            assert e <= TOL, f"phase {p} matrix {j}: rel err {e}"
            wi += 1


def test_chain_single_phase_is_qgemv(gpu, orc):
    torch, iflow = gpu
    say("[case] chain of one phase, 1024x1024")
    phases, host, chain, keep = build_chain(torch, iflow, [(1024, None, [1024])], synth.BASE_SEED + 520)
    iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)
    check_phases(torch, iflow, orc, phases, host, "single")


def test_chain_of_32_phases_many_launches(gpu, orc):
    """A chain of 32 tiny phases, each feeding the next (hand-overs dominate), launched many times in a row."""
    torch, iflow = gpu
    say("[case] chain of 32 dependent phases, 512 <-> 320 columns, 40 launches")
    spec = [(512, None, [320])]
    for p in range(1, 32):
        spec.append((320, (p - 1, 0), [512]) if p % 2 else (512, (p - 1, 0), [320]))
    phases, host, chain, keep = build_chain(torch, iflow, spec, synth.BASE_SEED + 700, sigma=0.05)
    for it in range(40):
        iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)
    check_phases(torch, iflow, orc, phases, host, "after 40 launches")
    with pytest.raises(iflow.IflowError) as ei:                 # the same matrix twice: two outputs overlap
        plan_chain(torch, iflow, phases + [phases[0]])
    assert ei.value.status == iflow.ERR_SHAPE


def test_chain_with_the_most_matrices(gpu, orc):
    """56 matrices in one launch: 14 phases of four, each phase reading one output of the phase before."""
    torch, iflow = gpu
    say("[case] chain of 14 phases x 4 matrices, 128x128")
    spec = [(128, None, [128] * 4)] + [(128, (p - 1, p % 4), [128] * 4) for p in range(1, 14)]
    phases, host, chain, keep = build_chain(torch, iflow, spec, synth.BASE_SEED + 800, sigma=0.08)
    for it in range(3):
        iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)
    check_phases(torch, iflow, orc, phases, host, "56 matrices")


def layer_spec(hidden, ffn):
    return [(hidden, None, [hidden, hidden, hidden]), (hidden, (0, 0), [hidden]),
            (hidden, (1, 0), [ffn, ffn]), (ffn, (2, 0), [hidden])]


def test_chain_decoder_layer_7b_and_graph_replay(gpu, orc):
    torch, iflow = gpu
    say("[case] chain 7B decoder layer: q/k/v -> o -> gate/up -> down, eager then five HIP-graph replays")
    spec = layer_spec(4096, 11008)
    phases, host, chain, keep = build_chain(torch, iflow, spec, synth.BASE_SEED + 540, sigma=0.012)
    fmt = iflow.Q3H_B64

    def reference():                       # the launches the chain replaces, on the same buffers
        outs = []
        for cols, x, mats in phases:
            ys = [torch.empty((m[1],), dtype=torch.float16, device="cuda") for m in mats]
            outs.append(ys)
        for p, (cols, x, mats) in enumerate(phases):
            src = spec[p][1]
            xin = x if src is None else outs[src[0]][src[1]]
            iflow.qgemv_multi(fmt, [m[0] for m in mats], [m[1] for m in mats], cols, xin, outs[p])
        torch.cuda.synchronize()
        return [[y.cpu().numpy().view(np.uint16) for y in ys] for ys in outs]

    def compare(what):
        ref = reference()
        for p, (_, _, mats) in enumerate(phases):
            for j, m in enumerate(mats):
                got = m[2].cpu().numpy().view(np.uint16)
                assert same_as_single_product(got, ref[p][j]), f"{what}: phase {p} matrix {j}: {(got != ref[p][j]).sum()} of {got.size} differ"

    iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)
    compare("eager")
    # sampled rows of the last phase against the oracle
    ofmt = orc.FORMATS["Q3H_B64"]
    cols, x, mats = phases[3]
    idx = synth.sample_rows(mats[0][1], 48, synth.BASE_SEED + 541)
    q, s, o = orc.quantize(ofmt, host[3][0][idx])
    ref = orc.gemm(orc.dequant(ofmt, q, s, o), x.cpu().numpy().view(np.uint16)[None, :])[0]
    got = mats[0][2].cpu().numpy().astype(np.float64)[idx]
    full = mats[0][2].cpu().numpy().astype(np.float64)
    rms = np.sqrt(np.mean(full ** 2))
    assert float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms))) <= TOL

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            iflow.qgemv_chain_launch(chain, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(5):
        x0 = phases[0][1]
        x0.copy_(torch.from_numpy(synth.activations(1, 4096, synth.BASE_SEED + 560 + rep)[0].view(np.int16)).cuda().view(torch.float16))
        for _, _, mats in phases:
            for m in mats:
                m[2].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        if rep % 2:
            graph.replay()                 # back-to-back replays: the second starts from the first one's workspace
        torch.cuda.synchronize()
        iflow.qgemv_chain_check(chain)
        compare(f"replay {rep}")


def test_chain_decoder_layer_70b_shapes(gpu, orc):
    """A 70B-shaped layer (hidden 8192, grouped k/v of 1024 rows, feed-forward 28672): seven strips of activations in
    the last phase, 57344 rows in the widest one.  Weights are drawn on the device (the host generator would take
    minutes for 0.86 G weights); every output must equal, bit for bit, what the separate launches give, and sampled
    rows of the first and last phase are checked against the oracle."""
    torch, iflow = gpu
    fmt, ofmt = iflow.Q3H_B64, orc.FORMATS["Q3H_B64"]
    hidden, kv, ffn = 8192, 1024, 28672
    say(f"[case] chain 70B-shaped layer hidden={hidden} kv={kv} ffn={ffn}")
    spec = [(hidden, None, [hidden, kv, kv]), (hidden, (0, 0), [hidden]),
            (hidden, (1, 0), [ffn, ffn]), (ffn, (2, 0), [hidden])]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 900)
    arena = Arena(torch, 2 * sum(r + 128 for _, _, rl in spec for r in rl))
    phases, kept = [], {}
    for p, (cols, src, row_list) in enumerate(spec):
        mats = []
        for j, rows in enumerate(row_list):
            wd = torch.randn((rows, cols), generator=gen, device="cuda", dtype=torch.float32) * 0.01
            n = iflow.packed_bytes(fmt, rows, cols)
            packed = torch.empty(n, dtype=torch.uint8, device="cuda")
            iflow.quantize(fmt, wd, rows, cols, packed, n)
            if (p, j) in ((0, 0), (3, 0)):
                idx = synth.sample_rows(rows, 32, synth.BASE_SEED + 901 + p)
                kept[(p, j)] = (idx, wd[torch.from_numpy(idx).cuda()].cpu().numpy())
            del wd
            mats.append((packed, rows, arena.take(rows)))
        if src is None:
            x = torch.from_numpy(synth.activations(1, cols, synth.BASE_SEED + 902)[0].view(np.int16)).cuda().view(torch.float16)
        else:
            x = phases[src[0]][2][src[1]][2]
        phases.append((cols, x, mats))
    chain, keep = plan_chain(torch, iflow, phases)
    for it in range(2):
        iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)
    xin = phases[0][1]
    for p, (cols, _, mats) in enumerate(phases):
        ys = [torch.empty((m[1],), dtype=torch.float16, device="cuda") for m in mats]
        iflow.qgemv_multi(fmt, [m[0] for m in mats], [m[1] for m in mats], cols, xin, ys)
        torch.cuda.synchronize()
        for j, m in enumerate(mats):
            got, ref = m[2].cpu().numpy().view(np.uint16), ys[j].cpu().numpy().view(np.uint16)
            assert same_as_single_product(got, ref), f"phase {p} matrix {j}: {(got != ref).sum()} of {got.size} differ"
            if (p, j) in kept:
                idx, w_rows = kept[(p, j)]
                q, s, o = orc.quantize(ofmt, w_rows)
                want = orc.gemm(orc.dequant(ofmt, q, s, o), xin.cpu().numpy().view(np.uint16)[None, :])[0]
                full = m[2].cpu().numpy().astype(np.float64)
                rms = np.sqrt(np.mean(full ** 2))
                e = float(np.max(np.abs(full[idx] - want) / np.maximum(np.abs(want), rms)))
                say(f"        phase {p}: max rel err on {len(idx)} sampled rows {e:.3e}")
                assert np.isfinite(full).all() and e <= TOL
        xin = ys[0]


def test_chain_benchmark_configuration_eight_layers(gpu, orc):
    """The launch the benchmark times: eight 7B-shaped layers (32 dependent phases, 56 matrices, 0.81 GB of codes) in one
    launch.  Every output must equal, bit for bit, what separate launches give on the same inputs; sampled rows of the
    first and the last layer are checked against the oracle, given the activations the GPU actually used."""
    torch, iflow = gpu
    fmt, ofmt = iflow.Q3H_B64, orc.FORMATS["Q3H_B64"]
    hidden, ffn, nlayers = 4096, 11008, 8
    say(f"[case] chain of {nlayers} 7B-shaped layers in one launch")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 1000)
    arena = Arena(torch, 2 * nlayers * (4 * (hidden + 128) + 2 * (ffn + 128) + (hidden + 128)))
    phases, kept = [], {}
    x0 = torch.from_numpy((synth.activations(1, hidden, synth.BASE_SEED + 1001)[0].astype(np.float32) * 2.0 ** -10)
                          .astype(np.float16).view(np.int16)).cuda().view(torch.float16)
    prev_down = None
    for layer in range(nlayers):
        base = len(phases)
        spec = [(hidden, None if layer == 0 else prev_down, [hidden] * 3), (hidden, (base, 0), [hidden]),
                (hidden, (base + 1, 0), [ffn, ffn]), (ffn, (base + 2, 0), [hidden])]
        for p, (cols, src, row_list) in enumerate(spec):
            mats = []
            for j, rows in enumerate(row_list):
                wd = torch.randn((rows, cols), generator=gen, device="cuda", dtype=torch.float32) * 0.02
                n = iflow.packed_bytes(fmt, rows, cols)
                packed = torch.empty(n, dtype=torch.uint8, device="cuda")
                iflow.quantize(fmt, wd, rows, cols, packed, n)
                if layer in (0, nlayers - 1) and j == 0:
                    idx = synth.sample_rows(rows, 16, synth.BASE_SEED + 1002 + p)
                    kept[(base + p, j)] = (idx, wd[torch.from_numpy(idx).cuda()].cpu().numpy())
                del wd
                mats.append((packed, rows, arena.take(rows)))
            x = x0 if src is None else phases[src[0]][2][src[1]][2]
            phases.append((cols, x, mats))
        prev_down = (base + 3, 0)
    chain, keep = plan_chain(torch, iflow, phases)
    for it in range(2):
        iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)
    for p, (cols, x, mats) in enumerate(phases):
        ys = [torch.empty((m[1],), dtype=torch.float16, device="cuda") for m in mats]
        iflow.qgemv_multi(fmt, [m[0] for m in mats], [m[1] for m in mats], cols, x, ys)
        torch.cuda.synchronize()
        for j, m in enumerate(mats):
            got, ref = m[2].cpu().numpy().view(np.uint16), ys[j].cpu().numpy().view(np.uint16)
            assert same_as_single_product(got, ref), f"phase {p} matrix {j}: {(got != ref).sum()} of {got.size} differ"
            if (p, j) in kept:
                idx, w_rows = kept[(p, j)]
                q, s, o = orc.quantize(ofmt, w_rows)
                want = orc.gemm(orc.dequant(ofmt, q, s, o), x.cpu().numpy().view(np.uint16)[None, :])[0]
                full = m[2].cpu().numpy().astype(np.float64)
                assert np.isfinite(full).all(), f"phase {p}: non-finite outputs"
                rms = np.sqrt(np.mean(full ** 2))
                e = float(np.max(np.abs(full[idx] - want) / np.maximum(np.abs(want), rms)))
                assert e <= TOL, f"phase {p}: rel err {e}"


def test_chain_check_reports_a_recorded_timeout(gpu, orc):
    """The error path of iflow_qgemv_chain_check, forced from the host: the word a phase raises when its bounded wait expires
    is set with a device copy (no kernel waits for anything), the check reports IFLOW_ERR_TIMEOUT until the chain is planned
    again, and planning again clears it."""
    torch, iflow = gpu
    say("[case] chain check: error word set by the host")
    phases, host, chain, keep = build_chain(torch, iflow, [(256, None, [64])], synth.BASE_SEED + 1200)
    plan, ws = keep
    iflow.qgemv_chain_launch(chain)
    iflow.qgemv_chain_check(chain)                             # a normal launch: no record
    ws.view(torch.int32)[1] = 1                                # what a phase writes when it gives up its wait
    torch.cuda.synchronize()
    with pytest.raises(iflow.IflowError) as ei:
        iflow.qgemv_chain_check(chain)
    assert ei.value.status == iflow.ERR_TIMEOUT
    iflow.qgemv_chain_launch(chain)                            # the record stays: later launches do not clear it
    with pytest.raises(iflow.IflowError):
        iflow.qgemv_chain_check(chain)
    chain2 = iflow.qgemv_chain_plan(iflow.Q3H_B64, phases, plan, plan.numel(), ws, ws.numel())
    iflow.qgemv_chain_launch(chain2)
    iflow.qgemv_chain_check(chain2)
    check_phases(torch, iflow, orc, phases, host, "after planning again")
