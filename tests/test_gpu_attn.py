"""GPU parity of iflow_attn_decode (one decode step of grouped-query attention over an fp16 key/value cache) against the
plain definition in oracle/attention.py."""
import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_parity import TOL, gpu, say  # noqa: F401

pytestmark = pytest.mark.gpu


def dev16(torch, a16):
    return torch.from_numpy(np.ascontiguousarray(a16).view(np.int16)).cuda().view(torch.float16)


def rel(got, ref):
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), np.maximum(rms, 1e-30))))


def make(n_heads, n_kv, max_seq, seed, q_scale=1.0, d=128):
    rng = np.random.default_rng(seed)
    q = (q_scale * rng.standard_normal((n_heads, d))).astype(np.float16)
    k = rng.standard_normal((n_kv, max_seq, d)).astype(np.float16)
    v = rng.standard_normal((n_kv, max_seq, d)).astype(np.float16)
    return q, k, v


def run(torch, iflow, q, k, v, T, scale, ws=None):
    n_heads, n_kv, max_seq, d = q.shape[0], k.shape[0], k.shape[1], q.shape[1]
    nbytes = iflow.attn_decode_workspace_bytes(n_heads)
    if ws is None:
        ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")       # scratch: NaN patterns to start with
    out = torch.full((n_heads, d), float("nan"), dtype=torch.float16, device="cuda")
    iflow.attn_decode(dev16(torch, q), dev16(torch, k), dev16(torch, v), n_heads, n_kv, d, T, max_seq, scale, out, ws, nbytes)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), ws


@pytest.mark.parametrize("n_heads,n_kv,T,max_seq", [(32, 32, 1, 64), (32, 32, 17, 64), (8, 8, 64, 64), (8, 4, 130, 200),
                                                    (32, 32, 1000, 1024), (64, 8, 777, 1024), (16, 4, 4096, 4096), (4, 1, 5000, 8192)])
def test_attention_decode_against_the_definition(gpu, n_heads, n_kv, T, max_seq):
    torch, iflow = gpu
    from oracle import attention as att
    say(f"[case] attention decode heads={n_heads} kv_heads={n_kv} seq_len={T} max_seq={max_seq}")
    q, k, v = make(n_heads, n_kv, max_seq, synth.BASE_SEED + 1500 + T)
    scale = 1.0 / np.sqrt(128.0)
    got, _ = run(torch, iflow, q, k, v, T, scale)
    ref = att.gqa_decode(q.view(np.uint16), k.view(np.uint16), v.view(np.uint16), T, scale)
    e = rel(got, ref)
    say(f"        max rel err {e:.3e}")
    assert np.isfinite(got).all() and e <= TOL


@pytest.mark.parametrize("n_heads,n_kv,d,T,max_seq", [
    (128, 8, 64, 1000, 1024),      # sixteen 64-component query heads per key/value head (the paper's Falcon-40B: Table 3, Table 5)
    (71, 1, 64, 777, 1024),        # multi-query attention: every head shares one key/value head (five pieces of sixteen heads)
    (32, 32, 64, 130, 200),        # multi-head attention at 64 components
    (16, 8, 64, 1, 64), (24, 8, 64, 65, 128), (40, 8, 64, 4096, 4096),       # groups of 2, 3 and 5 at 64 components
    (24, 8, 128, 300, 512), (48, 8, 128, 1000, 1024), (56, 8, 128, 129, 256), (128, 8, 128, 2049, 4096),   # groups of 3, 6, 7 and 16 at 128
    (40, 2, 128, 555, 1024), (33, 1, 128, 64, 64),                           # groups of 20 and 33: several pieces, the last ragged
])
def test_attention_other_head_dimensions_and_group_sizes(gpu, n_heads, n_kv, d, T, max_seq):
    """Section "Grouped-query attention": H heads in G groups, any ratio; head dimension 64 next to 128."""
    torch, iflow = gpu
    from oracle import attention as att
    say(f"[case] attention decode heads={n_heads} kv_heads={n_kv} head_dim={d} seq_len={T} max_seq={max_seq}")
    q, k, v = make(n_heads, n_kv, max_seq, synth.BASE_SEED + 1700 + T + n_heads, d=d)
    scale = 1.0 / np.sqrt(float(d))
    got, _ = run(torch, iflow, q, k, v, T, scale)
    ref = att.gqa_decode(q.view(np.uint16), k.view(np.uint16), v.view(np.uint16), T, scale)
    e = rel(got, ref)
    say(f"        max rel err {e:.3e}")
    assert np.isfinite(got).all() and e <= TOL


def test_attention_peaked_softmax_and_reused_workspace(gpu):
    """Large scores (one position dominates, the running maximum moves a lot) and several launches of different lengths
    on one workspace (left as the previous launch wrote it)."""
    torch, iflow = gpu
    from oracle import attention as att
    n_heads, n_kv, max_seq = 16, 8, 3000
    q, k, v = make(n_heads, n_kv, max_seq, synth.BASE_SEED + 1600, q_scale=6.0)
    ws = None
    for T in (3000, 65, 1, 2049, 3000):
        say(f"[case] attention, peaked scores, seq_len={T}, shared workspace")
        got, ws = run(torch, iflow, q, k, v, T, 0.5, ws)
        ref = att.gqa_decode(q.view(np.uint16), k.view(np.uint16), v.view(np.uint16), T, 0.5)
        e = rel(got, ref)
        assert np.isfinite(got).all() and e <= TOL, f"seq_len {T}: {e}"


def test_attention_one_workspace_for_different_head_counts(gpu):
    """One workspace, sized for the largest head count, serves launches of different head counts, group sizes and lengths
    one after the other with no host synchronization between them: stream order alone keeps a launch's partial results
    apart from the next one's."""
    torch, iflow = gpu
    from oracle import attention as att
    nbytes = iflow.attn_decode_workspace_bytes(64)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    scale = 1.0 / np.sqrt(128.0)
    cases = [(64, 8, 2000), (32, 32, 900), (8, 4, 1500), (64, 8, 1999), (16, 4, 2048), (32, 32, 901)]
    pending = []
    for n, (n_heads, n_kv, T) in enumerate(cases):
        say(f"[case] attention, shared workspace, heads={n_heads} kv_heads={n_kv} seq_len={T}")
        q, k, v = make(n_heads, n_kv, 2048, synth.BASE_SEED + 1650 + n)
        out = torch.full((n_heads, 128), float("nan"), dtype=torch.float16, device="cuda")
        iflow.attn_decode(dev16(torch, q), dev16(torch, k), dev16(torch, v), n_heads, n_kv, 128, T, 2048, scale, out, ws, nbytes)
        pending.append((q, k, v, T, out))
    torch.cuda.synchronize()
    for q, k, v, T, out in pending:
        ref = att.gqa_decode(q.view(np.uint16), k.view(np.uint16), v.view(np.uint16), T, scale)
        got = out.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all() and rel(got, ref) <= TOL, f"heads {q.shape[0]}, seq_len {T}"


def test_attention_graph_replay(gpu):
    torch, iflow = gpu
    from oracle import attention as att
    n_heads, n_kv, max_seq, T = 32, 8, 2048, 1500
    say("[case] attention under HIP-graph replay")
    q, k, v = make(n_heads, n_kv, max_seq, synth.BASE_SEED + 1700)
    qd, kd, vd = dev16(torch, q), dev16(torch, k), dev16(torch, v)
    nbytes = iflow.attn_decode_workspace_bytes(n_heads)
    ws = torch.zeros((nbytes,), dtype=torch.uint8, device="cuda")
    out = torch.zeros((n_heads, 128), dtype=torch.float16, device="cuda")
    stream = torch.cuda.Stream()
    scale = 1.0 / np.sqrt(128.0)
    with torch.cuda.stream(stream):
        iflow.attn_decode(qd, kd, vd, n_heads, n_kv, 128, T, max_seq, scale, out, ws, nbytes, stream=stream.cuda_stream)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            iflow.attn_decode(qd, kd, vd, n_heads, n_kv, 128, T, max_seq, scale, out, ws, nbytes, stream=stream.cuda_stream)
    for rep in range(3):
        q2 = make(n_heads, n_kv, 1, synth.BASE_SEED + 1710 + rep)[0]
        qd.copy_(dev16(torch, q2))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        graph.replay()
        torch.cuda.synchronize()
        ref = att.gqa_decode(q2.view(np.uint16), k.view(np.uint16), v.view(np.uint16), T, scale)
        assert rel(out.cpu().numpy().astype(np.float64), ref) <= TOL
