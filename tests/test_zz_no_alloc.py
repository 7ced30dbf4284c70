"""iflow_attn_decode_static - the entry point for callers that cannot allocate (its partial results live in an array inside
the library) - against iflow_attn_decode with a caller's workspace: the same kernels, so the outputs must be equal bit for
bit, and both must meet the oracle's definition within the product tolerance.  Two calls in a row on the shared array, the
second with a smaller input (fewer heads, fewer positions, fewer position ranges), then a third, larger one again."""
import numpy as np
import pytest

from paper_2401_08294_amd import synth
from test_gpu_attn import dev16, make, rel
from test_gpu_parity import TOL, gpu, say  # noqa: F401

pytestmark = pytest.mark.gpu


def both(torch, iflow, n_heads, n_kv, T, max_seq, seed):
    from oracle import attention as att
    q, k, v = make(n_heads, n_kv, max_seq, seed)
    scale = 1.0 / np.sqrt(128.0)
    qd, kd, vd = dev16(torch, q), dev16(torch, k), dev16(torch, v)
    nbytes = iflow.attn_decode_workspace_bytes(n_heads)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    want = torch.full((n_heads, 128), float("nan"), dtype=torch.float16, device="cuda")
    got = torch.full((n_heads, 128), float("nan"), dtype=torch.float16, device="cuda")
    iflow.attn_decode(qd, kd, vd, n_heads, n_kv, 128, T, max_seq, scale, want, ws, nbytes)
    iflow.attn_decode_static(qd, kd, vd, n_heads, n_kv, 128, T, max_seq, scale, got)
    torch.cuda.synchronize()
    a, b = want.cpu().numpy(), got.cpu().numpy()
    assert np.isfinite(b.astype(np.float64)).all()
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), "static-array call differs from the workspace call"
    ref = att.gqa_decode(q.view(np.uint16), k.view(np.uint16), v.view(np.uint16), T, scale)
    e = rel(b.astype(np.float64), ref)
    say(f"        heads={n_heads}/{n_kv} seq_len={T}: bit-equal to iflow_attn_decode, max rel err vs oracle {e:.3e}")
    assert e <= TOL


def test_static_array_call_twice_in_a_row_second_smaller(gpu):
    torch, iflow = gpu
    say("[case] iflow_attn_decode_static: 64/8 heads x 3000 positions, then 8/8 heads x 100 positions, then 32/32 x 2049")
    both(torch, iflow, 64, 8, 3000, 3072, synth.BASE_SEED + 1700)
    both(torch, iflow, 8, 8, 100, 128, synth.BASE_SEED + 1701)        # smaller: one position range per head, no merge launch
    both(torch, iflow, 32, 32, 2049, 2112, synth.BASE_SEED + 1702)


def test_static_array_call_rejects_more_heads_than_the_array_holds(gpu):
    torch, iflow = gpu
    say("[case] iflow_attn_decode_static: 256 heads are refused (the array holds 128)")
    q = torch.zeros((256, 128), dtype=torch.float16, device="cuda")
    k = torch.zeros((32, 64, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros((256, 128), dtype=torch.float16, device="cuda")
    with pytest.raises(iflow.IflowError) as ei:
        iflow.attn_decode_static(q, k, k, 256, 32, 128, 64, 64, 0.1, out)
    assert ei.value.status == iflow.ERR_SIZE
    assert iflow.ATTN_STATIC_MAX_HEADS == 128
