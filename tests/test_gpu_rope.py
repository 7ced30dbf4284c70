"""GPU parity: rotary position embedding + cache append (iflow_rope_append) against oracle/rope.py, through the C ABI.

Bar: the oracle rounds the exact fp64 rotation to fp16 once; the kernel computes the same rotation in fp64 with its own
sine and cosine and rounds once, so the two may differ by one fp16 step where the exact value sits within 1e-15 of a
rounding boundary - allowed for at most one value in a thousand; everything else bit-exact.  Rows of the caches other
than `position` must be untouched, the value row an exact copy.
"""
import sys

import numpy as np
import pytest

from paper_2401_08294_amd import synth

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2401_08294_amd import iflow
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    iflow.lib()
    return torch, iflow


def dev16(torch, a16):
    return torch.from_numpy(np.ascontiguousarray(a16).view(np.int16)).cuda()


def close_bits(got16, ref16):
    """fp16 bit patterns: equal, except at most 0.1 % of the values one step apart."""
    got16, ref16 = np.asarray(got16, np.uint16).ravel(), np.asarray(ref16, np.uint16).ravel()
    diff = got16 != ref16
    if not diff.any():
        return True
    g = got16[diff].view(np.float16).astype(np.float64)
    r = ref16[diff].view(np.float16).astype(np.float64)
    step = np.maximum(np.abs(r), 2.0 ** -14) * 2.0 ** -10
    return bool(np.all(np.abs(g - r) <= step) and diff.mean() <= 1e-3)


@pytest.mark.parametrize("n_heads,n_kv,position,max_seq", [(32, 32, 0, 8), (32, 32, 1, 8), (32, 8, 1000, 2048), (64, 8, 4095, 4096),
                                                          (8, 1, 123457, 131072), (2, 2, (1 << 20) - 1, 1 << 20)])
@pytest.mark.parametrize("mode", [0, 1])
def test_rope_append_against_the_definition(gpu, n_heads, n_kv, position, max_seq, mode):
    check_rope_append(gpu, n_heads, n_kv, position, max_seq, mode, 128)


def check_rope_append(gpu, n_heads, n_kv, position, max_seq, mode, d):
    torch, iflow = gpu
    from oracle import rope as R
    say(f"[case] rope_append heads={n_heads} kv_heads={n_kv} head_dim={d} position={position} max_seq={max_seq} pairing={mode}")
    rng = np.random.default_rng(synth.BASE_SEED + 1800 + position % 1000 + mode)
    base = 10000.0
    rows = min(max_seq, 6)                                      # the test's caches hold a window of rows around `position`
    q = rng.standard_normal((n_heads, d)).astype(np.float16)
    k = rng.standard_normal((n_kv, d)).astype(np.float16)
    v = rng.standard_normal((n_kv, d)).astype(np.float16)
    # device caches of the full size would be up to 2 x 256 MB here: fine on the device, but compare only a window on the host
    kc = torch.zeros((n_kv, max_seq, d), dtype=torch.float16, device="cuda")
    vc = torch.zeros((n_kv, max_seq, d), dtype=torch.float16, device="cuda")
    lo = max(0, min(position - 2, max_seq - rows))
    window_k = rng.standard_normal((n_kv, rows, d)).astype(np.float16)
    window_v = rng.standard_normal((n_kv, rows, d)).astype(np.float16)
    kc[:, lo:lo + rows] = torch.from_numpy(window_k).cuda()
    vc[:, lo:lo + rows] = torch.from_numpy(window_v).cuda()
    qd = dev16(torch, q.view(np.uint16))
    iflow.rope_append(qd, dev16(torch, k.view(np.uint16)), dev16(torch, v.view(np.uint16)), n_heads, n_kv, d, position, max_seq, base,
                      mode, kc, vc)
    torch.cuda.synchronize()
    kref, vref = window_k.view(np.uint16).copy(), window_v.view(np.uint16).copy()
    full_k = np.zeros((n_kv, rows, d), np.uint16); full_v = np.zeros((n_kv, rows, d), np.uint16)
    full_k[:], full_v[:] = kref, vref
    # the oracle works on the window, with the position relative to it
    qref = R.rope(q.view(np.uint16), position, base, mode)
    full_k[:, position - lo] = R.rope(k.view(np.uint16), position, base, mode)
    full_v[:, position - lo] = v.view(np.uint16)
    got_q = qd.cpu().numpy().view(np.uint16)
    got_k = kc[:, lo:lo + rows].cpu().numpy().view(np.uint16)
    got_v = vc[:, lo:lo + rows].cpu().numpy().view(np.uint16)
    assert close_bits(got_q, qref), "rotated queries differ"
    assert np.array_equal(got_v, full_v), "value rows differ"
    others = np.arange(rows) != position - lo
    assert np.array_equal(got_k[:, others], full_k[:, others]), "a key row other than `position` was touched"
    assert close_bits(got_k[:, position - lo], full_k[:, position - lo]), "rotated keys differ"
    # nothing outside the window was written either (the caches started as zeros)
    if lo > 0:
        assert not kc[:, :lo].any().item() and not vc[:, :lo].any().item()
    if lo + rows < max_seq:
        assert not kc[:, lo + rows:].any().item() and not vc[:, lo + rows:].any().item()


@pytest.mark.parametrize("d,n_heads,n_kv,position,max_seq", [(64, 128, 8, 1000, 2048), (64, 71, 1, 4095, 4096), (96, 12, 4, 77, 128),
                                                            (256, 8, 2, 30000, 32768), (16, 4, 4, 3, 8)])
@pytest.mark.parametrize("mode", [0, 1])
def test_rope_append_other_head_dimensions(gpu, d, n_heads, n_kv, position, max_seq, mode):
    """Head dimensions other than 128 (64: the paper's Falcon models)."""
    check_rope_append(gpu, n_heads, n_kv, position, max_seq, mode, d)


def test_decode_steps_with_rope_and_attention(gpu):
    """Five decode steps end to end: rope_append then attn_decode on the device, the same composition in the oracle."""
    torch, iflow = gpu
    from oracle import attention as att
    from oracle import rope as R
    n_heads, n_kv, max_seq, base, mode = 16, 4, 64, 10000.0, 1
    rng = np.random.default_rng(synth.BASE_SEED + 1900)
    kc = torch.zeros((n_kv, max_seq, 128), dtype=torch.float16, device="cuda")
    vc = torch.zeros((n_kv, max_seq, 128), dtype=torch.float16, device="cuda")
    okc = np.zeros((n_kv, max_seq, 128), np.uint16); ovc = np.zeros((n_kv, max_seq, 128), np.uint16)
    nbytes = iflow.attn_decode_workspace_bytes(n_heads)
    ws = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
    out = torch.empty((n_heads, 128), dtype=torch.float16, device="cuda")
    scale = 128 ** -0.5
    for pos in range(5):
        say(f"[case] decode step {pos}: rope_append + attn_decode")
        q = rng.standard_normal((n_heads, 128)).astype(np.float16)
        k = rng.standard_normal((n_kv, 128)).astype(np.float16)
        v = rng.standard_normal((n_kv, 128)).astype(np.float16)
        qd = dev16(torch, q.view(np.uint16))
        iflow.rope_append(qd, dev16(torch, k.view(np.uint16)), dev16(torch, v.view(np.uint16)), n_heads, n_kv, 128, pos, max_seq, base, mode, kc, vc)
        iflow.attn_decode(qd, kc, vc, n_heads, n_kv, 128, pos + 1, max_seq, scale, out, ws, nbytes)
        torch.cuda.synchronize()
        qr = R.rope_append(q.view(np.uint16), k.view(np.uint16), v.view(np.uint16), pos, base, mode, okc, ovc)
        ref = att.gqa_decode(qr, okc, ovc, pos + 1, scale)
        got = out.cpu().numpy().astype(np.float64)
        err = np.max(np.abs(got - ref) / np.maximum(np.abs(ref), np.sqrt(np.mean(ref ** 2))))
        assert np.isfinite(got).all() and err <= 2e-3, (pos, err)
