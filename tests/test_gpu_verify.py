"""GPU parity of dk_verify_greedy against the oracle: token ids and accept counts are compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26289_amd import binding as dk
from paper_2605_26289_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _run(logits_host_f32: np.ndarray, dtype: str, tokens: np.ndarray, cu: np.ndarray, row_stride=None, want_argmax=True):
    rows, vocab = logits_host_f32.shape
    stride = row_stride or vocab
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    buf = torch.full((max(rows, 1), stride), float("nan"), dtype=tdt, device="cuda")  # padding must never win
    if rows:
        buf[:rows, :vocab] = torch.from_numpy(logits_host_f32).to("cuda", tdt)
    n = len(cu) - 1
    cu_d = torch.from_numpy(cu.astype(np.int32)).cuda()
    tok_d = torch.from_numpy(tokens.astype(np.int32)).cuda() if rows else torch.zeros(1, dtype=torch.int32, device="cuda")
    keep = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
    am = torch.full((max(rows, 1),), -7, dtype=torch.int32, device="cuda") if want_argmax else None
    code = dk.BF16 if dtype == "bf16" else dk.F32
    ws = torch.empty(dk.verify_workspace_bytes(rows, vocab, code), dtype=torch.uint8, device="cuda")
    dk.verify_greedy(n, rows, cu_d, buf, code, vocab, stride, tok_d, keep, nxt, ws, argmax_out=am)
    torch.cuda.synchronize()
    return keep.cpu().numpy()[:n], nxt.cpu().numpy()[:n], (am.cpu().numpy()[:rows] if am is not None else None)


def _case(seed, deltas, vocab, dtype, ties=False, stride=None, want_argmax=True, hit=0.6):
    rng = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(deltas)]).astype(np.int64)
    rows = int(cu[-1])
    x = wl.normal(rng, (rows, vocab), dtype)
    if ties:  # few distinct values: many exact ties, plus infinities and a NaN
        x = wl.round_to_bf16(np.round(x * 2) / 2)
        for _ in range(max(1, rows // 2)):
            x[rng.integers(rows), rng.integers(vocab)] = np.inf
        if rows > 2:
            x[1, :] = -np.inf
            x[2, rng.integers(vocab)] = np.nan
    ref_am = oracle.greedy_argmax(x)
    toks = rng.integers(0, vocab, size=rows)
    for b, d in enumerate(deltas):
        for s in range(max(0, d - 1)):
            if rng.random() < hit:
                toks[cu[b] + 1 + s] = ref_am[cu[b] + s]
    keep, nxt, am = _run(x, dtype, toks, cu, stride, want_argmax)
    rk, rn, ra = oracle.verify_batch(x, toks, cu)
    assert np.array_equal(keep, rk), (keep, rk)
    assert np.array_equal(nxt, rn)
    if want_argmax:
        assert np.array_equal(am, ra)
    return keep


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("vocab,stride", [(1, 8), (7, 8), (8, None), (1000, None), (4099, 4104), (16384, None),
                                          (16385, 16392), (40000, None)])
def test_argmax_and_accept_small_vocabularies(vocab, stride, dtype):
    _case(vocab, [9, 1, 0, 3, 9, 2], vocab, dtype, ties=False, stride=stride)
    _case(vocab + 1, [9, 1, 0, 3, 9, 2], vocab, dtype, ties=True, stride=stride)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_config5_shape_full_vocabulary(dtype):
    """64 slots x (1 + 8 drafts) rows over a 128 256-entry vocabulary (the size Sec. 3.4 quotes as 128k)."""
    keep = _case(5, [9] * 64, 128256, dtype, hit=0.85)
    assert keep.min() >= 1 and keep.max() == 9 and len(set(keep.tolist())) > 2


def test_all_right_all_wrong_and_plain_decode():
    assert _case(11, [12] * 5, 3000, "bf16", hit=1.0).tolist() == [12] * 5       # k = 11 as in the paper's example
    assert _case(12, [9] * 5, 3000, "bf16", hit=0.0).max() <= 2                   # random drafts almost never match
    assert _case(13, [1] * 7, 3000, "bf16").tolist() == [1] * 7                   # k = 0: plain decode steps
    _case(14, [0, 0, 5], 100, "f32", ties=True, want_argmax=False)                 # empty slots, no argmax output
    _case(15, [150, 70], 512, "bf16", ties=True)                                   # more rows than lanes per slot


def test_argument_errors():
    ws = torch.empty(dk.verify_workspace_bytes(4, 64, dk.BF16), dtype=torch.uint8, device="cuda")
    cu = torch.tensor([0, 4], dtype=torch.int32, device="cuda")
    lg = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    tk = torch.zeros(4, dtype=torch.int32, device="cuda")
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(dk.DeltaKVError) as e:
        dk.verify_greedy(1, 4, cu, lg, dk.BF16, 64, 60, tk, out, out, ws)  # stride < vocab
    assert e.value.name == "INVALID"
    with pytest.raises(dk.DeltaKVError) as e:
        dk.verify_greedy(1, 4, cu, lg, dk.BF16, 60, 62, tk, out, out, ws)  # rows not 16-byte multiples
    assert e.value.name == "UNSUPPORTED"
    with pytest.raises(dk.DeltaKVError) as e:
        dk.verify_greedy(1, 4, cu, lg, dk.BF16, 64, 64, tk, out, out, ws[:256])
    assert e.value.name == "WORKSPACE"
    with pytest.raises(dk.DeltaKVError) as e:
        dk.verify_greedy(1, 4, cu, lg, 5, 64, 64, tk, out, out, ws)
    assert e.value.name == "UNSUPPORTED"
    dk.verify_greedy(0, 0, None, None, dk.BF16, 64, 64, None, None, None, None)  # empty batch: nothing to do
