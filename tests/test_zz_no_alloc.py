"""ecco_kv_attend_gqa_noalloc (the entry point for callers that cannot allocate) against ecco_kv_attend_gqa, through
the C ABI: same kernels, so the outputs must be the same bits.  Two calls in a row share the library's static device
array, the second with a smaller input; then the limit and the argument errors.  Runs last in the suite and must also
pass alone in a fresh process.
"""
from __future__ import annotations

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2505_06901_amd as E  # noqa: E402
from paper_2505_06901_amd import workloads as W  # noqa: E402


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def _t16(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.float16)).to(dev)


def test_noalloc_equals_workspace_call_twice_in_a_row(dev, oracle):
    B, Hkv, grp, T = 3, 2, 4, 1500
    Hq = Hkv * grp
    k, v = W.kv_cache(B, Hkv, T, 128, seed=23)
    mk = E.ecco_model_to_device(E.ecco_fit_patterns(k[:, :, :256], 16, 12, 5), 0)
    mv = E.ecco_model_to_device(E.ecco_fit_patterns(v[:, :, :256], 16, 12, 6), 0)
    kb, km = E.ecco_encode(mk, _t16(k, dev)); vb, vm = E.ecco_encode(mv, _t16(v, dev))
    kb, vb = kb.view(B, Hkv, T, 64), vb.view(B, Hkv, T, 64)
    km, vm = km.view(B, Hkv, T), vm.view(B, Hkv, T)
    q = W.activation(B * Hq, 128, 123).reshape(B, Hq, 128)
    qd = _t16(q, dev)
    # first call: 5 splits over the long sequences; second call right behind it on the same stream: a smaller input
    # (fewer sequences, heads, tokens and splits), which reuses the front of the same array
    seq1 = torch.tensor([T, 0, 333], dtype=torch.int32, device=dev)
    want1 = E.ecco_kv_attend_gqa(mk, mv, qd, kb, km, vb, vm, seq1, B, Hq, Hkv, T, n_splits=5)
    B2, T2 = 2, 700
    kb2, km2, vb2, vm2 = (a[:B2, :, :T2].contiguous() for a in (kb, km, vb, vm))
    q2 = qd[:B2].contiguous()
    seq2 = torch.tensor([T2, 100], dtype=torch.int32, device=dev)
    want2 = E.ecco_kv_attend_gqa(mk, mv, q2, kb2, km2, vb2, vm2, seq2, B2, Hq, Hkv, T2, n_splits=2)
    torch.cuda.synchronize()
    out1 = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=dev)
    out2 = torch.full((B2, Hq, 128), float("nan"), dtype=torch.float32, device=dev)
    before = torch.cuda.memory_allocated()
    E.ecco_kv_attend_gqa_noalloc(mk, mv, qd, kb, km, vb, vm, seq1, B, Hq, Hkv, T, 5, out1)
    E.ecco_kv_attend_gqa_noalloc(mk, mv, q2, kb2, km2, vb2, vm2, seq2, B2, Hq, Hkv, T2, 2, out2)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out1, want1)
    assert torch.equal(out2, want2)
    # and against the oracle, to the bar of the other attention tests (the oracle encodes for itself)
    ok, okm = oracle.encode(mk.centroids, mk.code_lens, k.view(np.uint16))
    ov, ovm = oracle.encode(mv.centroids, mv.code_lens, v.view(np.uint16))
    ref = oracle.kv_attend_gqa(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16), ok, okm, ov, ovm,
                               seq1.cpu().numpy(), B, Hq, Hkv, T)
    got = out1.cpu().numpy()
    assert not got[1].any()
    for b in (0, 2):
        for h in range(Hq):
            assert np.linalg.norm(got[b, h] - ref[b, h]) <= 1e-3 * np.linalg.norm(ref[b, h]), (b, h)
    # a third call, larger again, and one without splits (which uses no scratch at all)
    out3 = torch.empty_like(out1)
    E.ecco_kv_attend_gqa_noalloc(mk, mv, qd, kb, km, vb, vm, seq1, B, Hq, Hkv, T, 5, out3)
    assert torch.equal(out3, want1)
    E.ecco_kv_attend_gqa_noalloc(mk, mv, qd, kb, km, vb, vm, seq1, B, Hq, Hkv, T, 1, out3)
    assert torch.equal(out3, E.ecco_kv_attend_gqa(mk, mv, qd, kb, km, vb, vm, seq1, B, Hq, Hkv, T, n_splits=1))


def test_noalloc_limit_and_errors(dev):
    B, Hkv, T = 1, 1, 64
    k, v = W.kv_cache(B, Hkv, T, 128, seed=29)
    m = E.ecco_model_to_device(E.ecco_fit_patterns(k, 4, 12, 1), 0)
    kb, km = E.ecco_encode(m, _t16(k, dev)); vb, vm = E.ecco_encode(m, _t16(v, dev))
    seq = torch.tensor([T], dtype=torch.int32, device=dev)
    # B * Hq * n_splits * 520 bytes must fit 8 MiB: 16 heads x 256 splits x 4 sequences = 16384 partial results do not
    Hq = 16
    big_B = 4
    q = torch.zeros((big_B, Hq, 128), dtype=torch.float16, device=dev)
    out = torch.zeros((big_B, Hq, 128), dtype=torch.float32, device=dev)
    assert big_B * Hq * 256 * 520 > E.GQA_SCRATCH_BYTES
    with pytest.raises(E.EccoError) as e:
        E.ecco_kv_attend_gqa_noalloc(m, m, q, kb, km, vb, vm, seq, big_B, Hq, 1, T, 256, out)
    assert e.value.status == -2
    assert not out.any()  # nothing was launched
    # the largest size that fits is accepted (B = 1 here: one sequence, 16 heads, 256 splits of a 64-token cache)
    assert 1 * Hq * 256 * 520 <= E.GQA_SCRATCH_BYTES
    got = E.ecco_kv_attend_gqa_noalloc(m, m, q[:1].contiguous(), kb, km, vb, vm, seq, 1, Hq, 1, T, 256, out[:1].contiguous())
    want = E.ecco_kv_attend_gqa(m, m, q[:1].contiguous(), kb, km, vb, vm, seq, 1, Hq, 1, T, n_splits=256)
    assert torch.equal(got, want)
    with pytest.raises(E.EccoError) as e:
        E.ecco_kv_attend_gqa_noalloc(m, m, q, kb, km, vb, vm, seq, 1, 5, 2, T, 2, out)
    assert e.value.status == -2
    with pytest.raises(E.EccoError) as e:
        E.ecco_kv_attend_gqa_noalloc(m, m, None, kb, km, vb, vm, seq, 1, Hq, 1, T, 2, out)
    assert e.value.status == -1
