"""Parity of the HIP path against the CPU oracle, through the C ABI, on one MI355X.

Bars: encoded blocks / meta words and decoded indices bit-exact; dequantised FP16 bit-exact;
GEMV and attention outputs within rel-L2 1e-3 of the double-precision oracle.
"""
from __future__ import annotations

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2505_06901_amd as E  # noqa: E402
from paper_2505_06901_amd import workloads as W  # noqa: E402
from helpers import pack_raw  # noqa: E402

REL_L2 = 1e-3


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def t16(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.float16)).to(dev)


def tu8(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).to(dev)


def ti32(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).to(dev)


def rel_l2(got, want):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    return np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)


def assert_gemv_close(oracle, m, ob, om, rows, cols, x, y, tag=None):
    """y (batch x rows, from the HIP path) against the double-precision oracle on the oracle's own blocks: rel-L2 over
    the whole output and per batch row, and element by element |y - ref| <= 1e-3 * sum_c |w_rc| |x_c| (a norm alone
    does not see one bad row among thousands)."""
    want = oracle.gemv(m.centroids, m.code_lens, ob, om, rows, cols, x.view(np.uint16))
    assert y.shape == want.shape, tag
    assert rel_l2(y, want) <= REL_L2, tag
    for b in range(want.shape[0]):
        assert rel_l2(y[b], want[b]) <= REL_L2, (tag, b)
    dec = oracle.decode(m.centroids, m.code_lens, ob, om).view(np.float16).reshape(rows, cols)
    bound = np.abs(x.astype(np.float32)) @ np.abs(dec.astype(np.float32)).T
    err = np.abs(y.astype(np.float64) - want)
    worst = np.unravel_index(np.argmax(err - REL_L2 * bound), err.shape)
    assert (err <= REL_L2 * bound.astype(np.float64)).all(), (tag, worst, err[worst], bound[worst])
    return want


def assert_attn_close(oracle, mv, ovb, ovm, seq, B, Hq, Hkv, T, out, want, tag=None):
    """Attention output against the double-precision oracle: rel-L2 over the whole output and per (sequence, head), and
    element by element |o - ref| <= 1e-3 * max_{t < seq_len} |V_t,d| (the output is a convex mix of those rows)."""
    assert out.shape == want.shape, tag
    assert np.isfinite(out).all(), tag
    assert rel_l2(out, want) <= REL_L2, tag
    vdec = np.abs(oracle.decode(mv.centroids, mv.code_lens, ovb, ovm).view(np.float16).astype(np.float64)).reshape(B, Hkv, T, 128)
    for b in range(B):
        n = int(min(max(seq[b], 0), T))
        for h in range(Hq):
            if n == 0:
                assert not out[b, h].any(), (tag, b, h)
                continue
            assert rel_l2(out[b, h], want[b, h]) <= REL_L2, (tag, b, h)
            bound = vdec[b, h // (Hq // Hkv), :n].max(axis=0)
            err = np.abs(out[b, h].astype(np.float64) - want[b, h])
            assert (err <= REL_L2 * bound).all(), (tag, b, h, int(np.argmax(err - REL_L2 * bound)))


def enc_both(dev, oracle, m, x):
    """Encodes x (any shape, groups of 128 along the last axis) on the GPU and with the oracle, requires the same
    bytes, and returns (blocks, meta) as device tensors and as the oracle's arrays -- which are what the oracle's
    consumers are then given: no oracle input comes from the HIP path."""
    ob, om = oracle.encode(m.centroids, m.code_lens, np.ascontiguousarray(x).reshape(-1, 128).view(np.uint16))
    blocks, meta = E.ecco_encode(m, t16(x, dev))
    assert np.array_equal(np_meta(meta), om) and np.array_equal(np_blocks(blocks), ob)
    return blocks, meta, ob, om


def np_blocks(t):
    return t.cpu().numpy().reshape(-1, 64)


def np_meta(t):
    return t.cpu().numpy().view(np.uint32).reshape(-1)


# ---------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def tiny(dev, oracle):
    w = W.config_weight("tiny")
    m = E.ecco_model_to_device(E.ecco_fit_patterns(w, 16, 12, 0), 0)
    ob, om = oracle.encode(m.centroids, m.code_lens, w.view(np.uint16))
    return dict(w=w, m=m, ob=ob, om=om)


def test_tiny_encode_bit_exact(dev, oracle, tiny):
    blocks, meta = E.ecco_encode(tiny["m"], t16(tiny["w"], dev))
    torch.cuda.synchronize()
    assert np.array_equal(np_meta(meta), tiny["om"])
    assert np.array_equal(np_blocks(blocks), tiny["ob"])
    # determinism: a second run gives the same bytes
    b2, m2 = E.ecco_encode(tiny["m"], t16(tiny["w"], dev))
    assert torch.equal(b2, blocks) and torch.equal(m2, meta)


def test_tiny_decode_bit_exact(dev, oracle, tiny):
    m = tiny["m"]
    blocks, meta = tu8(tiny["ob"], dev), ti32(tiny["om"], dev)
    idx = E.ecco_decode_indices(m, blocks, meta).cpu().numpy()
    oidx, _ = oracle.decode_indices(m.code_lens, m.S, tiny["ob"], tiny["om"])
    assert np.array_equal(idx, oidx)
    dec = E.ecco_decode(m, blocks, meta).cpu().numpy().view(np.uint16)
    assert np.array_equal(dec, oracle.decode(m.centroids, m.code_lens, tiny["ob"], tiny["om"]))


@pytest.mark.parametrize("batch", [1, 2, 5, 8, 16])
def test_tiny_gemv(dev, oracle, tiny, batch):
    m = tiny["m"]
    x = W.activation(batch, 1024, 100)
    y = E.ecco_decode_gemv(m, tu8(tiny["ob"], dev), ti32(tiny["om"], dev), 64, 1024, t16(x, dev)).cpu().numpy()
    assert_gemv_close(oracle, m, tiny["ob"], tiny["om"], 64, 1024, x, y)


def test_gemv_unit_vector_ties_to_decode(dev, oracle, tiny):
    m = tiny["m"]
    dec = oracle.decode(m.centroids, m.code_lens, tiny["ob"], tiny["om"]).view(np.float16).reshape(64, 1024)
    for j in (0, 127, 128, 640, 1023):
        x = np.zeros((1, 1024), np.float16); x[0, j] = 1
        y = E.ecco_decode_gemv(m, tu8(tiny["ob"], dev), ti32(tiny["om"], dev), 64, 1024, t16(x, dev)).cpu().numpy()
        assert np.allclose(y[0], dec[:, j].astype(np.float64), rtol=2e-3, atol=1e-7)


# ---------------------------------------------------------------------------------------------------
def _skewed_model(oracle, S, seed):
    """Hand-built model whose codebooks reach 12 bits (exercises codes longer than the short table)."""
    rng = np.random.default_rng(seed)
    cent = np.sort(rng.uniform(-1, 1, (S, 16)), axis=1)
    cent[:, 0], cent[:, 15] = -1, 1
    lens = np.zeros((S, 16), np.uint8)
    probs = np.zeros((S, 16))
    for p in range(S):
        base = 2.2 + 1.2 * rng.random()
        counts = np.array([int(base ** k) + 1 for k in range(16)], np.uint64)[rng.permutation(16)]
        lens[p] = oracle.limited_lengths(counts, 12)
        probs[p] = counts / counts.sum()
    return cent.astype(np.float16), lens, probs


def _skewed_data(cent, probs, n_groups, seed):
    rng = np.random.default_rng(seed)
    S = cent.shape[0]
    p = rng.integers(0, S, n_groups)
    x = np.zeros((n_groups, 128), np.float64)
    for g in range(n_groups):
        idx = rng.choice(16, 128, p=probs[p[g]])
        idx[rng.integers(128)] = 15  # the +1 centroid is present, so the scale is what we say
        x[g] = cent[p[g]].astype(np.float64)[idx] * (0.01 + rng.random()) * (1 + 0.002 * rng.standard_normal(128))
    return x.astype(np.float16)


def test_long_codes_all_paths(dev, oracle):
    S = 7
    cent, lens, probs = _skewed_model(oracle, S, 1)
    assert lens.max() == 12
    m = E.ecco_model_to_device(E.ecco_model_create(cent, lens), 0)
    n = 256 * 3 + 77  # several workgroups and a ragged tail
    x = _skewed_data(cent, probs, n, 2)
    ob, om = oracle.encode(cent.view(np.uint16), lens, x.view(np.uint16))
    oidx, used = oracle.decode_indices(lens, S, ob, om)
    long_used = (lens[(om >> 16) & 63][np.arange(n)[:, None], oidx] > 8) & (((om >> 22) & 1) == 0)[:, None]
    assert long_used.sum() > 200  # codes beyond the 8-bit table really occur in Huffman-mode blocks
    blocks, meta = E.ecco_encode(m, t16(x, dev))
    assert np.array_equal(np_meta(meta), om) and np.array_equal(np_blocks(blocks), ob)
    assert np.array_equal(E.ecco_decode_indices(m, blocks, meta).cpu().numpy(), oidx)
    assert np.array_equal(E.ecco_decode(m, blocks, meta).cpu().numpy().view(np.uint16),
                          oracle.decode(cent.view(np.uint16), lens, ob, om))
    # gemv over the same blocks viewed as a 7-column-group matrix (ragged: 121 rows)
    rows, cols = n // 7, 7 * 128
    xb = W.activation(3, cols, 9)
    y = E.ecco_decode_gemv(m, blocks[: rows * 7], meta[: rows * 7], rows, cols, t16(xb, dev)).cpu().numpy()
    assert_gemv_close(oracle, m, ob[: rows * 7], om[: rows * 7], rows, cols, xb, y)


def test_long_codes_in_attention(dev, oracle):
    """Models whose codes reach 12 bits, for K, for V and for both: the long-code variants of both attention kernels."""
    B, H, T = 2, 2, 150
    short = _kv_setup(dev, oracle, B, H, T, 8)
    k, v = short[0], short[1]
    cent, lens, probs = _skewed_model(oracle, 5, 3)
    long_m = E.ecco_model_to_device(E.ecco_model_create(cent, lens), 0)
    kl = _skewed_data(cent, probs, B * H * T, 4).reshape(B, H, T, 128)
    vl = _skewed_data(cent, probs, B * H * T, 5).reshape(B, H, T, 128)
    q = W.activation(B * H * 2, 128, 107).reshape(B, 2 * H, 128)
    seq = np.array([T, 77], np.int32)
    for mk, mv, kk, vv in [(long_m, short[3], kl, v), (short[2], long_m, k, vl), (long_m, long_m, kl, vl)]:
        kb, km, okb, okm = enc_both(dev, oracle, mk, kk); vb, vm, ovb, ovm = enc_both(dev, oracle, mv, vv)
        args = (okb, okm, ovb, ovm, seq)
        want = oracle.kv_attend(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, np.ascontiguousarray(q[:, :H]).view(np.uint16), *args, B, H, T)
        out = E.ecco_kv_attend(mk, mv, t16(q[:, :H], dev), kb, km, vb, vm, ti32(seq, dev), B, H, T).cpu().numpy()
        assert_attn_close(oracle, mv, ovb, ovm, seq, B, H, H, T, out, want)
        want = oracle.kv_attend_gqa(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16), *args, B, 2 * H, H, T)
        out = E.ecco_kv_attend_gqa(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, 2 * H, H, T, n_splits=2).cpu().numpy()
        assert_attn_close(oracle, mv, ovb, ovm, seq, B, 2 * H, H, T, out, want)


def test_long_code_attention_repeatable(dev, oracle):
    """Both attention kernels with long codes in K and in V, over many units per wavefront: right against the oracle
    and the same bits on every launch."""
    B, H, T = 2, 2, 1500
    cent, lens, probs = _skewed_model(oracle, 5, 3)
    m = E.ecco_model_to_device(E.ecco_model_create(cent, lens), 0)
    kl = _skewed_data(cent, probs, B * H * T, 6).reshape(B, H, T, 128)
    vl = _skewed_data(cent, probs, B * H * T, 7).reshape(B, H, T, 128)
    q = W.activation(B * H * 2, 128, 109).reshape(B, 2 * H, 128)
    seq = np.array([T, 1111], np.int32)
    kb, km, okb, okm = enc_both(dev, oracle, m, kl); vb, vm, ovb, ovm = enc_both(dev, oracle, m, vl)
    args = (okb, okm, ovb, ovm, seq)
    want = oracle.kv_attend(m.centroids, m.code_lens, m.centroids, m.code_lens, np.ascontiguousarray(q[:, :H]).view(np.uint16), *args, B, H, T)
    qd, sd = t16(q[:, :H], dev), ti32(seq, dev)
    first = E.ecco_kv_attend(m, m, qd, kb, km, vb, vm, sd, B, H, T)
    assert_attn_close(oracle, m, ovb, ovm, seq, B, H, H, T, first.cpu().numpy(), want)
    for _ in range(15):
        assert torch.equal(first, E.ecco_kv_attend(m, m, qd, kb, km, vb, vm, sd, B, H, T))
    want = oracle.kv_attend_gqa(m.centroids, m.code_lens, m.centroids, m.code_lens, q.view(np.uint16), *args, B, 2 * H, H, T)
    qd = t16(q, dev)
    for n_splits in (1, 3):
        first = E.ecco_kv_attend_gqa(m, m, qd, kb, km, vb, vm, sd, B, 2 * H, H, T, n_splits=n_splits)
        assert_attn_close(oracle, m, ovb, ovm, seq, B, 2 * H, H, T, first.cpu().numpy(), want, n_splits)
        for _ in range(15):
            assert torch.equal(first, E.ecco_kv_attend_gqa(m, m, qd, kb, km, vb, vm, sd, B, 2 * H, H, T, n_splits=n_splits)), n_splits


def test_corrupt_blocks_decode_like_oracle(dev, oracle):
    S = 5
    cent, lens, _ = _skewed_model(oracle, S, 3)
    m = E.ecco_model_to_device(E.ecco_model_create(cent, lens), 0)
    rng = np.random.default_rng(4)
    n = 1000
    blocks = rng.integers(0, 256, (n, 64), dtype=np.uint8)
    blocks[::7] = 0xFF
    blocks[1::7] = 0
    meta = rng.integers(0, 2**32, n, dtype=np.uint64).astype(np.uint32) & np.uint32(0xFFFFBFFF)  # finite scales
    oidx, _ = oracle.decode_indices(lens, S, blocks, meta)
    idx = E.ecco_decode_indices(m, tu8(blocks, dev), ti32(meta, dev)).cpu().numpy()
    assert np.array_equal(idx, oidx)
    dec = E.ecco_decode(m, tu8(blocks, dev), ti32(meta, dev)).cpu().numpy().view(np.uint16)
    assert np.array_equal(dec, oracle.decode(cent.view(np.uint16), lens, blocks, meta))


def test_dequant_every_scale(dev, oracle):
    """All finite positive scales x 16 centroids through raw-mode blocks: FP16 bit-exact (subnormals kept)."""
    cent = np.array([[-1.0, -0.75, -0.52, -0.33, -0.2, -0.1, -0.031, -0.0007, 0.0, 0.011, 0.09, 0.21, 0.37, 0.5, 0.83, 1.0]],
                    np.float16)
    lens = np.full((1, 16), 4, np.uint8)
    m = E.ecco_model_to_device(E.ecco_model_create(cent, lens), 0)
    scales = np.arange(0, 0x7C00, dtype=np.uint32)
    nib = np.arange(128) % 16
    blocks = np.tile(pack_raw(nib), (scales.size, 1))
    meta = (scales | (1 << 22)).astype(np.uint32)
    dec = E.ecco_decode(m, tu8(blocks, dev), ti32(meta, dev)).cpu().numpy().view(np.uint16)
    assert np.array_equal(dec, oracle.decode(cent.view(np.uint16), lens, blocks, meta))


def test_edge_cases(dev, oracle, tiny):
    m = tiny["m"]
    # empty input: no-ops
    e16 = torch.empty((0, 128), dtype=torch.float16, device=dev)
    b, mt = E.ecco_encode(m, e16)
    assert b.numel() == 0 and mt.numel() == 0
    assert E.ecco_decode(m, b, mt).numel() == 0
    # all-zero groups, a lone outlier, the largest finite FP16 values, subnormals
    x = np.zeros((6, 128), np.float16)
    x[1, 5] = 3.0
    x[2] = 65504.0; x[2, ::2] = -65504.0
    x[3] = np.float16(6e-8); x[3, 7] = np.float16(-1.2e-7)
    x[4] = np.linspace(-1, 1, 128)
    x[5, 100] = -0.0
    ob, om = oracle.encode(m.centroids, m.code_lens, x.view(np.uint16))
    blocks, meta = E.ecco_encode(m, t16(x, dev))
    assert np.array_equal(np_meta(meta), om) and np.array_equal(np_blocks(blocks), ob)
    dec = E.ecco_decode(m, blocks, meta).cpu().numpy().view(np.uint16)
    assert np.array_equal(dec, oracle.decode(m.centroids, m.code_lens, ob, om))
    # argument errors come back as statuses
    with pytest.raises(E.EccoError) as e:
        E.ecco_decode_gemv(m, blocks, meta, 6, 100, torch.zeros((1, 100), dtype=torch.float16, device=dev))
    assert e.value.status == -2
    with pytest.raises(E.EccoError) as e:
        E.ecco_decode_gemv(m, blocks, meta, 6, 128, torch.zeros((17, 128), dtype=torch.float16, device=dev))
    assert e.value.status == -2
    mis = torch.empty(6 * 64 + 64, dtype=torch.uint8, device=dev)[16:16 + 6 * 64]
    with pytest.raises(E.EccoError) as e:
        E.ecco_decode(m, mis, meta)
    assert e.value.status == -3


def test_ragged_matrix_shapes(dev, oracle, tiny):
    # rows that do not fill a 16-row block or a workgroup's band, odd numbers of column groups (a unit of the batch
    # kernel then has one column group only), a single group, every batch size class; decode on ragged group counts
    m = tiny["m"]
    for rows, gpr, seed in [(1, 1, 21), (5, 1, 22), (17, 3, 23), (33, 5, 24), (300, 33, 25), (16, 64, 26)]:
        cols = gpr * 128
        w = W.weight_matrix(rows, cols, 0.02, 0.001, 10.0, seed)
        ob, om = oracle.encode(m.centroids, m.code_lens, w.reshape(-1, 128).view(np.uint16))
        blocks, meta = E.ecco_encode(m, t16(w, dev))
        assert np.array_equal(np_blocks(blocks), ob) and np.array_equal(np_meta(meta), om)
        assert np.array_equal(E.ecco_decode(m, blocks, meta).cpu().numpy().view(np.uint16),
                              oracle.decode(m.centroids, m.code_lens, ob, om))
        oidx, _ = oracle.decode_indices(m.code_lens, m.S, ob, om)
        assert np.array_equal(E.ecco_decode_indices(m, blocks, meta).cpu().numpy(), oidx)
        for batch in (1, 3, 16):
            x = W.activation(batch, cols, seed + 100)
            y = E.ecco_decode_gemv(m, blocks, meta, rows, cols, t16(x, dev)).cpu().numpy()
            assert_gemv_close(oracle, m, ob, om, rows, cols, x, y, (rows, gpr, batch))


@pytest.mark.parametrize("S", [1, 3])
def test_smallest_models(dev, oracle, S):
    """One pattern (nothing to choose) and three (fewer table items than any workgroup has threads, not a power of
    two): every entry point of the two-chain format against the oracle."""
    w = W.weight_matrix(48, 640, 0.02, 0.001, 10.0, 41)
    m = E.ecco_model_to_device(E.ecco_fit_patterns(w, S, 12, 7), 0)
    assert m.S == S
    ob, om = oracle.encode(m.centroids, m.code_lens, w.reshape(-1, 128).view(np.uint16))
    blocks, meta = E.ecco_encode(m, t16(w, dev))
    assert np.array_equal(np_blocks(blocks), ob) and np.array_equal(np_meta(meta), om)
    assert ((om >> 16) & 0x3F).max() < S
    assert np.array_equal(E.ecco_decode(m, blocks, meta).cpu().numpy().view(np.uint16), oracle.decode(m.centroids, m.code_lens, ob, om))
    sb, sm = E.ecco_encode_minmax(m, t16(w, dev))
    wb, wm = oracle.encode_minmax(m.centroids, m.code_lens, w.reshape(-1, 128).view(np.uint16))
    assert np.array_equal(np_blocks(sb), wb) and np.array_equal(np_meta(sm), wm)
    for batch in (1, 8):
        x = W.activation(batch, 640, 141 + batch)
        y = E.ecco_decode_gemv(m, blocks, meta, 48, 640, t16(x, dev)).cpu().numpy()
        assert_gemv_close(oracle, m, ob, om, 48, 640, x, y, batch)
    # the same model for K and V: append two tokens to an empty cache, then attend (plain and grouped, two splits)
    B, H, T = 2, 2, 40
    k, v = W.kv_cache(B, H, T, 128, seed=43)
    kb, km, okb, okm = enc_both(dev, oracle, m, k); vb, vm, ovb, ovm = enc_both(dev, oracle, m, v)
    q = W.activation(B * H * 2, 128, 143).reshape(B, 2 * H, 128)
    seq = np.array([T, 17], np.int32)
    args = (okb, okm, ovb, ovm, seq)
    want = oracle.kv_attend(m.centroids, m.code_lens, m.centroids, m.code_lens, np.ascontiguousarray(q[:, :H]).view(np.uint16), *args, B, H, T)
    out = E.ecco_kv_attend(m, m, t16(q[:, :H], dev), kb, km, vb, vm, ti32(seq, dev), B, H, T).cpu().numpy()
    assert_attn_close(oracle, m, ovb, ovm, seq, B, H, H, T, out, want)
    want = oracle.kv_attend_gqa(m.centroids, m.code_lens, m.centroids, m.code_lens, q.view(np.uint16), *args, B, 2 * H, H, T)
    out = E.ecco_kv_attend_gqa(m, m, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, 2 * H, H, T, n_splits=2).cpu().numpy()
    assert_attn_close(oracle, m, ovb, ovm, seq, B, 2 * H, H, T, out, want)


def test_widest_matrix(dev, oracle, tiny):
    """cols = 65536, the documented maximum: 512 column groups per row, 16 column tiles per band in the batch-1 kernel,
    256 units per 16-row block in the batched one; and one column group more is refused."""
    m = tiny["m"]
    rows, cols = 37, 65536
    w = W.weight_matrix(rows, cols, 0.02, 0.001, 10.0, 31)
    ob, om = oracle.encode(m.centroids, m.code_lens, w.reshape(-1, 128).view(np.uint16))
    blocks, meta = E.ecco_encode(m, t16(w, dev))
    assert np.array_equal(np_blocks(blocks), ob) and np.array_equal(np_meta(meta), om)
    for batch in (1, 4, 16):
        x = W.activation(batch, cols, 131 + batch)
        y = E.ecco_decode_gemv(m, blocks, meta, rows, cols, t16(x, dev)).cpu().numpy()
        assert_gemv_close(oracle, m, ob, om, rows, cols, x, y, batch)
    with pytest.raises(E.EccoError) as e:
        E.ecco_decode_gemv(m, blocks, meta, 1, cols + 128, t16(np.zeros((1, cols + 128), np.float16), dev))
    assert e.value.status == -2


# ---------------------------------------------------------------------------------------------------
def _kv_setup(dev, oracle, B, H, T, S):
    k, v = W.kv_cache(B, H, T, 128, seed=3)
    mk = E.ecco_model_to_device(E.ecco_fit_patterns(k[:, :, : max(8, T // 8)], S, 12, 3), 0)
    mv = E.ecco_model_to_device(E.ecco_fit_patterns(v[:, :, : max(8, T // 8)], S, 12, 3), 0)
    return k, v, mk, mv


def test_kv_append_matches_oracle(dev, oracle):
    B, H, T = 3, 5, 9
    k, v, mk, mv = _kv_setup(dev, oracle, B, H, T, 8)
    kb = torch.zeros((B, H, T, 64), dtype=torch.uint8, device=dev); km = torch.zeros((B, H, T), dtype=torch.int32, device=dev)
    vb = torch.zeros_like(kb); vm = torch.zeros_like(km)
    okb = np.zeros((B, H, T, 64), np.uint8); okm = np.zeros((B, H, T), np.uint32)
    ovb = np.zeros_like(okb); ovm = np.zeros_like(okm)
    seq = np.array([0, 4, T], np.int32)  # the last sequence is full: nothing may be written
    for step in range(5):
        cur = np.minimum(seq + step, T).astype(np.int32)
        tok = np.minimum(cur, T - 1)
        kn = np.stack([k[b, :, tok[b]] for b in range(B)]); vn = np.stack([v[b, :, tok[b]] for b in range(B)])
        E.ecco_kv_append(mk, mv, t16(kn, dev), t16(vn, dev), kb, km, vb, vm, ti32(cur, dev), B, H, T)
        oracle.kv_append(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, kn.view(np.uint16), vn.view(np.uint16),
                         okb, okm, ovb, ovm, cur, B, H, T)
    torch.cuda.synchronize()
    assert np.array_equal(kb.cpu().numpy(), okb) and np.array_equal(km.cpu().numpy().view(np.uint32), okm)
    assert np.array_equal(vb.cpu().numpy(), ovb) and np.array_equal(vm.cpu().numpy().view(np.uint32), ovm)
    assert okm[2].sum() == 0 and okm[0, :, :5].all()


def test_minmax_selector_matches_oracle(dev, oracle, tiny):
    """Min/max pattern selector: blocks and meta words bit-exact against the oracle, bulk and append, S = 16 and 64."""
    # bulk, weights (S = 16) on a ragged group count; K cache with S = 64 (one lane per pattern, all lanes used)
    m = tiny["m"]
    w = tiny["w"].reshape(-1, 128)[: 4 * 61 + 3]
    ob, om = oracle.encode_minmax(m.centroids, m.code_lens, w.view(np.uint16))
    blocks, meta = E.ecco_encode_minmax(m, t16(w, dev))
    assert np.array_equal(np_meta(meta), om) and np.array_equal(np_blocks(blocks), ob)
    assert not np.array_equal(om, tiny["om"][: om.size])  # the two selectors do differ on this input
    assert np.array_equal(E.ecco_decode(m, blocks, meta).cpu().numpy().view(np.uint16),
                          oracle.decode(m.centroids, m.code_lens, ob, om))
    k, v = W.kv_cache(2, 4, 160, 128, seed=3)
    m64 = E.ecco_model_to_device(E.ecco_fit_patterns(k[:, :, :96], 64, 12, 3), 0)
    x = k.reshape(-1, 128).copy()
    x[7] = 0                                   # all-zero group: scale 0, every fitness 0, pattern 0
    x[8] = np.float16(0.5)                     # constant group: min = max = absmax
    x[9] = -np.abs(x[9])                       # all negative
    ob, om = oracle.encode_minmax(m64.centroids, m64.code_lens, x.view(np.uint16))
    blocks, meta = E.ecco_encode_minmax(m64, t16(x, dev))
    assert np.array_equal(np_meta(meta), om) and np.array_equal(np_blocks(blocks), ob)
    assert (om[7] & 0x3FFFFF) == 0  # scale 0 and pattern 0 (the mode bit depends on the code of index 0)
    # append: five steps, a full sequence writes nothing; B*H not a multiple of the wavefronts per workgroup
    B, H, T = 3, 5, 9
    k, v, mk, mv = _kv_setup(dev, oracle, B, H, T, 8)
    kb = torch.zeros((B, H, T, 64), dtype=torch.uint8, device=dev); km = torch.zeros((B, H, T), dtype=torch.int32, device=dev)
    vb = torch.zeros_like(kb); vm = torch.zeros_like(km)
    okb = np.zeros((B, H, T, 64), np.uint8); okm = np.zeros((B, H, T), np.uint32)
    ovb = np.zeros_like(okb); ovm = np.zeros_like(okm)
    seq = np.array([0, 4, T], np.int32)
    for step in range(5):
        cur = np.minimum(seq + step, T).astype(np.int32)
        tok = np.minimum(cur, T - 1)
        kn = np.stack([k[b, :, tok[b]] for b in range(B)]); vn = np.stack([v[b, :, tok[b]] for b in range(B)])
        E.ecco_kv_append_minmax(mk, mv, t16(kn, dev), t16(vn, dev), kb, km, vb, vm, ti32(cur, dev), B, H, T)
        oracle.kv_append(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, kn.view(np.uint16), vn.view(np.uint16),
                         okb, okm, ovb, ovm, cur, B, H, T, minmax=True)
    torch.cuda.synchronize()
    assert np.array_equal(kb.cpu().numpy(), okb) and np.array_equal(km.cpu().numpy().view(np.uint32), okm)
    assert np.array_equal(vb.cpu().numpy(), ovb) and np.array_equal(vm.cpu().numpy().view(np.uint32), ovm)
    assert okm[2].sum() == 0 and okm[0, :, :5].all()


def test_act_codec_matches_oracle(dev, oracle):
    """2x activation codec: encoded blocks and decoded FP16 bit-exact; edge groups; arbitrary bytes; statuses."""
    rng = np.random.default_rng(31)
    edge = [np.full(64, 0.3), np.zeros(64), np.full(64, -65504.0),
            np.concatenate([[65504.0, -65504.0], rng.uniform(-65504, 65504, 62)]),
            np.concatenate([[65504.0, 60000.0], rng.uniform(60000, 65504, 62)]),
            np.concatenate([[6e-8, 0.0], np.zeros(62)]), np.concatenate([[1000.0, 1000.5], np.full(62, 1000.0)]),
            np.concatenate([[-6e-8, 6e-8], rng.uniform(-3e-6, 3e-6, 62)]), -np.abs(rng.normal(0, 3, 64)),
            np.array([-16 + 0.5 * i for i in range(63)] + [15.75])]
    n = 8192 * 64 + 4099   # more pieces than one pass of the grid, and a ragged tail
    x = W.activation(n, 64, 104)
    x[: len(edge)] = np.array(edge).astype(np.float16)
    scale = (10.0 ** rng.uniform(-4, 3, n)).astype(np.float32)          # group magnitudes over seven decades
    x[len(edge):] = (x[len(edge):].astype(np.float32) * scale[len(edge):, None]).astype(np.float16)
    x[40:60] += np.float16(7.0)                                          # groups away from zero: the zero point matters
    want_blocks = oracle.act_encode(x.view(np.uint16))
    blocks = E.ecco_act_encode(t16(x, dev))
    torch.cuda.synchronize()
    got_blocks = blocks.cpu().numpy()
    bad = np.nonzero((got_blocks != want_blocks).any(axis=1))[0]
    assert bad.size == 0, (bad[:8], got_blocks[bad[0]], want_blocks[bad[0]])
    want = oracle.act_decode(want_blocks)
    got = E.ecco_act_decode(blocks).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, want)
    assert (((got >> 10) & 0x1F) != 31).all()
    # arbitrary bytes: any block with a finite scale and zero point decodes as the rule says (infinities included)
    junk = rng.integers(0, 256, (4096, 64), dtype=np.uint8)
    junk[:64, 32:] = 0xFF                                                # reserved bits set: ignored
    side = np.zeros(4096, np.uint32)
    for i in range(32):
        side |= (junk[:, i].astype(np.uint32) >> 7) << i
    ok = (((side >> 10) & 0x1F) != 31) & (((side >> 26) & 0x1F) != 31)
    assert ok.sum() > 3000
    got = E.ecco_act_decode(tu8(junk, dev)).cpu().numpy().view(np.uint16)
    want = oracle.act_decode(junk)
    assert np.array_equal(got[ok], want[ok])
    # nothing to do / bad arguments
    E.ecco_act_encode(torch.empty((0, 64), dtype=torch.float16, device=dev))
    mis = torch.empty(64 + 8, dtype=torch.float16, device=dev)[4:68]
    with pytest.raises(E.EccoError) as e:
        E.ecco_act_encode(mis)
    assert e.value.status == -3
    misb = torch.empty(128, dtype=torch.uint8, device=dev)[16:80]
    with pytest.raises(E.EccoError) as e:
        E.ecco_act_decode(misb)
    assert e.value.status == -3


def test_kv_attend_matches_oracle(dev, oracle):
    B, H, T = 4, 3, 700  # several 256-token chunks and a ragged tail
    k, v, mk, mv = _kv_setup(dev, oracle, B, H, T, 16)
    kb, km, okb, okm = enc_both(dev, oracle, mk, k); vb, vm, ovb, ovm = enc_both(dev, oracle, mv, v)
    q = W.activation(B * H, 128, 103).reshape(B, H, 128)
    seq = np.array([T, 1, 0, 300], np.int32)
    out = E.ecco_kv_attend(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, H, T).cpu().numpy()
    want = oracle.kv_attend(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16),
                            okb, okm, ovb, ovm, seq, B, H, T)
    assert not out[2].any()
    assert_attn_close(oracle, mv, ovb, ovm, seq, B, H, H, T, out, want)
    # one token: the output is the decoded V_0 (up to FP32 rounding of p = 1)
    vdec = oracle.decode(mv.centroids, mv.code_lens, ovb, ovm).view(np.float16).reshape(B, H, T, 128)
    assert np.allclose(out[1], vdec[1, :, 0].astype(np.float64), rtol=1e-6, atol=1e-9)


def test_attend_ignores_cache_behind_seq_len(dev, oracle):
    """Slots at or behind seq_len may hold anything, NaN scales included: both attention kernels must not read them into the result."""
    B, H, T = 2, 2, 100
    k, v, mk, mv = _kv_setup(dev, oracle, B, H, T, 8)
    kb, km, okb, okm = enc_both(dev, oracle, mk, k); vb, vm, ovb, ovm = enc_both(dev, oracle, mv, v)
    seq = np.array([70, 33], np.int32)
    q = W.activation(B * H, 128, 105).reshape(B, H, 128)
    want = oracle.kv_attend(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16),
                            okb, okm, ovb, ovm, seq, B, H, T)
    kb, vb = kb.view(B, H, T, 64), vb.view(B, H, T, 64)
    km, vm = km.view(B, H, T), vm.view(B, H, T)
    for b in range(B):
        for a in (kb, vb):
            a[b, :, seq[b]:] = 0xFF
        for a in (km, vm):
            a[b, :, seq[b]:] = -1          # every bit set: scale bits 0xFFFF (a NaN), pattern 63, raw flag
    out = E.ecco_kv_attend(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, H, T).cpu().numpy()
    assert_attn_close(oracle, mv, ovb, ovm, seq, B, H, H, T, out, want)
    out = E.ecco_kv_attend_gqa(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, H, H, T, n_splits=3).cpu().numpy()
    assert_attn_close(oracle, mv, ovb, ovm, seq, B, H, H, T, out, want)


@pytest.mark.parametrize("grp,n_splits", [(1, 1), (4, 1), (8, 3), (16, 2), (3, 5)])
def test_kv_attend_gqa_matches_oracle(dev, oracle, grp, n_splits):
    B, Hkv, T = 3, 2, 1500 if grp >= 8 else 700   # several spans for the larger groups (span = 7680 / group tokens), ragged tails
    Hq = Hkv * grp
    k, v, mk, mv = _kv_setup(dev, oracle, B, Hkv, T, 16)
    kb, km, okb, okm = enc_both(dev, oracle, mk, k); vb, vm, ovb, ovm = enc_both(dev, oracle, mv, v)
    q = W.activation(B * Hq, 128, 106).reshape(B, Hq, 128)
    seq = np.array([T, 0, 333], np.int32)
    out = E.ecco_kv_attend_gqa(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, Hq, Hkv, T, n_splits=n_splits).cpu().numpy()
    want = oracle.kv_attend_gqa(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16),
                                okb, okm, ovb, ovm, seq, B, Hq, Hkv, T)
    assert out.shape == want.shape and not out[1].any()
    assert_attn_close(oracle, mv, ovb, ovm, seq, B, Hq, Hkv, T, out, want)
    if grp == 1 and n_splits == 1:
        # the plain kernel answers the same question
        ref = E.ecco_kv_attend(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, Hq, T).cpu().numpy()
        assert_attn_close(oracle, mv, ovb, ovm, seq, B, Hq, Hkv, T, ref, want)
        # argument errors
        with pytest.raises(E.EccoError) as e:
            E.ecco_kv_attend_gqa(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, 5, 2, T)
        assert e.value.status == -2
        with pytest.raises(E.EccoError) as e:
            E.ecco_kv_attend_gqa(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, 34, 2, T)
        assert e.value.status == -2


def test_gqa_long_context(dev, oracle):
    """One sequence of 20 000 tokens, 8 query heads over 2 key/value heads, 16 token splits (several spans per split)."""
    B, Hkv, grp, T = 1, 2, 4, 20000
    k, v = W.kv_cache(B, Hkv, T, 128, seed=13)
    mk = E.ecco_model_to_device(E.ecco_fit_patterns(k[:, :, :512], 16, 12, 3), 0)
    mv = E.ecco_model_to_device(E.ecco_fit_patterns(v[:, :, :512], 16, 12, 4), 0)
    kb, km, okb, okm = enc_both(dev, oracle, mk, k); vb, vm, ovb, ovm = enc_both(dev, oracle, mv, v)
    q = W.activation(B * Hkv * grp, 128, 108).reshape(B, Hkv * grp, 128)
    for seq_len, splits in [(T, 16), (T - 4321, 3), (T, 1)]:
        seq = np.array([seq_len], np.int32)
        out = E.ecco_kv_attend_gqa(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, Hkv * grp, Hkv, T, n_splits=splits).cpu().numpy()
        want = oracle.kv_attend_gqa(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16),
                                    okb, okm, ovb, ovm, seq, B, Hkv * grp, Hkv, T)
        assert_attn_close(oracle, mv, ovb, ovm, seq, B, Hkv * grp, Hkv, T, out, want, (seq_len, splits))
    # the plain kernel on the same cache: 20 000 tokens are three spans of its running softmax
    q1 = np.ascontiguousarray(q[:, :Hkv])
    for seq_len in (T, 8192, 8193):
        seq = np.array([seq_len], np.int32)
        out = E.ecco_kv_attend(mk, mv, t16(q1, dev), kb, km, vb, vm, ti32(seq, dev), B, Hkv, T).cpu().numpy()
        want = oracle.kv_attend(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q1.view(np.uint16),
                                okb, okm, ovb, ovm, seq, B, Hkv, T)
        assert_attn_close(oracle, mv, ovb, ovm, seq, B, Hkv, Hkv, T, out, want, seq_len)


# ---------------------------------------------------------------------------------------------------
# full-size workloads: every group, every row and every output element against the oracle
def _check_weight_case(dev, oracle, w, m, ob, om, batches, x_seed, tag):
    """Encode, decode (values and indices) and the fused GEMV of the matrix `w` under model `m`, all groups and all
    rows against the oracle's blocks `ob`, `om` (which the oracle made from `w` itself)."""
    rows, cols = w.shape
    blocks, meta = E.ecco_encode(m, t16(w, dev))
    assert np.array_equal(np_meta(meta), om), tag
    assert np.array_equal(np_blocks(blocks), ob), tag
    oidx, _ = oracle.decode_indices(m.code_lens, m.S, ob, om)
    assert np.array_equal(E.ecco_decode_indices(m, blocks, meta).cpu().numpy(), oidx), tag
    del oidx
    odec = oracle.decode(m.centroids, m.code_lens, ob, om)
    assert np.array_equal(E.ecco_decode(m, blocks, meta).cpu().numpy().view(np.uint16), odec), tag
    absw = np.abs(odec.view(np.float16).astype(np.float32)).reshape(rows, cols)
    del odec
    for batch in batches:
        x = W.activation(batch, cols, x_seed)
        y = E.ecco_decode_gemv(m, blocks, meta, rows, cols, t16(x, dev)).cpu().numpy()
        want = oracle.gemv(m.centroids, m.code_lens, ob, om, rows, cols, x.view(np.uint16))
        assert y.shape == want.shape
        assert rel_l2(y, want) <= REL_L2, (tag, batch)
        for b in range(batch):
            assert rel_l2(y[b], want[b]) <= REL_L2, (tag, batch, b)
        # element by element: |y - ref| <= 1e-3 * sum_c |w_rc| |x_c|
        bound = (np.abs(x.astype(np.float32)) @ absw.T).astype(np.float64)
        err = np.abs(y.astype(np.float64) - want)
        assert (err <= REL_L2 * bound).all(), (tag, batch, np.unravel_index(np.argmax(err - REL_L2 * bound), err.shape))
    return blocks, meta


def _full_weight_case(dev, oracle, name, which, rows_limit=None, batches=(1,)):
    c = W.CONFIGS[name]
    w = W.config_weight(name, which, rows=rows_limit)
    m = E.ecco_model_to_device(E.ecco_fit_patterns(w, c["S"], 12, c["seeds"][which]), 0)
    assert oracle.verify_model(m.centroids, m.code_lens) == 0
    ob, om = oracle.encode(m.centroids, m.code_lens, w.view(np.uint16))
    # what the format promises for every block: pattern ids in range, the second chain starts inside the block and at
    # bit 256 exactly in raw blocks
    assert ((om >> 16) & 63).max() < m.S
    israw = ((om >> 22) & 1) == 1
    assert ((om >> 23)[israw] == 256).all() and (om >> 23).max() < 512 - 64
    _check_weight_case(dev, oracle, w, m, ob, om, batches, c["x_seed"], name)
    return w, m, ob, om


def test_full_proj7b(dev, oracle):
    _full_weight_case(dev, oracle, "proj7b", 0, batches=(1,))


def test_full_mlp_up(dev, oracle):
    _full_weight_case(dev, oracle, "mlp", 0, batches=(1, 8, 16))


def test_full_mlp_down(dev, oracle):
    _full_weight_case(dev, oracle, "mlp", 1, batches=(1, 8, 16))


def test_proj70b_row_slab(dev, oracle):
    # the 70B-class projection at its real row length (224 column groups), first 1024 rows: four rows per workgroup
    _full_weight_case(dev, oracle, "proj70b", 0, rows_limit=1024, batches=(1, 16))


@pytest.fixture(scope="module")
def proj70b(dev, oracle):
    """The 70B-class projection, 8192 x 28672 = 1 835 008 groups: the tensor, the library's fit, the oracle's blocks."""
    c = W.CONFIGS["proj70b"]
    w = W.config_weight("proj70b", 0)
    m = E.ecco_model_to_device(E.ecco_fit_patterns(w, c["S"], 12, c["seeds"][0]), 0)
    assert oracle.verify_model(m.centroids, m.code_lens) == 0
    ob, om = oracle.encode(m.centroids, m.code_lens, w.view(np.uint16))
    return dict(w=w, m=m, ob=ob, om=om)


def test_full_proj70b(dev, oracle, proj70b):
    """The full shape in the launch shapes the benchmark times (batch 1: 32 rows x 7 column tiles = 224 units per
    workgroup; batch 16: two 16-row blocks per workgroup): every block, every decoded value and every output element
    against the oracle."""
    w, m, ob, om = (proj70b[k] for k in ("w", "m", "ob", "om"))
    assert ((om >> 16) & 63).max() < m.S
    israw = ((om >> 22) & 1) == 1
    assert ((om >> 23)[israw] == 256).all() and (om >> 23).max() < 512 - 64
    _check_weight_case(dev, oracle, w, m, ob, om, (1, 16), W.CONFIGS["proj70b"]["x_seed"], "proj70b")


def test_decode_sweep_sizes_beyond_the_matrix(dev, oracle, proj70b):
    """The standalone decoder at the two sweep sizes beyond the matrix, 2^21 and 2^22 groups: further rows of the same
    seeded stream under the same model, encoded by the oracle, every decoded value against the oracle."""
    m, ob, om = (proj70b[k] for k in ("m", "ob", "om"))
    c = W.CONFIGS["proj70b"]
    rows, cols = c["shapes"][0]
    gpr = cols // 128
    n_total = 1 << 22
    extra_rows = -(-(n_total - rows * gpr) // gpr)
    w2 = W.weight_matrix(extra_rows, cols, c["sigma"], c["outlier_frac"], c["outlier_mult"], c["seeds"][0], row_start=rows)
    ob2, om2 = oracle.encode(m.centroids, m.code_lens, w2.view(np.uint16))
    del w2
    ob_all = np.concatenate([ob, ob2])[:n_total]
    om_all = np.concatenate([om, om2])[:n_total]
    del ob2, om2
    blocks, meta = tu8(ob_all, dev), ti32(om_all, dev)
    for n in (1 << 21, n_total):
        got = E.ecco_decode(m, blocks[:n], meta[:n]).cpu().numpy().view(np.uint16)
        step = 1 << 19  # compared in pieces: the oracle's output of one piece at a time
        for s0 in range(0, n, step):
            want = oracle.decode(m.centroids, m.code_lens, ob_all[s0:s0 + step], om_all[s0:s0 + step])
            assert np.array_equal(got[s0:s0 + step], want), (n, s0)
        del got


@pytest.fixture(scope="module")
def kvfull(dev, oracle):
    """The KV configuration at full size (8 sequences x 32 heads x 4096 tokens, patterns fitted on a 512-token prefix):
    the caches, the library's fits, and the oracle's blocks of every token."""
    c = W.CONFIGS["kv"]
    B, H, T, S = c["batch"], c["heads"], c["tokens"], c["S"]
    k, v = W.kv_cache(B, H, T, 128, c["seeds"][0])
    cal = c["calib_tokens"]
    mk = E.ecco_model_to_device(E.ecco_fit_patterns(k[:, :, :cal], S, 12, c["seeds"][0]), 0)
    mv = E.ecco_model_to_device(E.ecco_fit_patterns(v[:, :, :cal], S, 12, c["seeds"][0] + 1), 0)
    assert oracle.verify_model(mk.centroids, mk.code_lens) == 0 and oracle.verify_model(mv.centroids, mv.code_lens) == 0
    okb, okm = oracle.encode(mk.centroids, mk.code_lens, k.view(np.uint16))
    ovb, ovm = oracle.encode(mv.centroids, mv.code_lens, v.view(np.uint16))
    return dict(B=B, H=H, T=T, k=k, v=v, mk=mk, mv=mv, okb=okb, okm=okm, ovb=ovb, ovm=ovm,
                q=W.activation(B * H, 128, c["q_seed"]).reshape(B, H, 128),
                seq=np.array([T, T, T - 1, 2500, 33, 1, T, 777], np.int32))


def test_full_kv_cache_encode_and_attend(dev, oracle, kvfull):
    """Bulk encode of both caches (1 M groups each) and single-query attention over them in the launch shape the
    benchmark times: every block and every output element of every head against the oracle; then the append of one
    token per sequence on every head."""
    B, H, T, k, v, mk, mv, q, seq = (kvfull[n] for n in ("B", "H", "T", "k", "v", "mk", "mv", "q", "seq"))
    okb, okm, ovb, ovm = (kvfull[n] for n in ("okb", "okm", "ovb", "ovm"))
    kb, km = E.ecco_encode(mk, t16(k, dev)); vb, vm = E.ecco_encode(mv, t16(v, dev))
    assert np.array_equal(np_blocks(kb), okb) and np.array_equal(np_meta(km), okm)
    assert np.array_equal(np_blocks(vb), ovb) and np.array_equal(np_meta(vm), ovm)
    kb = kb.view(B, H, T, 64); vb = vb.view(B, H, T, 64); km = km.view(B, H, T); vm = vm.view(B, H, T)
    out = E.ecco_kv_attend(mk, mv, t16(q, dev), kb, km, vb, vm, ti32(seq, dev), B, H, T).cpu().numpy()
    want = oracle.kv_attend(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16),
                            okb, okm, ovb, ovm, seq, B, H, T)
    assert_attn_close(oracle, mv, ovb, ovm, seq, B, H, H, T, out, want)
    # append of one token per sequence at the last slot, on every head, against the oracle's append on its own caches
    kb2, km2, vb2, vm2 = kb.clone(), km.clone(), vb.clone(), vm.clone()
    kn = np.ascontiguousarray(k[:, :, 7]); vn = np.ascontiguousarray(v[:, :, 7])
    pos = np.full(B, T - 1, np.int32)
    E.ecco_kv_append(mk, mv, t16(kn, dev), t16(vn, dev), kb2, km2, vb2, vm2, ti32(pos, dev), B, H, T)
    torch.cuda.synchronize()
    akb, akm = okb.reshape(B, H, T, 64).copy(), okm.reshape(B, H, T).copy()
    avb, avm = ovb.reshape(B, H, T, 64).copy(), ovm.reshape(B, H, T).copy()
    oracle.kv_append(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, kn.view(np.uint16), vn.view(np.uint16),
                     akb, akm, avb, avm, pos, B, H, T)
    assert np.array_equal(kb2.cpu().numpy(), akb) and np.array_equal(np_meta(km2).reshape(B, H, T), akm)
    assert np.array_equal(vb2.cpu().numpy(), avb) and np.array_equal(np_meta(vm2).reshape(B, H, T), avm)
    # the same values in another slot encode to the same bytes
    assert torch.equal(kb2[:, :, T - 1], kb[:, :, 7]) and torch.equal(km2[:, :, T - 1], km[:, :, 7])


def test_full_kv_cache_grouped_and_minmax(dev, oracle, kvfull):
    """Grouped queries in the benchmark's shape (the 32 query heads over the caches of the first 8 heads, 4 token splits):
    every output element against the oracle.  Then the min/max selector over the whole K cache (1 M groups, the bulk
    launch the benchmark times) and as an append: every block against the oracle."""
    B, H, T, k, v, mk, mv, q, seq = (kvfull[n] for n in ("B", "H", "T", "k", "v", "mk", "mv", "q", "seq"))
    grp, Hkv, splits = 4, H // 4, 4
    okb, okm = kvfull["okb"].reshape(B, H, T, 64)[:, :Hkv].copy(), kvfull["okm"].reshape(B, H, T)[:, :Hkv].copy()
    ovb, ovm = kvfull["ovb"].reshape(B, H, T, 64)[:, :Hkv].copy(), kvfull["ovm"].reshape(B, H, T)[:, :Hkv].copy()
    gkb, gkm, gvb, gvm = tu8(okb, dev), ti32(okm, dev), tu8(ovb, dev), ti32(ovm, dev)
    outg = E.ecco_kv_attend_gqa(mk, mv, t16(q, dev), gkb, gkm, gvb, gvm, ti32(seq, dev), B, H, Hkv, T, n_splits=splits).cpu().numpy()
    want = oracle.kv_attend_gqa(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, q.view(np.uint16),
                                okb, okm, ovb, ovm, seq, B, H, Hkv, T)
    assert_attn_close(oracle, mv, ovb.reshape(-1, 64), ovm.reshape(-1), seq, B, H, Hkv, T, outg, want)
    mb, mm = E.ecco_encode_minmax(mk, t16(k, dev))
    ob, om = oracle.encode_minmax(mk.centroids, mk.code_lens, k.view(np.uint16))
    assert np.array_equal(np_blocks(mb), ob) and np.array_equal(np_meta(mm), om)
    kb3, km3 = tu8(kvfull["okb"], dev).view(B, H, T, 64), ti32(kvfull["okm"], dev).view(B, H, T)
    vb3, vm3 = tu8(kvfull["ovb"], dev).view(B, H, T, 64), ti32(kvfull["ovm"], dev).view(B, H, T)
    kn = np.ascontiguousarray(k[:, :, 7]); vn = np.ascontiguousarray(v[:, :, 7])
    pos = np.full(B, T - 1, np.int32)
    E.ecco_kv_append_minmax(mk, mv, t16(kn, dev), t16(vn, dev), kb3, km3, vb3, vm3, ti32(pos, dev), B, H, T)
    akb, akm = kvfull["okb"].reshape(B, H, T, 64).copy(), kvfull["okm"].reshape(B, H, T).copy()
    avb, avm = kvfull["ovb"].reshape(B, H, T, 64).copy(), kvfull["ovm"].reshape(B, H, T).copy()
    oracle.kv_append(mk.centroids, mk.code_lens, mv.centroids, mv.code_lens, kn.view(np.uint16), vn.view(np.uint16),
                     akb, akm, avb, avm, pos, B, H, T, minmax=True)
    assert np.array_equal(kb3.cpu().numpy(), akb) and np.array_equal(np_meta(km3).reshape(B, H, T), akm)
    assert np.array_equal(vb3.cpu().numpy(), avb) and np.array_equal(np_meta(vm3).reshape(B, H, T), avm)
    # token 7's block by the bulk min/max encoder equals the appended one
    assert np.array_equal(akb[:, :, T - 1].reshape(-1, 64), ob.reshape(B, H, T, 64)[:, :, 7].reshape(-1, 64))


def test_repeated_launches_are_identical(dev, oracle):
    # the fused kernels fix their summation order, so every launch must give the same bits; a timing-dependent
    # slip (a race between wavefronts, a missed wait) shows up here as a launch that differs
    c = W.CONFIGS["mlp"]
    rows, cols = c["shapes"][0]
    w = W.config_weight("mlp", 0)
    m = E.ecco_model_to_device(E.ecco_fit_patterns(w, c["S"], 12, c["seeds"][0]), 0)
    blocks, meta = E.ecco_encode(m, t16(w, dev))
    dec = E.ecco_decode(m, blocks, meta).float().reshape(rows, cols)
    for batch in (1, 2, 16):
        x = t16(W.activation(batch, cols, 11), dev)
        first = E.ecco_decode_gemv(m, blocks, meta, rows, cols, x)
        ref = x.float() @ dec.T
        assert float((first - ref).norm() / ref.norm()) <= REL_L2
        for _ in range(40):
            again = E.ecco_decode_gemv(m, blocks, meta, rows, cols, x)
            assert torch.equal(first, again), batch


@pytest.mark.parametrize("rows,cols", [(8192, 4096), (12288, 4352)])
def test_batched_gemv_all_wavefronts_busy_repeatable(dev, oracle, rows, cols):
    """The batched kernel where every one of its sixteen wavefronts has units and a workgroup has two or three row
    blocks, under a 16-pattern model (the per-wavefront slices then straddle the 64 KB mark of the LDS): every row block
    of every launch right against the decoded matrix (the decoder is checked against the oracle elsewhere), and twenty
    launches bit for bit.  A timing-dependent slip in this regime shows as single wrong row blocks that move from launch
    to launch."""
    wt = W.config_weight("tiny")
    m = E.ecco_model_to_device(E.ecco_fit_patterns(wt, 16, 12, 0), 0)
    w = W.weight_matrix(rows, cols, 0.02, 1e-3, 10.0, 5)
    blocks, meta = E.ecco_encode(m, t16(w, dev))
    dec = E.ecco_decode(m, blocks, meta).float().reshape(rows, cols)
    for batch in (4, 16):
        xb = t16(W.activation(batch, cols, 60 + batch), dev)
        ref = xb.float() @ dec.T
        bound = xb.float().abs() @ dec.abs().T
        first = E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb)
        assert bool(((first - ref).abs() <= REL_L2 * bound + 1e-30).all()), batch
        for _ in range(20):
            assert torch.equal(first, E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb)), batch


@pytest.mark.parametrize("rows,cols", [(37, 8192), (8200, 1024), (48, 4096), (16400, 256)])
def test_batched_gemv_repeatable_with_long_codes(dev, oracle, rows, cols):
    """The batched kernel's long-code variant on shapes with several units per wavefront (37 x 8192), with three row
    blocks per workgroup and a ragged last one (8200 x 1024), and with one unit per wavefront: right against the
    batch-1 kernel's rows, and the same bits on every launch.  16400 x 256: five row blocks per workgroup (two rounds
    of the workgroup's reduction) and one unit per row block, so fifteen of the sixteen wavefronts have none."""
    S = 7
    cent, lens, probs = _skewed_model(oracle, S, 1)
    assert lens.max() == 12
    m = E.ecco_model_to_device(E.ecco_model_create(cent, lens), 0)
    n = rows * cols // 128
    x = _skewed_data(cent, probs, 4096, 5)
    x = np.tile(x, (-(-n // 4096), 1))[:n]
    blocks, meta = E.ecco_encode(m, t16(x, dev))
    for batch in (4, 16):
        xb = t16(W.activation(batch, cols, 40 + batch), dev)
        ref = torch.stack([E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb[b:b + 1].contiguous())[0] for b in range(batch)])
        first = E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb)
        assert float((first - ref).norm() / ref.norm()) <= REL_L2, batch
        for _ in range(10):
            assert torch.equal(first, E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb)), batch


def test_batched_gemv_random_shapes(dev, oracle):
    """Thirty seeded shapes (1 to 20 000 rows, 1 to 86 column groups, batch 2 to 16) under three models (long codes,
    16 and 64 fitted patterns): the batched kernel against the batch-1 kernel row by row, and three launches bit for bit.
    (The batch-1 kernel is checked against the oracle elsewhere; this test is about the batched kernel's indexing.)"""
    rng = np.random.default_rng(0)
    cent, lens, probs = _skewed_model(oracle, 7, 1)
    models = [(E.ecco_model_to_device(E.ecco_model_create(cent, lens), 0), (cent, probs))]
    w = W.weight_matrix(512, 4096, 0.02, 1e-3, 10.0, 77)
    models += [(E.ecco_model_to_device(E.ecco_fit_patterns(w, S, 12, 5), 0), None) for S in (16, 64)]
    for case in range(30):
        m, skew = models[case % 3]
        rows = int(rng.choice([1, 3, 15, 16, 17, 47, 300, 1000, 4097, 8200, 12290, 20000]))
        gpr = int(rng.choice([1, 2, 3, 7, 8, 31, 32, 33, 64, 86]))
        if rows * gpr > 400000:
            gpr = max(1, 400000 // rows)
        cols, n = gpr * 128, rows * gpr
        base = _skewed_data(skew[0], skew[1], 2048, case) if skew else \
            W.weight_matrix(16, 128 * 128, 0.02, 1e-3, 10.0, 1000 + case).reshape(-1, 128)
        x = np.ascontiguousarray(np.tile(base, (-(-n // base.shape[0]), 1))[:n])
        blocks, meta = E.ecco_encode(m, t16(x, dev))
        batch = int(rng.integers(2, 17))
        xb = t16(W.activation(batch, cols, 500 + case), dev)
        ref = torch.stack([E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb[b:b + 1].contiguous())[0] for b in range(batch)])
        first = E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb)
        assert float((first - ref).norm() / ref.norm()) <= REL_L2, (case, rows, gpr, batch)
        for _ in range(2):
            assert torch.equal(first, E.ecco_decode_gemv(m, blocks, meta, rows, cols, xb)), (case, rows, gpr, batch)


def test_graph_replay_matches_eager(dev, oracle, tiny):
    """Every entry point of the two-chain format recorded into one HIP graph and replayed three times on inputs that
    change between the replays (with eager work and synchronisation in between): every replay must give the bits the
    eager calls give on the same inputs."""
    m = tiny["m"]
    rows, cols = 64, 1024
    B, H, T = 2, 4, 96
    k, v, mk, mv = _kv_setup(dev, oracle, B, H, T, 8)

    def inputs(seed):
        w = W.weight_matrix(rows, cols, 0.02, 0.001, 10.0, seed)
        x = W.activation(8, cols, seed + 1)
        q = W.activation(B * H, 128, seed + 2).reshape(B, H, 128)
        kn = W.activation(B * H, 128, seed + 3).reshape(B, H, 128)
        vn = W.activation(B * H, 128, seed + 4).reshape(B, H, 128)
        return [t16(a, dev) for a in (w, x, q, kn, vn)]

    w_in, x_in, q_in, kn_in, vn_in = inputs(50)
    kb, km = E.ecco_encode(mk, t16(k, dev)); vb, vm = E.ecco_encode(mv, t16(v, dev))
    kb0, km0, vb0, vm0 = kb.clone(), km.clone(), vb.clone(), vm.clone()
    seq = ti32(np.array([T - 1, 40], np.int32), dev)
    blocks = torch.empty((rows * cols // 128, 64), dtype=torch.uint8, device=dev)
    meta = torch.empty((rows * cols // 128,), dtype=torch.int32, device=dev)
    dec = torch.empty((rows, cols), dtype=torch.float16, device=dev)
    y1 = torch.empty((1, rows), dtype=torch.float32, device=dev)
    y8 = torch.empty((8, rows), dtype=torch.float32, device=dev)
    att = torch.empty((B, H, 128), dtype=torch.float32, device=dev)
    gqa = torch.empty((B, H, 128), dtype=torch.float32, device=dev)
    gqa_na = torch.empty((B, H, 128), dtype=torch.float32, device=dev)
    ws = torch.empty((B * H * 2 * 130 * 4,), dtype=torch.uint8, device=dev)  # ecco_kv_attend_gqa_workspace(B, Hq, 2) bytes
    ab = torch.empty((rows * cols // 64, 64), dtype=torch.uint8, device=dev)
    adec = torch.empty((rows, cols), dtype=torch.float16, device=dev)

    outs = lambda: [t.clone() for t in (blocks, meta, dec, y1, y8, att, gqa, gqa_na, ab, adec, kb, km, vb, vm)]
    seq1 = seq + 1  # built outside the capture: the graph holds kernels of the library only
    def run_all():  # what is recorded: calls of the library only
        E.ecco_encode(m, w_in, blocks, meta)
        E.ecco_decode(m, blocks, meta, dec)
        E.ecco_decode_gemv(m, blocks, meta, rows, cols, x_in[:1], y1)
        E.ecco_decode_gemv(m, blocks, meta, rows, cols, x_in, y8)
        E.ecco_kv_append(mk, mv, kn_in, vn_in, kb, km, vb, vm, seq, B, H, T)
        E.ecco_kv_attend(mk, mv, q_in, kb, km, vb, vm, seq1, B, H, T, att)
        E.ecco_kv_attend_gqa(mk, mv, q_in, kb, km, vb, vm, seq1, B, H, H // 2, T, 2, ws, gqa)
        E.ecco_kv_attend_gqa_noalloc(mk, mv, q_in, kb, km, vb, vm, seq1, B, H, H // 2, T, 2, gqa_na)  # splits in the static array
        E.ecco_act_encode(w_in, ab)
        E.ecco_act_decode(ab, adec)

    run_all()  # warm-up outside the capture (kernel attributes are set on first use)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    for rep, seed in enumerate((60, 70, 80)):
        new = inputs(seed)
        for dst, src in zip((w_in, x_in, q_in, kn_in, vn_in), new):
            dst.copy_(src)
        for dst, src in zip((kb, km, vb, vm), (kb0, km0, vb0, vm0)):
            dst.copy_(src)
        run_all()
        torch.cuda.synchronize()
        want = outs()
        for t in (blocks, meta, dec, y1, y8, att, gqa, gqa_na, ab, adec):
            t.zero_()
        for dst, src in zip((kb, km, vb, vm), (kb0, km0, vb0, vm0)):
            dst.copy_(src)
        _ = (dec.float() @ dec.float().T).sum().item()  # eager work of the program's own between the replays
        g.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(outs(), want)):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (rep, i)
        assert torch.equal(gqa, gqa_na), rep
