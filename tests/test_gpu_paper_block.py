"""Parity of the self-contained block format (include/ecco_paper_block.h) against its CPU oracle, through the C ABI, on
one MI355X: encoded blocks and decoded FP16 bit-exact."""
from __future__ import annotations

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2505_06901_amd as E  # noqa: E402
from paper_2505_06901_amd import workloads as W  # noqa: E402
from test_paper_block_pins import _groups, _model  # noqa: E402


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def pb():
    from oracle import paper_block as P
    return P


def _both(pb, om):
    """The library's model object for an oracle-side model description."""
    return E.ecco_pb_model_to_device(E.ecco_pb_model_create(om.cent, om.lens, om.kp_lens, om.texp), 0)


def _t16(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.float16)).to(dev)


def _check_roundtrip(pb, dev, om, m, x):
    want_blocks = pb.encode(om, x.view(np.uint16))
    got_blocks = E.ecco_pb_encode(m, _t16(x, dev)).cpu().numpy()
    bad = np.nonzero((got_blocks != want_blocks).any(axis=1))[0]
    assert bad.size == 0, (bad[:8], got_blocks[bad[0]], want_blocks[bad[0]])
    want, n_coded, n_out = pb.decode(om, want_blocks)
    got = E.ecco_pb_decode(m, torch.from_numpy(want_blocks).to(dev)).cpu().numpy().view(np.uint16)
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, (bad[:8], n_coded[bad[0]], n_out[bad[0]], np.nonzero(got[bad[0]] != want[bad[0]])[0][:8])
    return n_coded, n_out


def test_hand_models_bit_exact(pb, dev):
    for S, texp, seed, skew in [(5, -9, 1, 2.4), (1, -6, 2, 1.6), (64, -8, 3, 3.0)]:
        om = _model(pb, S=S, texp=texp, seed=seed, skew=skew)
        m = _both(pb, om)
        x = _groups(seed + 10, 64 * 5 + 37, scale=2.0 ** texp * 40)           # several passes of 64 blocks and a ragged tail
        x[0] = 0
        x[1] = np.float16(2.0 ** texp * 480)                                  # every element at the largest scale
        x[2, 5] = -x[2, 5]; x[2, 77] = -np.abs(x[2]).max() * np.float16(1.0)   # the largest magnitude is negative
        x[3] = (np.arange(128) - 64).astype(np.float16) * np.float16(2.0 ** texp)
        x[4, :] = np.float16(6e-8)                                            # below the smallest scale: everything rounds to 0
        x[5] = np.float16(-0.0)
        n_coded, n_out = _check_roundtrip(pb, dev, om, m, x)
        assert (n_coded < 128).any() or S == 1 or skew < 2, "no clipped block in this input"
        assert (n_out > 0).any(), "no padded block in this input"
        # arbitrary bytes decode identically
        junk = np.random.default_rng(seed).integers(0, 256, (64 * 3 + 5, 64), dtype=np.uint8)
        want, _, _ = pb.decode(om, junk)
        got = E.ecco_pb_decode(m, torch.from_numpy(junk).to(dev)).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, want)


def test_fitted_model_bit_exact(pb, dev):
    w = W.config_weight("tiny")                                               # 64 x 1024, N(0, 0.02) with outliers
    m = E.ecco_pb_model_to_device(E.ecco_pb_fit(w, 16, 0), 0)
    om = pb.Model(m.centroids, m.code_lens, m.kp_lens, m.texp)
    assert pb.verify_model(om) == 0
    n_coded, n_out = _check_roundtrip(pb, dev, om, m, w.reshape(-1, 128))
    # reconstruction is close: relative squared error of a 15-level non-uniform quantiser with outliers kept in FP8
    dec = E.ecco_pb_decode(m, E.ecco_pb_encode(m, _t16(w, dev))).float().cpu().numpy().reshape(w.shape)
    rel = np.square(dec - w.astype(np.float32)).sum() / np.square(w.astype(np.float32)).sum()
    assert rel < 0.02, rel
    # argument errors
    with pytest.raises(E.EccoError) as e:
        E.ecco_pb_decode(m, torch.empty(128 + 16, dtype=torch.uint8, device=dev)[16:144])
    assert e.value.status == -3
    E.ecco_pb_encode(m, torch.empty((0, 128), dtype=torch.float16, device=dev))


def test_full_projection(pb, dev):
    """The 4096 x 4096 projection (131 072 groups), model fitted with S = 64, in the launch shape the benchmark times:
    every block against the oracle's encoder, every decoded value against its decoder, every row of the fused
    matrix-vector product against its double-precision product, by norm and element by element."""
    w = W.config_weight("proj7b")
    m = E.ecco_pb_model_to_device(E.ecco_pb_fit(w, 64, 1), 0)
    om = pb.Model(m.centroids, m.code_lens, m.kp_lens, m.texp)
    assert pb.verify_model(om) == 0
    want_blocks = pb.encode(om, w.reshape(-1, 128).view(np.uint16))
    blocks = E.ecco_pb_encode(m, _t16(w, dev))
    assert np.array_equal(blocks.cpu().numpy(), want_blocks)
    want, n_coded, n_out = pb.decode(om, want_blocks)
    dec = E.ecco_pb_decode(m, blocks).cpu().numpy().view(np.uint16)
    assert np.array_equal(dec, want)
    assert (n_coded < 128).any() and (n_out > 0).any()
    x = W.activation(1, 4096, 101).reshape(-1)
    y = E.ecco_pb_decode_gemv(m, blocks, 4096, 4096, _t16(x, dev)).cpu().numpy().astype(np.float64)
    ref = pb.gemv(om, want_blocks, 4096, 4096, x.view(np.uint16))
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) <= 1e-3
    # element by element: |y - ref| <= 1e-3 * sum_c |w_rc| |x_c| over the decoded weights
    bound = np.abs(want.view(np.float16).reshape(4096, 4096).astype(np.float32)) @ np.abs(x.astype(np.float32))
    err = np.abs(y - ref)
    assert (err <= 1e-3 * bound.astype(np.float64)).all(), int(np.argmax(err - 1e-3 * bound))
    # whole-output properties: finite values, bounded by the tensor's largest magnitude times the FP8 rounding slack
    assert (((dec >> 10) & 0x1F) != 31).all()
    top = float(np.abs(w.astype(np.float32)).max())
    assert float(np.abs(dec.view(np.float16).astype(np.float32)).max()) <= top * 1.07


def test_fused_gemv_matches_oracle(pb, dev):
    """Decode fused into the matrix-vector product: rel-L2 <= 1e-3 against the double-precision oracle; ragged shapes, a band
    that ends inside a pass of 64 blocks, blocks with clipped values and padded entries, arbitrary bytes."""
    om = _model(pb, S=6, texp=-9, seed=21, skew=2.6)
    m = _both(pb, om)
    rng = np.random.default_rng(22)
    for rows, gpr in [(1, 1), (5, 3), (17, 32), (40, 33), (300, 2), (64, 64), (9, 70), (700, 5), (11, 512)]:  # 512: the widest matrix allowed
        cols = gpr * 128
        w = _groups(rows * 7 + gpr, rows * gpr, scale=2.0 ** -9 * 30).reshape(rows, cols)
        blocks = pb.encode(om, w.view(np.uint16))
        x = W.activation(1, cols, 200 + gpr).reshape(cols)
        want = pb.gemv(om, blocks, rows, cols, x.view(np.uint16))
        got = E.ecco_pb_decode_gemv(m, torch.from_numpy(blocks).to(dev), rows, cols, _t16(x, dev)).cpu().numpy()
        err = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
        assert got.shape == (rows,) and err <= 1e-3, (rows, gpr, err)
        dec = pb.decode(om, blocks)[0].view(np.float16).reshape(rows, cols).astype(np.float32)
        bound = (np.abs(dec) @ np.abs(x.astype(np.float32))).astype(np.float64)
        assert (np.abs(got - want) <= 1e-3 * bound + 1e-30).all(), (rows, gpr)
    # arbitrary bytes (repeated positions among the padded entries included): same values as a sequential reader
    rows, gpr = 37, 4
    junk = rng.integers(0, 256, (rows * gpr, 64), dtype=np.uint8)
    x = W.activation(1, gpr * 128, 300).reshape(-1)
    want = pb.gemv(om, junk, rows, gpr * 128, x.view(np.uint16))
    got = E.ecco_pb_decode_gemv(m, torch.from_numpy(junk).to(dev), rows, gpr * 128, _t16(x, dev)).cpu().numpy()
    assert np.linalg.norm(got - want) / np.linalg.norm(want) <= 1e-3
    # unit vectors pick single decoded columns, padded entries included
    w = _groups(5, 8 * 2, scale=2.0 ** -9 * 30).reshape(8, 256)
    blocks = pb.encode(om, w.view(np.uint16))
    dec, n_coded, n_out = pb.decode(om, blocks)
    assert (n_out > 0).any()
    dec = dec.view(np.float16).reshape(8, 256).astype(np.float64)
    for j in (0, 100, 128, 255):
        e = np.zeros(256, np.float16); e[j] = 1
        got = E.ecco_pb_decode_gemv(m, torch.from_numpy(blocks).to(dev), 8, 256, _t16(e, dev)).cpu().numpy()
        assert np.allclose(got, dec[:, j], rtol=2e-3, atol=1e-9), j
    with pytest.raises(E.EccoError) as e:
        E.ecco_pb_decode_gemv(m, torch.from_numpy(blocks).to(dev), 8, 200, _t16(np.zeros(200, np.float16), dev))
    assert e.value.status == -2
