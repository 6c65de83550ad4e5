"""CPU-side checks of libecco: the C ABI loads and exports what include/ecco.h declares, the CPU fit
meets the model invariants and agrees with the oracle's fit where the paper's steps fix the result,
models serialise, and argument errors are reported before anything is launched.  No GPU needed."""
from __future__ import annotations

import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2505_06901_amd as E
from paper_2505_06901_amd import binding, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_exported():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    declared = set(re.findall(r"\b(ecco_[a-z_A-Z0-9]+)\s*\(", text))
    declared -= {"ecco_model", "ecco_status", "ecco_pb_model"}  # type names that precede a parenthesis in comments
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert binding.strerror(0) == "ok" and "shape" in binding.strerror(-2)


@pytest.fixture(scope="module")
def tiny_model():
    w = W.config_weight("tiny")
    return w, E.ecco_fit_patterns(w, 16, 12, 0)


def test_fit_invariants_and_oracle_agreement(oracle, tiny_model):
    w, m = tiny_model
    cent, lens = m.centroids, m.code_lens
    assert m.S == 16 and cent.shape == (16, 16)
    assert oracle.verify_model(cent, lens) == 0          # the oracle's independent verifier
    ocent, olens, ohist, _ = oracle.fit(w.view(np.uint16), 16, 12, 0)
    # both follow the same stated steps with the same seed: the shared patterns agree exactly here
    assert np.array_equal(cent, ocent)
    # code lengths may differ in ties; the cost on the oracle's counts must be the same (optimal cost is unique)
    for p in range(16):
        if ohist[p].sum():
            assert ((ohist[p] + 1) * lens[p]).sum() == ((ohist[p] + 1) * olens[p]).sum()
        else:
            assert (lens[p] == 4).all()
    m2 = E.ecco_fit_patterns(w, 16, 12, 0)
    assert np.array_equal(m2.centroids, cent) and np.array_equal(m2.code_lens, lens)


def test_fit_respects_length_limit(oracle):
    # one-sided, very peaked data make rare indices: unlimited Huffman would exceed 6 bits
    rng = np.random.default_rng(0)
    x = (rng.standard_t(1.2, size=(400, 128)) * 0.01).astype(np.float16)
    x = np.clip(x, -60000, 60000)
    m = E.ecco_fit_patterns(x, 4, 6, 3)
    assert m.code_lens.max() <= 6
    assert oracle.verify_model(m.centroids, m.code_lens) == 0
    m12 = E.ecco_fit_patterns(x, 4, 12, 3)
    assert oracle.verify_model(m12.centroids, m12.code_lens) == 0
    assert m12.code_lens.max() > 6


def test_fit_subsamples_large_inputs(oracle):
    w = W.weight_matrix(1100, 8192, 0.02, 1e-3, 10.0, seed=5)  # 70 400 groups > 65 536
    m = E.ecco_fit_patterns(w, 8, 12, 7)
    assert oracle.verify_model(m.centroids, m.code_lens) == 0


def test_model_roundtrip_and_validation(tiny_model):
    _, m = tiny_model
    blob = E.ecco_model_save(m)
    assert len(blob) == 16 + 16 * 16 * 3
    m2 = E.ecco_model_load(blob)
    assert np.array_equal(m2.centroids, m.centroids) and np.array_equal(m2.code_lens, m.code_lens)
    bad = bytearray(blob); bad[0] ^= 1
    with pytest.raises(E.EccoError) as e:
        E.ecco_model_load(bytes(bad))
    assert e.value.status == -5
    with pytest.raises(E.EccoError):
        E.ecco_model_load(blob[:-1])
    cent, lens = m.centroids, m.code_lens
    c2 = cent.copy(); c2[3, 4], c2[3, 5] = cent[3, 5] + 1, cent[3, 4]  # unsorted
    with pytest.raises(E.EccoError):
        E.ecco_model_create(c2, lens)
    l2 = lens.copy(); l2[0, 0] += 1                                     # Kraft sum < 1
    with pytest.raises(E.EccoError):
        E.ecco_model_create(cent, l2)
    c3 = cent.copy(); c3[0, 15] = 0x3E00                                # 1.5
    with pytest.raises(E.EccoError):
        E.ecco_model_create(c3, lens)
    c4 = cent.copy(); c4[0, 15] = 0x7C00                                # inf
    with pytest.raises(E.EccoError):
        E.ecco_model_create(c4, lens)
    assert E.ecco_model_create(cent, lens).S == 16


def test_argument_errors_without_gpu(tiny_model):
    w, m = tiny_model
    L = binding.lib()
    h = m.handle
    null = C.c_void_p(0)
    fake = C.c_void_p(0x1000)   # never dereferenced: the calls must fail before any launch
    out = C.c_void_p(0)
    a = w.view(np.uint16)
    assert L.ecco_fit_patterns(null, 128, 4, 12, 0, C.byref(out)) == -1
    assert L.ecco_fit_patterns(a.ctypes.data_as(C.c_void_p), 100, 4, 12, 0, C.byref(out)) == -2
    assert L.ecco_fit_patterns(a.ctypes.data_as(C.c_void_p), 1280, 65, 12, 0, C.byref(out)) == -1
    assert L.ecco_fit_patterns(a.ctypes.data_as(C.c_void_p), 1280, 4, 13, 0, C.byref(out)) == -1
    nan = np.full(128, 0x7E00, np.uint16)
    assert L.ecco_fit_patterns(nan.ctypes.data_as(C.c_void_p), 128, 1, 12, 0, C.byref(out)) == -1
    # model not on a device -> EINVAL for every GPU entry point
    assert L.ecco_decode(h, fake, fake, 1, fake, null) == -1
    assert L.ecco_encode(h, fake, 1, fake, fake, null) == -1
    assert L.ecco_decode_gemv(h, fake, fake, 1, 128, fake, 1, fake, null) == -1
    assert L.ecco_kv_append(h, h, fake, fake, fake, fake, fake, fake, fake, 1, 1, 1, null) == -1
    assert L.ecco_kv_attend(h, h, fake, fake, fake, fake, fake, fake, 1, 1, 1, fake, null) == -1
    assert L.ecco_decode(null, fake, fake, 1, fake, null) == -1
    assert L.ecco_decode(h, null, fake, 1, fake, null) == -1
    assert L.ecco_model_to_device(null, 0) == -1
    assert L.ecco_model_to_device(h, -1) == -1
    # sizes (ESHAPE) and alignment (EALIGN) are judged before the model's device, so they show without a GPU
    odd = C.c_void_p(0x1004)
    assert L.ecco_decode_gemv(h, fake, fake, 1, 100, fake, 1, fake, null) == -2      # cols % 128
    assert L.ecco_decode_gemv(h, fake, fake, 1, 128, fake, 17, fake, null) == -2     # batch
    assert L.ecco_decode_gemv(h, fake, fake, 0, 128, fake, 1, fake, null) == -2      # rows
    assert L.ecco_decode_gemv(h, fake, fake, 1, 65536 + 128, fake, 1, fake, null) == -2
    assert L.ecco_decode_gemv(h, odd, fake, 1, 128, fake, 1, fake, null) == -3       # blocks not 64-byte aligned
    assert L.ecco_decode_gemv(h, fake, fake, 1, 128, odd, 1, fake, null) == -3       # x not 16-byte aligned
    assert L.ecco_decode(h, odd, fake, 1, fake, null) == -3
    assert L.ecco_decode(h, fake, fake, 1, odd, null) == -3
    assert L.ecco_decode(h, fake, fake, 1 << 31, fake, null) == -2
    assert L.ecco_decode(h, null, null, 0, null, null) == -1                         # nothing to do, but no device either
    assert L.ecco_encode(h, fake, 1, odd, fake, null) == -3
    assert L.ecco_encode_minmax(h, fake, 1, odd, fake, null) == -3
    assert L.ecco_kv_append(h, h, fake, fake, fake, fake, fake, fake, fake, 0, 1, 1, null) == -2
    assert L.ecco_kv_append(h, h, fake, fake, odd, fake, fake, fake, fake, 1, 1, 1, null) == -3
    assert L.ecco_kv_append_minmax(h, h, fake, fake, fake, fake, fake, fake, fake, 1, 0, 1, null) == -2
    assert L.ecco_kv_attend(h, h, fake, fake, fake, fake, fake, fake, 1, 1, 0, fake, null) == -2
    assert L.ecco_kv_attend(h, h, odd, fake, fake, fake, fake, fake, 1, 1, 1, fake, null) == -3
    assert L.ecco_kv_attend(h, null, fake, fake, fake, fake, fake, fake, 1, 1, 1, fake, null) == -1
    gqa = lambda Hq, Hkv, splits, ws, q=fake: L.ecco_kv_attend_gqa(h, h, q, fake, fake, fake, fake, fake, 1, Hq, Hkv, 8, splits, ws, fake, null)
    assert gqa(6, 4, 1, null) == -2          # Hq % Hkv
    assert gqa(34, 2, 1, null) == -2         # more than 16 query heads per key/value head
    assert gqa(8, 2, 0, null) == -2 and gqa(8, 2, 257, fake) == -2
    assert gqa(8, 2, 2, null) == -1          # splits need a workspace
    assert gqa(8, 2, 2, odd) == -3
    assert gqa(8, 2, 1, null) == -1          # all fine up to the model, which is on no device
    assert L.ecco_kv_attend_gqa_workspace(2, 8, 3) == 2 * 8 * 3 * 130 * 4
    # split count: a workgroup per compute unit (an unknown device counts as 256), 256 tokens per split at least
    assert L.ecco_kv_attend_gqa_splits(-1, 8, 8, 4096) == 4
    assert L.ecco_kv_attend_gqa_splits(-1, 1, 32, 32768) == 8
    assert L.ecco_kv_attend_gqa_splits(-1, 64, 8, 4096) == 1
    assert L.ecco_kv_attend_gqa_splits(-1, 1, 4, 300) == 2
    assert L.ecco_kv_attend_gqa_splits(-1, 1, 1, 1 << 20) == 256
    assert L.ecco_kv_attend_gqa_splits(-1, 0, 4, 300) == -2
    # the activation codec and the streaming reference take no model: everything but the launch is host logic
    assert L.ecco_act_encode(null, 1, fake, null) == -1 and L.ecco_act_decode(fake, 1, null, null) == -1
    assert L.ecco_act_encode(fake, (1 << 40) + 1, fake, null) == -2
    assert L.ecco_act_encode(odd, 1, fake, null) == -3 and L.ecco_act_decode(odd, 1, fake, null) == -3
    assert L.ecco_act_encode(null, 0, null, null) == 0 and L.ecco_act_decode(null, 0, null, null) == 0
    assert L.ecco_read_stream(fake, 24, fake, null) == -2 and L.ecco_read_stream(odd, 32, fake, null) == -3
    assert L.ecco_read_stream(fake, 0, fake, null) == 0
    one = C.c_int(0)
    assert L.ecco_device_info(0, None, C.byref(one), C.byref(one)) == -1 and L.ecco_device_info(-1, C.byref(one), C.byref(one), C.byref(one)) == -1


def test_paper_block_argument_errors_without_gpu():
    w = W.config_weight("tiny")
    m = E.ecco_pb_fit(w, 4, 0)
    L = binding.lib()
    h = m.handle
    null, fake, odd = C.c_void_p(0), C.c_void_p(0x1000), C.c_void_p(0x1004)
    assert L.ecco_pb_decode(null, fake, 1, fake, null) == -1
    assert L.ecco_pb_decode(h, fake, 1, fake, null) == -1            # model on no device
    assert L.ecco_pb_decode(h, null, 1, fake, null) == -1
    assert L.ecco_pb_decode(h, fake, 1 << 31, fake, null) == -2
    assert L.ecco_pb_decode(h, odd, 1, fake, null) == -3 and L.ecco_pb_decode(h, fake, 1, odd, null) == -3
    assert L.ecco_pb_encode(h, fake, 1, odd, null) == -3
    assert L.ecco_pb_encode(h, fake, 1, fake, null) == -1
    assert L.ecco_pb_decode_gemv(h, fake, 1, 100, fake, fake, null) == -2
    assert L.ecco_pb_decode_gemv(h, fake, 0, 128, fake, fake, null) == -2
    assert L.ecco_pb_decode_gemv(h, fake, 1, 65536 + 128, fake, fake, null) == -2
    assert L.ecco_pb_decode_gemv(h, fake, 1, 128, odd, fake, null) == -3
    assert L.ecco_pb_decode_gemv(h, fake, 1, 128, fake, fake, null) == -1
    assert L.ecco_pb_model_to_device(null, 0) == -1


def test_paper_block_fit_invariants():
    """The CPU fit of the self-contained block format: a valid model (checked by the oracle's verifier), deterministic."""
    from oracle import paper_block as P
    w = W.config_weight("tiny")
    m = E.ecco_pb_fit(w, 16, 0)
    om = P.Model(m.centroids, m.code_lens, m.kp_lens, m.texp)
    assert P.verify_model(om) == 0
    assert m.S == 16 and -15 <= m.texp <= 7
    top = float(np.abs(w.astype(np.float32)).max())
    assert top / 2.0 ** m.texp <= 480 and (m.texp == -15 or top / 2.0 ** (m.texp - 1) > 480)   # the smallest power of two that fits
    lens = m.code_lens
    assert lens.min() >= 2 and lens.max() <= 8
    m2 = E.ecco_pb_fit(w, 16, 0)
    assert np.array_equal(m2.centroids, m.centroids) and np.array_equal(m2.code_lens, lens) and np.array_equal(m2.kp_lens, m.kp_lens)
    # the tables survive a trip through ecco_pb_model_create; bad tables are refused
    m3 = E.ecco_pb_model_create(m.centroids, lens, m.kp_lens, m.texp)
    assert np.array_equal(m3.centroids, m.centroids)
    blob = E.ecco_pb_model_save(m)
    assert len(blob) == 16 + 16 * (30 + 64 + 1) and blob[:4] == b"ECP0"
    m4 = E.ecco_pb_model_load(blob)
    assert (m4.S, m4.texp) == (m.S, m.texp) and np.array_equal(m4.code_lens, lens) and np.array_equal(m4.kp_lens, m.kp_lens)
    for broken in (blob[:-1], b"XXXX" + blob[4:], blob[:496] + b"\x00" + blob[497:]):  # short, bad magic, a code length of 0
        with pytest.raises(E.EccoError) as e:
            E.ecco_pb_model_load(broken)
        assert e.value.status == -5
    bad = lens.copy(); bad[0, 0, 0] = 1
    with pytest.raises(E.EccoError) as e:
        E.ecco_pb_model_create(m.centroids, bad, m.kp_lens, m.texp)
    assert e.value.status == -5
    with pytest.raises(E.EccoError) as e:
        E.ecco_pb_model_create(m.centroids, lens, m.kp_lens, 9)
    assert e.value.status == -5
    # codebooks compress: on the fit data nearly all values fit and some blocks have room for padded entries
    blocks = P.encode(om, w.view(np.uint16))
    dec, n_coded, n_out = P.decode(om, blocks)
    assert n_coded.mean() > 120 and (n_out > 0).mean() > 0.05


def test_build_rejects_register_spills(monkeypatch):
    """The build reads the compiler's resource remarks: scratch memory or spilled registers in any kernel stop it
    (scalar spills are tolerated in the one kernel that is known to have them)."""
    from paper_2505_06901_amd import build as B

    monkeypatch.delenv("ECCO_ALLOW_SCRATCH", raising=False)

    def remarks(name, scratch=0, sgpr=0, vgpr=0):
        pre = "x.hip:1:1: remark: "
        return "\n".join([pre + "Function Name: %s [-Rpass-analysis=kernel-resource-usage]" % name,
                          pre + "    TotalSGPRs: 60 [-Rpass-analysis=kernel-resource-usage]",
                          pre + "    ScratchSize [bytes/lane]: %d [-Rpass-analysis=kernel-resource-usage]" % scratch,
                          pre + "    SGPRs Spill: %d [-Rpass-analysis=kernel-resource-usage]" % sgpr,
                          pre + "    VGPRs Spill: %d [-Rpass-analysis=kernel-resource-usage]" % vgpr])

    B._check_kernel_resources(remarks("_Z11gemm_kernelILb0EEvv"), False)
    for bad in (dict(scratch=52), dict(sgpr=8), dict(vgpr=3)):
        with pytest.raises(RuntimeError, match="spills"):
            B._check_kernel_resources(remarks("_Z11gemm_kernelILb1EEvv", **bad), False)
    B._check_kernel_resources(remarks("_ZN12_GLOBAL__N_120kv_attend_gqa_kernelILb1ELb1EEEvv", sgpr=4), False)
    with pytest.raises(RuntimeError, match="spills"):
        B._check_kernel_resources(remarks("_ZN12_GLOBAL__N_120kv_attend_gqa_kernelILb1ELb1EEEvv", vgpr=1), False)
    with pytest.raises(RuntimeError, match="no kernel resource remarks"):
        B._check_kernel_resources("nothing here", False)


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: any other --gpus value ends with a message before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout)


def test_build_flags_a_64_bit_shift_by_the_last_allocated_register():
    """The build's check of generated code: a 64-bit shift whose amount is the last register of its kernel's allocation
    (next_free_vgpr rounded up to 8) is reported; the same shift by a lower register, by the top register of a kernel
    whose allocation is larger, and a 32-bit shift are not."""
    from paper_2505_06901_amd import build

    def kernel(name, body, n):
        return "\n".join(["\t.type\t%s,@function" % name, "%s:" % name, *["\t" + b for b in body], "\ts_endpgm",
                          "\t.amdhsa_kernel %s" % name, "\t\t.amdhsa_next_free_vgpr %d" % n, "\t.end_amdhsa_kernel"])

    asm = "\n".join([
        kernel("k_hit", ["v_lshlrev_b64 v[2:3], v119, v[4:5]", ".LBB0_1:", "v_ashrrev_i64 v[6:7], v119, v[6:7] ; comment v119"], 120),
        kernel("k_lower", ["v_lshlrev_b64 v[2:3], v118, v[4:5]", "v_lshlrev_b32_e32 v1, v119, v2", "v_add_u32_e32 v119, v1, v2"], 120),
        kernel("k_room", ["v_lshrrev_b64 v[2:3], v112, v[4:5]"], 113),       # allocation 120, last register v119 unused
        kernel("k_rounded", ["v_lshrrev_b64 v[2:3], v119, v[4:5]"], 118),    # would not assemble to 118, but the rule is the allocation's
    ])
    hits = build.last_register_shifts(asm)
    assert [h[0] for h in hits] == ["k_hit", "k_hit", "k_rounded"]
    assert hits[0][1].startswith("v_lshlrev_b64") and hits[1][1].startswith("v_ashrrev_i64")
