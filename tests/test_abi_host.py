"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, rejects bad
arguments before touching a device, and its host packer round-trips every bit width."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2512_17073_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2512_17073_amd import build
        build.build(verbose=False)
    return binding.lib()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "moe_lrc.h")).read()
    declared = set(re.findall(r"\b(moe_lrc_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def _cfg(**kw):
    base = dict(hidden=256, ffn=512, n_experts=8, n_shared=0, top_k=2, top_n=1, bits=3, shared_bits=4,
                group=64, rank=8, renormalize=0, max_tokens=16, residency=0)
    base.update(kw)
    return binding.Config(*[base[n] for n, _ in binding.Config._fields_])


@pytest.mark.parametrize("kw,code", [
    (dict(bits=5), -1), (dict(bits=1), -1), (dict(top_n=3), -1), (dict(top_k=0), -1), (dict(top_k=9), -1),
    (dict(rank=12), -1), (dict(rank=1032), -1), (dict(n_experts=0), -1), (dict(n_experts=300), -1),
    (dict(max_tokens=0), -1), (dict(residency=3), -1), (dict(renormalize=2), -1), (dict(n_shared=9), -1),
    (dict(n_shared=1, shared_bits=7), -1),
    (dict(group=32), -2), (dict(hidden=200), -2), (dict(ffn=500), -2), (dict(group=128, hidden=320), -2),
    (dict(hidden=16448), -2), (dict(ffn=65600), -2),
])
def test_config_errors_before_any_device_work(lib, kw, code):
    h = C.c_void_p()
    cfg = _cfg(**kw)
    rc = lib.moe_lrc_layer_create(C.byref(cfg), C.byref(h))
    assert rc == code, (kw, rc, binding.last_error())
    assert not h.value
    assert binding.last_error()


def test_null_arguments(lib):
    h = C.c_void_p()
    assert lib.moe_lrc_layer_create(None, C.byref(h)) == -1
    assert lib.moe_lrc_layer_create(C.byref(_cfg()), None) == -1
    assert lib.moe_lrc_layer_destroy(None) == 0
    assert lib.moe_lrc_set_gate(None, None, None) == -1
    assert lib.moe_lrc_set_expert(None, 0, 0, None, None, None, None, None) == -1
    assert lib.moe_lrc_route(None, None, 1, None, None, None) == -1
    assert lib.moe_lrc_permute(None, None, 1, None, None, None, None, None, None) == -1
    assert lib.moe_lrc_expert_ffn(None, None, 1, None, None, None, None, 0, None) == -1
    assert lib.moe_lrc_combine(None, None, None, None, None, 1, None, None, 0, None) == -1
    assert lib.moe_lrc_forward(None, None, 1, None, None, 0, None) == -1
    assert lib.moe_lrc_debug_unpack(None, 0, 0, None, None) == -1
    assert lib.moe_lrc_get_stats(None, None) == -1
    assert lib.moe_lrc_workspace_bytes(None, 4) == 0
    assert lib.moe_lrc_pack_codes(2, 64, 16, None, None) == -1


def test_stack_offline_and_hook_argument_errors_need_no_device(lib):
    # every one of these is refused on its arguments, before any device call
    h = C.c_void_p()
    one = (C.c_void_p * 1)(None)
    assert lib.moe_lrc_stack_create(None, 1, 8, 0, C.byref(h)) == -1
    assert lib.moe_lrc_stack_create(one, 1, 8, 0, None) == -1
    assert lib.moe_lrc_stack_create(one, 0, 8, 0, C.byref(h)) == -1          # no layers
    assert lib.moe_lrc_stack_create(one, 1, 8, 4, C.byref(h)) == -1          # unknown flag
    assert not h.value
    assert lib.moe_lrc_stack_destroy(None) == 0
    assert lib.moe_lrc_stack_step(None, None, 1, None, None, None) == -1
    assert lib.moe_lrc_stack_get_stats(None, None) == -1
    assert lib.moe_lrc_stack_reset(None) == -1
    assert lib.moe_lrc_forward_noalloc(None, None, 1, None, None) == -1
    assert lib.moe_lrc_offline_quantize(None, 64, 16, 2, 64, None, None, None, None, None) == -1
    dummy = C.c_void_p(256)                                                  # never dereferenced: shape errors come first
    assert lib.moe_lrc_offline_quantize(dummy, 64, 16, 5, 64, dummy, dummy, dummy, None, None) == -1     # bits
    assert lib.moe_lrc_offline_quantize(dummy, 100, 16, 2, 64, dummy, dummy, dummy, None, None) == -2    # K not a multiple of group
    qr = lib.moe_lrc_offline_quantize_refined
    assert qr(None, 64, 16, 2, 64, 20, 0.7, 10.0, 1.01, None, None, None, None, None) == -1
    assert qr(dummy, 64, 16, 2, 64, -1, 0.7, 10.0, 1.01, dummy, dummy, dummy, None, None) == -1         # steps
    assert qr(dummy, 64, 16, 2, 64, 20, 1.5, 10.0, 1.01, dummy, dummy, dummy, None, None) == -1         # p
    assert qr(dummy, 64, 16, 2, 64, 20, 0.7, 0.0, 1.01, dummy, dummy, dummy, None, None) == -1          # beta
    assert qr(dummy, 64, 16, 2, 64, 20, 0.7, 10.0, 0.5, dummy, dummy, dummy, None, None) == -1          # kappa
    assert qr(dummy, 100, 16, 2, 64, 20, 0.7, 10.0, 1.01, dummy, dummy, dummy, None, None) == -2        # K not a multiple of group
    assert lib.moe_lrc_offline_factors(None, 64, 64, 8, None, 16, 2, None, None, None, None, None) == -1
    assert lib.moe_lrc_offline_factors(dummy, 64, 64, 8, dummy, 4, 2, dummy, dummy, None, None, None) == -2   # sketch narrower than the rank
    assert lib.moe_lrc_offline_factors(dummy, 64, 64, 8, dummy, 80, 2, dummy, dummy, None, None, None) == -2  # sketch wider than the matrix
    assert lib.moe_lrc_offline_factors(dummy, 64, 64, 8, dummy, 16, 9, dummy, dummy, None, None, None) == -1  # power iterations
    assert lib.moe_lrc_offline_kurtosis(None, 10, None) == -1
    k = C.c_double()
    assert lib.moe_lrc_offline_kurtosis(dummy, 0, C.byref(k)) == -1
    assert lib.moe_lrc_calibrate(9, 1 << 20, 1, C.byref(k)) == -1            # unknown kind
    assert lib.moe_lrc_calibrate(4, 3, 1, C.byref(k)) == -1                  # FMAs per MFMA not in {0, 2, 4, 8, 16}
    assert lib.moe_lrc_calibrate(5, 3, 1, C.byref(k)) == -1                  # sub-step: row tiles not 1 or 2
    assert lib.moe_lrc_calibrate(0, 1 << 20, 0, C.byref(k)) == -1            # reps
    assert lib.moe_lrc_selftest_half_rounding(None, 1, None) == -1
    assert binding.last_error()


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_roundtrip_exhaustive_block(lib, bits):
    # one packing block is 256 x 16: put every code value at every lane-local position
    K, N = 256, 16
    levels = 1 << bits
    for shift in range(levels):
        codes = ((np.arange(K)[:, None] * 7 + np.arange(N)[None, :] * 3 + shift) % levels).astype(np.uint8)
        packed = binding.pack_codes(bits, codes)
        assert packed.size == K * N * bits // 8          # dense: exactly `bits` per weight
        np.testing.assert_array_equal(binding.unpack_codes(bits, K, N, packed), codes)
    # single-code impulses: each position maps to its own bits and nothing else
    for pos in range(0, K, 5):
        codes = np.zeros((K, N), np.uint8)
        codes[pos, pos % N] = levels - 1
        packed = binding.pack_codes(bits, codes)
        assert int(np.unpackbits(packed).sum()) == bits
        np.testing.assert_array_equal(binding.unpack_codes(bits, K, N, packed), codes)


@pytest.mark.parametrize("bits,K,N", [(2, 1408, 64), (3, 768, 48), (4, 320, 32), (3, 64, 16)])
def test_pack_roundtrip_random_and_ragged_k(lib, bits, K, N):
    rng = np.random.default_rng(bits * 1000 + K)
    codes = rng.integers(0, 1 << bits, size=(K, N), dtype=np.uint8)
    packed = binding.pack_codes(bits, codes)
    kp = (K + 255) // 256 * 256
    assert packed.size == kp * N * bits // 8
    np.testing.assert_array_equal(binding.unpack_codes(bits, K, N, packed), codes)


def test_pack_rejects_out_of_range_codes(lib):
    codes = np.full((256, 16), 4, np.uint8)
    with pytest.raises(binding.MoeLrcError) as ei:
        binding.pack_codes(2, codes)
    assert ei.value.code == -1
    with pytest.raises(binding.MoeLrcError):
        binding.pack_codes(2, np.zeros((256, 10), np.uint8))     # N not a multiple of 16


def test_bench_refuses_more_than_one_gpu():
    # this build runs on one GPU: bench.py says so and exits before touching a device
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
