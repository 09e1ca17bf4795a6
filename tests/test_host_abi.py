"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, builds the same
tables as the oracle, and rejects bad arguments without a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_02905_amd import eoq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(eoq.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return eoq.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "eoq.h")).read()
    declared = set(re.findall(r"\b(eoq_[a-z_0-9]+)\s*\(", header))
    assert declared == set(eoq.EXPORTS), declared ^ set(eoq.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_pilot_k(lib):
    assert eoq.eoq_pilot_k(128) == 11 == oracle.pilot_k(128)
    assert eoq.eoq_pilot_k(64) == 7 == oracle.pilot_k(64)
    for d in (16, 32, 96, 256, 1024):
        assert eoq.eoq_pilot_k(d) == oracle.pilot_k(d)


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_codebook_bit_exact_with_oracle(lib, bits):
    ctx = eoq.Context(n=512, bits=bits)
    cent, bnd = ctx.eoq_codebook()
    cb = oracle.lloyd_max_gaussian(bits)
    assert np.array_equal(cent, cb.centroids_f32)
    assert np.array_equal(bnd, cb.bounds_f32)


@pytest.mark.parametrize("seed", [260502906, 1, 2 ** 63 + 12345])
def test_rotation_matches_oracle_and_is_orthogonal(lib, seed):
    ctx = eoq.Context(n=512, bits=2, rot_seed=seed)
    P = ctx.eoq_rotation()
    Po = oracle.haar_rotation(128, seed)
    assert np.max(np.abs(P.astype(np.float64) - Po)) <= 2.0 ** -24      # at most one float32 ulp of entries < 1
    assert np.mean(P == Po.astype(np.float32)) > 0.999
    P64 = P.astype(np.float64)
    assert np.max(np.abs(P64.T @ P64 - np.eye(128))) <= 1e-6


def test_unsupported_shapes_are_rejected(lib):
    h = C.c_void_p()
    for n, d, bits, r_max in [(512, 64, 2, 32), (100, 128, 2, 32), (512, 128, 5, 32), (512, 128, 0, 32),
                              (512, 128, 2, 0), (512, 128, 2, 33), (8192, 128, 2, 32), (64, 128, 2, 8)]:
        assert lib.eoq_create(C.byref(h), n, d, bits, 1, r_max) == eoq.EOQ_ERR_UNSUPPORTED
        assert not h
    assert lib.eoq_create(None, 512, 128, 2, 1, 32) == eoq.EOQ_ERR_ARG


def test_workspace_size_and_host_only_context(lib):
    ctx = eoq.Context(n=512, bits=2, r_max=32)
    assert ctx.eoq_workspace_bytes(0) == 16
    assert ctx.eoq_workspace_bytes(10) == 10 * (128 * 8 + 32 * 128 * 4) + 16 + 48 + 64 + 10 * 128 * 16
    assert lib.eoq_last_error(ctx._h) == b""
    assert lib.eoq_rotation(ctx._h, None) == eoq.EOQ_ERR_ARG
    import torch
    if not torch.cuda.is_available():
        # no device: the hot calls fail with a status, they do not crash
        st = lib.eoq_decompress(ctx._h, eoq._Packed(), 1, None, None)
        assert st == eoq.EOQ_ERR_HIP
        assert b"HIP device" in lib.eoq_last_error(ctx._h)


def test_projection_table_matches_the_oracle_stream():
    """Phi of TQ_prod: the library's own generator (seed rot_seed + 1) against the oracle's, as binary16 tables."""
    ctx = eoq.Context(n=128, bits=2, rot_seed=77)
    got = ctx.eoq_projection()
    want = oracle.gaussian_projection(128, 78).astype(np.float16).astype(np.float32)
    assert got.shape == (128, 128) and np.array_equal(got, got.astype(np.float16).astype(np.float32))
    assert np.count_nonzero(got != want) <= 2     # a libm difference in the last bit can only show at a rounding boundary
