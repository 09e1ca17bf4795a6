"""Helpers shared by the GPU parity tests: run the CPU oracle over blocks (process pool) and
move records between the oracle's per-block form and the library's batched device layout."""
from __future__ import annotations

import math
import multiprocessing
import os
from concurrent.futures import ProcessPoolExecutor

import numpy as np

import oracle

ROT_SEED = 260502906
_CACHE = {}


def oracle_tables(bits: int, d: int = 128, seed: int = ROT_SEED):
    key = (bits, d, seed)
    if key not in _CACHE:
        Pi = oracle.haar_rotation(d, seed).astype(np.float32).astype(np.float64)   # the stored float32 table
        _CACHE[key] = (Pi, oracle.lloyd_max_gaussian(bits))
    return _CACHE[key]


def _init_worker():
    # one BLAS thread per worker: the pool is the parallelism
    for var in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
        os.environ[var] = "1"
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except Exception:
        pass


def _one(args):
    S, bits, r_max, seed, factor_bits, loss = args
    Pi, cb = oracle_tables(bits, S.shape[1], seed)
    rec = oracle.compress_block(S, Pi, cb, r_max, factor_bits=factor_bits, loss=loss)
    # what the quantiser compared with the boundaries (Alg. 1 line 5, in the float32 of the stored table): kept so
    # that a code the GPU decides differently can be checked to sit on a decision boundary
    rec.t32 = (rec.z * math.sqrt(S.shape[1])).astype(np.float32)
    rec.R = None
    rec.z = None
    return rec


def oracle_compress(blocks: np.ndarray, bits: int, r_max: int = 32, seed: int = ROT_SEED, workers: int | None = None,
                    factor_bits: int = 16, loss: str = "frobenius"):
    """blocks: [B, n, d] float64 (exactly the values handed to the GPU). Returns a list of BlockRecord."""
    jobs = [(blocks[b], bits, r_max, seed, factor_bits, loss) for b in range(blocks.shape[0])]
    workers = workers or min(8, os.cpu_count() or 1)
    if len(jobs) <= 2 or workers == 1:
        return [_one(j) for j in jobs]
    # spawn, not fork: the parent may already hold a HIP context, which a forked child cannot use or inherit safely
    with ProcessPoolExecutor(workers, mp_context=multiprocessing.get_context("spawn"), initializer=_init_worker) as ex:
        return list(ex.map(_one, jobs, chunksize=max(1, len(jobs) // (4 * workers))))


def records_to_packed(recs, r_max: int, device):
    """Oracle records -> the library's device layout (eoq.Packed)."""
    import torch
    from paper_2605_02905_amd import eoq
    B, n, d, bits = len(recs), recs[0].n, recs[0].d, recs[0].bits
    codes = np.stack([oracle.pack_codes(r.codes, bits) for r in recs])
    norms = np.stack([oracle.fp16_bits(r.rho16) for r in recs]).view(np.float16)
    rank = np.array([r.rank for r in recs], dtype=np.int32)
    phi = np.zeros((B, r_max), dtype=np.float32)
    sigma = np.zeros((B, r_max), dtype=np.float32)
    lfac = np.zeros((B, r_max, n), dtype=np.float16)
    rfac = np.zeros((B, r_max, d), dtype=np.float16)
    for b, r in enumerate(recs):
        phi[b, :r.rank] = r.phi
        sigma[b, :r.rank] = r.sigma
        lfac[b, :r.rank] = r.lfac
        rfac[b, :r.rank] = r.rfac
    t = lambda a: torch.from_numpy(a).to(device)
    return eoq.Packed(t(codes), t(norms), t(rank), t(phi), t(sigma), t(lfac), t(rfac),
                      torch.zeros(B, dtype=torch.int32, device=device))


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.linalg.norm(a - b) / np.linalg.norm(a))


# A code index may differ from the oracle's only where the rotated coordinate sits on a cell boundary: the GPU rotates
# the row in binary16 (relative rounding 2^-11 per entry: 2.8e-4 rms on z sqrt(d), whose scale is 1) against the oracle's
# float64, and the two residuals differ by the binary16 rounding of the stored factors.  Seven standard deviations:
BOUNDARY_MARGIN = 2e-3


def compare_compress(blocks64: np.ndarray, rec, lam_gpu: np.ndarray, recs, bits: int, r_max: int = 32,
                     lowrank_tol: float = 5e-3, boundary_margin: float = BOUNDARY_MARGIN):
    """Parity of eoq_compress against oracle records.  Returns a dict of statistics; asserts the bars:
    ranks bit-exact, eigenvalues within 1e-9 of the largest (the retained ones and the next within 1e-12), shrunk values within
    1e-3 relative, code mismatches <= 0.1 % of entries, every mismatch an adjacent index whose coordinate lies within
    `boundary_margin` (in units of the N(0,1) table) of the boundary between the two cells."""
    B, n, d = blocks64.shape
    rank_g = rec.rank.cpu().numpy()
    rank_o = np.array([r.rank for r in recs])
    assert np.array_equal(rank_g, rank_o), f"rank mismatch at blocks {np.nonzero(rank_g != rank_o)[0][:10]}: " \
        f"gpu {rank_g[rank_g != rank_o][:10]} oracle {rank_o[rank_g != rank_o][:10]}"
    flags = rec.flags.cpu().numpy()
    flags_o = np.array([r.flags for r in recs])
    assert np.array_equal(flags & 3, flags_o & 3)
    stats_sweeps = (flags >> 8) & 0xFF
    assert not np.any(flags & 4), "eigensolver hit its sweep limit"
    phi_g = rec.phi.cpu().numpy().astype(np.float64)
    sig_g = rec.sigma.cpu().numpy().astype(np.float64)
    codes_g = rec.codes.cpu().numpy()
    norms_g = rec.norms.cpu().numpy().astype(np.float64)
    lfac_g = rec.lfac.cpu().numpy().astype(np.float64)
    rfac_g = rec.rfac.cpu().numpy().astype(np.float64)
    bounds64 = oracle_tables(bits, d)[1].bounds_f32.astype(np.float64)
    stats = dict(max_phi_rel=0.0, max_sigma_rel=0.0, max_lam_rel=0.0, max_lam_top_rel=0.0, mismatches=0, entries=0, max_lowrank_abs=0.0,
                 max_code_step=0, max_boundary_dist=0.0,
                 norm_ulp_diffs=0, max_sweeps=int(stats_sweeps.max()), mean_sweeps=float(stats_sweeps.mean()))
    for b, r in enumerate(recs):
        lam_o = r.lam
        stats["max_lam_rel"] = max(stats["max_lam_rel"], float(np.max(np.abs(lam_gpu[b] - lam_o)) / lam_o[0]) if lam_o[0] > 0 else 0.0)
        # the retained eigenvalues and the first one below them feed the shrinker, the eigenvector solves and the
        # test for repeated eigenvalues
        top = min(r.rank + 1, len(lam_o))
        stats["max_lam_top_rel"] = max(stats["max_lam_top_rel"],
                                       float(np.max(np.abs(lam_gpu[b][:top] - lam_o[:top])) / lam_o[0]) if lam_o[0] > 0 else 0.0)
        if r.rank:
            stats["max_phi_rel"] = max(stats["max_phi_rel"], float(np.max(np.abs(phi_g[b, :r.rank] - r.phi) / np.maximum(r.phi, 1e-300))))
            stats["max_sigma_rel"] = max(stats["max_sigma_rel"], float(np.max(np.abs(sig_g[b, :r.rank] - r.sigma) / r.sigma)))
            # eigenvector signs are arbitrary: compare the product of the stored factors
            lo_g = lfac_g[b, :r.rank].T @ rfac_g[b, :r.rank]
            lo_o = r.lfac.T @ r.rfac
            stats["max_lowrank_abs"] = max(stats["max_lowrank_abs"], float(np.max(np.abs(lo_g - lo_o)) / np.max(np.abs(lo_o))))
        cg = oracle.unpack_codes(codes_g[b], bits, d)
        diff = cg != r.codes
        stats["mismatches"] += int(np.count_nonzero(diff))
        stats["entries"] += n * d
        if diff.any():
            go, oo = cg[diff].astype(np.int64), r.codes[diff].astype(np.int64)
            stats["max_code_step"] = max(stats["max_code_step"], int(np.max(np.abs(go - oo))))
            # cells c and c + 1 meet at boundary number c
            dist = np.abs(r.t32[diff].astype(np.float64) - bounds64[np.minimum(np.minimum(go, oo), len(bounds64) - 1)])
            stats["max_boundary_dist"] = max(stats["max_boundary_dist"], float(dist.max()))
        # stored norms: binary16 of the same real number up to the kernel's float32 rounding
        dn = np.abs(norms_g[b] - r.rho16)
        stats["norm_ulp_diffs"] += int(np.count_nonzero(dn > 0))
        assert np.all(dn <= 2e-3 * np.maximum(r.rho16, 1e-30) + 1e-7), b
    assert stats["max_lam_rel"] <= 1e-9, stats
    assert stats["max_lam_top_rel"] <= 1e-12, stats
    assert stats["max_phi_rel"] <= 1e-3, stats
    assert stats["max_sigma_rel"] <= 1e-3, stats
    assert stats["mismatches"] <= 1e-3 * stats["entries"], stats
    assert stats["max_code_step"] <= 1, stats
    assert stats["max_boundary_dist"] <= boundary_margin, stats
    assert stats["max_lowrank_abs"] <= lowrank_tol, stats
    return stats


def log_stats(name: str, stats: dict):
    """Append parity statistics to parity_stats.jsonl in the run-output folder at the repository root, if present."""
    import json
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = os.path.join(root, "gpurun_out")
    if os.path.isdir(out):
        with open(os.path.join(out, "parity_stats.jsonl"), "a") as fh:
            fh.write(json.dumps({"case": name, **{k: (float(v) if isinstance(v, (float, np.floating)) else int(v))
                                                  for k, v in stats.items()}}) + "\n")


def compare_factor_codes(rec, fq, recs):
    """4-bit factors of eoq_compress_q4 against oracle records made with factor_bits = 4.  The sign of a singular
    vector is arbitrary: per component the sign is taken from the two decoded right vectors and the sign bits of
    that component are compared after that flip; magnitude indices are compared as they are.  Asserts codebooks
    and phi16 within one binary16 unit, code mismatches <= 0.1 % of the factor entries, and that the record's
    lfac / rfac are exactly what the device's own codes expand to.  Returns statistics."""
    lc = rec_np(fq.lcodes)
    rc = rec_np(fq.rcodes)
    book = rec_np(fq.fbook).astype(np.float64)
    phi16 = rec_np(fq.phi16).astype(np.float64)
    lfac = rec_np(rec.lfac)
    rfac = rec_np(rec.rfac)
    st = dict(entries=0, mismatches=0, book_levels=0, book_exact=0, phi_exact=0, comps=0)
    for b, r in enumerate(recs):
        k = r.rank
        if k == 0:
            assert not np.any(book[b])
            continue
        n, d = r.n, r.d
        lcg = oracle.unpack_nibbles(lc[b, :k])          # [k, n]
        rcg = oracle.unpack_nibbles(rc[b, :k])          # [k, d]
        # the record's factors are exactly the expansion of the device's own codes
        assert np.array_equal(oracle.fp16_round(oracle.factor_decode(lcg, book[b, 0]) * phi16[b, :k, None]).astype(np.float16),
                              lfac[b, :k]), b
        assert np.array_equal(oracle.factor_decode(rcg, book[b, 1]).astype(np.float16), rfac[b, :k]), b
        # codebooks and phi16: binary16 of the same real numbers up to float32 rounding of the inputs
        ulp = np.spacing(np.abs(r.fbook).astype(np.float16)).astype(np.float64)
        assert np.all(np.abs(book[b] - r.fbook) <= ulp), (b, book[b], r.fbook)
        assert np.all(np.diff(book[b], axis=1) > 0)
        st["book_levels"] += 16
        st["book_exact"] += int(np.count_nonzero(book[b] == r.fbook))
        assert np.all(np.abs(phi16[b, :k] - r.phi16) <= np.spacing(r.phi16.astype(np.float16)).astype(np.float64)), b
        st["phi_exact"] += int(np.count_nonzero(phi16[b, :k] == r.phi16))
        st["comps"] += k
        sgn = np.sign(np.sum(rfac[b, :k].astype(np.float64) * r.rfac, axis=1))
        assert np.all(sgn != 0)
        flip = np.where(sgn < 0, 8, 0).astype(np.uint8)[:, None]
        st["mismatches"] += int(np.count_nonzero((lcg ^ flip) != r.lcodes)) + int(np.count_nonzero((rcg ^ flip) != r.rcodes))
        st["entries"] += k * (n + d)
    assert st["mismatches"] <= 1e-3 * max(st["entries"], 1), st
    return st


def rec_np(t):
    return t.detach().cpu().numpy()


def packed_to_records(rec, idx, bits: int):
    """Blocks `idx` of a device record (eoq.Packed) as oracle BlockRecords, field for field: what a reader of the
    stored record sees."""
    out = []
    rank = rec_np(rec.rank)
    for b in idx:
        k = int(rank[b])
        n, d = rec.norms.shape[1], rec.rfac.shape[2]
        out.append(oracle.BlockRecord(
            n, d, bits, k, 0, rec_np(rec.phi[b, :k]).astype(np.float64), rec_np(rec.sigma[b, :k]).astype(np.float64),
            rec_np(rec.lfac[b, :k]).astype(np.float64), rec_np(rec.rfac[b, :k]).astype(np.float64),
            oracle.unpack_codes(rec_np(rec.codes[b]), bits, d), rec_np(rec.norms[b]).astype(np.float64)))
    return out
