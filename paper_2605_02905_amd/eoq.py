"""ctypes binding of the C-ABI library (include/eoq.h).  Argument marshalling only:
every step of the path runs in the HIP kernels of libeoq.so.  PyTorch supplies device
memory and the current stream."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# EOQ_LIB_PATH names another build of the same library (e.g. the host-sanitizer build the README describes)
LIB_PATH = os.environ.get("EOQ_LIB_PATH") or os.path.join(_HERE, "libeoq.so")

EOQ_OK, EOQ_ERR_ARG, EOQ_ERR_UNSUPPORTED, EOQ_ERR_WORKSPACE, EOQ_ERR_HIP = range(5)
EOQ_F16, EOQ_F32 = 0, 1
EOQ_LOSS_FROBENIUS, EOQ_LOSS_OPERATOR, EOQ_LOSS_NUCLEAR = 0, 1, 2
FLAG_RANK_CLAMPED, FLAG_SHRINK_GUARD, FLAG_NO_CONVERGE, FLAG_NONFINITE = 1, 2, 4, 16

EXPORTS = ["eoq_create", "eoq_destroy", "eoq_pilot_k", "eoq_workspace_bytes", "eoq_rotation", "eoq_projection",
           "eoq_codebook", "eoq_qjl_encode", "eoq_scores_prod",
           "eoq_compress", "eoq_compress_static", "eoq_static_max_blocks", "eoq_compress_q4", "eoq_compress_chunk", "eoq_expand_factors", "eoq_decompress", "eoq_scores", "eoq_scores_stream", "eoq_softmax", "eoq_attend_workspace_bytes", "eoq_attend", "eoq_attend_stream", "eoq_set_solver", "eoq_set_loss", "eoq_profile", "eoq_stage_ms", "eoq_ceiling", "eoq_last_error"]


class EoqError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"eoq status {status}: {msg}")
        self.status = status


class _Packed(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("norms", C.c_void_p), ("rank", C.c_void_p), ("phi", C.c_void_p),
                ("sigma", C.c_void_p), ("lfac", C.c_void_p), ("rfac", C.c_void_p), ("flags", C.c_void_p)]


class _FactorCodes(C.Structure):
    _fields_ = [("lcodes", C.c_void_p), ("rcodes", C.c_void_p), ("fbook", C.c_void_p), ("phi16", C.c_void_p)]


class _Qjl(C.Structure):
    _fields_ = [("signs", C.c_void_p), ("norms", C.c_void_p)]


class ChunkLayout(C.Structure):
    """eoq_chunk_layout of include/eoq.h (strides in elements, record slots in blocks)."""
    _fields_ = [("in_group_stride", C.c_int64), ("in_group_size", C.c_int32), ("in_block_stride", C.c_int64),
                ("in_token_stride", C.c_int64), ("out_first", C.c_int64), ("out_stride", C.c_int64)]


_lib = None


def lib():
    """Load libeoq.so (built by `__graft_entry__.build()`); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        L.eoq_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int]
        L.eoq_create.restype = C.c_int
        L.eoq_destroy.argtypes = [C.c_void_p]
        L.eoq_destroy.restype = None
        L.eoq_pilot_k.argtypes = [C.c_int]
        L.eoq_pilot_k.restype = C.c_int
        L.eoq_workspace_bytes.argtypes = [C.c_void_p, C.c_int64]
        L.eoq_workspace_bytes.restype = C.c_size_t
        L.eoq_rotation.argtypes = [C.c_void_p, C.c_void_p]
        L.eoq_rotation.restype = C.c_int
        L.eoq_projection.argtypes = [C.c_void_p, C.c_void_p]
        L.eoq_projection.restype = C.c_int
        L.eoq_qjl_encode.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, _Packed, _Qjl, C.c_void_p]
        L.eoq_qjl_encode.restype = C.c_int
        L.eoq_scores_prod.argtypes = [C.c_void_p, _Packed, _Qjl, C.c_int64, C.c_int, C.c_int64, C.c_void_p, C.c_int,
                                      C.c_void_p, C.c_void_p]
        L.eoq_scores_prod.restype = C.c_int
        L.eoq_codebook.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.eoq_codebook.restype = C.c_int
        L.eoq_compress.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, _Packed, C.c_void_p, C.c_size_t,
                                   C.c_void_p]
        L.eoq_compress.restype = C.c_int
        L.eoq_compress_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, _Packed, C.c_void_p]
        L.eoq_compress_static.restype = C.c_int
        L.eoq_static_max_blocks.argtypes = [C.c_void_p]
        L.eoq_static_max_blocks.restype = C.c_int64
        L.eoq_compress_q4.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, _Packed, _FactorCodes, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
        L.eoq_compress_q4.restype = C.c_int
        L.eoq_compress_chunk.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, ChunkLayout, _Packed,
                                         C.POINTER(_FactorCodes), C.c_void_p, C.c_size_t, C.c_void_p]
        L.eoq_compress_chunk.restype = C.c_int
        L.eoq_expand_factors.argtypes = [C.c_void_p, _Packed, _FactorCodes, C.c_int64, C.c_void_p]
        L.eoq_expand_factors.restype = C.c_int
        L.eoq_decompress.argtypes = [C.c_void_p, _Packed, C.c_int64, C.c_void_p, C.c_void_p]
        L.eoq_decompress.restype = C.c_int
        L.eoq_scores.argtypes = [C.c_void_p, _Packed, C.c_int64, C.c_int, C.c_int64, C.c_void_p, C.c_int,
                                 C.c_void_p, C.c_void_p]
        L.eoq_scores.restype = C.c_int
        L.eoq_scores_stream.argtypes = [C.c_void_p, _Packed, C.c_int64, C.c_int, C.c_int64, C.c_int64, C.c_void_p,
                                        C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_void_p, C.c_int64, C.c_void_p]
        L.eoq_scores_stream.restype = C.c_int
        L.eoq_softmax.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p]
        L.eoq_softmax.restype = C.c_int
        L.eoq_attend_workspace_bytes.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int64]
        L.eoq_attend_workspace_bytes.restype = C.c_size_t
        L.eoq_attend.argtypes = [C.c_void_p, _Packed, C.c_int64, C.c_int, C.c_int64, C.c_int64, C.c_void_p, C.c_int64,
                                 C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.eoq_attend.restype = C.c_int
        L.eoq_attend_stream.argtypes = [C.c_void_p, _Packed, C.c_int64, C.c_int, C.c_int64, C.c_int64, C.c_void_p, C.c_int64,
                                        C.c_int64, C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t,
                                        C.c_void_p]
        L.eoq_attend_stream.restype = C.c_int
        L.eoq_set_solver.argtypes = [C.c_void_p, C.c_int]
        L.eoq_set_solver.restype = C.c_int
        L.eoq_set_loss.argtypes = [C.c_void_p, C.c_int]
        L.eoq_set_loss.restype = C.c_int
        L.eoq_profile.argtypes = [C.c_void_p, C.c_int]
        L.eoq_profile.restype = C.c_int
        L.eoq_stage_ms.argtypes = [C.c_void_p, C.c_void_p]
        L.eoq_stage_ms.restype = C.c_int
        L.eoq_ceiling.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        L.eoq_ceiling.restype = C.c_int
        L.eoq_last_error.argtypes = [C.c_void_p]
        L.eoq_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def eoq_pilot_k(d: int) -> int:
    return lib().eoq_pilot_k(d)


@dataclass
class Packed:
    """Device tensors of a compressed batch (layout: include/eoq.h, eoq_packed)."""
    codes: torch.Tensor   # uint8  [B, n, bits*d/8]
    norms: torch.Tensor   # int16  [B, n]  (binary16 bit patterns; .view(torch.float16) to read)
    rank: torch.Tensor    # int32  [B]
    phi: torch.Tensor     # float32 [B, r_max]
    sigma: torch.Tensor   # float32 [B, r_max]
    lfac: torch.Tensor    # float16 [B, r_max, n]
    rfac: torch.Tensor    # float16 [B, r_max, d]
    flags: torch.Tensor   # int32  [B]

    def c_struct(self) -> _Packed:
        return _Packed(*(t.data_ptr() for t in (self.codes, self.norms, self.rank, self.phi, self.sigma,
                                                 self.lfac, self.rfac, self.flags)))

    @staticmethod
    def empty(B: int, n: int, d: int, bits: int, r_max: int, device) -> "Packed":
        kw = dict(device=device)
        return Packed(torch.empty(B, n, bits * d // 8, dtype=torch.uint8, **kw),
                      torch.empty(B, n, dtype=torch.float16, **kw),
                      torch.empty(B, dtype=torch.int32, **kw),
                      torch.empty(B, r_max, dtype=torch.float32, **kw),
                      torch.empty(B, r_max, dtype=torch.float32, **kw),
                      torch.zeros(B, r_max, n, dtype=torch.float16, **kw),
                      torch.zeros(B, r_max, d, dtype=torch.float16, **kw),
                      torch.empty(B, dtype=torch.int32, **kw))

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in (self.codes, self.norms, self.rank, self.phi, self.sigma,
                                                          self.lfac, self.rfac, self.flags))


@dataclass
class FactorCodes:
    """Device tensors of the 4-bit SVD factors of a batch (layout: include/eoq.h, eoq_factor_codes)."""
    lcodes: torch.Tensor  # uint8   [B, r_max, n/2]
    rcodes: torch.Tensor  # uint8   [B, r_max, d/2]
    fbook: torch.Tensor   # float16 [B, 2, 8]
    phi16: torch.Tensor   # float16 [B, r_max]

    def c_struct(self) -> _FactorCodes:
        return _FactorCodes(*(t.data_ptr() for t in (self.lcodes, self.rcodes, self.fbook, self.phi16)))

    @staticmethod
    def empty(B: int, n: int, d: int, r_max: int, device) -> "FactorCodes":
        kw = dict(device=device)
        return FactorCodes(torch.zeros(B, r_max, n // 2, dtype=torch.uint8, **kw),
                           torch.zeros(B, r_max, d // 2, dtype=torch.uint8, **kw),
                           torch.zeros(B, 2, 8, dtype=torch.float16, **kw),
                           torch.zeros(B, r_max, dtype=torch.float16, **kw))

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in (self.lcodes, self.rcodes, self.fbook, self.phi16))


@dataclass
class Qjl:
    """Device tensors of the TQ_prod side information of a batch (layout: include/eoq.h, eoq_qjl)."""
    signs: torch.Tensor   # uint8   [B, n, d/8]
    norms: torch.Tensor   # float16 [B, n]

    def c_struct(self) -> _Qjl:
        return _Qjl(self.signs.data_ptr(), self.norms.data_ptr())

    @staticmethod
    def empty(B: int, n: int, d: int, device) -> "Qjl":
        return Qjl(torch.empty(B, n, d // 8, dtype=torch.uint8, device=device),
                   torch.empty(B, n, dtype=torch.float16, device=device))


def _stream_ptr(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


class Context:
    """eoq_create / eoq_destroy plus the calls that take the context."""

    def __init__(self, n: int, d: int = 128, bits: int = 2, rot_seed: int = 260502906, r_max: int = 32):
        self.n, self.d, self.bits, self.r_max, self.rot_seed = n, d, bits, r_max, rot_seed
        self._h = C.c_void_p()
        st = lib().eoq_create(C.byref(self._h), n, d, bits, rot_seed, r_max)
        if st != EOQ_OK:
            self._h = C.c_void_p()
            raise EoqError(st, "eoq_create failed")

    def close(self):
        if self._h:
            lib().eoq_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != EOQ_OK:
            raise EoqError(st, lib().eoq_last_error(self._h).decode())

    # -- tables ------------------------------------------------------------
    def eoq_rotation(self) -> np.ndarray:
        out = np.empty((self.d, self.d), dtype=np.float32)
        self._check(lib().eoq_rotation(self._h, out.ctypes.data))
        return out

    def eoq_projection(self) -> np.ndarray:
        out = np.empty((self.d, self.d), dtype=np.float32)
        self._check(lib().eoq_projection(self._h, out.ctypes.data))
        return out

    def eoq_codebook(self):
        cent = np.empty(1 << self.bits, dtype=np.float32)
        bnd = np.empty((1 << self.bits) - 1, dtype=np.float32)
        self._check(lib().eoq_codebook(self._h, cent.ctypes.data, bnd.ctypes.data))
        return cent, bnd

    def eoq_workspace_bytes(self, B: int) -> int:
        return lib().eoq_workspace_bytes(self._h, B)

    # -- hot calls ---------------------------------------------------------
    def eoq_compress(self, blocks: torch.Tensor, out: Packed | None = None, workspace: torch.Tensor | None = None):
        """blocks: device tensor [B, n, d], float16 or float32, contiguous.  Returns (Packed, workspace)."""
        assert blocks.is_cuda and blocks.is_contiguous() and blocks.shape[1:] == (self.n, self.d)
        B = blocks.shape[0]
        dtype = {torch.float16: EOQ_F16, torch.float32: EOQ_F32}[blocks.dtype]
        if out is None:
            out = Packed.empty(B, self.n, self.d, self.bits, self.r_max, blocks.device)
        need = self.eoq_workspace_bytes(B)
        if workspace is None:
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=blocks.device)
        self._check(lib().eoq_compress(self._h, blocks.data_ptr(), dtype, B, out.c_struct(), workspace.data_ptr(),
                                       workspace.numel(), _stream_ptr(blocks.device)))
        return out, workspace

    def eoq_static_max_blocks(self) -> int:
        return lib().eoq_static_max_blocks(self._h)

    def eoq_compress_static(self, blocks: torch.Tensor, out: Packed) -> Packed:
        """eoq_compress with the workspace inside the library (no allocation: `out` must be given)."""
        assert blocks.is_cuda and blocks.is_contiguous() and blocks.shape[1:] == (self.n, self.d)
        dtype = {torch.float16: EOQ_F16, torch.float32: EOQ_F32}[blocks.dtype]
        self._check(lib().eoq_compress_static(self._h, blocks.data_ptr(), dtype, blocks.shape[0], out.c_struct(),
                                              _stream_ptr(blocks.device)))
        return out

    def eoq_compress_q4(self, blocks: torch.Tensor, out: Packed | None = None, fq: FactorCodes | None = None,
                        workspace: torch.Tensor | None = None):
        """blocks: device tensor [B, n, d], float16, contiguous.  Returns (Packed, FactorCodes, workspace)."""
        assert blocks.is_cuda and blocks.is_contiguous() and blocks.shape[1:] == (self.n, self.d)
        B = blocks.shape[0]
        dtype = {torch.float16: EOQ_F16, torch.float32: EOQ_F32}[blocks.dtype]
        if out is None:
            out = Packed.empty(B, self.n, self.d, self.bits, self.r_max, blocks.device)
        if fq is None:
            fq = FactorCodes.empty(B, self.n, self.d, self.r_max, blocks.device)
        if workspace is None:
            workspace = torch.empty(max(self.eoq_workspace_bytes(B), 16), dtype=torch.uint8, device=blocks.device)
        self._check(lib().eoq_compress_q4(self._h, blocks.data_ptr(), dtype, B, out.c_struct(), fq.c_struct(),
                                          workspace.data_ptr(), workspace.numel(), _stream_ptr(blocks.device)))
        return out, fq, workspace

    def eoq_compress_chunk(self, chunk: torch.Tensor, B: int, layout: ChunkLayout, out: Packed,
                           fq: FactorCodes | None = None, workspace: torch.Tensor | None = None):
        """B blocks placed by `layout` inside the device tensor `chunk` (any shape, float16 or float32), written to
        the record slots `layout` names of the store `out` (and `fq`).  Returns the workspace."""
        assert chunk.is_cuda and chunk.is_contiguous()
        dtype = {torch.float16: EOQ_F16, torch.float32: EOQ_F32}[chunk.dtype]
        last = B - 1
        reach = ((last // layout.in_group_size) * layout.in_group_stride + (last % layout.in_group_size) * layout.in_block_stride
                 + (self.n - 1) * layout.in_token_stride + self.d)
        assert B == 0 or reach <= chunk.numel(), "layout reaches past the end of the chunk tensor"
        assert B == 0 or layout.out_first + last * layout.out_stride < out.rank.shape[0], "layout names a slot past the store"
        if workspace is None:
            workspace = torch.empty(max(self.eoq_workspace_bytes(B), 16), dtype=torch.uint8, device=chunk.device)
        fqs = fq.c_struct() if fq is not None else None
        self._check(lib().eoq_compress_chunk(self._h, chunk.data_ptr(), dtype, B, layout, out.c_struct(),
                                             C.byref(fqs) if fqs is not None else None, workspace.data_ptr(),
                                             workspace.numel(), _stream_ptr(chunk.device)))
        return workspace

    def eoq_expand_factors(self, rec: Packed, fq: FactorCodes):
        B = rec.rank.shape[0]
        self._check(lib().eoq_expand_factors(self._h, rec.c_struct(), fq.c_struct(), B,
                                             _stream_ptr(rec.codes.device)))
        return rec

    def eoq_decompress(self, rec: Packed, out: torch.Tensor | None = None) -> torch.Tensor:
        B = rec.rank.shape[0]
        if out is None:
            out = torch.empty(B, self.n, self.d, dtype=torch.float16, device=rec.codes.device)
        self._check(lib().eoq_decompress(self._h, rec.c_struct(), B, out.data_ptr(), _stream_ptr(out.device)))
        return out

    def eoq_scores(self, keys: Packed, q: torch.Tensor, n_kv_heads: int, out: torch.Tensor | None = None):
        """q: [n_seq, n_q_heads, d] float16 device.  Returns [n_seq, n_q_heads, blocks_per_head * n] float32."""
        assert q.is_cuda and q.is_contiguous() and q.dtype == torch.float16
        n_seq, n_q_heads, _ = q.shape
        B = keys.rank.shape[0]
        bph = B // (n_seq * n_kv_heads)
        assert bph * n_seq * n_kv_heads == B
        if out is None:
            out = torch.empty(n_seq, n_q_heads, bph * self.n, dtype=torch.float32, device=q.device)
        self._check(lib().eoq_scores(self._h, keys.c_struct(), n_seq, n_kv_heads, bph, q.data_ptr(), n_q_heads,
                                     out.data_ptr(), _stream_ptr(q.device)))
        return out

    def eoq_scores_stream(self, keys: Packed, q: torch.Tensor, n_kv_heads: int, block_capacity: int,
                          blocks_filled: int, tail: torch.Tensor | None, tail_len: int, out: torch.Tensor | None = None):
        """keys: store of [n_seq * n_kv_heads * block_capacity] slots; tail: [n_seq, n_kv_heads, tail_capacity, d]
        float16 device (or None).  Returns [n_seq, n_q_heads, score_stride] float32 with score_stride = out's last
        dimension (blocks_filled * n + tail_len when `out` is not given)."""
        assert q.is_cuda and q.is_contiguous() and q.dtype == torch.float16
        n_seq, n_q_heads, _ = q.shape
        assert keys.rank.shape[0] >= n_seq * n_kv_heads * block_capacity
        tail_cap = 0
        if tail is not None:
            assert tail.is_cuda and tail.is_contiguous() and tail.dtype == torch.float16
            assert tail.shape[0] == n_seq and tail.shape[1] == n_kv_heads and tail.shape[3] == self.d
            tail_cap = tail.shape[2]
        if out is None:
            out = torch.empty(n_seq, n_q_heads, blocks_filled * self.n + tail_len, dtype=torch.float32, device=q.device)
        assert out.is_contiguous() and out.shape[:2] == (n_seq, n_q_heads)
        self._check(lib().eoq_scores_stream(self._h, keys.c_struct(), n_seq, n_kv_heads, block_capacity, blocks_filled,
                                            tail.data_ptr() if tail is not None else None, tail_cap, tail_len,
                                            q.data_ptr(), n_q_heads, out.data_ptr(), out.shape[2],
                                            _stream_ptr(q.device)))
        return out

    def eoq_qjl_encode(self, blocks: torch.Tensor, rec: Packed, out: Qjl | None = None) -> Qjl:
        """blocks: the float16 device blocks `rec` was compressed from.  Returns the TQ_prod side information."""
        assert blocks.is_cuda and blocks.is_contiguous() and blocks.dtype == torch.float16
        assert blocks.shape[1:] == (self.n, self.d) and rec.rank.shape[0] == blocks.shape[0]
        B = blocks.shape[0]
        if out is None:
            out = Qjl.empty(B, self.n, self.d, blocks.device)
        self._check(lib().eoq_qjl_encode(self._h, blocks.data_ptr(), B, rec.c_struct(), out.c_struct(),
                                         _stream_ptr(blocks.device)))
        return out

    def eoq_scores_prod(self, keys: Packed, qjl: Qjl, q: torch.Tensor, n_kv_heads: int, out: torch.Tensor | None = None):
        assert q.is_cuda and q.is_contiguous() and q.dtype == torch.float16
        n_seq, n_q_heads, _ = q.shape
        B = keys.rank.shape[0]
        bph = B // (n_seq * n_kv_heads)
        assert bph * n_seq * n_kv_heads == B and qjl.norms.shape[0] == B
        if out is None:
            out = torch.empty(n_seq, n_q_heads, bph * self.n, dtype=torch.float32, device=q.device)
        self._check(lib().eoq_scores_prod(self._h, keys.c_struct(), qjl.c_struct(), n_seq, n_kv_heads, bph,
                                          q.data_ptr(), n_q_heads, out.data_ptr(), _stream_ptr(q.device)))
        return out

    def eoq_softmax(self, scores: torch.Tensor, length: int | None = None) -> torch.Tensor:
        """In-place softmax over the first `length` entries (default: all) of every row of a contiguous float32
        device tensor [..., row_stride]."""
        assert scores.is_cuda and scores.is_contiguous() and scores.dtype == torch.float32
        stride = scores.shape[-1]
        rows = scores.numel() // stride if stride else 0
        self._check(lib().eoq_softmax(self._h, scores.data_ptr(), rows, stride if length is None else length, stride,
                                      _stream_ptr(scores.device)))
        return scores

    def eoq_attend_workspace_bytes(self, n_seq: int, n_kv_heads: int, blocks_per_head: int) -> int:
        return lib().eoq_attend_workspace_bytes(self._h, n_seq, n_kv_heads, blocks_per_head)

    def eoq_attend(self, values: Packed, weights: torch.Tensor, n_kv_heads: int, block_capacity: int | None = None,
                   blocks_filled: int | None = None, out: torch.Tensor | None = None,
                   workspace: torch.Tensor | None = None) -> torch.Tensor:
        """weights: [n_seq, n_q_heads, weight_stride] float32 device.  Returns [n_seq, n_q_heads, d] float32."""
        assert weights.is_cuda and weights.is_contiguous() and weights.dtype == torch.float32
        n_seq, n_q_heads, stride = weights.shape
        if block_capacity is None:
            block_capacity = values.rank.shape[0] // (n_seq * n_kv_heads)
        if blocks_filled is None:
            blocks_filled = block_capacity
        assert values.rank.shape[0] >= n_seq * n_kv_heads * block_capacity
        if out is None:
            out = torch.empty(n_seq, n_q_heads, self.d, dtype=torch.float32, device=weights.device)
        need = self.eoq_attend_workspace_bytes(n_seq, n_kv_heads, blocks_filled)
        if workspace is None:
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=weights.device)
        self._check(lib().eoq_attend(self._h, values.c_struct(), n_seq, n_kv_heads, block_capacity, blocks_filled,
                                     weights.data_ptr(), stride, n_q_heads, out.data_ptr(), workspace.data_ptr(),
                                     workspace.numel(), _stream_ptr(weights.device)))
        return out

    def eoq_attend_stream(self, values: Packed, weights: torch.Tensor, n_kv_heads: int, block_capacity: int,
                          blocks_filled: int, tail: torch.Tensor | None, tail_len: int, out: torch.Tensor | None = None,
                          workspace: torch.Tensor | None = None) -> torch.Tensor:
        """eoq_attend plus the float16 tail values [n_seq, n_kv_heads, tail_capacity, d] (weights behind the blocks')."""
        assert weights.is_cuda and weights.is_contiguous() and weights.dtype == torch.float32
        n_seq, n_q_heads, stride = weights.shape
        assert values.rank.shape[0] >= n_seq * n_kv_heads * block_capacity
        tail_cap = 0
        if tail is not None:
            assert tail.is_cuda and tail.is_contiguous() and tail.dtype == torch.float16
            assert tail.shape[0] == n_seq and tail.shape[1] == n_kv_heads and tail.shape[3] == self.d
            tail_cap = tail.shape[2]
        if out is None:
            out = torch.empty(n_seq, n_q_heads, self.d, dtype=torch.float32, device=weights.device)
        if workspace is None:
            need = self.eoq_attend_workspace_bytes(n_seq, n_kv_heads, blocks_filled)
            workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=weights.device)
        self._check(lib().eoq_attend_stream(self._h, values.c_struct(), n_seq, n_kv_heads, block_capacity, blocks_filled,
                                            tail.data_ptr() if tail is not None else None, tail_cap, tail_len,
                                            weights.data_ptr(), stride, n_q_heads, out.data_ptr(), workspace.data_ptr(),
                                            workspace.numel(), _stream_ptr(weights.device)))
        return out

    def eoq_set_solver(self, solver: int):
        self._check(lib().eoq_set_solver(self._h, solver))

    def eoq_set_loss(self, loss: int):
        """EOQ_LOSS_FROBENIUS (0), EOQ_LOSS_OPERATOR (1) or EOQ_LOSS_NUCLEAR (2)."""
        self._check(lib().eoq_set_loss(self._h, loss))

    def eoq_profile(self, enable: bool = True):
        self._check(lib().eoq_profile(self._h, 1 if enable else 0))

    def eoq_stage_ms(self) -> dict:
        out = (C.c_float * 6)()
        self._check(lib().eoq_stage_ms(self._h, out))
        return dict(zip(("spectral", "encode", "decode", "scores", "attend", "softmax"), (float(x) for x in out)))

    def eoq_ceiling(self, kind: int, buf: torch.Tensor, iters: int = 1) -> dict:
        """One micro-benchmark of include/eoq.h's eoq_ceiling on the device buffer `buf` (uint8)."""
        assert buf.is_cuda and buf.is_contiguous()
        out = (C.c_double * 4)()
        self._check(lib().eoq_ceiling(self._h, kind, buf.data_ptr(), buf.numel() * buf.element_size(), iters, out))
        return {"ms": out[0], "work_a": out[1], "work_b": out[2], "compute_units": int(out[3])}

    def spectrum(self, workspace: torch.Tensor, B: int) -> torch.Tensor:
        """Gram eigenvalues [B, d] (float64) that eoq_compress leaves at the head of its workspace."""
        return workspace[: B * self.d * 8].view(torch.float64).view(B, self.d)
