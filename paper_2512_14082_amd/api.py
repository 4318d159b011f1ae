"""Thin Python binding over ``libunisparse.so`` (ctypes; argument marshalling only).

Every function has the name and meaning of the C entry point it calls (see
``include/unisparse.h``); all arithmetic of the hot path runs in the HIP kernels.  PyTorch is
used for device memory and the current stream, nothing else.  There is no CPU fallback: if the
library has not been built, or no MI355X is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libunisparse.so")

TOP_P = 0
TOP_K = 1
HEAD_DIM = 128

EXPORTS = [
    "unisparse_create", "unisparse_destroy", "unisparse_status_string", "unisparse_mask_row_words",
    "unisparse_mask_words", "unisparse_score_elems", "unisparse_workspace_bytes", "unisparse_workspace_bytes_min",
    "unisparse_avgpool_seq",
    "unisparse_pool_seq_varlen",
    "unisparse_build_mask", "unisparse_build_mask_static", "unisparse_select_blocks", "unisparse_sparse_attn",
    "unisparse_sparse_attn_ws", "unisparse_attn_workspace_bytes", "unisparse_full_attn",
    "unisparse_attn",
]


class UnisparseError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"unisparse status {code}: {msg}")
        self.code = code


class _Problem(ctypes.Structure):
    _fields_ = [("num_seqs", ctypes.c_int32), ("cu_seqlens", ctypes.POINTER(ctypes.c_int32)),
                ("n_heads_q", ctypes.c_int32), ("n_heads_kv", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("causal", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class _Tensor(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("stride_tok", ctypes.c_int64), ("stride_head", ctypes.c_int64)]


class _Select(ctypes.Structure):
    _fields_ = [("c_q", ctypes.c_int32), ("c_k", ctypes.c_int32), ("c_h", ctypes.c_int32), ("mode", ctypes.c_int32),
                ("threshold", ctypes.c_double), ("budget_frac", ctypes.c_double), ("pool", ctypes.c_int32),
                ("proxy_tiles", ctypes.c_int32), ("query_pool_pass", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("rand_q", ctypes.c_void_p), ("rand_k", ctypes.c_void_p)]


_lib = None


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    """dlopen the HIP library and declare the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not built: run `python -m paper_2512_14082_amd.build`")
    lib = ctypes.CDLL(path)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    PP, SP = ctypes.POINTER(_Problem), ctypes.POINTER(_Select)
    lib.unisparse_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.unisparse_create.restype = ctypes.c_int
    lib.unisparse_destroy.argtypes = [vp]
    lib.unisparse_destroy.restype = None
    lib.unisparse_status_string.argtypes = [ctypes.c_int]
    lib.unisparse_status_string.restype = ctypes.c_char_p
    for name in ("unisparse_mask_row_words", "unisparse_mask_words", "unisparse_attn_workspace_bytes"):
        getattr(lib, name).argtypes = [PP]
        getattr(lib, name).restype = sz
    for name in ("unisparse_score_elems", "unisparse_workspace_bytes", "unisparse_workspace_bytes_min"):
        getattr(lib, name).argtypes = [PP, SP]
        getattr(lib, name).restype = sz
    lib.unisparse_avgpool_seq.argtypes = [vp, _Tensor, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, vp, vp]
    lib.unisparse_avgpool_seq.restype = ctypes.c_int
    lib.unisparse_pool_seq_varlen.argtypes = [vp, PP, _Tensor, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp]
    lib.unisparse_pool_seq_varlen.restype = ctypes.c_int
    lib.unisparse_build_mask.argtypes = [vp, PP, SP, _Tensor, _Tensor, vp, sz, vp, vp, vp]
    lib.unisparse_build_mask.restype = ctypes.c_int
    lib.unisparse_build_mask_static.argtypes = [vp, PP, SP, _Tensor, _Tensor, vp, vp]
    lib.unisparse_build_mask_static.restype = ctypes.c_int
    lib.unisparse_select_blocks.argtypes = [vp, PP, SP, vp, vp, vp]
    lib.unisparse_select_blocks.restype = ctypes.c_int
    lib.unisparse_sparse_attn.argtypes = [vp, PP, _Tensor, _Tensor, _Tensor, vp, _Tensor, vp, vp]
    lib.unisparse_sparse_attn.restype = ctypes.c_int
    lib.unisparse_sparse_attn_ws.argtypes = [vp, PP, _Tensor, _Tensor, _Tensor, vp, _Tensor, vp, vp, sz, vp]
    lib.unisparse_sparse_attn_ws.restype = ctypes.c_int
    lib.unisparse_full_attn.argtypes = [vp, PP, _Tensor, _Tensor, _Tensor, _Tensor, vp, vp]
    lib.unisparse_full_attn.restype = ctypes.c_int
    lib.unisparse_attn.argtypes = [vp, PP, SP, _Tensor, _Tensor, _Tensor, vp, sz, vp, _Tensor, vp, vp]
    lib.unisparse_attn.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(code: int):
    if code != 0:
        raise UnisparseError(code, load_library().unisparse_status_string(code).decode())


@dataclass
class Problem:
    """Geometry of a packed batch (``unisparse_problem``)."""
    cu_seqlens: Sequence[int]
    n_heads_q: int
    n_heads_kv: int
    block_size: int
    causal: bool
    softmax_scale: float = 0.0
    head_dim: int = HEAD_DIM

    def __post_init__(self):
        self._cu = (ctypes.c_int32 * len(self.cu_seqlens))(*[int(x) for x in self.cu_seqlens])
        self._c = _Problem(len(self.cu_seqlens) - 1, ctypes.cast(self._cu, ctypes.POINTER(ctypes.c_int32)),
                           self.n_heads_q, self.n_heads_kv, self.head_dim, self.block_size, int(self.causal),
                           float(self.softmax_scale))

    @property
    def c(self):
        return ctypes.byref(self._c)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def n_rows(self) -> int:
        return sum(-(-(int(self.cu_seqlens[b + 1]) - int(self.cu_seqlens[b])) // self.block_size)
                   for b in range(len(self.cu_seqlens) - 1))

    @property
    def n_cols(self) -> int:
        return -(-max(int(self.cu_seqlens[b + 1]) - int(self.cu_seqlens[b])
                      for b in range(len(self.cu_seqlens) - 1)) // self.block_size)


@dataclass
class Select:
    """Selection parameters (``unisparse_select``)."""
    c_q: int = 8
    c_k: int = 8
    c_h: int = 1
    mode: int = TOP_P
    threshold: float = 0.9
    budget_frac: float = 0.25
    pool: int = 0          # 0 = average pooling (Eq. (1)), 1 = max pooling, 2 = stochastic pooling
    rand_q: Optional[torch.Tensor] = None   # stochastic pooling: float32 device uniforms [H, composite queries]
    rand_k: Optional[torch.Tensor] = None   # and [H_kv, composite keys]
    proxy_tiles: int = 0   # tuning of the score kernel: 0 = automatic, 1 / 2 = 32-row tiles per wavefront
    query_pool_pass: int = 0   # tuning: 0 = queries pooled inside the score kernel where possible, 1 = in their own pass

    @property
    def c(self):
        self._c = _Select(self.c_q, self.c_k, self.c_h, self.mode, float(self.threshold), float(self.budget_frac),
                          self.pool, self.proxy_tiles, self.query_pool_pass, 0, _rand_ptr(self.rand_q),
                          _rand_ptr(self.rand_k))
        return ctypes.byref(self._c)


def _rand_ptr(r: Optional[torch.Tensor]):
    if r is None:
        return None
    if not r.is_cuda or r.dtype != torch.float32 or not r.is_contiguous():
        raise ValueError("expected a contiguous float32 device tensor of uniform numbers")
    return r.data_ptr()


def _view(t: torch.Tensor, layout: str) -> _Tensor:
    """[T, H, d] ("thd") or [H, T, d] ("htd") bf16 CUDA tensor -> unisparse_tensor."""
    if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 3 or t.stride(2) != 1:
        raise ValueError("expected a bf16 device tensor with contiguous last dimension")
    if layout == "thd":
        return _Tensor(t.data_ptr(), t.stride(0), t.stride(1))
    if layout == "htd":
        return _Tensor(t.data_ptr(), t.stride(1), t.stride(0))
    raise ValueError("layout must be 'thd' or 'htd'")


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """Owns a ``unisparse_ctx``.  All launches go to torch's current stream."""

    def __init__(self, device: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("unisparse needs an MI355X; no HIP device is visible")
        self.lib = load_library()
        self.handle = ctypes.c_void_p()
        self.device = device
        _check(self.lib.unisparse_create(ctypes.byref(self.handle), device))

    def close(self):
        if self.handle:
            self.lib.unisparse_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- sizes ---------------------------------------------------------------------------------
    def mask_row_words(self, p: Problem) -> int:
        return int(self.lib.unisparse_mask_row_words(p.c))

    def mask_words(self, p: Problem) -> int:
        return int(self.lib.unisparse_mask_words(p.c))

    def score_elems(self, p: Problem, s: Select) -> int:
        return int(self.lib.unisparse_score_elems(p.c, s.c))

    def workspace_bytes(self, p: Problem, s: Select) -> int:
        return int(self.lib.unisparse_workspace_bytes(p.c, s.c))

    def alloc_mask(self, p: Problem) -> torch.Tensor:
        return torch.zeros((p.n_heads_q, p.n_rows, max(1, self.mask_row_words(p))), dtype=torch.int64,
                           device=f"cuda:{self.device}")

    def workspace_bytes_min(self, p: Problem, s: Select) -> int:
        return int(self.lib.unisparse_workspace_bytes_min(p.c, s.c))

    def alloc_workspace(self, p: Problem, s: Select, minimal: bool = False) -> torch.Tensor:
        """Workspace of build_mask: the size that lets it compute the scores in one sweep, or (minimal) the least
        it accepts."""
        n = self.workspace_bytes_min(p, s) if minimal else self.workspace_bytes(p, s)
        return torch.empty(max(256, n), dtype=torch.uint8, device=f"cuda:{self.device}")

    # ---- entry points --------------------------------------------------------------------------
    def avgpool_seq(self, x: torch.Tensor, c: int, layout: str = "htd") -> torch.Tensor:
        T = x.shape[0] if layout == "thd" else x.shape[1]
        H = x.shape[1] if layout == "thd" else x.shape[0]
        out = torch.empty((H, T // c, HEAD_DIM), dtype=torch.bfloat16, device=x.device)
        _check(self.lib.unisparse_avgpool_seq(self.handle, _view(x, layout), H, T, c, out.data_ptr(), _stream()))
        return out

    def pool_seq_varlen(self, p: Problem, x: torch.Tensor, c: int, layout: str = "htd", pool: int = 0,
                        rand: Optional[torch.Tensor] = None) -> torch.Tensor:
        H = x.shape[1] if layout == "thd" else x.shape[0]
        n_out = sum(-(-(int(p.cu_seqlens[b + 1]) - int(p.cu_seqlens[b])) // c) for b in range(len(p.cu_seqlens) - 1))
        out = torch.empty((H, n_out, p.head_dim), dtype=torch.bfloat16, device=x.device)
        _check(self.lib.unisparse_pool_seq_varlen(self.handle, p.c, _view(x, layout), H, c, pool, _rand_ptr(rand),
                                                  out.data_ptr(), _stream()))
        return out

    def build_mask(self, p: Problem, s: Select, q: torch.Tensor, k: torch.Tensor, layout: str = "htd",
                   workspace: Optional[torch.Tensor] = None, mask: Optional[torch.Tensor] = None,
                   want_score: bool = False) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
        ws = workspace if workspace is not None else self.alloc_workspace(p, s)
        m = mask if mask is not None else self.alloc_mask(p)
        score = None
        sp = None
        if want_score:
            score = torch.empty((p.n_heads_q // s.c_h, p.n_rows, max(1, p.n_cols)), dtype=torch.float32,
                                device=q.device)
            sp = score.data_ptr()
        _check(self.lib.unisparse_build_mask(self.handle, p.c, s.c, _view(q, layout), _view(k, layout),
                                             ws.data_ptr(), ws.numel(), m.data_ptr(), sp, _stream()))
        return m, score

    def build_mask_static(self, p: Problem, s: Select, q: torch.Tensor, k: torch.Tensor, mask: torch.Tensor,
                          layout: str = "htd") -> torch.Tensor:
        """``unisparse_build_mask_static``: the mask into the caller's ``mask``; nothing is allocated."""
        _check(self.lib.unisparse_build_mask_static(self.handle, p.c, s.c, _view(q, layout), _view(k, layout),
                                                    mask.data_ptr(), _stream()))
        return mask

    def tune(self, p: Problem, s: Select, q: torch.Tensor, k: torch.Tensor, layout: str = "htd", reps: int = 3) -> Select:
        """Time ``build_mask`` with each tiling of the score kernel this problem admits (``proxy_tiles`` 1 and 2) and
        set the faster one in ``s`` (the library's own choice, ``proxy_tiles = 0``, is a fixed rule).  Both tilings
        compute identical masks; only the launch shape differs.  Synchronises the device."""
        ws, m = self.alloc_workspace(p, s), self.alloc_mask(p)
        best, best_ms = 0, float("inf")
        for tiles in (2, 1):
            if tiles == 1 and (p.head_dim != 128 or p.block_size // s.c_q > 32):
                continue
            s.proxy_tiles = tiles
            self.build_mask(p, s, q, k, layout, workspace=ws, mask=m)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                self.build_mask(p, s, q, k, layout, workspace=ws, mask=m)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            if ms < best_ms:
                best, best_ms = tiles, ms
        s.proxy_tiles = best
        return s

    def select_blocks(self, p: Problem, s: Select, score: torch.Tensor, mask: Optional[torch.Tensor] = None):
        m = mask if mask is not None else self.alloc_mask(p)
        _check(self.lib.unisparse_select_blocks(self.handle, p.c, s.c, score.data_ptr(), m.data_ptr(), _stream()))
        return m

    def attn_workspace_bytes(self, p: Problem) -> int:
        return int(self.lib.unisparse_attn_workspace_bytes(p.c))

    def sparse_attn(self, p: Problem, q, k, v, mask: torch.Tensor, layout: str = "htd",
                    out: Optional[torch.Tensor] = None, want_lse: bool = False,
                    workspace: Optional[torch.Tensor] = None):
        """``unisparse_sparse_attn``, or ``unisparse_sparse_attn_ws`` when a workspace tensor (uint8, device) is given."""
        o = out if out is not None else torch.empty_like(q)
        lse = torch.empty((p.n_heads_q, p.total_tokens), dtype=torch.float32, device=q.device) if want_lse else None
        if workspace is None:
            _check(self.lib.unisparse_sparse_attn(self.handle, p.c, _view(q, layout), _view(k, layout), _view(v, layout),
                                                  mask.data_ptr(), _view(o, layout),
                                                  lse.data_ptr() if want_lse else None, _stream()))
        else:
            _check(self.lib.unisparse_sparse_attn_ws(self.handle, p.c, _view(q, layout), _view(k, layout),
                                                     _view(v, layout), mask.data_ptr(), _view(o, layout),
                                                     lse.data_ptr() if want_lse else None, workspace.data_ptr(),
                                                     workspace.numel(), _stream()))
        return o, lse

    def full_attn(self, p: Problem, q, k, v, layout: str = "htd", out: Optional[torch.Tensor] = None,
                  want_lse: bool = False):
        o = out if out is not None else torch.empty_like(q)
        lse = torch.empty((p.n_heads_q, p.total_tokens), dtype=torch.float32, device=q.device) if want_lse else None
        _check(self.lib.unisparse_full_attn(self.handle, p.c, _view(q, layout), _view(k, layout), _view(v, layout),
                                            _view(o, layout), lse.data_ptr() if want_lse else None, _stream()))
        return o, lse

    def attn(self, p: Problem, s: Select, q, k, v, layout: str = "htd", workspace=None, mask=None, out=None):
        ws = workspace if workspace is not None else self.alloc_workspace(p, s)
        m = mask if mask is not None else self.alloc_mask(p)
        o = out if out is not None else torch.empty_like(q)
        _check(self.lib.unisparse_attn(self.handle, p.c, s.c, _view(q, layout), _view(k, layout), _view(v, layout),
                                       ws.data_ptr(), ws.numel(), m.data_ptr(), _view(o, layout), None, _stream()))
        return o, m


# ---- host-side helpers for tests and reports (format conversion only) ------------------------------

def bits_to_device(bits, device="cuda:0") -> torch.Tensor:
    """uint16 bf16 bit patterns (numpy) -> bf16 device tensor of the same shape."""
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def unpack_mask(mask_words: torch.Tensor, n_cols: int):
    """int64 [H, NQ, W] device/host tensor -> numpy uint8 [H, NQ, n_cols]."""
    import numpy as np
    w = mask_words.detach().cpu().numpy().view(np.uint64)
    H, NQ, W = w.shape
    bits = np.unpackbits(w.view(np.uint8).reshape(H, NQ, W * 8), axis=-1, bitorder="little")
    return np.ascontiguousarray(bits[..., :n_cols])


def pack_mask(mask_u8, device="cuda:0") -> torch.Tensor:
    """numpy uint8 [H, NQ, NK] -> int64 device tensor [H, NQ, ceil(NK / 64)]."""
    import numpy as np
    H, NQ, NK = mask_u8.shape
    W = max(1, (NK + 63) // 64)
    padded = np.zeros((H, NQ, W * 64), dtype=np.uint8)
    padded[..., :NK] = mask_u8
    words = np.packbits(padded, axis=-1, bitorder="little").view(np.uint64).reshape(H, NQ, W)
    return torch.from_numpy(words.view(np.int64).copy()).to(device)
