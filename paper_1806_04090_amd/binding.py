"""Thin ctypes binding over libatomo.so (the C ABI declared in include/atomo.h).

Argument marshalling only: every step of the method runs in the HIP kernels behind the C ABI.
PyTorch is used for device memory (tensors) and streams.  There is no CPU fallback: importing this
module without a built library, or calling it without a GPU, raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ATOMO_LIB: load this build of the library instead (the host-sanitizer build of build.py, for instance)
LIB_PATH = os.environ.get("ATOMO_LIB") or os.path.join(_HERE, "libatomo.so")

ATOMO_OK, ATOMO_EINVAL, ATOMO_ECAPACITY, ATOMO_ENOCONV, ATOMO_EHIP, ATOMO_ENOMEM, ATOMO_ETOOLARGE = 0, -1, -2, -3, -4, -5, -6
ATOMO_KIND_SVD, ATOMO_KIND_ENTRYWISE, ATOMO_KIND_LQ = 0, 1, 2


class AtomoError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} (status {status})")


class atomo_mat(C.Structure):
    _fields_ = [("rows", C.c_int32), ("cols", C.c_int32), ("ld", C.c_int64), ("data", C.c_void_p)]


class atomo_svd_msg(C.Structure):
    _fields_ = [("rows", C.c_int32), ("cols", C.c_int32), ("capacity", C.c_int32), ("count", C.c_void_p),
                ("idx", C.c_void_p), ("w", C.c_void_p), ("U", C.c_void_p), ("V", C.c_void_p)]


class atomo_ew_msg(C.Structure):
    _fields_ = [("n", C.c_int64), ("capacity", C.c_int64), ("count", C.c_void_p), ("idx", C.c_void_p),
                ("val", C.c_void_p)]


class atomo_lq_msg(C.Structure):
    _fields_ = [("n", C.c_int64), ("capacity", C.c_int64), ("count", C.c_void_p), ("idx", C.c_void_p),
                ("norm", C.c_void_p)]


class atomo_svd_options(C.Structure):
    _fields_ = [("max_sweeps", C.c_int32), ("stop_cosine", C.c_float), ("max_inner_sweeps", C.c_int32),
                ("inner_reduction", C.c_float), ("full_period", C.c_int32), ("block_order", C.c_int32),
                ("stream_ids", C.POINTER(C.c_uint64)), ("adaptive", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """The loaded C-ABI library; raises if it has not been built (python -m paper_1806_04090_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1806_04090_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.atomo_create.argtypes = [C.POINTER(vp), C.c_int]
        L.atomo_destroy.argtypes = [vp]
        L.atomo_reserve.argtypes = [vp, C.c_size_t]
        L.atomo_svd_workspace_bytes.argtypes = [C.POINTER(atomo_mat), C.c_int, C.POINTER(C.c_size_t)]
        L.atomo_entrywise_workspace_bytes.argtypes = [C.c_int64, C.POINTER(C.c_size_t)]
        L.atomo_status.argtypes = [vp, vp, C.POINTER(C.c_int32)]
        L.atomo_last_hip_error.argtypes = [vp]
        L.atomo_strerror.argtypes = [C.c_int]
        L.atomo_strerror.restype = C.c_char_p
        L.atomo_probabilities.argtypes = [vp, vp, C.POINTER(C.c_int64), C.c_int, C.c_double, vp, vp]
        L.atomo_encode_svd.argtypes = [vp, C.POINTER(atomo_mat), C.c_int, C.c_double, C.c_uint64, C.c_uint64,
                                       C.POINTER(atomo_svd_options), C.POINTER(atomo_svd_msg), vp, vp, vp]
        L.atomo_encode_entrywise.argtypes = [vp, vp, C.c_double, C.c_uint64, C.c_uint64, C.POINTER(atomo_ew_msg),
                                             vp, vp]
        L.atomo_encode_entrywise_noalloc.argtypes = L.atomo_encode_entrywise.argtypes
        L.atomo_encode_lq.argtypes = [vp, vp, C.c_double, C.c_uint64, C.c_uint64, C.POINTER(atomo_lq_msg), vp, vp]
        L.atomo_decode.argtypes = [vp, C.c_int, vp, C.c_int, C.c_float, vp, C.c_int64, vp]
        L.atomo_decode_svd_batch.argtypes = [vp, C.POINTER(atomo_svd_msg), C.POINTER(C.c_int32), C.c_int, C.c_float,
                                             C.POINTER(vp), C.POINTER(C.c_int64), vp]
        L.atomo_apply_svd_batch.argtypes = L.atomo_decode_svd_batch.argtypes
        L.atomo_svd_sweeps.argtypes = [vp, vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int]
        L.atomo_last_counters.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.atomo_measure_mfma_fp32.argtypes = [vp, C.POINTER(C.c_double), vp]
        L.atomo_profile_enable.argtypes = [vp, C.c_int]
        L.atomo_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        for name in ("atomo_last_counters", "atomo_svd_sweeps", "atomo_profile_enable", "atomo_profile_read", "atomo_create", "atomo_destroy", "atomo_reserve", "atomo_svd_workspace_bytes",
                     "atomo_entrywise_workspace_bytes", "atomo_status", "atomo_last_hip_error", "atomo_probabilities",
                     "atomo_encode_svd", "atomo_encode_entrywise", "atomo_encode_entrywise_noalloc", "atomo_encode_lq", "atomo_decode",
                     "atomo_decode_svd_batch", "atomo_apply_svd_batch", "atomo_measure_mfma_fp32"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().atomo_strerror(status).decode()


def _check(status: int, what: str):
    if status != ATOMO_OK:
        raise AtomoError(status, what)


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> int:
    st = torch.cuda.current_stream() if stream is None else stream
    return int(st.cuda_stream)


def _f32_cuda(t: torch.Tensor, what: str) -> torch.Tensor:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32):
        raise TypeError(f"{what} must be a float32 CUDA tensor")
    return t


# ------------------------------------------------------------------------------------- messages

@dataclass
class SvdMessage:
    """Kept singular triplets of one matrix; buffers are device tensors owned by this object."""
    rows: int
    cols: int
    capacity: int
    count: torch.Tensor   # int32 [1]
    idx: torch.Tensor     # int32 [capacity]
    w: Optional[torch.Tensor]   # float32 [capacity]; None: folded form, U holds (sigma / p) u
    U: torch.Tensor       # float32 [capacity, rows]
    V: torch.Tensor       # float32 [capacity, cols]

    def c_struct(self) -> atomo_svd_msg:
        """The C descriptor, built once (the buffers of a message are not replaced after allocation)."""
        c = self.__dict__.get("_c")
        if c is None:
            c = atomo_svd_msg(self.rows, self.cols, self.capacity, self.count.data_ptr(), self.idx.data_ptr(),
                              None if self.w is None else self.w.data_ptr(), self.U.data_ptr(), self.V.data_ptr())
            self.__dict__["_c"] = c
        return c

    def to_host(self) -> dict:
        k = min(int(self.count.item()), self.capacity)
        return {"count": int(self.count.item()), "idx": self.idx[:k].cpu().numpy(),
                "w": None if self.w is None else self.w[:k].cpu().numpy(),
                "U": self.U[:k].cpu().numpy().T.copy(), "V": self.V[:k].cpu().numpy().T.copy()}


@dataclass
class EntrywiseMessage:
    n: int
    capacity: int
    count: torch.Tensor   # int64 [1]
    idx: torch.Tensor     # uint32 stored as int32 bits [capacity]
    val: torch.Tensor     # float32 [capacity]

    def c_struct(self) -> atomo_ew_msg:
        return atomo_ew_msg(self.n, self.capacity, self.count.data_ptr(), self.idx.data_ptr(), self.val.data_ptr())

    def to_host(self) -> dict:
        k = min(int(self.count.item()), self.capacity)
        return {"count": int(self.count.item()), "idx": self.idx[:k].cpu().numpy().view("uint32").astype("int64"),
                "val": self.val[:k].cpu().numpy()}


@dataclass
class LqMessage:
    """One l_q-quantised gradient: kept coordinates (sign in bit 31 of the index) and the shared magnitude."""
    n: int
    capacity: int
    count: torch.Tensor   # int64 [1]
    idx: torch.Tensor     # uint32 stored as int32 bits [capacity]
    norm: torch.Tensor    # float32 [1]

    def c_struct(self) -> atomo_lq_msg:
        return atomo_lq_msg(self.n, self.capacity, self.count.data_ptr(), self.idx.data_ptr(), self.norm.data_ptr())

    def to_host(self) -> dict:
        k = min(int(self.count.item()), self.capacity)
        words = self.idx[:k].cpu().numpy().view("uint32")
        return {"count": int(self.count.item()), "idx": (words & 0x7FFFFFFF).astype("int64"),
                "sign": np.where(words >> 31, -1, 1).astype("int8"), "norm": float(self.norm.item())}


def default_capacity(s: float, n_atoms: int) -> int:
    """Room for the expected s kept atoms plus a wide margin (the count is Poisson-binomial with mean <= s)."""
    return int(min(n_atoms, math.ceil(s) + 8 * math.ceil(math.sqrt(s)) + 8))


def alloc_svd_message(rows: int, cols: int, capacity: int, device, folded: bool = False) -> SvdMessage:
    """folded: no weight array; the encoder writes (sigma / p) u into U (rows + cols reals per atom)."""
    return SvdMessage(rows, cols, capacity,
                      torch.zeros(1, dtype=torch.int32, device=device),
                      torch.zeros(capacity, dtype=torch.int32, device=device),
                      None if folded else torch.zeros(capacity, dtype=torch.float32, device=device),
                      torch.zeros(capacity, rows, dtype=torch.float32, device=device),
                      torch.zeros(capacity, cols, dtype=torch.float32, device=device))


def alloc_entrywise_message(n: int, capacity: int, device) -> EntrywiseMessage:
    return EntrywiseMessage(n, capacity,
                            torch.zeros(1, dtype=torch.int64, device=device),
                            torch.zeros(capacity, dtype=torch.int32, device=device),
                            torch.zeros(capacity, dtype=torch.float32, device=device))


def alloc_lq_message(n: int, capacity: int, device) -> LqMessage:
    return LqMessage(n, capacity,
                     torch.zeros(1, dtype=torch.int64, device=device),
                     torch.zeros(capacity, dtype=torch.int32, device=device),
                     torch.zeros(1, dtype=torch.float32, device=device))


def lq_capacity(n: int, q: float) -> int:
    """Room for an l_q message of a length-n gradient: the budget |g|_1 / |g|_q is at most n^(1 - 1/q) for
    q >= 1 (Hoelder), n otherwise, plus a margin for the spread of the count."""
    s = float(n) if (q < 1.0 or math.isinf(q)) else float(n) ** (1.0 - 1.0 / q)
    return default_capacity(s, n)


# -------------------------------------------------------------------------------------- context

class Context:
    """Owns an atomo_ctx (device workspace, latched device flags) on one GPU."""

    def __init__(self, device: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("libatomo needs a GPU: no HIP device is visible and there is no CPU fallback")
        self.device = torch.device("cuda", device)
        self._h = C.c_void_p()
        _check(lib().atomo_create(C.byref(self._h), device), "atomo_create")

    def close(self):
        if self._h:
            lib().atomo_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reserve(self, nbytes: int):
        _check(lib().atomo_reserve(self._h, nbytes), "atomo_reserve")

    KERNEL_CLASSES = ("svd_prepare", "svd_gram", "svd_eig", "svd_update", "svd_refresh", "svd_finalize", "decode_svd",
                      "ew_hist", "ew_solve", "ew_sample", "ew_decode", "svd_thin")

    def measure_mfma_fp32(self) -> float:
        """TFLOP/s of a loop of fp32 matrix-core instructions on this GPU (blocks for about a millisecond)."""
        out = C.c_double(0.0)
        _check(lib().atomo_measure_mfma_fp32(self._h, C.byref(out), _stream_handle(None)), "atomo_measure_mfma_fp32")
        return out.value

    def profile_enable(self, enable: bool):
        _check(lib().atomo_profile_enable(self._h, 1 if enable else 0), "atomo_profile_enable")

    def profile_read(self) -> dict:
        """{kernel class: (total GPU ms, bracketed launches)} since the last read (HIP events)."""
        n = len(self.KERNEL_CLASSES)
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        _check(lib().atomo_profile_read(self._h, ms, cnt), "atomo_profile_read")
        return {name: (ms[i], cnt[i]) for i, name in enumerate(self.KERNEL_CLASSES)}

    def last_counters(self):
        """(block-pair eigenproblems solved, Jacobi steps of 32 rotations taken, 64 x 64 tiles rotated by the row
        updates of the data-space matrices) as of the last status() call."""
        a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        _check(lib().atomo_last_counters(self._h, C.byref(a), C.byref(b), C.byref(c)), "atomo_last_counters")
        return int(a.value), int(b.value), int(c.value)

    def svd_sweeps(self, n_mats: int, stream: Optional[torch.cuda.Stream] = None) -> List[int]:
        """Jacobi sweeps each matrix of the last atomo_encode_svd took (waits for the stream)."""
        out = (C.c_int32 * n_mats)()
        _check(lib().atomo_svd_sweeps(self._h, _stream_handle(stream), out, None, n_mats), "atomo_svd_sweeps")
        return list(out)

    def svd_refreshes(self, n_mats: int, stream: Optional[torch.cuda.Stream] = None) -> List[int]:
        """How often each matrix of the last atomo_encode_svd had its full Gram matrix formed from the data."""
        sweeps = (C.c_int32 * n_mats)()
        out = (C.c_int32 * n_mats)()
        _check(lib().atomo_svd_sweeps(self._h, _stream_handle(stream), sweeps, out, n_mats), "atomo_svd_sweeps")
        return list(out)

    def status(self, stream: Optional[torch.cuda.Stream] = None):
        """Waits for the stream; returns (status, largest Jacobi sweep count of the last SVD encode)."""
        sweeps = C.c_int32(0)
        st = lib().atomo_status(self._h, _stream_handle(stream), C.byref(sweeps))
        return st, int(sweeps.value)


# ---------------------------------------------------------------------------------- entry points

def atomo_probabilities(ctx: Context, lam: torch.Tensor, offsets: Sequence[int], s: float,
                        out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Algorithm 1 on each segment lam[offsets[k]:offsets[k+1]]; returns p (same order as lam)."""
    lam = _f32_cuda(lam, "lam").contiguous()
    p = torch.empty_like(lam) if out is None else _f32_cuda(out, "out")
    offs = (C.c_int64 * len(offsets))(*[int(o) for o in offsets])
    _check(lib().atomo_probabilities(ctx._h, lam.data_ptr(), offs, len(offsets) - 1, float(s), p.data_ptr(),
                                     _stream_handle(stream)), "atomo_probabilities")
    return p


def atomo_encode_svd(ctx: Context, mats: Sequence[torch.Tensor], s: float, seed: int, stream_base: int = 0,
                     msgs: Optional[List[SvdMessage]] = None, sigma_out: Optional[torch.Tensor] = None,
                     p_out: Optional[torch.Tensor] = None, max_sweeps: Optional[int] = None,
                     stop_cosine: Optional[float] = None, max_inner_sweeps: int = 0, inner_reduction: float = 0.0,
                     full_period: int = 0, block_order: int = 0, stream_ids: Optional[Sequence[int]] = None,
                     adaptive: int = 0, stream=None) -> List[SvdMessage]:
    """Spectral-ATOMO encode of a list of 2-D float32 CUDA tensors (row stride = tensor stride).
    stream_ids: one Philox stream id per matrix instead of stream_base + index.
    block_order: 0 = block pairs by weight (default), 1 = the fixed tournament, for the matrices that iterate in Gram space.
    adaptive: k > 0 enqueues only the sweeps that earlier calls with the same shapes needed, plus k (see atomo.h)."""
    n = len(mats)
    c_mats = (atomo_mat * n)()
    for j, g in enumerate(mats):
        _f32_cuda(g, f"mats[{j}]")
        if g.dim() != 2 or g.stride(1) != 1:
            raise ValueError("each gradient must be a 2-D tensor with unit column stride")
        c_mats[j] = atomo_mat(g.shape[0], g.shape[1], g.stride(0) if g.shape[0] > 1 else g.shape[1], g.data_ptr())
    if msgs is None:
        msgs = [alloc_svd_message(g.shape[0], g.shape[1], default_capacity(s, min(g.shape)), g.device) for g in mats]
    c_msgs = (atomo_svd_msg * n)(*[m.c_struct() for m in msgs])
    opt = None
    if (max_sweeps is not None or stop_cosine is not None or max_inner_sweeps or inner_reduction or full_period
            or block_order or stream_ids is not None or adaptive):
        ids = None
        if stream_ids is not None:
            if len(stream_ids) != n:
                raise ValueError("stream_ids needs one entry per matrix")
            ids = (C.c_uint64 * n)(*[int(x) & (2 ** 64 - 1) for x in stream_ids])
        opt = C.byref(atomo_svd_options(0 if max_sweeps is None else max_sweeps,
                                        0.0 if stop_cosine is None else stop_cosine,
                                        max_inner_sweeps, inner_reduction, int(full_period), int(block_order), ids,
                                        int(adaptive)))
    _check(lib().atomo_encode_svd(ctx._h, c_mats, n, float(s), int(seed) & (2 ** 64 - 1),
                                  int(stream_base) & (2 ** 64 - 1), opt, c_msgs,
                                  None if sigma_out is None else sigma_out.data_ptr(),
                                  None if p_out is None else p_out.data_ptr(), _stream_handle(stream)),
           "atomo_encode_svd")
    return msgs


def atomo_encode_entrywise(ctx: Context, g: torch.Tensor, s: float, seed: int, stream_id: int = 0,
                           msg: Optional[EntrywiseMessage] = None, p_out: Optional[torch.Tensor] = None,
                           stream=None) -> EntrywiseMessage:
    """Entry-wise ATOMO encode of a flat float32 CUDA tensor."""
    g = _f32_cuda(g, "g")
    if not g.is_contiguous():
        raise ValueError("g must be contiguous")
    n = g.numel()
    if msg is None:
        msg = alloc_entrywise_message(n, default_capacity(s, n), g.device)
    cm = msg.c_struct()
    _check(lib().atomo_encode_entrywise(ctx._h, g.data_ptr(), float(s), int(seed) & (2 ** 64 - 1),
                                        int(stream_id) & (2 ** 64 - 1), C.byref(cm),
                                        None if p_out is None else p_out.data_ptr(), _stream_handle(stream)),
           "atomo_encode_entrywise")
    return msg


def atomo_encode_entrywise_noalloc(ctx: Context, g: torch.Tensor, s: float, seed: int, stream_id: int,
                                   msg: EntrywiseMessage, p_out: Optional[torch.Tensor] = None, stream=None) -> EntrywiseMessage:
    """atomo_encode_entrywise through the entry point that allocates nothing: the caller brings the message
    buffers, the library's scratch is its fixed per-GPU array (at most 2^24 elements)."""
    g = _f32_cuda(g, "g")
    if not g.is_contiguous():
        raise ValueError("g must be contiguous")
    cm = msg.c_struct()
    _check(lib().atomo_encode_entrywise_noalloc(ctx._h, g.data_ptr(), float(s), int(seed) & (2 ** 64 - 1),
                                                int(stream_id) & (2 ** 64 - 1), C.byref(cm),
                                                None if p_out is None else p_out.data_ptr(), _stream_handle(stream)),
           "atomo_encode_entrywise_noalloc")
    return msg


def atomo_encode_lq(ctx: Context, g: torch.Tensor, q: float, seed: int, stream_id: int = 0,
                    msg: Optional[LqMessage] = None, p_out: Optional[torch.Tensor] = None, stream=None) -> LqMessage:
    """l_q quantisation of a flat float32 CUDA tensor: q = 2 is 1-bit QSGD, q = float('inf') TernGrad."""
    g = _f32_cuda(g, "g")
    if not g.is_contiguous():
        raise ValueError("g must be contiguous")
    n = g.numel()
    if msg is None:
        msg = alloc_lq_message(n, lq_capacity(n, q), g.device)
    cm = msg.c_struct()
    _check(lib().atomo_encode_lq(ctx._h, g.data_ptr(), float(q), int(seed) & (2 ** 64 - 1),
                                 int(stream_id) & (2 ** 64 - 1), C.byref(cm),
                                 None if p_out is None else p_out.data_ptr(), _stream_handle(stream)),
           "atomo_encode_lq")
    return msg


def atomo_decode(ctx: Context, msgs, scale: float = 1.0, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Sums the messages (all SvdMessage of one shape, or all EntrywiseMessage / LqMessage of one length) into a
    dense tensor."""
    msgs = list(msgs)
    first = msgs[0]
    if isinstance(first, SvdMessage):
        if out is None:
            out = torch.empty(first.rows, first.cols, dtype=torch.float32, device=first.U.device)
        _f32_cuda(out, "out")
        c_msgs = (atomo_svd_msg * len(msgs))(*[m.c_struct() for m in msgs])
        _check(lib().atomo_decode(ctx._h, ATOMO_KIND_SVD, C.cast(c_msgs, C.c_void_p), len(msgs), float(scale),
                                  out.data_ptr(), out.stride(0) if out.shape[0] > 1 else out.shape[1],
                                  _stream_handle(stream)), "atomo_decode")
        return out
    if isinstance(first, LqMessage):
        if out is None:
            out = torch.empty(first.n, dtype=torch.float32, device=first.idx.device)
        _f32_cuda(out, "out")
        c_msgs = (atomo_lq_msg * len(msgs))(*[m.c_struct() for m in msgs])
        _check(lib().atomo_decode(ctx._h, ATOMO_KIND_LQ, C.cast(c_msgs, C.c_void_p), len(msgs), float(scale),
                                  out.data_ptr(), 0, _stream_handle(stream)), "atomo_decode")
        return out
    if out is None:
        out = torch.empty(first.n, dtype=torch.float32, device=first.val.device)
    _f32_cuda(out, "out")
    c_msgs = (atomo_ew_msg * len(msgs))(*[m.c_struct() for m in msgs])
    _check(lib().atomo_decode(ctx._h, ATOMO_KIND_ENTRYWISE, C.cast(c_msgs, C.c_void_p), len(msgs), float(scale),
                              out.data_ptr(), 0, _stream_handle(stream)), "atomo_decode")
    return out


def atomo_decode_svd_batch(ctx: Context, groups: Sequence[Sequence[SvdMessage]], scale: float = 1.0,
                           outs: Optional[List[torch.Tensor]] = None, stream=None) -> List[torch.Tensor]:
    """One launch for a whole layer set: groups[o] are the messages summed into outs[o]."""
    flat = [m for grp in groups for m in grp]
    first = [0]
    for grp in groups:
        first.append(first[-1] + len(grp))
    if outs is None:
        outs = [torch.empty(grp[0].rows, grp[0].cols, dtype=torch.float32, device=grp[0].U.device) for grp in groups]
    c_msgs = (atomo_svd_msg * len(flat))(*[m.c_struct() for m in flat])
    c_first = (C.c_int32 * len(first))(*first)
    c_outs = (C.c_void_p * len(outs))(*[o.data_ptr() for o in outs])
    c_lds = (C.c_int64 * len(outs))(*[o.stride(0) if o.shape[0] > 1 else o.shape[1] for o in outs])
    _check(lib().atomo_decode_svd_batch(ctx._h, c_msgs, c_first, len(outs), float(scale), c_outs, c_lds,
                                        _stream_handle(stream)), "atomo_decode_svd_batch")
    return outs


def atomo_apply_svd_batch(ctx: Context, groups: Sequence[Sequence[SvdMessage]], alpha: float,
                          params: List[torch.Tensor], stream=None) -> List[torch.Tensor]:
    """params[o] += alpha * (sum of the decoded messages of groups[o]), in place, one launch for the layer set."""
    flat = [m for grp in groups for m in grp]
    first = [0]
    for grp in groups:
        first.append(first[-1] + len(grp))
    for p, grp in zip(params, groups):
        if p.dtype != torch.float32 or tuple(p.shape) != (grp[0].rows, grp[0].cols) or p.stride(1) != 1:
            raise ValueError("params must be float32 rows x cols tensors with unit column stride")
    c_msgs = (atomo_svd_msg * len(flat))(*[m.c_struct() for m in flat])
    c_first = (C.c_int32 * len(first))(*first)
    c_params = (C.c_void_p * len(params))(*[p.data_ptr() for p in params])
    c_lds = (C.c_int64 * len(params))(*[p.stride(0) if p.shape[0] > 1 else p.shape[1] for p in params])
    _check(lib().atomo_apply_svd_batch(ctx._h, c_msgs, c_first, len(params), float(alpha), c_params, c_lds,
                                       _stream_handle(stream)), "atomo_apply_svd_batch")
    return params
