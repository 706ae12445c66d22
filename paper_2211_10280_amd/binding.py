"""ctypes binding of libtensair.so -- argument marshalling only.

Every function here has the name of the C entry point it forwards to
(``include/tensair.h``); PyTorch supplies device memory and the stream, nothing
else.  There is no CPU fallback: if the shared library is missing, ``lib()``
raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtensair.so")

F32, BF16 = 0, 1
OK, EINVAL, ECAPACITY, EHIP, EDATA = 0, -1, -2, -3, -4
MAX_PEERS = 31
MAX_VOCAB = (1 << 28) - 64
MAX_DENSE = 1 << 33
STATIC_MAX_VOCAB = 1 << 21
STATIC_MAX_PEERS = 15
RESAMPLE_NEGATIVES = 1
STOCHASTIC_ROUNDING = 2

SYMBOLS = [
    "tensair_workspace_bytes", "tensair_capacity_in", "tensair_capacity_out", "tensair_model_init",
    "tensair_model_rebind", "tensair_model_alias", "tensair_pair_count", "tensair_sgns_grad",
    "tensair_dasgd_apply", "tensair_step", "tensair_status", "tensair_model_destroy",
    "tensair_last_error", "tensair_profile", "tensair_profile_read", "tensair_copy_probe",
    "tensair_prefetch", "tensair_grad_add", "tensair_dense_apply", "tensair_lookup",
    "tensair_cosine_difference", "tensair_grad_pack", "tensair_dasgd_apply_packed", "tensair_step_packed",
    "tensair_dasgd_apply_static", "tensair_stream_probe", "tensair_aligned_row_stride",
]

PROFILE_TAGS = {1: "keys", 2: "forward", 3: "sort", 4: "segments", 5: "reduce_in", 6: "reduce_out",
                8: "apply_index", 9: "apply_update", 11: "add_index", 12: "add_rows", 14: "pack"}


class TensairError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libtensair error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [("vocab", C.c_int64), ("dim", C.c_int32), ("row_stride", C.c_int32),
                ("dtype", C.c_int32), ("window", C.c_int32), ("negatives", C.c_int32),
                ("max_centers", C.c_int32), ("max_peers", C.c_int32), ("worker_id", C.c_uint32),
                ("seed", C.c_uint64), ("flags", C.c_uint32)]


class SparseRows(C.Structure):
    _fields_ = [("capacity", C.c_int64), ("n_rows", C.c_void_p), ("row_ids", C.c_void_p),
                ("row_grads", C.c_void_p)]


class SparseGrad(C.Structure):
    _fields_ = [("in_", SparseRows), ("out", SparseRows)]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2211_10280_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32
        L.tensair_aligned_row_stride.argtypes = [i32, i32]
        L.tensair_aligned_row_stride.restype = i32
        L.tensair_workspace_bytes.argtypes = [C.POINTER(Config)]
        L.tensair_workspace_bytes.restype = C.c_size_t
        L.tensair_capacity_in.argtypes = [C.POINTER(Config), i32]
        L.tensair_capacity_in.restype = i64
        L.tensair_capacity_out.argtypes = [C.POINTER(Config), i32]
        L.tensair_capacity_out.restype = i64
        L.tensair_model_init.argtypes = [C.POINTER(vp), C.POINTER(Config), vp, vp, C.c_int, vp, vp,
                                         C.c_size_t, vp]
        L.tensair_model_init.restype = C.c_int
        L.tensair_model_rebind.argtypes = [vp, vp, vp, u32]
        L.tensair_model_rebind.restype = C.c_int
        L.tensair_model_alias.argtypes = [vp, vp, vp]
        L.tensair_model_alias.restype = C.c_int
        L.tensair_pair_count.argtypes = [vp, i64, i64, i32]
        L.tensair_pair_count.restype = i64
        L.tensair_sgns_grad.argtypes = [vp, vp, i64, i64, i32, u32, C.POINTER(SparseGrad), vp, vp, vp, vp, vp]
        L.tensair_sgns_grad.restype = C.c_int
        L.tensair_dasgd_apply.argtypes = [vp, C.POINTER(SparseGrad), C.POINTER(SparseGrad), i32,
                                          C.c_float, vp]
        L.tensair_dasgd_apply.restype = C.c_int
        L.tensair_step.argtypes = [vp, vp, i64, i64, i32, u32, C.POINTER(SparseGrad), i32, C.c_float,
                                   C.POINTER(SparseGrad), vp, vp]
        L.tensair_step.restype = C.c_int
        L.tensair_prefetch.argtypes = [vp, vp, i64, i64, i32, u32, vp]
        L.tensair_prefetch.restype = C.c_int
        L.tensair_grad_add.argtypes = [vp, C.POINTER(SparseGrad), C.POINTER(SparseGrad), C.POINTER(SparseGrad), vp]
        L.tensair_grad_add.restype = C.c_int
        L.tensair_dense_apply.argtypes = [vp, i32, i64, C.POINTER(vp), i32, C.c_float, vp]
        L.tensair_dense_apply.restype = C.c_int
        L.tensair_lookup.argtypes = [vp, i32, vp, i64, vp, vp]
        L.tensair_lookup.restype = C.c_int
        L.tensair_cosine_difference.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp]
        L.tensair_cosine_difference.restype = C.c_int
        # a packed gradient has the layout of a sparse one (its rows are bfloat16 instead of fp32)
        L.tensair_grad_pack.argtypes = [vp, C.POINTER(SparseGrad), C.POINTER(SparseGrad), vp]
        L.tensair_grad_pack.restype = C.c_int
        L.tensair_dasgd_apply_packed.argtypes = L.tensair_dasgd_apply.argtypes
        L.tensair_dasgd_apply_packed.restype = C.c_int
        L.tensair_step_packed.argtypes = [vp, vp, i64, i64, i32, u32, C.POINTER(SparseGrad), i32, C.c_float,
                                          C.POINTER(SparseGrad), C.POINTER(SparseGrad), vp, vp]
        L.tensair_step_packed.restype = C.c_int
        L.tensair_dasgd_apply_static.argtypes = [vp, vp, i64, i32, i32, i32, C.POINTER(SparseGrad),
                                                 C.POINTER(SparseGrad), i32, C.c_float, vp, vp]
        L.tensair_dasgd_apply_static.restype = C.c_int
        L.tensair_status.argtypes = [vp, vp]
        L.tensair_status.restype = C.c_int
        L.tensair_model_destroy.argtypes = [vp]
        L.tensair_model_destroy.restype = C.c_int
        L.tensair_profile.argtypes = [vp, C.c_int]
        L.tensair_profile.restype = C.c_int
        L.tensair_profile_read.argtypes = [vp, vp, vp, i32]
        L.tensair_profile_read.restype = C.c_int
        L.tensair_copy_probe.argtypes = [vp, vp, C.c_size_t, vp]
        L.tensair_copy_probe.restype = C.c_int
        L.tensair_stream_probe.argtypes = [vp, vp, C.c_size_t, i32, vp]
        L.tensair_stream_probe.restype = C.c_int
        L.tensair_last_error.argtypes = []
        L.tensair_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise TensairError(rc, lib().tensair_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


# ---------------------------------------------------------------- device buffers
class GradBuffers:
    """Device memory of one tensair_sparse_grad (caller-owned, as the ABI asks)."""

    ROWS = torch.float32

    def __init__(self, cap_in: int, cap_out: int, dim: int, device="cuda"):
        self.dim = dim
        self.n_rows = torch.zeros(2, dtype=torch.int32, device=device)     # [in, out]
        self.in_ids = torch.empty(max(cap_in, 1), dtype=torch.int32, device=device)
        self.in_rows = torch.empty((max(cap_in, 1), dim), dtype=self.ROWS, device=device)
        self.out_ids = torch.empty(max(cap_out, 1), dtype=torch.int32, device=device)
        self.out_rows = torch.empty((max(cap_out, 1), dim), dtype=self.ROWS, device=device)
        self.cap_in, self.cap_out = cap_in, cap_out
        self.c = SparseGrad()
        self.c.in_ = SparseRows(cap_in, self.n_rows.data_ptr(), self.in_ids.data_ptr(), self.in_rows.data_ptr())
        self.c.out = SparseRows(cap_out, self.n_rows.data_ptr() + 4, self.out_ids.data_ptr(),
                                self.out_rows.data_ptr())

    def sizes(self):
        n = self.n_rows.cpu()
        return int(n[0]), int(n[1])

    def to_host(self):
        """((ids_in, rows_in), (ids_out, rows_out)) as numpy arrays trimmed to n_rows."""
        ui, uo = self.sizes()
        return ((self.in_ids[:ui].cpu().numpy(), self.in_rows[:ui].cpu().numpy()),
                (self.out_ids[:uo].cpu().numpy(), self.out_rows[:uo].cpu().numpy()))

    def ids_to_host(self):
        """(ids_in, ids_out) as numpy arrays trimmed to n_rows (the rows stay on the device)."""
        ui, uo = self.sizes()
        return self.in_ids[:ui].cpu().numpy(), self.out_ids[:uo].cpu().numpy()

    def load(self, ids_in, rows_in, ids_out, rows_out):
        """Fill from host arrays (e.g. a gradient received from a peer)."""
        ui, uo = len(ids_in), len(ids_out)
        assert ui <= self.cap_in and uo <= self.cap_out
        self.in_ids[:ui] = torch.from_numpy(np.ascontiguousarray(ids_in, dtype=np.int32)).to(self.in_ids.device)
        self.out_ids[:uo] = torch.from_numpy(np.ascontiguousarray(ids_out, dtype=np.int32)).to(self.in_ids.device)
        if ui:
            self.in_rows[:ui] = torch.from_numpy(np.ascontiguousarray(rows_in, dtype=np.float32)).to(self.in_ids.device)
        if uo:
            self.out_rows[:uo] = torch.from_numpy(np.ascontiguousarray(rows_out, dtype=np.float32)).to(self.in_ids.device)
        self.n_rows.copy_(torch.tensor([ui, uo], dtype=torch.int32))


class PackedBuffers(GradBuffers):
    """Device memory of one tensair_packed_grad: the same, with bfloat16 rows (kept as int16 bits)."""
    ROWS = torch.int16

    def to_host(self):
        (ii, ri), (io, ro) = super().to_host()
        return (ii, ri.view(np.uint16)), (io, ro.view(np.uint16))

    def load(self, ids_in, bits_in, ids_out, bits_out):
        """Fill from host arrays; the rows are uint16 bfloat16 bits."""
        ui, uo = len(ids_in), len(ids_out)
        assert ui <= self.cap_in and uo <= self.cap_out
        dev = self.in_ids.device
        self.in_ids[:ui] = torch.from_numpy(np.ascontiguousarray(ids_in, dtype=np.int32)).to(dev)
        self.out_ids[:uo] = torch.from_numpy(np.ascontiguousarray(ids_out, dtype=np.int32)).to(dev)
        if ui:
            self.in_rows[:ui] = torch.from_numpy(np.ascontiguousarray(bits_in, dtype=np.uint16).view(np.int16)).to(dev)
        if uo:
            self.out_rows[:uo] = torch.from_numpy(np.ascontiguousarray(bits_out, dtype=np.uint16).view(np.int16)).to(dev)
        self.n_rows.copy_(torch.tensor([ui, uo], dtype=torch.int32))


# ---------------------------------------------------------------- C entry points, same names
def tensair_aligned_row_stride(dim: int, dtype: int) -> int:
    n = lib().tensair_aligned_row_stride(dim, dtype)
    if n < 0:
        raise TensairError(EINVAL, "aligned_row_stride: bad dim or dtype")
    return n


def tensair_workspace_bytes(cfg: Config) -> int:
    n = lib().tensair_workspace_bytes(C.byref(cfg))
    if n == 0:
        raise TensairError(EINVAL, lib().tensair_last_error().decode())
    return n


def tensair_capacity_in(cfg: Config, n_centers: int) -> int:
    return lib().tensair_capacity_in(C.byref(cfg), n_centers)


def tensair_capacity_out(cfg: Config, n_centers: int) -> int:
    return lib().tensair_capacity_out(C.byref(cfg), n_centers)


def tensair_model_init(cfg: Config, w_in, w_out, fill_tables: bool, unigram_counts: np.ndarray,
                       workspace, stream=None):
    counts = np.ascontiguousarray(unigram_counts, dtype=np.uint64)
    h = C.c_void_p()
    _check(lib().tensair_model_init(C.byref(h), C.byref(cfg), _ptr(w_in), _ptr(w_out), int(fill_tables),
                                    counts.ctypes.data_as(C.c_void_p), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))
    return h


def tensair_model_rebind(h, w_in, w_out, worker_id: int):
    _check(lib().tensair_model_rebind(h, _ptr(w_in), _ptr(w_out), worker_id))


def tensair_model_alias(h, vocab: int):
    thr = np.zeros(vocab, dtype=np.uint32)
    alias = np.zeros(vocab, dtype=np.int32)
    _check(lib().tensair_model_alias(h, thr.ctypes.data_as(C.c_void_p), alias.ctypes.data_as(C.c_void_p)))
    return thr, alias


def tensair_pair_count(h, n_tokens: int, center_begin: int, n_centers: int) -> int:
    p = lib().tensair_pair_count(h, n_tokens, center_begin, n_centers)
    if p < 0:
        raise TensairError(EINVAL, lib().tensair_last_error().decode())
    return p


def tensair_sgns_grad(h, tokens, center_begin: int, n_centers: int, epoch: int, grad: GradBuffers,
                      mean_loss=None, negatives_dbg=None, seg_offsets_in=None, seg_offsets_out=None,
                      stream=None):
    _check(lib().tensair_sgns_grad(h, _ptr(tokens), tokens.numel(), center_begin, n_centers, epoch,
                                   C.byref(grad.c), _ptr(mean_loss), _ptr(negatives_dbg),
                                   _ptr(seg_offsets_in), _ptr(seg_offsets_out), _stream(stream)))


def _peer_array(peers):
    arr = (SparseGrad * max(len(peers), 1))()
    for i, p in enumerate(peers):
        arr[i] = p.c
    return arr


def tensair_dasgd_apply(h, own, peers, lr: float, stream=None):
    arr = _peer_array(peers)
    _check(lib().tensair_dasgd_apply(h, C.byref(own.c) if own is not None else None, arr, len(peers),
                                     C.c_float(lr), _stream(stream)))


def tensair_dasgd_apply_static(w_in, w_out, dim: int, own, peers, lr: float, status=None, stream=None):
    """w_in, w_out: [vocab, row_stride] tables of the same dtype; status: int32 tensor of one element or None."""
    dt = F32 if w_in.dtype == torch.float32 else BF16
    arr = _peer_array(peers)
    _check(lib().tensair_dasgd_apply_static(_ptr(w_in), _ptr(w_out), w_in.shape[0], dim, w_in.shape[1], dt,
                                            C.byref(own.c) if own is not None else None, arr, len(peers),
                                            C.c_float(lr), _ptr(status), _stream(stream)))


def tensair_step(h, tokens, center_begin: int, n_centers: int, epoch: int, peers, lr: float,
                 own_out: GradBuffers, mean_loss=None, stream=None):
    arr = _peer_array(peers)
    _check(lib().tensair_step(h, _ptr(tokens), tokens.numel(), center_begin, n_centers, epoch, arr,
                              len(peers), C.c_float(lr), C.byref(own_out.c), _ptr(mean_loss),
                              _stream(stream)))


def tensair_grad_pack(h, g: GradBuffers, out: PackedBuffers, stream=None):
    _check(lib().tensair_grad_pack(h, C.byref(g.c), C.byref(out.c), _stream(stream)))


def tensair_dasgd_apply_packed(h, own, peers, lr: float, stream=None):
    arr = _peer_array(peers)
    _check(lib().tensair_dasgd_apply_packed(h, C.byref(own.c) if own is not None else None, arr, len(peers),
                                            C.c_float(lr), _stream(stream)))


def tensair_step_packed(h, tokens, center_begin: int, n_centers: int, epoch: int, peers, lr: float,
                        own_out: GradBuffers, own_msg_out=None, mean_loss=None, stream=None):
    arr = _peer_array(peers)
    _check(lib().tensair_step_packed(h, _ptr(tokens), tokens.numel(), center_begin, n_centers, epoch, arr,
                                     len(peers), C.c_float(lr), C.byref(own_out.c),
                                     C.byref(own_msg_out.c) if own_msg_out is not None else None, _ptr(mean_loss),
                                     _stream(stream)))


def tensair_prefetch(h, tokens, center_begin: int, n_centers: int, epoch: int, stream=None):
    _check(lib().tensair_prefetch(h, _ptr(tokens), tokens.numel(), center_begin, n_centers, epoch,
                                  _stream(stream)))


def tensair_grad_add(h, a: GradBuffers, b: GradBuffers, out: GradBuffers, stream=None):
    _check(lib().tensair_grad_add(h, C.byref(a.c), C.byref(b.c), C.byref(out.c), _stream(stream)))


def tensair_dense_apply(theta, grads, lr: float, stream=None):
    """theta: 1-D float32 or bfloat16 tensor; grads: list of float32 tensors of the same length."""
    dt = F32 if theta.dtype == torch.float32 else BF16
    arr = (C.c_void_p * max(len(grads), 1))(*[g.data_ptr() for g in grads])
    _check(lib().tensair_dense_apply(_ptr(theta), dt, theta.numel(), arr, len(grads), C.c_float(lr),
                                     _stream(stream)))


def tensair_lookup(h, table: int, ids, out, stream=None):
    _check(lib().tensair_lookup(h, table, _ptr(ids), ids.numel(), _ptr(out), _stream(stream)))


def tensair_cosine_difference(a, b, dim: int, diff, stream=None):
    """a, b: [vocab, row_stride] tables of the same dtype; diff: float32 [vocab]."""
    dt = F32 if a.dtype == torch.float32 else BF16
    _check(lib().tensair_cosine_difference(_ptr(a), _ptr(b), dt, a.shape[0], dim, a.shape[1], _ptr(diff),
                                           _stream(stream)))


def tensair_status(h, stream=None):
    _check(lib().tensair_status(h, _stream(stream)))


def tensair_profile(h, level: int):
    _check(lib().tensair_profile(h, level))


def tensair_profile_read(h, max_records: int = 65536):
    """[(tag name, milliseconds), ...] since the previous read."""
    tags = np.zeros(max_records, dtype=np.int32)
    ms = np.zeros(max_records, dtype=np.float32)
    n = lib().tensair_profile_read(h, tags.ctypes.data_as(C.c_void_p), ms.ctypes.data_as(C.c_void_p), max_records)
    if n < 0:
        raise TensairError(n, lib().tensair_last_error().decode())
    return [(PROFILE_TAGS.get(int(tags[i]), str(int(tags[i]))), float(ms[i])) for i in range(n)]


def tensair_copy_probe(dst, src, nbytes: int, stream=None):
    _check(lib().tensair_copy_probe(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


def tensair_stream_probe(dst, src, nbytes: int, mode: int, stream=None):
    _check(lib().tensair_stream_probe(_ptr(dst), _ptr(src), nbytes, mode, _stream(stream)))


def tensair_model_destroy(h):
    _check(lib().tensair_model_destroy(h))


# ---------------------------------------------------------------- convenience owner of the buffers
class Model:
    """Owns the device memory a tensair_model needs (tables, workspace) and forwards to the
    C entry points.  No arithmetic happens here."""

    def __init__(self, vocab, dim, dtype, window, negatives, max_centers, max_peers, seed,
                 unigram_counts, worker_id=0, row_stride=None, tables=None, device="cuda", flags=0):
        self.cfg = Config(vocab, dim, row_stride or dim, dtype, window, negatives, max_centers,
                          max_peers, worker_id, seed, flags)
        tdt = torch.float32 if dtype == F32 else torch.bfloat16
        if tables is None:
            self.w_in = torch.empty((vocab, self.cfg.row_stride), dtype=tdt, device=device)
            self.w_out = torch.empty((vocab, self.cfg.row_stride), dtype=tdt, device=device)
            fill = True
        else:
            self.w_in, self.w_out = tables
            fill = False
        nbytes = tensair_workspace_bytes(self.cfg)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.h = tensair_model_init(self.cfg, self.w_in, self.w_out, fill, unigram_counts, self.workspace)
        self.device = device

    def grad_buffers(self, n_centers=None) -> GradBuffers:
        n = self.cfg.max_centers if n_centers is None else n_centers
        return GradBuffers(tensair_capacity_in(self.cfg, n), tensair_capacity_out(self.cfg, n),
                           self.cfg.dim, self.device)

    def rebind(self, w_in, w_out, worker_id):
        tensair_model_rebind(self.h, w_in, w_out, worker_id)

    def alias(self):
        return tensair_model_alias(self.h, self.cfg.vocab)

    def pair_count(self, n_tokens, begin, n):
        return tensair_pair_count(self.h, n_tokens, begin, n)

    def sgns_grad(self, tokens, begin, n, epoch, grad, **kw):
        tensair_sgns_grad(self.h, tokens, begin, n, epoch, grad, **kw)

    def dasgd_apply(self, own, peers, lr):
        tensair_dasgd_apply(self.h, own, peers, lr)

    def step(self, tokens, begin, n, epoch, peers, lr, own_out, mean_loss=None):
        tensair_step(self.h, tokens, begin, n, epoch, peers, lr, own_out, mean_loss)

    def grad_pack(self, g, out):
        tensair_grad_pack(self.h, g, out)

    def dasgd_apply_packed(self, own, peers, lr):
        tensair_dasgd_apply_packed(self.h, own, peers, lr)

    def step_packed(self, tokens, begin, n, epoch, peers, lr, own_out, own_msg_out=None, mean_loss=None):
        tensair_step_packed(self.h, tokens, begin, n, epoch, peers, lr, own_out, own_msg_out, mean_loss)

    def packed_buffers(self, n_centers=None) -> PackedBuffers:
        n = self.cfg.max_centers if n_centers is None else n_centers
        return PackedBuffers(tensair_capacity_in(self.cfg, n), tensair_capacity_out(self.cfg, n),
                             self.cfg.dim, self.device)

    def lookup(self, table, ids, out):
        tensair_lookup(self.h, table, ids, out)

    def grad_add(self, a, b, out):
        tensair_grad_add(self.h, a, b, out)

    def prefetch(self, tokens, begin, n, epoch):
        tensair_prefetch(self.h, tokens, begin, n, epoch)

    def status(self):
        tensair_status(self.h)

    def close(self):
        if self.h is not None:
            tensair_model_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
