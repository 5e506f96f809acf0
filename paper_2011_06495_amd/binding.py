"""Thin ctypes binding of the C ABI in include/mv.h (libmv.so).

Argument marshalling only: every step of the vote step runs in the library's
HIP kernels.  PyTorch tensors supply device memory and the stream.  There is no
fallback: if libmv.so has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmv.so")

MV_OK, MV_ERR_INVALID_ARG, MV_ERR_UNSUPPORTED, MV_ERR_ALLOC, MV_ERR_DEVICE, MV_ERR_STATE = range(6)
MV_F32, MV_BF16 = 0, 1
MV_REDUCE_MEAN, MV_REDUCE_SUM = 0, 1
MV_FLAG_ADD_DROP = 1

# every symbol include/mv.h declares
ABI_SYMBOLS = (
    "mv_workspace_bytes", "mv_begin", "mv_vote_step", "mv_ad_vote_step", "mv_rs_vote_step", "mv_end", "mv_release", "mv_status_string",
    "mv_kernel_count", "mv_kernel_name", "mv_set_profiling", "mv_set_spin_limit", "mv_step_kernel_ms",
    "mv_last_step_row_stats", "mv_probe_copy",
    "mv_codec_stream_bits", "mv_codec_scratch_bytes", "mv_codec_encode", "mv_codec_decode", "mv_codec_decode_static",
    "mv_quant_scratch_bytes", "mv_quant_encode", "mv_quant_decode",
)


class mv_config(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("device", ctypes.c_int32),
        ("n_workers", ctypes.c_int32),
        ("grad_dtype", ctypes.c_int32),
        ("d", ctypes.c_int64),
        ("k", ctypes.c_int64),
        ("reduce", ctypes.c_int32),
        ("flags", ctypes.c_int32),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
    ]


class MvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


_lib: Optional[ctypes.CDLL] = None


def load() -> ctypes.CDLL:
    """Loads libmv.so (built by paper_2011_06495_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it first (python -m paper_2011_06495_amd.build); "
            "there is no CPU fallback" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u32p = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.POINTER(ctypes.c_uint32)
    L.mv_workspace_bytes.argtypes = [ctypes.POINTER(mv_config)]
    L.mv_workspace_bytes.restype = ctypes.c_size_t
    L.mv_begin.argtypes = [ctypes.POINTER(mv_config), ctypes.POINTER(vp)]
    L.mv_begin.restype = i32
    L.mv_vote_step.argtypes = [vp, vp, i64, vp, i64, vp, vp, vp, vp, vp]
    L.mv_vote_step.restype = i32
    L.mv_ad_vote_step.argtypes = [vp, vp, i64, vp, i64, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    L.mv_ad_vote_step.restype = i32
    L.mv_rs_vote_step.argtypes = [vp, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp]
    L.mv_rs_vote_step.restype = i32
    L.mv_end.argtypes = [vp]
    L.mv_end.restype = i32
    L.mv_release.argtypes = [vp]
    L.mv_release.restype = None
    L.mv_status_string.argtypes = [i32]
    L.mv_status_string.restype = ctypes.c_char_p
    L.mv_kernel_count.argtypes = []
    L.mv_kernel_count.restype = i32
    L.mv_kernel_name.argtypes = [i32]
    L.mv_kernel_name.restype = ctypes.c_char_p
    L.mv_set_profiling.argtypes = [vp, i32]
    L.mv_set_profiling.restype = i32
    L.mv_set_spin_limit.argtypes = [vp, ctypes.c_uint32]
    L.mv_set_spin_limit.restype = i32
    L.mv_step_kernel_ms.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_float), i32]
    L.mv_step_kernel_ms.restype = i32
    L.mv_last_step_row_stats.argtypes = [vp, u32p, u32p, u32p]
    L.mv_last_step_row_stats.restype = i32
    u64 = ctypes.c_uint64
    L.mv_codec_stream_bits.argtypes = [i64, i64, i64]
    L.mv_codec_stream_bits.restype = u64
    L.mv_codec_scratch_bytes.argtypes = [u64, i32]
    L.mv_codec_scratch_bytes.restype = ctypes.c_size_t
    L.mv_codec_encode.argtypes = [vp, i64, vp, i64, i64, i32, i64, i64, vp, i64, vp, vp]
    L.mv_codec_encode.restype = i32
    L.mv_codec_decode.argtypes = [vp, i64, vp, u64, i32, i64, i64, vp, i64, i64, vp, vp, ctypes.c_size_t, vp]
    L.mv_codec_decode.restype = i32
    L.mv_codec_decode_static.argtypes = [vp, i64, vp, u64, i32, i64, i64, vp, i64, i64, vp, vp]
    L.mv_codec_decode_static.restype = i32
    L.mv_quant_scratch_bytes.argtypes = [i64, i32, i32]
    L.mv_quant_scratch_bytes.restype = ctypes.c_size_t
    L.mv_quant_encode.argtypes = [vp, i64, i64, i32, i32, vp, i64, vp, vp, ctypes.c_size_t, vp]
    L.mv_quant_encode.restype = i32
    L.mv_quant_decode.argtypes = [vp, i64, i64, i32, i32, vp, vp, i64, vp]
    L.mv_quant_decode.restype = i32
    L.mv_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.mv_probe_copy.restype = i32
    _lib = L
    return L


def status_string(status: int) -> str:
    return load().mv_status_string(int(status)).decode()


def make_config(n_workers: int, d: int, k: int, grad_dtype: int = MV_F32, reduce: int = MV_REDUCE_MEAN,
                device: int = 0, workspace: int = 0, workspace_bytes: int = 0, flags: int = 0) -> mv_config:
    return mv_config(ctypes.sizeof(mv_config), device, n_workers, grad_dtype, d, k, reduce, flags,
                     workspace or None, workspace_bytes)


def mv_workspace_bytes(cfg: mv_config) -> int:
    return int(load().mv_workspace_bytes(ctypes.byref(cfg)))


def mv_begin(cfg: mv_config) -> int:
    """Returns the context handle (an integer address); raises MvError."""
    h = ctypes.c_void_p()
    st = load().mv_begin(ctypes.byref(cfg), ctypes.byref(h))
    if st != MV_OK:
        raise MvError(st, "mv_begin")
    return h.value


def _dev_ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def mv_vote_step(ctx: int, grads, err, worker_idx, votes, mask_idx, agg_vals, stream=None,
                 ld_g: Optional[int] = None, ld_e: Optional[int] = None) -> None:
    """Enqueues one vote step on `stream` (a torch.cuda.Stream; None = torch's
    current stream).  Tensors are torch device tensors; `grads` and `err` are
    2-D with unit column stride (the row stride is taken from the tensor unless
    given).  worker_idx and votes may be None."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(err.device)
    st = load().mv_vote_step(
        ctx, _dev_ptr(grads), grads.stride(0) if ld_g is None else ld_g,
        _dev_ptr(err), err.stride(0) if ld_e is None else ld_e,
        _dev_ptr(worker_idx), _dev_ptr(votes), _dev_ptr(mask_idx), _dev_ptr(agg_vals),
        stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_vote_step")


def mv_rs_vote_step(ctx: int, grads, err, rand_exp, worker_idx, votes, mask_idx, agg_vals, stream=None,
                    ld_g: Optional[int] = None, ld_e: Optional[int] = None) -> None:
    """Enqueues one step of majority voting with random selection: as mv_vote_step,
    the mask drawn in proportion to the votes with the caller's Exp(1) numbers
    `rand_exp` (d float32 on the device)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(err.device)
    st = load().mv_rs_vote_step(
        ctx, _dev_ptr(grads), grads.stride(0) if ld_g is None else ld_g,
        _dev_ptr(err), err.stride(0) if ld_e is None else ld_e, _dev_ptr(rand_exp),
        _dev_ptr(worker_idx), _dev_ptr(votes), _dev_ptr(mask_idx), _dev_ptr(agg_vals),
        stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_rs_vote_step")


def mv_ad_vote_step(ctx: int, grads, err, k_ad: int, vote_bits, msum, add_idx, drop_idx, counts, mask_idx,
                    agg_vals, stream=None, ld_g: Optional[int] = None, ld_e: Optional[int] = None) -> None:
    """Enqueues one add-drop vote step (Algorithm 2).  vote_bits: N x ld_bits int32
    device tensor (the standing votes' bitmaps), msum: uint8 device tensor."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(err.device)
    st = load().mv_ad_vote_step(
        ctx, _dev_ptr(grads), grads.stride(0) if ld_g is None else ld_g,
        _dev_ptr(err), err.stride(0) if ld_e is None else ld_e, int(k_ad),
        _dev_ptr(vote_bits), vote_bits.stride(0), _dev_ptr(msum), _dev_ptr(add_idx), _dev_ptr(drop_idx),
        _dev_ptr(counts), _dev_ptr(mask_idx), _dev_ptr(agg_vals), stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_ad_vote_step")


def mv_end(ctx: int) -> None:
    st = load().mv_end(ctx)
    if st != MV_OK:
        raise MvError(st, "mv_end")


def mv_release(ctx: int) -> None:
    load().mv_release(ctx)


def kernel_names():
    L = load()
    return [L.mv_kernel_name(i).decode() for i in range(L.mv_kernel_count())]


def mv_set_profiling(ctx: int, level: int) -> None:
    st = load().mv_set_profiling(ctx, level)
    if st != MV_OK:
        raise MvError(st, "mv_set_profiling")


def mv_set_spin_limit(ctx: int, polls: int) -> None:
    st = load().mv_set_spin_limit(ctx, polls)
    if st != MV_OK:
        raise MvError(st, "mv_set_spin_limit")


def mv_step_kernel_ms(ctx: int, steps_back: int = 0):
    n = load().mv_kernel_count()
    buf = (ctypes.c_float * n)()
    st = load().mv_step_kernel_ms(ctx, steps_back, buf, n)
    if st != MV_OK:
        raise MvError(st, "mv_step_kernel_ms")
    return list(buf)


def mv_last_step_row_stats(ctx: int, n_workers: int):
    a, b, c = ((ctypes.c_uint32 * n_workers)() for _ in range(3))
    st = load().mv_last_step_row_stats(ctx, a, b, c)
    if st != MV_OK:
        raise MvError(st, "mv_last_step_row_stats")
    return list(a), list(b), list(c)


def mv_probe_copy(dst, src, stream=None) -> None:
    """Plain streaming copy src -> dst (torch device tensors of equal byte size)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(src.device)
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    st = load().mv_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_probe_copy")


def mv_codec_stream_bits(n: int, d: int, block_len: int) -> int:
    return int(load().mv_codec_stream_bits(n, d, block_len))


def mv_codec_scratch_bytes(max_bits: int, rows: int) -> int:
    return int(load().mv_codec_scratch_bytes(max_bits, rows))


def mv_codec_encode(idx, n: int, d: int, block_len: int, streams, n_bits, counts=None, counts_stride: int = 1,
                    stream=None) -> None:
    """idx: rows x ld int32 device tensor of ascending coordinates; streams: rows x ld_words
    int32 device tensor (out); n_bits: rows int64 device tensor (out); counts: optional
    int32 device tensor with the rows' lengths at stride counts_stride."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(idx.device)
    st = load().mv_codec_encode(_dev_ptr(idx), idx.stride(0), _dev_ptr(counts), counts_stride, n, idx.shape[0], d,
                                block_len, _dev_ptr(streams), streams.stride(0), _dev_ptr(n_bits),
                                stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_codec_encode")


def mv_codec_decode(streams, n_bits, max_bits: int, d: int, block_len: int, idx_out, max_n: int, counts_out,
                    scratch, stream=None) -> None:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(streams.device)
    st = load().mv_codec_decode(_dev_ptr(streams), streams.stride(0), _dev_ptr(n_bits), max_bits, streams.shape[0],
                                d, block_len, _dev_ptr(idx_out), idx_out.stride(0), max_n, _dev_ptr(counts_out),
                                _dev_ptr(scratch), scratch.numel() * scratch.element_size(), stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_codec_decode")


MV_CODEC_STATIC_SCRATCH_BYTES = 16 << 20


def mv_codec_decode_static(streams, n_bits, max_bits: int, d: int, block_len: int, idx_out, max_n: int, counts_out,
                           stream=None) -> None:
    """mv_codec_decode on the library's own scratch array: allocates nothing."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(streams.device)
    st = load().mv_codec_decode_static(_dev_ptr(streams), streams.stride(0), _dev_ptr(n_bits), max_bits,
                                       streams.shape[0], d, block_len, _dev_ptr(idx_out), idx_out.stride(0), max_n,
                                       _dev_ptr(counts_out), stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_codec_decode_static")


def mv_quant_scratch_bytes(n: int, rows: int, q: int) -> int:
    return int(load().mv_quant_scratch_bytes(n, rows, q))


def mv_quant_encode(vals, q: int, streams, means, scratch, stream=None) -> None:
    """vals: rows x n float32 device tensor; streams: rows x ld_words int32 (out);
    means: rows x 2**(q-1) float32 (out)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(vals.device)
    st = load().mv_quant_encode(_dev_ptr(vals), vals.stride(0), vals.shape[1], vals.shape[0], q, _dev_ptr(streams),
                                streams.stride(0), _dev_ptr(means), _dev_ptr(scratch),
                                scratch.numel() * scratch.element_size(), stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_quant_encode")


def mv_quant_decode(streams, n: int, q: int, means, out, stream=None) -> None:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(out.device)
    st = load().mv_quant_decode(_dev_ptr(streams), streams.stride(0), n, streams.shape[0], q, _dev_ptr(means),
                                _dev_ptr(out), out.stride(0), stream.cuda_stream)
    if st != MV_OK:
        raise MvError(st, "mv_quant_decode")
