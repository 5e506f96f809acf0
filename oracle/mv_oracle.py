"""ctypes front end of the CPU oracle (oracle/mv_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
benchmark's cpu_baseline leg import this module.  It never imports the HIP
package and the HIP package never imports it.

All arrays are numpy arrays on the host.  Function names follow the steps of
Algorithm 1 of the paper (error compensation, local top-K mask, vote count,
global mask, aggregate, error update).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mv_oracle.c")
_LIB = os.path.join(_HERE, "libmv_oracle.so")

# No -ffast-math, no contraction: the oracle's fp32 arithmetic must be the
# plain IEEE operations the paper's 32-bit values imply.
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *_CFLAGS, _SRC, "-o", tmp, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i32, i64, vp, dbl = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_double
        L.mvo_widen_bf16.argtypes = [vp, vp, i64]
        L.mvo_widen_bf16.restype = None
        L.mvo_error_compensate.argtypes = [vp, vp, vp, i64]
        L.mvo_error_compensate.restype = None
        L.mvo_row_topk.argtypes = [vp, i64, i64, vp]
        L.mvo_row_topk.restype = i32
        L.mvo_votes.argtypes = [vp, i32, i64, i64, vp]
        L.mvo_votes.restype = i32
        L.mvo_mask.argtypes = [vp, i64, i64, vp]
        L.mvo_mask.restype = i32
        L.mvo_aggregate.argtypes = [vp, i64, i32, vp, i64, i32, vp]
        L.mvo_aggregate.restype = None
        L.mvo_error_update.argtypes = [vp, i64, vp, i64, vp]
        L.mvo_error_update.restype = None
        L.mvo_vote_step.argtypes = [vp, i64, i32, vp, i64, i32, i64, i64, i32, vp, vp, vp, vp, i32]
        L.mvo_vote_step.restype = i32
        L.mvo_rs_mask_draws.argtypes = [vp, i64, i64, vp, i64, vp]
        L.mvo_rs_mask_draws.restype = i64
        L.mvo_rs_mask_keys.argtypes = [vp, i64, i64, vp, vp]
        L.mvo_rs_mask_keys.restype = i32
        L.mvo_rs_vote_step.argtypes = [vp, i64, i32, vp, i64, i32, i64, i64, i32, vp, vp, vp, vp, vp, i32]
        L.mvo_rs_vote_step.restype = i32
        L.mvo_ad_vote_step.argtypes = [vp, i64, i32, vp, i64, i32, i64, i64, i64, i32, vp, vp, vp, vp, vp, vp, vp,
                                       vp, vp, i32]
        L.mvo_ad_vote_step.restype = i32
        L.mvo_codec_offset_bits.argtypes = [i64]
        L.mvo_codec_offset_bits.restype = i32
        L.mvo_codec_encode.argtypes = [vp, i64, i64, i64, vp, i64]
        L.mvo_codec_encode.restype = i64
        L.mvo_codec_decode.argtypes = [vp, i64, i64, i64, vp, i64]
        L.mvo_codec_decode.restype = i64
        L.mvo_quant_edges.argtypes = [vp, i64, i32, vp]
        L.mvo_quant_edges.restype = i32
        L.mvo_quant_encode.argtypes = [vp, i64, i32, vp, vp]
        L.mvo_quant_encode.restype = i32
        L.mvo_quant_decode.argtypes = [vp, i64, i32, vp, vp]
        L.mvo_quant_decode.restype = None
        L.mvo_quant_pack.argtypes = [vp, i64, i32, vp]
        L.mvo_quant_pack.restype = None
        L.mvo_bits_per_position.argtypes = [dbl]
        L.mvo_bits_per_position.restype = i32
        L.mvo_q_val.argtypes = [dbl, dbl, dbl]
        L.mvo_q_val.restype = dbl
        L.mvo_q_loc.argtypes = [dbl, dbl]
        L.mvo_q_loc.restype = dbl
        L.mvo_compression.argtypes = [dbl, dbl]
        L.mvo_compression.restype = dbl
        L.mvo_max_threads.argtypes = []
        L.mvo_max_threads.restype = i32
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ---------------------------------------------------------------- steps

def widen_bf16(g_bf16: np.ndarray) -> np.ndarray:
    g = _c(g_bf16, np.uint16)
    out = np.empty(g.shape, np.float32)
    lib().mvo_widen_bf16(_ptr(g), _ptr(out), g.size)
    return out


def error_compensate(delta: np.ndarray, e: np.ndarray) -> np.ndarray:
    delta, e = _c(delta, np.float32), _c(e, np.float32)
    assert delta.shape == e.shape
    out = np.empty_like(delta)
    lib().mvo_error_compensate(_ptr(delta), _ptr(e), _ptr(out), delta.size)
    return out


def row_topk(delta_bar_row: np.ndarray, K: int) -> np.ndarray:
    row = _c(delta_bar_row, np.float32)
    assert row.ndim == 1
    idx = np.empty(K, np.uint32)
    rc = lib().mvo_row_topk(_ptr(row), row.size, K, _ptr(idx))
    if rc != 0:
        raise ValueError("mvo_row_topk rejected its arguments")
    return idx


def votes(worker_idx: np.ndarray, d: int) -> np.ndarray:
    w = _c(worker_idx, np.uint32)
    assert w.ndim == 2
    out = np.empty(d, np.uint8)
    rc = lib().mvo_votes(_ptr(w), w.shape[0], w.shape[1], d, _ptr(out))
    if rc != 0:
        raise ValueError("mvo_votes rejected its arguments")
    return out


def mask(votes_: np.ndarray, K: int) -> np.ndarray:
    v = _c(votes_, np.uint8)
    out = np.empty(K, np.uint32)
    rc = lib().mvo_mask(_ptr(v), v.size, K, _ptr(out))
    if rc != 0:
        raise ValueError("mvo_mask rejected its arguments")
    return out


def aggregate(delta_bar: np.ndarray, mask_idx: np.ndarray, reduce_mean: bool = True) -> np.ndarray:
    a = _c(delta_bar, np.float32)
    m = _c(mask_idx, np.uint32)
    assert a.ndim == 2
    out = np.empty(m.size, np.float32)
    lib().mvo_aggregate(_ptr(a), a.shape[1], a.shape[0], _ptr(m), m.size, int(reduce_mean), _ptr(out))
    return out


def error_update(delta_bar_row: np.ndarray, mask_idx: np.ndarray) -> np.ndarray:
    a = _c(delta_bar_row, np.float32)
    m = _c(mask_idx, np.uint32)
    out = np.empty_like(a)
    lib().mvo_error_update(_ptr(a), a.size, _ptr(m), m.size, _ptr(out))
    return out


# ---------------------------------------------------------------- whole step

@dataclass
class StepResult:
    worker_idx: np.ndarray  # N x K uint32, rows ascending
    votes: np.ndarray       # d uint8
    mask_idx: np.ndarray    # K uint32 ascending
    agg: np.ndarray         # K float32
    err: np.ndarray         # N x d float32 (e_{t+1})


def vote_step(grads: np.ndarray, err: np.ndarray, K: int, reduce_mean: bool = True,
              threads: int = 1) -> StepResult:
    """One vote step.  grads: N x d float32, or uint16 holding bf16 patterns.
    err: N x d float32 (not modified; the new error buffer is returned)."""
    assert grads.ndim == 2 and err.shape == grads.shape
    is_bf16 = grads.dtype == np.uint16
    g = _c(grads, np.uint16 if is_bf16 else np.float32)
    e = np.array(err, dtype=np.float32, order="C", copy=True)
    N, d = g.shape
    widx = np.empty((N, K), np.uint32)
    v = np.empty(d, np.uint8)
    m = np.empty(K, np.uint32)
    agg = np.empty(K, np.float32)
    rc = lib().mvo_vote_step(_ptr(g), d, int(is_bf16), _ptr(e), d, N, d, K, int(reduce_mean),
                             _ptr(widx), _ptr(v), _ptr(m), _ptr(agg), int(threads))
    if rc != 0:
        raise ValueError("mvo_vote_step rejected its arguments")
    return StepResult(widx, v, m, agg, e)


# ---------------------------------------------------------------- random selection (Algorithm 1, S_rand-weighted)

def rs_mask_draws(votes: np.ndarray, K: int, u: np.ndarray):
    """The sequential sampler: draws positions in proportion to their votes, with the
    uniform numbers u, until K distinct ones are selected.  Returns (mask ascending,
    draws used)."""
    v = _c(votes, np.uint8)
    uu = _c(u, np.float64)
    m = np.empty(K, np.uint32)
    used = lib().mvo_rs_mask_draws(_ptr(v), v.size, K, _ptr(uu), uu.size, _ptr(m))
    if used < 0:
        raise ValueError("mvo_rs_mask_draws: bad arguments, fewer than K voted positions or too few numbers")
    return m, int(used)


def rs_mask_keys(votes: np.ndarray, K: int, rand_exp: np.ndarray) -> np.ndarray:
    """The K voted positions whose exponential clocks rand_exp[j] / votes[j] ring first."""
    v = _c(votes, np.uint8)
    r = _c(rand_exp, np.float32)
    assert r.size == v.size
    m = np.empty(K, np.uint32)
    if lib().mvo_rs_mask_keys(_ptr(v), v.size, K, _ptr(r), _ptr(m)) != 0:
        raise ValueError("mvo_rs_mask_keys: bad arguments or fewer than K voted positions")
    return m


def rs_vote_step(grads: np.ndarray, err: np.ndarray, K: int, rand_exp: np.ndarray, reduce_mean: bool = True,
                 threads: int = 1) -> StepResult:
    """One vote step whose mask is selected at random in proportion to the votes."""
    assert grads.ndim == 2 and err.shape == grads.shape
    is_bf16 = grads.dtype == np.uint16
    g = _c(grads, np.uint16 if is_bf16 else np.float32)
    e = np.array(err, dtype=np.float32, order="C", copy=True)
    N, d = g.shape
    r = _c(rand_exp, np.float32)
    assert r.size == d
    widx = np.empty((N, K), np.uint32)
    v = np.empty(d, np.uint8)
    m = np.empty(K, np.uint32)
    agg = np.empty(K, np.float32)
    rc = lib().mvo_rs_vote_step(_ptr(g), d, int(is_bf16), _ptr(e), d, N, d, K, int(reduce_mean), _ptr(r),
                                _ptr(widx), _ptr(v), _ptr(m), _ptr(agg), int(threads))
    if rc != 0:
        raise ValueError("mvo_rs_vote_step rejected its arguments")
    return StepResult(widx, v, m, agg, e)


# ---------------------------------------------------------------- add-drop voting (Algorithm 2)

@dataclass
class AdStepResult:
    worker_idx: np.ndarray  # N x K uint32: supp(M_n), ascending
    add_idx: list           # per worker: ascending uint32 array of the added positions
    drop_idx: list          # per worker: ascending uint32 array of the dropped positions
    vote: np.ndarray        # N x d uint8 0/1: M~_{n,t}
    msum: np.ndarray        # d uint8: M^sum_t
    mask_idx: np.ndarray
    agg: np.ndarray
    err: np.ndarray


def ad_vote_step(grads: np.ndarray, err: np.ndarray, K: int, K_ad: int, vote: np.ndarray, msum: np.ndarray,
                 reduce_mean: bool = True, threads: int = 1) -> AdStepResult:
    """One iteration of majority voting with add-drop.  `vote` (N x d, 0/1) and
    `msum` (d) are the state before the step; they are not modified, the new
    state is returned."""
    assert grads.ndim == 2 and err.shape == grads.shape
    is_bf16 = grads.dtype == np.uint16
    g = _c(grads, np.uint16 if is_bf16 else np.float32)
    e = np.array(err, dtype=np.float32, order="C", copy=True)
    N, d = g.shape
    vt = np.array(vote, dtype=np.uint8, order="C", copy=True).reshape(N, d)
    ms = np.array(msum, dtype=np.uint8, order="C", copy=True).reshape(d)
    widx = np.empty((N, K), np.uint32)
    add = np.zeros((N, K_ad), np.uint32)
    drop = np.zeros((N, K_ad), np.uint32)
    n_add = np.zeros(N, np.int64)
    n_drop = np.zeros(N, np.int64)
    m = np.empty(K, np.uint32)
    agg = np.empty(K, np.float32)
    rc = lib().mvo_ad_vote_step(_ptr(g), d, int(is_bf16), _ptr(e), d, N, d, K, K_ad, int(reduce_mean),
                                _ptr(vt), _ptr(ms), _ptr(widx), _ptr(add), _ptr(drop), _ptr(n_add),
                                _ptr(n_drop), _ptr(m), _ptr(agg), int(threads))
    if rc != 0:
        raise ValueError("mvo_ad_vote_step rejected its arguments or state")
    return AdStepResult(widx, [add[n, : n_add[n]].copy() for n in range(N)],
                        [drop[n, : n_drop[n]].copy() for n in range(N)], vt, ms, m, agg, e)


# ---------------------------------------------------------------- sparse position code (Sec. 4.3.1)

def codec_offset_bits(block_len: int) -> int:
    return int(lib().mvo_codec_offset_bits(int(block_len)))


def codec_stream_bits(n: int, d: int, block_len: int) -> int:
    """Length of the stream of n positions: n (1 + B) + number of blocks."""
    return n * (1 + codec_offset_bits(block_len)) + (d + block_len - 1) // block_len


def codec_encode(idx: np.ndarray, d: int, block_len: int):
    """Returns (words, n_bits): the stream as uint32 words, bit k = bit k % 32 of word k // 32."""
    idx = _c(idx, np.uint32)
    n_bits = codec_stream_bits(idx.size, d, block_len)
    words = np.zeros((n_bits + 31) // 32 + 1, np.uint32)
    got = lib().mvo_codec_encode(_ptr(idx), idx.size, d, block_len, _ptr(words), words.size)
    if got < 0:
        raise ValueError("mvo_codec_encode rejected its arguments")
    assert got == n_bits
    return words, int(got)


def codec_decode(words: np.ndarray, n_bits: int, d: int, block_len: int, max_n: int) -> np.ndarray:
    words = _c(words, np.uint32)
    out = np.empty(max(1, max_n), np.uint32)
    n = lib().mvo_codec_decode(_ptr(words), n_bits, d, block_len, _ptr(out), max_n)
    if n < 0:
        raise ValueError("mvo_codec_decode: malformed stream")
    return out[:n].copy()


# ---------------------------------------------------------------- fractional quantisation (Sec. 4.3.2)

def quant_edges(v: np.ndarray, q: int) -> np.ndarray:
    v = _c(v, np.float32)
    edges = np.zeros(1 << (q - 1), np.float64)
    if lib().mvo_quant_edges(_ptr(v), v.size, q, _ptr(edges)) != 0:
        raise ValueError("mvo_quant_edges rejected its arguments")
    return edges


def quant_encode(v: np.ndarray, q: int):
    """Returns (codes uint8, means float32[L]): code = (interval - 1) | sign << (q - 1)."""
    v = _c(v, np.float32)
    codes = np.zeros(v.size, np.uint8)
    means = np.zeros(1 << (q - 1), np.float32)
    if lib().mvo_quant_encode(_ptr(v), v.size, q, _ptr(codes), _ptr(means)) != 0:
        raise ValueError("mvo_quant_encode rejected its arguments")
    return codes, means


def quant_decode(codes: np.ndarray, q: int, means: np.ndarray) -> np.ndarray:
    codes, means = _c(codes, np.uint8), _c(means, np.float32)
    out = np.empty(codes.size, np.float32)
    lib().mvo_quant_decode(_ptr(codes), codes.size, q, _ptr(means), _ptr(out))
    return out


def quant_pack(codes: np.ndarray, q: int) -> np.ndarray:
    codes = _c(codes, np.uint8)
    words = np.zeros((codes.size * q + 31) // 32, np.uint32)
    lib().mvo_quant_pack(_ptr(codes), codes.size, q, _ptr(words))
    return words


# ---------------------------------------------------------------- comm load

def bits_per_position(inv_phi: float) -> int:
    return int(lib().mvo_bits_per_position(float(inv_phi)))


def q_val(q_bits: float, phi: float, d: float) -> float:
    return float(lib().mvo_q_val(q_bits, phi, d))


def q_loc(phi: float, d: float) -> float:
    return float(lib().mvo_q_loc(phi, d))


def compression(qbar_loc: float, qbar_val: float) -> float:
    return float(lib().mvo_compression(qbar_loc, qbar_val))


def max_threads() -> int:
    return int(lib().mvo_max_threads())
