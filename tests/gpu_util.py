"""Helpers of the GPU parity tests: device buffers with guard bands, one call of
the HIP path through the C ABI, and element-by-element comparison with the
oracle's result."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from paper_2011_06495_amd import binding as B

GUARD = 64            # guard elements after every output buffer
SENTINEL_U32 = 0xDEADBEEF
SENTINEL_F32 = -12345.5


def round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


@dataclass
class GpuOut:
    worker_idx: np.ndarray
    votes: np.ndarray
    mask_idx: np.ndarray
    agg: np.ndarray
    err: np.ndarray


class GpuStepper:
    """Owns a context and the device buffers of one (N, d, K) problem."""

    def __init__(self, N: int, d: int, K: int, bf16: bool = False, reduce: int = B.MV_REDUCE_MEAN,
                 extra_ld: int = 0, own_workspace: bool = False, want_worker_idx: bool = True,
                 want_votes: bool = True):
        self.N, self.d, self.K, self.bf16 = N, d, K, bf16
        dev = torch.device("cuda:0")
        self.dev = dev
        self.ld_g = round_up(d, 8 if bf16 else 4) + extra_ld * (8 if bf16 else 4)
        self.ld_e = round_up(d, 4) + extra_ld * 4
        self.g = torch.zeros((N, self.ld_g), dtype=torch.int16 if bf16 else torch.float32, device=dev)
        self.e = torch.full((N, self.ld_e), SENTINEL_F32, dtype=torch.float32, device=dev)
        self.widx = torch.full((N * K + GUARD,), SENTINEL_U32 - (1 << 32), dtype=torch.int32, device=dev) \
            if want_worker_idx else None
        self.votes = torch.full((d + GUARD,), 0x5A, dtype=torch.uint8, device=dev) if want_votes else None
        self.mask = torch.full((K + GUARD,), SENTINEL_U32 - (1 << 32), dtype=torch.int32, device=dev)
        self.agg = torch.full((K + GUARD,), SENTINEL_F32, dtype=torch.float32, device=dev)
        cfg = B.make_config(N, d, K, B.MV_BF16 if bf16 else B.MV_F32, reduce)
        self.ws = None
        if own_workspace:
            nbytes = B.mv_workspace_bytes(cfg)
            assert nbytes > 0
            self.ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
            base = round_up(self.ws.data_ptr(), 256)
            cfg = B.make_config(N, d, K, B.MV_BF16 if bf16 else B.MV_F32, reduce,
                                workspace=base, workspace_bytes=nbytes)
        self.ctx = B.mv_begin(cfg)

    def set_error(self, e_host: np.ndarray) -> None:
        self.e[:, : self.d].copy_(torch.from_numpy(np.ascontiguousarray(e_host, np.float32)))

    def set_grads(self, g_host: np.ndarray) -> None:
        if self.bf16:
            t = torch.from_numpy(np.ascontiguousarray(g_host, np.uint16).view(np.int16))
        else:
            t = torch.from_numpy(np.ascontiguousarray(g_host, np.float32))
        self.g[:, : self.d].copy_(t)

    def step(self, stream=None) -> None:
        B.mv_vote_step(self.ctx, self.g, self.e, self.widx, self.votes, self.mask, self.agg,
                       stream=stream, ld_g=self.ld_g, ld_e=self.ld_e)

    def step_rs(self, rand_exp_host: np.ndarray, stream=None) -> None:
        """One step of majority voting with random selection with the given Exp(1) numbers."""
        r = torch.from_numpy(np.ascontiguousarray(rand_exp_host, np.float32)).to(self.dev)
        assert r.numel() == self.d
        B.mv_rs_vote_step(self.ctx, self.g, self.e, r, self.widx, self.votes, self.mask, self.agg,
                          stream=stream, ld_g=self.ld_g, ld_e=self.ld_e)
        torch.cuda.synchronize()          # r must outlive the step

    def fetch(self, check_guards: bool = True) -> GpuOut:
        torch.cuda.synchronize()
        N, d, K = self.N, self.d, self.K
        widx = None
        if self.widx is not None:
            w = self.widx.cpu().numpy().view(np.uint32)
            if check_guards:
                assert np.all(w[N * K:] == SENTINEL_U32), "write past the end of worker_idx"
            widx = w[: N * K].reshape(N, K).copy()
        votes = None
        if self.votes is not None:
            v = self.votes.cpu().numpy()
            if check_guards:
                assert np.all(v[d:] == 0x5A), "write past the end of votes"
            votes = v[:d].copy()
        m = self.mask.cpu().numpy().view(np.uint32)
        a = self.agg.cpu().numpy()
        e = self.e.cpu().numpy()
        if check_guards:
            assert np.all(m[K:] == SENTINEL_U32), "write past the end of mask_idx"
            assert np.all(a[K:] == np.float32(SENTINEL_F32)), "write past the end of agg_vals"
            assert np.all(e[:, d:] == np.float32(SENTINEL_F32)), "write into the row padding of err"
        return GpuOut(widx, votes, m[:K].copy(), a[:K].copy(), e[:, :d].copy())

    def row_stats(self):
        return B.mv_last_step_row_stats(self.ctx, self.N)

    def close(self) -> None:
        if self.ctx:
            B.mv_end(self.ctx)
            B.mv_release(self.ctx)
            self.ctx = 0

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def assert_matches_oracle(got: GpuOut, ref, what: str = "") -> None:
    """Bit-exact on index sets, votes, mask, error buffer; the aggregate is
    bit-exact too because both sides sum the workers in order 0..N-1 in fp32."""
    if got.worker_idx is not None:
        bad = np.flatnonzero((got.worker_idx != ref.worker_idx).any(axis=1))
        assert bad.size == 0, "%s worker_idx differs in rows %s" % (what, bad[:8])
    if got.votes is not None:
        assert np.array_equal(got.votes, ref.votes), "%s votes differ" % what
    assert np.array_equal(got.mask_idx, ref.mask_idx), "%s mask differs" % what
    assert np.array_equal(got.err.view(np.uint32), ref.err.view(np.uint32)), "%s error buffer differs" % what
    # spec tolerance: 1e-6 relative; with the summation order fixed it is exact
    fin = np.isfinite(ref.agg)                            # an infinite aggregate is compared by its bits below
    scale = np.maximum(np.abs(ref.agg[fin]), np.finfo(np.float32).tiny)
    assert np.all(np.abs(got.agg[fin].astype(np.float64) - ref.agg[fin]) <= 1e-6 * scale), "%s agg beyond 1e-6" % what
    assert np.array_equal(got.agg.view(np.uint32), ref.agg.view(np.uint32)), "%s agg not bit-exact" % what
