"""Parity of mv_ad_vote_step (majority voting with add-drop, Algorithm 2) against
the oracle: added and dropped coordinate lists, the standing votes, the cumulative
vote sum, the mask, the aggregate and the error buffer, every step of a sequence
with the state carried on the device."""
import sys

import numpy as np
import pytest
import torch

from paper_2011_06495_amd import binding as B
from paper_2011_06495_amd import workloads as W
from tests.gpu_util import GUARD, SENTINEL_F32, SENTINEL_U32, round_up

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


class GpuAdStepper:
    def __init__(self, N, d, K, k_ad_max, bf16=False):
        self.N, self.d, self.K, self.k_ad_max, self.bf16 = N, d, K, k_ad_max, bf16
        dev = torch.device("cuda:0")
        self.ld_g = round_up(d, 8 if bf16 else 4)
        self.ld_e = round_up(d, 4)
        self.ld_bits = round_up((d + 31) // 32, 4)
        self.g = torch.zeros((N, self.ld_g), dtype=torch.int16 if bf16 else torch.float32, device=dev)
        self.e = torch.full((N, self.ld_e), SENTINEL_F32, dtype=torch.float32, device=dev)
        self.e[:, :d] = 0
        self.bits = torch.zeros((N, self.ld_bits), dtype=torch.int32, device=dev)
        self.msum = torch.zeros(round_up(d, 16), dtype=torch.uint8, device=dev)
        self.add = torch.full((N * k_ad_max + GUARD,), SENTINEL_U32 - (1 << 32), dtype=torch.int32, device=dev)
        self.drop = torch.full((N * k_ad_max + GUARD,), SENTINEL_U32 - (1 << 32), dtype=torch.int32, device=dev)
        self.counts = torch.zeros(2 * N, dtype=torch.int32, device=dev)
        self.mask = torch.full((K + GUARD,), SENTINEL_U32 - (1 << 32), dtype=torch.int32, device=dev)
        self.agg = torch.full((K + GUARD,), SENTINEL_F32, dtype=torch.float32, device=dev)
        self.ctx = B.mv_begin(B.make_config(N, d, K, B.MV_BF16 if bf16 else B.MV_F32, flags=B.MV_FLAG_ADD_DROP))

    def step(self, g_host, k_ad):
        if self.bf16:
            t = torch.from_numpy(np.ascontiguousarray(g_host, np.uint16).view(np.int16))
        else:
            t = torch.from_numpy(np.ascontiguousarray(g_host, np.float32))
        self.g[:, : self.d].copy_(t)
        self.k_ad = k_ad
        B.mv_ad_vote_step(self.ctx, self.g, self.e, k_ad, self.bits, self.msum, self.add, self.drop, self.counts,
                          self.mask, self.agg, ld_g=self.ld_g, ld_e=self.ld_e)
        torch.cuda.synchronize()

    def compare(self, ref, what):
        N, d, K, k_ad = self.N, self.d, self.K, self.k_ad
        counts = self.counts.cpu().numpy().astype(np.int64)
        add = self.add.cpu().numpy().view(np.uint32)
        drop = self.drop.cpu().numpy().view(np.uint32)
        assert np.all(add[N * self.k_ad_max:] == SENTINEL_U32) and np.all(drop[N * self.k_ad_max:] == SENTINEL_U32)
        for n in range(N):
            na, nd = counts[2 * n], counts[2 * n + 1]
            assert na == ref.add_idx[n].size and nd == ref.drop_idx[n].size, "%s row %d counts" % (what, n)
            assert np.array_equal(add[n * k_ad: n * k_ad + na], ref.add_idx[n]), "%s row %d add list" % (what, n)
            assert np.array_equal(drop[n * k_ad: n * k_ad + nd], ref.drop_idx[n]), "%s row %d drop list" % (what, n)
        bits = self.bits.cpu().numpy().view(np.uint32)
        vote = np.unpackbits(bits.view(np.uint8), axis=1, bitorder="little")[:, :d]
        assert np.array_equal(vote, ref.vote), "%s standing votes" % what
        assert not np.unpackbits(bits.view(np.uint8), axis=1, bitorder="little")[:, d:].any()
        ms = self.msum.cpu().numpy()
        assert np.array_equal(ms[:d], ref.msum) and not ms[d:].any(), "%s msum" % what
        m = self.mask.cpu().numpy().view(np.uint32)
        assert np.all(m[K:] == SENTINEL_U32)
        assert np.array_equal(m[:K], ref.mask_idx), "%s mask" % what
        a = self.agg.cpu().numpy()
        assert np.array_equal(a[:K].view(np.uint32), ref.agg.view(np.uint32)), "%s agg" % what
        e = self.e.cpu().numpy()
        assert np.all(e[:, d:] == np.float32(SENTINEL_F32))
        assert np.array_equal(e[:, :d].view(np.uint32), ref.err.view(np.uint32)), "%s err" % what

    def close(self):
        B.mv_end(self.ctx)
        B.mv_release(self.ctx)


def run_ad_sequence(oracle, w, k_ads, threads=8, spin_limit=None):
    k_ad_max = max(k_ads)
    gs = GpuAdStepper(w.N, w.d, w.K, k_ad_max, bf16=(w.grad_dtype == "bf16"))
    try:
        if spin_limit is not None:
            B.mv_set_spin_limit(gs.ctx, spin_limit)
        vote = np.zeros((w.N, w.d), np.uint8)
        msum = np.zeros(w.d, np.uint8)
        e = W.zero_error(w)
        for t, k_ad in enumerate(k_ads):
            g = W.gradients(w, t, threads=threads)
            gs.step(g, k_ad)
            ref = oracle.ad_vote_step(g, e, w.K, k_ad, vote, msum, threads=threads)
            gs.compare(ref, "%s step %d k_ad %d" % (w.name, t, k_ad))
            vote, msum, e = ref.vote, ref.msum, ref.err
    finally:
        gs.close()


@pytest.mark.parametrize("name,d,N", [("C2", 150007, 6), ("C4", 200003, 8), ("C5", 120005, 5), ("C3", 257003, 7)])
def test_add_drop_reduced_workloads(oracle, name, d, N):
    kw = dict(lattice_shift=6) if name == "C4" else {}
    w = W.WORKLOADS[name].with_size(d, N=N, K=max(40, d // 500), **kw)
    k_ad = max(1, w.K // 10)
    say("add-drop %s N=%d d=%d K=%d K_ad=%d" % (name, w.N, w.d, w.K, k_ad))
    # from the empty state: small steps first (the mask reaches into unvoted coordinates),
    # then a full vote, then the paper's regime phi_ad = phi / 10
    run_ad_sequence(oracle, w, [k_ad, k_ad, w.K, k_ad, k_ad, 1, k_ad])


def test_add_drop_when_nothing_waits_for_anything(oracle):
    """No polls allowed: rows whose threshold is not seen at the first look are selected from memory,
    and the mask is found from the blocks' counts by the last kernel (with few votes standing, the
    mask's vote level is 0 and reaches over many blocks).  Same results."""
    w = W.C2.with_size(150007, N=6, K=300)
    say("add-drop without polls N=%d d=%d K=%d" % (w.N, w.d, w.K))
    run_ad_sequence(oracle, w, [30, 30, w.K, 30, 1], spin_limit=0)


@pytest.mark.parametrize("d,K,N", [(1, 1, 1), (33, 5, 2), (1025, 40, 3), (4099, 4099, 2), (70001, 700, 4)])
def test_add_drop_edge_shapes(oracle, d, K, N):
    say("add-drop edge d=%d K=%d N=%d" % (d, K, N))
    rng = np.random.default_rng(d + K)
    gs = GpuAdStepper(N, d, K, K)
    try:
        vote = np.zeros((N, d), np.uint8)
        msum = np.zeros(d, np.uint8)
        e = np.zeros((N, d), np.float32)
        for t, k_ad in enumerate([K, max(1, K // 7), 1, K]):
            g = rng.standard_normal((N, d)).astype(np.float32)
            gs.step(g, k_ad)
            ref = oracle.ad_vote_step(g, e, K, k_ad, vote, msum)
            gs.compare(ref, "edge step %d" % t)
            vote, msum, e = ref.vote, ref.msum, ref.err
    finally:
        gs.close()


def test_add_drop_degenerate_rows(oracle):
    """Rows of equal magnitudes: the row's top-K comes from memory; ties decide
    everything, lowest coordinate first."""
    N, d, K, k_ad = 3, 90001, 300, 30
    say("add-drop degenerate N=%d d=%d K=%d" % (N, d, K))
    rng = np.random.default_rng(3)
    gs = GpuAdStepper(N, d, K, K)
    try:
        vote = np.zeros((N, d), np.uint8)
        msum = np.zeros(d, np.uint8)
        e = np.zeros((N, d), np.float32)
        for t in range(4):
            g = np.zeros((N, d), np.float32)
            g[0] = 1.5 if t % 2 == 0 else rng.choice(np.array([1.0, 2.0], np.float32), size=d)
            g[1] = rng.standard_normal(d).astype(np.float32)
            g[2] = rng.choice(np.array([-1.0, 1.0, 3.0], np.float32), size=d)
            e[:] = 0                                   # frozen scale: keep the rows degenerate
            gs.e[:, :d] = 0
            gs.step(g, k_ad)
            ref = oracle.ad_vote_step(g, e, K, k_ad, vote, msum)
            gs.compare(ref, "degenerate step %d" % t)
            vote, msum = ref.vote, ref.msum
    finally:
        gs.close()


def test_add_drop_with_infinite_magnitudes(oracle):
    """Infinities order above every finite magnitude in the additions (largest first) and in the
    removals (smallest first); at a coordinate all workers' infinities have one sign, so no NaN arises."""
    N, d, K, k_ad = 3, 60001, 400, 40
    say("add-drop infinities N=%d d=%d K=%d K_ad=%d" % (N, d, K, k_ad))
    rng = np.random.default_rng(31)
    sign = np.where(rng.integers(0, 2, size=d) == 1, np.float32(np.inf), np.float32(-np.inf))
    gs = GpuAdStepper(N, d, K, K)
    try:
        vote = np.zeros((N, d), np.uint8)
        msum = np.zeros(d, np.uint8)
        e = np.zeros((N, d), np.float32)
        for t, ka in enumerate([K, k_ad, k_ad, k_ad]):
            g = rng.standard_normal((N, d)).astype(np.float32)
            if t in (0, 2):                                   # new infinities while the standing votes move
                hot = rng.choice(d, size=60, replace=False)
                g[t % N, hot] = sign[hot]
                g[(t + 1) % N, hot[:20]] = sign[hot[:20]]
            gs.step(g, ka)
            ref = oracle.ad_vote_step(g, e, K, ka, vote, msum)
            assert not np.isnan(ref.err).any() and not np.isnan(ref.agg).any()
            gs.compare(ref, "infinities step %d" % t)
            vote, msum, e = ref.vote, ref.msum, ref.err
        assert np.isinf(e).any() or np.isinf(ref.agg).any()
    finally:
        gs.close()


def test_add_drop_needs_the_flag_and_valid_arguments():
    ctx = B.mv_begin(B.make_config(2, 1000, 10))
    dev = torch.device("cuda:0")
    g = torch.zeros((2, 1000), device=dev)
    e = torch.zeros((2, 1000), device=dev)
    bits = torch.zeros((2, 32), dtype=torch.int32, device=dev)
    msum = torch.zeros(1008, dtype=torch.uint8, device=dev)
    out = torch.zeros(64, dtype=torch.int32, device=dev)
    agg = torch.zeros(16, device=dev)
    with pytest.raises(B.MvError) as ei:
        B.mv_ad_vote_step(ctx, g, e, 2, bits, msum, out, out, out, out, agg)
    assert ei.value.status == B.MV_ERR_STATE
    B.mv_end(ctx)
    B.mv_release(ctx)
    ctx = B.mv_begin(B.make_config(2, 1000, 10, flags=B.MV_FLAG_ADD_DROP))
    for k_ad in (0, 11):
        with pytest.raises(B.MvError) as ei:
            B.mv_ad_vote_step(ctx, g, e, k_ad, bits, msum, out, out, out, out, agg)
        assert ei.value.status == B.MV_ERR_INVALID_ARG
    small_bits = torch.zeros((2, 28), dtype=torch.int32, device=dev)
    with pytest.raises(B.MvError):
        B.mv_ad_vote_step(ctx, g, e, 2, small_bits, msum, out, out, out, out, agg)
    B.mv_end(ctx)
    B.mv_release(ctx)
