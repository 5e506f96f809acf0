"""Parity of the GPU fractional quantiser (Sec. 4.3.2) against the oracle: the
packed codes bit-exact (the interval edges come from correctly rounded fp64
operations on both sides), the interval means and the reproduced values within
1e-6 relative (the means are fp64 sums whose grouping differs)."""
import sys

import numpy as np
import pytest
import torch

from paper_2011_06495_amd import binding as B
from paper_2011_06495_amd import workloads as W

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def gpu_quant(oracle, vals, q):
    rows, n = vals.shape
    L = 1 << (q - 1)
    dev = torch.device("cuda:0")
    v = torch.from_numpy(vals).to(dev)
    ld_words = (n * q + 31) // 32 + 2
    streams = torch.full((rows, ld_words), 0x5A5A5A5A, dtype=torch.int32, device=dev)
    means = torch.full((rows, L), -1.0, dtype=torch.float32, device=dev)
    scratch = torch.empty(B.mv_quant_scratch_bytes(n, rows, q), dtype=torch.uint8, device=dev)
    out = torch.full((rows, n + 4), 7.0, dtype=torch.float32, device=dev)
    B.mv_quant_encode(v, q, streams, means, scratch)
    B.mv_quant_decode(streams, n, q, means, out)
    torch.cuda.synchronize()
    sw = streams.cpu().numpy().view(np.uint32)
    mu = means.cpu().numpy()
    o = out.cpu().numpy()
    nw = (n * q + 31) // 32
    for r in range(rows):
        codes, ref_mu = oracle.quant_encode(vals[r], q)
        words = oracle.quant_pack(codes, q)
        assert np.array_equal(sw[r, :nw], words), "row %d codes" % r
        assert np.all(sw[r, nw:] == 0x5A5A5A5A)
        assert np.all(np.abs(mu[r] - ref_mu) <= 1e-6 * np.abs(ref_mu)), "row %d means" % r
        ref_out = oracle.quant_decode(codes, q, ref_mu)
        assert np.array_equal(np.signbit(o[r, :n]), np.signbit(ref_out))
        assert np.all(np.abs(o[r, :n] - ref_out) <= 1e-6 * np.abs(ref_out)), "row %d reproduction" % r
        assert np.all(o[r, n:] == 7.0)


@pytest.mark.parametrize("q", [2, 3, 4, 5, 8])
@pytest.mark.parametrize("n,rows", [(1, 1), (33, 3), (1000, 2), (11174, 4)])
def test_quant_random_values(oracle, q, n, rows):
    say("quant q=%d n=%d rows=%d" % (q, n, rows))
    rng = np.random.default_rng(q * 1000 + n)
    vals = (rng.standard_normal((rows, n)) * np.exp(rng.standard_normal((rows, n)))).astype(np.float32)
    if n > 20:
        vals[:, ::17] = 0.0
        vals[0, 5] = -0.0
    gpu_quant(oracle, vals, q)


def test_quant_degenerate_rows(oracle):
    say("quant degenerate")
    n = 300
    vals = np.zeros((4, n), np.float32)
    vals[1] = -2.5                                              # one magnitude
    vals[2, :] = np.where(np.arange(n) % 2, 4.0, 1.0)          # values exactly on the ends of the range
    vals[3] = np.float32(2.0) ** -np.arange(n, dtype=np.float32).clip(0, 100)   # many octaves
    for q in (2, 4):
        gpu_quant(oracle, vals, q)


def test_quant_on_the_values_a_vote_step_sends(oracle):
    """The uplink values of Algorithm 1: every worker's compensated vector on the
    global mask, quantised with the paper's q = 4."""
    w = W.C3.with_size(300007, N=8)
    say("quant on masked values N=%d K=%d" % (w.N, w.K))
    g, e = W.gradients(w, 0), W.zero_error(w)
    ref = oracle.vote_step(g, e, w.K)
    sent = np.ascontiguousarray((g + e)[:, ref.mask_idx].astype(np.float32))
    gpu_quant(oracle, sent, 4)
