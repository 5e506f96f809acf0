"""mv_codec_decode_static (the decoder on the library's own scratch array, for callers that
cannot allocate) against mv_codec_decode on the same streams: decoded lists and counts equal
element by element, on two calls in a row, the second on a smaller input; sizes beyond the
array are refused.  Collected last: it shares one process with the other GPU tests and must
pass after them as well as alone."""
import sys

import numpy as np
import pytest
import torch

from paper_2011_06495_amd import binding as B

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def encode_lists(rng, rows, n, d, block_len):
    dev = torch.device("cuda:0")
    idx = torch.full((rows, n), -1, dtype=torch.int32, device=dev)
    counts = torch.zeros(rows, dtype=torch.int32, device=dev)
    lists = []
    for r in range(rows):
        m = n if r == 0 else int(rng.integers(0, n + 1))
        l = np.sort(rng.choice(d, m, replace=False)).astype(np.uint32)
        lists.append(l)
        if m:
            idx[r, :m] = torch.from_numpy(l.astype(np.int64)).to(torch.int32)
        counts[r] = m
    max_bits = B.mv_codec_stream_bits(n, d, block_len)
    streams = torch.zeros((rows, (max_bits + 31) // 32 + 2), dtype=torch.int32, device=dev)
    n_bits = torch.zeros(rows, dtype=torch.int64, device=dev)
    B.mv_codec_encode(idx, n, d, block_len, streams, n_bits, counts=counts)
    torch.cuda.synchronize()
    return lists, streams, n_bits, max_bits


def decode_both_ways(rng, rows, n, d, block_len):
    dev = torch.device("cuda:0")
    lists, streams, n_bits, max_bits = encode_lists(rng, rows, n, d, block_len)
    need = B.mv_codec_scratch_bytes(max_bits, rows)
    assert need <= B.MV_CODEC_STATIC_SCRATCH_BYTES
    # every buffer exists before the call under test, which must not allocate
    out_a = torch.full((rows, n + 8), -1, dtype=torch.int32, device=dev)
    out_b = torch.full((rows, n + 8), -1, dtype=torch.int32, device=dev)
    cnt_a = torch.full((rows,), -7, dtype=torch.int32, device=dev)
    cnt_b = torch.full((rows,), -7, dtype=torch.int32, device=dev)
    scratch = torch.empty(need, dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    held = torch.cuda.memory_allocated(dev), torch.cuda.memory_reserved(dev)
    B.mv_codec_decode_static(streams, n_bits, max_bits, d, block_len, out_b, n, cnt_b)
    torch.cuda.synchronize()
    assert (torch.cuda.memory_allocated(dev), torch.cuda.memory_reserved(dev)) == held
    B.mv_codec_decode(streams, n_bits, max_bits, d, block_len, out_a, n, cnt_a, scratch)
    torch.cuda.synchronize()
    a, b = out_a.cpu().numpy().view(np.uint32), out_b.cpu().numpy().view(np.uint32)
    ca, cb = cnt_a.cpu().numpy(), cnt_b.cpu().numpy()
    assert np.array_equal(ca, cb), "counts differ: %s / %s" % (ca, cb)
    assert np.array_equal(a, b), "decoded lists differ in rows %s" % np.flatnonzero((a != b).any(axis=1))[:8]
    for r, l in enumerate(lists):                       # and both are the lists that were encoded
        assert cb[r] == l.size and np.array_equal(b[r, : l.size], l), "row %d" % r
        assert np.all(b[r, l.size:] == 0xFFFFFFFF)


def test_decode_on_the_static_scratch_matches_decode_on_a_buffer_twice_in_a_row():
    rng = np.random.default_rng(20)
    say("static scratch: 16 rows of 11174 positions among 11173962, blocks of 1000")
    decode_both_ways(rng, 16, 11174, 11_173_962, 1000)
    say("static scratch: 3 rows of 500 positions among 70001, blocks of 128 (smaller, right after)")
    decode_both_ways(rng, 3, 500, 70001, 128)
    say("static scratch: 1 row, 1 position")
    decode_both_ways(rng, 1, 1, 1, 1)


def test_sizes_beyond_the_static_scratch_are_refused_and_nothing_runs():
    dev = torch.device("cuda:0")
    rows, n, d, block_len = 64, 200_000, 100_000_000, 1000
    max_bits = B.mv_codec_stream_bits(n, d, block_len)
    assert B.mv_codec_scratch_bytes(max_bits, rows) > B.MV_CODEC_STATIC_SCRATCH_BYTES
    ld_words = (max_bits + 31) // 32
    streams = torch.zeros((rows, ld_words), dtype=torch.int32, device=dev)
    n_bits = torch.zeros(rows, dtype=torch.int64, device=dev)
    out = torch.full((rows, n), -1, dtype=torch.int32, device=dev)
    cnt = torch.full((rows,), -7, dtype=torch.int32, device=dev)
    with pytest.raises(B.MvError) as err:
        B.mv_codec_decode_static(streams, n_bits, max_bits, d, block_len, out, n, cnt)
    assert err.value.status == B.MV_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert int(cnt.min()) == -7 and int(cnt.max()) == -7 and int(out.max()) == -1
    with pytest.raises(B.MvError) as err:                # the argument checks of mv_codec_decode apply
        B.mv_codec_decode_static(streams, n_bits, max_bits, d, 0, out, n, cnt)
    assert err.value.status == B.MV_ERR_INVALID_ARG
