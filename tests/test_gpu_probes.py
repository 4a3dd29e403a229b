"""The measurement aids of the library (no part of the method): the two read-only streaming probes fold every
word they read into their sums, the MFMA probe issues the number of matrix instructions it says, and all three
turn malformed calls into error codes on the host."""
import pytest
import torch

from paper_2605_22566_amd import binding as B
from paper_2605_22566_amd import runner as R
from paper_2605_22566_amd import workload as W

pytestmark = pytest.mark.gpu


def _session():
    return R.Session(W.small_layered(1, W.Shape(8, 2, 128), num_req=1))


def _code(fn):
    with pytest.raises(B.GraphFlowError) as e:
        fn()
    return e.value.code


def _word_sum(sums):
    return int(sums.to(torch.int64).sum().item()) & 0xffffffff


def test_read_probes_sum_every_word():
    sess = _session()
    dev = sess.device
    nbytes = (3 << 20) + 4096 + 16                       # no multiple of the grid's footprint: the tail loop runs
    words = torch.randint(0, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, device=dev)
    want = int(words.to(torch.int64).sum().item()) & 0xffffffff
    for num_wg in (1, 7, 64):
        sums = torch.full((num_wg,), -1, dtype=torch.int32, device=dev)
        B.gf_hbm_read_probe(sess.ctx, words, nbytes, sums, num_wg)
        torch.cuda.synchronize()
        assert _word_sum(sums) == want
    # tiles: every tile once, in a shuffled order, by any number of workgroups; ids outside the buffer are folded in
    tile = 2048
    n = (3 << 20) // tile
    gen = torch.Generator(device=dev)
    gen.manual_seed(3)
    ids = torch.randperm(n, generator=gen, device=dev).to(torch.int32)
    want = int(words[: n * tile // 4].to(torch.int64).sum().item()) & 0xffffffff
    for num_wg in (1, 5, 32):
        sums = torch.full((num_wg,), -1, dtype=torch.int32, device=dev)
        B.gf_hbm_tile_probe(sess.ctx, words, tile, n, ids, n, sums, num_wg)
        torch.cuda.synchronize()
        assert _word_sum(sums) == want
    far = ids + 5 * n                                       # the same tiles after folding
    sums = torch.zeros(4, dtype=torch.int32, device=dev)
    B.gf_hbm_tile_probe(sess.ctx, words, tile, n, far, n, sums, 4)
    torch.cuda.synchronize()
    assert _word_sum(sums) == want


def test_mfma_probe_issues_what_it_says():
    sess = _session()
    dev = sess.device
    num_wg, rounds = 3, 5
    sums = torch.full((num_wg * 256,), -1.0, dtype=torch.float32, device=dev)
    ones = torch.ones(8192, dtype=torch.bfloat16, device=dev)
    B.gf_mfma_probe(sess.ctx, ones, ones.numel() * 2, rounds, sums, num_wg)
    torch.cuda.synchronize()
    # every MFMA adds 16 (a contraction over 16 ones) to the 16 accumulator elements a lane holds; a round issues 8
    assert torch.equal(sums, torch.full_like(sums, 16.0 * 16 * 8 * rounds))
    # with the softmax's vector instructions riding along: the same MFMAs, plus four values in [0, 1) and a sum of
    # 8 * rounds exponentials of such values, each scaled by 0.001
    mixed = torch.full_like(sums, -1.0)
    B.gf_mfma_probe(sess.ctx, ones, ones.numel() * 2, rounds, mixed, num_wg, softmax_mix=1)
    torch.cuda.synchronize()
    extra = mixed - sums
    assert bool(((extra > 0) & (extra < 4 + 0.002 * 8 * rounds + 0.1)).all())      # 0.1: rounding of the fold at 1e4
    zeros = torch.zeros(512, dtype=torch.bfloat16, device=dev)        # one 1 KB fragment, used by everybody
    B.gf_mfma_probe(sess.ctx, zeros, 1024, rounds, sums, num_wg)
    torch.cuda.synchronize()
    assert torch.equal(sums, torch.zeros_like(sums))
    B.gf_mfma_probe(sess.ctx, ones, ones.numel() * 2, 0, sums, num_wg)    # no round: the accumulators stay zero
    torch.cuda.synchronize()
    assert torch.equal(sums, torch.zeros_like(sums))


def test_probe_argument_checks():
    sess = _session()
    dev = sess.device
    buf = torch.zeros(4096, dtype=torch.bfloat16, device=dev)
    sums = torch.zeros(256, dtype=torch.int32, device=dev)
    fsums = torch.zeros(256, dtype=torch.float32, device=dev)
    ids = torch.zeros(4, dtype=torch.int32, device=dev)
    assert _code(lambda: B.gf_hbm_read_probe(sess.ctx, buf, 24, sums, 1)) == B.GF_ERR_BAD_SHAPE          # not 16-byte
    assert _code(lambda: B.gf_hbm_read_probe(sess.ctx, None, 4096, sums, 1)) == B.GF_ERR_NULL
    assert _code(lambda: B.gf_hbm_tile_probe(sess.ctx, buf, 1000, 4, ids, 4, sums, 1)) == B.GF_ERR_BAD_SHAPE
    assert _code(lambda: B.gf_hbm_tile_probe(sess.ctx, buf, 1024, 0, ids, 4, sums, 1)) == B.GF_ERR_BAD_SHAPE
    assert _code(lambda: B.gf_hbm_tile_probe(sess.ctx, buf, 1024, 4, None, 4, sums, 1)) == B.GF_ERR_NULL
    assert _code(lambda: B.gf_mfma_probe(sess.ctx, buf, 1000, 1, fsums, 1)) == B.GF_ERR_BAD_SHAPE
    assert _code(lambda: B.gf_mfma_probe(sess.ctx, buf, 0, 1, fsums, 1)) == B.GF_ERR_BAD_SHAPE
    assert _code(lambda: B.gf_mfma_probe(sess.ctx, buf, 1024, -1, fsums, 1)) == B.GF_ERR_BAD_SHAPE
    assert _code(lambda: B.gf_mfma_probe(sess.ctx, buf, 1024, 1, fsums, 1, softmax_mix=2)) == B.GF_ERR_BAD_SHAPE
    assert _code(lambda: B.gf_mfma_probe(sess.ctx, None, 1024, 1, fsums, 1)) == B.GF_ERR_NULL
    assert _code(lambda: B.gf_mfma_probe(sess.ctx, buf, 1024, 1, None, 1)) == B.GF_ERR_NULL
    B.gf_mfma_probe(sess.ctx, None, 1024, 1, None, 0)               # no workgroup: nothing read, nothing launched
    B.gf_hbm_read_probe(sess.ctx, None, 0, None, 1)
