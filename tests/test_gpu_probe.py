"""The bandwidth probes move the bytes they claim to: every variant of the flat copy, the
read and the write pass, the row-chunk and tile copies and the multi-read pass is checked
against numpy on small buffers with NaN wherever nothing may be written.  (The probes
compute nothing of the method, so the oracle has no part in this.)"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def combo():
    import paper_1908_07782_amd as c
    assert torch.cuda.is_available()
    c.lib()
    return c


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


SHAPES = [(4, 1000, 1024), (3, 70_001, 70_016), (16, 33_000, 33_024)]
MAPPINGS = [(flight, adjacent, run, through) for flight in (1, 2, 4, 8) for adjacent in (0, 1)
            for run, through in ((0, 0), (3, 0), (16, 1), (128, 1))]


@pytest.mark.parametrize("N,P,ld", SHAPES)
def test_flat_copy_read_and_write_cover_every_word_once(combo, N, P, ld):
    rng = np.random.default_rng(N * 1000 + P)
    src_h = rng.standard_normal((N, ld)).astype(np.float32)
    src = torch.from_numpy(src_h).cuda()
    for flight, adjacent, run, through in MAPPINGS:
        cols = (run << 4) | (through << 1) | adjacent
        dst = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
        combo.bandwidth_probe(combo.PROBE_COPY, dst, src, P, cols=cols, param=flight)
        assert np.array_equal(bits(dst.cpu().numpy()), bits(src_h)), (flight, adjacent, run, through)
        dst.fill_(float("nan"))
        combo.bandwidth_probe(combo.PROBE_WRITE, dst, None, P, cols=cols, param=flight)
        want = np.tile(np.array([1, 2, 3, 4], np.float32), N * ld // 4).reshape(N, ld)
        assert np.array_equal(dst.cpu().numpy(), want), (flight, adjacent, run, through)
        if through:
            continue                                       # the read pass has no stores to speak of
        per_block = 1024 * flight
        blocks = -(-N * ld // per_block)
        out = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
        combo.bandwidth_probe(combo.PROBE_READ, out, src, P, cols=cols, param=flight)
        got = out.cpu().numpy().reshape(-1)
        flat = np.zeros(blocks * per_block, np.float64)
        flat[:N * ld] = src_h.reshape(-1)
        want = flat.reshape(blocks, per_block).sum(axis=1)
        scale = np.abs(flat).reshape(blocks, per_block).sum(axis=1)
        assert np.all(np.abs(got[:blocks] - want) <= 1e-5 * scale + 1e-30), (flight, adjacent, run)
        assert np.isnan(got[blocks:]).all()


@pytest.mark.parametrize("N,P,ld", SHAPES)
@pytest.mark.parametrize("cols", [64, 128, 1024])
def test_strip_copies_touch_whole_strips_only(combo, N, P, ld, cols):
    if P < cols:
        pytest.skip("no whole strip")
    rng = np.random.default_rng(N + P + cols)
    src_h = rng.standard_normal((N, ld)).astype(np.float32)
    src = torch.from_numpy(src_h).cuda()
    strips = P // cols
    dst = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
    for run in (0, 1, 4, 16):                      # strip i -> workgroup i, or XCD runs of `run` strips
        dst.fill_(float("nan"))
        combo.bandwidth_probe(combo.PROBE_ROW_CHUNKS, dst, src, P, cols=cols, param=run)
        got = dst.cpu().numpy()
        assert np.array_equal(bits(got[:, :strips * cols]), bits(src_h[:, :strips * cols])), run
        assert np.isnan(got[:, strips * cols:]).all(), run
        dst.fill_(float("nan"))
        combo.bandwidth_probe(combo.PROBE_TILES, dst, src, P, cols=cols, param=run)
        got = dst.cpu().numpy().reshape(-1)
        n = strips * N * cols
        assert np.array_equal(bits(got[:n]), bits(src_h.reshape(-1)[:n])), run
        assert np.isnan(got[n:]).all(), run


@pytest.mark.parametrize("N,P,ld", SHAPES)
@pytest.mark.parametrize("k", [1, 2, 3])
def test_multi_read_pass_adds_k_rows_in_order(combo, N, P, ld, k):
    if P < 1024:
        pytest.skip("no whole tile")
    rng = np.random.default_rng(N + P + k)
    src_h = rng.standard_normal((N, ld)).astype(np.float32)
    src = torch.from_numpy(src_h).cuda()
    dst = torch.full((N, ld), float("nan"), dtype=torch.float32, device="cuda")
    combo.bandwidth_probe(combo.PROBE_MULTI_READ, dst, src, P, param=k)
    got = dst.cpu().numpy()
    covered = P // 1024 * 1024
    want = src_h[:, :covered].copy()
    for j in range(1, k):
        want = want + np.roll(src_h, -j, axis=0)[:, :covered]       # fp32 adds, in row order
    assert np.array_equal(bits(got[:, :covered]), bits(want))
    assert np.isnan(got[:, covered:]).all()


def test_lds_read_probe_reads_what_it_says(combo):
    """Every thread of a workgroup reads iters x 8 words of the 8 KiB block, 64 lanes on 64
    consecutive words; the checksum is the sum of the word indices read plus the number of reads."""
    iters, wgs = 4, 37
    dst = torch.full((4, 1024), float("nan"), dtype=torch.float32, device="cuda")
    combo.bandwidth_probe(combo.PROBE_LDS_READ, dst, None, 1000, cols=wgs, param=iters)
    got = dst.cpu().numpy().reshape(-1)
    want = 0
    for t in range(256):
        idx = t
        for it in range(iters):
            for u in range(8):
                want += ((idx + u * 64) & 511) + 1
            idx = (idx + 64) & 511
    assert np.array_equal(got[:wgs], np.full(wgs, float(want), np.float32))
    assert np.isnan(got[wgs:]).all()
