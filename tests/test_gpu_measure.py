"""GPU checks of the measurement aids (include/lrd_measure.h): the kernels behind bench.py's in-run peaks
do the work their byte / flop counts claim, and the event log records every product of a call."""
import numpy as np
import pytest
import torch

from paper_2309_03824_amd import binding as lrd

pytestmark = pytest.mark.gpu


def test_stream_copy_and_write_move_the_bytes_they_count():
    n = (1 << 20) + 48                      # not a multiple of a workgroup's 32 KiB
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    lrd.measure_stream(src, dst, n, lrd.STREAM_COPY)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    dst.fill_(7)
    guard = dst.clone()
    lrd.measure_stream(None, dst, n - 16, lrd.STREAM_WRITE)
    torch.cuda.synchronize()
    words = dst[: n - 16].view(torch.int32).view(-1, 4).cpu().numpy()
    assert np.all(words[:, 1:] == np.array([1, 2, 3]))       # every 16-byte word was written
    assert torch.equal(dst[n - 16:], guard[n - 16:])         # and nothing past the size given
    before = dst.clone()
    lrd.measure_stream(src, dst, n, lrd.STREAM_READ)
    torch.cuda.synchronize()
    assert torch.equal(dst, before)                          # the read pass stores nothing (almost surely)


def test_lds_read_loop_reads_the_words_it_counts():
    """The loop's checksum equals what its documented access pattern reads from an LDS array holding its own
    word indices (so the reads are real, in bounds, and eight per round)."""
    wgs, iters = 3, 4
    sink = torch.zeros(wgs * 256, dtype=torch.int32, device="cuda")
    nbytes = lrd.measure_lds_read(sink, wgs, iters)
    torch.cuda.synchronize()
    assert nbytes == wgs * 256 * iters * 8 * 16
    got = sink.cpu().numpy().astype(np.uint32).reshape(wgs, 256)
    lane = np.arange(256, dtype=np.int64) & 63
    base = (lane & 31) * 144 + (lane >> 5) * 16
    want = np.zeros(256, dtype=np.int64)
    for it in range(iters):
        a = base + ((it & 1) << 14)
        for q, off in enumerate((0, 32, 64, 96, 4608, 4640, 4672, 4704)):
            want += (a + off) // 4 + (q & 3)                 # component q & 3 of the 16-byte word
    want = (want & 0xFFFFFFFF).astype(np.uint32)
    for w in range(wgs):
        assert np.array_equal(got[w], want)


def test_mfma_loop_counts_its_flops_and_event_log_records_products():
    sink = torch.zeros(8 * 256, dtype=torch.float32, device="cuda")
    flops = lrd.measure_mfma_loop(sink, 8, 10)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 10 * 4 * 2.0 * 32 * 32 * 16     # workgroups x waves x rounds x 4 instructions
    assert torch.all(torch.isfinite(sink))
    T, n_in, n_out, r = 256, 64, 128, 16
    bf = torch.bfloat16
    X, V, U = (torch.randn(s, device="cuda").to(bf) for s in ((T, n_in), (r, n_in), (n_out, r)))
    Y, H = torch.empty(T, n_out, dtype=bf, device="cuda"), torch.empty(T, r, dtype=bf, device="cuda")
    ws = torch.empty(lrd.linear_workspace_bytes(T, n_in, n_out, r, lrd.BF16, 0) + 16, dtype=torch.uint8, device="cuda")
    with lrd.ProfileLog(8) as log:
        lrd.linear_fwd(X, V, U, None, Y, H, ws)
        torch.cuda.synchronize()
    rows = log.rows()
    assert [(r_["M"], r_["N"], r_["K"]) for r_ in rows] == [(T, r, n_in), (T, n_out, r)]
    assert all(r_["us"] > 0 and r_["batch"] == 1 and r_["kernel"] for r_ in rows)
