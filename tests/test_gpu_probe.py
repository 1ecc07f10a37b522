"""The measuring helpers of the C ABI (matrix-pipe-only loop, copy, read, shader-clock sampling):
they run, validate their arguments and report plausible figures.  They are not part of the linear."""
import pytest
import torch

from paper_2410_06511_amd import f8

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,mfma_per_iter,cycles", [(0, 64, 32), (1, 32, 64)])
def test_mfma_probe_runs_at_one_instruction_per_issue_slot(shape, mfma_per_iter, cycles):
    """With operands in registers the matrix pipe is the only limit: a 16x16x128 fp8 MFMA takes 32
    cycles of its SIMD, a 32x32x64 one 64 (both 2048 flop per cycle and SIMD)."""
    ops = torch.full((1 << 20,), 0x38, dtype=torch.uint8, device="cuda")
    ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
    iters = 500
    flops = f8.probe_mfma(ops, iters, ticks, shape=shape)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == cus * 4 * iters * 64 * 2 * 16 * 16 * 128
    c, r = ticks.cpu().tolist()
    assert r > 0 and 0.99 * cycles <= c / (iters * mfma_per_iter) <= 1.05 * cycles


def test_mfma_probe_rejects_bad_arguments():
    ops = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    for kw, code in ((dict(shape=2), 4), (dict(shape=0, n=3 << 18), 2), (dict(shape=0, n=1 << 16), 2), (dict(shape=0, iters=1 << 20), 2)):
        with pytest.raises(f8.F8Error) as e:
            f8.probe_mfma(ops[: kw.get("n", 1 << 20)], kw.get("iters", 1), shape=kw["shape"])
        assert e.value.code == code


def test_copy_and_read_probes():
    src = torch.randint(0, 256, (1 << 22,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    f8.probe_copy(src, dst)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    f8.probe_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    with pytest.raises(f8.F8Error) as e:
        f8.probe_copy(src[:24], dst[:24])      # not a multiple of 16 bytes
    assert e.value.code == 2


def test_clock_probe_brackets_a_region():
    """Two samples around some work: most compute units are seen in both, and the mean shader clock
    between them is a possible one for this chip."""
    clk = torch.zeros((2, 4 * f8.PROBE_CLOCK_SLOTS), dtype=torch.int64, device="cuda")
    ops = torch.full((1 << 20,), 0x38, dtype=torch.uint8, device="cuda")
    f8.probe_clock(clk[0])
    f8.probe_mfma(ops, 2000)
    f8.probe_clock(clk[1])
    torch.cuda.synchronize()
    c = clk.cpu()
    both = ((c[0].view(-1, 4)[:, 0] == 1) & (c[1].view(-1, 4)[:, 0] == 1)).sum().item()
    assert both >= 128
    ghz = f8.clock_ghz_between(c[0], c[1])
    assert 0.4 <= ghz <= 2.6
