"""The calibration kernels behind bench.py's measured ceilings: they run to completion on small
buffers, report the bytes / flops of a launch, leave their inputs as they were, copy what they
are asked to copy, and refuse sizes their launch shapes do not cover."""
import pytest

pytestmark = pytest.mark.gpu


def test_hbm_modes_on_a_small_buffer():
    import torch
    import paper_2504_09285_amd as dsv
    n = 8 << 20
    g = torch.Generator(device="cpu").manual_seed(5)
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, generator=g).cuda()
    keep = src.clone()
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    dsv.dsv_calib_hbm(0, dst, src, n)          # read only
    torch.cuda.synchronize()
    assert torch.equal(src, keep) and int(dst.max()) == 0
    dsv.dsv_calib_hbm(2, dst, src, n)          # copy
    torch.cuda.synchronize()
    assert torch.equal(dst, keep) and torch.equal(src, keep)


def test_paged_read_reports_its_bytes_and_touches_nothing():
    import torch
    import paper_2504_09285_amd as dsv
    for blocks in (64, 1024):
        n = blocks * 32768
        k = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
        v = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        sink = torch.zeros(16, dtype=torch.float32, device="cuda")
        assert dsv.dsv_calib_paged_read(k, v, sink) == 2.0 * n
        torch.cuda.synchronize()
        assert int(k.min()) == 3 and int(k.max()) == 3 and int(v.min()) == 7 and int(v.max()) == 7
        assert float(sink.abs().max()) == 0.0


@pytest.mark.parametrize("nbytes", [0, 32768, 63 * 32768, 96 * 32768, 64 * 32768 + 16])
def test_paged_read_refuses_sizes_that_are_not_a_power_of_two_of_blocks(nbytes):
    import torch
    import paper_2504_09285_amd as dsv
    k = torch.zeros(max(nbytes, 16), dtype=torch.uint8, device="cuda")[:nbytes]
    v = torch.zeros(max(nbytes, 16), dtype=torch.uint8, device="cuda")[:nbytes]
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(dsv.DsvError):
        dsv.dsv_calib_paged_read(k, v, sink)
    torch.cuda.synchronize()


def test_mfma_loop_reports_its_flops():
    import torch
    import paper_2504_09285_amd as dsv
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    flops = dsv.dsv_calib_mfma(10, sink)
    torch.cuda.synchronize()
    assert flops > 0 and float(sink.abs().max()) == 0.0


def test_mfma_loop_on_caller_operands_reports_its_flops_and_checks_its_arguments():
    import torch
    import paper_2504_09285_amd as dsv
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    ops = torch.randn(4096, generator=g, device="cuda").to(torch.bfloat16)
    keep = ops.clone()
    fixed = dsv.dsv_calib_mfma(16, sink)
    assert dsv.dsv_calib_mfma_data(16, ops, sink, shape=0) == fixed      # same launch shape, same count
    assert dsv.dsv_calib_mfma_data(16, ops, sink, shape=1) == fixed      # 16x16x32: twice the MFMAs of half the size
    with pytest.raises(dsv.DsvError):
        dsv.dsv_calib_mfma_data(16, ops, sink, shape=2)
    torch.cuda.synchronize()
    assert torch.equal(ops, keep) and float(sink.abs().max()) == 0.0
    for iters, operands in ((12, ops), (0, ops), (16, ops[:64]), (16, ops[1:4001])):   # not a multiple of 8; too few; misaligned
        with pytest.raises(dsv.DsvError):
            dsv.dsv_calib_mfma_data(iters, operands, sink)
    torch.cuda.synchronize()
