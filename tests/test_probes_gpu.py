"""The measurement entry points (matrix-instruction rate, synthetic tile streams, clock samples) run and report
plausible values. They compute nothing of the method, so there is nothing to compare with the oracle: the checks
are that every launch completes, the samples are written, and the counts are those the header states."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_counter_rate_and_matrix_probe(mepic):
    khz = mepic.device_counter_khz()
    assert 1_000 <= khz <= 10_000_000
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    for random_operands in (False, True):
        sink.zero_()
        flop = mepic.probe_mfma_bf16(200, sink, random_operands=random_operands)
        torch.cuda.synchronize()
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        assert flop == n_cu * 8 * 200 * 4 * 2 * 32 * 32 * 16
        clocks, ticks = float(sink[1]), float(sink[2])
        assert clocks >= 200 * 4 * 32 * 0.9            # a product occupies the matrix pipe for 32 clocks
        assert ticks > 0 and 0.3 < clocks / (ticks / (khz * 1e3)) / 1e9 < 3.5    # a clock rate between 0.3 and 3.5 GHz
        assert float(sink[0]) == 0.0


@pytest.mark.parametrize("structure", [0, 1, 2])
def test_tile_stream_probe_runs(mepic, structure):
    buf = torch.zeros(1 << 14, dtype=torch.float32, device="cuda")
    mepic.probe_tile_stream(structure, 50, buf)
    torch.cuda.synchronize()
    assert float(buf[1]) >= 50 * 32 * 32 * 0.9 and float(buf[2]) > 0
    assert float(buf[0]) == 0.0 and float(buf[3:].abs().max()) == 0.0      # the buffer is only read


def test_prefill_clock_sample_is_written(mepic):
    import workloads as W
    from paper_2512_16822_amd.device_case import DeviceCase, align_with_library
    st = W.prefill_structure("clock_sample", 5, B=2, Hq=8, Hkv=2, D=128, P=16, theta=5e5, n_chunks=2, chunk_tokens=256,
                             pool=3, q_tokens=64)
    aligned, _ = align_with_library(mepic, st)
    dc = DeviceCase(mepic, W.assemble(st, aligned, poison=False))
    dc.ws.zero_()
    mepic.attn_prefill(dc.params)
    torch.cuda.synchronize()
    assert mepic.last_kernel() == "prefill_mfma_bf16"
    off = mepic.attn_workspace_size(dc.params, True) - 16
    clocks, ticks = [int(x) for x in dc.ws[off:off + 16].view(torch.int64).cpu()]
    assert clocks > 0 and ticks > 0 and clocks / ticks < 40        # core clocks per 10 ns tick: below 4 GHz
