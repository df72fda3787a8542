"""The step-mix probe (a measurement aid of the library): argument checks and a short run of every mix."""
import pytest
import torch

import paper_2505_19578_amd as sp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def buffers():
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    operands = torch.randn(sp.SP_PROBE_OPERAND_BYTES // 2, generator=g, device="cuda").to(torch.bfloat16)
    sink = torch.full((sp.SP_PROBE_SINK_BYTES // 4,), float("nan"), dtype=torch.float32, device="cuda")
    return operands, sink


def test_every_mix_runs_and_counts_its_flops(buffers):
    operands, sink = buffers
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for mix, name in enumerate(sp.SP_PROBE_MIXES):
        print(f"probe mix {mix} ({name})", flush=True)
        sink.fill_(float("nan"))
        flops = sp.sp_probe_step_mix(mix, operands, 50, sink)
        torch.cuda.synchronize()
        wg_per_cu, g = (1, 64) if name == "step_64q" else (2, 32)
        n_lanes = cus * wg_per_cu * 256
        assert flops == cus * wg_per_cu * 4 * 50 * g * 2 * 32 * 32 * 16
        # every lane of the grid wrote its accumulators' sum: finite for bounded operands
        assert torch.isfinite(sink[:n_lanes]).all()
        assert torch.isnan(sink[n_lanes:]).all()


def test_arguments_are_checked(buffers):
    operands, sink = buffers
    with pytest.raises(sp.SpError):
        sp.sp_probe_step_mix(len(sp.SP_PROBE_MIXES), operands, 10, sink)
    with pytest.raises(sp.SpError):
        sp.sp_probe_step_mix(0, operands, 0, sink)
    with pytest.raises(sp.SpError):
        sp.sp_probe_step_mix(0, operands[: 1 << 20], 10, sink)
    with pytest.raises(sp.SpError):
        sp.sp_probe_step_mix(0, operands, 10, sink[: 1 << 10])
    with pytest.raises(sp.SpError):
        sp.sp_probe_step_mix(0, operands[1:], 10, sink)       # 2-byte offset: not 16-byte aligned
