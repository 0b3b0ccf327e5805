"""The calibration probe behind `bench.py --stage ceiling`: every mode runs to completion on both kinds of operands
and leaves the sink untouched (it measures rates; there is nothing to compare with an oracle)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4])
def test_probe_modes_run(gpu_lib, mode):
    av = gpu_lib
    g = torch.Generator(device="cuda").manual_seed(1)
    for buf in (torch.randn((4, 512, 4096), device="cuda", generator=g).to(torch.bfloat16),
                torch.zeros((4, 512, 4096), dtype=torch.bfloat16, device="cuda")):
        sink = torch.zeros(1, device="cuda")
        print(f"[case] probe mode {mode}", flush=True)
        av.aurora_probe_contraction(mode, buf, 64, 8, sink)
        av.aurora_probe_contraction(mode, buf, 300, 3, sink)
        torch.cuda.synchronize()
        assert float(sink.item()) == 0.0
