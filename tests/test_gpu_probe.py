"""The MFMA-only measurement kernel runs and reports a plausible rate."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("changing", [False, True])
def test_mfma_probe_runs(changing):
    """The MFMA-only measurement kernels: run, report their FLOP count and a clock reading."""
    import paper_2604_17397_amd as P
    flops, cycles = P.probe_mfma(500, changing=changing)
    torch.cuda.synchronize()
    assert flops == 256 * 4 * 500 * 16 * 32768.0
    assert int(cycles.item()) > 500 * 16 * 8   # at least a quarter of the MFMA-bound cycle count
    with pytest.raises(P.SdvgError):
        P.probe_mfma(0, changing=changing)
