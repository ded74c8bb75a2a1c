"""GPU parity, bit-exact: sdvg_buffer_snapshot (clone / restore of an opaque buffer) against the
CPU oracle's byte copy."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 4096 + 5, (64 << 20) + 3])
def test_buffer_snapshot_matches_oracle(n):
    """Snapshot / restore of an opaque buffer: bit-exact, margins untouched, round trip."""
    import paper_2604_17397_amd as P
    g = torch.Generator(device="cuda")
    g.manual_seed(1234 + n % 97)
    src = torch.randint(0, 256, (n + 32,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.full((n + 48,), 0xA5, dtype=torch.uint8, device="cuda")
    h_dst = dst.cpu().numpy().copy()
    oracle.buffer_copy(h_dst, src.cpu().numpy(), n)
    P.buffer_snapshot(dst, src, n)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy(), h_dst)
    # clone -> corrupt -> restore
    live = src[:n].clone() if n else src[:0].clone()
    snap = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    P.buffer_snapshot(snap, live, n)
    orig = live.cpu().numpy().copy()
    if n:
        live[::3] ^= 0xFF
    P.buffer_snapshot(live, snap, n)
    torch.cuda.synchronize()
    assert np.array_equal(live.cpu().numpy(), orig)
