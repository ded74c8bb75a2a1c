"""Helpers for the GPU parity tests: bit-exact host <-> device transfer and error metrics."""
import numpy as np
import torch

import sdvg_inputs as si


def to_dev_bf16(bits):
    """uint16 bf16 bit patterns (numpy) -> bfloat16 device tensor holding the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def bits_of(t):
    """bfloat16 tensor (any device) -> uint16 bit patterns (numpy)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def attn_errors(gpu_bits, ref):
    """max |err| and relative RMS of a bf16 GPU output against the fp64 oracle output."""
    g = si.bf16_bits_to_f64(gpu_bits)
    err = g - ref
    return float(np.max(np.abs(err))), float(np.sqrt(np.sum(err * err) / np.sum(ref * ref)))


def attn_errors_by_head(gpu_bits, ref):
    """(max |err|, pooled rel-RMS, worst single head's rel-RMS, that head) for outputs shaped
    [rows, heads, dim]. Heads whose reference is all zero are skipped for the per-head figure."""
    g = si.bf16_bits_to_f64(gpu_bits)
    err = g - ref
    num = np.sum(err * err, axis=(0, 2))
    den = np.sum(ref * ref, axis=(0, 2))
    per_head = np.sqrt(np.where(den > 0, num / np.where(den > 0, den, 1.0), 0.0))
    worst = int(np.argmax(per_head))
    return (float(np.max(np.abs(err))), float(np.sqrt(num.sum() / den.sum())), float(per_head[worst]), worst)


# Tolerances of the bf16 attention path: absolute and relative-RMS bounds on the output.
# bf16 P and bf16 output rounding are each ~2^-9 relative; sums over many keys average it down.
BF16_MAX_ABS = 2e-2
BF16_REL_RMS = 1e-2
F32_MAX_ABS = 1e-4
