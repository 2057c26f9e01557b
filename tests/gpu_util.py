"""Helpers shared by the GPU parity tests: host <-> device plumbing and the
floating-point parity bar for bf16 outputs."""
import numpy as np
import torch

from paper_2501_04052_amd import synth

TOL = 8e-3          # max relative error on bf16 GEMM outputs (fp32 accumulation)


def bf16_bits_to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev_to_bf16_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def max_rel_err(y_gpu_bits, y_ref_f64):
    """|y_gpu - bf16(y_ref)| / max(|bf16(y_ref)|, 0.01 rms(y_ref)): the floor keeps outputs
    that are tiny through cancellation from turning summation-order noise into a 'relative' error."""
    ref16 = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(y_ref_f64.astype(np.float32))).astype(np.float64)
    got = synth.bf16_bits_to_f32(y_gpu_bits).astype(np.float64)
    rms = float(np.sqrt(np.mean(y_ref_f64 ** 2))) if y_ref_f64.size else 0.0
    den = np.maximum(np.abs(ref16), 0.01 * rms + 1e-300)
    return float(np.max(np.abs(got - ref16) / den)) if got.size else 0.0


def tensor_to_host(t):
    scales = t.scales.cpu().numpy()
    if scales.dtype == np.int16:                       # 16-bit scale words of the FP16-scale format
        scales = scales.view(np.uint16)
    return (t.codes.cpu().numpy(), scales, np.float32(t.tensor_scale.cpu().numpy()[0]))
