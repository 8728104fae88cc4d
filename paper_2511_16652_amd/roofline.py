"""Roofline bookkeeping for the EGGROLL hot path (host-side arithmetic only, no GPU code).

Closed forms follow the paper's appendix "Arithmetic Intensity Analysis": operations divided by
bytes read or written, for a linear layer M in R^{d_out x d_in}, a batch of B inputs and `s` bytes
per element.
"""
from __future__ import annotations

import math

# MI355X published peaks used as roofline denominators
HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "i8": 5000.0, "f32": 157.3}
# plain vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def intensity_standard(B, d_in, d_out, s=2):
    """Standard batched inference u M^T."""
    return (2.0 * B * d_in * d_out) / (s * (B * d_in + B * d_out + d_out * d_in))


def intensity_gaussian_es(d_in, d_out, s=2):
    """Full-rank Gaussian matrix ES with pre-generated perturbations (independent of B)."""
    return (2.0 * d_in * d_out) / (s * (d_in + d_out + d_out * d_in))


def intensity_eggroll(B, d_in, d_out, r, s=2):
    """EGGROLL with pre-generated factors and the B x r intermediate written and read."""
    ops = 2.0 * B * d_in * d_out + 2.0 * B * (d_in + d_out) * r + B * d_out
    byts = s * (B * d_in + B * (d_in + d_out + 2) * r + d_out * d_in + B * d_out)
    return ops / byts


def critical_batch_standard(A, m):
    """Smallest batch reaching intensity A for a square m x m layer, s = 2."""
    return math.ceil(A * m / (m - 2.0 * A))


def critical_batch_eggroll(A, m, r):
    return math.ceil(A * m / (m - 2.0 * A + 2.0 * r + 0.5 - r * A * (2.0 + 2.0 / m)))


def flop_overhead(r, m):
    """Extra operations of EGGROLL relative to the shared GEMM, square m x m layer."""
    return (4.0 * r + 1.0) / (2.0 * m)


def forward_flops(R, d_in, d_out, r):
    """Algorithmic operations of one perturbed forward over R rows."""
    return 2.0 * R * d_in * d_out + 2.0 * R * (d_in + d_out) * r + R * d_out


def forward_bytes(R, d_in, d_out, r, s):
    """Algorithmic HBM bytes of one perturbed forward when the noise is regenerated in-kernel:
    X read, W read once, Y written, the R x r fp32 intermediate written and read."""
    return s * (R * d_in + d_out * d_in + R * d_out) + 8.0 * R * r


def update_flops(N, d_in, d_out, r):
    return 2.0 * N * r * d_in * d_out


def update_bytes(N, d_in, d_out):
    """fitness read + fp32 G written."""
    return 4.0 * N + 4.0 * d_out * d_in
