"""The paper's roofline model for software-decoded weight formats, as plain
arithmetic (Sec. 3.3 "Efficiency", eq. "theoretical-speedup"; App. D
"Theoretical model of software-decoded formats").  Used to put measured numbers
next to the model's prediction for a given accelerator; no kernel depends on it.
"""
from __future__ import annotations


def kernel_time(P_w: float, h: int, m: int, r_compute: float, r_transfer: float) -> float:
    """t = max(t_compute, t_transfer) for Y^T = W X^T with W h x h at P_w bits per
    weight and batch m: 2 m h^2 / R_compute versus P_w h^2 / (8 R_transfer)."""
    return max(2.0 * m * h * h / r_compute, P_w * h * h / (8.0 * r_transfer))


def speedup(P_w1: float, P_w2: float, m: float, nu: float) -> float:
    """Speed-up from P_w1 to P_w2 bits per weight at batch m on a device with
    nu = R_compute / R_transfer (op/s per byte/s)."""
    return max(1.0, P_w1 * nu / (16.0 * m)) / max(1.0, P_w2 * nu / (16.0 * m))


def memory_bound_batch(P_w: float, nu: float) -> float:
    """Largest batch for which a P_w-bit kernel is still bound by weight transfer."""
    return P_w * nu / 16.0


def effective_bandwidth(operand_bytes: float, seconds: float) -> float:
    """App. E: operand sizes divided by the time taken (bytes/s)."""
    return operand_bytes / seconds
