"""Shared helpers of the GPU parity tests: tolerance metrics and fixtures."""
import numpy as np


def rel_max(a, b) -> float:
    """max|a-b| / max|b| per tensor (near-zero entries make elementwise ratios meaningless)."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-12))


def rel_l2(a, b) -> float:
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-12))


def rel_scalar(a, b) -> float:
    return abs(float(a) - float(b)) / max(abs(float(b)), 1e-12)


def top2_gap(q) -> np.ndarray:
    """Gap between the best and second-best entry of each row."""
    s = np.sort(np.asarray(q, np.float64), axis=1)
    return s[:, -1] - s[:, -2] if s.shape[1] > 1 else np.full(s.shape[0], np.inf)
