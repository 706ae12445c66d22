"""Comparison helpers shared by the GPU parity tests (no method arithmetic)."""
import numpy as np

# Tolerances (BASELINE the benchmark spec): integers bit-exact; fp32 tables relative error <= 1e-4
# after N steps; bf16 tables <= 2 ulp.  The per-call gradient rows and the table *delta* are
# checked as well so that the table check cannot pass vacuously (the tables barely move).
TOL_TABLE = 1e-4
TOL_DELTA = 1e-3
TOL_ROWS = 1e-4
TOL_LOSS = 2e-5
BF16_ULP = 2


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def rows_rel(a, b, floor=1e-12):
    """max over rows of ||a_r - b_r|| / max(||b_r||, floor)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if a.size == 0:
        return 0.0
    num = np.linalg.norm(a - b, axis=1)
    den = np.maximum(np.linalg.norm(b, axis=1), floor)
    return float((num / den).max())


def bf16_ordered(u16):
    """Map bf16 bit patterns to integers whose difference is the distance in ulps."""
    u = np.asarray(u16).astype(np.int64)
    mag = u & 0x7FFF
    return np.where(u & 0x8000, -mag, mag)


def bf16_ulp_dist(a, b):
    return int(np.abs(bf16_ordered(a) - bf16_ordered(b)).max()) if np.asarray(a).size else 0


def bf16_to_f32(u16):
    return (np.asarray(u16).astype(np.uint32) << 16).view(np.float32)
