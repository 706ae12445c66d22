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
# chains of N steps on bf16 tables: the two sides round differently in about 1e-3 of the updated
# elements per step (fp32 vs fp64 accumulation of the gradient lands on the other side of a
# rounding boundary), independently from step to step, so among 10^7..10^9 elements a few collect
# three such differences.  The chain tests therefore bound the fraction of elements beyond 2 ulp
# and the maximum; single applications from identical inputs are held to 2 ulp outright.
BF16_CHAIN_FRAC = 1e-6
BF16_CHAIN_MAX = 4
# the same chains with the peers' gradients sent as bfloat16 messages: a message element is a rounding
# decision taken from gradients that differ between the two sides by their own error (up to 1e-4 of a
# row, more once bf16 tables have drifted apart by a rounding), so an element within that distance of a
# rounding boundary -- a fraction of about error / 2^-8 -- comes out one bfloat16 step apart on the two
# sides.  One such step is 2^-8 of that peer's gradient element, which, against a table element that is
# itself a sum of a few such gradients times alpha, is of the order of one table ulp per flipped message,
# and more where the gradients cancel.  (From identical messages the application is held to 2 ulp.)
BF16_MSG_CHAIN_FRAC = 1e-4
BF16_MSG_CHAIN_MAX = 16


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def rows_rel(a, b, floor_frac=1e-3):
    """max over rows of ||a_r - b_r|| / max(||b_r||, floor_frac * rms row norm of b).

    The floor matters for rows that are the remainder of a cancellation: a row that is both the
    context (g = sigma - 1) and a negative (g = sigma) of the same center receives +-0.5/P * v and is
    left with ~1e-7 of either term, so its fp32 error is a fraction of the *terms*, not of the
    remainder.  Rows that small are compared on the scale of the gradient as a whole."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if a.size == 0:
        return 0.0
    num = np.linalg.norm(a - b, axis=1)
    nb = np.linalg.norm(b, axis=1)
    rms = float(np.sqrt((nb ** 2).mean()))
    den = np.maximum(nb, max(floor_frac * rms, 1e-30))
    return float((num / den).max())


def bf16_ordered(u16):
    """Map bf16 bit patterns to integers whose difference is the distance in ulps."""
    u = np.asarray(u16).astype(np.int64)
    mag = u & 0x7FFF
    return np.where(u & 0x8000, -mag, mag)


def bf16_ulp_dist(a, b):
    """Largest distance in bf16 ulps, bit patterns compared as ordered integers."""
    return int(np.abs(bf16_ordered(a) - bf16_ordered(b)).max()) if np.asarray(a).size else 0


def bf16_ulp_err(a, b, peak_bits=None, floor_frac=2.0 ** -7, full=False):
    """max |a - b| / ulp_bf16(m) with m = max(|a|, |b|, peak, floor).

    peak_bits (optional, uint16 magnitude bits) is the largest magnitude the element has had on the
    oracle side during a multi-step run: bf16 storage keeps an absolute error, so a one-ulp
    difference made while the value was large is still there after the value has shrunk, and is
    to be measured in the ulps of the time it was made.  floor = floor_frac * rms of b's nonzero
    elements covers elements that are the remainder of a cancellation (see rows_rel)."""
    fa, fb = bf16_to_f32(a), bf16_to_f32(b)
    nz = fb[fb != 0]
    if nz.size == 0:
        return float(np.abs(fa - fb).max() > 0)
    floor = np.float32(floor_frac * float(np.sqrt((nz.astype(np.float64) ** 2).mean())))
    mag = np.maximum(np.maximum(np.abs(fb), np.abs(fa)), floor)
    if peak_bits is not None:
        np.maximum(mag, bf16_to_f32(peak_bits), out=mag)
    ulp = np.exp2(np.floor(np.log2(mag)) - 7)
    err = np.abs(fa - fb) / ulp
    if not full:
        return float(err.max())
    return float(err.max()), float((err > BF16_ULP).mean()), float((err == 0).mean())


def bf16_to_f32(u16):
    return (np.asarray(u16).astype(np.uint32) << 16).view(np.float32)
