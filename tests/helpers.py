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
# Provisional bars of the runs from pre-trained tables (set from the arithmetic once measured):
FORCED_BEYOND = 1e-5


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


# ---------------------------------------------------------------- the same comparisons on the GPU
# (torch as test infrastructure: tables of 10^9 elements are compared where they already are)
def to_dev(w_np):
    """numpy table (float32, or uint16 bfloat16 bits) -> device tensor of the same bits"""
    import torch
    if w_np.dtype == np.uint16:
        return torch.from_numpy(w_np.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(w_np).cuda()


def _ordered_t(x):
    """Integers whose difference is the distance in units in the last place (f32 or bf16 tensor)."""
    import torch
    if x.dtype == torch.bfloat16:
        i = x.view(torch.int16).to(torch.int32)
        mag = i & 0x7FFF
    else:
        i = x.view(torch.int32).to(torch.int64)
        mag = i & 0x7FFFFFFF
    return torch.where(i < 0, -mag, mag)


def ulp_stats_t(got, want, w0=None, chunk=1 << 26):
    """Element-wise comparison of two device tables of the same type, in units in the last place of their own
    values (bit patterns as ordered integers): {max: largest distance, differ: fraction of elements that are
    not bit-identical, beyond2: fraction more than 2 apart, moved: elements of `want` that differ from `w0`}."""
    import torch
    g, w = got.reshape(-1), want.reshape(-1)
    z = w0.reshape(-1) if w0 is not None else None
    n = g.numel()
    mx = differ = beyond = moved = 0
    for lo in range(0, n, chunk):
        d = (_ordered_t(g[lo:lo + chunk]) - _ordered_t(w[lo:lo + chunk])).abs()
        mx = max(mx, int(d.max()))
        differ += int((d > 0).sum())
        beyond += int((d > 2).sum())
        if z is not None:
            moved += int((w[lo:lo + chunk] != z[lo:lo + chunk]).sum())
    return {"max": mx, "differ": differ / max(n, 1), "beyond2": beyond / max(n, 1), "moved": moved, "n": n}


def rel_l2_t(a, b, chunk=1 << 26):
    """|a - b|_2 / |b|_2 of two device tensors, accumulated in double."""
    import torch
    a, b = a.reshape(-1), b.reshape(-1)
    num = den = 0.0
    for lo in range(0, a.numel(), chunk):
        x, y = a[lo:lo + chunk].double(), b[lo:lo + chunk].double()
        num += float(((x - y) ** 2).sum())
        den += float((y ** 2).sum())
    return (num / den) ** 0.5 if den > 0 else num ** 0.5


def delta_rel_l2_t(got, want, w0, chunk=1 << 26):
    """The same on the change since w0: |(got - w0) - (want - w0)| / |want - w0|."""
    import torch
    g, w, z = got.reshape(-1), want.reshape(-1), w0.reshape(-1)
    num = den = 0.0
    for lo in range(0, g.numel(), chunk):
        x, y, o = g[lo:lo + chunk].double(), w[lo:lo + chunk].double(), z[lo:lo + chunk].double()
        num += float(((x - y) ** 2).sum())
        den += float(((y - o) ** 2).sum())
    return (num / den) ** 0.5 if den > 0 else num ** 0.5


def bf16_ulp_err_t(got, want, peak=None, floor_frac=2.0 ** -7, chunk=1 << 26):
    """bf16_ulp_err on device tensors: (max error, fraction beyond BF16_ULP, fraction bit-identical), the ulp
    taken at max(|a|, |b|, peak, floor_frac * rms of want's non-zero elements)."""
    import torch
    g, w = got.reshape(-1), want.reshape(-1)
    pk = peak.reshape(-1) if peak is not None else None
    n = g.numel()
    ss = cnt = 0.0
    for lo in range(0, n, chunk):
        y = w[lo:lo + chunk].double()
        ss += float((y ** 2).sum())
        cnt += float((y != 0).sum())
    if cnt == 0:
        return float((g.float() != w.float()).any()), 0.0, 1.0
    floor = floor_frac * (ss / cnt) ** 0.5
    mx, beyond, same = 0.0, 0, 0
    for lo in range(0, n, chunk):
        x, y = g[lo:lo + chunk].float(), w[lo:lo + chunk].float()
        mag = torch.maximum(torch.maximum(x.abs(), y.abs()), torch.tensor(floor, device=x.device))
        if pk is not None:
            mag = torch.maximum(mag, pk[lo:lo + chunk].float().abs())
        ulp = torch.exp2(torch.floor(torch.log2(mag)) - 7)
        err = (x - y).abs() / ulp
        mx = max(mx, float(err.max()))
        beyond += int((err > BF16_ULP).sum())
        same += int((err == 0).sum())
    return mx, beyond / n, same / n


def ulp_err_at_t(got, want, ref, chunk=1 << 26):
    """(max, fraction beyond 2) of |got - want| in units in the last place of max(|got|, |want|, |ref|): the error of
    one update W <- W - alpha * sum measured against the larger of the old and the new value (where the two
    cancel, the rounding of the fp32 sum, harmless against the operands, is many ulps of the remainder)."""
    import torch
    g, w, r = got.reshape(-1), want.reshape(-1), ref.reshape(-1)
    mant = 7 if got.dtype == torch.bfloat16 else 23
    tiny = torch.tensor(2.0 ** -126, device=g.device, dtype=torch.float64)
    mx, beyond = 0.0, 0
    for lo in range(0, g.numel(), chunk):
        x, y, z = g[lo:lo + chunk].double(), w[lo:lo + chunk].double(), r[lo:lo + chunk].double()
        mag = torch.maximum(torch.maximum(torch.maximum(x.abs(), y.abs()), z.abs()), tiny)
        err = (x - y).abs() / torch.exp2(torch.floor(torch.log2(mag)) - mant)
        mx = max(mx, float(err.max()))
        beyond += int((err > 2).sum())
    return mx, beyond / max(g.numel(), 1)
