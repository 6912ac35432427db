"""Seeded synthetic inputs: activations, weights, bias and relevance masks.

This module holds none of the method's arithmetic.  It only draws numbers
(numpy's counter-based Philox generator), rounds them to the storage type the
caller asks for *before* any implementation sees them, and paints masks whose
statistics follow the paper's census (Sec. II-B: on average 42-49 % of pixels
irrelevant, most images 40-50 %, in few large contiguous regions such as sky
or far/near depth ranges).  Both the GPU library's callers and the CPU oracle's
tests are fed from here, so they read identical bytes.

Masks are uint8 [N, H, W], nonzero = relevant.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 220710741

F32, BF16, F16, FP8 = 0, 1, 2, 3
DTYPE_NAMES = {F32: "f32", BF16: "bf16", F16: "f16", FP8: "fp8"}


def rng(*key: int) -> np.random.Generator:
    """Generator keyed by (BASE_SEED, *key); same key -> same stream."""
    return np.random.Generator(np.random.Philox(seed=np.random.SeedSequence([BASE_SEED, *key])))


# ---- storage types ---------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def f32_to_f16_bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def _fp8_table() -> np.ndarray:
    """Values of the 127 non-negative finite E4M3 codes 0x00..0x7E, ascending
    (OCP 8-bit floating point: bias 7, subnormals frac * 2^-9, no infinities,
    0x7F = NaN)."""
    codes = np.arange(127)
    e, frac = codes >> 3, codes & 7
    return np.where(e == 0, frac / 512.0, (1.0 + frac / 8.0) * np.exp2(e - 7.0)).astype(np.float32)


def f32_to_fp8_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> E4M3 codes (uint8): nearest value, ties to the even code,
    magnitudes beyond 448 clamp to 448, NaN -> 0x7F."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    table = _fp8_table().astype(np.float64)
    mag = np.minimum(np.abs(a).astype(np.float64), table[-1])
    hi = np.clip(np.searchsorted(table, mag, side="left"), 0, 126)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = mag - table[lo], table[hi] - mag
    code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(np.isnan(a), 0x7F, code).astype(np.uint8)
    return code | (np.signbit(a).astype(np.uint8) << 7)


def fp8_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint8)
    mag = np.append(_fp8_table(), np.float32(np.nan))[b & 0x7F]
    return np.where(b >> 7, -mag, mag).astype(np.float32)


def to_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    """Values -> the array both implementations read: float32, uint16 bits, or E4M3 bytes."""
    if dtype == F32:
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(a)
    if dtype == F16:
        return f32_to_f16_bits(a)
    if dtype == FP8:
        return f32_to_fp8_bits(a)
    raise ValueError("dtype %r" % (dtype,))


def from_storage(s: np.ndarray, dtype: int) -> np.ndarray:
    """Storage array -> the float32 values it holds (exact)."""
    if dtype == F32:
        return np.ascontiguousarray(s, dtype=np.float32)
    if dtype == BF16:
        return bf16_bits_to_f32(s)
    if dtype == F16:
        return f16_bits_to_f32(s)
    if dtype == FP8:
        return fp8_bits_to_f32(s)
    raise ValueError("dtype %r" % (dtype,))


# ---- tensors ---------------------------------------------------------------

def activations(shape, dtype: int, *key: int) -> np.ndarray:
    """ReLU(N(0,1)) in NHWC, in storage form."""
    g = rng(*key)
    a = g.standard_normal(size=shape, dtype=np.float32)
    np.maximum(a, 0.0, out=a)
    return to_storage(a, dtype)


def activations_large(shape, dtype: int, *key: int) -> np.ndarray:
    """The same distribution for tensors of a gigabyte and more, several times faster to draw: one
    random byte per element picks one of 256 equally likely values of ReLU(N(0,1)) (its quantiles
    at (i + 1/2) / 256), stored in the layer's type."""
    from statistics import NormalDist
    nd = NormalDist()
    levels = np.array([max(nd.inv_cdf((i + 0.5) / 256.0), 0.0) for i in range(256)], dtype=np.float32)
    table = to_storage(levels, dtype)
    g = rng(*key)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=table.dtype)
    step = 1 << 26
    for at in range(0, n, step):
        picks = g.integers(0, 256, size=min(step, n - at), dtype=np.uint8)
        out[at:at + picks.size] = table[picks]
    return out.reshape(shape)


def he_weights(c_out: int, kh: int, kw: int, c_in: int, dtype: int, *key: int) -> np.ndarray:
    """He-normal weights [C_out, KH, KW, C_in], std = sqrt(2 / (KH*KW*C_in))."""
    g = rng(*key)
    a = g.standard_normal(size=(c_out, kh, kw, c_in), dtype=np.float32)
    a *= np.float32(np.sqrt(2.0 / (kh * kw * c_in)))
    return to_storage(a, dtype)


def bias(c_out: int, *key: int) -> np.ndarray:
    """Small float32 bias, N(0, 0.01^2)."""
    return (rng(*key).standard_normal(size=(c_out,), dtype=np.float32) * np.float32(0.01))


def small_integers(shape, lo: int, hi: int, dtype: int, *key: int) -> np.ndarray:
    """Integers in [lo, hi]: exactly representable in every storage type."""
    a = rng(*key).integers(lo, hi + 1, size=shape).astype(np.float32)
    return to_storage(a, dtype)


# ---- masks -----------------------------------------------------------------

def irrelevant_fraction(mask: np.ndarray) -> float:
    return 1.0 - float(np.count_nonzero(mask)) / mask.size


def mask_band_and_boxes(n: int, h: int, w: int, target: float, *key: int,
                        n_boxes: int = 3) -> np.ndarray:
    """Irrelevant = `n_boxes` random axis-aligned boxes plus a top band.

    Box sides are uniform in [h/7, h/2] (8..28 at 56x56); the band height is the
    one whose irrelevant fraction is closest to `target`."""
    g = rng(*key)
    out = np.ones((n, h, w), dtype=np.uint8)
    for b in range(n):
        boxes = np.zeros((h, w), dtype=bool)
        for _ in range(n_boxes):
            bh = int(g.integers(max(1, h // 7), max(2, h // 2) + 1))
            bw = int(g.integers(max(1, w // 7), max(2, w // 2) + 1))
            r0 = int(g.integers(0, h - bh + 1))
            c0 = int(g.integers(0, w - bw + 1))
            boxes[r0:r0 + bh, c0:c0 + bw] = True
        best, best_err = 0, 2.0
        for band in range(h + 1):
            irr = boxes.copy()
            irr[:band, :] = True
            err = abs(irr.mean() - target)
            if err < best_err:
                best, best_err = band, err
        boxes[:best, :] = True
        out[b][boxes] = 0
    return out


def _paint_objects(h, w, sky, cy, cx, hy, hx, scale):
    rel = np.zeros((h, w), dtype=bool)
    for y, x, a, b in zip(cy, cx, hy, hx):
        r0 = max(sky, int(np.floor(y - a * scale)))
        r1 = min(h, int(np.ceil(y + a * scale)))
        c0 = max(0, int(np.floor(x - b * scale)))
        c1 = min(w, int(np.ceil(x + b * scale)))
        if r1 > r0 and c1 > c0:
            rel[r0:r1, c0:c1] = True
    return rel


def mask_objects(n: int, h: int, w: int, irrelevant, *key: int, max_boxes: int = 6) -> np.ndarray:
    """Relevant = union of 1..max_boxes "object + context" boxes below a top sky
    band; everything else irrelevant.  One scale factor per image is bisected so
    that the irrelevant fraction is `irrelevant` (a float, or one per image).
    Exactly all-relevant at 0 and all-irrelevant at 1."""
    g = rng(*key)
    fr = np.broadcast_to(np.asarray(irrelevant, dtype=np.float64), (n,))
    out = np.zeros((n, h, w), dtype=np.uint8)
    for b in range(n):
        f = float(fr[b])
        k = int(g.integers(1, max_boxes + 1))
        cy = g.uniform(0.25 * h, 0.95 * h, size=k)
        cx = g.uniform(0.05 * w, 0.95 * w, size=k)
        hy = g.uniform(0.5, 1.0, size=k)
        hx = g.uniform(0.5, 1.5, size=k)
        if f <= 0.0:
            out[b] = 1
            continue
        if f >= 1.0:
            continue
        sky = int(round(min(0.15, 0.5 * f) * h))
        lo, hi = 0.0, 4.0 * max(h, w)
        for _ in range(40):
            mid = 0.5 * (lo + hi)
            kept = _paint_objects(h, w, sky, cy, cx, hy, hx, mid).mean()
            if kept < 1.0 - f:
                lo = mid
            else:
                hi = mid
        out[b] = _paint_objects(h, w, sky, cy, cx, hy, hx, hi)
    return out


def mask_bernoulli(n: int, h: int, w: int, irrelevant: float, *key: int) -> np.ndarray:
    """Each pixel irrelevant independently with probability `irrelevant`: the
    most fragmented mask there is."""
    g = rng(*key)
    return (g.random(size=(n, h, w), dtype=np.float32) >= np.float32(irrelevant)).astype(np.uint8)


def mask_depth_ramp(n: int, h: int, w: int, target: float, *key: int) -> np.ndarray:
    """Synthetic depth d = 1 - row/H + 0.15 * smooth noise (far at the top);
    pixels beyond a far plane are irrelevant; 3..10 tall pedestrian-shaped boxes
    (aspect about 1 : 2.5) are forced relevant; the far plane is bisected so the
    irrelevant fraction is `target`."""
    g = rng(*key)
    out = np.zeros((n, h, w), dtype=np.uint8)
    rows = (np.arange(h, dtype=np.float64) + 0.5) / h
    for b in range(n):
        cells = g.standard_normal(size=(9, 9))
        # bilinear interpolation of an 8x8-cell value-noise lattice
        ys = np.linspace(0.0, 8.0, h, endpoint=False)
        xs = np.linspace(0.0, 8.0, w, endpoint=False)
        y0 = ys.astype(int)
        x0 = xs.astype(int)
        ty = (ys - y0)[:, None]
        tx = (xs - x0)[None, :]
        c00 = cells[y0][:, x0]
        c01 = cells[y0][:, x0 + 1]
        c10 = cells[y0 + 1][:, x0]
        c11 = cells[y0 + 1][:, x0 + 1]
        noise = (c00 * (1 - ty) * (1 - tx) + c01 * (1 - ty) * tx
                 + c10 * ty * (1 - tx) + c11 * ty * tx)
        depth = (1.0 - rows)[:, None] + 0.15 * noise
        ped = np.zeros((h, w), dtype=bool)
        for _ in range(int(g.integers(3, 11))):
            bw = int(g.integers(max(1, w // 60), max(2, w // 20) + 1))
            bh = min(h, int(2.5 * bw))
            r0 = int(g.integers(0, h - bh + 1))
            c0 = int(g.integers(0, w - bw + 1))
            ped[r0:r0 + bh, c0:c0 + bw] = True
        lo, hi = float(depth.min()) - 1.0, float(depth.max()) + 1.0
        for _ in range(40):
            mid = 0.5 * (lo + hi)
            irr = ((depth > mid) & ~ped).mean()
            if irr > target:
                lo = mid
            else:
                hi = mid
        out[b] = ~((depth > hi) & ~ped)
    return out
