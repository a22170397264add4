"""Counter-based dropout mask of the oracle (test infrastructure, independent of the HIP path).

The paper fuses dropout into the bias+dropout+residual+LayerNorm pattern (section 2.2 and the
appendix schedule) but leaves the random generator to the framework. The reading taken here: the
keep/drop decision of an element is a pure function of (seed, layer, site, element index), computed
with the published Philox4x32-10 block function (Salmon et al., SC'11), so the backward pass and an
independent implementation can regenerate it.

  element index  e = t*H + c                      (row-major position in the [T, H] tensor)
  counter        (lo32(e>>3), hi32(e>>3), site, layer_id),  key (lo32(seed), hi32(seed))
  16-bit draw    r16 = (out[(e & 7) >> 1] >> (16 * (e & 1))) & 0xffff
  keep           r16 >= thr,  thr = p * 65536 rounded to the nearest integer, halves away from zero, with p
                 the probability as the single-precision number the layer descriptor carries

All arithmetic is done on numpy uint64 arrays holding 32-bit quantities.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32 on arrays of counters; returns the four output words (uint64 arrays < 2^32)."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) for c in (c0, c1, c2, c3))
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0            # 64-bit product of two 32-bit numbers
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK32
        hi1, lo1 = p1 >> _SH32, p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def dropout_threshold(p: float) -> int:
    """16-bit threshold of a drop probability. The probability travels in a single-precision descriptor field,
    so it is rounded to single precision first; its product with 2^16 is then exact in double precision and is
    rounded to the nearest integer with halves going up (p >= 0, so up is away from zero)."""
    return int(np.floor(float(np.float32(p)) * 65536.0 + 0.5))


def keep_mask(n_elements: int, p: float, seed: int, site: int, layer_id: int) -> np.ndarray:
    """Boolean keep mask for elements e = 0..n_elements-1 of one dropout site."""
    e = np.arange(n_elements, dtype=np.uint64)
    blk = e >> np.uint64(3)
    out = philox4x32_10(blk & _MASK32, blk >> _SH32, np.full_like(blk, site), np.full_like(blk, layer_id),
                        seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = np.stack(out, axis=0)                           # [4, n]
    sel = ((e & np.uint64(7)) >> np.uint64(1)).astype(np.int64)
    w = words[sel, np.arange(n_elements)]
    r16 = (w >> (np.uint64(16) * (e & np.uint64(1)))) & np.uint64(0xFFFF)
    return r16 >= np.uint64(dropout_threshold(p))
