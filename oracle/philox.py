"""Philox-4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11), written from the
published description with Python integers (test oracle).  Counter words (slot, seq, step_lo, step_hi),
key words (seed_lo, seed_hi); the uniform of a slot is the top 24 bits of output word 0 times 2^-24,
so it lies in [0, 1) and is exactly representable in fp32."""

M0, M1 = 0xD2511F53, 0xCD9E8D57          # round multipliers
W0, W1 = 0x9E3779B9, 0xBB67AE85          # key schedule increments (golden ratio, sqrt(3)-1)
MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    c0, c1, c2, c3 = counter
    k0, k1 = key
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & MASK, p1 & MASK, ((p0 >> 32) ^ c3 ^ k1) & MASK, p0 & MASK
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def uniform24(seed, seq, step, slot):
    """The uniform in [0,1) on the 2^-24 grid for (seed, sequence, step counter, slot)."""
    out = philox4x32_10((slot & MASK, seq & MASK, step & MASK, (step >> 32) & MASK),
                        (seed & MASK, (seed >> 32) & MASK))
    return (out[0] >> 8) * (2.0 ** -24)
