"""GF(2^128) arithmetic on Python integers and what tests build from it: the pre-counter block
J0 of an IV that is not 96 bits long (SP 800-38D 7.1 step 2), and 16-byte IVs solved for a wanted
J0, which put the 32-bit counter wherever a test needs it (just below its wrap, say).

Independent of the oracle and of the GPU library: a block is read as a polynomial whose
coefficient of x^i is bit i counted from the most significant bit of byte 0."""

_R = (1 << 128) | (1 << 7) | (1 << 2) | (1 << 1) | 1   # x^128 + x^7 + x^2 + x + 1


def to_poly(block: bytes) -> int:
    v = int.from_bytes(block, "big")
    return int(format(v, "0128b")[::-1], 2)      # coefficient of x^i at integer bit i


def from_poly(p: int) -> bytes:
    return int(format(p, "0128b")[::-1], 2).to_bytes(16, "big")


def mul(a: int, b: int) -> int:
    r = 0
    while b:
        if b & 1:
            r ^= a
        b >>= 1
        a <<= 1
        if a >> 128:
            a ^= _R
    return r


def inverse(a: int) -> int:
    """a^(2^128 - 2) by square and multiply"""
    r, e, s = 1, (1 << 128) - 2, a
    while e:
        if e & 1:
            r = mul(r, s)
        s = mul(s, s)
        e >>= 1
    return r


def ghash(h: bytes, data: bytes) -> bytes:
    assert len(data) % 16 == 0
    hp, y = to_poly(h), 0
    for i in range(0, len(data), 16):
        y = mul(y ^ to_poly(data[i:i + 16]), hp)
    return from_poly(y)


def j0_of(h: bytes, iv: bytes) -> bytes:
    if len(iv) == 12:
        return iv + b"\x00\x00\x00\x01"
    pad = (-len(iv)) % 16
    return ghash(h, iv + bytes(pad) + bytes(8) + (8 * len(iv)).to_bytes(8, "big"))


def iv_for_j0(h: bytes, j0: bytes) -> bytes:
    """the 16-byte IV whose pre-counter block is j0:  J0 = IV H^2 + L H  with L the length block"""
    hp = to_poly(h)
    length_block = to_poly(bytes(8) + (128).to_bytes(8, "big"))
    inv_h2 = inverse(mul(hp, hp))
    return from_poly(mul(to_poly(j0) ^ mul(length_block, hp), inv_h2))
