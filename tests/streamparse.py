"""Independent pure-Python reader of the compressed container, token by token.

Written from the container description alone (header fields, value plane, block directory, per-block
flags plane and payload plane, LSB-first bits); it calls nothing from the oracle or the HIP path, so
it pins the byte layout both of them must produce.  Slow: use on small streams only.
"""
import struct
from fractions import Fraction


def bitlen(x):
    return int(x).bit_length()


def level_len(i, M, l):
    return -((-i * M) >> l)          # ceil(i*M / 2^l)


def _bits(buf, pos, n):
    v = 0
    for k in range(n):
        v |= ((buf[(pos + k) >> 3] >> ((pos + k) & 7)) & 1) << k
    return v


def parse(stream):
    s = bytes(stream)
    assert len(s) >= 64
    magic, version, l, tau, KB, nb = struct.unpack_from("<4sBBHII", s, 0)
    base, S = struct.unpack_from("<dd", s, 16)
    n, d, total, rsv = struct.unpack_from("<QQQQ", s, 32)
    assert magic == b"FSGD" and version == 1 and 1 <= tau <= 256 and rsv == 0
    assert total == len(s), (total, len(s))
    assert nb == -(-d // KB)
    # value plane: d tokens of w = 1 + ceil(log2 tau) bits, low bits code-1, top bit the sign; reported
    # as sign << 7 | code-1 for every w up to 8 (tau <= 128), and as the 9-bit token itself above that;
    # "code" (1..tau) and "negative" give the two parts whatever w is
    w = 1 + (tau - 1).bit_length()
    dir_off = 64 + 8 * (-(-(d * w) // 64))
    plane = s[64:dir_off]
    toks = [_bits(plane, j * w, w) for j in range(d)]
    codes = [((t >> (w - 1)) << 7) | (t & ((1 << (w - 1)) - 1)) for t in toks] if w <= 8 else toks
    code = [(t & ((1 << (w - 1)) - 1)) + 1 for t in toks]
    negative = [bool(t >> (w - 1)) for t in toks]
    assert _bits(plane, d * w, 8 * len(plane) - d * w) == 0, "value-plane padding must be zero"
    blocks_off = dir_off + 16 * nb
    keys, tokens, off_expect = [], [], 0
    payload_at = []          # absolute bit position in the stream of every key's binary delta
    last = 0
    for blk in range(nb):
        off8, pre, M, pbits = struct.unpack_from("<IIII", s, dir_off + 16 * blk)
        cnt = min(KB, d - blk * KB)
        assert off8 == off_expect and pre == last and 1 <= M <= 32
        fwords = -(-(cnt * l) // 64)
        pwords = -(-pbits // 64)
        fl = s[blocks_off + 8 * off8: blocks_off + 8 * (off8 + fwords)]
        pl = s[blocks_off + 8 * (off8 + fwords): blocks_off + 8 * (off8 + fwords + pwords)]
        pos, key, maxd = 0, pre, 0
        for i in range(cnt):
            level = _bits(fl, i * l, l) + 1
            ln = level_len(level, M, l)
            delta = _bits(pl, pos, ln)
            payload_at.append(8 * (blocks_off + 8 * (off8 + fwords)) + pos)
            pos += ln
            key += delta
            maxd = max(maxd, delta)
            keys.append(key)
            tokens.append((level, ln, delta, M))
        assert pos == pbits
        assert max(1, bitlen(maxd)) == M, "M must be the bit length of the block's largest delta"
        assert _bits(fl, cnt * l, 64 * fwords - cnt * l) == 0, "flag padding must be zero"
        assert _bits(pl, pbits, 64 * pwords - pbits) == 0, "payload padding must be zero"
        last = key
        off_expect = off8 + fwords + pwords
    assert blocks_off + 8 * off_expect == total
    return dict(l=l, tau=tau, KB=KB, nb=nb, w=w, base=base, S=S, n=n, d=d, total=total,
                codes=codes, code=code, negative=negative, keys=keys, tokens=tokens, payload_at=payload_at)


def exact_code(abs_v, S, base, limit=4096):
    """ceil(log_b(S/|v|)) by exact rationals: the least integer c >= 0 with |v| * b^c >= S.

    Returns (c, margin) where margin is the relative distance of log-space position from the nearest
    boundary, so callers can skip values that sit on a boundary to within float64 round-off."""
    a, s, b = Fraction(abs_v), Fraction(S), Fraction(base)
    c, p = 0, Fraction(1)
    while a * p < s:
        p *= b
        c += 1
        if c > limit:
            return None, 0.0
    hi = float(a * p / s) - 1.0                      # >= 0: how far past the boundary it passed
    lo = 1.0 - float(a * p / b / s) if c > 0 else 1.0  # > 0: how far short of the previous one
    return c, min(abs(hi), abs(lo))


def with_zero_delta(stream, rank):
    """A copy of `stream` (a uint8 array) in which the binary delta of key number `rank` is all zeros, so
    that the key repeats its predecessor: a stream no encoder writes (Eq. 4 is taken over distinct keys)."""
    info = parse(stream)
    out = stream.copy()
    pos, ln = info["payload_at"][rank], info["tokens"][rank][1]
    for k in range(ln):
        out[(pos + k) >> 3] &= ~(1 << ((pos + k) & 7)) & 0xFF
    return out
