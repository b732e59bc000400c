"""Second, independent statement of the stream format in pure Python.

Test infrastructure only.  The paper names the entropy coder (ANS, Sec. 2.2)
but gives no stream layout, so the layout used here cannot be pinned to the
paper ("parity unpinned").  To keep a slip in the C oracle from going
unnoticed, this file states the same format a second time, organised
differently (one state at a time over explicit symbol lists, Python integers,
linear search through the cumulative table) and the tests require both to
produce the same bytes on small inputs.  It imports nothing from the C oracle.
"""
import struct

PROB_BITS = 12
M = 1 << PROB_BITS
CHUNK = 4096
K = 16
G = 8
L = 1 << 16


def exponent(u):
    """Alg. 1 "split": the 8 bits under the sign bit of a bf16 word."""
    return (u >> 7) & 0xFF


def quantise(cnt, guard=0):
    """Counts -> integer frequencies summing to M (0 for absent symbols).  With guard > 0 the
    exponents up to that far outside the occupied range, and exponent 0, are kept codable (f = 1)."""
    total = sum(cnt)
    if total == 0:
        return [0] * 256
    present = [s for s in range(256) if cnt[s]]
    kept = set(present)
    if guard:
        kept |= set(range(max(0, present[0] - guard), min(255, present[-1] + guard) + 1)) | {0}
    f = [max(1, cnt[s] * M // total) if s in kept else 0 for s in range(256)]
    rest = M - sum(f)
    if rest > 0:
        top = max(range(256), key=lambda s: (cnt[s], -s))
        f[top] += rest
    for _ in range(-rest if rest < 0 else 0):
        top = max(range(256), key=lambda s: (f[s], -s))
        f[top] -= 1
    return f


def starts(freq):
    c, out = 0, []
    for f in freq:
        out.append(c)
        c += f
    return out


def state_symbols(m, j, k_states=K, g=G):
    """Local indices coded by state j, in decoding order."""
    return [i for i in range(m) if (i % (k_states * g)) // g == j]


def encode_state(symbols, freq):
    """Symbols of one state in decoding order -> (final state, words in decoding order)."""
    start = starts(freq)
    x = L
    emitted = []
    for s in reversed(symbols):
        f = freq[s]
        assert f > 0
        if x >= ((L >> PROB_BITS) << 16) * f:
            emitted.append(x & 0xFFFF)
            x >>= 16
        q, r = divmod(x, f)
        x = q * M + start[s] + r
        assert L <= x < (L << 16)
    emitted.reverse()
    return x, emitted


def decode_state(count, freq, x, words):
    start = starts(freq)
    out = []
    pos = 0
    for _ in range(count):
        slot = x % M
        s = 0
        while not (start[s] <= slot < start[s] + freq[s]):
            s += 1
        out.append(s)
        x = freq[s] * (x // M) + slot - start[s]
        if x < L:
            x = x * 65536 + words[pos]
            pos += 1
    assert x == L and pos == len(words)
    return out


def pack_signmant(words16, k):
    """Sec. 2.3 / App. D: (k+1)-bit signed field, 8/(k+1) per byte, low bits first."""
    width = k + 1
    per = 8 // width
    out = bytearray((len(words16) * width + 7) // 8)
    for i, u in enumerate(words16):
        field = ((u >> 15) << k) | ((u & 0x7F) >> (7 - k))
        out[i // per] |= field << ((i % per) * width)
    return bytes(out)


def _pad(b):
    return b + bytes((-len(b)) % 16)


def _f32(bits):
    return struct.unpack("<f", struct.pack("<I", bits & 0xFFFFFFFF))[0]


def _bits(value):
    """IEEE binary32 bit pattern of a Python float (rounds to nearest even, as struct does)."""
    try:
        return struct.unpack("<I", struct.pack("<f", value))[0]
    except OverflowError:
        return 0x7F800000 if value > 0 else 0xFF800000


def bf16_round(bits32):
    if (bits32 & 0x7FFFFFFF) > 0x7F800000:
        return (bits32 >> 16) | 0x40
    return ((bits32 + 0x7FFF + ((bits32 >> 16) & 1)) >> 16) & 0xFFFF


def block_coefficients(words16, block):
    """Sec. 2.3: per block, the mantissa of the weight of largest magnitude (first on ties)."""
    out = []
    for b in range(0, len(words16), block):
        blk = words16[b:b + block]
        best = max(range(len(blk)), key=lambda i: (blk[i] & 0x7FFF, -i))
        out.append(blk[best] & 0x7F)
    return out


def scale(words16, block, coef, divide):
    """bf16(w / c) or bf16(w * c), c = 1 + coef/128, in binary32 (Python doubles hold the exact
    product, and a quotient of two bf16 values is never close enough to a binary32 tie for the
    extra rounding through double to matter)."""
    out = []
    for i, u in enumerate(words16):
        c = 1.0 + coef[i // block] / 128.0
        v = _f32(u << 16)
        if v != v:
            out.append(u | 0x40)
            continue
        r = v / c if divide else v * c
        out.append(bf16_round(_bits(r)))
    return out


def compress(words16, k=7, block=0, guard=0, freq=None, low=None, half=False):
    """List of bf16 words -> container bytes.  freq: an earlier table to code with.  low: the lower
    halves of binary32 words whose upper halves are words16 (stored as a raw plane).  half: the
    words are binary16 -- the symbol is a word's upper byte, its lower byte is stored raw."""
    if half and (k != 7 or block or low is not None):
        raise ValueError("binary16 is lossless only")
    coef = []
    if block:
        coef = block_coefficients(words16, block)
        words16 = scale(words16, block, coef, divide=True)
    n = len(words16)
    expo = [u >> 8 for u in words16] if half else [exponent(u) for u in words16]
    cnt = [0] * 256
    for e in expo:
        cnt[e] += 1
    if freq is None:
        freq = quantise(cnt, guard)
    freq = [int(v) for v in freq]
    nc = (n + CHUNK - 1) // CHUNK
    offsets, states, lens, payload = [], [], [], []
    for c in range(nc):
        chunk = expo[c * CHUNK:(c + 1) * CHUNK]
        offsets.append(len(payload))
        for j in range(K):
            syms = [chunk[i] for i in state_symbols(len(chunk), j)]
            x, run = encode_state(syms, freq)
            states.append(x)
            lens.append(len(run))
            payload.extend(run)
    offsets.append(len(payload))
    header = struct.pack("<IIQIIIIIIQIII", 0x315A554E, 1, n, k, PROB_BITS, CHUNK, K, G, nc, len(payload), block,
                         guard, 2 if half else (0 if low is None else 1))
    header += bytes(64 - len(header))
    out = header
    out += struct.pack("<256H", *freq)
    out += _pad(struct.pack(f"<{nc + 1}I", *offsets))
    out += struct.pack(f"<{nc * K}I", *states)
    out += bytes(lens)
    out += _pad(struct.pack(f"<{len(payload)}H", *payload))
    out += _pad(bytes(u & 0xFF for u in words16) if half else pack_signmant(words16, k))
    if low is not None:
        out += _pad(struct.pack(f"<{n}H", *low))
    if block:
        out += _pad(bytes(coef))
    return out


def decompress(blob):
    """Container bytes -> list of bf16 words."""
    magic, ver, n, k, pb, chunk, ks, g, nc, tw, block, _guard, elem = struct.unpack_from("<IIQIIIIIIQIII", blob, 0)
    f32, half = elem == 1, elem == 2
    assert (magic, ver, pb, chunk, ks, g) == (0x315A554E, 1, PROB_BITS, CHUNK, K, G)
    pos = 64
    freq = list(struct.unpack_from("<256H", blob, pos)); pos += 512
    offsets = struct.unpack_from(f"<{nc + 1}I", blob, pos); pos += ((nc + 1) * 4 + 15) // 16 * 16
    states = struct.unpack_from(f"<{nc * K}I", blob, pos); pos += nc * K * 4
    lens = blob[pos:pos + nc * K]; pos += nc * K
    payload = struct.unpack_from(f"<{tw}H", blob, pos); pos += (tw * 2 + 15) // 16 * 16
    sm = blob[pos:]
    after_sm = pos + ((n * (k + 1) + 7) // 8 + 15) // 16 * 16
    low = struct.unpack_from(f"<{n}H", blob, after_sm) if f32 else None
    coef = list(blob[after_sm:]) if block else []
    width, per = k + 1, 8 // (k + 1)
    out = [0] * n
    for c in range(nc):
        m = min(CHUNK, n - c * CHUNK)
        at = offsets[c]
        for j in range(K):
            idx = state_symbols(m, j)
            run = payload[at:at + lens[c * K + j]]
            at += lens[c * K + j]
            for i, e in zip(idx, decode_state(len(idx), freq, states[c * K + j], run)):
                gi = c * CHUNK + i
                field = (sm[gi // per] >> ((gi % per) * width)) & ((1 << width) - 1)
                if half:
                    out[gi] = (e << 8) | field           # symbol = upper byte, raw lower byte
                else:
                    out[gi] = ((field >> k) << 15) | (e << 7) | ((field & ((1 << k) - 1)) << (7 - k))
        assert at == offsets[c + 1]
    if block:
        out = scale(out, block, coef, divide=False)
    if f32:
        out = [(hi << 16) | lo for hi, lo in zip(out, low)]
    return out
