"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names what fixes the expected value: IEEE/numpy float semantics, a
library routine, a closed form, a hand-worked value in tests/golden/, brute
force on tiny inputs, or the independent pure-Python statement of the format.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy import stats

from oracle import oracle as O
from oracle import py_rans as P
from paper_2410_20650_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALL = np.arange(65536, dtype=np.uint16)


def as_float(words):
    """bf16 words -> the real numbers they denote, via numpy's fp32 (bf16 is its upper half)."""
    with np.errstate(invalid="ignore"):                         # signalling NaNs are fine here
        return (words.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------- split / merge (Alg. 1, App. D)

def test_split_agrees_with_ieee_meaning_of_every_pattern():
    s, e, m = O.split(ALL)
    v = as_float(ALL)
    finite = np.isfinite(v)
    normal = finite & (np.abs(v) >= 2.0 ** -126)
    # sign: numpy's signbit of the value
    assert np.array_equal(s.astype(bool), np.signbit(v))
    # normal numbers: |v| = 2^(E-127) * (1 + mant/128)
    frac, ex = np.frexp(np.abs(v[normal]))            # |v| = frac * 2^ex, frac in [0.5, 1)
    assert np.array_equal(e[normal], (ex - 1 + 127).astype(np.uint8))
    assert np.array_equal(m[normal], ((frac * 2 - 1) * 128).astype(np.uint8))
    # zeros and subnormals: exponent field 0, |v| = 2^-126 * mant/128
    sub = finite & ~normal
    assert np.all(e[sub] == 0)
    assert np.array_equal(m[sub], (np.abs(v[sub]) * 2.0 ** 126 * 128).astype(np.uint8))
    # Inf / NaN: exponent field all ones; Inf has mantissa 0
    assert np.all(e[~finite] == 255)
    assert np.array_equal(m[~finite] == 0, np.isinf(v[~finite]))


def test_merge_inverts_split_on_every_pattern():
    assert np.array_equal(O.merge(*O.split(ALL)), ALL)


# ---------------------------------------------------------------- truncation (Sec. 2.3)

@pytest.mark.parametrize("k", [7, 3, 1, 0])
def test_truncate_is_round_toward_zero_to_k_mantissa_bits(k):
    t = O.truncate(ALL, k)
    v, vt = as_float(ALL), as_float(t)
    normal = np.isfinite(v) & (np.abs(v) >= 2.0 ** -126)
    # independent definition on the reals: largest multiple of 2^(E-127-k) not above |v|
    _, ex = np.frexp(np.abs(v[normal]))
    ulp = np.ldexp(1.0, ex - 1 - k)
    expect = np.copysign(np.floor(np.abs(v[normal]) / ulp) * ulp, v[normal])
    assert np.array_equal(vt[normal], expect)
    # the paper's bound: relative change below 2^-k, sign and binade kept
    rel = np.abs(v[normal] - vt[normal]) / np.abs(v[normal])
    assert rel.max() < 2.0 ** -k
    assert np.array_equal(np.signbit(vt), np.signbit(v))
    assert np.array_equal(np.frexp(np.abs(vt[normal]))[1], ex)
    assert np.array_equal(O.truncate(t, k), t)                 # idempotent
    if k == 7:
        assert np.array_equal(t, ALL)


# ---------------------------------------------------------------- signed-mantissa packing (Sec. 2.3, App. D)

@pytest.mark.parametrize("k", [7, 3, 1, 0])
@pytest.mark.parametrize("n", [0, 1, 5, 8, 13, 65536])
def test_pack_signmant_layout(k, n):
    w = ALL[:n] if n <= 65536 else ALL
    if n and n < 65536:
        w = np.random.default_rng(n + k).integers(0, 65536, n).astype(np.uint16)
    packed = O.pack_signmant(w, k)
    assert packed.size == math.ceil(n * (k + 1) / 8)
    # unpack with numpy's bit unpacker: field i occupies bits [i*(k+1), (i+1)*(k+1)) LSB first
    bits = np.unpackbits(packed, bitorder="little")
    assert np.all(bits[n * (k + 1):] == 0)                      # padding is zero
    fields = bits[: n * (k + 1)].reshape(n, k + 1)
    v = as_float(w)
    assert np.array_equal(fields[:, k].astype(bool), np.signbit(v))   # sign is the top bit
    kept = (fields[:, :k] << np.arange(k)).sum(axis=1) if k else np.zeros(n, int)
    _, _, mant = O.split(w)
    assert np.array_equal(kept, mant >> (7 - k))
    assert packed.tobytes() == P.pack_signmant([int(u) for u in w], k)


# ---------------------------------------------------------------- statistics (Sec. 2.2, Eq. 1)

def test_histogram_matches_bincount_of_float_exponents():
    w = inputs.bits(inputs.gaussian_bf16(200_000, seed=11))
    v = as_float(w)
    _, ex = np.frexp(np.abs(v))                                 # all values are normal here
    assert np.all(np.abs(v[v != 0]) >= 2.0 ** -126)
    field = np.where(v == 0, 0, ex - 1 + 127)
    assert np.array_equal(O.histogram(w), np.bincount(field, minlength=256).astype(np.uint64))
    assert int(O.histogram(w).sum()) == w.size
    assert O.histogram(np.zeros(0, np.uint16)).sum() == 0


def test_entropy_closed_cases():
    c = np.zeros(256, np.uint64)
    assert O.entropy(c) == 0.0
    c[17] = 5
    assert O.entropy(c) == 0.0
    c[200] = 5
    assert O.entropy(c) == pytest.approx(1.0, abs=1e-12)
    assert O.entropy(np.full(256, 3, np.uint64)) == pytest.approx(8.0, abs=1e-12)
    c = np.zeros(256, np.uint64)
    c[:4] = [4, 2, 1, 1]                                        # 1/2, 1/4, 1/8, 1/8 -> 1.75 bits
    assert O.entropy(c) == pytest.approx(1.75, abs=1e-12)
    f = np.zeros(256, np.uint16)
    f[:4] = [2048, 1024, 512, 512]
    assert O.cross_entropy(c, f) == pytest.approx(1.75, abs=1e-12)
    f[:4] = [1024, 1024, 1024, 1024]
    assert O.cross_entropy(c, f) == pytest.approx(2.0, abs=1e-12)


def gaussian_exponent_pmf(std):
    """P(exponent field = E) for bf16(round-to-nearest-even(N(0, std^2))), from the normal CDF.

    A value rounds into binade E when 2^(E-127) * (1 - 2^-9) <= |x| < 2^(E-126) * (1 - 2^-9)
    (half of the last bf16 step below a power of two already rounds up to it).
    """
    p = np.zeros(256)
    shift = 1.0 - 2.0 ** -9
    for E in range(1, 255):
        lo, hi = 2.0 ** (E - 127) * shift, 2.0 ** (E - 126) * shift
        p[E] = 2 * (stats.norm.cdf(hi / std) - stats.norm.cdf(lo / std))
    p[0] = 1 - p.sum()
    return p


def test_exponent_entropy_of_gaussian_weights_matches_closed_form():
    p = gaussian_exponent_pmf(0.02)
    h_closed = -(p[p > 0] * np.log2(p[p > 0])).sum()
    assert h_closed == pytest.approx(2.545, abs=2e-3)           # "less than 3 bits" (Sec. 2.1)
    w = inputs.bits(inputs.gaussian_bf16(4_000_000, seed=12))
    cnt = O.histogram(w)
    assert O.entropy(cnt) == pytest.approx(h_closed, abs=5e-3)
    emp = cnt / cnt.sum()
    assert np.abs(emp - p).max() < 2e-3
    # mantissa and sign carry (almost) their full width, as Fig. 1 reports
    s, _, m = O.split(w)
    pm = np.bincount(m, minlength=128) / m.size
    assert -(pm[pm > 0] * np.log2(pm[pm > 0])).sum() > 6.95
    assert abs(s.mean() - 0.5) < 2e-3


# ---------------------------------------------------------------- frequency table

def test_quantise_closed_cases():
    c = np.zeros(256, np.uint64)
    assert O.quantise(c).sum() == 0
    c[42] = 9
    f = O.quantise(c)
    assert f[42] == 4096 and f.sum() == 4096
    c[7] = 9
    f = O.quantise(c)
    assert f[7] == 2048 and f[42] == 2048
    f = O.quantise(np.full(256, 123, np.uint64))
    assert np.all(f == 16)
    # 255 singletons and one huge count: every singleton keeps f = 1, the rest goes to the big one
    c = np.ones(256, np.uint64)
    c[100] = 10 ** 9
    f = O.quantise(c)
    assert f[100] == 4096 - 255 and np.all(np.delete(f, 100) == 1)
    # three equal counts: floor gives 1365 each, the shortfall of 1 goes to the lowest symbol
    c = np.zeros(256, np.uint64)
    c[[9, 3, 200]] = 50
    f = O.quantise(c)
    assert (f[3], f[9], f[200]) == (1366, 1365, 1365)


def test_quantise_excess_is_taken_from_the_largest():
    # 200 symbols with count 1 and 56 with count 100: floors are 0 -> 1 for the rare ones,
    # floor(100*4096/5800) = 70 for the common ones; 200 + 56*70 = 4120 > 4096, so 24 units
    # come off the largest entries, lowest symbol first.
    c = np.ones(256, np.uint64)
    c[:56] = 100
    f = O.quantise(c)
    assert f.sum() == 4096
    assert np.all(f[56:] == 1)
    assert np.all(f[:24] == 69) and np.all(f[24:56] == 70)


def test_quantise_properties_and_second_implementation():
    rng = np.random.default_rng(5)
    for trial in range(200):
        k = int(rng.integers(1, 257))
        c = np.zeros(256, np.uint64)
        idx = rng.choice(256, k, replace=False)
        c[idx] = (rng.pareto(0.7, k) * 10 + 1).astype(np.uint64)
        f = O.quantise(c)
        assert f.sum() == 4096
        assert np.array_equal(f > 0, c > 0)
        assert list(f) == P.quantise([int(x) for x in c])
        # never costs much more than the empirical entropy
        assert O.cross_entropy(c, f) >= O.entropy(c) - 1e-9


# ---------------------------------------------------------------- rANS step arithmetic (Sec. 2.2)

def golden_steps():
    rows = []
    with open(os.path.join(GOLDEN, "rans_steps.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if line:
                f, c, x0, x1 = (int(t) for t in line[:4])
                rows.append((f, c, x0, x1, None if line[4] == "-" else int(line[4])))
    return rows


def test_rans_steps_match_hand_worked_values():
    rows = golden_steps()
    assert len(rows) == 8
    for f, c, x0, x1, word in rows:
        assert O.rans_encode_step(x0, f, c) == (x1, word)
        # and the decoder undoes exactly that step
        back, consumed = O.rans_decode_step(x1, f, c, 0 if word is None else word)
        assert back == x0 and consumed == (word is not None)


def test_rans_step_is_a_bijection_that_keeps_the_state_interval():
    rng = np.random.default_rng(9)
    for _ in range(20000):
        f = int(rng.integers(1, 4096))
        c = int(rng.integers(0, 4096 - f + 1))
        x = int(rng.integers(1 << 16, 1 << 32))
        xn, word = O.rans_encode_step(x, f, c)
        assert (1 << 16) <= xn < (1 << 32)
        assert c <= xn % 4096 < c + f                           # the slot names the symbol
        back, consumed = O.rans_decode_step(xn, f, c, word or 0)
        assert back == x and consumed == (word is not None)


def test_equal_halves_turn_the_state_into_the_binary_number():
    # With two symbols of frequency M/2 every step appends one bit: starting from 2^16 the
    # state after n <= 15 steps is 2^(16+n) + 2048 * (the bits read as a binary number).
    freq = np.zeros(256, np.uint16)
    freq[[10, 20]] = 2048
    for bits in itertools.product([0, 1], repeat=6):
        sym = [10 if b == 0 else 20 for b in bits]
        states, lens, runs = O.encode_chunk(sym, freq, k_states=1, g=1)
        value = 0
        for b in reversed(bits):                                # the coder runs back to front
            value = 2 * value + b
        assert int(states[0]) == (1 << (16 + len(bits))) + 2048 * value
        assert lens[0] == 0


def test_single_symbol_chunk_never_emits():
    freq = np.zeros(256, np.uint16)
    freq[121] = 4096
    states, lens, runs = O.encode_chunk(np.full(4096, 121, np.uint8), freq)
    assert np.all(states == 65536) and np.all(lens == 0)
    assert np.all(O.decode_chunk(4096, freq, states, runs) == 121)


def test_chunk_codec_brute_force_small_alphabets():
    tables = [{0: 4096}, {0: 2048, 1: 2048}, {0: 4095, 1: 1}, {0: 1, 1: 4095},
              {3: 1, 7: 2, 9: 4093}, {3: 1365, 7: 1365, 9: 1366}, {0: 1, 128: 1, 255: 4094}]
    for table in tables:
        freq = np.zeros(256, np.uint16)
        for s, f in table.items():
            freq[s] = f
        alphabet = sorted(table)
        for n in range(0, 9):
            for seq in itertools.product(alphabet, repeat=n):
                for K, G in ((1, 1), (2, 2), (3, 1)):
                    states, lens, runs = O.encode_chunk(seq, freq, k_states=K, g=G, words_cap=16)
                    back = O.decode_chunk(n, freq, states, runs, k_states=K, g=G)
                    assert tuple(back) == seq
                    # the independent per-state coder gives the same states and words
                    for j in range(K):
                        mine = [seq[i] for i in P.state_symbols(n, j, K, G)]
                        x, words = P.encode_state(mine, [int(f) for f in freq])
                        assert x == int(states[j]) and words == list(runs[j])


def test_long_rare_symbol_run_hits_the_word_capacity_bound():
    # 4096 symbols of frequency 1 cost 12 bits each: 256 per state -> exactly 192 words per state
    freq = np.zeros(256, np.uint16)
    freq[0] = 4095
    freq[255] = 1
    states, lens, runs = O.encode_chunk(np.full(4096, 255, np.uint8), freq, words_cap=192)
    assert np.all(lens == 192)
    assert np.all(O.decode_chunk(4096, freq, states, runs) == 255)


def test_no_state_emits_more_than_193_words_for_256_symbols():
    # The bound the format's run lengths rest on (one byte per run, slots of 200 words), in two parts.
    # 1) The two inequalities of the argument, checked on the oracle's own step for every frequency at the
    #    edges of its ranges and at random states (integers only):
    #      a step without a word:  x' + 1 <= 4096 (x + 1)                  (log2(x + 1) grows by at most 12)
    #      a step with a word:     the state falls to y = x >> 16 >= 16 before it is advanced, so
    #                              y + 1 <= (17/16) y <= (17/16) (x + 1) / 65536, and then the same growth
    #    With t words among 256 steps:  16 <= log2(x_end + 1) <= log2(65537) + 256 * 12 - t (16 - log2(17/16)),
    #    so t <= (log2(65537) - 16 + 3072) / (16 - log2(17/16)) = 193.06.
    rng = np.random.default_rng(7)
    for f in range(1, 4097):
        limit = f << 20
        cums = (0, 4096 - f)
        quiet = [1 << 16, min(limit, 1 << 32) - 1] + [int(v) for v in rng.integers(1 << 16, min(limit, 1 << 32), 3)]
        for x in quiet:
            for c in cums:
                xn, word = O.rans_encode_step(x, f, c)
                assert word is None and (1 << 16) <= xn < (1 << 32)
                assert xn + 1 <= 4096 * (x + 1)
        if limit < (1 << 32):
            loud = [limit, (1 << 32) - 1, limit | 0xFFFF] + [int(v) for v in rng.integers(limit, 1 << 32, 3)]
            for x in loud:
                for c in cums:
                    xn, word = O.rans_encode_step(x, f, c)
                    y = x >> 16
                    assert word == (x & 0xFFFF) and y >= 16 * f
                    assert 16 * (y + 1) <= 17 * y and 65536 * y <= x
                    assert (1 << 16) <= xn < (1 << 32) and xn + 1 <= 4096 * (y + 1)
    assert math.floor((math.log2(65537) - 16 + 256 * 12) / (16 - math.log2(17 / 16))) == 193
    # 2) A search for a long run (a heuristic, the proof is part 1): per step and per number of words so
    #    far, the largest states reached are kept and every choice of a rare symbol is tried.  It finds
    #    192, the all-rare case of the test above, and nothing beyond the bound.
    choices = [(f, c) for f in (1, 2, 3, 4, 8) for c in (0, 4096 - f)]
    front = {0: {1 << 16}}
    for _ in range(256):
        nxt = {}
        for words, states in front.items():
            for x in states:
                for f, c in choices:
                    xn, word = O.rans_encode_step(x, f, c)
                    nxt.setdefault(words + (word is not None), set()).add(xn)
        front = {wd: set(sorted(st)[-6:]) for wd, st in nxt.items() if wd >= max(nxt) - 2}
    assert 192 <= max(front) <= 193


# ---------------------------------------------------------------- container: both statements of the format agree

@pytest.mark.parametrize("k", [7, 3, 1, 0])
@pytest.mark.parametrize("n", [0, 1, 7, 130, 4096, 4097, 9001])
def test_c_oracle_and_python_codec_write_identical_bytes(n, k):
    w = inputs.bits(inputs.gaussian_bf16(n, seed=100 + n)) if n else np.zeros(0, np.uint16)
    blob = O.compress(w, k, threads=2)
    mine = P.compress([int(u) for u in w], k)
    assert blob.tobytes() == mine
    assert P.decompress(mine) == [int(u) for u in O.truncate(w, k)]
    assert np.array_equal(O.decompress(np.frombuffer(mine, np.uint8), n), O.truncate(w, k))


def test_python_codec_decodes_heavy_tailed_blob_from_c_oracle():
    w = inputs.bits(inputs.student_t4_bf16(6000, seed=3))
    blob = O.compress(w, 3)
    assert P.decompress(blob.tobytes()) == [int(u) for u in O.truncate(w, 3)]


# ---------------------------------------------------------------- invariants of the whole path

@pytest.mark.parametrize("k", [7, 3, 1, 0])
def test_round_trip_of_every_bf16_pattern(k):
    blob = O.compress(ALL, k, threads=4)
    assert np.array_equal(O.decompress(blob, 65536, threads=3), O.truncate(ALL, k))
    perm = np.random.default_rng(k).permutation(ALL)
    assert np.array_equal(O.decompress(O.compress(perm, k), 65536), O.truncate(perm, k))


@pytest.mark.parametrize("n", [1, 2, 127, 128, 129, 4095, 4096 * 3 + 1, 100_003])
def test_lossless_round_trip_ragged_sizes(n):
    for gen in (inputs.gaussian_bf16, inputs.student_t4_bf16, inputs.random_bits_bf16):
        w = inputs.bits(gen(n, seed=n))
        for threads in (1, 5):
            assert np.array_equal(O.decompress(O.compress(w, 7, threads), n, threads), w)


def test_threads_do_not_change_the_bytes():
    w = inputs.bits(inputs.gaussian_bf16(300_000, seed=77))
    assert np.array_equal(O.compress(w, 7, threads=1), O.compress(w, 7, threads=8))


def test_size_against_entropy_bound_config1():
    # Config 1: 1024 x 1024, N(0, 0.02^2), lossless.
    w = inputs.bits(inputs.gaussian_bf16((1024, 1024), seed=inputs.seed_for(1)))
    n = w.size
    blob = O.compress(w, 7, threads=8)
    cnt = O.histogram(w)
    info = O.blob_info(blob)
    H, CE = O.entropy(cnt), O.cross_entropy(cnt, info["freq"])
    assert 0 <= CE - H < 0.01                                   # cost of the 12-bit table
    n_states = (n // 4096) * 16
    coded_bits = 16 * info["total_words"] + 32 * n_states
    # information content under the table, plus between 16 and 32 bits of flush per state
    assert n * CE + 16 * n_states - 0.002 * n <= coded_bits <= n * CE + 32 * n_states + 0.002 * n
    bits_per_weight = 8 * blob.size / n
    assert bits_per_weight <= 1.02 * (H + 8)                    # the stated target
    assert bits_per_weight - (H + 8) == pytest.approx(0.14, abs=0.03)


def test_lossy_size_and_bound():
    w = inputs.bits(inputs.student_t4_bf16(500_000, seed=inputs.seed_for(4)))
    H = O.entropy(O.histogram(w))
    assert H == pytest.approx(2.708, abs=0.02)
    for k in (3, 1, 0):
        blob = O.compress(w, k, threads=4)
        bpw = 8 * blob.size / w.size
        assert H + (k + 1) < bpw < H + (k + 1) + 0.2
        # same exponents, hence the same table and words, for every k
        sec, sec7 = O.sections(blob), O.sections(O.compress(w, 7, threads=4))
        b7 = O.compress(w, 7, threads=4)
        for name in ("freq", "offsets", "states", "lens", "words"):
            assert np.array_equal(blob[slice(*sec[name])], b7[slice(*sec7[name])])


def test_corruption_is_detected():
    w = inputs.bits(inputs.gaussian_bf16(50_000, seed=5))
    blob = O.compress(w, 7)
    sec = O.sections(blob)
    rng = np.random.default_rng(1)
    detected = 0
    for trial in range(40):
        bad = blob.copy()
        name = ("states", "words", "lens")[trial % 3]
        lo, hi = sec[name]
        pos = int(rng.integers(lo, hi - 16))
        bad[pos] ^= 1 << int(rng.integers(0, 8))
        try:
            out = O.decompress(bad, w.size)
            assert not np.array_equal(out, w) or name == "lens"
        except O.OracleError as err:
            assert err.code == O.ECORRUPT
            detected += 1
    assert detected >= 30                                       # final-state check catches nearly all
    with pytest.raises(O.OracleError):
        O.decompress(blob[:-16], w.size)
    with pytest.raises(O.OracleError):
        O.decompress(blob, w.size + 1)
    with pytest.raises(O.OracleError):
        O.compress(w, 5)


# ---------------------------------------------------------------- block-wise normalisation (Sec. 2.3)

def torch_bf16(words):
    import torch
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int16).copy()).view(torch.bfloat16)


def test_block_coefficient_is_the_mantissa_of_the_largest_weight():
    w = inputs.bits(inputs.student_t4_bf16(10_000 + 37, seed=21))
    v = np.abs(as_float(w))
    for block in (32, 64, 128, 256, 512):
        coef = O.block_coefficients(w, block)
        assert coef.size == math.ceil(w.size / block)
        for b in range(coef.size):
            seg = slice(b * block, min((b + 1) * block, w.size))
            first_max = int(np.argmax(v[seg]))                 # numpy returns the first maximum
            frac, _ = np.frexp(v[seg][first_max])
            assert coef[b] == int((frac * 2 - 1) * 128)        # 1.mantissa of that weight
    with pytest.raises(O.OracleError):
        O.block_coefficients(w, 48)


def test_normalisation_arithmetic_matches_torch_bf16():
    # every non-NaN bf16 pattern divided / multiplied by every coefficient class, against PyTorch's
    # IEEE float32 division / product and its round-to-nearest-even bf16 conversion
    import torch
    words = ALL[~np.isnan(as_float(ALL))]
    t = torch_bf16(words)
    for coef in (0, 1, 37, 64, 100, 127):
        c = 1.0 + coef / 128.0
        co = np.full(math.ceil(words.size / 32), coef, np.uint8)
        ours = O.normalise(words, 32, co)
        ref = (t.float() / c).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(ours, ref), coef
        ours = O.denormalise(words, 32, co)
        ref = (t.float() * c).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        keep = ~np.isnan(as_float(ref))
        assert np.array_equal(ours[keep], ref[keep]), coef


@pytest.mark.parametrize("k", [3, 1, 0])
def test_largest_weight_of_every_block_survives_lossy_compression(k):
    w = inputs.bits(inputs.student_t4_bf16(50_000, seed=22))
    v = as_float(w)
    plain_err = np.abs(as_float(O.truncate(w, k)) - v).mean()
    previous = None
    for block in (512, 128, 32):
        blob = O.compress(w, k, threads=3, block=block)
        out = O.decompress(blob, w.size, threads=2)
        assert np.array_equal(out, O.lossy_blockwise(w, k, block))
        for b in range(math.ceil(w.size / block)):
            seg = slice(b * block, min((b + 1) * block, w.size))
            i = int(np.argmax(np.abs(v[seg])))
            assert out[seg][i] == w[seg][i]                     # "invariant to rounding and truncation"
        # sign kept, relative change bounded by the truncation step plus the two bf16 roundings
        vo = as_float(out)
        assert np.array_equal(np.signbit(vo), np.signbit(v))
        assert (np.abs(vo - v) / np.abs(v)).max() < 2.0 ** -k + 2.0 ** -7
        # smaller blocks reproduce the weights better (block-size study) and cost 8 bits per block
        err = np.abs(vo - v).mean()
        assert err < plain_err and (previous is None or err < previous)
        previous = err
        sec = O.sections(blob)
        assert sec["coef"][1] - sec["coef"][0] == (math.ceil(w.size / block) + 15) // 16 * 16
        assert sec["coef"][1] == blob.size


@pytest.mark.parametrize("k,block,n", [(3, 512, 4096 + 77), (1, 32, 1000), (0, 128, 5000), (3, 64, 0), (0, 512, 1)])
def test_blockwise_containers_of_both_codecs_agree(k, block, n):
    w = inputs.bits(inputs.gaussian_bf16(n, seed=300 + n)) if n else np.zeros(0, np.uint16)
    blob = O.compress(w, k, block=block)
    mine = P.compress([int(u) for u in w], k, block)
    assert blob.tobytes() == mine
    assert P.decompress(mine) == [int(u) for u in O.lossy_blockwise(w, k, block)]
    assert np.array_equal(O.decompress(blob, n), O.lossy_blockwise(w, k, block))


def test_blockwise_rejects_lossless_and_odd_blocks():
    w = inputs.bits(inputs.gaussian_bf16(1000, seed=1))
    with pytest.raises(O.OracleError):
        O.compress(w, 7, block=512)
    with pytest.raises(O.OracleError):
        O.compress(w, 3, block=100)
    every = O.compress(ALL, 3, block=64)
    assert np.array_equal(O.decompress(every, 65536), O.lossy_blockwise(ALL, 3, 64))


# ---------------------------------------------------------------- tables kept across weight updates (Alg. 1 recompresses every step)

def test_guarded_quantise_closed_cases():
    # one exponent, guard 2: five codable symbols in the band plus exponent 0 (an update can cancel to
    # +-0); floors give 4096 + 5 ones, the excess of 5 comes off the only large entry
    c = np.zeros(256, np.uint64)
    c[120] = 77
    f = O.quantise(c, guard=2)
    assert {s: int(f[s]) for s in np.nonzero(f)[0]} == {0: 1, 118: 1, 119: 1, 120: 4091, 121: 1, 122: 1}
    # the band is clipped at both ends of the byte range
    c = np.zeros(256, np.uint64)
    c[0] = 5
    f = O.quantise(c, guard=3)
    assert list(f[:5]) == [4093, 1, 1, 1, 0] and f.sum() == 4096
    c = np.zeros(256, np.uint64)
    c[255] = 5
    f = O.quantise(c, guard=1)
    assert list(f[253:]) == [0, 1, 4094] and f[0] == 1 and f.sum() == 4096
    # two equal halves with a hole between them, guard 1: symbols 99..105 and 0 are codable, the six
    # empty ones get 1, and the excess of 6 is taken alternately from the two large entries,
    # the lower symbol first: three units each
    c = np.zeros(256, np.uint64)
    c[[100, 104]] = 1000
    f = O.quantise(c, guard=1)
    assert {s: int(f[s]) for s in np.nonzero(f)[0]} == {0: 1, 99: 1, 100: 2045, 101: 1, 102: 1, 103: 1, 104: 2045,
                                                        105: 1}
    # nothing to add when every exponent already occurs
    assert np.all(O.quantise(np.full(256, 9, np.uint64), guard=5) == 16)
    assert O.quantise(np.zeros(256, np.uint64), guard=4).sum() == 0


def test_guarded_quantise_properties_and_second_implementation():
    rng = np.random.default_rng(11)
    for trial in range(150):
        k = int(rng.integers(1, 40))
        lo = int(rng.integers(0, 256 - k))
        c = np.zeros(256, np.uint64)
        idx = lo + rng.choice(k, max(1, k // 2), replace=False)
        c[idx] = (rng.pareto(0.7, idx.size) * 10 + 1).astype(np.uint64)
        guard = int(rng.integers(0, 6))
        f = O.quantise(c, guard=guard)
        assert f.sum() == 4096
        present = np.nonzero(c)[0]
        want = np.zeros(256, bool)
        if guard:
            want[max(0, present[0] - guard): min(255, present[-1] + guard) + 1] = True
            want[0] = True
        else:
            want[present] = True
        assert np.array_equal(f > 0, want)
        assert list(f) == P.quantise([int(x) for x in c], guard)
        if guard == 0:
            assert np.array_equal(f, O.quantise(c))
        # the band costs at most its share of the probability mass
        assert O.cross_entropy(c, f) <= O.cross_entropy(c, O.quantise(c)) + math.log2(4096 / (4096 - 2 * guard - k - 1)) + 1e-9


@pytest.mark.parametrize("k", [7, 3, 0])
@pytest.mark.parametrize("n", [1, 130, 4097, 20_000])
def test_compression_with_an_earlier_table(n, k):
    old = inputs.bits(inputs.gaussian_bf16(n, seed=300 + n))
    new = inputs.bits(inputs.synthetic_update(inputs.gaussian_bf16(n, seed=300 + n), seed=7))
    guard = 8
    first = O.compress(old, k, guard=guard)
    table = O.blob_info(first)["freq"]
    assert np.array_equal(table, O.quantise(O.histogram(old), guard=guard))
    assert int(first[52:56].view("<u4")[0]) == guard
    assert np.all(table[O.split(new)[1]] > 0)                   # seeds chosen so that the update stays inside the band
    blob = O.compress(new, k, guard=guard, freq=table)
    # decoding needs nothing but the container: the values are the new ones
    assert np.array_equal(O.decompress(blob, n), O.truncate(new, k))
    assert np.array_equal(O.blob_info(blob)["freq"], table)
    # second statement of the format, given the same table
    assert blob.tobytes() == P.compress([int(u) for u in new], k, guard=guard, freq=[int(v) for v in table])
    assert P.decompress(blob.tobytes()) == [int(u) for u in O.truncate(new, k)]


def test_own_table_reproduces_plain_compression():
    w = inputs.bits(inputs.student_t4_bf16(30_000, seed=21))
    plain = O.compress(w, 7)
    again = O.compress(w, 7, freq=O.blob_info(plain)["freq"])
    assert np.array_equal(plain, again)
    guarded = O.compress(w, 7, guard=3)
    again = O.compress(w, 7, guard=3, freq=O.blob_info(guarded)["freq"])
    assert np.array_equal(guarded, again)
    assert not np.array_equal(O.blob_info(plain)["freq"], O.blob_info(guarded)["freq"])


def test_stale_table_is_refused_when_an_exponent_has_no_room():
    w = inputs.bits(inputs.gaussian_bf16(5000, seed=2))
    table = O.quantise(O.histogram(w), guard=1)
    top = int(np.nonzero(table)[0][-1])
    bad = w.copy()
    bad[1234] = np.uint16((top + 1) << 7)                      # one weight two binades above the band's end
    with pytest.raises(O.OracleError) as err:
        O.compress(bad, 7, guard=1, freq=table)
    assert err.value.code == O.ESTALE
    ok = w.copy()
    ok[1234] = np.uint16(top << 7)                             # the band's last exponent is still codable
    assert np.array_equal(O.decompress(O.compress(ok, 7, guard=1, freq=table), ok.size), ok)
    with pytest.raises(O.OracleError):                          # a table that does not sum to 4096
        O.compress(w, 7, freq=np.ones(256, np.uint16))


def test_size_under_a_stale_table_is_the_cross_entropy():
    # coded bits = information content of the NEW exponents under the OLD table + flush
    n = 64 * 4096
    base = inputs.gaussian_bf16(n, seed=9)
    old, new = inputs.bits(base), inputs.bits(inputs.synthetic_update(base, seed=10))
    table = O.quantise(O.histogram(old), guard=8)
    blob = O.compress(new, 7, guard=8, freq=table, threads=4)
    info = O.blob_info(blob)
    CE = O.cross_entropy(O.histogram(new), table)
    n_states = (n // 4096) * 16
    coded_bits = 16 * info["total_words"] + 32 * n_states
    assert n * CE + 16 * n_states - 0.002 * n <= coded_bits <= n * CE + 32 * n_states + 0.002 * n
    # a small update barely moves the exponent distribution: under 0.01 bit per weight lost
    fresh = O.compress(new, 7, threads=4)
    assert 0 <= 8 * (blob.size - fresh.size) / n < 0.01


# ---------------------------------------------------------------- linear layer on a compressed weight (Sec. 2.2, compressed forward pass)

def test_linear_oracle_one_hot_activations_pick_weight_columns():
    from oracle import linear as L
    out_f, in_f = 24, 256                                       # not square: a transposed operand cannot pass
    w = inputs.bits(inputs.gaussian_bf16(out_f * in_f, seed=41))
    blob = O.compress(w, 7)
    picks = [0, 1, 17, 255, 128]
    x = np.zeros((len(picks), in_f), np.uint16)
    for t, k in enumerate(picks):
        x[t, k] = 0x3F80                                        # bf16 1.0
    y = L.linear(blob, out_f, in_f, x)
    assert y.shape == (len(picks), out_f)
    wf = as_float(w).reshape(out_f, in_f)
    for t, k in enumerate(picks):
        assert np.array_equal(y[t], wf[:, k])
    # the bias is added once to every token
    b = np.arange(out_f, dtype=np.float64) * 0.5 - 3
    assert np.array_equal(L.linear(blob, out_f, in_f, x, bias=b), y + b)


@pytest.mark.parametrize("k", [7, 3, 0])
def test_linear_oracle_against_exact_rational_arithmetic(k):
    # bf16 values are dyadic rationals: Fractions give the exact sum, whatever the order
    from fractions import Fraction
    from oracle import linear as L
    out_f, in_f, tokens = 5, 128, 3
    w = inputs.bits(inputs.student_t4_bf16(out_f * in_f, seed=42))
    x = inputs.bits(inputs.gaussian_bf16(tokens * in_f, seed=43, std=1.0)).reshape(tokens, in_f)
    blob = O.compress(w, k)
    y = L.linear(blob, out_f, in_f, x)
    mag = L.magnitude(blob, out_f, in_f, x)
    w_hat = [Fraction(float(v)) for v in as_float(O.truncate(w, k))]   # the lossy variant multiplies the truncated weights
    xs = [[Fraction(float(v)) for v in as_float(row)] for row in x]
    for t in range(tokens):
        for o in range(out_f):
            exact = sum(w_hat[o * in_f + i] * xs[t][i] for i in range(in_f))
            assert abs(Fraction(float(y[t, o])) - exact) <= Fraction(float(mag[t, o])) * Fraction(in_f, 2 ** 52)
            assert float(mag[t, o]) >= abs(float(exact))


@pytest.mark.parametrize("k,block", [(3, 32), (1, 64), (0, 512)])
def test_linear_oracle_on_blockwise_normalised_weights_against_exact_rational_arithmetic(k, block):
    # the paper's default lossy form: the layer multiplies what the three steps of the normalisation give
    # back (normalise, truncate, de-normalise), here taken from their own definition, not from a container
    from fractions import Fraction
    from oracle import linear as L
    out_f, in_f, tokens = 6, 256, 2
    w = inputs.bits(inputs.student_t4_bf16(out_f * in_f, seed=46))
    x = inputs.bits(inputs.gaussian_bf16(tokens * in_f, seed=47, std=1.0)).reshape(tokens, in_f)
    blob = O.compress(w, k, block=block)
    y = L.linear(blob, out_f, in_f, x)
    mag = L.magnitude(blob, out_f, in_f, x)
    values = O.lossy_blockwise(w, k, block)
    assert not np.array_equal(values, O.truncate(w, k))                 # the normalisation does change the values
    w_hat = [Fraction(float(v)) for v in as_float(values)]
    xs = [[Fraction(float(v)) for v in as_float(row)] for row in x]
    for t in range(tokens):
        for o in range(out_f):
            exact = sum(w_hat[o * in_f + i] * xs[t][i] for i in range(in_f))
            assert abs(Fraction(float(y[t, o])) - exact) <= Fraction(float(mag[t, o])) * Fraction(in_f, 2 ** 52)


def test_linear_oracle_row_sums_and_linearity():
    from oracle import linear as L
    out_f, in_f = 16, 512
    w = inputs.bits(inputs.gaussian_bf16(out_f * in_f, seed=44))
    blob = O.compress(w, 7)
    ones = np.full((1, in_f), 0x3F80, np.uint16)
    y = L.linear(blob, out_f, in_f, ones)
    rows = as_float(w).reshape(out_f, in_f)
    for o in range(out_f):
        assert y[0, o] == pytest.approx(math.fsum(rows[o]), rel=1e-12, abs=1e-15)
    # tokens are independent of each other: stacking activations stacks outputs
    x = inputs.bits(inputs.gaussian_bf16(4 * in_f, seed=45, std=1.0)).reshape(4, in_f)
    whole = L.linear(blob, out_f, in_f, x)
    for t in range(4):
        assert np.array_equal(whole[t], L.linear(blob, out_f, in_f, x[t:t + 1])[0])
    # negating the activations (flip the bf16 sign bit) negates the output exactly
    assert np.array_equal(L.linear(blob, out_f, in_f, x ^ 0x8000), -whole)


# ---------------------------------------------------------------- binary32 tensors (beyond the paper, which uses BFloat16 only)

def test_f32_round_trip_and_layout():
    rng = np.random.default_rng(77)
    for n in (0, 1, 9, 4097, 30_000):
        w = (rng.standard_normal(n) * 0.02).astype(np.float32).view(np.uint32)
        blob = O.compress_f32(w, threads=3)
        assert np.array_equal(O.decompress_f32(blob, n, threads=2), w)
        # the upper halves are a bf16 tensor compressed as usual; the container differs from that
        # one only by the element-type word and the plane of lower halves, which is stored raw
        high, low = (w >> 16).astype(np.uint16), (w & 0xFFFF).astype(np.uint16)
        plain = O.compress(high, 7, threads=3)
        sec, sec16 = O.sections(blob), O.sections(plain)
        for name in ("freq", "offsets", "states", "lens", "words", "signmant"):
            assert np.array_equal(blob[slice(*sec[name])], plain[slice(*sec16[name])]), name
        lo, hi = sec["low"]
        assert np.array_equal(blob[lo: lo + 2 * n].view("<u2"), low)
        assert blob.size == plain.size + (hi - lo)
        # second statement of the format
        assert blob.tobytes() == P.compress([int(u) for u in high], 7, low=[int(u) for u in low])
        assert P.decompress(blob.tobytes()) == [int(u) for u in w]
        # the two element types do not decode each other's containers
        with pytest.raises(O.OracleError):
            O.decompress(blob, n)
        with pytest.raises(O.OracleError):
            O.decompress_f32(plain, n)


def test_f32_special_values_and_size():
    # every upper half combined with a few lower halves: zeros, subnormals, Inf, NaN payloads
    high = np.arange(65536, dtype=np.uint32)
    for low in (0, 1, 0x8000, 0xFFFF, 0x1234):
        w = (high << 16) | np.uint32(low)
        assert np.array_equal(O.decompress_f32(O.compress_f32(w), w.size), w)
    # Gaussian weights: 8 exponent bits shrink to their entropy, the other 24 bits stay
    w = (np.random.default_rng(3).standard_normal(1 << 20) * 0.02).astype(np.float32).view(np.uint32)
    blob = O.compress_f32(w, threads=8)
    H = O.entropy(O.histogram((w >> 16).astype(np.uint16)))
    assert H + 24 < 8 * blob.size / w.size < 1.01 * (H + 24)


def test_f32_guard_band_and_kept_table():
    rng = np.random.default_rng(78)
    n = 20_000
    w0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    w1 = (w0 - 1e-4 * rng.standard_normal(n).astype(np.float32)).view(np.uint32)
    w0 = w0.view(np.uint32)
    first = O.compress_f32(w0, guard=8)
    table = O.blob_info(first)["freq"]
    high0 = (w0 >> 16).astype(np.uint16)
    assert np.array_equal(table, O.quantise(O.histogram(high0), guard=8))
    kept = O.compress_f32(w1, threads=2, guard=8, freq=table)
    assert np.array_equal(O.decompress_f32(kept, n), w1)
    # the same bytes as the bf16 container of the upper halves under the same table, plus the plane
    high1, low1 = (w1 >> 16).astype(np.uint16), (w1 & 0xFFFF).astype(np.uint16)
    plain = O.compress(high1, 7, guard=8, freq=table)
    sec, sec16 = O.sections(kept), O.sections(plain)
    for name in ("freq", "offsets", "states", "lens", "words", "signmant"):
        assert np.array_equal(kept[slice(*sec[name])], plain[slice(*sec16[name])]), name
    assert kept.tobytes() == P.compress([int(u) for u in high1], 7, guard=8, freq=[int(f) for f in table],
                                        low=[int(u) for u in low1])
    # an exponent outside the table: refused, as for bf16
    w2 = w1.copy()
    w2[5] = np.uint32((int(np.nonzero(table)[0][-1]) + 1) << 23)
    with pytest.raises(O.OracleError) as err:
        O.compress_f32(w2, guard=8, freq=table)
    assert err.value.code == O.ESTALE


# ---------------------------------------------------------------- the weight update of the backward loop (Alg. 1)

def _round_nearest_even(value, bits):
    """The real `value` (a Fraction) rounded to `bits` significant binary digits, ties to even
    (normal range only): rounding written out on the rationals."""
    from fractions import Fraction
    if value == 0:
        return Fraction(0)
    sign = -1 if value < 0 else 1
    mag = abs(value)
    e = mag.numerator.bit_length() - mag.denominator.bit_length()
    if Fraction(2) ** e > mag:
        e -= 1
    assert Fraction(2) ** e <= mag < Fraction(2) ** (e + 1)
    scaled = mag / Fraction(2) ** (e - bits + 1)               # in [2^(bits-1), 2^bits)
    whole, rest = divmod(scaled, 1)
    if rest > Fraction(1, 2) or (rest == Fraction(1, 2) and whole % 2 == 1):
        whole += 1
    return sign * whole * Fraction(2) ** (e - bits + 1)


def test_update_closed_cases_from_golden_file():
    from oracle import update as U
    rows = [line.split() for line in open(os.path.join(os.path.dirname(__file__), "golden", "sgd_update.txt"))
            if line.strip() and not line.startswith("#")]
    assert len(rows) >= 10
    for w, g, lr, want in rows:
        got = U.sgd_update(np.array([int(w, 16)], np.uint16), np.array([int(g, 16)], np.uint16), float.fromhex(lr))
        assert int(got[0]) == int(want, 16), (w, g, lr, want, hex(int(got[0])))


def test_update_matches_exact_rational_arithmetic():
    from fractions import Fraction
    from oracle import update as U
    w = inputs.bits(inputs.gaussian_bf16(400, seed=102))
    g = inputs.bits(inputs.gaussian_bf16(400, seed=103, std=1.0))
    as_real = lambda u: Fraction(float((np.uint32(u) << 16).view(np.float32)))
    for lr in (1e-3, 0.37, 2.0 ** -6):
        lr32 = Fraction(float(np.float32(lr)))
        got = U.sgd_update(w, g, lr)
        for i in range(w.size):
            step = _round_nearest_even(lr32 * as_real(g[i]), 24)            # the product, rounded to binary32
            new = _round_nearest_even(as_real(w[i]) - step, 24)             # the difference, rounded to binary32
            want = _round_nearest_even(new, 8)                              # to bf16
            assert as_real(got[i]) == want, (i, lr)


def test_update_against_torch_and_invariants():
    import torch
    from oracle import update as U
    w = inputs.all_patterns_bf16()
    wb = inputs.bits(w)
    for seed, lr in ((1, 1e-2), (2, 3.0), (3, 1e-30)):
        g = inputs.random_bits_bf16(65536, seed=110 + seed)
        got = U.sgd_update(wb, inputs.bits(g), lr)
        ref32 = w.float() - torch.tensor(lr, dtype=torch.float32) * g.float()   # library float32 arithmetic
        ref = inputs.bits(ref32.to(torch.bfloat16))                             # library rounding to bf16
        nan = torch.isnan(ref32).numpy()
        assert np.array_equal(got[~nan], ref[~nan])
        assert np.all(got[nan] == 0x7FC0)
    # a zero gradient changes nothing (NaNs become the canonical one)
    zero = np.zeros(65536, np.uint16)
    same = U.sgd_update(wb, zero, 0.5)
    is_nan = (wb & 0x7FFF) > 0x7F80
    assert np.array_equal(same[~is_nan], wb[~is_nan]) and np.all(same[is_nan] == 0x7FC0)
    # flipping the sign of the gradient and of the rate together changes nothing
    g = inputs.bits(inputs.gaussian_bf16(65536, seed=120, std=1.0))
    assert np.array_equal(U.sgd_update(wb, g, 0.01), U.sgd_update(wb, g ^ 0x8000, -0.01))


def test_training_step_container_follows_the_kept_table_rules():
    from oracle import update as U
    n = 30_000
    w0 = inputs.bits(inputs.gaussian_bf16(n, seed=130))
    g = inputs.bits(inputs.gaussian_bf16(n, seed=131, std=1.0))
    first = O.compress(w0, 7, guard=8)
    new_container, rebuilt, new = U.training_step(first, g, 1e-4)
    assert rebuilt == 0
    assert np.array_equal(new, U.sgd_update(w0, g, 1e-4))
    assert np.array_equal(O.decompress(new_container, n), new)
    assert np.array_equal(O.blob_info(new_container)["freq"], O.blob_info(first)["freq"])   # the table was kept
    # a step large enough to leave the guard band: fresh statistics
    big, rebuilt, new = U.training_step(first, g, 1e6)
    assert rebuilt == 1
    assert np.array_equal(O.decompress(big, n), U.sgd_update(w0, g, 1e6))
    assert np.array_equal(big, O.compress(new, 7, guard=8))


# ---------------------------------------------------------------- binary16 tensors (beyond the paper)

def test_f16_round_trip_layout_and_size():
    rng = np.random.default_rng(91)
    for n in (0, 1, 9, 4097, 30_000):
        w = (rng.standard_normal(n) * 0.02).astype(np.float16).view(np.uint16)
        blob = O.compress_f16(w, threads=3)
        assert np.array_equal(O.decompress_f16(blob, n, threads=2), w)
        sec = O.sections(blob)
        # the raw plane is the words' lower bytes, the table is over their upper bytes
        lo, _ = sec["signmant"]
        assert np.array_equal(blob[lo: lo + n], (w & 0xFF).astype(np.uint8))
        if n:
            counts = np.bincount(w >> 8, minlength=256).astype(np.uint64)
            assert np.array_equal(O.blob_info(blob)["freq"], O.quantise(counts))
        # second statement of the format (upper byte / lower byte, written out directly)
        assert blob.tobytes() == P.compress([int(u) for u in w], 7, half=True)
        assert P.decompress(blob.tobytes()) == [int(u) for u in w]
        # element types do not decode each other's containers
        with pytest.raises(O.OracleError):
            O.decompress(blob, n)
        with pytest.raises(O.OracleError):
            O.decompress_f16(O.compress(w, 7), n)
    # every 16-bit pattern: zeros, subnormals, infinities, NaN payloads
    every = np.arange(65536, dtype=np.uint16)
    assert np.array_equal(O.decompress_f16(O.compress_f16(every), 65536), every)
    # Gaussian weights: the upper byte (sign, 5 exponent bits, 2 mantissa bits) shrinks to its entropy
    w = (np.random.default_rng(4).standard_normal(1 << 20) * 0.02).astype(np.float16).view(np.uint16)
    blob = O.compress_f16(w, threads=8)
    counts = np.bincount(w >> 8, minlength=256).astype(np.uint64)
    H = O.entropy(counts)
    assert 5.3 < H < 5.8                                     # 1 sign + ~2.55 exponent + ~2 mantissa bits
    assert H + 8 < 8 * blob.size / w.size < 1.02 * (H + 8)


def test_f16_guard_band_and_kept_table():
    rng = np.random.default_rng(92)
    n = 20_000
    w0 = (rng.standard_normal(n) * 0.02).astype(np.float16)
    w1 = (w0.astype(np.float32) - 1e-4 * rng.standard_normal(n).astype(np.float32)).astype(np.float16).view(np.uint16)
    w0 = w0.view(np.uint16)
    first = O.compress_f16(w0, guard=4)
    table = O.blob_info(first)["freq"]
    assert np.array_equal(table, O.quantise(np.bincount(w0 >> 8, minlength=256).astype(np.uint64), guard=4))
    kept = O.compress_f16(w1, threads=2, guard=4, freq=table)
    assert np.array_equal(O.decompress_f16(kept, n), w1)
    assert np.array_equal(O.blob_info(kept)["freq"], table)
    assert kept.tobytes() == P.compress([int(u) for u in w1], 7, guard=4, freq=[int(f) for f in table], half=True)
    w2 = w1.copy()
    # the band runs from the smallest occupied upper byte (small positive values) to the largest
    # (the most negative values) plus the guard; the largest-magnitude negative number lies beyond it
    w2[7] = np.uint16(0xFBFF)
    assert table[0xFB] == 0 and table[0x7B] == 1
    with pytest.raises(O.OracleError) as err:
        O.compress_f16(w2, guard=4, freq=table)
    assert err.value.code == O.ESTALE
