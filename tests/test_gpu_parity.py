"""GPU parity: the HIP path against the CPU oracle, through the C ABI (-m gpu).

Integer/byte work throughout, so the bar is bit-exact: decoded bf16 words equal the oracle's
(0 ULP, lossy truncation included) and the exported container equals the oracle's byte for byte.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2410_20650_amd import inputs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
KS = [7, 3, 1, 0]


@pytest.fixture(scope="module")
def nz():
    from paper_2410_20650_amd import binding
    return binding


def roundtrip_and_compare(nz, w: torch.Tensor, k: int, threads: int = 16, block: int = 0):
    """Compress on the GPU, compare container and decoded words with the oracle's."""
    words = inputs.bits(w)
    n = words.size
    blob = nz.neuzip_compress_blockwise(w, k, block)
    assert blob.block_size == block and blob.mantissa_bits == k and blob.elems == n
    got = nz.neuzip_export(blob)
    want = O.compress(words, k, threads=threads, block=block)
    assert got.size == want.size == blob.compressed_bytes
    if not np.array_equal(got, want):
        sec = O.sections(want)
        bad = [name for name, (lo, hi) in sec.items() if not np.array_equal(got[lo:hi], want[lo:hi])]
        raise AssertionError(f"container differs from the oracle's in sections {bad} (n={n}, k={k})")
    out = torch.full_like(w, float("nan"))
    nz.neuzip_decompress(blob, out)
    nz.neuzip_check(blob)
    expect = O.lossy_blockwise(words, k, block) if block else O.truncate(words, k)
    assert np.array_equal(inputs.bits(out), expect), f"decoded words differ (n={n}, k={k}, block={block})"
    # the oracle reads the GPU's container, the GPU reads the oracle's
    assert np.array_equal(O.decompress(got, n, threads=threads), expect)
    theirs = nz.neuzip_import(want)
    out2 = torch.zeros_like(w)
    nz.neuzip_decompress(theirs, out2)
    nz.neuzip_check(theirs)
    assert np.array_equal(inputs.bits(out2), expect)
    return blob


def test_config1_gaussian_1024x1024(nz):
    w = inputs.gaussian_bf16((1024, 1024), inputs.seed_for(1), device=DEV)
    blob = roundtrip_and_compare(nz, w, 7)
    words = inputs.bits(w)
    cnt = O.histogram(words)
    assert np.array_equal(nz.neuzip_histogram(blob).astype(np.uint64), cnt)
    assert np.array_equal(nz.neuzip_frequencies(blob), O.quantise(cnt))
    bits_per_weight = 8 * blob.compressed_bytes / words.size
    assert bits_per_weight <= 1.02 * (O.entropy(cnt) + 8)
    assert blob.device_bytes < 1.01 * blob.compressed_bytes + 16384   # tables, alignment, 1/64 of headroom for the words


@pytest.mark.parametrize("k", KS)
@pytest.mark.parametrize("n", [1, 7, 8, 9, 127, 128, 129, 4095, 4096, 4097, 3 * 4096 + 1001,
                               32 * 4096, 33 * 4096 + 5, 1_000_003])
def test_ragged_sizes(nz, n, k):
    w = inputs.gaussian_bf16(n, 7000 + n, device=DEV)
    roundtrip_and_compare(nz, w, k)


def test_seeded_random_sizes_and_distributions(nz):
    # sizes anywhere between one element and a few hundred chunks, value distributions drawn per case
    rng = np.random.default_rng(7700)
    for case in range(24):
        n = int(rng.integers(1, 2 ** int(rng.integers(1, 21))))
        k = int(rng.choice(KS))
        kind = case % 3
        if kind == 0:
            w = inputs.gaussian_bf16(n, 7701 + case, std=float(10.0 ** rng.uniform(-4, 1)), device=DEV)
        elif kind == 1:
            w = inputs.student_t4_bf16(n, 7701 + case, device=DEV)
        else:
            w = inputs.random_bits_bf16(n, 7701 + case, device=DEV)
        block = int(rng.choice([0, 32, 128, 512])) if k != 7 else 0
        roundtrip_and_compare(nz, w, k, block=block)


@pytest.mark.parametrize("k", KS)
def test_every_bf16_pattern(nz, k):
    w = inputs.all_patterns_bf16(device=DEV)
    roundtrip_and_compare(nz, w, k)
    perm = torch.randperm(65536, generator=torch.Generator().manual_seed(k)).to(DEV)
    roundtrip_and_compare(nz, w[perm].contiguous(), k)


@pytest.mark.parametrize("k", KS)
def test_heavy_tailed(nz, k):
    w = inputs.student_t4_bf16(700_001, inputs.seed_for(4), device=DEV)
    roundtrip_and_compare(nz, w, k)


@pytest.mark.parametrize("n", [5, 4096, 40_000, 300_000])
def test_uniform_exponents_take_the_unstaged_path(nz, n):
    # 8 bits per symbol: the word runs of 32 chunks exceed the LDS window
    w = inputs.random_bits_bf16(n, 99 + n, device=DEV)
    roundtrip_and_compare(nz, w, 7)
    roundtrip_and_compare(nz, w, 0)


@pytest.mark.parametrize("n", [1, 100, 4096, 200_000 + 3])
def test_single_exponent_tensor(nz, n):
    w = inputs.constant_bf16(n, 0.75, device=DEV)
    blob = roundtrip_and_compare(nz, w, 7)
    assert nz.neuzip_frequencies(blob).max() == 4096
    # same exponent, varying sign and mantissa
    g = torch.Generator(device=DEV).manual_seed(n)
    v = (torch.rand(n, generator=g, device=DEV) + 1.0) * (torch.randint(0, 2, (n,), generator=g, device=DEV) * 2 - 1)
    roundtrip_and_compare(nz, v.to(torch.bfloat16), 3)


def test_rare_symbols_and_long_runs(nz):
    # one dominant exponent and 200 rare ones: frequencies of 1, 12-bit codes, runs near the 192-word cap
    n = 64 * 4096
    g = torch.Generator(device=DEV).manual_seed(5)
    expo = torch.full((n,), 120, dtype=torch.int32, device=DEV)
    rare = torch.randint(0, n, (600,), generator=g, device=DEV)
    expo[rare] = torch.randint(1, 201, (600,), generator=g, device=DEV, dtype=torch.int32)
    expo[4096 * 3: 4096 * 4] = torch.arange(4096, device=DEV, dtype=torch.int32) % 200 + 1   # a chunk of rare symbols only
    mant = torch.randint(0, 128, (n,), generator=g, device=DEV, dtype=torch.int32)
    sign = torch.randint(0, 2, (n,), generator=g, device=DEV, dtype=torch.int32)
    u = (sign << 15) | (expo << 7) | mant
    w = (u - 65536 * (u >= 32768)).to(torch.int16).view(torch.bfloat16)
    roundtrip_and_compare(nz, w, 7)
    roundtrip_and_compare(nz, w, 1)


@pytest.mark.parametrize("k", [3, 1, 0])
@pytest.mark.parametrize("block", [32, 64, 128, 256, 512])
def test_blockwise_normalisation(nz, k, block):
    # Sec. 2.3: lossy variant with one 8-bit coefficient per block
    for n in (1, 33, 4096, 4097 + block // 2, 300_007):
        w = inputs.student_t4_bf16(n, 9000 + n + block, device=DEV)
        roundtrip_and_compare(nz, w, k, block=block)


@pytest.mark.parametrize("k", [3, 0])
def test_blockwise_normalisation_on_every_pattern(nz, k):
    # subnormals, zeros, infinities and NaNs go through the same arithmetic as on the CPU
    w = inputs.all_patterns_bf16(device=DEV)
    roundtrip_and_compare(nz, w, k, block=64)
    perm = torch.randperm(65536, generator=torch.Generator().manual_seed(7 + k)).to(DEV)
    roundtrip_and_compare(nz, w[perm].contiguous(), k, block=512)


def test_blockwise_keeps_the_largest_weight_of_each_block(nz):
    n, block = 1 << 20, 512
    w = inputs.student_t4_bf16(n, 9100, device=DEV)
    blob = nz.neuzip_compress_blockwise(w, 0, block)
    out = torch.empty_like(w)
    nz.neuzip_decompress(blob, out)
    a = w.float().view(-1, block)
    idx = a.abs().argmax(dim=1, keepdim=True)
    assert torch.equal(torch.gather(out.float().view(-1, block), 1, idx), torch.gather(a, 1, idx))
    # 8 bits per block; the exponent stream changes a little because normalised weights are coded
    plain = nz.neuzip_compress(w, 0)
    sec = O.sections(nz.neuzip_export(blob))
    assert sec["coef"][1] - sec["coef"][0] == n // block
    assert abs(blob.compressed_bytes - plain.compressed_bytes - n // block) < 0.02 * plain.compressed_bytes
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress_blockwise(w, 7, block)
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress_blockwise(w, 3, 48)
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress(w, 0, blob=blob)                      # a normalised blob is not reused as a plain one


def test_empty_tensor(nz):
    w = torch.empty(0, dtype=torch.bfloat16, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    got = nz.neuzip_export(blob)
    assert np.array_equal(got, O.compress(np.zeros(0, np.uint16), 7))
    nz.neuzip_decompress(blob, w)
    assert nz.neuzip_import(got).elems == 0


def test_blob_reuse_and_recompression(nz):
    w = inputs.gaussian_bf16(500_000, 31, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    for step in range(3):
        w = inputs.synthetic_update(w, 40 + step)
        same = nz.neuzip_compress(w, 7, blob=blob)
        assert same is blob
        assert np.array_equal(nz.neuzip_export(blob), O.compress(inputs.bits(w), 7, threads=8))
        out = torch.empty_like(w)
        nz.neuzip_decompress(blob, out)
        assert torch.equal(out.view(torch.int16), w.view(torch.int16))
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress(w[:1000].contiguous(), 7, blob=blob)      # different size
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress(w, 3, blob=blob)                         # different precision


def test_forward_schedule_into_one_scratch(nz):
    # Alg. 1 forward loop at small scale: every layer goes through the same temporary buffer
    shapes = [(256, 512), (64, 512), (64, 512), (256, 512), (896, 256), (896, 256), (256, 896)]
    tensors = [inputs.gaussian_bf16(s, inputs.seed_for(3, i), device=DEV) for i, s in enumerate(shapes)]
    blobs = [nz.neuzip_compress(t, 7) for t in tensors]
    scratch = torch.zeros(max(t.numel() for t in tensors), dtype=torch.bfloat16, device=DEV)
    # one call runs the whole sequence; what is left in the scratch is the last layer
    at = nz.neuzip_decompress_sequence(blobs, scratch)
    last = tensors[-1]
    assert torch.equal(scratch[at[-1]: at[-1] + last.numel()].view(torch.int16), last.reshape(-1).view(torch.int16))
    # layer by layer with a consumer in between sees every layer intact
    for t, b in zip(tensors, blobs):
        assert nz.neuzip_decompress_sequence([b], scratch) == [0]
        assert torch.equal(scratch[: t.numel()].view(torch.int16), t.reshape(-1).view(torch.int16))
    # a space that holds them all: neighbours are placed one behind the other (256-byte boundaries)
    # and share launches of up to 8; with 10 tensors the last two start at the front again
    more = tensors + [inputs.gaussian_bf16(s, inputs.seed_for(3, 40 + i), device=DEV) for i, s in enumerate([(3, 7), (130, 100), (64, 512)])]
    more_blobs = blobs + [nz.neuzip_compress(t, 7) for t in more[len(tensors):]]
    roomy = torch.zeros(sum(t.numel() + 128 for t in more), dtype=torch.bfloat16, device=DEV)
    at = nz.neuzip_decompress_sequence(more_blobs, roomy)
    expect, run = [], 0
    for i, t in enumerate(more):
        if i == 8:
            run = 0
        expect.append(run)
        run = (run + t.numel() + 127) // 128 * 128
    assert at == expect
    for i in list(range(2, 8)) + [8, 9]:                  # what the second group did not overwrite, and that group
        t = more[i]
        assert torch.equal(roomy[at[i]: at[i] + t.numel()].view(torch.int16), t.reshape(-1).view(torch.int16)), i
    for b in more_blobs:
        nz.neuzip_check(b)
    small = torch.zeros(1000, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_decompress_sequence(blobs, small)


def test_batch_of_a_layer_in_one_launch(nz):
    # the weights a layer uses together, mixed sizes and precisions, ragged tails, an empty tensor
    shapes = [(256, 512), (64, 512), (64, 515), (256, 512), (896, 256), (896, 256), (256, 896), (3, 7), (0,),
              (1024, 1024), (33, 4096)]
    ks = [7, 7, 3, 7, 7, 0, 7, 1, 7, 7, 3]
    tensors = [inputs.gaussian_bf16(s, inputs.seed_for(3, 50 + i), device=DEV) for i, s in enumerate(shapes)]
    blobs = [nz.neuzip_compress(t, k) for t, k in zip(tensors, ks)]
    # one scratch buffer holds the whole layer: destinations are consecutive 256-byte aligned pieces
    sizes = [(t.numel() + 127) // 128 * 128 for t in tensors]
    scratch = torch.full((sum(sizes),), float("nan"), dtype=torch.bfloat16, device=DEV)
    dsts, at = [], 0
    for t, size in zip(tensors, sizes):
        dsts.append(scratch[at: at + t.numel()])
        at += size
    nz.neuzip_decompress_batch(blobs, dsts)
    for t, k, d, b in zip(tensors, ks, dsts, blobs):
        assert np.array_equal(inputs.bits(d), O.truncate(inputs.bits(t), k))
        nz.neuzip_check(b)
    # nothing outside the destinations was touched
    at = 0
    for t, size in zip(tensors, sizes):
        assert torch.isnan(scratch[at + t.numel(): at + size].float()).all()
        at += size
    with pytest.raises(ValueError):
        nz.neuzip_decompress_batch(blobs[:2], dsts[:1])
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_decompress_batch(blobs[:1], [scratch[1:1 + tensors[0].numel()]])   # misaligned


def test_decompression_can_be_captured_in_a_hip_graph(nz):
    # decompress allocates nothing and records no memset node, so a per-layer schedule can be
    # captured once and replayed; every replay is checked against the eager result, with eager
    # work and synchronisation in between
    shapes = [(300, 512), (64, 512), (1000, 1000)]
    tensors = [inputs.gaussian_bf16(s, inputs.seed_for(3, 80 + i), device=DEV) for i, s in enumerate(shapes)]
    blobs = [nz.neuzip_compress(t, 7) for t in tensors]
    outs = [torch.zeros(t.numel(), dtype=torch.bfloat16, device=DEV) for t in tensors]
    scratch = torch.zeros(max(t.numel() for t in tensors), dtype=torch.bfloat16, device=DEV)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        nz.neuzip_decompress_batch(blobs, outs, stream=side)          # warm up outside the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            nz.neuzip_decompress_batch(blobs, outs, stream=side)
            at = nz.neuzip_decompress_sequence(blobs, scratch, stream=side)
    for replay in range(4):
        for o in outs:
            o.fill_(float(replay))                                    # eager work between replays
        scratch.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, o in zip(tensors, outs):
            assert torch.equal(o.view(torch.int16), t.reshape(-1).view(torch.int16)), replay
        last = tensors[-1]
        assert torch.equal(scratch[at[-1]: at[-1] + last.numel()].view(torch.int16), last.reshape(-1).view(torch.int16))
    for b in blobs:
        nz.neuzip_check(b)


@pytest.mark.parametrize("k,block", [(7, 0), (3, 0), (0, 128)])
def test_compress_batch_matches_one_by_one(nz, k, block):
    # a layer's weights in one pass of the pipeline: same containers as tensor by tensor, which are
    # the oracle's; more tensors than one group holds, ragged and empty ones included
    shapes = [(256, 512), (64, 515), (1, 1), (0,), (896, 256), (33, 4096), (7, 9), (512, 512), (1000, 37),
              (300, 300), (2, 4096)]
    tensors = [inputs.student_t4_bf16(s, inputs.seed_for(5, 200 + i), device=DEV) for i, s in enumerate(shapes)]
    blobs = nz.neuzip_compress_batch(tensors, k, block)
    assert len(blobs) == len(tensors)
    for t, b in zip(tensors, blobs):
        words = inputs.bits(t)
        assert np.array_equal(nz.neuzip_export(b), O.compress(words, k, threads=4, block=block))
        out = torch.empty_like(t)
        nz.neuzip_decompress(b, out)
        nz.neuzip_check(b)
        expect = O.lossy_blockwise(words, k, block) if block else O.truncate(words, k)
        assert np.array_equal(inputs.bits(out), expect)
        if t.numel():
            assert np.array_equal(nz.neuzip_histogram(b).astype(np.uint64), O.histogram(expect if False else
                                  (O.normalise(words, block, O.block_coefficients(words, block)) if block else words)))
    # recompression into the same blobs after an update
    updated = [inputs.synthetic_update(t, 900 + i) for i, t in enumerate(tensors)]
    again = nz.neuzip_compress_batch(updated, k, block, blobs=blobs)
    assert all(a is b for a, b in zip(again, blobs))
    for t, b in zip(updated, blobs):
        assert np.array_equal(nz.neuzip_export(b), O.compress(inputs.bits(t), k, threads=4, block=block))
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress_batch(updated[:2], k, block, blobs=[blobs[0], blobs[0]])
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress_batch(updated[:2], k, block, blobs=[blobs[1], blobs[0]])   # sizes do not match


def test_other_stream(nz):
    s = torch.cuda.Stream()
    w = inputs.gaussian_bf16(300_000, 3, device=DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        blob = nz.neuzip_compress(w, 7, stream=s)
        out = torch.empty_like(w)
        nz.neuzip_decompress(blob, out, stream=s)
    s.synchronize()
    assert torch.equal(out.view(torch.int16), w.view(torch.int16))


def test_argument_errors(nz):
    w = inputs.gaussian_bf16(10_000, 1, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    with pytest.raises(nz.NeuzipError) as e:
        nz.neuzip_compress(w, 5)
    assert e.value.code == nz.EINVAL
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_decompress(blob, torch.empty(9_999, dtype=torch.bfloat16, device=DEV))
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_decompress(blob, torch.empty(10_008, dtype=torch.bfloat16, device=DEV)[1:10_001])  # misaligned
    with pytest.raises(TypeError):
        nz.neuzip_compress(w.to(torch.float64), 7)
    with pytest.raises(TypeError):
        nz.neuzip_compress_batch([w, w.float()], 7)                # one element type per call


def test_import_rejects_malformed_containers(nz):
    w = inputs.bits(inputs.gaussian_bf16(50_000, 5))
    good = O.compress(w, 7)
    sec = O.sections(good)
    for name, delta in (("header", 0), ("freq", 2), ("offsets", 4), ("lens", 3)):
        bad = good.copy()
        bad[sec[name][0] + delta] ^= 0x10
        with pytest.raises(nz.NeuzipError) as e:
            nz.neuzip_import(bad)
        assert e.value.code == nz.ECORRUPT
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_import(good[:-16])


def test_damaged_words_are_reported_by_check(nz):
    # the container is structurally valid, only coded bits are flipped: the decoder stays in bounds,
    # and a state that does not come back to its start raises the flag
    w = inputs.bits(inputs.gaussian_bf16(200_000, 6))
    good = O.compress(w, 7)
    lo, hi = O.sections(good)["words"]
    bad = good.copy()
    rng = np.random.default_rng(2)
    for pos in rng.integers(lo, hi - 16, 50):
        bad[pos] ^= 0x5A
    blob = nz.neuzip_import(bad)
    out = torch.empty(w.size, dtype=torch.bfloat16, device=DEV)
    nz.neuzip_decompress(blob, out)
    with pytest.raises(nz.NeuzipError) as e:
        nz.neuzip_check(blob)
    assert e.value.code == nz.ECORRUPT
    nz.neuzip_check(blob)  # flag is cleared by the report


def test_host_threads_on_their_own_streams(nz):
    # calls that touch different blobs may come from different host threads: four threads, each
    # with its own stream and tensors, compress (serialised inside the library: one workspace),
    # recompress and decompress at the same time; every result is checked against the oracle's
    import threading
    errors = []

    def worker(idx):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(6):
                    n = 50_000 + 4099 * idx + 17 * rep
                    w = inputs.gaussian_bf16(n, 7700 + 10 * idx + rep, device=DEV)
                    stream.synchronize()
                    blob = nz.neuzip_compress(w, 7 if rep % 2 == 0 else 3, stream)
                    out = torch.empty_like(w)
                    nz.neuzip_decompress(blob, out, stream)
                    nz.neuzip_check(blob, stream)
                    k = blob.mantissa_bits
                    if not np.array_equal(inputs.bits(out), O.truncate(inputs.bits(w), k)):
                        errors.append((idx, rep, "values"))
                    if not np.array_equal(nz.neuzip_export(blob, stream), O.compress(inputs.bits(w), k)):
                        errors.append((idx, rep, "container"))
                    nz.neuzip_free(blob)
        except Exception as exc:                                # surfaced in the main thread
            errors.append((idx, repr(exc)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads)
    assert errors == []


def test_stream_probe_moves_the_bytes_and_rejects_what_is_no_decoders_mix(nz):
    # the measuring aid: writes its pattern over whole 8 KB chunks of the output, reads the input, no more
    out = torch.zeros(64 * 8192 // 2 + 8, dtype=torch.bfloat16, device=DEV)          # 64 chunks + the sink word
    guard = torch.full((4096,), 7, dtype=torch.uint8, device=DEV)
    inp = torch.full((64 * 5504,), 3, dtype=torch.uint8, device=DEV)                  # a lossless container's share
    nz.neuzip_stream_probe(inp, out)
    torch.cuda.synchronize()
    words = out.view(torch.int32)
    assert int(words[0].item()) == 0x03030303                                       # the field bytes it read
    turn = words[: 64 * 2048].reshape(-1, 4)[:, 3]                                   # the turn number, in every 16-byte piece
    assert int(turn.sum().item()) == 64 * 16 * sum(range(32)) and int(turn.max().item()) == 31
    assert bool((guard == 7).all()) and bool((inp == 3).all())
    tiny = torch.zeros(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_stream_probe(tiny, out)                                           # less than a byte per 8 outputs
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_stream_probe(inp, tiny)                                           # no whole chunk of output
