"""The checker's Bloom filter against what its definition and the mathematics fix.

The format (section 2.2 of the paper names Bloom filters; the layout is the library's, stated in
include/lsm_index.h) is re-derived here with Python integers from that statement, independently of
the C code: block and bit positions of given keys, the filter bytes of a tiny run, no false
negatives, and a false-positive rate near the one the block size and the bits per key predict.
"""
import math

import numpy as np

import brute

M64 = (1 << 64) - 1


def _mix(x):
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & M64
    x ^= x >> 31
    return x


def _place(key: bytes, n_blocks: int):
    h = 0x5EED251116138
    for i in range(4):
        h = _mix(h ^ int.from_bytes(key[8 * i:8 * i + 8], "big"))
    g = _mix(h ^ 0x9E3779B97F4A7C15)
    return ((h >> 32) * n_blocks) >> 32, [(g >> (7 * j)) & 127 for j in range(6)]


def test_splitmix_output_function_reference_values():
    # first outputs of splitmix64 seeded with 0 (published test vector of the generator): out_n = mix(n * golden)
    gold = 0x9E3779B97F4A7C15
    assert _mix(gold) == 0xE220A8397B1DCDAF
    assert _mix((2 * gold) & M64) == 0x6E789E6AA1B965F4
    assert _mix((3 * gold) & M64) == 0x06C45D188009454F


def test_block_count(oracle):
    assert oracle.bloom_blocks(0, 16) == 1
    assert oracle.bloom_blocks(8, 16) == 1 and oracle.bloom_blocks(9, 16) == 2
    assert oracle.bloom_blocks(1000, 10) == math.ceil(10000 / 128)
    assert oracle.bloom_blocks(10, 0) == 0
    assert oracle.bloom_blocks(1 << 40, 16) == 0  # 2^37 blocks: too many


def test_filter_bytes_of_a_small_run_follow_the_definition(oracle):
    rs = np.random.RandomState(5)
    keys = sorted({bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(40)})
    run = brute.run_from_raw([brute.pack_entry(k, i, brute.PUT) for i, k in enumerate(keys)])
    for n_blocks in (1, 3, 7, 64):
        want = np.zeros((n_blocks, 16), dtype=np.uint8)
        for k in keys:
            block, bits = _place(k, n_blocks)
            for b in bits:
                want[block, b // 8] |= 1 << (b % 8)
        got = oracle.build_bloom(run, n_blocks)
        assert np.array_equal(got, want)


def test_no_false_negatives_and_plausible_false_positive_rate(oracle):
    rs = np.random.RandomState(6)
    keys = sorted({bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(20000)})
    run = brute.run_from_raw([brute.pack_entry(k, i, brute.TOMBSTONE if i % 5 == 0 else brute.PUT) for i, k in enumerate(keys)])
    n_blocks = oracle.bloom_blocks(len(keys), 16)
    filt = oracle.build_bloom(run, n_blocks)
    assert all(oracle.bloom_may_contain(filt, k) for k in keys)  # tombstones included: they must shadow
    absent = [bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(20000)]
    fp = sum(oracle.bloom_may_contain(filt, k) for k in absent) / len(absent)
    # blocked filter, 128-bit blocks, 8 keys per block on average, 6 bits per key: Poisson-weighted (1 - e^{-6j/128})^6
    expect = sum(math.exp(-8) * 8 ** j / math.factorial(j) * (1 - math.exp(-6 * j / 128)) ** 6 for j in range(60))
    assert 0.5 * expect < fp < 1.6 * expect and fp < 0.02
    # membership answers agree with the bit-level definition
    for k in absent[:200] + keys[:200]:
        block, bits = _place(k, n_blocks)
        assert oracle.bloom_may_contain(filt, k) == all(filt[block, b // 8] >> (b % 8) & 1 for b in bits)


def test_a_dropped_or_shifted_bit_is_noticed(oracle):
    """Plant mistakes in a copy of the definition and see that the byte comparison above would catch them."""
    rs = np.random.RandomState(7)
    keys = sorted({bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(64)})
    run = brute.run_from_raw([brute.pack_entry(k, i, brute.PUT) for i, k in enumerate(keys)])
    got = oracle.build_bloom(run, 5)
    for shift, nbits in ((6, 6), (7, 5)):  # wrong stride between bit fields; one bit missing
        wrong = np.zeros((5, 16), dtype=np.uint8)
        for k in keys:
            h = 0x5EED251116138
            for i in range(4):
                h = _mix(h ^ int.from_bytes(k[8 * i:8 * i + 8], "big"))
            g = _mix(h ^ 0x9E3779B97F4A7C15)
            for j in range(nbits):
                b = (g >> (shift * j)) & 127
                wrong[((h >> 32) * 5) >> 32, b // 8] |= 1 << (b % 8)
        assert not np.array_equal(got, wrong)
