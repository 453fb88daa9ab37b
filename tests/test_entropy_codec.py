"""The library's host-side entropy codec (Sec. 3.1, entropy-coding paragraph) against the oracle: bucket
probabilities, optimal code lengths and their mean, the bit stream itself, round trips, random access to a
vector, and the paper's figure of about 5 % at b = 4 on quantised data.  No GPU involved."""
import ctypes as C

import numpy as np
import pytest

import workloads as W
from oracle import turboquant_oracle as o


@pytest.fixture(scope="module")
def ent():
    import os
    from paper_2504_19874_amd import _lib
    if not os.path.exists(_lib.LIB_PATH):
        from paper_2504_19874_amd import build
        build.build_library(verbose=False)
    from paper_2504_19874_amd import entropy
    return entropy


@pytest.mark.parametrize("d,bits", [(128, 1), (128, 2), (128, 4), (1536, 3), (1536, 4), (3072, 4), (64, 5)])
def test_masses_and_code_match_the_oracle(ent, d, bits):
    c32, _, _ = o.codebook_fp32(d, bits)
    p_or = o.bucket_masses(c32.astype(np.float64), d)  # both sides from the stored (fp32) table
    p = ent.bucket_masses(d, bits, c32)
    assert abs(p.sum() - 1) < 1e-12 and np.max(np.abs(p - p_or)) < 1e-12
    code = ent.PrefixCode(p)
    L_or = o.huffman_lengths(p)
    # an optimal code's mean length is unique even where equal probabilities leave the lengths a choice
    assert abs(code.mean_bits - float((p * L_or).sum())) < 1e-12
    assert sum(2.0 ** -int(l) for l in code.lengths) == 1.0
    assert np.array_equal(code.codewords, o.canonical_codewords(code.lengths))
    assert np.array_equal(code.lengths, L_or)  # the same tie rule on both sides


@pytest.mark.parametrize("d,bits,n", [(128, 4, 50), (96, 3, 7), (64, 1, 3), (160, 2, 33)])
def test_stream_equals_the_oracle_bit_for_bit_and_round_trips(ent, d, bits, n):
    rng = np.random.default_rng(d + bits)
    c64, _, _ = o.lloyd_max_codebook(max(d, 3), bits)
    p = o.bucket_masses(c64, d)
    code = ent.PrefixCode(p)
    idx = rng.choice(1 << bits, size=(n, d), p=p).astype(np.int32)
    words = o.pack_planes(idx, bits)
    stream, offs = code.encode(words, d)
    bits_or, starts_or = o.prefix_encode(idx, code.lengths, code.codewords)
    assert list(offs) == starts_or
    got_bits = np.unpackbits(stream)[: len(bits_or)]
    assert np.array_equal(got_bits, np.array(bits_or, dtype=np.uint8))
    assert stream.size == (len(bits_or) + 7) // 8 and not np.unpackbits(stream)[len(bits_or):].any()
    assert np.array_equal(code.decode(stream, d, n), words)
    assert np.array_equal(o.prefix_decode(list(got_bits), code.lengths, code.codewords, n, d), idx)
    # any one vector from its bit offset
    k = n // 2
    assert np.array_equal(code.decode(stream, d, 1, int(offs[k])), words[k:k + 1])


def test_saving_on_quantised_vectors_is_what_the_paper_states(ent, paper):
    """Codes of random unit vectors from the oracle's quantiser at b = 4: the stream is about 5 % shorter than 4
    bits per coordinate, and close to the code's expected length."""
    d, bits, n = 128, 4, 4000
    Pi = o.rotation_from_gaussian(W.gaussian_matrix(d, 100))
    c32, t32, _ = o.codebook_fp32(d, bits)
    idx, _, _ = o.quant_mse(W.unit_gaussian_rows(n, d, 5), Pi, t32, normalise=False)
    code = ent.PrefixCode(ent.bucket_masses(d, bits, c32))
    stream, offs = code.encode(o.pack_planes(idx, bits), d)
    per_coord = int(offs[-1]) / (n * d)
    assert abs(per_coord - code.mean_bits) < 0.01
    assert abs((1 - per_coord / bits) - paper["prefix_saving_b4"]) < 0.01
    assert np.array_equal(o.unpack_planes(code.decode(stream, d, n), bits, d), idx)


def test_codec_rejects_bad_streams_and_arguments(ent):
    from paper_2504_19874_amd import _lib
    lib = _lib.load()
    p = np.array([0.5, 0.25, 0.125, 0.125])
    code = ent.PrefixCode(p)
    assert list(code.lengths) == [1, 2, 3, 3] and list(code.codewords) == [0, 2, 6, 7]
    idx = np.array([[3] * 32], dtype=np.int32)
    stream, offs = code.encode(o.pack_planes(idx, 2), 32)
    assert int(offs[1]) == 96
    out = np.zeros((1, 2), dtype=np.uint32)
    vp = lambda a: a.ctypes.data_as(C.c_void_p)
    # a stream cut short
    assert lib.tq_entropy_decode(32, 2, vp(code.lengths), vp(stream), stream.size - 1, 0, 1, vp(out)) == 1
    # lengths that are no prefix code (Kraft sum above 1)
    bad = np.array([1, 1, 1, 1], dtype=np.uint8)
    assert lib.tq_entropy_decode(32, 2, vp(bad), vp(stream), stream.size, 0, 1, vp(out)) == 1
    # too little room for the stream
    small = np.zeros(4, dtype=np.uint8)
    used = C.c_size_t(0)
    w = o.pack_planes(idx, 2)
    assert lib.tq_entropy_encode(32, 2, vp(code.lengths), vp(code.codewords), vp(w), 1, vp(small), small.size,
                                 C.byref(used), None) == 4
    assert lib.tq_prefix_code_build(0, vp(p), vp(bad), vp(out), None) == 1
    assert lib.tq_bucket_masses(2, 2, vp(np.zeros(4, dtype=np.float32)), vp(p)) == 1
    # a distribution whose rarest symbols would need more than 32 bits
    tiny = np.array([2.0 ** -k for k in range(1, 41)] + [2.0 ** -40] + [0.0] * 23)
    L = np.zeros(64, dtype=np.uint8)
    cw = np.zeros(64, dtype=np.uint32)
    assert lib.tq_prefix_code_build(64, vp(tiny), vp(L), vp(cw), None) == 2
