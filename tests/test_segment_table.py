"""Host segment-table builder of the library vs the oracle's brute-force enumeration: integer
work, compared bit for bit.  Needs no GPU."""
import numpy as np
import pytest

import oracle
from paper_2502_11034_amd import binding as B
from paper_2502_11034_amd import workloads as W


def compare(numels, chunk):
    begin, tensor, index = B.adagc_build_segment_table(numels, chunk)
    ref_chunks, ref_begin = oracle.enumerate_chunks(numels, chunk)
    assert begin.tolist() == ref_begin
    assert len(tensor) == len(ref_chunks)
    ref_tensor = np.array([c[0] for c in ref_chunks], dtype=np.int64)
    ref_first = np.array([c[1] for c in ref_chunks], dtype=np.int64)
    ref_len = np.array([c[2] for c in ref_chunks], dtype=np.int64)
    first = index.astype(np.int64) * chunk
    length = np.minimum(chunk, np.asarray(numels, dtype=np.int64)[tensor.astype(np.int64)] - first)
    assert np.array_equal(tensor.astype(np.int64), ref_tensor)
    assert np.array_equal(first, ref_first)
    assert np.array_equal(length, ref_len)
    assert int(length.sum()) == int(sum(numels))


def test_chunk_constant():
    assert B.adagc_chunk_elems() == 16384


@pytest.mark.parametrize("chunk", [1, 7, 16, 16384])
def test_small_ragged_lists(chunk):
    rng = np.random.default_rng(0)
    numels = [int(x) for x in rng.integers(1, 100, 50)] + [1, chunk, chunk + 1, 2 * chunk, 2 * chunk - 1]
    compare(numels, chunk)


@pytest.mark.parametrize("make", [W.tiny_transformer_list, W.gpt2_small_list, W.llama3_8b_list])
def test_model_lists(make):
    numels = [s.numel for s in make()]
    compare(numels, B.adagc_chunk_elems())


def test_llama3_8b_counts():
    numels = [s.numel for s in W.llama3_8b_list()]
    assert len(numels) == 291 and sum(numels) == 8030261248
    begin, tensor, index = B.adagc_build_segment_table(numels)
    assert begin[-1] == sum(-(-n // 16384) for n in numels)


def test_ragged_stress_list():
    numels = [s.numel for s in W.ragged_stress_list()]
    assert len(numels) == 20001
    compare(numels, B.adagc_chunk_elems())


def test_permutation_permutes_rows():
    rng = np.random.default_rng(1)
    numels = [int(x) for x in rng.integers(1, 70000, 30)]
    perm = rng.permutation(len(numels))
    b0, t0, i0 = B.adagc_build_segment_table(numels)
    b1, t1, i1 = B.adagc_build_segment_table([numels[p] for p in perm])
    for k, p in enumerate(perm):
        assert np.array_equal(i1[b1[k]:b1[k + 1]], i0[b0[p]:b0[p + 1]])
        assert (t1[b1[k]:b1[k + 1]] == k).all()


def test_builder_rejects_bad_input():
    with pytest.raises(B.AdagcError) as e:
        B.adagc_build_segment_table([4, 0, 3])
    assert e.value.code == B.ADAGC_ERR_INVALID_ARG
    with pytest.raises(B.AdagcError):
        B.adagc_build_segment_table([4, -1])
    with pytest.raises(B.AdagcError):
        B.adagc_build_segment_table([4], 0)
    with pytest.raises(B.AdagcError):
        B.adagc_build_segment_table([])
    # more than 2^32-1 chunks
    with pytest.raises(B.AdagcError) as e:
        B.adagc_build_segment_table([2 ** 40], 1)
    assert e.value.code == B.ADAGC_ERR_TOO_LARGE


# --------------------------------------------------------------------------- visiting order (host only)

@pytest.mark.parametrize("parts", [1, 2, 3, 4, 5, 8, 16, 1021])
@pytest.mark.parametrize("run", [1, 2, 7, 8, 64])
def test_visiting_order_is_a_permutation(parts, run):
    for n in (1, 2, 7, 8, 9, 50, 63, 64, 65, 1000, 7686, 100003):
        order = B.adagc_build_visiting_order(n, parts, run)
        assert np.array_equal(np.sort(order), np.arange(n, dtype=np.uint32)), (n, parts, run)


def test_visiting_order_shapes():
    assert list(B.adagc_build_visiting_order(10, 1, 1)) == list(range(10))
    # 2 parts of 32 chunks, runs of 8: XCD 0 (positions 0, 8, 16, ...) walks chunks 0..7 of the first half,
    # XCD 1 walks chunks 0..7 of the second half, XCD 2 walks chunks 8..15 of the first half, ...
    order = B.adagc_build_visiting_order(64, 2, 8)
    assert list(order[0::8][:8]) == list(range(0, 8))
    assert list(order[1::8][:8]) == list(range(32, 40))
    assert list(order[2::8][:8]) == list(range(8, 16))
    assert list(order[7::8][:8]) == list(range(56, 64))
    # 8 parts: one XCD per part, the run length does not matter
    assert np.array_equal(B.adagc_build_visiting_order(4096, 8, 8), B.adagc_build_visiting_order(4096, 8, 1))
    assert list(B.adagc_build_visiting_order(4096, 8, 1)[:9]) == [0, 512, 1024, 1536, 2048, 2560, 3072, 3584, 1]
    # parts that do not divide 8: position k -> part k mod parts
    assert list(B.adagc_build_visiting_order(9, 3, 5)) == [0, 3, 6, 1, 4, 7, 2, 5, 8]
    # more parts than chunks: list order
    assert list(B.adagc_build_visiting_order(5, 8, 8)) == [0, 1, 2, 3, 4]


def test_visiting_order_rejects_bad_arguments():
    for args in ((0, 2, 8), (-1, 2, 8), (10, 0, 8), (10, 2, 0), (10, -2, 8)):
        with pytest.raises(B.AdagcError) as e:
            B.adagc_build_visiting_order(*args)
        assert e.value.code == B.ADAGC_ERR_INVALID_ARG
