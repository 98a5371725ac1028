"""Host logic of the GEMM stage: which of its two kernels a problem takes, and the static schedule
of the one that keeps its weight tile in LDS (every round exactly once, evenly dealt, a block
seldom changing its channel tile).  No GPU needed."""
import collections

import pytest

from paper_2503_06545_amd import binding as qc

BLOCKS = 256


def all_rounds(M, N):
    return [qc.gemm_schedule(M, N, b) for b in range(BLOCKS)]


@pytest.mark.parametrize("M,N", [(131072, 3456), (131072, 4608), (131072, 1152), (65536, 4608), (16384, 3456),
                                 (80037, 3401), (700, 392), (1, 1), (4096, 128), (100000, 129), (9000, 7000),
                                 (513, 5000)])
def test_every_round_is_dealt_exactly_once(M, N):
    n_tiles, chunks = -(-N // 128), -(-(-(-M // 256) * 256) // 512)
    seen = collections.Counter(r for rounds in all_rounds(M, N) for r in rounds)
    assert set(seen) == {(nt, c) for nt in range(n_tiles) for c in range(chunks)}
    assert set(seen.values()) == {1}


def test_block_out_of_range_and_bad_sizes_are_rejected():
    assert qc.qc_debug_gemm_schedule(1024, 128, BLOCKS, None, 0) == -1
    assert qc.qc_debug_gemm_schedule(1024, 128, -1, None, 0) == -1
    assert qc.qc_debug_gemm_schedule(0, 128, 0, None, 0) == -1
    assert qc.qc_debug_gemm_schedule(1024, 128, 0, None, -1) == -1


@pytest.mark.parametrize("M,N", [(131072, 3456), (131072, 4608), (65536, 4608)])
def test_paper_shapes_are_dealt_evenly_and_keep_their_channel_tile(M, N):
    rounds = all_rounds(M, N)
    counts = [len(r) for r in rounds]
    assert max(counts) == min(counts) == (N // 128) * (M // 512) // BLOCKS
    # a block changes its weight tile a handful of times at most
    changes = [sum(1 for a, b in zip(r, r[1:]) if a[0] != b[0]) for r in rounds]
    assert max(changes) <= 6 and sorted(changes)[len(changes) // 2] <= 1
    # at any step the blocks of one XCD (block b runs on XCD b % 8) read few distinct chunks:
    # what the XCD's L2 holds
    for xcd in range(8):
        mine = [rounds[b] for b in range(xcd, BLOCKS, 8)]
        for step in range(0, counts[0], 5):
            assert len({r[step][1] for r in mine}) <= 8


def test_which_problems_take_the_resident_kernel():
    # hidden 1152 (short reduction): QKV, fc1 and the out-projection at full size; not a token
    # count that leaves a block fewer than 6 rounds
    assert qc.qc_debug_gemm_kernel(131072, 1152, 3456, 8) == 2
    assert qc.qc_debug_gemm_kernel(131072, 1152, 4608, 8) == 2
    assert qc.qc_debug_gemm_kernel(131072, 1152, 4608, 4) == 2
    assert qc.qc_debug_gemm_kernel(65536, 1152, 4608, 8) == 2
    assert qc.qc_debug_gemm_kernel(131072, 1152, 1152, 8) == 2
    assert qc.qc_debug_gemm_kernel(32768, 1152, 3456, 8) == 2
    assert qc.qc_debug_gemm_kernel(16384, 1152, 3456, 8) == 1
    assert qc.qc_debug_gemm_kernel(16384, 1152, 4608, 8) == 1
    # fc2: a 128 x 4608 weight tile does not fit in LDS with 8-bit codes, nor with 4-bit ones
    assert qc.qc_debug_gemm_kernel(131072, 4608, 1152, 8) == 1
    assert qc.qc_debug_gemm_kernel(131072, 4608, 1152, 4) == 1
    # 4-bit codes fit up to K = 2304
    assert qc.qc_debug_gemm_kernel(131072, 2304, 4608, 4) == 2
    assert qc.qc_debug_gemm_kernel(131072, 2304, 4608, 8) == 1
    assert qc.qc_debug_gemm_kernel(131072, 2305, 4608, 4) == 0      # odd K with 4 bits
    assert qc.qc_debug_gemm_kernel(0, 1152, 4608, 8) == 0
