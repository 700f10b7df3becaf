"""Pins for the CPU oracle (the MPI_Alltoallv definition in oracle/alltoallv_oracle.c).

The oracle is checked against things other than itself: an element-wise decode of a payload
that names its own origin, numpy's transpose for the uniform case, byte conservation, canary
bytes, and the error behaviour MPI's statement of the problem implies.  The last tests plant
plausible mistakes in a copy of the definition and show that the pins reject them.
"""
import numpy as np
import pytest

import oracle
import workloads as wl


def _random_counts(P, seed, max_elems=9, zero_frac=0.3):
    rng = np.random.default_rng(seed)
    c = rng.integers(0, max_elems + 1, size=(P, P))
    c[rng.random((P, P)) < zero_frac] = 0
    return (4 * c).astype(np.int32)


def decode_check(recv, lay, canary=0xA5):
    """Independent statement of the result for the traceable payload: element k of the region
    rank j receives from rank i must read (i<<20)|(j<<10)|k, and nothing else may change."""
    touched = np.zeros(recv.size, dtype=bool)
    for j in range(lay.P):
        for i in range(lay.P):
            n = int(lay.sendcounts[i, j])
            o = int(lay.rdispls[j, i])
            got = recv[o:o + n].view("<i4")
            k = np.arange(n // 4)
            want = (i << 20) | (j << 10) | k
            if not np.array_equal(got, want):
                return False
            if touched[o:o + n].any():
                return False
            touched[o:o + n] = True
    return bool((recv[~touched] == canary).all())


@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 7, 8, 9])
@pytest.mark.parametrize("variant", ["dense", "gaps", "permuted"])
def test_traceable_payload_decodes(P, variant):
    counts = _random_counts(P, 100 + P)
    kw = {"dense": {}, "gaps": {"gap": 12}, "permuted": {"gap": 8, "permute_seed": 7}}[variant]
    lay = wl.make_layout(counts, **kw)
    send = wl.payload_traceable_int32(lay)
    recv = np.full(lay.recv_bytes, 0xA5, dtype=np.uint8)
    assert oracle.alltoallv(send, lay.sendcounts, lay.sdispls, recv, lay.recvcounts, lay.rdispls) == 0
    assert decode_check(recv, lay)


def test_config1_shape_decodes():
    lay = wl.make_layout(wl.make_counts(1))
    assert lay.P == 16 and lay.sendcounts.max() <= 256 and (lay.sendcounts % 4 == 0).all()
    send = wl.payload_traceable_int32(lay)
    recv = np.full(lay.recv_bytes, 0xA5, dtype=np.uint8)
    assert oracle.alltoallv(send, lay.sendcounts, lay.sdispls, recv, lay.recvcounts, lay.rdispls) == 0
    assert decode_check(recv, lay)


@pytest.mark.parametrize("P,S", [(1, 8), (4, 1), (6, 24), (16, 256)])
def test_uniform_case_is_a_block_transpose(P, S):
    """All blocks S bytes: the textbook all-to-all, i.e. a transpose of S-byte cells."""
    lay = wl.make_layout(wl.counts_constant(P, S))
    send = wl.payload_position_hash(5, lay.send_bytes)
    recv = np.zeros(lay.recv_bytes, dtype=np.uint8)
    assert oracle.alltoallv(send, lay.sendcounts, lay.sdispls, recv, lay.recvcounts, lay.rdispls) == 0
    want = send[:P * P * S].reshape(P, P, S).transpose(1, 0, 2)
    assert np.array_equal(recv[:P * P * S].reshape(P, P, S), want)


@pytest.mark.parametrize("cfg,P", [(2, 24), (3, 16), (4, 12)])
def test_conservation_and_blockwise_equality(cfg, P):
    """Total bytes are conserved and each received region equals the sent block, byte sizes with
    arbitrary alignment included (configuration-2 style counts)."""
    counts = wl.make_counts(cfg, P)
    lay = wl.make_layout(counts, gap=3, permute_seed=11)
    send = wl.payload_position_hash(99, lay.send_bytes)
    recv = np.full(lay.recv_bytes, 0x5A, dtype=np.uint8)
    assert oracle.alltoallv(send, lay.sendcounts, lay.sdispls, recv, lay.recvcounts, lay.rdispls) == 0
    written = np.zeros(lay.recv_bytes, dtype=bool)
    for i in range(P):
        for j in range(P):
            n = int(counts[i, j])
            s = send[lay.sdispls[i, j]:lay.sdispls[i, j] + n]
            r = recv[lay.rdispls[j, i]:lay.rdispls[j, i] + n]
            assert np.array_equal(s, r)
            written[lay.rdispls[j, i]:lay.rdispls[j, i] + n] = True
    assert int(written.sum()) == lay.payload_bytes == int(lay.recvcounts.astype(np.int64).sum())
    assert (recv[~written] == 0x5A).all()
    # the multiset of payload bytes is unchanged
    sent = np.concatenate([send[lay.sdispls[i, j]:lay.sdispls[i, j] + counts[i, j]]
                           for i in range(P) for j in range(P)])
    assert np.array_equal(np.bincount(sent, minlength=256), np.bincount(recv[written], minlength=256))


def test_send_buffer_and_metadata_are_read_only():
    lay = wl.make_layout(_random_counts(6, 3))
    send = wl.payload_traceable_int32(lay)
    keep = (send.copy(), lay.sendcounts.copy(), lay.sdispls.copy(), lay.recvcounts.copy(), lay.rdispls.copy())
    recv = np.zeros(lay.recv_bytes, dtype=np.uint8)
    oracle.alltoallv(send, lay.sendcounts, lay.sdispls, recv, lay.recvcounts, lay.rdispls)
    for a, b in zip(keep, (send, lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)):
        assert np.array_equal(a, b)


def test_error_codes_and_nothing_written():
    lay = wl.make_layout(_random_counts(5, 8, zero_frac=0.0))
    send = wl.payload_traceable_int32(lay)
    recv = np.full(lay.recv_bytes, 0xA5, dtype=np.uint8)
    bad = lay.recvcounts.copy()
    bad[2, 3] += 4
    bad[3, 2] -= 4
    assert oracle.check_counts(lay.sendcounts, bad) == oracle.ERR_COUNT_MISMATCH
    lib = oracle._load()
    rc = lib.oracle_alltoallv(oracle._p(send), oracle._p(lay.sendcounts), oracle._p(lay.sdispls),
                              oracle._p(recv), oracle._p(bad), oracle._p(lay.rdispls), lay.P)
    assert rc == oracle.ERR_COUNT_MISMATCH and (recv == 0xA5).all()
    neg = lay.sendcounts.copy()
    neg[1, 1] = -4
    assert oracle.check_counts(neg, np.ascontiguousarray(neg.T)) == oracle.ERR_NEGATIVE_COUNT


def test_receiver_subset_matches_full_and_leaves_other_ranks_alone():
    counts = wl.make_counts(2, 12)
    lay = wl.make_layout(counts)
    send = wl.payload_position_hash(3, lay.send_bytes)
    full = np.zeros(lay.recv_bytes, dtype=np.uint8)
    oracle.alltoallv(send, lay.sendcounts, lay.sdispls, full, lay.recvcounts, lay.rdispls)
    part = np.full(lay.recv_bytes, 0xA5, dtype=np.uint8)
    sel = [1, 7, 11]
    assert oracle.alltoallv_receivers(send, lay.sendcounts, lay.sdispls, part, lay.recvcounts,
                                      lay.rdispls, sel) == 0
    for j in range(12):
        lo = int(lay.rdispls[j, 0])
        hi = int(lay.rdispls[j, 11] + lay.recvcounts[j, 11])
        if j in sel:
            assert np.array_equal(part[lo:hi], full[lo:hi])
        else:
            assert (part[lo:hi] == 0xA5).all()


# ---- planted mistakes: the pins above must reject plausible wrong oracles -------------------
def _mutant(kind, send, lay, recv):
    P = lay.P
    for i in range(P):
        for j in range(P):
            n = int(lay.sendcounts[i, j])
            so, ro = int(lay.sdispls[i, j]), int(lay.rdispls[j, i])
            if kind == "no_transpose":          # writes where rank i would receive from j
                ro = int(lay.rdispls[i, j])
                n = min(n, int(lay.recvcounts[i, j]))
            elif kind == "wrong_count":         # uses the receiver's row of sendcounts
                n = int(lay.sendcounts[j, i])
            elif kind == "off_by_one_block":    # reads the neighbouring block
                so = int(lay.sdispls[i, (j + 1) % P])
            elif kind == "drops_last_sender" and i == P - 1:
                continue
            n = max(0, min(n, recv.size - ro, send.size - so))
            recv[ro:ro + n] = send[so:so + n]


@pytest.mark.parametrize("kind", ["no_transpose", "wrong_count", "off_by_one_block", "drops_last_sender"])
def test_planted_mistakes_fail_the_decode_pin(kind):
    lay = wl.make_layout(_random_counts(6, 21, zero_frac=0.1), gap=8)
    send = wl.payload_traceable_int32(lay)
    recv = np.full(lay.recv_bytes, 0xA5, dtype=np.uint8)
    _mutant(kind, send, lay, recv)
    assert not decode_check(recv, lay)


# ---- the input generators themselves ----------------------------------------------------------
def test_generators_are_seeded_and_shaped():
    c3 = wl.make_counts(3, 256)
    assert c3.min() >= 0 and c3.max() <= 16384 and (c3 % 4 == 0).all()
    assert 0.18 < (c3 == 0).mean() < 0.25          # ~21.5 % empty blocks
    c4 = wl.make_counts(4, 256).astype(np.float64)
    assert abs(c4.mean() - 1024) < 8 and abs(c4.std() - 256) < 8 and (c4 % 4 == 0).all()
    c2 = wl.make_counts(2, 128)
    assert c2.min() >= 0 and c2.max() <= 1024 and (c2 % 4 != 0).any()
    assert (wl.make_counts(5, 8) == 256).all()
    assert np.array_equal(wl.make_counts(4, 64), wl.make_counts(4, 64))
    a = wl.payload_position_hash(17, 1000, start=0)
    b = wl.payload_position_hash(17, 100, start=333)
    assert np.array_equal(a[333:433], b)


def test_fft_patterns_have_the_stated_totals():
    """Section "Fast Fourier transform": N1 = ceil(0.78125 P) ceil(0.625 P) 8 and
    N2 = ((P - 1) 32 + 8) P complex values of two FP64 each ... the count matrices must add up
    to the stated problem sizes (N1 counts FP64 values, N2 complex values)."""
    import math
    for P in (8, 64, 200):
        n1 = wl.counts_fft_n1(P)
        assert int(n1.sum()) // 8 == math.ceil(0.78125 * P) * math.ceil(0.625 * P) * 8
        assert (n1[math.ceil(0.625 * P):] == 0).all() and (n1[:, math.ceil(0.78125 * P):] == 0).all()
        n2 = wl.counts_fft_n2(P)
        assert int(n2.sum()) // 16 == ((P - 1) * 32 + 8) * P


def test_torch_payload_matches_numpy_payload():
    import torch

    n = 8 * 1000 + 5
    t = wl.payload_position_hash_torch(77, n, "cpu", chunk_words=300)
    assert np.array_equal(t.numpy(), wl.payload_position_hash(77, n))
