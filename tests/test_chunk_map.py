"""The chunk map (which tokens a chunk id stands for) on the host: csrc/chunk_map.hpp compiled with plain g++.
Paper Sec. 1: a sequence of L tokens is cut into ceil(L / C) chunks of at most C tokens."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def locate(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("chunk_map") / "chunk_map_host.so")
    subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", os.path.join(HERE, "host", "chunk_map_host.cpp"), "-o", so],
                   check=True)
    lib = ctypes.CDLL(so)
    lib.chunk_map_locate.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_uint32, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int)]

    def call(C, total, cps, seqlens, chunks, bc):
        tok0, valid = ctypes.c_int64(), ctypes.c_int()
        if seqlens is None:
            lib.chunk_map_locate(C, total, cps, 0, None, None, bc, ctypes.byref(tok0), ctypes.byref(valid))
        else:
            s = np.ascontiguousarray(seqlens, dtype=np.int64)
            c = np.ascontiguousarray(chunks, dtype=np.int64)
            lib.chunk_map_locate(C, total, 0, len(s) - 1, s.ctypes.data, c.ctypes.data, bc, ctypes.byref(tok0), ctypes.byref(valid))
        return tok0.value, valid.value

    return call


@pytest.mark.parametrize("C", [16, 32, 64, 128])
@pytest.mark.parametrize("Tlen", [1, 63, 64, 65, 300])
def test_fixed_layout(locate, C, Tlen):
    cps = -(-Tlen // C)
    for b in range(3):
        for k in range(cps):
            tok0, valid = locate(C, Tlen, cps, None, None, b * cps + k)
            assert tok0 == b * Tlen + k * C
            assert valid == min(C, Tlen - k * C)


@pytest.mark.parametrize("C", [32, 64, 128])
def test_packed_sequences_chunk_by_chunk(locate, C):
    lens = [5, 0, 200, C, 0, 0, 2 * C + 1, 1]
    seqlens = np.concatenate([[0], np.cumsum(lens)])
    chunks = np.concatenate([[0], np.cumsum([-(-n // C) for n in lens])])
    total = int(seqlens[-1])
    bc = 0
    for s, n in enumerate(lens):                      # walk the sequences the plain way
        for k in range(-(-n // C)):
            tok0, valid = locate(C, total, 0, seqlens, chunks, bc)
            assert tok0 == seqlens[s] + k * C and valid == min(C, n - k * C), (s, k)
            bc += 1
    assert bc == chunks[-1]


@pytest.mark.parametrize("C", [64, 128])
def test_surplus_chunk_ids_and_bad_offsets_stay_inside_the_buffers(locate, C):
    """Chunk ids at or beyond the last one, trailing empty sequences and offset arrays that disagree with each other must
    still give rows inside [0, total): the kernels read rows tok0 .. tok0 + valid - 1 without any further check."""
    lens = [70, 0, 3, 0, 0]
    seqlens = np.concatenate([[0], np.cumsum(lens)])
    chunks = np.concatenate([[0], np.cumsum([-(-n // C) for n in lens])])
    total = int(seqlens[-1])
    for bc in list(range(int(chunks[-1]), int(chunks[-1]) + 5)) + [10 ** 6, 2 ** 31 - 1]:
        tok0, valid = locate(C, total, 0, seqlens, chunks, bc)
        assert 0 <= tok0 and tok0 + valid <= total and 1 <= valid <= C, (bc, tok0, valid)
    rng = np.random.default_rng(7)
    for _ in range(500):                             # garbage offsets of every kind
        n_seq = int(rng.integers(1, 6))
        bad_s = rng.integers(-500, 500, size=n_seq + 1)
        bad_c = rng.integers(-5, 10, size=n_seq + 1)
        tot = int(rng.integers(1, 300))
        bc = int(rng.integers(0, 12))
        tok0, valid = locate(C, tot, 0, bad_s, bad_c, bc)
        assert 0 <= tok0 and tok0 + valid <= tot and 1 <= valid <= C, (bad_s, bad_c, tot, bc, tok0, valid)
