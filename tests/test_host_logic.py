"""The launcher's host-side planning (csrc/sr_host.h) compiled alone for the CPU: the cut of a tensor
slice into launch-sized pieces, the index-range checks and the LDS reservation behind the cap on
resident waves.  Properties are checked against definitions written out here, on random and on
edge inputs."""
import ctypes as C
import os
import random
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def host(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    so = str(tmp_path_factory.mktemp("host") / "libhostlogic.so")
    subprocess.run([gxx, "-O1", "-std=c++17", "-Wall", "-Werror", "-fPIC", "-shared",
                    os.path.join(HERE, "host_logic_driver.cpp"), "-o", so], check=True)
    L = C.CDLL(so)
    L.plan_pieces.argtypes = [C.c_ulonglong] * 3 + [C.POINTER(C.c_ulonglong), C.c_longlong, C.c_longlong]
    L.plan_pieces.restype = C.c_longlong
    L.range_wraps.argtypes = [C.c_ulonglong] * 2
    L.blocks_spanned.argtypes = [C.c_ulonglong] * 2
    L.blocks_spanned.restype = C.c_ulonglong
    L.chunks_of.argtypes = [C.c_ulonglong] * 2
    L.chunks_of.restype = C.c_longlong
    L.occupancy_lds.argtypes = [C.c_uint]
    L.occupancy_lds.restype = C.c_uint
    return L


def pieces(L, numel, off, bpp, cap=4096, fail_at=-1):
    buf = (C.c_ulonglong * (3 * cap))()
    n = L.plan_pieces(numel, off, bpp, buf, cap, fail_at)
    return n, [(buf[3 * i], buf[3 * i + 1], buf[3 * i + 2]) for i in range(max(0, min(n, cap)))]


def check_cut(L, numel, off, bpp):
    n, ps = pieces(L, numel, off, bpp)
    nblk = (off + numel - 1) // 8 - off // 8 + 1
    assert L.blocks_spanned(numel, off) == nblk
    assert n == -(-nblk // bpp), (numel, off, bpp)                 # as few pieces as the limit allows
    at = 0
    for i, (local, cnt, goff) in enumerate(ps):
        assert local == at and goff == off + at and cnt >= 1        # consecutive, counter index follows
        if i > 0:
            assert goff % 8 == 0                                    # later pieces start on a block boundary
        assert (goff + cnt - 1) // 8 - goff // 8 + 1 <= bpp         # no piece spans more blocks than allowed
        at += cnt
    assert at == numel                                              # the pieces tile the slice exactly


def test_pieces_tile_the_slice_on_edge_cases(host):
    for numel, off, bpp in [(1, 0, 1), (1, 7, 1), (8, 0, 1), (9, 7, 1), (16, 1, 2), (17, 7, 2), (64, 0, 8), (64, 5, 8),
                            (1000, 3, 1), (512 * 5, 0, 64), (512 * 5 + 1, 7, 64), (7, 1, 100),
                            (1 << 40, (1 << 62) + 5, 1 << 33), (12345, (1 << 64) - 8 - 12345, 10)]:
        check_cut(host, numel, off, bpp)


def test_pieces_tile_the_slice_on_random_inputs(host):
    rng = random.Random(5)
    for _ in range(3000):
        bpp = rng.choice([1, 2, 3, 7, 64, 1000])
        numel = rng.randrange(1, 8 * bpp * rng.choice([1, 2, 9, 40]) + 9)
        off = rng.choice([0, rng.randrange(0, 64), rng.randrange(0, 1 << 63)])
        check_cut(host, numel, off, bpp)


def test_a_failing_piece_stops_the_walk(host):
    n, _ = pieces(host, 1000, 3, 4, fail_at=5)
    assert n == -1 - 5
    n, _ = pieces(host, 1000, 3, 4, fail_at=10 ** 6)
    assert n == -(-((1002 // 8) - 0 + 1) // 4)


def test_index_range_check(host):
    top = (1 << 64) - 1
    for off, numel, want in [(0, 1, 0), (top - 8 - 10, 10, 0), (top - 8 - 10 + 1, 10, 1), (0, top - 8, 0), (0, top - 7, 1),
                             (1 << 63, 1 << 63, 1), ((1 << 63) - 9, 1 << 63, 0), ((1 << 63) - 8, 1 << 63, 1)]:
        assert host.range_wraps(off, numel) == want, (off, numel)
        if not want:
            assert off + numel + 8 <= top                           # the definition: a rounded-up end still fits


def test_chunk_count_and_its_overflow_guard(host):
    top = (1 << 64) - 1
    for numel in (0, 1, 65535, 65536, 65537, 1 << 40):
        assert host.chunks_of(numel, 65536) == -(-numel // 65536)
    assert host.chunks_of(top - 65535, 65536) == (top - 65535 + 65535) // 65536
    assert host.chunks_of(top - 65534, 65536) == -1
    assert host.chunks_of(top, 65536) == -1


def test_lds_reservation_is_the_largest_that_admits_the_asked_number_of_waves(host):
    """LDS is granted in units of 1280 bytes, 128 per CU: the reservation is a whole number of units,
    `waves` workgroups of that size fit, and one unit more per workgroup would not let them."""
    unit, units = 1280, 128
    assert host.occupancy_lds(0) == 0 and host.occupancy_lds(32) == 0 and host.occupancy_lds(100) == 0
    for waves in range(3, 32):
        b = host.occupancy_lds(waves)
        assert b % unit == 0 and 0 < b <= 64 * 1024
        per = b // unit
        assert per * waves <= units < (per + 1) * waves
    # the settings the library uses, in units per workgroup (what the hardware sees)
    assert [host.occupancy_lds(w) // unit for w in (18, 11, 16, 24)] == [7, 11, 8, 5]
    assert host.occupancy_lds(1) == host.occupancy_lds(2) == host.occupancy_lds(3)   # 64 KiB per launch at most
