"""The work split of the streaming expert kernels (csrc/stream_sched.h), compiled for the host and run on the
CPU: whatever the numbers of experts per class, the layer shape and the number of workgroups, every tile of
every class must be taken by exactly one workgroup (fixed ranges) or lie in exactly one drawn unit."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "native", "stream_sched_host.cpp")
HDR = os.path.join(HERE, "..", "paper_2505_19645_amd", "csrc", "stream_sched.h")


@pytest.fixture(scope="module")
def sched(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("sched") / "libsched.so")
    subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-Wall", "-Werror", "-fsanitize=undefined",
                    "-fno-sanitize-recover=undefined", "-o", so, SRC], check=True)
    L = C.CDLL(so)
    L.moesd_test_stream_schedule.argtypes = [C.c_int] * 14 + [C.POINTER(C.c_int)]
    L.moesd_test_unit_range.argtypes = [C.c_int] * 6 + [C.POINTER(C.c_int)]
    return L


def split(L, mode, d, I, S, T, part_k, shared_stream, ns, n64, n128, G, dyn, fp8=0):
    rows = []
    for b in range(G):
        out = (C.c_int * 24)()
        L.moesd_test_stream_schedule(mode, d, I, S, T, part_k, shared_stream, ns, n64, n128, G, b, dyn, fp8, out)
        rows.append(list(out))
    return np.array(rows)


def check(L, mode, d, I, S, T, part_k, shared_stream, ns, n64, n128, G, dyn, fp8=0):
    r = split(L, mode, d, I, S, T, part_k, shared_stream, ns, n64, n128, G, dyn, fp8)
    label = dict(mode=mode, d=d, I=I, S=S, T=T, ns=ns, n64=n64, n128=n128, G=G, dyn=dyn)
    parts = -(-S // part_k) if (mode == 1 and S > 0) else 1
    for ci, (n_e, rows_per) in enumerate(((n128, 128), (n64, 64))):
        n_sh, per_s, per_r = r[0, 6 * ci + 3], r[0, 6 * ci + 4], r[0, 6 * ci + 5]
        assert (r[:, 6 * ci + 3] == n_sh).all()
        n_tiles = n_sh + n_e * per_r
        taken = np.zeros(n_tiles, int)
        for b in range(G):
            n_mine, id0, stride = r[b, 6 * ci: 6 * ci + 3]
            ids = id0 + stride * np.arange(n_mine)
            assert (ids < n_tiles).all() and (ids >= 0).all(), (label, ci, b)
            taken[ids] += 1
        assert (taken == 1).all(), (label, "wide class", rows_per)
        # where the shared expert is
        want_sh = 0
        if S > 0 and ((ci == 1 and 16 < T <= 64) or (ci == 0 and T > 64 and shared_stream)):
            want_sh = per_s * parts * (-(-T // rows_per) if ci == 0 else 1)
        assert n_sh == want_sh, (label, ci)
    # the small line: fixed ranges are consecutive, start at 0 and end where the drawn part begins
    dyn_on, n_units, n_double, ut, pool0, n_tiles = r[0, 18:24]
    assert (r[:, 18:24] == r[0, 18:24]).all()
    n_stat = pool0 if dyn_on else n_tiles
    pos = 0
    for b in range(G):
        n_mine, id0, stride = r[b, 12:15]
        assert stride == 1 and n_mine >= 0 and id0 == pos, (label, b, id0, pos)
        pos += n_mine
    assert pos == n_stat, label
    want_small = ns * r[0, 17] + (r[0, 16] * parts * -(-T // 16) if (S > 0 and T <= 16) else 0)
    assert n_tiles == want_small, label
    srows = 64 if fp8 else 32          # weight rows of a small tile
    assert r[0, 17] == (-(-I // (srows // 2)) if mode == 0 else -(-d // srows)), label
    if dyn_on:
        assert dyn and n_units >= G and pool0 % ut == 0
        end = pool0
        for u in range(n_units):
            t = (C.c_int * 2)()
            L.moesd_test_unit_range(n_units, n_double, ut, pool0, n_tiles, u, t)
            assert t[0] == end and t[1] > t[0], (label, u)
            assert (t[1] - t[0]) * 1 >= ut
            end = t[1]
        assert end == n_tiles
        t = (C.c_int * 2)()
        for u in (-1, n_units, n_units + 7):
            L.moesd_test_unit_range(n_units, n_double, ut, pool0, n_tiles, u, t)
            assert t[0] == t[1]
    return r


def test_benchmark_shapes(sched):
    # (d, I, S) of the five benchmark shapes at a few token counts, 256 workgroups, classes as uniform routing gives
    for d, I, S, E, K in ((256, 512, 0, 8, 2), (2048, 1408, 5632, 60, 4), (3584, 2560, 20480, 64, 8),
                          (4096, 14336, 0, 8, 2), (7168, 2048, 2048, 256, 8)):
        part_k = -(-I // 256) * 256
        for T in (1, 16, 17, 64, 100, 128, 300, 640, 2560):
            rows = T * K / E
            n = min(E, T * K)
            ns, n64, n128 = (n, 0, 0) if rows <= 12 else (n // 2, n - n // 2, 0) if rows <= 24 else \
                (0, n, 0) if rows <= 56 else (0, n // 2, n - n // 2) if rows <= 100 else (0, 0, n // 2)
            for mode in (0, 1):
                for ss in (0, 1):
                    check(sched, mode, d, I, S, T, part_k, ss, ns, n64, n128, 256, 1)


def test_random_splits(sched):
    rng = np.random.default_rng(12)
    for _ in range(400):
        d = 8 * int(rng.integers(8, 900))
        I = 8 * int(rng.integers(2, 1800))
        S = 0 if rng.random() < 0.4 else 8 * int(rng.integers(2, 2600))
        part_k = -(-I // 256) * 256
        T = int(rng.choice([1, 5, 16, 17, 40, 64, 65, 128, 129, 500, 3000]))
        G = int(rng.choice([1, 7, 32, 104, 256, 304]))
        ns, n64, n128 = (int(rng.integers(0, m)) for m in (300, 70, 70))
        if rng.random() < 0.3:
            n64 = n128 = 0
        if rng.random() < 0.2:
            ns = 0
        fp8 = int(rng.random() < 0.3)
        check(sched, int(rng.integers(0, 2)), d, I, S, T, part_k, int(rng.integers(0, 2)), ns, n64, n128, G,
              int(rng.integers(0, 2)), fp8)


def test_long_small_line_is_drawn_and_balanced(sched):
    # like the headline point of the largest benchmark shape, without its shared expert: 214 experts with few
    # rows each and nothing else
    r = check(sched, 0, 7168, 2048, 0, 64, 2048, 1, 214, 0, 0, 256, 1)
    assert r[0, 18] == 1                      # units are drawn
    n_mine = r[:, 12]
    assert n_mine.max() - n_mine.min() <= r[0, 21]   # equal fixed shares up to one unit
    # wide tiles shift the small line towards the workgroups that hold fewer of them
    r = check(sched, 1, 2048, 1408, 5632, 100, 1536, 1, 40, 20, 3, 256, 0)
    wide = r[:, 0] + r[:, 6]
    small = r[:, 12]
    assert small[wide == wide.min()].mean() > small[wide == wide.max()].mean()
