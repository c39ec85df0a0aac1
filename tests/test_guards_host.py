"""The clamps that keep corrupt caller-owned arrays from taking a kernel outside its buffers
(csrc/guards.hpp), compiled for the host and tested on the CPU over negative, oversized and boundary values.
The kernels include the same header, so the GPU test with corrupt tables is the second line of defence, not
the first."""
import ctypes as C
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_07486_amd", "csrc")
INT_MIN, INT_MAX = -(1 << 31), (1 << 31) - 1


@pytest.fixture(scope="module")
def g(tmp_path_factory):
    d = tmp_path_factory.mktemp("guards")
    src = d / "guards_host.c"
    src.write_text('#include "guards.hpp"\n'
                   "int h_clamp_ctx(int n, int mp) { return clamp_ctx(n, mp); }\n"
                   "int h_clamp_page(int pg, int last) { return clamp_page(pg, last); }\n"
                   "int h_clamp_token(int n, int N) { return clamp_token(n, N); }\n"
                   "int h_clamp_count(int c, int C, int N) { return clamp_count(c, C, N); }\n"
                   "int h_clamp_tail(int t, int N) { return clamp_tail(t, N); }\n"
                   "int h_clamp_row(int n, int mp, long long stride) { return clamp_row(n, mp, stride); }\n")
    lib = d / "libguards.so"
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-fsanitize=undefined",
                    "-fno-sanitize-recover=undefined", "-x", "c", "-shared", "-fPIC", "-I", CSRC, str(src), "-o", str(lib)],
                   check=True)
    L = C.CDLL(str(lib))
    L.h_clamp_row.argtypes = [C.c_int, C.c_int, C.c_longlong]
    return L


EDGE = [INT_MIN, INT_MIN + 1, -(1 << 20), -17, -1, 0, 1, 15, 16, 17, 4095, 4096, 4097, (1 << 25) - 1, 1 << 25,
        (1 << 25) + 1, 1 << 30, INT_MAX - 1, INT_MAX]


def test_context_length_stays_inside_the_block_table(g):
    for mp in (0, 1, 7, 256, 2048, (1 << 25) // 16, INT_MAX // 16, INT_MAX):   # the last two: no int overflow in 16 * mp
        cap = min(16 * mp, INT_MAX)
        for n in EDGE:
            r = g.h_clamp_ctx(n, mp)
            assert 0 <= r <= cap
            assert r == n if 0 <= n <= cap else r in (0, cap)
            if r > 0:
                assert (r - 1) // 16 < mp          # the page index of the last token is a valid column of the table


def test_page_ids_stay_inside_the_pool(g):
    for last in (0, 1, 12344, INT_MAX - 1, INT_MAX):
        for pg in EDGE:
            r = g.h_clamp_page(pg, last)
            assert 0 <= r <= last
            assert r == pg if 0 <= pg <= last else r in (0, last)


def test_token_indices_stay_inside_the_sequence(g):
    for N in (0, 1, 2, 16, 4097, 1 << 25, INT_MAX):
        for n in EDGE:
            r = g.h_clamp_token(n, N)
            assert 0 <= r <= max(N - 1, 0)
            if 0 <= n < N:
                assert r == n


def test_counts_and_tail_starts(g):
    for N in (0, 1, 100, INT_MAX):
        for Cb in (1, 256, 65536):
            for c in EDGE:
                r = g.h_clamp_count(c, Cb, N)
                assert 0 <= r <= Cb and (N > 0 or r == 0)
                if 0 <= c <= Cb and N > 0:
                    assert r == c
        for t in EDGE:
            r = g.h_clamp_tail(t, N)
            assert 0 <= r <= N
            if 0 <= t <= N:
                assert r == t


def test_score_rows_never_exceed_their_stride_or_the_block_table(g):
    for mp in (0, 1, 2048, INT_MAX // 16):
        for stride in (0, 1, 16 * 2048, 16 * 2048 + 5, 1 << 40):
            for n in EDGE:
                r = g.h_clamp_row(n, mp, stride)
                assert 0 <= r <= min(16 * mp, stride, INT_MAX)
                if 0 <= n <= min(16 * mp, stride):
                    assert r == n
