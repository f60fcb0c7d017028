"""Host logic that sizes the launches (csrc/rk_internal.h), checked without a GPU.

A small host program that includes the library's own header is compiled with hipcc and prints what
the rules give for a table of shapes; the test checks the bounds every kernel relies on (at least
one workgroup, never more partial results than the merge has slots for, never more than there are
stretches of 128 rows) and the choices the measurements in the header's comments led to.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2411_05787_amd", "csrc")

PROGRAM = r"""
#include "rk_internal.h"
#include <cstdio>
using namespace rk;
int main() {
    const long rows[] = {1, 100, 128, 129, 512, 1024, 2048, 4096, 8192, 16384};
    const long problems[] = {1, 4, 8, 16, 24, 32, 64, 128, 256, 512, 4096};
    for (long r : rows) for (long p : problems) for (int tail : {0, 10, 128, 500})
        printf("merged %ld %d %ld %d %d %d\n", r, tail, p, merged_split_workgroups(r, tail, p, false),
               merged_split_workgroups(r, tail, p, true), (int)two_batches_pay(r, tail, p));
    for (long r : rows) for (long p : problems) for (int tail : {0, 10, 500}) {
        int own = -1;
        const int n = batched_tagged_workgroups(r, tail, &own, p);
        printf("batched %ld %d %ld %d %d\n", r, tail, p, n, own);
    }
    for (long r : {1L, 100L, 128L, 1024L, 2048L, 3072L, 4096L, 6144L, 8192L, 12288L, 16384L, 100000L}) for (long p : {1L, 4L, 8L})
        for (int tail : {0, 10, 128, 500}) {
            int own = -1;
            const int n = sliced_split_workgroups(r, tail, &own, p, 64);
            printf("sliced %ld %d %ld %d %d\n", r, tail, p, n, own);
        }
    const long lens[] = {1, 2000, 32768, 33008, 65536, 131072, 1000000};
    for (long l : lens) for (int b : {1, 2, 16}) for (int hkv : {1, 4, 8}) {
        rk_geom g{b, hkv * 4, hkv, 128, 1.0f};
        printf("emit %ld %d %d %d\n", l, b, hkv, emit_split_workgroups(&g, l));
    }
    return 0;
}
"""


@pytest.fixture(scope="module")
def table(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    d = tmp_path_factory.mktemp("sizes")
    src = d / "sizes.cpp"
    src.write_text(PROGRAM)
    exe = d / "sizes"
    # host code only: no offload architecture needed, nothing is launched
    r = subprocess.run([hipcc, "-O1", "-std=c++17", "-I", CSRC, "-x", "hip", "--offload-arch=gfx950", str(src), "-o", str(exe)],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stderr[-2000:]
    rows = [ln.split() for ln in out.stdout.splitlines()]
    return rows


def test_merged_split_bounds(table):
    seen = 0
    for kind, *v in table:
        if kind != "merged":
            continue
        rows, tail, problems, n16, n32, pays = map(int, v)
        counted = rows if tail <= 32 else rows + tail
        stretches = max((counted + 127) // 128, 1)
        for n in (n16, n32):
            assert 1 <= n <= 64
            assert n <= stretches or n == 32, (rows, tail, problems, n)
        if n32 != n16:
            assert n32 == 32 and pays == 1              # the only difference the ticketed form makes
        if pays:
            assert problems <= 8 and rows + (tail if tail > 128 else 0) > 2048
        seen += 1
    assert seen == 10 * 11 * 4


def test_batched_tagged_bounds_and_measured_choices(table):
    got = {}
    for kind, *v in table:
        if kind != "batched":
            continue
        rows, tail, problems, n, own = map(int, v)
        counted = rows if tail <= 128 else rows + tail
        assert own in (0, 1) and 1 <= n <= 64 and n <= max((counted + 127) // 128, 1)
        if tail == 0 or tail > 128:
            assert own == 0
        got[(rows, tail, problems)] = (n, own)
    # the shapes that were measured
    assert got[(2048, 10, 128)] == (2, 0) and got[(1024, 10, 128)] == (2, 0)      # 16 sequences x 8 KV heads: 256 workgroups, no tail workgroup
    assert got[(2048, 10, 64)] == (4, 0)                                        # 8 sequences: 256 workgroups
    assert sum(got[(2048, 10, 32)]) * 32 <= 256 and sum(got[(8192, 10, 32)]) * 32 <= 256    # 4 sequences: at most 256 workgroups
    assert got[(2048, 10, 16)][0] == 16 and got[(2048, 10, 24)][0] == 16        # 2 and 3 sequences: one tile per wavefront
    assert sum(got[(4096, 10, 16)]) * 16 <= 256                                 # 2 sequences, K = 4096: no CU with two workgroups


def test_headline_shapes(table):
    merged = {(int(v[0]), int(v[1]), int(v[2])): (int(v[3]), int(v[4])) for kind, *v in table if kind == "merged"}
    assert merged[(2048, 10, 8)] == (16, 16)            # cfg2's partial step: 16 workgroups + the tail's own
    assert merged[(4096, 10, 4)][1] == 32               # cfg3 (4 KV heads, 7 heads per group: ticketed)
    assert merged[(8192, 10, 8)][1] == 32               # cfg5: ticketed with 32 workgroups
    emit = {(int(v[0]), int(v[1]), int(v[2])): int(v[3]) for kind, *v in table if kind == "emit"}
    assert emit[(33008, 1, 8)] * 8 == 512               # cfg2's full-cache kernel: 512 workgroups
    assert emit[(65536, 1, 4)] * 4 == 512               # cfg3
    assert emit[(131072, 1, 8)] * 8 == 1024             # cfg5
    for (length, b, hkv), n in emit.items():
        assert 1 <= n <= 1024 and n <= max((length + 127) // 128, 1)


def test_sliced_split_bounds_and_measured_choices(table):
    """Sizing of the partial step for the merge by slices: within what the merge takes and what is resident at once,
    never more workgroups than stretches of 128 rows, and the choices the measurements led to."""
    got = {}
    for kind, *v in table:
        if kind != "sliced":
            continue
        rows, tail, problems, n, own = map(int, v)
        got[(rows, tail, problems)] = (n, own)
        assert own in (0, 1) and 1 <= n and n + own <= 64
        assert (n + own) * problems <= 512
        counted = rows if tail <= 128 else rows + tail
        assert n <= max((counted + 127) // 128, 1)
        if tail > 128:
            assert own == 0
    assert len(got) == 12 * 3 * 4
    assert got[(2048, 10, 8)] == (16, 1)          # 16 workgroups of one tile per wavefront and the tail's own
    assert got[(4096, 10, 8)] == (32, 0)          # 32 x 8 = 256 workgroups: the tail's would be the only ones beyond one per CU
    assert got[(4096, 10, 4)] == (32, 1)
    assert got[(8192, 10, 8)] == (64, 0)          # a 65th partial result would cost every wavefront a second tile
    assert got[(8192, 10, 4)] == (64, 0)
    assert got[(16384, 10, 8)] == (64, 0)         # two tiles per wavefront either way
    assert got[(3072, 10, 8)] == (24, 1)
