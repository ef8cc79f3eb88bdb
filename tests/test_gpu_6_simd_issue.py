"""The hardware facts behind the bounds of the expert and router kernels, measured by tests/microbench/simd_issue.hip
(register-only kernels; __graft_entry__.build() compiles it): a SIMD needs max(32, 12 + 4 n) cycles per 32x32x16 matrix
instruction that has n other vector instructions beside it, and of two wavefronts on a SIMD the one that arrived first
is served first."""
import os
import re
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "microbench", "simd_issue")


def test_simd_issue_law_and_oldest_first_arbitration():
    if not os.path.exists(EXE):   # built by __graft_entry__.build(); here only if nothing is built yet
        import __graft_entry__
        __graft_entry__.build_microbench()
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, r.stdout + r.stderr
    law = {(int(m.group(1)), int(m.group(2))): (float(m.group(3)), int(m.group(4)))
           for m in re.finditer(r"law n=(\d+) waves_per_simd=(\d) cycles_per_matrix_instruction=([\d.]+) expected=(\d+)", r.stdout)}
    assert sorted(law) == [(n, w) for n in (0, 4, 7, 9, 12) for w in (1, 2)]
    for (n, w), (got, want) in law.items():
        assert want == max(32, 12 + 4 * n)
        if w == 2:     # the configuration of the expert kernels: the law to within three cycles
            assert abs(got - want) <= 3.0, (n, w, got, want)
        else:          # one wavefront issues in order: never faster than the law, a few cycles per instruction slower
            assert want - 1.5 <= got <= want + 14.0, (n, w, got, want)
    m = re.search(r"arbitration first_wavefront=([\d.]+) second_wavefront=([\d.]+)", r.stdout)
    first, second = float(m.group(1)), float(m.group(2))
    assert 31.0 <= first <= 36.0 and 60.0 <= second <= 70.0, (first, second)
