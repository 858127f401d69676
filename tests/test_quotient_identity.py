"""The division-free code path of the GPU quantizer rests on an IEEE binary32 identity; this test
proves it by exhaustion on the CPU (every bf16 abs-max, every bf16 element below it, both code
widths: 1.4e9 pairs, a few seconds with OpenMP)."""
import os
import subprocess
import tempfile


def test_corrected_reciprocal_quotient_matches_ieee_division_for_all_bf16_pairs():
    src = os.path.join(os.path.dirname(__file__), "quotient_identity.c")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "quotient_identity")
        subprocess.run(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-o", exe, src, "-lm"], check=True)
        out = subprocess.run([exe], check=True, capture_output=True, text=True,
                             env=dict(os.environ, OMP_NUM_THREADS=str(min(8, os.cpu_count() or 1)))).stdout
    rows = [list(map(int, line.split())) for line in out.strip().splitlines()]
    assert [r[0] for r in rows] == [7, 127]
    for qmax, pairs, bad1, bad2, bad3 in rows:
        assert pairs > 500_000_000
        assert (bad1, bad2, bad3) == (0, 0, 0)
