"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a
standalone driver (oracle/sanitize_main.c) runs every mode on small and degenerate tensors."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    build = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
             "-static-libasan", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
             os.path.join(ROOT, "oracle", "sanitize_main.c"), os.path.join(ROOT, "oracle", "slicer_ref.c"),
             "-lm", "-o", exe]
    subprocess.run(build, check=True, capture_output=True, text=True)
    p = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                       env=dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1"))
    assert p.returncode == 0, (p.stdout + p.stderr)[-2000:]
    assert "clean" in p.stdout
