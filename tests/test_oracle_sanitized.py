"""The oracle's pins once more, on a build of oracle/spec_oracle.c with gcc's undefined-behaviour sanitizer
(every finding aborts): signed overflow, bad shifts, float-to-int conversions out of range and indexing the
compiler can see to be out of bounds stop the run instead of passing silently.  Host code only."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_the_undefined_behaviour_sanitizer(tmp_path):
    import oracle
    lib = str(tmp_path / "libspec_oracle_ubsan.so")
    subprocess.run(["gcc", *oracle.CFLAGS, "-g", "-fsanitize=undefined", "-fno-sanitize-recover=all",
                    "-o", lib, os.path.join(ROOT, "oracle", "spec_oracle.c"), "-lm"], check=True)
    pins = sorted(f for f in glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py"))
                  if os.path.basename(f) != os.path.basename(__file__))
    assert len(pins) >= 8
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *pins],
                         cwd=ROOT, env=dict(os.environ, ORACLE_LIB=lib), stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True, timeout=900)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "runtime error" not in run.stdout
