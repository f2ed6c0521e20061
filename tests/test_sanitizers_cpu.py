"""Address / undefined-behaviour sanitizer build of the host code: the CPU oracle (oracle/lba_ref.cpp) and the
host planner (paper_2401_14110_amd/csrc/lba_plan.cpp, which has no device code) are compiled together with
tests/sanitize_driver.cpp under -fsanitize=address,undefined; the driver replays the hand-worked pins of
tests/golden/ through that build, runs every oracle entry point on ragged shapes with both integer carriers, and
sweeps the planner over the format space and the shape limits.  CPU only: nothing here is ever run on a GPU."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(ROOT, "tests", "golden")


def _clang():
    for c in ("/opt/rocm/lib/llvm/bin/clang++", "/opt/rocm/llvm/bin/clang++"):
        if os.path.exists(c):
            return c
    return "clang++"


def test_oracle_and_planner_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    subprocess.run([_clang(), "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-pthread",
                    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2401_14110_amd", "csrc"),
                    os.path.join(ROOT, "oracle", "lba_ref.cpp"),
                    os.path.join(ROOT, "paper_2401_14110_amd", "csrc", "lba_plan.cpp"),
                    os.path.join(ROOT, "tests", "sanitize_driver.cpp"), "-o", exe], check=True)
    # the hand-worked roundings, with their expressions evaluated here (exact dyadic numbers) and handed over as hex floats
    rows = []
    for line in open(os.path.join(GOLD, "q_m7e4_b7_roundings.txt")):
        if line.strip() and not line.startswith("#"):
            x, f, r = (float(eval(t, {"__builtins__": {}})) for t in line.split())
            rows.append("%s %s %s\n" % (x.hex(), f.hex(), r.hex()))
    assert len(rows) >= 12
    rpath = tmp_path / "roundings.txt"
    rpath.write_text("".join(rows))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, str(rpath), os.path.join(GOLD, "chain_p1b.txt")], capture_output=True, text=True, env=env)
    assert run.returncode == 0, (run.returncode, run.stdout[-3000:], run.stderr[-3000:])
    assert "sanitize driver ok" in run.stdout
