"""AddressSanitizer + UndefinedBehaviorSanitizer passes on the CPU side (no GPU is used):
the oracle over the whole append -> score -> top-k -> gather -> assemble path at ragged shapes,
and the host side of the C ABI (argument validation) with fake device pointers and launcher
stubs.  Both drivers exit 0 only if no sanitizer report was raised
(-fno-sanitize-recover=all turns every report into an abort)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\nstdout:\n{r.stdout}\nstderr:\n{r.stderr[-4000:]}"
    return r.stdout


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c11", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=all", "-Wall", os.path.join(SAN, "oracle_driver.c"), "-lm", "-o", exe])
    out = _run([exe])
    assert "144 cases clean" in out


def test_abi_host_validation_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "abi_driver")
    _run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
          "-Xarch_host", "-fno-sanitize-recover=all", "-Wno-unused-result",
          "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2510_18269_amd", "csrc"),
          os.path.join(ROOT, "paper_2510_18269_amd", "csrc", "oqm_api.hip"),
          os.path.join(SAN, "abi_driver.cpp"), "-o", exe])
    # the HIP runtime's own start-up allocations are not this test's subject
    out = _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    assert "abi sanitizer driver: clean" in out
