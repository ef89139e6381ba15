"""The library's host code under AddressSanitizer + UBSan and under ThreadSanitizer (host side only; the device code
is compiled as usual but never runs: the driver uses RUDRA_FLAG_CONTROL_ONLY).  CPU only."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "tests", "csrc", "host_driver.cpp"), os.path.join(ROOT, "paper_1509_04210_amd", "csrc", "rudra_ps.hip")]
COMMON = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
VARIANTS = {
    "asan_ubsan": ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                   "-fno-sanitize-recover=undefined"],
    "tsan": ["-Xarch_host", "-fsanitize=thread"],
}


def _build_and_run(name, tmp):
    exe = os.path.join(tmp, f"host_driver_{name}")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    b = subprocess.run([hipcc, *COMMON, *VARIANTS[name], *SRC, "-o", exe, "-lpthread"], capture_output=True, text=True)
    if b.returncode != 0:
        return name, "build", b.stderr[-2000:]
    # verify_asan_link_order=0: whatever the environment preloads stays in place ahead of the sanitizer runtime
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", TSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    ok = r.returncode == 0 and "host driver ok" in r.stdout and "Sanitizer" not in r.stderr and "runtime error" not in r.stderr
    return name, "ok" if ok else "run", (r.stdout + r.stderr)[-2000:]


def test_host_code_is_clean_under_sanitizers(tmp_path):
    with ThreadPoolExecutor(max_workers=2) as pool:
        results = list(pool.map(lambda n: _build_and_run(n, str(tmp_path)), VARIANTS))
    for name, state, out in results:
        assert state == "ok", f"{name}: {state} failed\n{out}"
