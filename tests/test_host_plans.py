"""Host logic of the library without a GPU: the launch plans and workspace layouts over a sweep of
shapes (tests/host_plan_check.cpp linked against the library's objects), and the CPU oracle run
under AddressSanitizer and UndefinedBehaviorSanitizer (oracle/sanitize_check.cpp).
With AAAC_HOST_SANITIZE=1 the library's sources are recompiled for the plan check with the same
sanitizers on the host side (about a minute)."""
import os
import subprocess

import pytest

from paper_2605_08692_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def test_launch_plans_cover_every_layer_once(tmp_path):
    exe = str(tmp_path / "host_plan_check")
    driver = os.path.join(ROOT, "tests", "host_plan_check.cpp")
    inc = ["-I" + os.path.join(ROOT, "include"), "-I" + hip_build.CSRC]
    kernels = [s for s in hip_build.SOURCES if s != "aaac_api.hip"]
    if os.environ.get("AAAC_HOST_SANITIZE") == "1":
        host_san = [a for f in SAN for a in ("-Xarch_host", f)]
        cmd = [HIPCC] + hip_build.FLAGS + host_san + inc + ["-x", "hip", driver] + \
              [os.path.join(hip_build.CSRC, s) for s in kernels] + ["-o", exe]
    else:
        objs = [os.path.join(hip_build.OBJ, s + ".o") for s in kernels]
        if not all(os.path.exists(o) for o in objs):
            hip_build.build()
        cmd = [HIPCC, "--offload-arch=gfx950", "-std=c++17"] + inc + ["-x", "hip", driver, "-x", "none"] + objs + ["-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and "host_plan_check ok" in run.stdout, run.stdout[-2000:] + run.stderr[-2000:]


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    src = os.path.join(ROOT, "oracle", "sanitize_check.cpp")
    res = subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off"] + SAN + [src, "-o", exe],
                         capture_output=True, text=True)
    if res.returncode != 0 and "sanitize" in res.stderr and "cannot find" in res.stderr:
        pytest.skip("the sanitizer runtimes are not installed")
    assert res.returncode == 0, res.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and "sanitize_check ok" in run.stdout, run.stdout[-2000:] + run.stderr[-3000:]
