"""The library's host code (descriptions, plans, index maps, attention index data, scheduling front-end) under
AddressSanitizer + UndefinedBehaviorSanitizer, driven by tests/host_sanitize_driver.cpp on seeded random inputs.
Only host code is instrumented (the sanitizer flags follow -Xarch_host); the kernel objects are the ordinary ones
and are never launched: the run needs no GPU."""
import glob
import os
import shutil
import subprocess

import pytest

from paper_2603_26498_amd import build as B

HERE = os.path.dirname(os.path.abspath(__file__))
KERNEL_SOURCES = [s for s in B.SOURCES if s not in ("api.hip", "sched.cpp")]
SAN = ["-O1", "-g", "-fno-omit-frame-pointer"]
HOST_SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined"]


def _kernel_objects():
    """Ordinary objects of the kernel files, rebuilt when a source or header is newer than they are."""
    newest_header = max(os.path.getmtime(p) for p in glob.glob(os.path.join(B.CSRC, "*.h")) +
                        glob.glob(os.path.join(HERE, "..", "include", "*.h")))
    objs = [os.path.join(B.OBJ, os.path.splitext(s)[0] + ".o") for s in KERNEL_SOURCES]
    stale = [o for o, s in zip(objs, KERNEL_SOURCES)
             if not os.path.exists(o) or os.path.getmtime(o) < max(newest_header, os.path.getmtime(os.path.join(B.CSRC, s)))]
    if stale:
        B.build()
    return objs


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="hipcc not found")
def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hipcc = B._hipcc()
    objs = _kernel_objects()
    api_o, sched_o, drv_o, exe = (str(tmp_path / n) for n in ("api.o", "sched.o", "driver.o", "driver"))
    flags = [f for f in B.FLAGS if f != "-O3"]
    B._run([hipcc, *flags, *SAN, *HOST_SAN, "-c", os.path.join(B.CSRC, "api.hip"), "-o", api_o])
    plain = ["-std=c++17", "-Wno-option-ignored", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    B._run([hipcc, *SAN, *plain, "-x", "c++", "-c", os.path.join(B.CSRC, "sched.cpp"), "-o", sched_o])
    B._run([hipcc, *SAN, *plain, "-x", "c++", "-c", os.path.join(HERE, "host_sanitize_driver.cpp"), "-o", drv_o])
    B._run([hipcc, "--offload-arch=gfx950", "-Wno-option-ignored", "-fsanitize=address,undefined", api_o, sched_o, drv_o, *objs, "-o", exe])
    for seed in ("1", "2", "3"):
        r = subprocess.run([exe, seed], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
        assert r.returncode == 0 and "all expectations held" in r.stdout, r.stdout[-4000:]
