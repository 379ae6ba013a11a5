"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer.

Every source of the library is compiled with both sanitizers on its host code
(the device code is built as always and never launched), linked with a driver
that replays the host-only entry points - argument validation, the Gram-path
cost model, workspace sizes, the contraction's launch plan with its XCD work
ranges and token split, the stash layout - over the benchmark's shapes and a
set of edge cases.  The index arithmetic in there decides which tile a
workgroup stores to, so it has to be free of overflow and out-of-range reads.
No GPU is touched.  The numbers the sanitized build prints are compared with
the regular build's.
"""
import os
import re
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2512_23353_amd import build as libbuild
from paper_2512_23353_amd import isopo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def _build(tmp):
    if shutil.which("hipcc") is None:
        pytest.skip("no hipcc")
    # the library's own flags (device code as always), host code at -O1 with the sanitizers
    base = ["hipcc", *[f for f in libbuild.FLAGS if f != "-O3"], "-O1", "-g", *SAN]

    def one(src):
        obj = os.path.join(tmp, os.path.splitext(os.path.basename(src))[0] + ".o")
        r = subprocess.run([*base, "-x", "hip", "-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-4000:]
        return obj
    srcs = [os.path.join(libbuild.CSRC, s) for s in libbuild.SOURCES] + [os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp")]
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(one, srcs))
    exe = os.path.join(tmp, "host_sanitizer_driver")
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        "-o", exe, *objs], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    return exe


def test_host_code_under_address_and_ub_sanitizers(tmp_path):
    exe = _build(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    report = r.stdout[-3000:] + r.stderr[-6000:]
    assert r.returncode == 0, report
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, report
    assert "done failures=0" in r.stdout and "FAIL" not in r.stdout, report
    lines = r.stdout.splitlines()
    assert sum(" contraction per_seq=" in l for l in lines) >= 80

    # the regular build returns the same numbers for the cases whose inputs this test can rebuild
    def host_layer(lengths, d_in, d_out, dtype=isopo.BF16):
        off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
        return isopo.Layer(None, None, off, d_in=d_in, d_out=d_out, dtype=dtype, n_tokens=int(off[-1]))
    for tag, lengths, d_in, d_out in (("config4/gate", [2048] * 64, 1536, 8960), ("config4/k", [2048] * 64, 1536, 256),
                                      ("one_tile", [4096], 256, 256), ("empty_some", [0, 5, 0, 700, 0], 1536, 256),
                                      ("long_narrow", [100000, 31072], 256, 384)):
        lay = host_layer(lengths, d_in, d_out)
        chosen, full, mn = isopo.gram_plan(lay)
        line = next(l for l in lines if l.startswith(f"{tag} plan req=0 "))
        got = dict(kv.split("=") for kv in line.split()[2:])
        assert (int(got["full"]), int(got["min"])) == (full, mn)
        assert {1: "ghost", 2: "materialised"}[int(got["chosen"])] == chosen
        for per_seq in (0, 1):
            pl = isopo.contraction_plan(lay.ref(), bool(per_seq))
            line = next(l for l in lines if l.startswith(f"{tag} contraction per_seq={per_seq} tile="))
            got = dict(kv.split("=") for kv in line.split()[2:])
            assert [int(v) for v in got["xcd"].split(",")] == pl["xcd_start"]
            assert (int(got["tile"]), int(got["tiles"]), int(got["chunks"]), int(got["chunk_tokens"]), int(got["whole"]),
                    int(got["wgs"])) == (pl["tile"], pl["tiles"], pl["n_chunks"], pl["chunk_tokens"], pl["whole_tiles"],
                                         pl["workgroups"])
