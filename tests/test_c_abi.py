"""The boundary used from plain C (gcc, no C++ / Python in between), and from several
threads at once (maps are immutable and every builder returns a new one)."""
import os
import subprocess
import sys
import threading

import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from tests import chains

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_caller(tmp_path):
    exe = str(tmp_path / "c_abi_example")
    libdir = os.path.dirname(B.LIB_PATH)
    # the library depends on the HIP runtime; resolve it the way the Python binding does (torch's copy first)
    import torch
    rt_dirs = [os.path.join(os.path.dirname(torch.__file__), "lib"), "/opt/rocm/lib"]
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_example.c"), "-o", exe, B.LIB_PATH,
           "-Wl,--allow-shlib-undefined"] + [f"-Wl,-rpath,{d}" for d in [libdir] + rt_dirs]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, LD_LIBRARY_PATH=":".join(rt_dirs + [os.environ.get("LD_LIBRARY_PATH", "")]))
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("OK"), (r.stdout, r.stderr)


def test_builders_from_several_threads():
    errors = []

    def work(tid):
        try:
            for seed in range(tid * 25, tid * 25 + 25):
                src_shapes, ops = chains.random_chain(seed, extended=True)
                srcs = [np.arange(int(np.prod(s)), dtype=np.uint32).reshape(s) + 7 * i for i, s in enumerate(src_shapes)]
                m = B.amap_compose(src_shapes, 4, ops)
                got = B.amap_eval_host(m, srcs)
                if B.amap_describe(m).strided:
                    assert B.amap_plan_selfcheck(m, -1) == 0
                want = oracle.run_chain(srcs, ops)
                assert np.array_equal(got, want), seed
        except Exception as e:  # noqa: BLE001 - reported to the main thread
            errors.append((tid, repr(e)))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(6)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_gemm_refusals_name_their_reason():
    """The requirements of the GEMM entry points are checked on the host before anything is
    launched; a refusal leaves its reason for amap_last_error (no GPU needed to get that far)."""
    fake = [0x10000, 0x20000]           # aligned, never dereferenced: the calls return before any launch
    cases = [
        (B.amap_compose([(256, 68)], 2, []), 256, "multiples of 8"),
        (B.amap_compose([(256, 128)], 2, [("slice", 1, 0, 128, 2)]), 256, "aligned source runs"),
        (B.amap_compose([(256, 32), (256, 96)], 2, [("concat", 1)]), 64, "ends inside a k-step"),
        (B.amap_compose([(128, 64), (128, 64)], 2, [("concat", 0)]), 64, "span all of m"),
        (B.amap_compose([(256, 64)] * 9, 2, [("concat", 1)]), 64, "up to 8"),
    ]
    for m, n, word in cases:
        with pytest.raises(B.AmapError) as e:
            B.amap_gemm_gather(fake * 5, m, 0x900000, None, n, None, 0xA00000, 0)
        assert e.value.status == B.AMAP_E_UNSUPPORTED and word in str(e.value), str(e.value)
