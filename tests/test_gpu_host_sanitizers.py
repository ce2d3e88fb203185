"""Host orchestration of the library under AddressSanitizer + UndefinedBehaviorSanitizer (GPU only: the host code
drives real kernels).  The sanitized build (host code only; device code as shipped) is made by build(); the native
driver runs the whole path -- compression, factorization, solves, ADMM, the lockstep C-sweep at a second beta (cached
bases), label assignment, error estimate -- once per option set, and no run may produce a sanitizer report."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = os.path.join(ROOT, "paper_2108_04167_amd", "_asan", "hss_bench_native")

RUNS = [
    "4096 8 128 64 1.5 20 3",
    "4096 8 256 64 1.5 20 3 adaptive_start=128",
    "8192 3 128 64 0.5 20 3 sampling=1",
    "4096 12 128 64 1.5 20 3 clustering=1",
    "2048 54 512 256 3.0 20 3 merge_top=0 graph=1",
    "1024 90 128 16 4.0 20 3 sampling=1 ann_trees=2 clustering=1 cache_basis=0",
    "3001 123 128 64 4.0 20 3",                               # leaves of two sizes, features beyond the fused kernels
    "2500 8 128 64 1.5 20 3 sampling=1",
    "1000 300 128 64 6.0 10 2 clustering=1 adaptive_start=128",
    "4096 8 128 64 1.5 20 3 block_cache_mib=0",              # every release a hipFree, every reservation a hipMalloc
]


@pytest.mark.parametrize("args", RUNS)
def test_no_host_sanitizer_report(args):
    if not os.path.exists(DRIVER):
        pytest.skip("sanitized build absent (build() makes it)")
    env = dict(os.environ)
    # leak detection off (the GPU runtime keeps allocations until exit); the shadow gap must stay mappable for the runtime
    env["ASAN_OPTIONS"] = "detect_leaks=0:protect_shadow_gap=0:halt_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    res = subprocess.run([DRIVER] + args.split(), capture_output=True, text=True, env=env, timeout=150)
    reports = [l for l in res.stderr.splitlines() if "ERROR: AddressSanitizer" in l or "runtime error" in l]
    assert not reports, "\n".join(reports[:10])
    # the driver printed its summary, i.e. every library call returned without an error code.  (The process can still
    # end with exit code 1 from a check inside the sanitizer's own device allocator -- "dev_runtime_unloaded_" -- when
    # memory is recycled after the GPU runtime has unloaded: at exit, or when a helper thread of the runtime ends.  All
    # frames of that are the sanitizer's and libc's, after main has returned; none is this library's.)
    assert "stream_copy_kernel" in res.stdout and "compress" in res.stdout, res.stderr[-2000:]
    if res.returncode != 0:
        assert "CHECK failed" in res.stderr and "dev_runtime_unloaded_" in res.stderr, res.stderr[-2000:]
        assert "__cxa_finalize" in res.stderr or "AsanThread::Destroy" in res.stderr, res.stderr[-2000:]
        assert "hsssvm" not in res.stderr and "hss_" not in res.stderr, res.stderr[-2000:]
