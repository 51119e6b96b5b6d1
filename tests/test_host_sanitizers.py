"""The host code of the library under sanitizers (no GPU): tests/host_sanitizer_driver.cpp is built against
AddressSanitizer + UndefinedBehaviorSanitizer builds of the host sources (the producers with g++, the runtime
behind the C boundary with hipcc's host pass) and against a ThreadSanitizer build of the multi-threaded
producers, and must run clean."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1903_00757_amd", "csrc")
DRIVER = os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp")
INCLUDES = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
HIPCC = "/opt/rocm/bin/hipcc"


def run_clean(cmd, exe, env_extra):
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, **env_extra)
    done = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert done.returncode == 0, done.stdout + done.stderr
    assert "all checks passed" in done.stdout
    assert "runtime error" not in done.stderr and "Sanitizer" not in done.stderr, done.stderr


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not installed")
def test_producers_under_thread_sanitizer(tmp_path):
    """gv_augment, gv_augment_weighted and gv_redistribute_pool with several workers: no data race."""
    exe = str(tmp_path / "driver_tsan")
    # the runtime behind the context calls is not part of this build: the driver's context section is compiled out
    stub = tmp_path / "stubs.cpp"
    stub.write_text('#include "gvhot.h"\n'
                    'extern "C" { int gv_create(const gv_config *c, gv_ctx **out) { if (out) *out = nullptr; return c->dim % 32 ? GV_EINVAL : GV_EHIP; }\n'
                    'void gv_destroy(gv_ctx *) {} const char *gv_last_error(const gv_ctx *) { return "stub"; }\n'
                    'int gv_sync(gv_ctx *) { return GV_EINVAL; } int gv_train_pool(gv_ctx *) { return GV_EINVAL; }\n'
                    'int gv_auc(const float *p, uint64_t np, const float *q, uint64_t nq, double *out) {\n'
                    '  if (!np || !nq) return GV_EINVAL; double w = 0; for (uint64_t i = 0; i < np; ++i) for (uint64_t j = 0; j < nq; ++j)\n'
                    '  w += p[i] > q[j] ? 1.0 : (p[i] == q[j] ? 0.5 : 0.0); *out = w / (double)(np * nq); return GV_OK; } }\n')
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", *INCLUDES, DRIVER, os.path.join(CSRC, "gv_augment.cpp"),
           str(stub), "-o", exe, "-lpthread"]
    run_clean(cmd, exe, {"TSAN_OPTIONS": "halt_on_error=1"})


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_host_runtime_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """All host sources (producers, and the runtime behind the C boundary compiled by hipcc with the sanitizers
    on its host pass only); the kernels are linked unsanitized and never launched here."""
    exe = str(tmp_path / "driver_asan")
    # sanitizers on the host pass only; the device code is built as always
    host_flags = "-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined -Xarch_host -fno-omit-frame-pointer".split()
    plain_flags = "-fsanitize=address -fsanitize=undefined -fno-gpu-sanitize -fno-omit-frame-pointer".split()
    common = [HIPCC, "-std=c++17", "-O1", "-g", "--offload-arch=gfx950", "-munsafe-fp-atomics", "-Xclang", "-target-feature",
              "-Xclang", "-packed-fp32-ops", *INCLUDES]
    objects = []
    sources = [("gv_api.cpp", ["-x", "hip", *host_flags], "gv_api.o"), ("gv_augment.cpp", host_flags, "gv_augment.o")]
    # the kernels (two objects, see the head of gv_kernels.hip) are only linked, never launched: the objects of the
    # regular build will do when they are up to date
    kernel_sources = [os.path.join(CSRC, f) for f in ("gv_kernels.hip", "gv_internal.hpp")]
    for name, flags in (("gv_kernels.o", []), ("gv_kernels_tracked.o", ["-DGV_TRACK_LOSS=1"])):
        built = os.path.join(ROOT, "paper_1903_00757_amd", "_build", name)
        if os.path.exists(built) and all(os.path.getmtime(built) >= os.path.getmtime(f) for f in kernel_sources):
            objects.append(built)
        else:
            sources.append(("gv_kernels.hip", flags, name))
    for src, flags, name in sources:
        obj = str(tmp_path / name)
        subprocess.run([*common, *flags, "-c", os.path.join(CSRC, src), "-o", obj], check=True, capture_output=True, text=True)
        objects.append(obj)
    driver_obj = str(tmp_path / "driver.o")
    subprocess.run([HIPCC, "-std=c++17", "-O1", "-g", *INCLUDES, *plain_flags, "-c", DRIVER, "-o", driver_obj],
                   check=True, capture_output=True, text=True)
    cmd = [HIPCC, "--offload-arch=gfx950", *plain_flags, driver_obj, *objects, "-o", exe, "-lpthread"]
    # the HIP runtime keeps process-lifetime allocations: leak checking is about the library's own calls only
    run_clean(cmd, exe, {"ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1", "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1"})
