"""The library's HOST logic (argument checks, workspace planning, pointer tables, the sequencing of launches)
under AddressSanitizer + UndefinedBehaviorSanitizer.  `br_native_bench_san` is the C driver of the ABI linked with
every library source, host code instrumented (paper_2602_03515_amd.build.build_sanitized; device code is compiled
as usual).  Without a GPU it walks the planning and validation code; with one it runs every call of the ABI."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "paper_2602_03515_amd", "br_native_bench_san")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _exe():
    if not os.path.exists(EXE):
        from paper_2602_03515_amd.build import build_sanitized
        build_sanitized()
    return EXE


def test_host_logic_is_clean_under_asan_and_ubsan_without_a_gpu():
    res = subprocess.run([_exe(), "--host-only"], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "0 surprises" in res.stdout and "ERROR: AddressSanitizer" not in res.stdout and "runtime error" not in res.stdout


@pytest.mark.gpu
@pytest.mark.parametrize("math", [0, 1, 2])
def test_every_abi_call_is_clean_under_host_sanitizers_on_the_gpu(math):
    """Six steps with a refresh every second one on a layer of small ragged matrices (one factor's QR panels span two
    workgroups): br_init, br_accumulate_stats, br_refresh_basis, br_step and br_destroy with the host side instrumented."""
    if not os.path.exists(EXE):
        pytest.fail(f"{EXE} is missing: build it with `python -m paper_2602_03515_amd.build --sanitize` before the GPU run")
    res = subprocess.run([EXE, "--small", "--layers", "1", "--steps", "6", "--freq", "2", "--math", str(math)], env=ENV,
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "ms/step" in res.stdout and "ERROR: AddressSanitizer" not in res.stdout and "runtime error" not in res.stdout
