"""The host half of the library -- CSR validation, decomposition, packing, image self-check,
export, save / load / repack, the fibre builder -- compiled as a CPU-only program with
AddressSanitizer and UndefinedBehaviorSanitizer (every report fatal) and run on skewed, directed,
grid and malformed operands under many option sets.  No GPU, no kernel: the launchers are stubs
that abort if reached."""
import os
import subprocess

from paper_2307_05740_amd import _build


def _stale(binary: str) -> bool:
    if not os.path.exists(binary):
        return True
    built = os.path.getmtime(binary)
    deps = [os.path.join(_build.PKG_DIR, s) for s in _build.HOST_SOURCES]
    deps += [os.path.join(_build.PKG_DIR, "csrc", "arrow_internal.h"),
             os.path.join(_build.REPO_DIR, "include", "arrow.h"), os.path.join(_build.REPO_DIR, "include", "csf3.h")]
    return any(os.path.getmtime(d) > built for d in deps)


def test_host_code_is_clean_under_address_and_ub_sanitizers(tmp_path):
    binary = _build.HOST_CHECK + "_asan"
    if _stale(binary):
        _build.build_host_check(sanitize=True)
    syms = subprocess.run(["nm", "-C", binary], stdout=subprocess.PIPE, text=True, check=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms        # the sanitizers really are linked in
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    proc = subprocess.run([binary, str(tmp_path / "levels.arrow")], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                          text=True, env=env, timeout=600)
    assert proc.returncode == 0 and "host_check: ok" in proc.stdout, proc.stdout[-4000:]
