"""The library's host code under AddressSanitizer and UBSan, without a GPU: the layout transforms between canonical
bytes and device records (every weight width and exponent form, ragged sizes, ranks to 256), the C ABI's argument
checks, and the offline step's host arithmetic for every number format.  Also the same layout self test in the
normal build."""
import os
import subprocess

from paper_2402_02446_amd import binding, build


def test_layout_self_test_in_the_normal_build():
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    assert binding.lib().lqer_selftest_layouts() == 0


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    kern = os.path.join(build.BUILD, "kernels_tiled.o")
    if not os.path.exists(kern):
        build.build(verbose=False)
    exe = build.build_host_asan()
    res = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "host self test ok" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
