"""The library's host code (planning, weight packing, scheduler, graph capture, copy paths,
measurement aids, two-party runtime, teardown) replayed on the CPU against a stand-in HIP
runtime under AddressSanitizer and UBSan: the create / run / destroy sequences of the GPU
parity suite, including all four sets of seeded random chains. No GPU, no device code."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "hipstub"))


@pytest.fixture(scope="module")
def stub_dir(tmp_path_factory):
    import build_stub
    return build_stub.build(str(tmp_path_factory.mktemp("hipstub")))


def test_host_code_is_clean_under_sanitizers(stub_dir):
    import build_stub
    env = dict(os.environ)
    pre = [build_stub.asan_runtime()] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env["LD_PRELOAD"] = ":".join(pre)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=23"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, os.path.join(HERE, "hipstub", "replay.py"), stub_dir],
                       capture_output=True, text=True, env=env, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-6000:])
    assert r.returncode == 0, tail
    assert "REPLAY OK" in r.stdout, tail
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, tail
