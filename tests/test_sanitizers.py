"""The CPU checker and the library's host builder under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU): random
corpora with clones, save / load, top-k, tree drafts and the worked example, the
two implementations compared with each other along the way."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
         "-g", "-O1"]


def _have_sanitizer_runtime(tmp_path):
    src = tmp_path / "probe.c"
    src.write_text("int main(void){return 0;}\n")
    exe = tmp_path / "probe"
    p = subprocess.run(["gcc"] + FLAGS + [str(src), "-o", str(exe)], capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0")
    return p.returncode == 0 and subprocess.run([str(exe)], env=env).returncode == 0


def test_oracle_and_host_builder_under_asan_ubsan(tmp_path):
    if not (shutil.which("gcc") and shutil.which("g++")):
        pytest.skip("gcc / g++ not available")
    if not _have_sanitizer_runtime(tmp_path):
        pytest.skip("the sanitizer runtime (libasan / libubsan) is not installed")
    oracle_o = tmp_path / "sam_oracle.o"
    subprocess.check_call(["gcc", "-std=c11"] + FLAGS + ["-c", os.path.join(ROOT, "oracle", "sam_oracle.c"),
                                                          "-o", str(oracle_o)])
    exe = tmp_path / "sanitize_driver"
    subprocess.check_call(["g++", "-std=c++17", "-pthread"] + FLAGS + [
        os.path.join(ROOT, "tests", "sanitize_driver.cpp"),
        os.path.join(ROOT, "paper_2411_10666_amd", "csrc", "sam_host.cpp"),
        str(oracle_o), "-o", str(exe)])
    # (verify_asan_link_order=0: other preloaded libraries may sit in front of the runtime)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([str(exe), str(tmp_path / "corpus.sam")], capture_output=True, text=True,
                       env=env, timeout=600)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-4000:]
    assert p.stdout.strip().endswith("ok")
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr
