"""The host-side half of the C ABI (argument checks and dispatch) built with plain g++ against
stub launchers and run under AddressSanitizer and UndefinedBehaviorSanitizer.  No GPU involved."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_api_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "host_driver"
    src = [os.path.join(ROOT, "paper_2205_00119_amd", "csrc", "api.cpp"),
           os.path.join(ROOT, "tests", "host", "stub_launchers.cpp"),
           os.path.join(ROOT, "tests", "host", "driver.cpp")]
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    f"-I{os.path.join(ROOT, 'include')}", f"-I{os.path.join(ROOT, 'paper_2205_00119_amd', 'csrc')}",
                    "-o", str(exe), *src], check=True)
    # other preloaded libraries may sit in front of the sanitizer runtime; that is fine
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1")
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "host checks ok" in res.stdout
