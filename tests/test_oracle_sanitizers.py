"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a
small C++ driver calls every exported function on awkward shapes with exactly sized heap
buffers.  CPU only."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_selftest")
    src = [os.path.join(ROOT, "oracle", f) for f in ("combo_ref.cpp", "selftest.cpp")]
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", exe] + src,
                   check=True)
    env = dict(os.environ)
    # other preloaded libraries may precede the sanitizer runtime; that is fine here
    env["ASAN_OPTIONS"] = "detect_leaks=1:verify_asan_link_order=0"
    out = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "oracle selftest ok" in out.stdout
