"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a stand-alone C program (oracle/selftest.c)
linked with the oracle runs the five self-checks of the path on small inputs."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_selftest_under_sanitizers(tmp_path):
    exe = str(tmp_path / "selftest")
    cmd = ["gcc", "-std=c11", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
           os.path.join(ROOT, "oracle", "np_oracle.c"), os.path.join(ROOT, "oracle", "selftest.c"), "-lm", "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr[-2000:])
    assert "oracle selftest ok" in r.stdout
