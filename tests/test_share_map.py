"""Host logic of the attention stream decomposition (no GPU): the share map that
both the stream pass and the merge pass rely on is checked by brute force."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_share_map_brute_force():
    src = os.path.join(ROOT, "tests", "share_map_check.cpp")
    inc = os.path.join(ROOT, "paper_2602_11530_amd", "csrc")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as d:
        exe = os.path.join(d, "share_map_check")
        subprocess.check_call([hipcc, "-O1", "--offload-arch=gfx950", "-x", "hip", "-I", inc, src,
                               "-o", exe], stderr=subprocess.DEVNULL)
        out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    assert "bad=0" in out.stdout
