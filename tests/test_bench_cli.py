"""Host-side behaviour of bench.py that needs no GPU: more than one GPU is refused with a
message, and the byte accounting of a decode step matches the sizes the roofline is priced on."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_decode_step_byte_accounting():
    sys.path.insert(0, ROOT)
    import bench
    B, V, C = 256, 128256, 8000
    nb = bench.decode_step_bytes(B, V, C)
    wv, wc = (V + 31) // 32, (C + 31) // 32
    # logits read and written, class bits read, class ids read once, token bits written
    assert nb["mask_kernel"] == 2 * B * V * 2 + B * wc * 4 + V * 4 + B * wv * 4
    assert nb["step"] >= nb["mask_kernel"] and nb["step"] - nb["mask_kernel"] < 64 * 1024
    assert nb["mask_kernel"] == 136207360
