"""Host-side contract of bench.py: one GPU only, and the workload table it times is the input module's."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one MI355X" in (r.stderr + r.stdout)


def test_workload_accounting():
    sys.path.insert(0, ROOT)
    from paper_2505_18574_amd import inputs

    # ops: 2 M N K (convolution: of the implicit GEMM, padding taps included); bytes: operands once, output once
    c = inputs.GEMM_I8_SWEEP[0]
    assert c.ops == 2 * 3136 * 64 * 576 and c.bytes == 3136 * 576 + 576 * 64 + 4 * 64 + 3136 * 64
    v = inputs.CONV_I8[0]
    assert v.gemm_mnk == (8 * 56 * 56, 64, 576) and v.ops == 2 * 25088 * 64 * 576
    assert v.bytes == 8 * 56 * 56 * 64 + 576 * 64 + 4 * 64 + 25088 * 64
    g = inputs.GEMM_BF16[0]
    assert g.ops == 2 * 4096 ** 3 and g.bytes == 2 * 2 * 4096 * 4096 + 4 * 4096 * 4096
    b = inputs.BATCHED_F32
    assert b.bytes == 262144 * 1872 and b.ops == 262144 * 3756
