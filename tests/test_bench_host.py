"""Host-side logic of bench.py: the algorithmic bytes behind `roofline` follow the
paper's memory model (Sec. 4.4, Table 2), and runs on more than one GPU are refused."""
import os
import subprocess
import sys
import types

import pytest

from oracle import quant

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


@pytest.mark.parametrize("bits,group", [(2, 32), (4, 32), (1, 64), (2, 64)])
@pytest.mark.parametrize("lens", [[131072], [32768], [20000, 16384, 32768]])
def test_quant_bytes_follow_table2(bits, group, lens):
    args = types.SimpleNamespace(bits=bits, group=group)
    got = bench.quant_bytes_of(args, lens)
    want = 0.0
    for n in lens:
        nq, tail = quant.partition(n, 128, group)
        # Table 2 counts fp16 elements of one layer's K and V (8 KV heads, 128 channels) ...
        want += 2.0 * quant.table2_quant_elements(nq, 8, 128, 1, bits, group)
        want += 8 * tail * 2 * 128 * 2          # ... the fp16 tail: K and V rows of 128 fp16
        want += 2 * 32 * 128 * 2                # query in, output out (32 heads, fp16)
    assert got == want


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
