"""Host-side checks of bench.py (no GPU): the figures it derives by arithmetic, the files it names, its refusal of N > 1."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_algorithmic_bytes_of_a_decode_unit_step():
    """K and V rows of the c+1 slots, S read and written, positions, the retained list, q and o, the new rows."""
    c, d, e = 2048, 128, 2
    want = 2 * (c + 1) * d * e + 8 * (c + 1) + 4 * (c + 1) + 4 * c + (d * e + 4 * d) + 2 * d * e
    assert bench.algorithmic_bytes_per_unit(c, 1) == want == 1083148
    assert 256 * want == 277285888
    # G query heads: only q and o grow
    assert bench.algorithmic_bytes_per_unit(c, 4) - want == 3 * (d * e + 4 * d)


def test_prefill_flops_and_prompt_bytes():
    L, c, d, H = 512, 2048, 128, 32
    assert bench.prefill_flops_per_chunk(c) == 2 * 2 * L * (c + (L + 1) / 2) * d * H == 19331547136.0
    T, b = 32768, 64
    per_head = T * d * 2 + b * d * 2 + T * 4 + 2 * 2 * c * d * 2 + 2 * c * 4
    assert bench.prompt_bytes_per_call(T, c) == per_head * H == 340787200


def test_profiled_traffic_constants_name_files_that_hold_them():
    """Every traffic constant names a committed summary, and the counter readings it is built from appear there."""
    for what, t in bench.PROFILED_TRAFFIC.items():
        path = os.path.join(ROOT, t["source"])
        assert os.path.isfile(path), (what, t["source"])
        assert t["bytes"] > 0
    text = open(os.path.join(ROOT, bench.PROFILED_TRAFFIC["decode"]["source"])).read()
    m = re.search(r"decode_fused_kernel<bf16, 128, 1, false>\s+FETCH_SIZE\s+([\d.]+)\s+WRITE_SIZE\s+([\d.]+)", text)
    assert m, "the decode kernel's row is missing from the traffic summary"
    from_file = (float(m.group(1)) * 2 + float(m.group(2))) * 1024
    assert abs(from_file - bench.PROFILED_TRAFFIC["decode"]["bytes"]) / from_file < 1e-3
    # the decode kernel moves what the algorithm needs and no more
    assert 0.97 < bench.PROFILED_TRAFFIC["decode"]["bytes"] / 277285888 < 1.03


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr
