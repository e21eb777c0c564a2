"""The benchmark reads the HBM traffic of its roofline objects from the committed rocprofv3 summaries at run time:
every file it names must exist and carry the key, and the figure must be plausible against the algorithmic bytes."""

import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _value(fname, key="traffic_bytes_per_launch"):
    text = open(os.path.join(ROOT, "profiles", fname)).read()
    m = re.search(r"^%s\s*=\s*([0-9.eE+-]+)" % re.escape(key), text, re.M)
    assert m, "%s has no %s" % (fname, key)
    return float(m.group(1)), text


def test_bench_names_only_existing_profile_files():
    src = open(os.path.join(ROOT, "bench.py")).read()
    named = set(re.findall(r'"([A-Za-z0-9_]+\.txt)"', src))
    assert named, "bench.py names no profile summary"
    for f in named:
        assert os.path.exists(os.path.join(ROOT, "profiles", f)), f


def test_traffic_figures_against_algorithmic_bytes():
    # layer1 convolution of ResNet-18 b64: X + Y in bf16 + codes; GEMM: X + Y + codes; ternarize: 8.25 B per weight
    for fname, alg in (("resnet18_b64_forward_kernels.txt", 51389440), ("gemm_8192x4096x4096_kernels.txt", 138412032),
                       ("ternarize_2p28_hbm.txt", (1 << 28) * 8.25)):
        v, text = _value(fname)
        assert 0.9 * alg <= v <= 3.0 * alg, (fname, v, alg)
        assert "rocprofv3" in text and "bench.py" in text      # the summary states the command that made it


def test_bench_refuses_more_than_one_gpu():
    # this build runs on one GPU; asking for more ends with a message that says so (no GPU is touched before that)
    import subprocess
    import sys
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "ONE GPU" in (p.stderr + p.stdout)
