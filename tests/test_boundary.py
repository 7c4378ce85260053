"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and its host-only entry points behave as documented."""
import ctypes
import math
import os
import re
from fractions import Fraction

import pytest
import torch

from paper_2512_07090_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "tokfilt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None


def test_params_struct_matches_header_layout():
    # 6 int32, 9 int64, double, 2 int32, float, int32 with natural alignment
    assert ctypes.sizeof(B.tf_params) == 128
    assert B.tf_params.q_stride.offset == 24 and B.tf_params.prune_ratio.offset == 96
    assert B.tf_params.softmax_scale.offset == 112 and B.tf_params.anchor.offset == 116
    assert B.tf_params.ema_gamma.offset == 120 and B.tf_params.anchor_inclusive.offset == 124


def test_keep_count_host(golden_dir):
    for line in open(os.path.join(golden_dir, "keep_count_table.txt")):
        if line.strip() and not line.startswith("#"):
            n, r, m = line.split()
            assert B.tf_keep_count(int(n), float(r)) == int(m)
    for n in (1, 3, 10, 127, 4096, 32768):
        for num in range(100):
            assert B.tf_keep_count(n, num / 100.0) == math.ceil((1 - Fraction(num, 100)) * n)
    assert B.tf_keep_count(0, 0.5) == -1
    assert B.tf_keep_count(16, 1.0) == -1
    assert B.tf_keep_count(16, -0.1) == -1
    assert B.tf_keep_count(16, float("nan")) == -1


def test_workspace_bytes_and_shape_validation():
    good = B.make_params((2, 8, 300, 128), (2, 2, 300, 128), torch.bfloat16, 0.5)
    ws = B.tf_workspace_bytes(good)
    assert ws >= 2 * 2 * 2 * 300 * 4 + 2 * 300 and ws % 256 == 0

    def bad(**kw):
        p = B.make_params((2, 8, 300, 128), (2, 2, 300, 128), torch.bfloat16, 0.5)
        for k, v in kw.items():
            setattr(p, k, v)
        return B.tf_workspace_bytes(p)

    assert bad(head_dim=64) == 0
    assert bad(n_kv_heads=3) == 0
    assert bad(seq=0) == 0
    assert bad(prune_ratio=1.0) == 0
    assert bad(dtype=7) == 0
    assert bad(fusion=4) == 0
    assert bad(warmup=-1) == 0
    assert bad(anchor_inclusive=2) == 0
    assert bad(anchor=2) == 0
    assert bad(anchor=B.TF_ANCHOR_EMA, ema_gamma=1.0) == 0
    assert bad(anchor=B.TF_ANCHOR_EMA, ema_gamma=-0.1) == 0
    assert bad(anchor=B.TF_ANCHOR_EMA, ema_gamma=0.9) > 0
    p = B.make_params((2, 8, 300, 128), (2, 2, 300, 128), torch.bfloat16, 0.5)
    p.kv_stride[2] = 132                       # not a multiple of 8 elements
    assert B.tf_workspace_bytes(p) == 0


def test_status_strings():
    assert B.tf_status_string(B.TF_OK) == "ok"
    assert "workspace" in B.tf_status_string(B.TF_ERR_WORKSPACE_TOO_SMALL)
    assert B.tf_status_string(99) == "unknown status"


def test_product_path_has_no_oracle_dependency():
    # the package must never reach into the test oracle
    pkg = os.path.join(ROOT, "paper_2512_07090_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src
                assert "tokfilt_oracle" not in src


def test_tail_schedule_host_matches_oracle():
    import oracle
    for L, pg, y in ((32, 0.25, 0.5), (40, 0.33, 0.4), (40, 0.33, 0.6), (10, 0.3, 0.25), (7, 0.9, 0.5),
                     (1, 0.5, 1.0)):
        ratios, n_tail = B.tf_tail_schedule(L, pg, y)
        ref, n_ref = oracle.tail_schedule(L, pg, y)
        assert n_tail == n_ref and ratios == list(ref)
    for bad in ((0, 0.2, 0.5), (4, -0.1, 0.5), (4, 0.2, 0.0), (4, 0.2, 1.5)):
        with pytest.raises(B.TokfiltError):
            B.tf_tail_schedule(*bad)


def test_bench_reads_the_traffic_of_every_committed_counter_summary():
    """bench.py takes `roofline.traffic` from the counter summaries under profiles/: every
    workload's attention and scoring summary must hold a figure it can read."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    import bench
    from paper_2512_07090_amd import synth
    for w in synth.WORKLOADS:
        att = "attend_f32" if w.dtype == "f32" else "attend_bf16"
        for name in ("%s_%s_pmc.txt" % (att, w.name), "scan_score_%s_pmc.txt" % w.name):
            value, source = bench.read_traffic(name)
            assert value is not None and value > 1e5, name
            assert source == "profiles/" + name
