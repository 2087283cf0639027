"""CPU-only checks of the boundary: the library loads, exports every symbol the public header declares, and its
host-side validation rejects bad arguments without touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2605_08862_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2605_08862_amd import build
        build.build()
    return B.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "bubblespec.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(bs_[a-z_]+)\s*\(", header))
    assert declared >= {"bs_draft_lookup", "bs_verify_step", "bs_accept_resample", "bs_kv_commit"}
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)


def test_workspace_query_and_shape_validation(lib):
    ok = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=1024, vocab=4096, dtype=B.BS_F32)
    assert B.bs_workspace_bytes(B.make_desc(ok), 4, 4) > 0
    for bad in (dict(ok, head_dim=96), dict(ok, d_model=100), dict(ok, n_q_heads=5, n_kv_heads=2),
                dict(ok, dtype=7), dict(ok, vocab=1)):
        assert B.bs_workspace_bytes(B.make_desc(bad), 4, 4) == 0
    assert B.bs_workspace_bytes(B.make_desc(ok), 0, 4) == 0
    assert B.bs_workspace_bytes(B.make_desc(dict(ok, d_model=16384)), 4, 4) > 0
    assert B.bs_workspace_bytes(B.make_desc(dict(ok, d_model=16384 + 64)), 4, 4) == 0     # row kept in registers
    assert B.bs_workspace_bytes(B.make_desc(ok), 4, B.BS_MAX_K + 1) == 0
    big = dict(n_layers=28, d_model=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, d_ffn=18944, vocab=152064,
               dtype=B.BS_BF16)
    assert B.bs_workspace_bytes(B.make_desc(big), 128, 16) > 14e9          # holds the packed weights
    assert B.bs_workspace_bytes(B.make_desc(big), 128, 20) == 0            # 21 * 7 query rows > 128 per KV head


def test_null_arguments_are_rejected(lib):
    out = C.c_void_p()
    assert lib.bs_create(None, None, None, None, 0, 1, 1, None, C.byref(out)) == B.BS_EINVAL
    assert lib.bs_verify_step(None, 1, None, None, None, None, 0, None, None) == B.BS_EINVAL
    assert lib.bs_kv_commit(None, 1, None, None, None) == B.BS_EINVAL
    assert lib.bs_draft_lookup(None, 1, None, None, 4, 1, 4, None, None, None) == B.BS_EINVAL
    assert lib.bs_set_filter(None, 5, 0.9, None) == B.BS_EINVAL
    assert lib.bs_last_error(None) == b"null context"


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_bench_setup_guard_stops_on_non_finite_logits():
    """bench.py feeds the library's logits to torch.multinomial during set-up; a non-finite value must end the program
    on the host (SystemExit naming the step) before it reaches that device-asserting op.  Stub tensors, no GPU."""
    import torch
    import bench
    bench.check_finite(torch.zeros(3, 5), "stub")
    for bad in (float("inf"), float("-inf"), float("nan")):
        z = torch.zeros(3, 5)
        z[1, 2] = bad
        with pytest.raises(SystemExit) as e:
            bench.check_finite(z, "set-up decode step 4 of stub")
        assert "set-up decode step 4" in str(e.value) and e.value.code != 0
