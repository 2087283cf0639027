"""GPU parity at full depth in a launch configuration bench.py times (BASELINE configs[1]: 1.5B shape, 28 layers, batch 64,
context 2048, k = 8, dense bf16 proposal): sampled outputs the oracle can compute one by one.

* logits of two whole sequences (9 rows x 151936 each) against the full-depth fp64 oracle, max-abs <= 2e-2, their
  appended K/V rows, and the end-to-end ids of those sequences against the oracle on its own logits (counted);
* the sampler decisions of all 64 sequences against the oracle's rule applied to the device's own logits;
* properties that hold at any size: row packing, committed lengths, emitted counts.
(The 7B-shape and pool-stress configurations are covered at their real batch sizes, on two-layer slices, in
tests/test_gpu_launch_sizes.py.)"""
import pytest

from tests import helpers as H

pytestmark = pytest.mark.gpu


def test_bench_configuration_sampled_parity():
    wl, st, _ = H.run_bench_workload_case("s1p5b_b64_c2048_k8")
    assert st["rows"] == 576 and st["sampled"] == [0, 63]
    assert wl["desc"]["n_layers"] == 28
    wl["eng"].close()
