"""GPU parity at the launch sizes of the 7B-shape and pool-stress configurations.

The launchers pick kernel instantiations by the row limit M_max = B (k_max + 1) and the shape (row tiling of the
MFMA GEMMs, K splits, 96- or 192-row SwiGLU tiles, LM-head row tiling, query blocks and token chunks of the
attention work list), so a variant is only checked if a test runs at the batch that selects it.  Each case here is a
two-layer slice of the real per-layer shape with the full vocabulary at the REAL batch of the configuration, built
by the same workload builder bench.py times:

  * configuration 3: 7B shape, B = 32, context 8192, k = 8 (288 rows)
  * configuration 4: 7B shape, B = 128, lognormal contexts 512..32768, k_b ~ U{0..16} (row limit 2176)
  * Tab. 1 of the paper: 7B heads, B = 128, context 8192, 32 sequences with 4 drafts and 96 plain decodes
  * configuration 5: 1.5B shape, B = 256, context 16384, drafts from bs_draft_lookup on the device (row limit 4352)

Checked: Tier A (the oracle's rule on the device's own logits) on ALL sequences; Tier B (logits against the fp64
oracle, max-abs 2e-2) on sampled sequences: shortest context, longest context, a plain (k = 0) one, a full-length one;
Tier C (device ids against the oracle on its own logits) counted on those; and the properties that hold at any size
(row packing, accepted prefix = draft prefix, emitted counts, committed lengths, status word)."""
import numpy as np
import pytest

from oracle.lookup import lookup as oracle_lookup
from tests import helpers as H

pytestmark = pytest.mark.gpu
_run = lambda name: H.run_bench_workload_case(name, layers=2)


def test_config3_7b_batch32_context8192():
    wl, st, _ = _run("s7b_b32_c8192_k8")
    assert st["rows"] == 288
    wl["eng"].close()


def test_config4_7b_longtail_batch128():
    wl, st, _ = _run("s7b_longtail_b128_k0to16")
    assert st["row_limit"] == 2176 and 800 <= st["rows"] <= 1500
    assert max(st["contexts"]) > 20000 and min(st["contexts"]) <= 600         # the long tail is really in the batch
    wl["eng"].close()


def test_table1_mixed_batch_7b_heads():
    """The batch of the paper's Tab. 1: 128 requests at context 8192, 32 of them verifying 4 drafts."""
    wl, st, (_, k_b) = _run("s7b_tab1_b128_c8192")
    assert (k_b == 4).sum() == 32 and (k_b == 0).sum() == 96
    wl["eng"].close()


def test_config5_pool_stress_batch256():
    """Drafts come from bs_draft_lookup on the device (prebuilt index) and go into bs_verify_step with no host round
    trip.  The lookup is checked bit for bit against the brute-force oracle on sampled sequences and, for every
    sequence, against the pool itself (a draft must continue an occurrence of the matched context)."""
    wl, st, (drafts, k_b) = _run("s1p5b_pool_b256_c16384")
    assert st["sequences"] == 256 and st["row_limit"] == 4352
    toks, off, prb = wl["pool"]
    seq_prompt, tails = wl["seq_prompt_host"], wl["tails_host"]
    assert (k_b > 0).sum() >= 150 and (k_b == 0).sum() >= 10               # drafted and plain sequences in one launch
    for b in list(range(0, 256, 16)) + st["sampled"]:
        p = seq_prompt[b]
        ref = oracle_lookup([toks[off[r]:off[r + 1]] for r in range(prb[p], prb[p + 1])], tails[b], 4, 1, 16)
        assert k_b[b] == len(ref) and list(drafts[b][:k_b[b]]) == ref, (b, drafts[b], ref)
        assert (drafts[b][k_b[b]:] == -1).all()
    for b in range(256):                                                   # any size: the draft continues a pool match
        if k_b[b] == 0:
            continue
        p = seq_prompt[b]
        seg = toks[off[prb[p]]:off[prb[p + 1]]]
        pat = np.concatenate([tails[b][-1:], drafts[b][:k_b[b]]])
        hit = np.flatnonzero(seg[:len(seg) - len(pat) + 1] == pat[0])
        ok = any((seg[h:h + len(pat)] == pat).all() for h in hit)
        assert ok, b
    wl["eng"].close()
