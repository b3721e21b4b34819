"""One oracle-checked parity case for every compiled instantiation of the matrix-core attention kernel.

attn_mfma_kernel<D, KS, DB, waves, SOFTCAP, PAIRS, F16, COARSE, SOFT, NOREF> is compiled for
  (D, KS, DB) in {(64,4,2) d=64, (128,5,3) d=80, (128,6,3) d=96, (128,8,4) d=128, (256,16,8) d=256}
  x waves in {4, 8 (256-row tiles: n >= 262144, or two passes from 131072; not for d = 256, not with coarse classes)}
  x SOFTCAP x PAIRS (row_pairs asked for or not) x F16 (IEEE half or bf16) x COARSE (more than 256 membership sets,
  4 wavefronts only) x NOREF (softmax without a reference / with the running reference: both are launched, the
  data decide which one does a tile), plus the soft gate (SOFT: d in {64,80,96,128}, bf16/f16; tests/test_gpu_soft_gate.py).
The kernel reads its LDS operands with loads the compiler does not track, so every binary gets its own check
against the oracle here: all rows at small n (4 wavefronts), sampled rows at 262144 + 77 tokens (8 wavefronts).
"""
import itertools

import numpy as np
import pytest
import torch

from paper_2604_03260_amd import workloads
from paper_2604_03260_amd.workloads import Workload
from tests import harness

pytestmark = pytest.mark.gpu

DIMS = [64, 80, 96, 128, 256]


def run_case(wl, pairs, big_norms, rows=None):
    inp = workloads.make_inputs(wl, "cuda")
    if big_norms:
        # every Cauchy-Schwarz bound far above 60 (and the cap of 50 is above 60 in log2 units): the work-groups
        # of the no-reference instantiation all decline, the running-reference instantiation does every tile
        inp["k"] *= 12.0
    res = harness.run_gpu(wl, inp, want_pairs=pairs, want_lse=True)
    mq, mk = harness.check_assign(wl, inp, res)
    stats = harness.check_attn(wl, inp, res, mq, mk, rows=rows)
    if pairs:
        harness.check_pair_totals(wl, res, mq, mk)
    return stats


CASES4 = list(itertools.product(DIMS, [False, True], [False, True], ["bf16", "f16"], [False, True], [True, False]))


@pytest.mark.parametrize("d,softcap,pairs,dtype,coarse,noref", CASES4,
                         ids=["d%d-%s-%s-%s-%s-%s" % (d, "cap" if sc else "nocap", "pairs" if pr else "nopairs", dt,
                                                      "coarse" if co else "exact", "noref" if nr else "runref")
                              for d, sc, pr, dt, co, nr in CASES4])
def test_four_wavefront_instantiations_all_rows(d, softcap, pairs, dtype, coarse, noref):
    K, topk = (32, 2) if coarse else (8, 2)           # C(32,2) = 496 membership sets: classes of super-groups
    wl = Workload("inst4", 91, 1, 4, 2, 700 + d, d, dtype, K, topk, 48, softcap=50.0 if softcap else 0.0,
                  mixture=8 if coarse else 0)
    run_case(wl, pairs, big_norms=not noref)


CASES8 = list(itertools.product([64, 80, 96, 128], [False, True], [False, True], ["bf16", "f16"], [True, False]))


@pytest.mark.parametrize("d,softcap,pairs,dtype,noref", CASES8,
                         ids=["d%d-%s-%s-%s-%s" % (d, "cap" if sc else "nocap", "pairs" if pr else "nopairs", dt,
                                                   "noref" if nr else "runref") for d, sc, pr, dt, nr in CASES8])
def test_eight_wavefront_instantiations_sampled_rows(d, softcap, pairs, dtype, noref):
    wl = Workload("inst8", 92, 1, 2, 1, 262144 + 77, d, dtype, 4, 2, 1500, softcap=50.0 if softcap else 0.0)
    rows = workloads.sample_rows(wl, 96)
    run_case(wl, pairs, big_norms=not noref, rows=rows)
