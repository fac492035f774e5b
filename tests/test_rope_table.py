"""Product side of the rotary tables (CPU only, host arithmetic of libpz.so): the library's
pz_rope_yarn_table against the oracle's independent generator, its defaults and its argument checks.
The fused rotary + append kernel gets the library's table and the oracle its own (tests/test_gpu_rope.py),
so what this file bounds -- the gap between the two tables -- is what bounds the kernel's byte differences."""
import numpy as np

import oracle
import paper_2602_11937_amd as pz
from helpers import paper_values

D = 64


def test_binding_defaults_are_the_papers_factor_and_the_parents_context():
    pv = paper_values()
    prm = pz.YarnParams()
    assert prm.factor == pv["yarn_factor"] and prm.original_context == pv["yarn_original_context"]
    lc, ls = pz.pz_rope_yarn_table(prm, D, 3)
    oc, osn = oracle.yarn_table(D, 3)
    assert np.array_equal(lc, oc) and np.array_equal(ls, osn)


def test_library_table_generator_agrees_with_the_oracle():
    for factor in (1.0, 32.0, 56.0):
        oc, osn = oracle.yarn_table(D, 140000, factor=factor)
        lc, ls = pz.pz_rope_yarn_table(pz.YarnParams(factor=factor), D, 140000)
        # two independent double-precision evaluations, each rounded once to fp32: equal, or one unit in the
        # last place apart where the double values straddle a rounding boundary (|value| <= 1.41)
        assert np.max(np.abs(oc - lc)) <= 2.0 ** -23 and np.max(np.abs(osn - ls)) <= 2.0 ** -23
        same_row = np.all(oc == lc, axis=1) & np.all(osn == ls, axis=1)
        assert same_row.mean() > 0.99


def test_table_argument_checks():
    assert pz.pz_rope_yarn_table(pz.YarnParams(factor=0.5), D, 4, check=False)[0].sum() == 0
    assert pz.lib().pz_rope_yarn_table(None, 64, 4, 0, 0) == -1
