"""The synthetic workloads land on the block densities the benchmark's configurations name.

CPU only: the oracle's pattern generation on the full head / batch mean of every workload, i.e. on
the very map the benchmark and the GPU parity tests use.
"""
import numpy as np
import pytest

import oracle
import spion_inputs as si


@pytest.mark.parametrize("name", [w.name for w in si.WORKLOADS])
def test_achieved_density_matches_the_configuration(name):
    w = si.workload(name)
    Q, K, _, _ = si.make_qkv_do(w)
    A = si.make_score_map(w, Q, K)
    ref = oracle.generate_pattern(A, w.block, w.filt, w.thresh_mode, w.thresh_value)
    assert ref["nnzb"] == si.EXPECTED_NNZB[name]
    dens = ref["nnzb"] / float(w.nb * w.nb)
    if name in si.TARGET_DENSITY:
        assert abs(dens - si.TARGET_DENSITY[name]) <= 0.005, dens


def test_configuration_5_spans_sparse_to_dense_layers():
    dens = [si.EXPECTED_NNZB["cfg5_layer%d" % l] / 4096.0 for l in range(4)]
    assert dens == sorted(dens)
    assert 0.035 <= dens[0] <= 0.045 and dens[3] >= 0.20
    # the fill cannot keep more than the cells its walks reach, whatever the threshold: that share
    # bounds layer 3 below the 25 % the configuration names
    w = si.workload(5, 3)
    Q, K, _, _ = si.make_qkv_do(w)
    ps = oracle.pool_sum(oracle.conv_diag(oracle.quantize(si.make_score_map(w, Q, K)), w.filt), w.block)
    reach = oracle.fill(ps, oracle.make_thresh_int(int(ps.min()) - 1)).sum() / 4096.0
    assert dens[3] <= reach < 0.25


def test_one_minus_target_variant_is_the_sparser_one():
    for name, q in si.Q_ONE_MINUS_TARGET.items():
        w = si.workload(name, variant="one_minus_target")
        assert w.thresh_value == q and q > si.workload(name).thresh_value
        assert w.seed == si.workload(name).seed
