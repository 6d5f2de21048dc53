"""The seeded workloads keep the contract the kernels and the oracle assume (Section 2.1: a token names its top-k
experts; the readings: distinct experts per token, -1 = masked), and the generators are reproducible."""
import numpy as np
import pytest

import ep_inputs as g


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_every_workload_has_valid_routing(cid):
    cfg = g.config(cid)
    T = min(cfg.T, 512)
    idx, w = g.routing_all(cfg, T)
    assert idx.shape == (cfg.S, T, cfg.K) and w.shape == (cfg.S, T, cfg.K)
    g.validate_routing(idx, cfg.E)
    assert np.allclose(w.sum(axis=-1), 1.0, atol=1e-5)          # gate weights renormalised over the k chosen
    masked = g.mask_random(idx, 0.3, seed=cid)
    g.validate_routing(masked, cfg.E)
    assert (masked == -1).any() and ((masked == idx) | (masked == -1)).all()
    again, w2 = g.routing_all(cfg, T)
    assert np.array_equal(idx, again) and np.array_equal(w, w2)  # counter-based: the same call gives the same table


def test_validator_rejects_what_the_kernels_do_not_accept():
    ok = np.array([[[0, 3], [2, -1]]], dtype=np.int32)
    g.validate_routing(ok, 4)
    with pytest.raises(ValueError):
        g.validate_routing(ok.astype(np.int64), 4)
    with pytest.raises(ValueError):
        g.validate_routing(np.array([[[0, 4]]], dtype=np.int32), 4)
    with pytest.raises(ValueError):
        g.validate_routing(np.array([[[-2, 1]]], dtype=np.int32), 4)
    with pytest.raises(ValueError):
        g.validate_routing(np.array([[[1, 1]]], dtype=np.int32), 4)
    g.validate_routing(np.array([[[-1, -1]]], dtype=np.int32), 4)   # two masked entries are not a duplicate


def test_zipf_workload_is_as_skewed_as_the_design_notes_say():
    cfg = g.config(4, S=1)
    idx, _ = g.routing_all(cfg)
    counts = np.bincount(idx.ravel(), minlength=cfg.E)
    assert counts.sum() == cfg.T * cfg.K
    assert counts.max() > 0.9 * cfg.T and (counts == 0).sum() >= 1
