"""An interrupted sweep continued with pahq_acdc_sweep_resume reaches what the uninterrupted sweep reaches.

The pruning rule (paper, Appendix "Preliminaries"; Appendix "Integration with ACDC") decides receiver by receiver
in descending order, each decision given all earlier ones: after any receiver the state of the sweep is the removed
set alone.  So the sweep over the upper receivers, its removed set carried to a NEW model, and a resumed sweep there
over the rest must give the uninterrupted sweep's decisions one for one (the uninterrupted sweep itself is held to
the oracle's elsewhere).
"""
import os
import sys
import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "golden"))
sys.path.insert(0, os.path.dirname(__file__))
import workloads                                    # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,tau", [("mid_hi", 1e-3), ("mid_hi", 2e-2), ("cfg1_hi", 1e-3), ("midllama_hi", 5e-3)])
def test_resumed_sweep_equals_uninterrupted(name, tau):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    a = P.Model(shape, w, B, S, max_batch_edges=8)
    b = None
    try:
        a.clean_cache(clean, corrupt)
        n_recv = P.n_receivers(a.cfg)
        kept_full, n_full, tr_full = a.acdc_sweep(tau)
        assert 0 < kept_full.sum() < kept_full.size or n_full > 0
        for cut in (n_recv - 1, n_recv // 2, 1):                      # after the output node only / half way / all but receiver 0
            upper = np.arange(cut, n_recv, dtype=np.int32)
            lower = np.arange(0, cut, dtype=np.int32)
            kept1, n1, tr1 = a.acdc_sweep(tau, receivers=upper)
            state = a.get_removed()
            assert np.array_equal(state, 1 - kept1)
            b = P.Model(shape, w, B, S, max_batch_edges=8)
            b.clean_cache(clean, corrupt)
            b.set_removed(state)
            kept2, n2, tr2 = b.acdc_sweep(tau, receivers=lower, resume=True)
            assert n1 + n2 == n_full, (name, tau, cut)
            assert np.array_equal(kept2, kept_full), (name, tau, cut)
            assert tr1.tobytes() + tr2.tobytes() == tr_full.tobytes(), (name, tau, cut)
            # a receiver that is already decided cannot be named again, and a failed call changes nothing
            if state.any():
                touched = [r for r in upper if a_row_has_removed(P, a.cfg, state, int(r))]
                if touched:
                    with pytest.raises(P.PahqError):
                        b.acdc_sweep(tau, receivers=np.array(touched[:1], np.int32), resume=True)
                    assert np.array_equal(b.get_removed(), 1 - kept2)
            b.close(); b = None
    finally:
        a.close()
        if b is not None:
            b.close()


def a_row_has_removed(P, cfg, removed, r):
    e0 = P.edge_id(cfg, 0, r)          # a receiver's in-edges are consecutive in the canonical order
    return bool(removed[e0: e0 + P.n_upstream(cfg, r)].any())
