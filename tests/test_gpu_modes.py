"""GPU parity of the two precision modes next to PAHQ's per-edge evaluation:

* PAHQ_ALL_FP32 (no quantiser anywhere; the unaccelerated ACDC of the paper's runtime table): with no
  rounding to the e4m3 grid there is no code that can move, so device (binary32) and oracle (fp64)
  agree to rounding: logits and every cached sender output element by element, per-edge KL to
  2e-6 + 2e-5 |KL|, and whole sweeps decision by decision.  This is the test of attention, norms, GELU /
  SwiGLU, rotary positions, patching, gathering and the KL reduction that e4m3 code moves cannot blur.
* pahq_eval_circuit: the pruned graph under a SET of fp32 heads (Appendix "Integration with ACDC", last
  block of the algorithm) against oracle.Model.forward(pi = that set, removed, C)."""
import os
import sys
import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "golden"))
import workloads                                    # noqa: E402
from oracle.model import Model as OModel, ALL       # noqa: E402
from oracle.acdc import Acdc, MODE_ALL_FP32, MODE_PAHQ   # noqa: E402
from plain_forward import plain_forward             # noqa: E402
from fp32_spread import SpreadModel, circuit_kl_with_spread   # noqa: E402
from tolerance import check_kl_cases                # noqa: E402

pytestmark = pytest.mark.gpu

F32_ATOL, F32_RTOL = 2e-6, 2e-5        # binary32 against fp64 with nothing quantised (measured: below 0.4 of it)
NAMES = ["cfg1_hi", "mid_hi", "mid_hi2", "midllama_hi", "midllama_hi2"]


def rnd_removed(g, frac, seed, from_receiver=0):
    rng = np.random.default_rng(seed)
    R = g.empty_removed()
    for r in range(from_receiver, g.n_receivers):
        R[r, : g.n_upstream(r)] = rng.random(g.n_upstream(r)) < frac
    return R


@pytest.mark.parametrize("name", NAMES)
def test_all_fp32_mode(name):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    om = OModel(shape, w)
    g = om.g
    gm = P.Model(shape, w, B, S, precision=P.ALL_FP32, max_batch_edges=16)
    try:
        gm.clean_cache(clean, corrupt)
        # logits against a textbook forward that shares nothing with the oracle, element by element
        for which, tok in ((0, clean), (1, corrupt)):
            ref = plain_forward(shape, w, tok)
            got = gm.get_logits(which).astype(np.float64)
            assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max(), (name, which)
        # every cached sender output, element by element
        oc, _ = om.forward(clean, ALL)
        for s in range(g.n_senders):
            a = gm.get_sender_output(0, s).astype(np.float64)
            b = oc[s].reshape(a.shape)
            assert np.abs(a - b).max() <= 1e-4 * np.abs(b).max(), (name, s)
        # per-edge KL and the state's own KL, empty removed set and sweep-like states
        oa = Acdc(om, clean, corrupt, MODE_ALL_FP32)
        for frac in (0.0, 0.5):
            for r in range(g.n_receivers - 1, -1, -max(1, g.n_receivers // 8)):
                R = rnd_removed(g, frac, 100 + r, r) if frac else g.empty_removed()
                gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
                got = gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32))
                pairs = [(gm.eval_current(r), oa.kl_fast(r, R))] + [(got[u], oa.kl_edge(r, u, removed=R)) for u in range(g.n_upstream(r))]
                for gv, wv in pairs:
                    assert abs(gv - wv) <= F32_ATOL + F32_RTOL * abs(wv), (name, frac, r, gv, wv)
        gm.set_removed(np.zeros(g.n_edges(), np.uint8))
        # the sweep, decision by decision: a decision may differ only where the increment is within the
        # bound of tau (then every later state differs and the comparison stops)
        for tau in (1e-3, 3e-2):
            kept, n_evals, tr = gm.acdc_sweep(tau)
            o_removed, o_tr = oa.sweep(tau)
            equal = True
            for i in range(min(n_evals, len(o_tr))):
                ov, ou, okn, okc, orm = o_tr[i]
                t = tr[i]
                assert (t["receiver"], t["sender"]) == (ov, ou)
                assert abs(t["kl_new"] - okn) <= F32_ATOL + F32_RTOL * abs(okn)
                if bool(t["removed"]) != orm:
                    assert abs((okn - okc) - tau) <= 2 * (F32_ATOL + F32_RTOL * max(abs(okn), abs(okc))), (name, tau, i)
                    equal = False
                    break
            if equal:
                assert n_evals == len(o_tr)
                assert (kept == (~g.removed_to_flat(o_removed)).astype(np.uint8)).all()
                assert 0 < kept.sum() < g.n_edges()          # a circuit: some edges kept, some removed
            print(name, "all-fp32 sweep tau", tau, "equal" if equal else "diverged inside the bound", "kept", int(kept.sum()))
    finally:
        gm.close()


def test_all_fp32_clean_patch_is_exactly_zero():
    import paper_2510_23264_amd as P
    shape, w, clean, _ = workloads.make("mid_hi")
    B, S = clean.shape
    gm = P.Model(shape, w, B, S, precision=P.ALL_FP32, max_batch_edges=8)
    try:
        gm.clean_cache(clean, clean.copy())
        g = OModel(shape, w).g
        for r in (g.OUT, g.mlpin(1), g.headin(2, 1, 0)):
            gm.set_removed(g.removed_to_flat(rnd_removed(g, 0.5, 3, r)).astype(np.uint8))
            # every node computed: the clean run's own bits.  Dead nodes left out: their cached outputs enter
            # the stream's sums at another place, so the logits agree to rounding instead of bit for bit
            for skipping, limit in ((False, 0.0), (True, 1e-7)):
                gm.set_dead_node_skipping(skipping)
                assert (np.abs(gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32))) <= limit).all(), skipping
                assert abs(gm.eval_current(r)) <= limit, skipping
    finally:
        gm.close()


def head_sets(g, L, H, R):
    """(label, [L][H] flags or None for the library's own choice, the flags the oracle uses)."""
    z = lambda: np.zeros((L, H), np.uint8)
    one = z(); one[L - 1, 1 % H] = 1
    some = z(); some[0, 0] = some[L - 1, H - 1] = some[min(1, L - 1), 1 % H] = 1
    layer = z(); layer[min(1, L - 1), :] = 1
    full = z(); full[:] = 1
    derived = z()            # every head with a kept edge in and a kept edge out
    for l in range(L):
        for h in range(H):
            inn = any((~R[g.headin(l, h, c), : g.n_upstream(g.headin(l, h, c))]).any() for c in range(3))
            out = any(not R[r, g.head(l, h)] for r in g.receivers_downstream_of(g.head(l, h)))
            derived[l, h] = inn and out
    return [("none", z(), z()), ("one", one, one), ("several", some, some), ("a whole layer", layer, layer),
            ("all", full, full), ("derived", None, derived)]


@pytest.mark.parametrize("name", NAMES)
def test_eval_circuit_with_sets_of_fp32_heads(name):
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    om = SpreadModel(shape, w)
    g = om.g
    L, H = shape.n_layers, shape.n_heads
    gm = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=8)
    try:
        gm.clean_cache(clean, corrupt)
        assert gm.eval_circuit() == 0.0                       # nothing removed, no fp32 head: the cached clean run itself
        got, want, sigma = [], [], []
        for frac, seed in ((0.4, 7), (0.8, 8)):
            R = rnd_removed(g, frac, seed)                    # any removed set: the pass starts at the embedding
            kept = (~g.removed_to_flat(R)).astype(np.uint8)
            for label, flags, oracle_flags in head_sets(g, L, H, R):
                pi = frozenset((l, h) for l in range(L) for h in range(H) if oracle_flags[l, h])
                kl, logits = gm.eval_circuit(kept=kept, f32_heads=flags, want_logits=True)
                o_kl, o_logits, s = circuit_kl_with_spread(om, clean, corrupt, pi, R)
                got.append(kl); want.append(o_kl); sigma.append(s)
                # the logits of the pruned run: rounding-level agreement unless a code moved (then a
                # few per cent on single elements); a wrong head set or a wrong edge is far outside
                assert np.abs(logits - o_logits).max() <= 0.1 * np.abs(o_logits).max(), (name, frac, label)
        check_kl_cases(got, want, sigma, what=name + " circuit")
        # same edges, different head sets: the sets are seen (the values differ from each other)
        assert len({round(float(v), 9) for v in want[:5]}) >= 4
        assert (gm.get_removed() == 0).all()                  # the model's own removed set is untouched
        # the per-edge path still works afterwards (the head state is rebuilt)
        oa = Acdc(om, clean, corrupt, MODE_PAHQ)
        r = g.headin(L - 1, 0, 1)
        x = gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32))
        check_kl_cases(x, [oa.kl_edge(r, u) for u in range(g.n_upstream(r))], np.zeros(len(x)) + max(sigma), what=name + " after")
    finally:
        gm.close()


@pytest.mark.parametrize("name", ["cfg1_hi", "mid_hi", "midllama_hi"])
def test_logit_difference_metric(name):
    """The task metric of the paper's Appendix "Task Metrics" (logit of the answer minus logit of a distractor, as
    a drop below the clean reference) in place of the KL: per-edge values and states under PAHQ precision against
    the oracle (binding bound), exactly 0 for identical prompts, and in the all-fp32 mode to rounding, with sweeps
    that decide on it equal to the oracle's decision by decision."""
    import paper_2510_23264_amd as P
    import synth
    from oracle.acdc import METRIC_LOGIT_DIFF
    from fp32_spread import kl_with_spread
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    ans, dis = synth.make_answers(shape.vocab, B, "uniform", 77)
    om = SpreadModel(shape, w)
    g = om.g
    margs = dict(metric=METRIC_LOGIT_DIFF, answer=ans, distractor=dis)
    # ---- PAHQ precision
    gm = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=16)
    try:
        gm.set_metric(P.METRIC_LOGIT_DIFF, ans, dis)
        with pytest.raises(P.PahqError) as e:
            gm.eval_current(g.OUT)                           # the caches were dropped with the metric
        assert e.value.code == -2
        gm.clean_cache(clean, corrupt)
        cases = []
        for frac in (0.0, 0.5):
            for r in range(g.n_receivers - 1, -1, -max(1, g.n_receivers // 8)):
                R = rnd_removed(g, frac, 100 + r, r) if frac else g.empty_removed()
                cases.append((r, R, list(range(g.n_upstream(r)))))
        res = kl_with_spread(om, clean, corrupt, MODE_PAHQ, cases, seeds=6, **margs)
        got, want, sigma = [], [], []
        for (r, R, senders), o in zip(cases, res):
            gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
            vals = gm.eval_edges(r, np.array(senders, np.int32))
            got += [gm.eval_current(r)] + list(vals)
            want += [o["kl_current"]] + o["kl_new"]
            sigma += [o["sigma_current"]] + o["sigma_new"]
        worst = check_kl_cases(got, want, sigma, what=name + " logit difference")
        assert np.median(np.abs(want)) > 1e-3                # the values are large enough for the bound to bind
        print(name, "logit difference: median |value| %.3g, worst |d| / bound %.3f" % (np.median(np.abs(want)), worst))
        # its value for a pruned graph equals the one assembled from the oracle's logits
        kept = (~g.removed_to_flat(rnd_removed(g, 0.5, 5))).astype(np.uint8)
        gm.set_removed(np.zeros(g.n_edges(), np.uint8))
        v, lg = gm.eval_circuit(kept=kept, f32_heads=np.zeros((shape.n_layers, shape.n_heads), np.uint8), want_logits=True)
        ref = gm.get_logits(0)
        b = np.arange(B)
        assert abs(v - np.mean((ref[b, ans] - ref[b, dis]) - (lg[b, ans] - lg[b, dis]))) < 1e-5
        # identical prompts: exactly 0
        gm.clean_cache(clean, clean.copy())
        gm.set_removed(g.removed_to_flat(rnd_removed(g, 0.5, 3, g.mlpin(0) if shape.d_mlp else 3)).astype(np.uint8))
        r0 = g.mlpin(0) if shape.d_mlp else 3
        gm.set_dead_node_skipping(False)                      # every node computed: bit for bit the clean run
        assert (gm.eval_edges(r0, np.arange(g.n_upstream(r0), dtype=np.int32)) == 0.0).all() and gm.eval_current(r0) == 0.0
        gm.set_dead_node_skipping(True)
        # back to the KL: again a change of metric, again the caches go
        gm.set_metric(P.METRIC_KL)
        gm.clean_cache(clean, corrupt)
        gm.set_removed(np.zeros(g.n_edges(), np.uint8))
        oa_kl = Acdc(om, clean, corrupt, MODE_PAHQ)
        x = gm.eval_edges(g.OUT, np.arange(g.n_senders, dtype=np.int32))
        check_kl_cases(x, [oa_kl.kl_edge(g.OUT, u) for u in range(g.n_senders)], np.zeros(g.n_senders) + max(sigma), what="kl again")
    finally:
        gm.close()
    # ---- all-fp32: rounding-level agreement and equal sweeps
    gm = P.Model(shape, w, B, S, precision=P.ALL_FP32, max_batch_edges=16)
    try:
        gm.set_metric(P.METRIC_LOGIT_DIFF, ans, dis)
        gm.clean_cache(clean, corrupt)
        oa = Acdc(om, clean, corrupt, MODE_ALL_FP32, **margs)
        for r in (g.OUT, g.n_receivers // 2, 1):
            vals = gm.eval_edges(r, np.arange(g.n_upstream(r), dtype=np.int32))
            for u in range(g.n_upstream(r)):
                wv = oa.kl_edge(r, u)
                assert abs(vals[u] - wv) <= F32_ATOL + F32_RTOL * abs(wv), (name, r, u, vals[u], wv)
        for tau in (1e-2, 1e-1):
            kept, n_evals, tr = gm.acdc_sweep(tau)
            o_removed, o_tr = oa.sweep(tau)
            assert n_evals == len(o_tr) and all(bool(t["removed"]) == o[4] for t, o in zip(tr, o_tr)), (name, tau)
            assert (kept == (~g.removed_to_flat(o_removed)).astype(np.uint8)).all()
            print(name, "logit-difference sweep, all-fp32, tau", tau, "equal; kept", int(kept.sum()))
    finally:
        gm.close()


def test_threshold_grid_on_one_set_of_caches():
    """pahq_acdc_sweep_grid over the paper's 21-value threshold grid (scaled to the workload's KL range): every
    row equals the single sweep at that threshold, no cache pass is repeated, and in the all-fp32 mode every
    row equals the oracle's sweep (kept sets shrink as the threshold grows)."""
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make("cfg1_hi")
    B, S = clean.shape
    grid = P.tau_grid()
    assert grid.size == 21 and abs(grid[0] - 1e-3) < 1e-9 and abs(grid[-1] - 3.1623) < 1e-3
    om = OModel(shape, w)
    g = om.g
    for precision, mode in ((P.ALL_FP32, MODE_ALL_FP32), (P.PAHQ, MODE_PAHQ)):
        gm = P.Model(shape, w, B, S, precision=precision, max_batch_edges=16)
        try:
            gm.clean_cache(clean, corrupt)
            passes0 = gm.counters()[2]
            kept, n_evals = gm.acdc_sweep_grid(grid)
            sizes = kept.sum(axis=1)
            assert (np.diff(sizes.astype(int)) <= 0).all() and sizes[0] > sizes[-1]
            for i in (0, 7, 14, 20):
                k1, n1, _ = gm.acdc_sweep(float(grid[i]))
                assert n1 == n_evals[i] and (k1 == kept[i]).all()
            if precision == P.ALL_FP32:
                oa = Acdc(om, clean, corrupt, mode)
                for i in range(0, 21, 2):
                    o_removed, o_tr = oa.sweep(float(grid[i]))
                    assert len(o_tr) == n_evals[i] and (kept[i] == (~g.removed_to_flat(o_removed)).astype(np.uint8)).all(), i
        finally:
            gm.close()


@pytest.mark.parametrize("name", ["cfg1_hi", "mid_hi"])
def test_sender_side_precision_policy(name):
    """Eq. P_t as printed (fp32 for the source head of the evaluated edge) on the device against the oracle's
    pair_sender_policy / sweep_sender_policy: per-candidate (current, new) pairs under sweep-like states, and a
    whole sweep; and the two policies do give different numbers for the same edge."""
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt = workloads.make(name)
    B, S = clean.shape
    om = SpreadModel(shape, w)
    g = om.g
    gm = P.Model(shape, w, B, S, precision=P.PAHQ, max_batch_edges=8)
    try:
        gm.clean_cache(clean, corrupt)
        got, want, sigma = [], [], []
        for r, frac in ((g.OUT, 0.0), (g.n_receivers - 3, 0.5), (g.n_receivers // 2, 0.3)):
            R = rnd_removed(g, frac, 50 + r, r) if frac else g.empty_removed()
            gm.set_removed(g.removed_to_flat(R).astype(np.uint8))
            senders = list(range(g.n_upstream(r)))[:: max(1, g.n_upstream(r) // 6)]
            new, cur = gm.eval_edges_sender_policy(r, senders)
            base, devs = [], []
            for seed in range(5):                                  # the oracle's pairs and their binary32 spread
                om.set_spread(0.0 if seed == 0 else 2.0 ** -22, 1000 + seed)
                oa = Acdc(om, clean, corrupt, MODE_PAHQ)
                vals = [oa.pair_sender_policy(r, u, R) for u in senders]
                if seed == 0:
                    base = vals
                else:
                    devs.append([(c - b[0], n - b[1]) for (c, n), b in zip(vals, base)])
            om.set_spread(0.0, 0)
            sg = np.sqrt(np.mean(np.square(np.array(devs)), axis=0))          # [sender][cur|new]
            for k in range(len(senders)):
                got += [cur[k], new[k]]; want += [base[k][0], base[k][1]]; sigma += [sg[k][0], sg[k][1]]
        check_kl_cases(got, want, sigma, what=name + " sender policy")
        gm.set_removed(np.zeros(g.n_edges(), np.uint8))
        # the other policy gives other numbers for an edge out of a head
        r = g.headin(shape.n_layers - 1, 0, 1)
        u = g.head(0, 1)
        assert gm.eval_edges_sender_policy(r, [u])[0][0] != gm.eval_edges(r, [u])[0]
        # a sweep under it, decision by decision (a differing decision only inside the bound, as elsewhere)
        oa = Acdc(om, clean, corrupt, MODE_PAHQ)
        recv = [g.OUT, g.n_receivers - 2, g.n_receivers - 5]
        tau = 0.03
        kept, n_evals, tr = gm.acdc_sweep(tau, receivers=recv, sender_policy=True)
        o_removed, o_tr = oa.sweep_sender_policy(tau, receivers=recv)
        equal = True
        for i in range(min(n_evals, len(o_tr))):
            ov, ou, okn, okc, orm = o_tr[i]
            t = tr[i]
            assert (t["receiver"], t["sender"]) == (ov, ou)
            if bool(t["removed"]) != orm:
                from tolerance import bound, pooled
                assert abs((okn - okc) - tau) <= bound(max(abs(okn), abs(okc)), pooled(sigma)), (name, i)
                equal = False
                break
        if equal:
            assert n_evals == len(o_tr)
            rows = np.concatenate([np.arange(g.edge_offsets()[r], g.edge_offsets()[r + 1]) for r in recv])
            assert (kept[rows] == (~g.removed_to_flat(o_removed))[rows].astype(np.uint8)).all()
        print(name, "sender-policy sweep:", "equal" if equal else "diverged inside the bound", "evals", n_evals)
    finally:
        gm.close()
