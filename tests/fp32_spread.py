"""How far the oracle's own KL moves when the values entering its e4m3 quantisers are only known to
binary32 accuracy (test infrastructure; CPU only; calls nothing but oracle/).

A device that computes in binary32 cannot reproduce the fp64 oracle's quantiser inputs to better than
a unit in the last place or two: its own rounding of the value plus the accumulated rounding of the
sums, norms and activation functions that produced it.  Each such difference that straddles a rounding
boundary of the e4m3 grid moves one code by a whole grid step (2^-4 .. 2^-3 relative on that element),
and the KL of a candidate inherits a spread from these moves that no binary32 implementation can
avoid.  This module measures that spread on the oracle: every quantiser input is multiplied by
1 + EPS * xi, with xi a unit-variance number that is a fixed function of (seed, element position, the
element's binary32 bits) -- the same value at the same place gets the same perturbation in the
reference pass and in the candidate pass, as a deterministic device gives it the same rounding error --
and the KL is recomputed for several seeds.  sigma = rms deviation from the unperturbed oracle value.

EPS = 2^-22 (two binary32 ulps).  The parity bound the GPU tests use with it is stated once, in
tests/tolerance.py.
"""
import numpy as np

from oracle.model import Model
from oracle.acdc import Acdc

EPS = 2.0 ** -22


class SpreadModel(Model):
    """oracle.model.Model whose quantiser inputs carry a seeded relative perturbation (0 = none)."""
    eps, seed = 0.0, 0

    def set_spread(self, eps, seed):
        self.eps, self.seed = float(eps), int(seed)

    def _quant_act(self, x, nm="W_Q"):
        if self.eps:
            bits = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
            idx = np.arange(x.size, dtype=np.uint64).reshape(x.shape)
            with np.errstate(over="ignore"):
                h = bits * np.uint64(0x9E3779B97F4A7C15) + idx * np.uint64(0xBF58476D1CE4E5B9) \
                    + np.uint64((self.seed * 0x94D049BB133111EB) % (1 << 64))
                h ^= h >> np.uint64(30); h *= np.uint64(0xBF58476D1CE4E5B9)
                h ^= h >> np.uint64(27); h *= np.uint64(0x94D049BB133111EB)
                h ^= h >> np.uint64(31)
            xi = ((h >> np.uint64(11)).astype(np.float64) / 2.0 ** 53 - 0.5) * np.sqrt(12.0)
            x = x * (1.0 + self.eps * xi)
        return super()._quant_act(x, nm)


def kl_with_spread(model, clean, corrupt, mode, cases, seeds=4, eps=EPS, progress=None, **acdc_args):
    """cases: list of (receiver, removed matrix, [senders]).  Returns per case a dict with the oracle's
    kl_current, kl_new[], and the rms deviations sigma_current, sigma_new[], sigma_inc[] (of kl_new -
    kl_current) over `seeds` perturbed re-evaluations.  `model` must be a SpreadModel; acdc_args go to
    oracle.acdc.Acdc (the metric and its token ids)."""
    def run():
        oa = Acdc(model, clean, corrupt, mode, **acdc_args)          # fresh caches under the current perturbation
        out = []
        for r, R, senders in cases:
            cur = oa.kl_fast(r, R)
            out.append((cur, [oa.kl_edge(r, int(u), removed=R) for u in senders]))
            if progress:
                progress(r)
        return out
    model.set_spread(0.0, 0)
    base = run()
    dev_cur = [[] for _ in cases]
    dev_new = [[[] for _ in c[2]] for c in cases]
    dev_inc = [[[] for _ in c[2]] for c in cases]
    for s in range(seeds):
        model.set_spread(eps, 1000 + s)
        got = run()
        for i, ((c0, n0), (c1, n1)) in enumerate(zip(base, got)):
            dev_cur[i].append(c1 - c0)
            for k in range(len(n0)):
                dev_new[i][k].append(n1[k] - n0[k])
                dev_inc[i][k].append((n1[k] - c1) - (n0[k] - c0))
    model.set_spread(0.0, 0)
    rms = lambda v: float(np.sqrt(np.mean(np.square(v)))) if len(v) else 0.0
    return [dict(kl_current=base[i][0], kl_new=base[i][1], sigma_current=rms(dev_cur[i]),
                 sigma_new=[rms(v) for v in dev_new[i]], sigma_inc=[rms(v) for v in dev_inc[i]])
            for i in range(len(cases))]


def circuit_kl_with_spread(model, clean, corrupt, pi, removed, seeds=4, eps=EPS):
    """KL of the pruned graph under the set `pi` of fp32 heads (three forwards from the embedding:
    corrupted run, clean reference, pruned clean run, all under `pi`), its logits, and the rms deviation
    of that KL over `seeds` perturbed re-evaluations."""
    from oracle.model import log_softmax, kl_to_reference

    def run():
        C, _ = model.forward(corrupt, pi)
        _, ref = model.forward(clean, pi)
        _, lg = model.forward(clean, pi, removed=removed, C=C)
        return kl_to_reference(log_softmax(ref), lg), lg
    model.set_spread(0.0, 0)
    kl, logits = run()
    dev = []
    for s in range(seeds):
        model.set_spread(eps, 1000 + s)
        dev.append(run()[0] - kl)
    model.set_spread(0.0, 0)
    return kl, logits, float(np.sqrt(np.mean(np.square(dev)))) if dev else 0.0
