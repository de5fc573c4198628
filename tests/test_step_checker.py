"""The GPU-vs-oracle step checker itself, exercised on the CPU: a stand-in "device" (a second oracle
whose logits carry small seeded noise, as a reduced-precision path's would) must pass with its flips
classified, and planted decision bugs must fail."""
import numpy as np
import pytest
import torch

import helpers
from gpu_utils import StepChecker
from oracle import pacer_oracle as po
from paper_2602_01274_amd import synth


class NoisyOracle(po.PacerOracle):
    """The oracle with seeded noise on every logits row and hidden state it produces."""

    def __init__(self, *a, sigma=0.0, **kw):
        super().__init__(*a, **kw)
        self.rng = np.random.default_rng(1234)
        self.sigma = sigma

    def _target_rows(self, toks):
        lg = super()._target_rows(toks)
        return lg + self.sigma * self.rng.standard_normal(lg.shape)

    def _draft_one(self, tok):
        h, lg = super()._draft_one(tok)
        return h, lg + self.sigma * self.rng.standard_normal(lg.shape)


class FakeSession:
    """Looks like engine.Session to the checker; bug: a planted decision error."""

    def __init__(self, orc, bug=None):
        self.o, self.bug = orc, bug
        self.step_idx = [0]

    def prefill(self, tokens, seq=0):
        o = self.o
        o.tokens = []
        for kv in (o.kvT, o.kvD, o.kvB):
            kv.n = 0
        o.prefill(tokens)

    def tokens(self, seq=0):
        return list(self.o.tokens)

    def step(self, mode=0, seed=0, record=True, **kw):
        o = self.o
        o.mode, o.seed, o.step_idx = mode, seed, self.step_idx[0]
        r = o.step(**kw)
        self.step_idx[0] += 1
        g = r["gamma"]
        V, d = r["draft_logits"].shape[1], r["hidden"].shape[1]
        dl = np.zeros((g + 1, V))
        dl[:g] = r["draft_logits"]
        if r["bonus_draft_logits"] is not None:
            dl[g] = r["bonus_draft_logits"]
        hid = np.zeros((g + 1, d))
        hid[:g] = r["hidden"]
        n, z = r["n"], r["z"]
        if self.bug == "n_plus_one" and n < g:
            n += 1
        if self.bug == "z_is_draft" and n < g:
            z = r["draft_tokens"][n]
        return dict(gamma=g, n=n, z=z, len=len(o.tokens), alpha=[float(np.float32(a)) for a in r["alpha"]],
                    stops=[x["stop"] for x in r["rounds"]], draft_tokens=list(r["draft_tokens"]),
                    draft_logits=torch.tensor(dl, dtype=torch.float32), hidden=torch.tensor(hid, dtype=torch.float32),
                    target_logits=torch.tensor(r["target_logits"], dtype=torch.float32))


def _pair(mode, sigma, bug=None, seed=5):
    w = synth.workload("tiny")
    tgt, drf, mb = synth.make_pair(w, seed=0)
    prompt = synth.make_prompt(w["target"]["vocab"], 12, 1).tolist()
    ow = [helpers.to_oracle(m, cache=True) for m in (tgt, drf, mb)]
    o = helpers.build_oracle(w, ow[0], ow[1], ow[2], mode=mode, seed=seed, max_seq=256)
    args = dict(block=w["block"], gamma_max=w["gamma_max"], t0=w["t0"], rho=w["rho"], beta=w["beta"], mode=mode, seed=seed,
                max_seq=256, sigma=sigma)
    dev = NoisyOracle(ow[0], helpers.oracle_cfg(w["target"]), ow[1], helpers.oracle_cfg(w["draft"]), ow[2], **args)
    s = FakeSession(dev, bug)
    s.prefill(prompt)
    o.prefill(prompt)
    return StepChecker(s, o, 2e-2, 2e-2, mode=mode, seed=seed), s, o


@pytest.mark.parametrize("mode", [po.GREEDY, po.SAMPLE])
def test_exact_device_has_no_flips(mode):
    ck, s, o = _pair(mode, 0.0)
    for _ in range(12):
        ck.step()
    assert ck.flips == [] and ck.decisions > 50
    assert s.tokens() == o.tokens


@pytest.mark.parametrize("mode", [po.GREEDY, po.SAMPLE])
def test_noisy_device_flips_are_classified_and_teacher_forced(mode):
    """Noise of 1e-3 (standard deviation) on every logit, about 1e-2 of the logit RMS at its largest, inside the 2e-2 tolerance, flips
    some decisions; each must be explained by the deciding row's own error, and the run stays in step."""
    ck, s, o = _pair(mode, 1e-3)
    for _ in range(40):
        ck.step()
    assert s.tokens() == o.tokens
    assert ck.flips, "noise of this size is expected to flip at least one decision in 40 steps"
    for f in ck.flips:
        assert f[2] in ("tie", "within_error")
        if f[2] == "within_error":
            assert f[4] >= 1e-3


@pytest.mark.parametrize("bug", ["n_plus_one", "z_is_draft"])
@pytest.mark.parametrize("mode", [po.GREEDY, po.SAMPLE])
def test_planted_decision_bugs_fail(mode, bug):
    ck, s, o = _pair(mode, 0.0, bug)
    with pytest.raises(AssertionError):
        for _ in range(12):
            ck.step()
