"""Step-by-step comparison of the HIP path with the CPU oracle (teacher forced)."""
import numpy as np

from oracle import pacer_oracle as po
from oracle import philox


def rel_err(got, ref):
    """max |got - ref| over the array, divided by the RMS of the reference."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    return float(np.abs(got - ref).max() / np.sqrt(np.mean(ref ** 2)))


def top2_gap(row):
    s = np.sort(np.asarray(row))
    return float(s[-1] - s[-2])


def abs_err(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - np.asarray(ref, dtype=np.float64)).max())


class StepChecker:
    """Feeds the same committed prefix to both sides, compares every per-call tensor and every
    integer decision.  Integers must agree, except where the oracle's own margin at that decision
    (argmax gap of the deciding logits, |mean - t|, |r - p/q|) is
      * below `tie` (1e-3): a tie, logged in self.flips as ("tie", ...), or
      * below twice the logit error actually measured on the deciding rows of that very step
        (which is itself asserted to be within the tolerance): the GPU decided correctly on its
        own logits; logged as ("within_error", ...).
    After a logged flip the GPU sequence is re-prefilled with the oracle's prefix."""

    def __init__(self, sess, orc, tol_logits, tol_alpha, tie=1e-3, mode=po.GREEDY, seed=0, seq=0):
        self.s, self.o, self.seq = sess, orc, seq
        self.tol_logits, self.tol_alpha, self.tie = tol_logits, tol_alpha, tie
        self.mode, self.seed = mode, seed
        self.flips = []
        self.max_err = dict(draft_logits=0.0, hidden=0.0, target_logits=0.0, alpha=0.0)
        self.steps = 0

    def _resync(self):
        self.s.prefill(self.o.tokens, seq=self.seq)
        self.s.step_idx[self.seq] = self.o.step_idx

    def _explain(self, kind, margin, k, err=0.0):
        bound = max(self.tie, 2.0 * err)
        assert margin < bound, f"step {self.steps}: {kind} mismatch at {k}: oracle margin {margin}, measured error {err}"
        self.flips.append((self.steps, kind, "tie" if margin < self.tie else "within_error", k, margin))

    def step(self, **kw):
        step_idx = self.o.step_idx
        ro = self.o.step(**kw)
        rg = self.s.step(mode=self.mode, seed=self.seed, record=True, **kw)
        return self.check(ro, rg, step_idx)

    def check(self, ro, rg, step_idx):
        """Compare one finished step of this sequence (ro: oracle record, rg: GPU record)."""
        self.steps += 1
        beta = self.o.beta
        # --- drafting: compare row by row until the first differing draft token
        g = min(ro["gamma"], rg["gamma"])
        dl = rg["draft_logits"].cpu().numpy()
        hd = rg["hidden"].cpu().numpy()
        for k in range(g):
            self.max_err["draft_logits"] = max(self.max_err["draft_logits"], rel_err(dl[k], ro["draft_logits"][k]))
            self.max_err["hidden"] = max(self.max_err["hidden"], rel_err(hd[k], ro["hidden"][k]))
            assert rel_err(dl[k], ro["draft_logits"][k]) < self.tol_logits, (self.steps, k)
            assert rel_err(hd[k], ro["hidden"][k]) < self.tol_logits, (self.steps, k)
            if rg["draft_tokens"][k] != ro["draft_tokens"][k]:
                row = ro["draft_logits"][k]
                if self.mode == po.SAMPLE:
                    u = philox.vocab_uniforms(self.seed, self.seq, step_idx, k + 1, philox.PURPOSE_DRAFT, len(row))
                    row = row + philox.gumbel(u)
                self._explain("draft_token", top2_gap(row), k, abs_err(dl[k], ro["draft_logits"][k]))
                self._resync()
                return ro, rg
        # --- pre-verification
        na = min(len(ro["alpha"]), len(rg.get("alpha", [])))
        if na:
            ea = float(np.abs(np.array(rg["alpha"][:na]) - ro["alpha"][:na]).max())
            self.max_err["alpha"] = max(self.max_err["alpha"], ea)
            assert ea < self.tol_alpha, (self.steps, ea)
        if rg["gamma"] != ro["gamma"]:
            rnd = min(len(ro["rounds"]), len(rg["stops"])) - 1
            r = ro["rounds"][rnd]
            self._explain("stop", abs(r["stat"] - r["t"]), rnd, ea if na else 0.0)
            self._resync()
            return ro, rg
        # --- verification
        tl = rg["target_logits"].cpu().numpy()
        for k in range(ro["gamma"] + 1):
            e = rel_err(tl[k], ro["target_logits"][k])
            self.max_err["target_logits"] = max(self.max_err["target_logits"], e)
            assert e < self.tol_logits, (self.steps, k, e)
        if ro["bonus_draft_logits"] is not None:
            assert rel_err(dl[ro["gamma"]], ro["bonus_draft_logits"]) < self.tol_logits
        # --- acceptance
        if (rg["n"], rg["z"]) != (ro["n"], ro["z"]):
            gam = ro["gamma"]
            e_eff = abs_err(tl[:gam + 1], ro["target_logits"]) + abs(beta) * abs_err(
                dl[:gam], ro["draft_logits"]) if gam else abs_err(tl[:1], ro["target_logits"])
            if ro["bonus_draft_logits"] is not None:
                e_eff += abs(beta) * abs_err(dl[gam], ro["bonus_draft_logits"])
            if self.mode == po.GREEDY:
                eff = ro["target_logits"][:gam] + beta * ro["draft_logits"]
                rows = list(eff) + ([ro["target_logits"][gam] + beta * ro["bonus_draft_logits"]]
                                    if ro["bonus_draft_logits"] is not None else [])
                k = min(rg["n"], ro["n"])
                self._explain("accept", top2_gap(rows[k]), k, e_eff)
            else:
                k = min(rg["n"], ro["n"])
                if rg["n"] != ro["n"]:
                    self._explain("accept", abs(ro["r"][k] - ro["ratios"][k]), k, 2.0 * e_eff * max(1.0, ro["ratios"][k]))
                else:
                    self._explain("next_token", self._next_gap(ro, step_idx), k, e_eff)
            self._resync()
            return ro, rg
        assert rg["len"] == len(self.o.tokens)
        return ro, rg

    def _next_gap(self, ro, step_idx):
        n, gam, beta = ro["n"], ro["gamma"], self.o.beta
        V = ro["target_logits"].shape[1]
        u = philox.vocab_uniforms(self.seed, self.seq, step_idx, n + 1, philox.PURPOSE_NEXT, V)
        if n == gam:
            keys = ro["target_logits"][gam] + beta * ro["bonus_draft_logits"] + philox.gumbel(u)
        else:
            P = po.softmax(ro["target_logits"][n] + beta * ro["draft_logits"][n])
            Q = po.softmax(ro["draft_logits"][n])
            with np.errstate(divide="ignore"):
                keys = np.log(po.residual_dist(P, Q)) + philox.gumbel(u)
        return top2_gap(keys[np.isfinite(keys)])
