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


def _argmax_key_gap(keys, a, b):
    """|keys[a] - keys[b]|, infinite if either is not finite."""
    if not (np.isfinite(keys[a]) and np.isfinite(keys[b])):
        return float("inf")
    return float(abs(keys[a] - keys[b]))


class StepChecker:
    """Feeds the same committed prefix to both sides, compares every per-call tensor and every
    integer decision (draft tokens, stop flags, the accept count n, the new token z).

    Integers must agree.  Two classes of disagreement are excused, logged in self.flips and
    followed by re-prefilling the GPU sequence with the oracle's prefix (teacher forcing):

      "tie"           the oracle's own margin at the deciding quantity (gap of the top two of the
                      deciding logits row, |statistic - t| of the stop test, |r - p/q| of the
                      accept test) is below `tie` = 1e-3.  Not limited in number.
      "within_error"  the margin is below what the error measured ON THE DECIDING ROW ALONE can move
                      it (argmax: two entries move towards each other, so 2 x the row's max-abs
                      error; stop test: the largest alpha error of the deciding block; accept
                      test: the ratio's bound from the row's log-probability errors), AND the
                      decision recomputed in float64 from the GPU's own logits is the decision the
                      GPU took (its decision logic is right; its logits, themselves asserted to be
                      within tolerance, differ).  At most one per 50 compared decisions.

    After a draft-token flip the rest of the step is not comparable (the two sides drafted
    different tokens), but the verify rows and alphas that depend only on the common tokens
    still are, and are compared."""

    OWN_MARGIN = 1e-4     # below this the GPU's f32 decision arithmetic and its float64 recomputation may differ

    def __init__(self, sess, orc, tol_logits, tol_alpha, tie=1e-3, mode=po.GREEDY, seed=0, seq=0):
        self.s, self.o, self.seq = sess, orc, seq
        self.tol_logits, self.tol_alpha, self.tie = tol_logits, tol_alpha, tie
        self.mode, self.seed = mode, seed
        self.flips = []
        self.max_err = dict(draft_logits=0.0, hidden=0.0, target_logits=0.0, alpha=0.0)
        self.steps = 0
        self.decisions = 0

    # ---- bookkeeping ---------------------------------------------------------------------
    def ties(self):
        return [f for f in self.flips if f[2] == "tie"]

    def within_error(self):
        return [f for f in self.flips if f[2] == "within_error"]

    def allowed_within_error(self):
        return max(1, self.decisions // 50)

    def assert_flip_budget(self):
        assert len(self.within_error()) <= self.allowed_within_error(), (
            f"{len(self.within_error())} within_error flips in {self.decisions} decisions: {self.within_error()}")

    def summary(self):
        return (f"steps={self.steps} decisions={self.decisions} ties={self.ties()} "
                f"within_error={self.within_error()} max_err={self.max_err}")

    def _resync(self):
        self.s.prefill(self.o.tokens, seq=self.seq)
        self.s.step_idx[self.seq] = self.o.step_idx

    def _explain(self, kind, margin, k, bound, own_ok):
        """A disagreement of kind `kind` at index k.  margin: the oracle's margin; bound: what the
        deciding row's measured error can move; own_ok: the GPU's decision follows from its own logits."""
        if margin < self.tie:
            self.flips.append((self.steps, kind, "tie", k, margin))
            return
        assert margin < bound, (f"step {self.steps}: {kind} mismatch at {k}: oracle margin {margin:.3e} is neither a "
                                f"tie nor within the deciding row's error bound {bound:.3e}")
        assert own_ok, f"step {self.steps}: {kind} mismatch at {k}: the GPU's decision does not follow from its own logits"
        self.flips.append((self.steps, kind, "within_error", k, margin))

    # ---- one step ------------------------------------------------------------------------
    def step(self, **kw):
        step_idx = self.o.step_idx
        ro = self.o.step(**kw)
        rg = self.s.step(mode=self.mode, seed=self.seed, record=True, **kw)
        return self.check(ro, rg, step_idx)

    def _draft_keys(self, row, step_idx, k):
        if self.mode != po.SAMPLE:
            return np.asarray(row, dtype=np.float64)
        u = philox.vocab_uniforms(self.seed, self.seq, step_idx, k + 1, philox.PURPOSE_DRAFT, len(row))
        return np.asarray(row, dtype=np.float64) + philox.gumbel(u)

    def _check_alpha(self, ro, rg, upto):
        na = min(len(ro["alpha"]), len(rg.get("alpha", [])), upto)
        ea = 0.0
        if na:
            ea = float(np.abs(np.array(rg["alpha"][:na]) - ro["alpha"][:na]).max())
            self.max_err["alpha"] = max(self.max_err["alpha"], ea)
            assert ea < self.tol_alpha, (self.steps, ea)
        return na

    def _check_target_rows(self, ro, rg, n_rows):
        tl = rg["target_logits"].cpu().numpy()
        for k in range(n_rows):
            e = rel_err(tl[k], ro["target_logits"][k])
            self.max_err["target_logits"] = max(self.max_err["target_logits"], e)
            assert e < self.tol_logits, (self.steps, k, e)
        return tl

    def check(self, ro, rg, step_idx):
        """Compare one finished step of this sequence (ro: oracle record, rg: GPU record)."""
        self.steps += 1
        beta = self.o.beta
        b = self.o.b
        # --- drafting: compare row by row until the first differing draft token
        g = min(ro["gamma"], rg["gamma"])
        dl = rg["draft_logits"].cpu().numpy()
        hd = rg["hidden"].cpu().numpy()
        for k in range(g):
            self.max_err["draft_logits"] = max(self.max_err["draft_logits"], rel_err(dl[k], ro["draft_logits"][k]))
            self.max_err["hidden"] = max(self.max_err["hidden"], rel_err(hd[k], ro["hidden"][k]))
            assert rel_err(dl[k], ro["draft_logits"][k]) < self.tol_logits, (self.steps, k)
            assert rel_err(hd[k], ro["hidden"][k]) < self.tol_logits, (self.steps, k)
            self.decisions += 1
            if rg["draft_tokens"][k] != ro["draft_tokens"][k]:
                keys_o = self._draft_keys(ro["draft_logits"][k], step_idx, k)
                keys_g = self._draft_keys(dl[k], step_idx, k)
                yg = rg["draft_tokens"][k]
                own = int(np.argmax(keys_g))
                own_ok = own == yg or _argmax_key_gap(keys_g, own, yg) < self.OWN_MARGIN
                self._explain("draft_token", top2_gap(keys_o), k, 2.0 * abs_err(dl[k], ro["draft_logits"][k]), own_ok)
                # what depends only on the common tokens: alphas of the rows up to k, verify rows 0..k
                self._check_alpha(ro, rg, k + 1)
                self._check_target_rows(ro, rg, min(k, g) + 1)
                self._resync()
                return ro, rg
        # --- pre-verification
        na = self._check_alpha(ro, rg, 1 << 30)
        n_rounds = min(len(ro["rounds"]), len(rg.get("stops", [])))
        self.decisions += n_rounds
        if rg["gamma"] != ro["gamma"]:
            rnd = n_rounds - 1
            r = ro["rounds"][rnd]
            a_g = np.array(rg["alpha"][rnd * b:(rnd + 1) * b], dtype=np.float32)
            e_blk = float(np.abs(a_g.astype(np.float64) - ro["alpha"][rnd * b:(rnd + 1) * b]).max()) if na else 0.0
            own_stop, _ = self.o._halt(a_g, np.float32(r["t"]))          # the halting test on the GPU's own alphas, in f32
            self._explain("stop", abs(r["stat"] - r["t"]), rnd, e_blk, own_stop == bool(rg["stops"][rnd]))
            self._check_target_rows(ro, rg, g + 1)
            self._resync()
            return ro, rg
        # --- verification
        gam = ro["gamma"]
        tl = self._check_target_rows(ro, rg, gam + 1)
        if ro["bonus_draft_logits"] is not None:
            assert rel_err(dl[gam], ro["bonus_draft_logits"]) < self.tol_logits
        # --- acceptance
        self.decisions += 2
        if (rg["n"], rg["z"]) != (ro["n"], ro["z"]):
            k = min(rg["n"], ro["n"])
            dl_o_k = ro["draft_logits"][k] if k < gam else ro["bonus_draft_logits"]
            e_q = abs_err(dl[k], dl_o_k) if dl_o_k is not None else 0.0
            e_eff = abs_err(tl[k], ro["target_logits"][k]) + abs(beta) * e_q      # the deciding row alone
            eff_o = ro["target_logits"][k] + (beta * dl_o_k if dl_o_k is not None else 0.0)
            eff_g = tl[k].astype(np.float64) + beta * dl[k].astype(np.float64)
            if self.mode == po.GREEDY:
                # the GPU's n from its own logits: the first row whose argmax is not its draft
                own = int(np.argmax(eff_g))
                if rg["n"] < ro["n"]:          # GPU rejected y_k: its own argmax must differ from y_k
                    yk = ro["draft_tokens"][k]
                    own_ok = own != yk or _argmax_key_gap(eff_g, own, int(np.argsort(eff_g)[-2])) < self.OWN_MARGIN
                elif rg["n"] > ro["n"]:        # GPU accepted y_k
                    yk = ro["draft_tokens"][k]
                    own_ok = own == yk or _argmax_key_gap(eff_g, own, yk) < self.OWN_MARGIN
                else:                          # same n, other token
                    own_ok = own == rg["z"] or _argmax_key_gap(eff_g, own, rg["z"]) < self.OWN_MARGIN
                self._explain("accept" if rg["n"] != ro["n"] else "next_token", top2_gap(eff_o), k, 2.0 * e_eff, own_ok)
            elif rg["n"] != ro["n"]:
                yk = ro["draft_tokens"][k]
                ratio_o, rk = float(ro["ratios"][k]), float(ro["r"][k])
                lp_g = eff_g - (eff_g.max() + np.log(np.exp(eff_g - eff_g.max()).sum()))
                q_g = dl[k].astype(np.float64)
                lq_g = q_g - (q_g.max() + np.log(np.exp(q_g - q_g.max()).sum()))
                ratio_g = float(np.exp(lp_g[yk] - lq_g[yk]))
                own_rej = rk > ratio_g
                own_ok = own_rej == (rg["n"] == k) or abs(rk - ratio_g) < self.OWN_MARGIN * max(1.0, ratio_g)
                # log-ratio = (eff[y] - lse(eff)) - (q[y] - lse(q)): each of the four terms moves by at most its row's error
                delta = 2.0 * (e_eff + e_q)
                self._explain("accept", abs(rk - ratio_o), k, ratio_o * (np.exp(delta) - 1.0), own_ok)
            else:
                keys_o = self._next_keys(ro["target_logits"][k], dl_o_k, beta, k, gam, step_idx)
                keys_g = self._next_keys(tl[k], dl[k], beta, k, gam, step_idx)
                own = int(np.argmax(keys_g))
                own_ok = own == rg["z"] or _argmax_key_gap(keys_g, own, rg["z"]) < 10 * self.OWN_MARGIN
                fin = np.isfinite(keys_o) & np.isfinite(keys_g)
                e_keys = float(np.abs(keys_o[fin] - keys_g[fin]).max())
                self._explain("next_token", top2_gap(keys_o[np.isfinite(keys_o)]), k, 2.0 * e_keys, own_ok)
            self._resync()
            return ro, rg
        assert rg["len"] == len(self.o.tokens)
        return ro, rg

    def _next_keys(self, t_row, d_row, beta, n, gam, step_idx):
        """Gumbel-max keys of the emitted token at row n: log p (bonus row) or log max(0, p - q), plus the noise."""
        t_row = np.asarray(t_row, dtype=np.float64)
        d_row = np.asarray(d_row, dtype=np.float64)
        u = philox.vocab_uniforms(self.seed, self.seq, step_idx, n + 1, philox.PURPOSE_NEXT, len(t_row))
        if n == gam:
            return t_row + beta * d_row + philox.gumbel(u)
        P = po.softmax(t_row + beta * d_row)
        Q = po.softmax(d_row)
        with np.errstate(divide="ignore"):
            return np.log(po.residual_dist(P, Q)) + philox.gumbel(u)
