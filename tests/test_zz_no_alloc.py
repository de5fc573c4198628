"""The allocation-free acceptance entry point against pacer_accept_rollback, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2602_01274_amd import binding as B
from paper_2602_01274_amd import synth

pytestmark = pytest.mark.gpu


def _drafted_and_verified(s, seq, gamma, mode, seed):
    ctr = s.step_idx[seq]
    B.pacer_begin_step(s.ctx, seq)
    for _ in range(gamma):
        B.pacer_draft_step(s.ctx, [seq], mode, seed, ctr)
    B.pacer_verify(s.ctx, [seq], None, s.logits)
    return ctr


@pytest.mark.parametrize("mode", [B.GREEDY, B.SAMPLE])
def test_accept_noalloc_matches_accept_rollback(mode):
    """pacer_accept_noalloc (scratch in the library's device image, no workspace, no allocation) must give the n and
    the new token of pacer_accept_rollback on the same logits, bit for bit: two calls in a row on one stream, the
    second with a smaller window (the shared scratch then still holds the first call's rows), on a pair whose
    vocabulary spans all 16 chunks; strong coupling makes all-accepted steps (bonus row) occur, weak coupling rejections."""
    from paper_2602_01274_amd.engine import Session
    w = synth.workload("mid")
    tgt, drf, mb = synth.make_pair(w, seed=0, gain_jitter=0.1, n_layers_target=2)
    s = Session(w, tgt, drf, mb, max_seq=256)
    V = w["target"]["vocab"]
    s.prefill(synth.make_prompt(V, 40, 1).tolist())
    stream = torch.cuda.current_stream().cuda_stream
    out_n = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    out_z = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    seen = set()
    for gamma, beta in ((12, 3.0), (4, 3.0), (8, 12.0), (3, 12.0), (12, 0.5), (1, 12.0), (2, 1.0), (1, 1.0), (1, 0.0), (1, 1.0), (1, 0.5)):
        ctr = _drafted_and_verified(s, 0, gamma, mode, 11)
        B.pacer_accept_rollback(s.ctx, [0], mode, [beta], 11, ctr, s.logits, s.n_acc, s.next_tok)
        st = B.pacer_get_state(s.ctx, 0)
        n, z = st["n_accepted"], st["next_token"]
        # the rings still hold this step's draft logits (row gamma: the bonus forward's, if it ran) and tokens
        tl = s.logits[0, :gamma + 1].contiguous()
        dl = s.draft_logits(0)[:gamma + 1].contiguous()
        dt = s.draft_tokens(0)[:gamma].contiguous()
        bonus = n == gamma
        B.pacer_accept_noalloc(tl, dl, dt, gamma, bonus, V, mode, beta, 11, ctr, 0, out_n, out_z, stream)
        torch.cuda.synchronize()
        assert (int(out_n.item()), int(out_z.item())) == (n, z), (gamma, beta, n, z)
        if not bonus:
            # without the bonus row a rejection gives the same result, and with it too (the row is then skipped)
            B.pacer_accept_noalloc(tl, dl, dt, gamma, True, V, mode, beta, 11, ctr, 0, out_n, out_z, stream)
            torch.cuda.synchronize()
            assert (int(out_n.item()), int(out_z.item())) == (n, z)
        else:
            B.pacer_accept_noalloc(tl, dl, dt, gamma, False, V, mode, beta, 11, ctr, 0, out_n, out_z, stream)
            torch.cuda.synchronize()
            assert (int(out_n.item()), int(out_z.item())) == (gamma, -1)
        seen.add(bonus)
        s.step_idx[0] += 1
    assert seen == {True, False}, "both a rejection and an all-accepted step must have occurred"
    with pytest.raises(B.PacerError) as e:
        B.pacer_accept_noalloc(tl, dl, dt, 32, True, V, mode, 1.0, 0, 0, 0, out_n, out_z, stream)
    assert e.value.code == B.EOVERFLOW
    s.close()


class _LogitsOracle:
    """The oracle's own step (Alg. 1, verification part; Eq. 5) run on scripted logits: the draft and target
    "models" return rows of given arrays, so the acceptance arithmetic of oracle/pacer_oracle.py is what decides."""

    def __init__(self, tl, dl, beta, mode, seed, step_idx, seq):
        from oracle import pacer_oracle as po

        class Scripted(po.PacerOracle):
            def __init__(s):
                c = po.ModelCfg(1, 1, 1, 1, 1, tl.shape[1])
                super().__init__(None, c, None, c, None, block=1, gamma_max=tl.shape[0], t0=0.5, rho=1.0, beta=beta,
                                 mode=mode, seed=seed, seq=seq, max_seq=1)
                s.k = 0

                class NoCache:
                    n = 10 ** 9
                    def truncate(self, n): pass
                s.kvT = s.kvD = s.kvB = NoCache()
                s.tokens = [0]
                s.step_idx = step_idx

            def _draft_one(s, tok):
                s.k += 1
                return np.zeros(1), dl[s.k - 1]

            def _target_rows(s, toks):
                return tl[:len(toks)]

        self.o = Scripted()

    def step(self, gamma):
        return self.o.step(fixed_gamma=gamma)


@pytest.mark.parametrize("mode", [B.GREEDY, B.SAMPLE])
def test_accept_noalloc_against_oracle_on_scripted_logits(mode):
    """The acceptance kernels against the oracle's Eq. 5 arithmetic on logits that no model produced: the largest
    window the entry point takes (gamma 31, vocabulary 32000: all 16 chunks), strong and weak coupling, identical
    draft and target distributions (beta 0, equal logits: every draft is accepted with probability one and a rejection
    would find no residual mass), and a window of one.  Integers must be equal unless the oracle's margin is a tie."""
    import torch
    from oracle import philox
    from oracle import pacer_oracle as po
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(17)
    out_n = torch.zeros(1, dtype=torch.int32, device="cuda")
    out_z = torch.zeros(1, dtype=torch.int32, device="cuda")
    cases = [(31, 32000, 3.0, 1.0, False), (31, 32000, 0.5, 1.0, False), (16, 32000, 0.0, 1.0, True), (1, 1024, 1.0, 2.0, False),
             (8, 5000, 6.0, 0.5, False), (31, 1024, 12.0, 1.0, False), (5, 16, 1.0, 1.0, False)]
    seen_bonus = False
    for ci, (gamma, V, beta, scale, same) in enumerate(cases):
        for rep in range(3):
            dl = (rng.standard_normal((gamma + 1, V)) * scale).astype(np.float32).astype(np.float64)
            tl = dl.copy() if same else (rng.standard_normal((gamma + 1, V)) * scale).astype(np.float32).astype(np.float64)
            seed, step_idx, seq = 100 + ci, 7 + rep, (ci + rep) % 16
            ro = _LogitsOracle(tl, dl, beta, mode, seed, step_idx, seq).step(gamma)
            y = ro["draft_tokens"]
            t_dev = torch.tensor(tl, dtype=torch.float32, device="cuda")
            d_dev = torch.tensor(dl, dtype=torch.float32, device="cuda")
            y_dev = torch.tensor(y, dtype=torch.int32, device="cuda")
            B.pacer_accept_noalloc(t_dev, d_dev, y_dev, gamma, True, V, mode, beta, seed, step_idx, seq, out_n, out_z, stream)
            torch.cuda.synchronize()
            n, z = int(out_n.item()), int(out_z.item())
            seen_bonus |= ro["n"] == gamma
            if (n, z) != (ro["n"], ro["z"]):
                # excused only as a tie of the oracle's own deciding quantity (float32 kernels against float64)
                k = min(n, ro["n"])
                eff = tl[k] + beta * dl[k]
                if mode == B.GREEDY:
                    top = np.sort(eff)[-2:]
                    margin = top[1] - top[0]
                elif n != ro["n"]:
                    margin = abs(ro["r"][k] - ro["ratios"][k])
                else:
                    u = philox.vocab_uniforms(seed, seq, step_idx, k + 1, philox.PURPOSE_NEXT, V)
                    if k == gamma:
                        keys = eff + philox.gumbel(u)
                    else:
                        with np.errstate(divide="ignore"):
                            keys = np.log(po.residual_dist(po.softmax(eff), po.softmax(dl[k]))) + philox.gumbel(u)
                    top = np.sort(keys[np.isfinite(keys)])[-2:]
                    margin = top[1] - top[0]
                assert margin < 1e-3, (gamma, V, beta, same, (n, z), (ro["n"], ro["z"]), margin)
            if same and mode == B.SAMPLE:
                assert ro["n"] == gamma          # p == q: every ratio is 1
    assert seen_bonus


@pytest.mark.parametrize("mode", [B.GREEDY, B.SAMPLE])
def test_accept_noalloc_bad_values_do_not_index_out_of_range(mode):
    """The caller's buffers may hold anything.  A draft id outside the vocabulary is read as the nearest valid id
    (so p[y] and q[y] stay inside their rows); logits without a finite value leave the next token at 0x7fffffff.
    Neither may fault, and a sound call afterwards gives the result it gave before."""
    V, gamma = 1000, 6
    g = torch.Generator(device="cpu").manual_seed(3)
    tl = torch.randn(gamma + 1, V, generator=g).cuda()
    dl = torch.randn(gamma + 1, V, generator=g).cuda()
    dt = tl[:gamma].argmax(dim=1).to(torch.int32)
    stream = torch.cuda.current_stream().cuda_stream
    out_n = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    out_z = torch.full((1,), -7, dtype=torch.int32, device="cuda")

    def run(t, d, y):
        B.pacer_accept_noalloc(t, d, y, gamma, True, V, mode, 0.0, 5, 0, 0, out_n, out_z, stream)
        torch.cuda.synchronize()
        return int(out_n.item()), int(out_z.item())

    ref = run(tl, dl, dt)
    assert 0 <= ref[0] <= gamma and 0 <= ref[1] < V
    for bad in (V, V + 12345, -1, 2**31 - 1):
        y = dt.clone()
        y[2] = bad
        n, z = run(tl, dl, y)
        assert 0 <= n <= gamma and 0 <= z < V
        if mode == B.GREEDY:
            assert n <= 2                              # an id no argmax can equal is rejected at the latest there
    nan = torch.full_like(tl, float("nan"))
    n, z = run(nan, dl, dt)
    assert z == 0x7FFFFFFF and 0 <= n <= gamma
    assert run(tl, dl, dt) == ref
