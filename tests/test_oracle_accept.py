"""Pins for the acceptance rule (Eq. 5) and the stochastic path of the oracle (CPU only)."""
import itertools

import numpy as np
from scipy import stats

import helpers
from oracle import pacer_oracle as po
from paper_2602_01274_amd import synth


def test_emitted_token_law_is_exactly_p():
    """For any p, q: sum_y q(y) a(y) [v = y] + (1 - sum_y q(y) a(y)) p'(v) = p(v), with
    a = accept_prob and p' = residual_dist (exact enumeration, tiny vocabularies)."""
    rng = np.random.default_rng(0)
    for V in (2, 3, 7, 16):
        for _ in range(20):
            p, q = po.softmax(rng.standard_normal(V) * 2), po.softmax(rng.standard_normal(V) * 2)
            a = np.array([po.accept_prob(p, q, y) for y in range(V)])
            law = q * a + (1.0 - np.sum(q * a)) * po.residual_dist(p, q)
            assert np.max(np.abs(law - p)) < 1e-12
    # acceptance probability 1 when p >= q, ratio otherwise; p == q: always accepted
    p = np.array([.5, .3, .2]); q = np.array([.2, .3, .5])
    assert [po.accept_prob(p, q, y) for y in range(3)] == [1.0, 1.0, .2 / .5]
    assert np.allclose(po.residual_dist(p, q), [1.0, 0.0, 0.0])
    assert np.allclose(po.residual_dist(p, p), p)


def test_first_rejection_index():
    # n = min({i-1 : r_i > ratio_i} U {gamma})
    assert po.first_rejection(np.array([.9, .9, .1, .9]), np.array([.5, .5, .5, .5])) == 2
    assert po.first_rejection(np.array([.9, .9]), np.array([.5, .5])) == 2
    assert po.first_rejection(np.array([.4]), np.array([.5])) == 0
    assert po.first_rejection(np.array([.5]), np.array([.5])) == 1      # r == ratio accepts


T = dict(n_layers=1, d_model=16, n_heads=1, head_dim=16, d_ffn=32, vocab=5,
         rope_theta=10000.0, rms_eps=1e-5)


def _tiny(beta):
    w = dict(target=T, draft=T, share_embed_head=False, dtype="f32", block=2, gamma_max=4,
             beta=beta, t0=0.5, rho=1.05, mode="sample")
    tgt, drf, mb = synth.make_pair(w, seed=3)
    # spread the logits so that the laws are far from uniform and from each other
    tgt["head"] = tgt["head"] * 60.0
    drf["head"] = drf["head"] * 60.0
    return w, tgt, drf, mb


def _exact_ngram_law(w, tgt, drf, prompt, n):
    """Law of the next n tokens under autoregressive sampling of the effective target."""
    V = T["vocab"]
    law = {}
    ot, od, oc = helpers.to_oracle(tgt), helpers.to_oracle(drf), helpers.oracle_cfg(T)
    for seq in itertools.product(range(V), repeat=n):
        pr, ctx = 1.0, list(prompt)
        for tok in seq:
            kt, kd = po.KVCache(1, 16, 32), po.KVCache(1, 16, 32)
            lt = po.lm_forward(ot, oc, ctx, kt)[1][-1]
            ld = po.lm_forward(od, oc, ctx, kd)[1][-1]
            pr *= po.softmax(lt + w["beta"] * ld)[tok]
            ctx.append(tok)
        law[seq] = pr
    return law


_STOP_RULES = {
    "halting_test": None,                                   # the procedure's own decisions
    "adversarial": lambda k, a: k == 0 and a[0] > 0.5,      # a stop rule that looks at the pre-verification output
    "fixed3": "fixed3",                                     # vanilla speculative decoding, window 3
}


def _sample_ngrams(args):
    """Worker: 3-gram counts of the sampled procedure for seeds [lo, hi) under one stop rule (one oracle, reset per sample)."""
    rule, lo, hi, prompt = args
    from threadpoolctl import threadpool_limits
    threadpool_limits(1)                                    # 16-wide matrices: BLAS threads only get in each other's way
    w, tgt, drf, mb = _tiny(beta=1.0)
    fs = _STOP_RULES[rule]
    cached = [helpers.to_oracle(m, cache=True) for m in (tgt, drf, mb)]
    o = helpers.build_oracle(w, cached[0], cached[1], cached[2], mode=po.SAMPLE, seed=0, max_seq=32)
    cnt, acc = {}, 0
    for s in range(lo, hi):
        o.tokens, o.step_idx, o.seed = [], 0, 1000 + s
        for kv in (o.kvT, o.kvD, o.kvB):
            kv.n = 0
        o.prefill(prompt)
        out, recs = o.generate(3, fixed_gamma=3) if fs == "fixed3" else o.generate(3, force_stop=fs)
        cnt[tuple(out)] = cnt.get(tuple(out), 0) + 1
        acc += recs[0]["n"]
    return cnt, acc


def test_sampled_pacer_output_follows_the_target_law():
    """Sec. 2.2 (last sentence): the output distribution equals that of autoregressive decoding
    of the target.  3-gram law of the sampled procedure (30000 samples per stop rule, 125 cells: the smallest
    expected cell count is above 5, so every cell takes part), with the real halting test, with an adversarial
    stop rule that looks at the pre-verification output and with a fixed window, against exact enumeration."""
    from concurrent.futures import ProcessPoolExecutor
    import multiprocessing as mp
    w, tgt, drf, mb = _tiny(beta=1.0)
    prompt = [1, 4, 2]
    law = _exact_ngram_law(w, tgt, drf, prompt, 3)
    keys = sorted(law)
    exp = np.array([law[k] for k in keys])
    assert abs(exp.sum() - 1) < 1e-9 and exp.max() < 0.5
    n, workers = 30000, 8
    chunk = n // workers
    jobs = [(rule, i * chunk, (i + 1) * chunk, prompt) for rule in _STOP_RULES for i in range(workers)]
    with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as ex:
        res = list(ex.map(_sample_ngrams, jobs))
    for r, rule in enumerate(_STOP_RULES):
        cnt = dict.fromkeys(keys, 0)
        acc = 0
        for c, a in res[r * workers:(r + 1) * workers]:
            for k, v in c.items():
                cnt[k] += v
            acc += a
        obs = np.array([cnt[k] for k in keys], dtype=float)
        assert obs.sum() == n
        big = exp * n >= 5
        o2 = np.append(obs[big], obs[~big].sum()) if (~big).any() else obs
        e2 = np.append(exp[big], exp[~big].sum()) * n if (~big).any() else exp * n
        assert stats.chisquare(o2, e2).pvalue > 1e-3, rule
        assert 0 < acc / n < 3, rule          # both acceptances and rejections occurred


def test_sampled_first_token_is_not_the_draft_law():
    """Guard for the test above: with beta = 0 the draft law differs from the target law, and
    the procedure must still emit the target law (a p/q swap would emit the draft's)."""
    w, tgt, drf, mb = _tiny(beta=0.0)
    prompt = [0, 3]
    law = _exact_ngram_law(w, tgt, drf, prompt, 1)
    exp = np.array([law[(v,)] for v in range(5)])
    kd = po.KVCache(1, 16, 32)
    qlaw = po.softmax(po.lm_forward(helpers.to_oracle(drf), helpers.oracle_cfg(T), prompt, kd)[1][-1])
    assert np.abs(qlaw - exp).max() > 0.1
    n = 2000
    cnt = np.zeros(5)
    for s in range(n):
        o = helpers.build_oracle(w, tgt, drf, mb, mode=po.SAMPLE, seed=s, max_seq=32)
        o.prefill(prompt)
        cnt[o.generate(1)[0][0]] += 1
    assert stats.chisquare(cnt, exp * n).pvalue > 1e-3
    assert stats.chisquare(cnt, qlaw * n).pvalue < 1e-6
