"""GPU parity: the HIP path against the CPU oracle, call by call, on identical seeded inputs.
All of these go through the C ABI (binding -> libpacer.so)."""
import numpy as np
import pytest
import torch

import helpers
from gpu_utils import StepChecker, rel_err
from oracle import pacer_oracle as po
from paper_2602_01274_amd import synth

pytestmark = pytest.mark.gpu


def _session(w, tgt, drf, mb, max_seq, **kw):
    from paper_2602_01274_amd.engine import Session
    return Session(w, tgt, drf, mb, max_seq=max_seq, **kw)


def _run(name, n_prompt, n_new, tol_logits, tol_alpha, mode=po.GREEDY, seed=0, gain_jitter=0.1,
         max_seq=512, step_kw=None, w_over=None, n_layers_target=None, halting="mean", kv_fill=None):
    w = synth.workload(name)
    w.update(w_over or {})
    tgt, drf, mb = synth.make_pair(w, seed=0, gain_jitter=gain_jitter, n_layers_target=n_layers_target)
    prompt = synth.make_prompt(w["target"]["vocab"], n_prompt, 1).tolist()
    s = _session(w, tgt, drf, mb, max_seq, halting={"mean": 0, "any": 1, "last": 2}[halting], kv_fill=kv_fill)
    o = helpers.build_oracle(w, tgt, drf, mb, mode=mode, seed=seed, max_seq=max_seq, cache=True, halting=halting)
    s.prefill(prompt)
    o.prefill(prompt)
    ck = StepChecker(s, o, tol_logits, tol_alpha, mode=mode, seed=seed)
    start = len(o.tokens)
    gammas, ns = [], []
    while len(o.tokens) - start < n_new:
        ro, _ = ck.step(**(step_kw or {}))
        gammas.append(ro["gamma"])
        ns.append(ro["n"])
    toks = s.tokens()
    assert toks == o.tokens
    print(f"\n[{name} mode={mode}] gamma mean={np.mean(gammas):.2f} tau={np.mean(ns):.2f} {ck.summary()}")
    ck.assert_flip_budget()                            # ties (< 1e-3) are only logged; within_error: 1 per 50 decisions
    s.close()
    return ck, gammas, ns


def test_tiny_f32_greedy_steps_match_oracle():
    """Workload `tiny`: f32 pair, 32-token prompt, 64 new tokens, greedy, gamma_max 8, b 2."""
    ck, gammas, ns = _run("tiny", 32, 64, tol_logits=1e-4, tol_alpha=1e-4)
    assert len(set(gammas)) > 1          # the window really adapts
    assert 0 < np.mean(ns) < np.mean(gammas)
    both = {n == g for n, g in zip(ns, gammas)}
    assert both == {True, False}         # steps with a rejection and all-accepted steps (bonus row) both occurred


def test_tiny_f32_sampling_steps_match_oracle():
    _run("tiny", 32, 48, tol_logits=1e-4, tol_alpha=1e-4, mode=po.SAMPLE, seed=7)


def test_tiny_fixed_window_and_autoregressive_modes():
    _run("tiny", 9, 24, tol_logits=1e-4, tol_alpha=1e-4, step_kw=dict(fixed_gamma=5))
    _run("tiny", 1, 12, tol_logits=1e-4, tol_alpha=1e-4, step_kw=dict(fixed_gamma=1))


def test_tiny_forced_stop_patterns():
    _run("tiny", 20, 24, tol_logits=1e-4, tol_alpha=1e-4, step_kw=dict(force_stop=lambda k, a: False))
    _run("tiny", 20, 16, tol_logits=1e-4, tol_alpha=1e-4, step_kw=dict(force_stop=lambda k, a: True))


def test_largest_windows_the_library_takes():
    """gamma_max = 31 is the largest window a context accepts (32 verify rows = two full row tiles).  f32 pair with
    block size 1 (31 draft steps and 31 one-row pre-verification calls per step), bf16 pair with gamma_max 28 and
    b 4 (29 verify rows: two row tiles, not the 17-row form); every block is forced to pass so that each step uses
    the whole window."""
    ck, gammas, _ = _run("tiny", 11, 40, tol_logits=1e-4, tol_alpha=1e-4, w_over=dict(block=1, gamma_max=31),
                         step_kw=dict(force_stop=lambda k, a: False), max_seq=256)
    assert set(gammas) == {31}
    ck, gammas, _ = _run("mid", 90, 24, tol_logits=2e-2, tol_alpha=2e-2, w_over=dict(gamma_max=28),
                         step_kw=dict(force_stop=lambda k, a: False), max_seq=512)
    assert set(gammas) == {28}


def test_halting_variants_any_and_last():
    """Sec. 5.2's stricter criteria (any token / last token below t) next to the mean criterion."""
    g = {}
    for h in ("mean", "any", "last"):
        _, gammas, _ = _run("tiny", 20, 32, tol_logits=1e-4, tol_alpha=1e-4, halting=h)
        g[h] = np.mean(gammas)
    print("mean window per criterion:", g)
    assert g["any"] <= g["mean"] + 2      # per block 'any' stops whenever the mean does (step boundaries differ, so only roughly)


def test_halting_variants_bf16_path():
    """The same criteria through the bf16 path's pre-verification head kernel."""
    for h in ("any", "last"):
        _run("mid", 60, 16, tol_logits=2e-2, tol_alpha=2e-2, halting=h)


def test_mid_bf16_greedy_steps_match_oracle():
    """Workload `mid` (12-layer d768 V32000 target, 2-layer draft, bf16, b 4, gamma_max 12);
    the context crosses several 64-key attention tiles."""
    _run("mid", 150, 40, tol_logits=2e-2, tol_alpha=2e-2)


def test_mid_config_as_named_full_length(capsys):
    """Workload `mid` exactly as named: 12-layer d768 target, 2-layer draft, bf16, greedy, beta 3, 128-token prompt,
    256 new tokens, gamma_max 12, b 4: about 200 teacher-forced steps and 3000 integer decisions against the oracle."""
    w = synth.workload("mid")
    assert (w["prompt"], w["new"], w["gamma_max"], w["block"], w["mode"]) == (128, 256, 12, 4, "greedy")
    ck, gammas, ns = _run("mid", w["prompt"], w["new"], tol_logits=2e-2, tol_alpha=2e-2, gain_jitter=0.0, max_seq=640)
    with capsys.disabled():
        print(f"[mid as named] {ck.summary()}", flush=True)
    assert ck.decisions > 1500


def test_kv_buffers_full_of_nans_do_not_matter():
    """Attention reads whole 32-position groups of the cache, including slots past the sequence's end; the
    caller's buffers arrive here with every byte 0xFF (f16 and f32 NaNs) and the results must not change:
    the library clears what it is given.  Prompt lengths that leave partly filled groups, both paths."""
    _run("mid", 45, 12, tol_logits=2e-2, tol_alpha=2e-2, kv_fill=0xFF)
    _run("tiny", 21, 12, tol_logits=1e-4, tol_alpha=1e-4, kv_fill=0xFF)


def test_mid_bf16_sampling_steps_match_oracle():
    _run("mid", 70, 24, tol_logits=2e-2, tol_alpha=2e-2, mode=po.SAMPLE, seed=3)


def test_7b_width_two_layers_bf16():
    """Full width, heads, FFN and vocabulary of the 7B-shaped target (d 4096, 32 heads of 128,
    FFN 11008, V 32000) at a depth the oracle can afford; 68M-shaped draft; gamma_max 16, b 4."""
    _run("7b", 100, 20, tol_logits=2e-2, tol_alpha=2e-2, n_layers_target=2,
         w_over=dict(mode="greedy"))


def test_7b_width_two_layers_sampling():
    """The headline workload's own decoding mode (stochastic sampling at temperature 1) at its width and
    vocabulary (d 4096, V 32000, gamma_max 16, b 4, beta 3): Gumbel-max draft tokens, the accept test
    r <= p/q and the residual resampling of Eq. 5 over 32000 entries, against the oracle on the same
    Philox streams."""
    _run("7b", 100, 24, tol_logits=2e-2, tol_alpha=2e-2, n_layers_target=2, mode=po.SAMPLE, seed=3)


def test_7b_width_long_context_4100_keys():
    """The long-context workload's regime (4096-token prompt) at the 7B width: 4100 prompt tokens, so every
    cache offset and position beyond 4096 is exercised, full windows (17 verify rows over more than 4100
    keys: 8 key splits per head for the target, 4 for the draft and the pre-verification layer, combined by
    the block that finishes last), prompt ingestion in nine 512-row passes."""
    _run("7b", 4100, 10, tol_logits=2e-2, tol_alpha=2e-2, n_layers_target=2, max_seq=4352,
         w_over=dict(mode="greedy"), step_kw=dict(force_stop=lambda k, a: False))


def test_prompt_ingestion_1500_tokens_first_alpha_and_first_verify():
    """Prompt ingestion (three passes of up to 512 rows through the wide GEMMs, the last one ragged, 16 slots of 32
    positions in the attention kernel; the target's last layer stops after its K/V) is checked by what is computed
    from the caches it leaves: the pre-verification layer's first alpha values (its prefix rows), the draft logits
    and every row of the first verify pass, against the oracle, with the halting test deciding the windows."""
    ck, gammas, _ = _run("7b", 1500, 12, tol_logits=2e-2, tol_alpha=2e-2, n_layers_target=2, max_seq=1664,
                         w_over=dict(mode="greedy"))
    assert ck.max_err["alpha"] > 0.0 and ck.max_err["target_logits"] > 0.0      # both were really compared


def test_7b_width_full_window_and_long_prompt():
    """gamma = gamma_max = 16 every step (17 verify rows: one full row tile + row 16), on a 2100-token
    prompt: the target's attention splits its keys over 8 blocks per head, the draft's and the
    pre-verification layer's over 2, and the block that finishes last combines the partial results."""
    _run("7b", 2100, 12, tol_logits=2e-2, tol_alpha=2e-2, n_layers_target=2, max_seq=2304,
         w_over=dict(mode="greedy"), step_kw=dict(force_stop=lambda k, a: False))


def _run_batch(name, prompt_lens, betas, n_steps, tol_logits, tol_alpha, mode=po.GREEDY, seed=5, max_seq=512,
               n_layers_target=None, fixed_gamma=None, ragged=True):
    """Several sequences in lock step (ragged verify batch, per-sequence gamma, beta and length)
    against one oracle per sequence."""
    w = synth.workload(name)
    tgt, drf, mb = synth.make_pair(w, seed=0, gain_jitter=0.1, n_layers_target=n_layers_target)
    nb = len(prompt_lens)
    s = _session(w, tgt, drf, mb, max_seq, max_batch=nb)
    cks = []
    ow = [helpers.to_oracle(m, cache=True) for m in (tgt, drf, mb)]      # one set of float64 copies for all oracles
    for i, (pl, beta) in enumerate(zip(prompt_lens, betas)):
        prompt = synth.make_prompt(w["target"]["vocab"], pl, 10 + i).tolist()
        o = helpers.build_oracle(w, ow[0], ow[1], ow[2], mode=mode, seed=seed, max_seq=max_seq, cache=True, seq=i, beta=beta)
        s.prefill(prompt, seq=i)
        o.prefill(prompt)
        cks.append(StepChecker(s, o, tol_logits, tol_alpha, mode=mode, seed=seed, seq=i))
    gam, full = [], []
    for _ in range(n_steps):
        idx = [ck.o.step_idx for ck in cks]
        ros = [ck.o.step(**({} if fixed_gamma is None else {"fixed_gamma": fixed_gamma})) for ck in cks]
        rgs = s.step_batch(list(range(nb)), mode=mode, betas=betas, seed=seed, record=True, fixed_gamma=fixed_gamma)
        for ck, ro, rg, k in zip(cks, ros, rgs, idx):
            ck.check(ro, rg, k)
        gam.append([r["gamma"] for r in ros])
        full.append([r["n"] == r["gamma"] for r in ros])
    for i, ck in enumerate(cks):
        assert s.tokens(i) == ck.o.tokens
    ties = [f for ck in cks for f in ck.ties()]
    werr = [f for ck in cks for f in ck.within_error()]
    decisions = sum(ck.decisions for ck in cks)
    print(f"\n[batch {name} x{nb} mode={mode}] gammas={gam} max_err={[ck.max_err['target_logits'] for ck in cks]} "
          f"decisions={decisions} ties={ties} within_error={werr}")
    assert len(werr) <= max(1, decisions // 50)
    assert not ragged or len({tuple(g) for g in gam}) > 1 or len(set(gam[0])) > 1      # the batch really was ragged
    s.close()
    return full


def test_batch_tiny_f32_ragged():
    _run_batch("tiny", [5, 33, 70], [4.0, 1.0, 2.5], 10, 1e-4, 1e-4)
    _run_batch("tiny", [9, 64], [4.0, 3.0], 8, 1e-4, 1e-4, mode=po.SAMPLE)


def test_batch_tiny_f32_sixteen_sequences():
    """The largest batch the library takes (16 sequences), f32 path, ragged prompts from 1 token up."""
    _run_batch("tiny", [1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 4, 6, 10, 16, 26, 42],
               [4.0, 1.0, 2.5, 3.0, 0.0, 4.5, 2.0, 3.5, 1.5, 5.0, 4.0, 0.5, 2.5, 3.0, 1.0, 4.0], 4, 1e-4, 1e-4, max_seq=256)


def test_batch_mid_bf16_ragged():
    """The batched workload in miniature: ragged batch, per-sequence beta in [1, 5], prompt lengths
    spread over several attention tiles; 4 sequences x up to 13 verify rows = two 32-row GEMM chunks."""
    _run_batch("mid", [40, 75, 150, 260], [1.0, 2.3, 3.7, 5.0], 6, 2e-2, 2e-2)


def test_batch_mid_bf16_key_splits_differ_per_sequence():
    """Three sequences of 30, 420 and 700 prompt tokens in one launch: the target's attention splits the
    keys in blocks of 192, so the first sequence has one block per head (it writes its output itself), the
    second three and the third four (combined by the block that finishes last), step after step on the
    same counters."""
    _run_batch("mid", [30, 420, 700], [3.0, 2.0, 4.0], 5, 2e-2, 2e-2, max_seq=1024)


def test_batch_mid_bf16_bonus_row_for_part_of_the_batch():
    """Strong coupling and a short fixed window make all-accepted steps frequent: in most steps only some
    of the sequences take the extra draft forward and the bonus row (Alg. 1, the all-accepted branch), whose
    logits then sit at other slots than the sequences' indices in the second acceptance pass."""
    for mode in (po.GREEDY, po.SAMPLE):
        full = _run_batch("mid", [40, 75, 150, 33], [8.0, 1.0, 6.0, 10.0], 8, 2e-2, 2e-2, mode=mode, fixed_gamma=2, ragged=False)
        assert any(any(f) and not all(f) for f in full)
        assert any(not f[0] and any(f[1:]) for f in full)      # a later sequence without the first: slot != index


def test_7b_width_two_sequences_full_windows():
    """Two sequences with 17 verify rows each (fixed window of 16) at the 7B width: 34 rows go through the
    wide GEMM, and attention runs as two one-tile blocks per (head, sequence)."""
    _run_batch("7b", [40, 75], [3.0, 4.0], 2, 2e-2, 2e-2, n_layers_target=2, fixed_gamma=16, ragged=False, max_seq=160)


def test_7b_width_two_sequences_eighteen_rows():
    """Two sequences with 9 verify rows each at the 7B width: 18 rows are two row tiles of the streaming GEMM
    (not the 17-row form), with the down projection's K split across blocks."""
    _run_batch("7b", [40, 75], [3.0, 4.0], 2, 2e-2, 2e-2, n_layers_target=2, fixed_gamma=8, ragged=False, max_seq=160)


def test_batch_mid_bf16_eight_sequences_wide_gemm():
    """8 sequences x up to 13 verify rows = up to 104 rows: the wide GEMM with several row groups per
    output-tile group, ragged last row tile, per-sequence attention over different lengths."""
    _run_batch("mid", [40, 75, 150, 260, 33, 97, 201, 64], [1.0, 2.3, 3.7, 5.0, 4.0, 3.0, 2.0, 4.5], 4, 2e-2, 2e-2)


def test_13b_width_four_layers_batch_against_oracle():
    """The shapes of workload `13b_batch` (d 5120, 40 heads of 128, FFN 13824, V 32000) at a depth the oracle can
    afford, 12 sequences, ragged prompts and windows, per-sequence beta: up to 204 verify rows through the
    wide GEMM at the widths bench.py times (K 5120 and 13824, 960 / 320 / 1728 / 2000 output tiles; 3 and 4
    row tiles per block, K slices for the few-tile matrices)."""
    _run_batch("13b_batch", [18, 33, 47, 25, 60, 39, 21, 52, 30, 44, 27, 36],
               [1.0, 2.0, 3.0, 4.0, 5.0, 2.5, 3.5, 1.5, 4.5, 2.0, 3.0, 4.0], 2, 2e-2, 2e-2, max_seq=160, n_layers_target=4)


def test_13b_width_ragged_prompts_in_the_named_range():
    """The batched workload's prompt-length range (256 to 2048 tokens) at its width (d 5120, 40 heads) and a depth the
    oracle can afford: three sequences of 300, 1100 and 2048 prompt tokens in one ragged verify launch (different
    numbers of 512-row prompt passes, different key ranges per sequence in one attention launch), per-sequence beta."""
    _run_batch("13b_batch", [300, 1100, 2048], [1.5, 3.0, 4.5], 2, 2e-2, 2e-2, max_seq=2176, n_layers_target=2)


def test_13b_width_ten_full_windows_six_row_tiles_per_block():
    """Ten sequences x 17 verify rows = 170 rows = 11 row tiles: the down and gate/up GEMMs run in the 8-wave
    wide kernel with two row groups of six row tiles (the largest operand stage, 96 KiB of LDS)."""
    _run_batch("13b_batch", [18, 33, 47, 25, 60, 39, 21, 52, 30, 44], [1.0, 2.0, 3.0, 4.0, 5.0, 2.5, 3.5, 1.5, 4.5, 2.0], 1, 2e-2, 2e-2,
               max_seq=160, n_layers_target=2, fixed_gamma=16, ragged=False)


def test_33b_width_two_layers_bf16():
    """Shapes of the large pair (target d 7168, 56 heads of 128, FFN 19200, V 32256; 24-layer d 2048
    draft with 128-wide heads): tile counts and K lengths none of the other tests has."""
    _run("33b", 40, 10, tol_logits=2e-2, tol_alpha=2e-2, n_layers_target=2, max_seq=128, w_over=dict(mode="greedy"))


def test_33b_width_eight_sequences_down_projection_k_slices():
    """Eight sequences x 13 verify rows = 104 rows at the 33B width: the down projection (448 output tiles)
    runs in the 8-wave wide kernel with two K slices across blocks (56 tile groups x 2 row groups x 2)."""
    _run_batch("33b", [12, 20, 9, 16, 14, 22, 11, 18], [3.0, 2.0, 4.0, 3.5, 2.5, 3.0, 4.5, 1.5], 1, 2e-2, 2e-2,
               n_layers_target=2, fixed_gamma=12, ragged=False, max_seq=64)


def test_13b_batch_full_depth_batch_invariance():
    """Workload `13b_batch` at full size (40 layers, 16 sequences) in the launch configuration bench.py
    times.  Property that holds at any size: a sequence verified inside the ragged batch (wide GEMM,
    rows of 16 sequences) gets the logits and decisions it gets when stepped alone (weight-streaming
    GEMM) from the same state."""
    w = synth.workload("13b_batch")
    tgt, drf, mb = synth.make_pair(w, seed=0, device="cuda")
    nb = 16
    s = _session(w, tgt, drf, mb, 256, max_batch=nb)
    del tgt, drf, mb
    torch.cuda.empty_cache()
    lens = synth.make_lengths(20, 150, nb, 4)
    betas = synth.make_betas(1.0, 5.0, nb, 5)
    prompts = [synth.make_prompt(32000, n, 30 + i).tolist() for i, n in enumerate(lens)]

    def fresh():
        for i, p in enumerate(prompts):
            s.prefill(p, seq=i)
        s.step_idx = [0] * nb

    fresh()
    batched = s.step_batch(list(range(nb)), betas=betas, record=True)
    rows = sum(r["gamma"] + 1 for r in batched)
    assert rows > 32                                            # the wide kernel really ran
    fresh()
    worst = 0.0
    for i in (0, 5, 10, 15):
        solo = s.step_batch([i], betas=[betas[i]], record=True)[0]
        b = batched[i]
        g = min(solo["gamma"], b["gamma"])
        assert solo["draft_tokens"][:g] == b["draft_tokens"][:g]
        if solo["gamma"] != b["gamma"]:
            # the pre-verification layer ran 64 rows through the wide GEMM in the batch and 4 rows through the
            # streaming one alone: a different window is allowed only at a near-tie of the block mean
            k = g // w["block"] - 1
            mean = float(np.mean(b["alpha"][k * w["block"]:(k + 1) * w["block"]]))
            assert abs(mean - w["t0"] * w["rho"] ** k) < 2e-3, (i, solo["gamma"], b["gamma"], mean)
            continue
        ls, lb = solo["target_logits"].double(), b["target_logits"].double()
        err = ((ls - lb).abs().amax(dim=1) / lb.pow(2).mean(dim=1).sqrt()).max().item()
        worst = max(worst, err)
        if (solo["n"], solo["z"]) != (b["n"], b["z"]):
            # allowed only at a near-tie of the deciding row's top two effective logits
            k = min(solo["n"], b["n"])
            eff = (lb[k] + betas[i] * b["draft_logits"][k].double()).cpu().numpy()
            top = np.sort(eff)[-2:]
            assert top[1] - top[0] < 2e-2 * np.sqrt(np.mean(eff ** 2)), (i, solo["n"], b["n"], top)
    print(f"\n[13b_batch full depth] rows={rows} batched vs solo logits max err {worst:.2e}")
    assert worst < 5e-3
    s.close()


def _host_copy(x):
    if isinstance(x, dict):
        return {k: _host_copy(v) for k, v in x.items()}
    if isinstance(x, list):
        return [_host_copy(v) for v in x]
    return x.cpu()


def test_7b_full_depth_headline_settings_against_oracle_and_losslessness(capsys):
    """Workload `7b` as BASELINE names it: full size (32 layers, d 4096, FFN 11008, V 32000; 68M-shaped draft),
    512-token prompt, stochastic sampling at temperature 1, gamma_max 16, b 4, beta 3, in the launch
    configuration bench.py times (weights generated on the device).  (i) Two sampling steps and one greedy
    step at that context are compared with the oracle row by row (every logit of every verify row, every
    draft logit, alpha, every integer decision).  (ii) Property that holds at any size: greedy speculative
    decoding emits the tokens of target-only greedy decoding run through the same kernels; a mismatch must
    sit at a near-tie of the GPU's own deciding logits.  (iii) The long-context workload's length at full depth
    (4096-token prompt, 32 layers), again by a property that holds at any size: row i of one 17-row verify pass
    equals the i-th of 17 single-token target passes over the same tokens (the KV-cached parallel forward of
    Eq. 4 against Eq. 1 step by step), here through different kernels (17-row form and split keys against the
    one-row shapes)."""
    from paper_2602_01274_amd import binding as B

    def say(msg):
        with capsys.disabled():
            print(f"[7b full depth] {msg}", flush=True)
    w = synth.workload("7b")
    assert w["mode"] == "sample" and w["prompt"] == 512
    tgt, drf, mb = synth.make_pair(w, seed=0, device="cuda")
    s = _session(w, tgt, drf, mb, 4352)
    host = (_host_copy(tgt), _host_copy(drf), _host_copy(mb))
    del tgt, drf, mb
    torch.cuda.empty_cache()
    prompt = synth.make_prompt(32000, w["prompt"], 1).tolist()
    o = helpers.build_oracle(w, host[0], host[1], host[2], mode=po.SAMPLE, seed=3, max_seq=640)
    s.prefill(prompt)
    say("oracle: 511-row prompt pass through 32 layers ...")
    o.prefill(prompt)
    ck = StepChecker(s, o, 2e-2, 2e-2, mode=po.SAMPLE, seed=3)
    for i in range(2):
        ro, _ = ck.step()
        say(f"sampling step {i}: gamma {ro['gamma']} n {ro['n']} {ck.summary()}")
    o.mode = ck.mode = po.GREEDY
    ro, _ = ck.step()
    say(f"greedy step: gamma {ro['gamma']} n {ro['n']} {ck.summary()}")
    ck.assert_flip_budget()
    assert s.tokens() == o.tokens
    # (ii) losslessness on the GPU itself, longer run, 300-token prompt
    w["mode"] = "greedy"
    prompt = synth.make_prompt(32000, 300, 2).tolist()
    s.prefill(prompt)
    spec, recs = s.generate(40, record=True)
    s.prefill(prompt)
    ar, recs_ar = s.generate(40, fixed_gamma=0, record=True)
    if spec != ar:
        k = next(i for i in range(40) if spec[i] != ar[i])
        # the autoregressive run's logits at that token: gap between its top two effective logits
        r = recs_ar[k]
        eff = (r["target_logits"][0] + w["beta"] * r["draft_logits"][0]).double().cpu().numpy()
        top = np.sort(eff)[-2:]
        say(f"speculative and autoregressive runs part at token {k}: top-2 gap {top[1] - top[0]:.2e}")
        assert top[1] - top[0] < 2e-2 * np.sqrt(np.mean(eff ** 2))
    assert any(r["n"] > 0 for r in recs) and any(r["n"] < r["gamma"] for r in recs)
    # (iii) 4096-token prompt: one 17-row verify pass against 17 one-row passes over the same tokens
    prompt = synth.make_prompt(32000, 4096, 4).tolist()
    s.prefill(prompt)
    one = s.step(fixed_gamma=16, record=True)
    rows, y = one["target_logits"].double(), one["draft_tokens"]
    s.prefill(prompt)
    worst = 0.0
    for i in range(17):
        r = s.step(fixed_gamma=0, record=True)
        single = r["target_logits"][0].double()
        err = ((single - rows[i]).abs().max() / rows[i].pow(2).mean().sqrt()).item()
        worst = max(worst, err)
        if i < 16:      # teacher forcing: the committed token becomes the draft the 17-row pass verified
            B.pacer_force_commit(s.ctx, 0, len(prompt) + i, [y[i]])
    say(f"4096-token prompt: 17-row verify pass against 17 single-token passes, max err / RMS {worst:.2e}")
    assert worst < 1e-2                # two f16 paths with different summation orders: half the tolerance against the oracle
    s.close()


def test_verify_twice_gives_the_same_bits():
    """The K slices of the down projection and the attention's key splits are added by whichever block finishes
    last, always in slice order: two verify passes over the same drafts (the second re-writes the same cache
    rows) must agree bit for bit, for 13 rows (8 key splits per head) and for 17 (two row-tile blocks per head)."""
    import torch
    from paper_2602_01274_amd import binding as B
    w = synth.workload("7b")
    tgt, drf, mb = synth.make_pair(w, seed=0, gain_jitter=0.1, n_layers_target=3)
    s = _session(w, tgt, drf, mb, 768)
    s.prefill(synth.make_prompt(w["target"]["vocab"], 600, 1).tolist())
    for gamma in (12, 16):
        B.pacer_begin_step(s.ctx, 0)
        for _ in range(gamma):
            B.pacer_draft_step(s.ctx, [0], B.GREEDY, 0, s.step_idx[0])
        B.pacer_verify(s.ctx, [0], None, s.logits)
        torch.cuda.synchronize()
        first = s.logits[0, :gamma + 1].clone()
        for _ in range(3):
            B.pacer_verify(s.ctx, [0], None, s.logits)
            torch.cuda.synchronize()
            assert torch.equal(first, s.logits[0, :gamma + 1])
        assert torch.isfinite(first).all()
        B.pacer_accept_rollback(s.ctx, [0], B.GREEDY, [w["beta"]], 0, s.step_idx[0], s.logits, s.n_acc, s.next_tok)
        B.pacer_get_state(s.ctx, 0)
        s.step_idx[0] += 1
    s.close()


def test_verify_twice_gives_the_same_bits_batched_13b_width():
    """The same guard for the batched kernels: ten sequences x 17 rows = 170 rows at the 13B width put the down
    projection through the 8-wave wide kernel with three K slices across blocks (partial tiles added by the
    block that finishes last), and prompts of 40 to 1500 tokens give the sequences one to several key splits
    in one attention launch.  Repeated verify passes over the same drafts must agree bit for bit; the run
    stops at the first mismatch."""
    from paper_2602_01274_amd import binding as B
    w = synth.workload("13b_batch")
    tgt, drf, mb = synth.make_pair(w, seed=0, gain_jitter=0.1, n_layers_target=2)
    lens = [40, 1500, 90, 700, 33, 1100, 260, 64, 900, 130]
    nb = len(lens)
    s = _session(w, tgt, drf, mb, 1600, max_batch=nb)
    seqs = list(range(nb))
    for i, n in enumerate(lens):
        s.prefill(synth.make_prompt(w["target"]["vocab"], n, 70 + i).tolist(), seq=i)
    for gamma in (16, 12):
        for i in seqs:
            B.pacer_begin_step(s.ctx, i)
        for _ in range(gamma):
            B.pacer_draft_step(s.ctx, seqs, B.GREEDY, 0, s.step_idx[0])
        B.pacer_verify(s.ctx, seqs, None, s.logits)
        torch.cuda.synchronize()
        first = s.logits[:, :gamma + 1].clone()
        assert torch.isfinite(first).all()
        for rep in range(3):
            B.pacer_verify(s.ctx, seqs, None, s.logits)
            torch.cuda.synchronize()
            assert torch.equal(first, s.logits[:, :gamma + 1]), f"gamma {gamma}: repeat {rep} differs"
        B.pacer_accept_rollback(s.ctx, seqs, B.GREEDY, [3.0] * nb, 0, s.step_idx[0], s.logits, s.n_acc, s.next_tok)
        for i in seqs:
            B.pacer_get_state(s.ctx, i)
            s.step_idx[i] += 1
    s.close()


def test_verify_can_be_captured_into_a_hip_graph():
    """pacer_verify only enqueues kernels on the context's stream (no allocation, no memset, no host wait), so a
    caller may capture it.  Captured on a side stream, the graph is replayed several times with eager passes and
    synchronisations between the replays; every replay must reproduce the eager bits (a pass writes the same
    cache rows and the same logits rows again).  A draft step is not replayed here: its last kernel already
    embeds the token it chose into the buffer the step started from, so the same step cannot run twice."""
    from paper_2602_01274_amd import binding as B
    w = synth.workload("7b")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        tgt, drf, mb = synth.make_pair(w, seed=0, gain_jitter=0.1, n_layers_target=3)
        s = _session(w, tgt, drf, mb, 768)
        s.prefill(synth.make_prompt(w["target"]["vocab"], 600, 1).tolist())
        for gamma in (12, 16):
            B.pacer_begin_step(s.ctx, 0)
            for _ in range(gamma):
                B.pacer_draft_step(s.ctx, [0], B.GREEDY, 0, s.step_idx[0])
            B.pacer_verify(s.ctx, [0], None, s.logits)
            torch.cuda.synchronize()
            first = s.logits[0, :gamma + 1].clone()
            assert torch.isfinite(first).all()
            gv = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gv, stream=side):
                B.pacer_verify(s.ctx, [0], None, s.logits)
            for rep in range(3):
                s.logits.zero_()
                gv.replay()
                torch.cuda.synchronize()
                assert torch.equal(first, s.logits[0, :gamma + 1]), f"gamma {gamma}: graph replay {rep} differs from the eager pass"
                s.logits.zero_()
                B.pacer_verify(s.ctx, [0], None, s.logits)                # eager work between the replays
                torch.cuda.synchronize()
                assert torch.equal(first, s.logits[0, :gamma + 1])
            del gv
            B.pacer_accept_rollback(s.ctx, [0], B.GREEDY, [w["beta"]], 0, s.step_idx[0], s.logits, s.n_acc, s.next_tok)
            st = B.pacer_get_state(s.ctx, 0)
            assert 0 <= st["n_accepted"] <= gamma
            s.step_idx[0] += 1
        s.close()


def test_wait_stop_and_get_state_match_the_device_buffers():
    """The host-polled words (stop flags, accept results) carry what the kernels wrote to the caller's
    device buffers, call after call, also across a re-prefill (tickets are never reused)."""
    from paper_2602_01274_amd import binding as B
    w = synth.workload("tiny")
    tgt, drf, mb = synth.make_pair(w, seed=0)
    s = _session(w, tgt, drf, mb, 256, max_batch=3)
    seqs = [0, 1, 2]
    with pytest.raises(B.PacerError) as e:
        B.pacer_wait_stop(s.ctx, [0])                       # nothing to wait for yet
    assert e.value.code == B.ESTATE
    for rnd in range(3):
        for i in seqs:
            s.prefill(synth.make_prompt(1024, 10 + 7 * i + rnd, 50 + i).tolist(), seq=i)
        for step in range(3):
            for i in seqs:
                B.pacer_begin_step(s.ctx, i)
            for blk in range(2):
                for _ in range(w["block"]):
                    B.pacer_draft_step(s.ctx, seqs, B.GREEDY, 0, step)
                B.pacer_preverify_block(s.ctx, seqs, s.alpha, s.stop)
                flags = B.pacer_wait_stop(s.ctx, seqs)
                assert flags == s.stop[:3].tolist()
            B.pacer_verify(s.ctx, seqs, None, s.logits)
            B.pacer_accept_rollback(s.ctx, seqs, B.GREEDY, [4.0, 1.0, 2.5], 0, step, s.logits, s.n_acc, s.next_tok)
            for k, i in enumerate(seqs):
                st = B.pacer_get_state(s.ctx, i)
                assert st["n_accepted"] == int(s.n_acc[k].item()) and st["next_token"] == int(s.next_tok[k].item())
    s.close()


def test_draft_window_call_equals_the_call_by_call_loop():
    """pacer_draft_window (the inner loop of Alg. 1 inside the library) against the same loop issued call by call:
    same windows, same accept counts and same tokens, single sequence (both modes) and a ragged batch."""
    for name, mode, n_prompt in (("tiny", po.GREEDY, 20), ("tiny", po.SAMPLE, 33), ("mid", po.GREEDY, 70)):
        w = synth.workload(name)
        tgt, drf, mb = synth.make_pair(w, seed=0, n_layers_target=2 if name == "mid" else None)
        s = _session(w, tgt, drf, mb, 512)
        prompt = synth.make_prompt(w["target"]["vocab"], n_prompt, 3).tolist()
        runs = []
        for record in (True, False):
            s.prefill(prompt)
            toks, recs = s.generate(40, mode=mode, seed=9, record=record)
            runs.append((toks, [(r["gamma"], r["n"], r["z"]) for r in recs]))
        assert runs[0] == runs[1]
        assert len({g for g, _, _ in runs[0][1]}) > 1                 # windows of several lengths occurred
        s.close()
    w = synth.workload("tiny")
    tgt, drf, mb = synth.make_pair(w, seed=0)
    s = _session(w, tgt, drf, mb, 256, max_batch=4)
    seqs, betas = [0, 1, 2, 3], [4.0, 1.0, 2.5, 3.0]
    runs = []
    for record in (True, False):
        for i in seqs:
            s.prefill(synth.make_prompt(1024, 7 + 9 * i, 40 + i).tolist(), seq=i)
        s.step_idx = [0] * 4
        out = []
        for _ in range(8):
            out.append([(r["gamma"], r["n"], r["z"]) for r in s.step_batch(seqs, betas=betas, record=record)])
        runs.append((out, [s.tokens(i) for i in seqs]))
    assert runs[0] == runs[1]
    assert len({g for step in runs[0][0] for g, _, _ in step}) > 1
    s.close()


def test_force_stop_overrides_the_device_flag_once():
    """pacer_force_stop: the next pre-verification call of that sequence writes the forced flag (to the device buffer
    and to the host-polled word) instead of its own decision, alpha is still computed, and the force is used up:
    the call after it decides by the rule again (mean alpha <= t in f32, recomputed here from the kernel's alpha)."""
    from paper_2602_01274_amd import binding as B
    w = synth.workload("tiny")
    tgt, drf, mb = synth.make_pair(w, seed=0)
    s = _session(w, tgt, drf, mb, 256, max_batch=3)
    seqs = [0, 1, 2]
    for i in seqs:
        s.prefill(synth.make_prompt(1024, 12 + 5 * i, 80 + i).tolist(), seq=i)
        B.pacer_begin_step(s.ctx, i)

    def natural(blk):
        t = np.float32(w["t0"])
        for _ in range(blk):
            t = np.float32(t * np.float32(w["rho"]))
        out = []
        for a in s.alpha[:3].tolist():
            acc = np.float32(0.0)
            for v in a:
                acc = np.float32(acc + np.float32(v))
            out.append(int(np.float32(acc / np.float32(len(a))) <= t))
        return out

    for blk, forces in enumerate(([1, 0, -1], [-1, -1, -1], [0, 1, 1])):
        for _ in range(w["block"]):
            B.pacer_draft_step(s.ctx, seqs, B.GREEDY, 0, 0)
        for i, f in zip(seqs, forces):
            if f >= 0:
                B.pacer_force_stop(s.ctx, i, f)
        B.pacer_preverify_block(s.ctx, seqs, s.alpha, s.stop)
        flags = B.pacer_wait_stop(s.ctx, seqs)
        assert flags == s.stop[:3].tolist()
        nat = natural(blk)
        assert flags == [f if f >= 0 else n for f, n in zip(forces, nat)], (blk, flags, forces, nat)
        assert all(0.0 < v < 1.0 for a in s.alpha[:3].tolist() for v in a)
    with pytest.raises(B.PacerError) as e:
        B.pacer_force_stop(s.ctx, 0, 2)
    assert e.value.code == B.EINVAL
    s.close()


def test_pack_weight_counts_values_beyond_the_half_range():
    """bf16 weights are held as half floats: a value beyond 65504 (or an inf / NaN in the source) cannot be represented,
    and pacer_pack_weight reports how many there were instead of decoding garbage silently."""
    from paper_2602_01274_amd import binding as B
    src = (torch.randn(64, 128, device="cuda") * 0.02).to(torch.bfloat16)
    dst = torch.empty_like(src)
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    B.pacer_pack_weight(dst, src, B.T_WO, 0, cnt, stream)
    torch.cuda.synchronize()
    assert int(cnt.item()) == 0
    src[3, 5] = 1.0e6
    src[40, 127] = float("inf")
    src[17, 0] = -70000.0
    src[9, 9] = 65000.0          # still a finite half
    B.pacer_pack_weight(dst, src, B.T_WO, 0, cnt, stream)
    torch.cuda.synchronize()
    assert int(cnt.item()) == 3
    B.pacer_pack_weight(dst, src, B.T_WO, 0, None, stream)      # the counter is optional
    torch.cuda.synchronize()
    # the engine refuses such a model
    w = synth.workload("mid")
    tgt, drf, mb = synth.make_pair(w, seed=0, n_layers_target=1)
    tgt["layers"][0]["wo"][2, 2] = 3.0e5
    with pytest.raises(B.PacerError) as e:
        _session(w, tgt, drf, mb, 128)
    assert e.value.code == B.EINVAL and "not finite" in str(e.value)


def test_capacity_errors_are_reported_not_faulted():
    """KV capacity and window limits are host-checked: the calls fail with PACER_EOVERFLOW /
    PACER_ESTATE and leave the sequence usable."""
    from paper_2602_01274_amd import binding as B
    w = synth.workload("tiny")
    tgt, drf, mb = synth.make_pair(w, seed=0)
    s = _session(w, tgt, drf, mb, 64)                      # room for 64 positions only
    with pytest.raises(B.PacerError) as e:
        s.prefill(list(range(60)))                          # leaves no room for a step
    assert e.value.code == B.EOVERFLOW
    s.prefill(list(range(40)))
    B.pacer_begin_step(s.ctx, 0)
    for _ in range(w["gamma_max"]):
        B.pacer_draft_step(s.ctx, [0], B.GREEDY, 0, 0)
    with pytest.raises(B.PacerError) as e:
        B.pacer_draft_step(s.ctx, [0], B.GREEDY, 0, 0)      # beyond gamma_max
    assert e.value.code == B.EOVERFLOW
    with pytest.raises(B.PacerError) as e:
        B.pacer_accept_rollback(s.ctx, [0], B.GREEDY, [1.0], 0, 0, s.logits, s.n_acc, s.next_tok)   # not verified yet
    assert e.value.code == B.ESTATE
    with pytest.raises(B.PacerError) as e:
        B.pacer_preverify_block(s.ctx, [0], s.alpha, s.stop)   # 8 new drafts, block is 2
    assert e.value.code == B.ESTATE
    B.pacer_verify(s.ctx, [0], None, s.logits)
    B.pacer_accept_rollback(s.ctx, [0], B.GREEDY, [4.0], 0, 0, s.logits, s.n_acc, s.next_tok)
    st = B.pacer_get_state(s.ctx, 0)
    assert st["len"] == 40 + st["n_accepted"] + 1 and 0 <= st["n_accepted"] <= w["gamma_max"]
    while True:                                             # run into the end of the cache
        try:
            s.step()
        except B.PacerError as e2:
            assert e2.code == B.EOVERFLOW
            break
    assert B.pacer_get_state(s.ctx, 0)["len"] + w["gamma_max"] + 2 > 64
    s.close()


@pytest.mark.parametrize("name", ["tiny", "mid"])
def test_prompt_token_outside_the_vocabulary_is_reported_not_faulted(name):
    """Token ids live on the device, so the library cannot refuse a bad prompt up front.  No kernel may use such
    an id as an index: the prompt copy replaces it by a valid id and flags the sequence, the step's first
    read-back returns PACER_ENUMERIC, the sequence takes no further step, and a new prefill reopens it
    (f32 path: tiny, bf16 path: mid)."""
    from paper_2602_01274_amd import binding as B
    w = synth.workload(name)
    tgt, drf, mb = synth.make_pair(w, seed=0)
    V = w["target"]["vocab"]
    s = _session(w, tgt, drf, mb, 256)
    good = synth.make_prompt(V, 20, 1).tolist()
    for bad_id in (V + 7, -3, 2**31 - 1):
        bad = list(good)
        bad[5] = bad_id
        s.prefill(bad)
        with pytest.raises(B.PacerError) as e:
            s.step(mode=B.GREEDY)
        assert e.value.code == B.ENUMERIC, str(e.value)
        with pytest.raises(B.PacerError) as e:
            B.pacer_begin_step(s.ctx, 0)
        assert e.value.code == B.ENUMERIC
    s.prefill(good)
    r = s.step(mode=B.GREEDY)
    assert r["n"] >= 0 and 0 <= r["z"] < V
    s.close()


def test_logits_without_a_finite_value_are_reported_not_faulted():
    """A draft model whose final norm gain holds a NaN produces logits with no finite value: the token choice has
    no winner.  The chosen id must still be a valid index (the same kernel embeds it at once), and the step ends
    with PACER_ENUMERIC instead of tokens; the same for a target model with such a gain."""
    from paper_2602_01274_amd import binding as B
    w = synth.workload("mid")
    V = w["target"]["vocab"]
    prompt = synth.make_prompt(V, 20, 1).tolist()
    for which in ("draft", "target"):
        tgt, drf, mb = synth.make_pair(w, seed=0)
        m = drf if which == "draft" else tgt
        m["final_norm"] = m["final_norm"].clone()
        m["final_norm"][:] = float("nan")
        s = _session(w, tgt, drf, mb, 256)
        s.prefill(prompt)
        for mode in (B.GREEDY, B.SAMPLE):
            with pytest.raises(B.PacerError) as e:
                s.step(mode=mode)
            assert e.value.code == B.ENUMERIC, (which, mode, str(e.value))
            torch.cuda.synchronize()
            toks = s.draft_tokens(0)[:w["block"]]          # the drafts of the first block were made in either case
            assert int(toks.min()) >= 0 and int(toks.max()) < V
            s.prefill(prompt)
        s.close()
