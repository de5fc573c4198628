"""Seeded synthetic inputs: model shapes, random-init weights, prompts.

This module holds no arithmetic of the method.  It only produces the inputs that both the
HIP library (through the binding) and the CPU checker are fed with, so that the two see
identical bits.  The synthetic models stand in for the paper's real draft/target pairs
(Sec. 4.1, "Models") and the uniform-random prompts for its benchmark prompts
(Sec. 4.1, "Evaluation Datasets"), none of which are available here.

Recipe: every matrix and embedding ~ N(0, 0.02^2); RMSNorm gains = 1 (optionally
1 + 0.1*N(0,1) for tests that must notice a dropped gain); bf16 models round the matrices
to bf16 (round-to-nearest-even) once, here, so that every consumer loads the same values;
M_B's 2-class head ~ N(0, (1.5/sqrt(2d))^2); draft-position table row 0 = 0, other rows
N(0, 0.02^2); prompts are i.i.d. uniform token ids.  One generator stream per tensor, so
a tensor does not depend on the order of generation.
"""
import copy

import torch

# name -> dict(target=..., draft=..., block, gamma_max, beta, prompt, new, mode, dtype, share)
_SHAPES = {
    "tiny": dict(
        target=dict(n_layers=4, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024),
        draft=dict(n_layers=1, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024),
        share_embed_head=True, dtype="f32", block=2, gamma_max=8, beta=4.0,
        prompt=32, new=64, mode="greedy"),
    "mid": dict(
        target=dict(n_layers=12, d_model=768, n_heads=12, head_dim=64, d_ffn=2048, vocab=32000),
        draft=dict(n_layers=2, d_model=768, n_heads=12, head_dim=64, d_ffn=2048, vocab=32000),
        share_embed_head=True, dtype="bf16", block=4, gamma_max=12, beta=3.0,
        prompt=128, new=256, mode="greedy"),
    "7b": dict(
        target=dict(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32000),
        draft=dict(n_layers=2, d_model=768, n_heads=12, head_dim=64, d_ffn=3072, vocab=32000),
        share_embed_head=False, dtype="bf16", block=4, gamma_max=16, beta=3.0,
        prompt=512, new=512, mode="sample"),
    "7b_long": dict(
        target=dict(n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008, vocab=32000),
        draft=dict(n_layers=2, d_model=768, n_heads=12, head_dim=64, d_ffn=3072, vocab=32000),
        share_embed_head=False, dtype="bf16", block=4, gamma_max=16, beta=3.0,
        prompt=4096, new=256, mode="greedy"),
    "13b_batch": dict(
        target=dict(n_layers=40, d_model=5120, n_heads=40, head_dim=128, d_ffn=13824, vocab=32000),
        draft=dict(n_layers=2, d_model=768, n_heads=12, head_dim=64, d_ffn=3072, vocab=32000),
        share_embed_head=False, dtype="bf16", block=4, gamma_max=16, beta=None,
        prompt=(256, 2048), new=256, mode="greedy", batch=16),
    # a pair at the scale of the paper's larger experiments (Sec. 4.1: 1.3B draft, 33B target), where the
    # draft step itself streams gigabytes: Llama-shaped, multi-head attention, 33.6 B and 1.35 B parameters
    "33b": dict(
        target=dict(n_layers=54, d_model=7168, n_heads=56, head_dim=128, d_ffn=19200, vocab=32256),
        draft=dict(n_layers=24, d_model=2048, n_heads=16, head_dim=128, d_ffn=5504, vocab=32256),
        share_embed_head=False, dtype="bf16", block=4, gamma_max=16, beta=3.0,
        prompt=512, new=256, mode="sample"),
}
T0_DEFAULT = 0.5
RHO_DEFAULT = 1.05
ROPE_THETA = 10000.0
RMS_EPS = 1e-5


def workload(name):
    """A deep copy of the named workload description (shapes and decode settings)."""
    w = copy.deepcopy(_SHAPES[name])
    w["name"] = name
    w.setdefault("batch", 1)
    w["t0"], w["rho"] = T0_DEFAULT, RHO_DEFAULT
    for m in ("target", "draft"):
        w[m]["rope_theta"], w[m]["rms_eps"] = ROPE_THETA, RMS_EPS
    return w


def _stream(seed, model_id, layer, tensor_id, device):
    g = torch.Generator(device=device)
    g.manual_seed(((seed * 1009 + model_id) * 1009 + layer + 1) * 1009 + tensor_id)
    return g


def _normal(shape, std, seed, model_id, layer, tensor_id, device, store):
    g = _stream(seed, model_id, layer, tensor_id, device)
    if store == torch.bfloat16 and device != "cpu":
        # large models: draw straight into bf16 storage on the device, in slabs
        out = torch.empty(shape, dtype=torch.bfloat16, device=device)
        flat = out.view(-1)
        step = 1 << 26
        for s in range(0, flat.numel(), step):
            n = min(step, flat.numel() - s)
            flat[s:s + n] = (torch.randn(n, generator=g, device=device) * std).to(torch.bfloat16)
        return out
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std
    return t.to(store)


def _gain(d, seed, model_id, layer, tensor_id, device, jitter):
    if jitter == 0.0:
        return torch.ones(d, dtype=torch.float32, device=device)
    g = _stream(seed, model_id, layer, tensor_id, device)
    return 1.0 + jitter * torch.randn(d, generator=g, device=device, dtype=torch.float32)


def _layer(shape, seed, model_id, l, device, store, jitter):
    d, f = shape["d_model"], shape["d_ffn"]
    n = lambda s, tid: _normal(s, 0.02, seed, model_id, l, tid, device, store)
    return {
        "attn_norm": _gain(d, seed, model_id, l, 0, device, jitter),
        "wq": n((d, d), 1), "wk": n((d, d), 2), "wv": n((d, d), 3), "wo": n((d, d), 4),
        "ffn_norm": _gain(d, seed, model_id, l, 5, device, jitter),
        "wg": n((f, d), 6), "wu": n((f, d), 7), "wd": n((d, f), 8),
    }


def make_lm(shape, seed, model_id, dtype="bf16", device="cpu", gain_jitter=0.0, share=None):
    """Random-init decoder LM.  Linear weights are [out, in].  share: another LM whose
    embedding and LM head are reused (the tiny and mid pairs)."""
    store = torch.bfloat16 if dtype == "bf16" else torch.float32
    d, v = shape["d_model"], shape["vocab"]
    w = {"layers": [_layer(shape, seed, model_id, l, device, store, gain_jitter)
                    for l in range(shape["n_layers"])]}
    if share is not None:
        w["embed"], w["head"] = share["embed"], share["head"]
    else:
        w["embed"] = _normal((v, d), 0.02, seed, model_id, -1, 0, device, store)
        w["head"] = _normal((v, d), 0.02, seed, model_id, -1, 1, device, store)
    w["final_norm"] = _gain(d, seed, model_id, -1, 2, device, gain_jitter)
    return w


def make_preverify(draft_shape, gamma_max, seed, dtype="bf16", device="cpu", gain_jitter=0.0):
    """Random-init pre-verification layer of draft width: one decoder layer, final norm,
    2-class head, additive draft-position table (row 0 is the prefix row and stays zero)."""
    store = torch.bfloat16 if dtype == "bf16" else torch.float32
    d = draft_shape["d_model"]
    mb = {"layer": _layer(draft_shape, seed, 7, 0, device, store, gain_jitter),
          "final_norm": _gain(d, seed, 7, -1, 2, device, gain_jitter)}
    mb["cls"] = _normal((2, d), 1.5 / (2.0 * d) ** 0.5, seed, 7, -1, 3, device, torch.float32)
    pe = _normal((gamma_max + 1, d), 0.02, seed, 7, -1, 4, device, torch.float32)
    pe[0] = 0.0
    mb["posemb"] = pe
    return mb


def make_pair(w, seed=0, device="cpu", gain_jitter=0.0, n_layers_target=None):
    """(target, draft, preverify) weights of a workload.  n_layers_target truncates the
    target's depth (full-width models for tests that cannot afford the full depth)."""
    ts = dict(w["target"])
    if n_layers_target is not None:
        ts["n_layers"] = n_layers_target
    tgt = make_lm(ts, seed, 1, w["dtype"], device, gain_jitter)
    drf = make_lm(w["draft"], seed, 2, w["dtype"], device, gain_jitter,
                  share=tgt if w["share_embed_head"] else None)
    mb = make_preverify(w["draft"], w["gamma_max"], seed + 2, w["dtype"], device, gain_jitter)
    return tgt, drf, mb


def make_prompt(vocab, n, seed):
    g = torch.Generator()
    g.manual_seed(1_000_003 * (seed + 1))
    return torch.randint(0, vocab, (n,), generator=g, dtype=torch.int64).to(torch.int32)


def make_lengths(lo, hi, n, seed):
    g = torch.Generator()
    g.manual_seed(2_000_003 * (seed + 1))
    return torch.randint(lo, hi + 1, (n,), generator=g, dtype=torch.int64).tolist()


def make_betas(lo, hi, n, seed):
    g = torch.Generator()
    g.manual_seed(3_000_017 * (seed + 1))
    return (lo + (hi - lo) * torch.rand(n, generator=g, dtype=torch.float64)).tolist()
