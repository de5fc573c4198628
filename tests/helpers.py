"""Glue shared by the tests: turn the synthetic torch weights into the arrays the CPU
oracle takes (test-side only; the product path never touches the oracle)."""
import numpy as np
import torch

from oracle import pacer_oracle as po


class LazyF64:
    """A torch tensor (any float dtype, host) that widens to float64 only when used."""

    def __init__(self, t):
        self.t = t

    def __array__(self, dtype=None, copy=None):
        return self.t.detach().cpu().to(torch.float64).numpy()

    def __getitem__(self, idx):
        return self.t[torch.as_tensor(np.asarray(idx))].detach().cpu().to(torch.float64).numpy()


def to_oracle(w):
    if isinstance(w, dict):
        return {k: to_oracle(v) for k, v in w.items()}
    if isinstance(w, list):
        return [to_oracle(v) for v in w]
    return LazyF64(w)


def oracle_cfg(shape):
    return po.ModelCfg(shape["n_layers"], shape["d_model"], shape["n_heads"], shape["head_dim"],
                       shape["d_ffn"], shape["vocab"], shape["rope_theta"], shape["rms_eps"])


def build_oracle(w, tgt, drf, mb, mode=None, seed=0, max_seq=None, **kw):
    mode = mode if mode is not None else (po.SAMPLE if w["mode"] == "sample" else po.GREEDY)
    args = dict(block=w["block"], gamma_max=w["gamma_max"], t0=w["t0"], rho=w["rho"],
                beta=w["beta"], mode=mode, seed=seed,
                max_seq=max_seq or 4096)
    args.update(kw)
    return po.PacerOracle(to_oracle(tgt), oracle_cfg(w["target"]), to_oracle(drf),
                          oracle_cfg(w["draft"]), to_oracle(mb) if mb is not None else None, **args)
