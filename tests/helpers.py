"""Glue shared by the tests: turn the synthetic torch weights into the arrays the CPU
oracle takes (test-side only; the product path never touches the oracle)."""
import numpy as np
import torch

from oracle import pacer_oracle as po


class LazyF64:
    """A torch tensor (any float dtype, host) that widens to float64 only when used."""

    def __init__(self, t, cache=False):
        self.t = t
        self.cache = cache
        self._a = None

    def __array__(self, dtype=None, copy=None):
        if self._a is not None:
            return self._a
        a = self.t.detach().cpu().to(torch.float64).numpy()
        if self.cache:
            self._a = a
        return a

    def __getitem__(self, idx):
        return self.t[torch.as_tensor(np.asarray(idx))].detach().cpu().to(torch.float64).numpy()


def to_oracle(w, cache=False):
    """cache=True keeps the float64 copies (8 bytes per weight): small and mid models only."""
    if isinstance(w, LazyF64):          # already converted (several oracles sharing one set of float64 copies)
        return w
    if isinstance(w, dict):
        return {k: to_oracle(v, cache) for k, v in w.items()}
    if isinstance(w, list):
        return [to_oracle(v, cache) for v in w]
    return LazyF64(w, cache)


def oracle_cfg(shape):
    return po.ModelCfg(shape["n_layers"], shape["d_model"], shape["n_heads"], shape["head_dim"],
                       shape["d_ffn"], shape["vocab"], shape["rope_theta"], shape["rms_eps"])


def build_oracle(w, tgt, drf, mb, mode=None, seed=0, max_seq=None, cache=False, **kw):
    mode = mode if mode is not None else (po.SAMPLE if w["mode"] == "sample" else po.GREEDY)
    args = dict(block=w["block"], gamma_max=w["gamma_max"], t0=w["t0"], rho=w["rho"],
                beta=w["beta"], mode=mode, seed=seed,
                max_seq=max_seq or 4096)
    args.update(kw)
    ct = oracle_cfg(dict(w["target"], n_layers=len(tgt["layers"])))
    return po.PacerOracle(to_oracle(tgt, cache), ct, to_oracle(drf, cache),
                          oracle_cfg(w["draft"]), to_oracle(mb, cache) if mb is not None else None, **args)
