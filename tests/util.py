"""Test helpers: turn generated inputs into the oracle's float64 model (marshalling only)."""
import numpy as np
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


class LazyLayers:
    """Sequence of per-layer float64 weight dicts, built on demand (keeps one layer alive)."""

    def __init__(self, n, fn):
        self._n, self._fn = n, fn
        self._last = (None, None)

    def __len__(self):
        return self._n

    def __getitem__(self, l):
        if self._last[0] != l:
            self._last = (l, self._fn(l))
        return self._last[1]


def torch_model(shape, seed=0, gain_jitter=0.0, device="cpu"):
    """The stored weight bytes (torch tensors) of a whole model."""
    return {
        "layers": [gi.layer_weights(shape, seed, l, device, gain_jitter=gain_jitter)
                   for l in range(shape.n_layers)],
        "embed": gi.embedding(shape, seed, device),
        "lm_head": gi.lm_head(shape, seed, device),
        "final_norm": gi.final_norm(shape, seed, device, gain_jitter),
    }


def oracle_model(shape, tm) -> orc.OracleModel:
    layers = [{k: to_f64(v) for k, v in lw.items()} for lw in tm["layers"]]
    return orc.OracleModel(shape.n_heads, shape.head_dim, shape.rope_base, shape.rms_eps,
                           layers, to_f64(tm["embed"]), to_f64(tm["lm_head"]), to_f64(tm["final_norm"]))
