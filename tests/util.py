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
                           layers, to_f64(tm["embed"]), to_f64(tm["lm_head"]), to_f64(tm["final_norm"]),
                           n_kv_heads=shape.kv_heads, qk_norm=shape.qk_norm)


def gpu_model(shape, tm, max_B, cap, max_rows=0):
    """The HIP-side model built from the same stored weight bytes as `oracle_model`."""
    from paper_2604_02047_amd import ModelDesc
    from paper_2604_02047_amd.runner import GooseModel
    return GooseModel(ModelDesc.from_shape(shape), max_B, cap, lambda l: tm["layers"][l], tm["embed"],
                      tm["lm_head"], tm["final_norm"], max_rows=max_rows)


def load_prefix_cache(gm, cache):
    """Copies an oracle cache (list of (K,V) float64 [n_h,P,d]) into the device cache (rounded to its type)."""
    P = cache[0][0].shape[1]
    for l, (k, v) in enumerate(cache):
        gm.write_rows(l, torch.from_numpy(k), torch.from_numpy(v))
    gm.set_P(P)


def device_cache_as_oracle(gm, P):
    """The device cache's first P slots as an oracle cache (exact upcast of the stored values)."""
    kr, vr = gm.k_rows(0, P), gm.v_rows(0, P)
    return [(kr[l].to(torch.float64).cpu().numpy(), vr[l].to(torch.float64).cpu().numpy())
            for l in range(gm.desc.n_layers)]
