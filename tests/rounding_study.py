#!/usr/bin/env python3
"""Where does the 16-bit path's logit error come from?  (CPU only; test infrastructure.)

Re-runs the oracle's arithmetic (fp64 NumPy, same formulas as oracle/goose_oracle.py) on one
verification step of a benchmark shape, with bf16 rounding switched on at chosen points of the
layer -- the points at which the HIP path stores a 16-bit value -- and reports the largest logit
error of every variant relative to the exact pass, as a fraction of the logit scale max|logit|.

Rounding points of a decoder layer:
  xn1  normalised input of the q|k|v projection        xn2  normalised input of the gate/up projection
  q    rotated query                                   k    rotated key (what the cache stores)
  v    value (what the cache stores)                   p    unnormalised softmax probabilities
  o    attention output (input of the O projection)    h    SwiGLU output (input of the down projection)
  xf   normalised input of the LM head
"hilo" variants replace a rounding by the sum of two bf16 values (the value and its remainder),
which is what a two-term split of a projection's activation operand would carry.

The KV prefix of every variant is the same stored (bf16-rounded) prefix, produced by an exact
prefill, as in the GPU parity tests (the prefix is an input there).

    python tests/rounding_study.py [--shape 7b] [--B 64] [--P 1024] [--layers N]
"""
import argparse
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import goose_inputs as gi  # noqa: E402
from oracle import goose_oracle as orc  # noqa: E402

POINTS = ("xn1", "q", "k", "v", "p", "o", "xn2", "h", "xf")


def bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def hilo(a):
    hi = bf16(a)
    return hi + bf16(a - hi)


def rnd(a, mode):
    return a if mode == 0 else (bf16(a) if mode == 1 else hilo(a))


def layer(model, w, x, Kc, Vc, pos, allow, cfg):
    """oracle.decoder_layer with a rounding mode (0 exact, 1 bf16, 2 two-term) at every point."""
    T = x.shape[0]
    n_h, n_kv, d = model.n_heads, model.n_kv_heads, model.head_dim
    xn = rnd(orc.rmsnorm(x, w["g1"], model.rms_eps), cfg["xn1"])
    q = orc.rope((xn @ w["wq"].T).reshape(T, n_h, d), pos, model.rope_base)
    k = orc.rope((xn @ w["wk"].T).reshape(T, n_kv, d), pos, model.rope_base)
    v = (xn @ w["wv"].T).reshape(T, n_kv, d)
    q, k, v = rnd(q, cfg["q"]), rnd(k, cfg["k"]), rnd(v, cfg["v"])
    K = np.concatenate([Kc, k.transpose(1, 0, 2)], axis=1)
    V = np.concatenate([Vc, v.transpose(1, 0, 2)], axis=1)
    o = np.empty((T, n_h, d))
    group = n_h // n_kv
    for hd in range(n_h):
        s = q[:, hd, :] @ K[hd // group].T / np.sqrt(d)
        s = np.where(allow, s, -np.inf)
        e = np.exp(s - s.max(axis=-1, keepdims=True))
        o[:, hd, :] = (rnd(e, cfg["p"]) @ V[hd // group]) / e.sum(axis=-1, keepdims=True)
    o = rnd(o.reshape(T, n_h * d), cfg["o"])
    x = x + o @ w["wo"].T
    xn2 = rnd(orc.rmsnorm(x, w["g2"], model.rms_eps), cfg["xn2"])
    h = rnd(orc.silu(xn2 @ w["wg"].T) * (xn2 @ w["wu"].T), cfg["h"])
    return x + h @ w["wd"].T


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="7b")
    ap.add_argument("--B", type=int, default=64)
    ap.add_argument("--P", type=int, default=1024)
    ap.add_argument("--layers", type=int, default=0, help="first N layers only (0 = all)")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    shape = gi.SHAPES[args.shape]
    L = args.layers or shape.n_layers
    B, P = args.B, args.P
    tree = gi.tree_spine_7b(args.seed) if B == 64 else gi.tree_random(B, seed=args.seed, spine_len=min(16, B - 1))
    assert tree.B == B
    f64 = lambda t: t.to(torch.float64).numpy()  # noqa: E731

    def cfg(**kw):
        c = dict.fromkeys(POINTS, 0)
        c.update(kw)
        return c

    every = dict.fromkeys(POINTS, 1)
    variants = {"exact": cfg(), "all bf16 (the path as built before)": dict(every)}
    for pt in POINTS:
        variants[f"only {pt}"] = cfg(**{pt: 1})
    variants["only k,v (what bf16 storage of the cache forces)"] = cfg(k=1, v=1)
    variants["k,v,q,p (projection operands exact)"] = cfg(k=1, v=1, q=1, p=1)
    variants["all, projection operands two-term (xn1,xn2,o,h,xf)"] = dict(every, xn1=2, xn2=2, o=2, h=2, xf=2)
    variants["all, projection operands and q,p two-term"] = dict(every, xn1=2, xn2=2, o=2, h=2, xf=2, q=2, p=2)
    variants["all, xn1,xn2,xf two-term"] = dict(every, xn1=2, xn2=2, xf=2)
    variants["all, o,h two-term"] = dict(every, o=2, h=2)

    model = orc.OracleModel(shape.n_heads, shape.head_dim, shape.rope_base, shape.rms_eps, [None] * L, None, None,
                            None, n_kv_heads=shape.kv_heads)
    embed = f64(gi.embedding(shape, args.seed))
    prefix = gi.prefix_tokens(args.seed, P, shape.vocab)
    tokens = gi.draft_tokens_uniform(args.seed + 1, tree.parent, shape.vocab, 7)
    anc, depth = orc.ancestor_mask(tree.parent)
    allow = np.concatenate([np.ones((B, P), bool), anc], axis=1)
    pos = P + depth.astype(np.int64)
    xp = embed[prefix.astype(np.int64)]
    causal = np.tril(np.ones((P, P), bool))
    z = np.zeros((shape.kv_heads, 0, shape.head_dim))
    xs = {name: embed[tokens.astype(np.int64)].copy() for name in variants}
    t0 = time.time()
    for l in range(L):
        w = {k: f64(v) for k, v in gi.layer_weights(shape, args.seed, l).items()}
        # exact prefill of this layer; the cache keeps its bf16 rounding (the stored prefix is an input)
        xp, kp, vp = orc.decoder_layer(model, w, xp, z, z, np.arange(P), causal)
        Kc, Vc = bf16(kp), bf16(vp)
        for name, c in variants.items():
            xs[name] = layer(model, w, xs[name], Kc, Vc, pos, allow, c)
        ref = xs["exact"]
        line = ", ".join(f"{n.split(' ')[0]} {np.abs(xs[n] - ref).max() / np.abs(ref).max():.2e}"
                         for n in ("all bf16 (the path as built before)",))
        print(f"layer {l + 1}/{L} ({time.time() - t0:.0f}s): hidden-state error, {line}", flush=True)
        del w
    gf, wl = f64(gi.final_norm(shape, args.seed)), f64(gi.lm_head(shape, args.seed))
    logits = {n: rnd(orc.rmsnorm(xs[n], gf, shape.rms_eps), variants[n]["xf"]) @ wl.T for n in variants}
    ref = logits["exact"]
    scale = np.abs(ref).max()
    print(f"\n{shape.name}, {L} layers, B={B}, P={P}: logit scale {scale:.3f}")
    print(f"{'variant':62s} max|err|/scale   rms err/scale")
    for n in variants:
        e = logits[n] - ref
        print(f"{n:62s} {np.abs(e).max() / scale:10.3e}   {np.sqrt((e * e).mean()) / scale:10.3e}")


if __name__ == "__main__":
    main()
