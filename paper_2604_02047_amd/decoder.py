"""Sequencing of whole decoding cycles (Alg. "Decoding Loop") on top of the C ABI.

Every decision and every computation is a library call: the n-gram match, the routing, the tree
builder, tiers and moving average are host functions of libgoose; verification, harvest, walk and
compaction run on the GPU (goose_verify_step, goose_verify_step_batched).  This module only moves
small arrays between them: per cycle it uploads the trees (a few hundred bytes each) and reads back
the walks' results and the table rows the harvest touched.

GooseDecoder decodes one request; BatchedGooseDecoder decodes several with one pass over the
weights per cycle (the batch sweep of App. D), each request with its own KV cache, successor
tables and adaptive state, and drops a request from the batch as soon as it has its tokens.
"""
import numpy as np
import torch

from . import binding as gb
from .runner import GooseModel


class _Request:
    """The state of one request: KV cache and its length, successor tables (device, and a host mirror
    for the tree builder), the token sequence, the anchor and the spine-acceptance average."""

    def __init__(self, gm: GooseModel, K, kcache=None, vcache=None):
        V, dev = gm.desc.vocab, gm.device
        i32 = dict(dtype=torch.int32, device=dev)
        self.gm, self.K = gm, K
        self.kcache = gm.kcache if kcache is None else kcache
        self.vcache = gm.vcache if vcache is None else vcache
        self.P = 0
        self.d_P = torch.zeros(1, **i32)
        self.accept_len, self.bonus = torch.zeros(1, **i32), torch.zeros(1, **i32)
        self.path, self.argmax = torch.zeros(gm.max_B, **i32), torch.zeros(gm.max_B, **i32)
        self.d_ids = torch.full((V, K), -1, **i32)                       # written by the harvest kernel
        self.d_scores = torch.zeros((V, K), dtype=torch.float32, device=dev)
        self.h_ids = np.full((V, K), -1, np.int32)                       # host mirror for the tree builder
        self.h_scores = np.zeros((V, K), np.float32)
        self.seq, self.p_hat, self.anchor = [], 0.3, None
        self.trace = []

    def mirror_rows(self, tokens):
        idx = torch.as_tensor(np.unique(np.asarray(tokens, np.int64)), device=self.gm.device)
        self.h_ids[idx.cpu().numpy()] = self.d_ids[idx].cpu().numpy()
        self.h_scores[idx.cpu().numpy()] = self.d_scores[idx].cpu().numpy()

    def prefill(self, prompt):
        """Feeds the prompt through the verification path as chain trees (every row kept), harvests every
        position's logits, and returns the first generated token."""
        gm, c = self.gm, self.gm.ctx
        prompt = [int(t) for t in prompt]
        done, step = 0, gm.max_B
        while done < len(prompt):
            n = min(step, len(prompt) - done)
            chunk = prompt[done:done + n]
            t, p, s = gm.stage_tree(chunk, np.arange(-1, n - 1), np.ones(n, np.uint8))
            W = (n + 63) // 64
            mask = gm.mask.view(-1)[:n * W]
            c.goose_build_mask(p, n, done, mask, gm.depth, gm.pos)
            c.goose_embed(gm.embed, t, n, gm.x)
            for l in range(gm.desc.n_layers):
                c.goose_verify_layer(gm.packed_layer(l), gm.x, self.kcache[l], self.vcache[l], done, n, mask, gm.pos)
            logits = torch.empty((n, gm.desc.vocab), dtype=torch.float32, device=gm.device)
            c.goose_lm_head_argmax(gm.packed_head, gm.x, n, gm.argmax, logits, None)
            c.goose_harvest_topk(logits, gm.desc.vocab, t, n, self.K, self.d_ids, self.d_scores)
            done += n
        torch.cuda.synchronize()
        self.P = done
        self.d_P.fill_(done)
        self.mirror_rows(prompt)
        self.anchor = int(gm.argmax[n - 1].item())
        self.seq = prompt + [self.anchor]
        return self.anchor

    def plan(self, o):
        """The nodes of the next cycle (host side of Alg. "Decoding Loop", one library call): tokens, parent,
        is_spine, mode."""
        return gb.goose_plan_cycle(self.seq, o.lens, o.max_spine, self.anchor, self.h_ids, self.h_scores, o.B,
                                   self.p_hat, o.rho, o.D, o.min_score, o.bypass_len)

    def absorb(self, o, tokens, is_spine, mode, L, path, bonus, P):
        """Takes the walk's result of a cycle; returns the tokens the cycle emitted."""
        self.P = P
        self.mirror_rows(tokens)
        offered = int(is_spine.sum()) - 1
        acc_spine = int(is_spine[path[1:]].sum())
        self.p_hat = gb.goose_ema_update(self.p_hat, acc_spine, offered, o.alpha)
        emitted = [int(tokens[v]) for v in path[1:]] + [bonus]
        self.seq += emitted
        self.anchor = bonus
        self.trace.append({"mode": mode, "nodes": len(tokens), "accepted": L, "p_hat": self.p_hat})
        return emitted


def _require_room(P, n, cap):
    """A cycle writes cache slots [P, P + n): refuse it before anything is overwritten."""
    if P + n > cap:
        raise gb.GooseError(gb.GOOSE_ERR_CAPACITY, f"cycle of {n} nodes on {P} committed slots, capacity {cap}")


def _require_clean(flags):
    """The device-side checks of the cycle just run (bad parent array, cache length out of range)."""
    if flags:
        raise gb.GooseError(gb.GOOSE_ERR_CAPACITY if flags & gb.GOOSE_FLAG_CAPACITY else gb.GOOSE_ERR_NOT_TOPOLOGICAL,
                            f"the verification kernels flagged the cycle (goose_device_flags = {flags})")


class _Options:
    def __init__(self, gm, B, K, rho, D, min_score, bypass_len, lens, max_spine, alpha):
        assert B <= gm.max_B and 1 + max_spine <= gm.max_B
        self.B, self.K, self.rho, self.D, self.min_score = B, K, rho, D, min_score
        self.bypass_len, self.lens, self.max_spine, self.alpha = bypass_len, tuple(lens), max_spine, alpha


class GooseDecoder:
    def __init__(self, gm: GooseModel, B=60, K=10, rho=0.5, D=6, min_score=0.01, bypass_len=8, lens=(3, 4, 5),
                 max_spine=20, alpha=0.3):
        self.gm = gm
        self.o = _Options(gm, B, K, rho, D, min_score, bypass_len, lens, max_spine, alpha)
        self.req = _Request(gm, K)

    trace = property(lambda self: self.req.trace)
    seq = property(lambda self: self.req.seq)
    p_hat = property(lambda self: self.req.p_hat)

    @property
    def lens(self):
        return self.o.lens

    @lens.setter
    def lens(self, v):
        self.o.lens = tuple(v)

    def prefill(self, prompt):
        first = self.req.prefill(prompt)
        self.gm.set_P(self.req.P)
        return first

    def cycle(self):
        """One cycle; returns the tokens it emitted (accepted drafts and the bonus token)."""
        gm, q = self.gm, self.req
        tokens, parent, is_spine, mode = q.plan(self.o)
        n = len(tokens)
        _require_room(gm.P, n, gm.cap)
        t, p, s = gm.stage_tree(tokens, parent, is_spine)
        gm.verify_step_fused(t, p, s, n, gm.cap - n, succ_ids=q.d_ids, succ_scores=q.d_scores)
        _require_clean(gm.ctx.goose_device_flags())   # (synchronises the stream)
        L = int(gm.accept_len.item())
        gm.P = int(gm.d_P.item())
        return q.absorb(self.o, tokens, is_spine, mode, L, gm.path[:L + 1].cpu().numpy(), int(gm.bonus.item()), gm.P)

    def generate(self, prompt, n_new):
        out = [self.prefill(prompt)]
        while len(out) < n_new:
            out += self.cycle()
        return out


class BatchedGooseDecoder:
    """Several requests, one pass over the weights per cycle.  `gm` must have been created with
    max_rows >= the rows of a full batch (round_up(B, 32) per request)."""

    def __init__(self, gm: GooseModel, n_requests, B=32, K=10, rho=0.5, D=6, min_score=0.01, bypass_len=8,
                 lens=(3, 4, 5), max_spine=20, alpha=0.3):
        assert n_requests * ((max(B, 1 + max_spine) + 31) // 32 * 32) <= gm.ctx.max_rows
        self.gm = gm
        self.o = _Options(gm, B, K, rho, D, min_score, bypass_len, lens, max_spine, alpha)
        self.reqs = [_Request(gm, K, torch.zeros_like(gm.kcache), torch.zeros_like(gm.vcache))
                     for _ in range(n_requests)]
        self.argmax_all = torch.zeros(gm.ctx.max_rows, dtype=torch.int32, device=gm.device)
        self.passes = 0

    def cycle(self, active):
        """One batched cycle over the requests `active` (indices); returns {index: emitted tokens}."""
        gm = self.gm
        plans, table = [], []
        for i in active:
            q = self.reqs[i]
            tokens, parent, is_spine, mode = q.plan(self.o)
            _require_room(q.P, len(tokens), gm.cap)
            t, p, s = gm.stage_tree(tokens, parent, is_spine)
            plans.append((tokens, is_spine, mode))
            table.append({"tokens": t, "parent": p, "is_spine": s, "B": len(tokens), "P_max": gm.cap - len(tokens),
                          "kcache": q.kcache, "vcache": q.vcache, "P": q.d_P, "accept_len": q.accept_len,
                          "path": q.path, "bonus": q.bonus, "succ_ids": q.d_ids, "succ_scores": q.d_scores})
        gm.ctx.goose_verify_step_batched(gm.model_ptrs(), table, self.argmax_all)
        _require_clean(gm.ctx.goose_device_flags())   # (synchronises the stream)
        self.passes += 1
        out = {}
        for i, (tokens, is_spine, mode) in zip(active, plans):
            q = self.reqs[i]
            L = int(q.accept_len.item())
            out[i] = q.absorb(self.o, tokens, is_spine, mode, L, q.path[:L + 1].cpu().numpy(), int(q.bonus.item()),
                              int(q.d_P.item()))
        return out

    def generate(self, prompts, n_new):
        """Returns one token list per prompt, each at least n_new long; a request leaves the batch when done."""
        assert len(prompts) == len(self.reqs)
        outs = [[q.prefill(p)] for q, p in zip(self.reqs, prompts)]
        active = list(range(len(prompts)))
        while active:
            for i, emitted in self.cycle(active).items():
                outs[i] += emitted
            active = [i for i in active if len(outs[i]) < n_new]
        return outs
