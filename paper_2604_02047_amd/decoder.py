"""Sequencing of whole decoding cycles (Alg. "Decoding Loop") on top of the C ABI.

Every decision and every computation is a library call: the n-gram match, the routing, the tree
builder, tiers and moving average are host functions of libgoose; verification, harvest, walk and
compaction run on the GPU (goose_verify_step).  This module only moves small arrays between them:
per cycle it uploads the tree (a few hundred bytes) and reads back the walk's result and the table
rows the harvest touched.
"""
import numpy as np
import torch

from . import binding as gb
from .runner import GooseModel


class GooseDecoder:
    def __init__(self, gm: GooseModel, B=60, K=10, rho=0.5, D=6, min_score=0.01, bypass_len=8, lens=(3, 4, 5),
                 max_spine=20, alpha=0.3):
        assert B <= gm.max_B and 1 + max_spine <= gm.max_B
        self.gm, self.B, self.K = gm, B, K
        self.rho, self.D, self.min_score = rho, D, min_score
        self.bypass_len, self.lens, self.max_spine, self.alpha = bypass_len, tuple(lens), max_spine, alpha
        V, dev = gm.desc.vocab, gm.device
        self.d_ids = torch.full((V, K), -1, dtype=torch.int32, device=dev)      # written by the harvest kernel
        self.d_scores = torch.zeros((V, K), dtype=torch.float32, device=dev)
        self.h_ids = np.full((V, K), -1, np.int32)                               # host mirror for the tree builder
        self.h_scores = np.zeros((V, K), np.float32)
        self.seq, self.p_hat, self.anchor = [], 0.3, None
        self.trace = []

    def _mirror_rows(self, tokens):
        idx = torch.as_tensor(np.unique(np.asarray(tokens, np.int64)), device=self.gm.device)
        self.h_ids[idx.cpu().numpy()] = self.d_ids[idx].cpu().numpy()
        self.h_scores[idx.cpu().numpy()] = self.d_scores[idx].cpu().numpy()

    def prefill(self, prompt):
        """Feeds the prompt through the verification path as chain trees (every row kept), harvests every
        position's logits, and returns the first generated token."""
        gm, c = self.gm, self.gm.ctx
        prompt = [int(t) for t in prompt]
        gm.set_P(0)
        done, step = 0, gm.max_B
        while done < len(prompt):
            n = min(step, len(prompt) - done)
            chunk = prompt[done:done + n]
            t, p, s = gm.stage_tree(chunk, np.arange(-1, n - 1), np.ones(n, np.uint8))
            W = (n + 63) // 64
            mask = gm.mask.view(-1)[:n * W]
            c.goose_build_mask(p, n, gm.P, mask, gm.depth, gm.pos)
            c.goose_embed(gm.embed, t, n, gm.x)
            for l in range(gm.desc.n_layers):
                c.goose_verify_layer(gm.packed_layer(l), gm.x, gm.kcache[l], gm.vcache[l], gm.P, n, mask, gm.pos)
            logits = torch.empty((n, gm.desc.vocab), dtype=torch.float32, device=gm.device)
            c.goose_lm_head_argmax(gm.packed_head, gm.x, n, gm.argmax, logits, None)
            c.goose_harvest_topk(logits, gm.desc.vocab, t, n, self.K, self.d_ids, self.d_scores)
            done += n
            gm.set_P(done)
        torch.cuda.synchronize()
        self._mirror_rows(prompt)
        self.anchor = int(gm.argmax[n - 1].item())
        self.seq = prompt + [self.anchor]
        return self.anchor

    def cycle(self):
        """One cycle; returns the tokens it emitted (accepted drafts and the bonus token)."""
        gm = self.gm
        draft, consensus = gb.goose_context_match(self.seq, self.lens, self.max_spine)
        has_succ = bool(((self.h_ids[self.anchor] >= 0) & (self.h_scores[self.anchor] >= self.min_score)).any())
        mode = gb.goose_cycle_mode(len(draft), consensus, self.bypass_len, has_succ)
        if mode == gb.MODE_BYPASS:
            n = 1 + len(draft)
            tokens = np.concatenate([[self.anchor], draft]).astype(np.int32)
            parent = np.arange(-1, n - 1, dtype=np.int32)
            is_spine = np.ones(n, np.uint8)
        elif mode == gb.MODE_TREE:
            r = gb.goose_spine_ratio_tier(self.p_hat)
            tokens, parent, is_spine = gb.goose_build_spine_tree(self.anchor, draft, self.h_ids, self.h_scores, self.B,
                                                                 r, self.rho, self.D, self.min_score)
        else:
            tokens, parent, is_spine = (np.array([self.anchor], np.int32), np.array([-1], np.int32),
                                        np.ones(1, np.uint8))
        n = len(tokens)
        t, p, s = gm.stage_tree(tokens, parent, is_spine)
        gm.verify_step_fused(t, p, s, n, gm.cap - n, succ_ids=self.d_ids, succ_scores=self.d_scores)
        torch.cuda.synchronize()
        L = int(gm.accept_len.item())
        path = gm.path[:L + 1].cpu().numpy()
        bonus = int(gm.bonus.item())
        gm.P = int(gm.d_P.item())
        self._mirror_rows(tokens)
        offered = int(is_spine.sum()) - 1
        acc_spine = int(is_spine[path[1:]].sum())
        self.p_hat = gb.goose_ema_update(self.p_hat, acc_spine, offered, self.alpha)
        emitted = [int(tokens[v]) for v in path[1:]] + [bonus]
        self.seq += emitted
        self.anchor = bonus
        self.trace.append({"mode": mode, "nodes": n, "accepted": L, "p_hat": self.p_hat})
        return emitted

    def generate(self, prompt, n_new):
        out = [self.prefill(prompt)]
        while len(out) < n_new:
            out += self.cycle()
        return out
