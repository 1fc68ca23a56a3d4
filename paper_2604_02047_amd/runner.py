"""Device-memory plumbing around the C ABI: allocates the caches, packs weights, stages a tree.

Nothing here computes anything of the method: tensors are allocated with torch, handed to the
library, and read back.  Weights come from a caller-supplied function so that checkpoints or
synthetic generators can both feed it.
"""
import numpy as np
import torch

from . import layout
from .binding import GooseContext, ModelDesc


def _torch_dtype(name):
    return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[name]


class GooseModel:
    """A model resident in HBM: packed weights, KV cache, and per-step staging buffers."""

    def __init__(self, desc: ModelDesc, max_B: int, cap: int, layer_fn, embed, lm_head, final_norm,
                 device="cuda:0", max_rows: int = 0):
        self.desc, self.max_B, self.cap = desc, max_B, cap
        self.device = torch.device(device)
        self.dt = _torch_dtype(desc.dtype)
        self.ctx = GooseContext(desc, max_B, cap, max_rows)
        lb = self.ctx.goose_packed_layer_bytes()
        self.layer_bytes = lb
        self.packed_layers = torch.zeros(desc.n_layers * lb, dtype=torch.uint8, device=self.device)
        for l in range(desc.n_layers):
            raw = {k: v.to(self.device).contiguous() for k, v in layer_fn(l).items()}
            self.ctx.goose_pack_layer(raw, self.packed_layers[l * lb:(l + 1) * lb])
            torch.cuda.synchronize()
            del raw
        self.embed = embed.to(self.device).contiguous()
        self.packed_head = torch.zeros(self.ctx.goose_packed_lm_head_bytes(), dtype=torch.uint8, device=self.device)
        wl, gf = lm_head.to(self.device).contiguous(), final_norm.to(self.device).contiguous()
        self.ctx.goose_pack_lm_head(gf, wl, self.packed_head)
        torch.cuda.synchronize()
        del wl, gf
        assert cap % 64 == 0, "cap must be a multiple of 64"
        # One head's cache is cap * head_dim elements.  fp32 models: K[slot][d] and V transposed, Vt[d][slot];
        # bf16 / fp16 models: 32-key blocks in MFMA operand order (layout.py), kept here as flat vectors.
        self.tiled = desc.dtype in ("bf16", "f16")
        kvh = desc.kv_heads  # caches hold key/value heads (fewer than query heads under grouped queries)
        if self.tiled:
            self.kcache = torch.zeros((desc.n_layers, kvh, cap * desc.head_dim), dtype=self.dt, device=self.device)
            self.vcache = torch.zeros_like(self.kcache)
        else:
            self.kcache = torch.zeros((desc.n_layers, kvh, cap, desc.head_dim), dtype=self.dt, device=self.device)
            self.vcache = torch.zeros((desc.n_layers, kvh, desc.head_dim, cap), dtype=self.dt, device=self.device)
        self.P = 0
        i32 = dict(dtype=torch.int32, device=self.device)
        self.d_P = torch.zeros(1, **i32)
        self.mask = torch.zeros((128, 2), dtype=torch.int64, device=self.device)
        self.depth = torch.zeros(128, **i32)
        self.pos = torch.zeros(128, **i32)
        self.x = torch.zeros((max_B, desc.hidden), dtype=torch.float32, device=self.device)
        self.argmax = torch.zeros(128, **i32)
        self.accept_len = torch.zeros(1, **i32)
        self.path = torch.zeros(128, **i32)
        self.bonus = torch.zeros(1, **i32)
        self.margin = torch.zeros(128, dtype=torch.float32, device=self.device)

    def packed_layer(self, l):
        return self.packed_layers[l * self.layer_bytes:(l + 1) * self.layer_bytes]

    def _slots(self, a, b):
        return torch.arange(a, b, device=self.device)

    def k_rows(self, a, b):
        """Key rows of slots [a,b) as [layer][head][slot][d] (a copy in logical order)."""
        if not self.tiled:
            return self.kcache[:, :, a:b].clone()
        return self.kcache[:, :, layout.k_offsets(self._slots(a, b), self.desc.head_dim)]

    def v_rows(self, a, b):
        """Value rows of slots [a,b) as [layer][head][slot][d] (a copy in logical order)."""
        if not self.tiled:
            return self.vcache[:, :, :, a:b].transpose(2, 3).contiguous()
        return self.vcache[:, :, layout.v_offsets(self._slots(a, b), self.desc.head_dim)]

    def write_rows(self, l, k, v):
        """Stores logical rows k, v [head][n][d] of layer l into slots [0,n) (values cast to the cache type)."""
        n = k.shape[1]
        k, v = k.to(self.dt).to(self.device), v.to(self.dt).to(self.device)
        if not self.tiled:
            self.kcache[l, :, :n] = k
            self.vcache[l, :, :, :n] = v.transpose(1, 2)
        else:
            self.kcache[l][:, layout.k_offsets(self._slots(0, n), self.desc.head_dim)] = k
            self.vcache[l][:, layout.v_offsets(self._slots(0, n), self.desc.head_dim)] = v

    def set_P(self, P: int):
        self.P = int(P)
        self.d_P.fill_(self.P)

    def model_ptrs(self):
        return {"embed": self.embed, "packed_layers": self.packed_layers, "packed_head": self.packed_head,
                "kcache": self.kcache, "vcache": self.vcache}

    def stage_tree(self, tokens, parent, is_spine):
        dev = self.device
        t = torch.as_tensor(np.asarray(tokens, dtype=np.int32), device=dev)
        p = torch.as_tensor(np.asarray(parent, dtype=np.int32), device=dev)
        s = None if is_spine is None else torch.as_tensor(np.asarray(is_spine, dtype=np.uint8), device=dev)
        return t, p, s

    # ---- one step through the individual entry points (host-known P)
    def verify_step_calls(self, tokens, parent, is_spine, want_logits=False, commit=True, layer_hook=None):
        """build_mask -> embed -> verify_layer x L -> lm_head_argmax -> accept -> compact_kv."""
        B = len(parent)
        c, d = self.ctx, self.desc
        t, p, s = self.stage_tree(tokens, parent, is_spine)
        W = (B + 63) // 64
        mask = self.mask.view(-1)[:B * W]
        c.goose_build_mask(p, B, self.P, mask, self.depth, self.pos)
        c.goose_embed(self.embed, t, B, self.x)
        for l in range(d.n_layers):
            c.goose_verify_layer(self.packed_layer(l), self.x, self.kcache[l], self.vcache[l], self.P, B, mask,
                                 self.pos)
            if layer_hook is not None:
                layer_hook(l, self.x[:B])
        logits = torch.empty((B, d.vocab), dtype=torch.float32, device=self.device) if want_logits else None
        c.goose_lm_head_argmax(self.packed_head, self.x, B, self.argmax, logits, self.margin)
        c.goose_accept(p, t, s, self.argmax, B, self.accept_len, self.path, self.bonus)
        out = {"mask": mask.clone().view(B, W), "depth": self.depth[:B].clone(), "pos": self.pos[:B].clone(),
               "argmax": self.argmax[:B].clone(), "margin": self.margin[:B].clone(), "logits": logits,
               "tail_k": self.k_rows(self.P, self.P + B),
               "tail_v": self.v_rows(self.P, self.P + B)}
        if commit:
            new_P = torch.zeros(1, dtype=torch.int32, device=self.device)
            c.goose_compact_kv(self.kcache, self.vcache, self.P, self.path, self.accept_len, new_P)
            torch.cuda.synchronize()
            self.set_P(int(new_P.item()))
        torch.cuda.synchronize()
        out["accept_len"] = int(self.accept_len.item())
        out["path"] = self.path[:B].cpu().numpy().copy()
        out["bonus"] = int(self.bonus.item())
        return out

    # ---- one step through goose_verify_step (P lives on the device)
    def verify_step_fused(self, t, p, s, B, P_max, next_root=None, logits=None, margin=None, succ_ids=None,
                          succ_scores=None):
        io = {"tokens": t, "parent": p, "is_spine": s, "P": self.d_P, "argmax": self.argmax,
              "accept_len": self.accept_len, "path": self.path, "bonus": self.bonus, "next_root": next_root,
              "logits": logits, "margin": margin, "succ_ids": succ_ids, "succ_scores": succ_scores,
              "harvest_k": 0 if succ_ids is None else succ_ids.shape[1]}
        self.ctx.goose_verify_step(self.model_ptrs(), io, B, P_max)
