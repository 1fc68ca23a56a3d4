"""Bit-exact parity of the integer steps (ancestor mask, greedy walk, KV compaction) with the oracle."""
import numpy as np
import pytest
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2604_02047_amd import GooseContext, ModelDesc
    c = GooseContext(ModelDesc.from_shape(gi.SHAPES["tiny"]), 128, 4096)
    yield c
    c.close()


def _trees():
    out = [gi.tree_single(), gi.tree_chain(2), gi.tree_chain(64), gi.tree_chain(65), gi.tree_chain(128),
           gi.tree_star(128), gi.tree_star(33), gi.tree_tiny_spine(), gi.tree_spine_13b(), gi.tree_spine_33b(),
           gi.tree_spine_stress(), gi.tree_balanced()]
    out += [gi.tree_spine_7b(s) for s in range(4)]
    out += [gi.tree_random(B, B) for B in (3, 17, 63, 64, 65, 100, 127, 128)]
    return out


def test_mask_depth_pos_bit_exact(ctx):
    dev = "cuda:0"
    for n, tree in enumerate(_trees()):
        B, P = tree.B, 7 + 13 * n
        W = (B + 63) // 64
        parent = torch.as_tensor(tree.parent, device=dev)
        mask = torch.full((B * W,), -1, dtype=torch.int64, device=dev)
        depth = torch.full((B,), -1, dtype=torch.int32, device=dev)
        pos = torch.full((B,), -1, dtype=torch.int32, device=dev)
        ctx.goose_build_mask(parent, B, P, mask, depth, pos)
        torch.cuda.synchronize()
        anc, odepth = orc.ancestor_mask(tree.parent)
        assert np.array_equal(mask.cpu().numpy().view(np.uint64).reshape(B, W), orc.mask_words(anc)), n
        assert np.array_equal(depth.cpu().numpy(), odepth), n
        assert np.array_equal(pos.cpu().numpy(), P + odepth), n
        # same result with P read from device memory
        dP = torch.tensor([P], dtype=torch.int32, device=dev)
        pos2 = torch.zeros_like(pos)
        ctx.goose_build_mask(parent, B, 0, mask, depth, pos2, d_P=dP)
        torch.cuda.synchronize()
        assert torch.equal(pos, pos2)
    assert ctx.goose_device_flags() == 0


def test_bad_parent_array_sets_flag_and_stays_in_bounds(ctx):
    dev = "cuda:0"
    parent = torch.tensor([-1, 0, 5, 1, -3, 2], dtype=torch.int32, device=dev)  # 5 >= 2 and -3 are invalid
    mask = torch.zeros(6, dtype=torch.int64, device=dev)
    depth = torch.zeros(6, dtype=torch.int32, device=dev)
    pos = torch.zeros(6, dtype=torch.int32, device=dev)
    ctx.goose_build_mask(parent, 6, 0, mask, depth, pos)
    assert ctx.goose_device_flags() & 1
    assert ctx.goose_device_flags() == 0  # reading clears it


def test_accept_bit_exact(ctx):
    dev = "cuda:0"
    rng = np.random.default_rng(5)
    multi = 0
    for trial in range(200):
        B = int(rng.integers(1, 129))
        tree = gi.tree_random(B, trial, spine_len=int(rng.integers(0, min(B, 20) + 1)))
        vocab = 2 if trial % 2 else 8
        tokens = rng.integers(0, vocab, B).astype(np.int32)  # duplicates among siblings allowed on purpose
        x_hat = rng.integers(0, vocab, B).astype(np.int32)
        use_tag = trial % 3 != 0
        acc, bonus = orc.greedy_walk(tree.parent, tokens, tree.is_spine if use_tag else None, x_hat)
        out_len = torch.full((1,), -7, dtype=torch.int32, device=dev)
        out_path = torch.full((B,), -7, dtype=torch.int32, device=dev)
        out_bonus = torch.full((1,), -7, dtype=torch.int32, device=dev)
        ctx.goose_accept(torch.as_tensor(tree.parent, device=dev), torch.as_tensor(tokens, device=dev),
                         torch.as_tensor(tree.is_spine, device=dev) if use_tag else None,
                         torch.as_tensor(x_hat, device=dev), B, out_len, out_path, out_bonus)
        torch.cuda.synchronize()
        L = int(out_len.item())
        assert L == len(acc), trial
        assert out_path.cpu().numpy().tolist() == [0] + acc + [-1] * (B - 1 - L), trial
        assert int(out_bonus.item()) == bonus, trial
        multi += L >= 2
    assert multi > 15


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compact_kv_bit_exact(dtype):
    from paper_2604_02047_amd import GooseContext, ModelDesc
    dev = "cuda:0"
    shape = gi.SHAPES["tiny"] if dtype == "f32" else gi.SHAPES["tiny_bf16"]
    cap = 320
    c = GooseContext(ModelDesc.from_shape(shape), 128, cap)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    kdims = (shape.n_layers, shape.n_heads, cap, shape.head_dim)
    rng = np.random.default_rng(1)
    cases = [[0], [0, 1, 2, 3], [0, 2, 3], [0, 5, 9, 64, 127], [0, 127], list(range(0, 128, 1))[:40],
             [0, 3, 4, 5, 6, 40, 41]]
    for n, path in enumerate(cases):
        P = int(rng.integers(0, cap - 128))
        k0 = torch.randn(kdims, device=dev).to(tdt)              # logical [layer][head][slot][d]
        v0 = torch.randn(kdims, device=dev).to(tdt)
        if dtype == "f32":   # stored as K[slot][d] and V transposed [d][slot]
            k, vt = k0.clone(), v0.transpose(2, 3).contiguous()
        else:                # stored in operand-ordered 32-key blocks
            from paper_2604_02047_amd import layout
            slots = torch.arange(cap, device=dev)
            ko, vo = layout.k_offsets(slots, shape.head_dim), layout.v_offsets(slots, shape.head_dim)
            assert sorted(ko.flatten().tolist()) == list(range(cap * shape.head_dim))   # a permutation of the cache
            assert sorted(vo.flatten().tolist()) == list(range(cap * shape.head_dim))
            k = torch.zeros((kdims[0], kdims[1], cap * shape.head_dim), dtype=tdt, device=dev)
            vt = torch.zeros_like(k)
            k[:, :, ko] = k0
            vt[:, :, vo] = v0
        L = len(path) - 1
        dpath = torch.full((128,), -1, dtype=torch.int32, device=dev)
        dpath[:L + 1] = torch.tensor(path, dtype=torch.int32)
        dlen = torch.tensor([L], dtype=torch.int32, device=dev)
        newP = torch.zeros(1, dtype=torch.int32, device=dev)
        if n % 2:
            c.goose_compact_kv(k, vt, P, dpath, dlen, newP)
        else:  # P from device memory, updated in place
            newP.fill_(P)
            c.goose_compact_kv(k, vt, 0, dpath, dlen, newP, d_P=newP)
        torch.cuda.synchronize()
        if dtype == "f32":
            v = vt.transpose(2, 3)
        else:
            k, v = k[:, :, ko], vt[:, :, vo]
        assert int(newP.item()) == P + L + 1
        idx = torch.tensor(path, device=dev) + P
        # slots [0,P) untouched, [P, P+L] are the path rows, byte for byte
        assert torch.equal(k[:, :, :P], k0[:, :, :P]) and torch.equal(v[:, :, :P], v0[:, :, :P])
        assert torch.equal(k[:, :, P:P + L + 1], k0[:, :, idx]) and torch.equal(v[:, :, P:P + L + 1], v0[:, :, idx])
        # and identical to the oracle's commit of the same rows
        nl = kdims[0]
        cache = [(k0[l, :, :P].double().cpu().numpy(), v0[l, :, :P].double().cpu().numpy()) for l in range(nl)]
        new_kv = [(k0[l, :, P:P + 128].double().cpu().numpy(), v0[l, :, P:P + 128].double().cpu().numpy())
                  for l in range(nl)]
        ref = orc.commit_path(cache, new_kv, path)
        for l in range(nl):
            assert np.array_equal(k[l, :, :P + L + 1].double().cpu().numpy(), ref[l][0])
            assert np.array_equal(v[l, :, :P + L + 1].double().cpu().numpy(), ref[l][1])
    c.close()


def test_cache_length_from_device_memory_out_of_range_sets_the_capacity_flag(ctx):
    """A device-resident cache length cannot be refused by the host: one slot past what fits (P + B > cap),
    past the bound the launch was sized for, or negative, the kernels must say so."""
    from paper_2604_02047_amd.binding import GOOSE_FLAG_CAPACITY
    dev = "cuda:0"
    tree = gi.tree_chain(16)
    parent = torch.as_tensor(tree.parent, device=dev)
    mask = torch.zeros(16, dtype=torch.int64, device=dev)
    depth = torch.zeros(16, dtype=torch.int32, device=dev)
    pos = torch.zeros(16, dtype=torch.int32, device=dev)
    cap = 4096
    assert ctx.goose_device_flags() == 0
    for P, bad in ((cap - 16, False), (cap - 15, True), (-1, True), (0, False)):
        dP = torch.tensor([P], dtype=torch.int32, device=dev)
        ctx.goose_build_mask(parent, 16, 0, mask, depth, pos, d_P=dP)
        assert bool(ctx.goose_device_flags() & GOOSE_FLAG_CAPACITY) == bad, P
    # a commit that would run past the cache
    from paper_2604_02047_amd import GooseContext, ModelDesc
    shape = gi.SHAPES["tiny_bf16"]
    c = GooseContext(ModelDesc.from_shape(shape), 64, 128)
    k = torch.zeros((shape.n_layers, shape.n_heads, 128 * shape.head_dim), dtype=torch.bfloat16, device=dev)
    v = torch.zeros_like(k)
    path = torch.tensor([0, 1, 2] + [-1] * 61, dtype=torch.int32, device=dev)
    L = torch.tensor([2], dtype=torch.int32, device=dev)
    for P, bad in ((125, False), (126, True)):
        dP = torch.tensor([P], dtype=torch.int32, device=dev)
        c.goose_compact_kv(k, v, 0, path, L, dP, d_P=dP)
        assert bool(c.goose_device_flags() & GOOSE_FLAG_CAPACITY) == bad, P
    c.close()
