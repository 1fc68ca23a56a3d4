"""The skinny-M projection kernel alone against an fp64 product of the same bf16 inputs."""
import numpy as np
import pytest
import torch

import paper_2604_02047_amd as g

pytestmark = pytest.mark.gpu


def _a_rows(B):
    """Rows the operand buffer must hold: whole 32-row tiles, whole 128-row chunks beyond 128 rows."""
    return (B + 31) // 32 * 32 if B <= 128 else (B + 127) // 128 * 128


def _operand(a32, rows, Kp, dt, terms, dev):
    """fp32 rows [B][K] -> (device operand in `terms` terms with `rows` rows, the exact values it carries as fp64)."""
    B, K = a32.shape
    if terms == 1:
        a = torch.zeros((rows, Kp), dtype=dt)
        a[:B, :K] = a32.to(dt)
        return a.to(dev), a[:B, :K].double().numpy()
    src = torch.zeros((rows, Kp), dtype=torch.float32, device=dev)
    src[:B, :K] = a32.to(dev)
    a2 = torch.full((rows, 2 * Kp), float("nan"), dtype=dt, device=dev)
    g.goose_split_operand(src, rows, Kp, Kp, a2, 2 * Kp)
    torch.cuda.synchronize()
    groups = a2.view(rows, Kp // 8, 2, 8).double().cpu()      # [row][group][hi|lo][8]
    carried = (groups[:, :, 0] + groups[:, :, 1]).reshape(rows, Kp)
    hi = groups[:, :, 0].reshape(rows, Kp)
    assert torch.equal(hi[:B, :K].to(dt), a32.to(dt))                       # hi is the plain rounding
    assert (carried[:B, :K] - a32.double()).abs().max() <= 2.0 ** -15 * a32.abs().max()   # hi + lo: 16 more bits
    return a2, carried[:B, :K].numpy()


def _run(B, N, K, nw, ks, seed=0, dt=torch.bfloat16, terms=1):
    dev = "cuda:0"
    gen = torch.Generator(device="cpu").manual_seed(seed)
    Kp, Np, rows = (K + 127) // 128 * 128, (N + 31) // 32 * 32, (B + 31) // 32 * 32
    a, a_exact = _operand(torch.randn((B, K), generator=gen), _a_rows(B), Kp, dt, terms, dev)
    w = (torch.randn((N, K), generator=gen) * 0.05).to(dt)
    ref = a_exact @ w.double().numpy().T
    packed = torch.zeros(g.goose_packed_matrix_bytes(N, K), dtype=torch.uint8, device=dev)
    g.goose_pack_matrix(w.to(dev), N, K, packed)
    part = torch.full((ks, rows, Np), float("nan"), dtype=torch.float32, device=dev)
    if terms == 1:
        g.goose_gemm_packed(a, Kp, packed, N, K, B, nw, ks, part)
    else:
        g.goose_gemm_packed_ex(a, Kp * terms, terms, packed, N, K, B, nw, ks, part)
    torch.cuda.synchronize()
    out = part[:, :B, :N].double().sum(0).cpu().numpy()
    scale = np.abs(ref).max()
    err = np.abs(out - ref).max()
    # fp32 accumulation of exact bf16 products: only summation-order rounding remains
    assert err <= 2e-5 * scale * max(1.0, np.sqrt(K) / 16), (B, N, K, nw, ks, err, scale)


@pytest.mark.parametrize("B", [1, 16, 33, 64, 80, 128])
def test_gemm_row_tiles(B):
    _run(B, 256, 512, 2, 1)
    _run(B, 288, 1024, 4, 2)


@pytest.mark.parametrize("B", [129, 200, 256, 300, 512])
def test_gemm_row_chunks(B):
    """More than 128 rows: chunks of 128 rows, each its own workgroups (dealt so that the chunks of a
    column group share an XCD); grids that are no multiple of 8 workgroups, ragged last chunk."""
    _run(B, 256, 512, 2, 1)
    _run(B, 288, 1024, 4, 2)
    _run(B, 1000, 1000, 4, 3)
    _run(B, 4096, 2048, 4, 4)


@pytest.mark.parametrize("stages,ks", [(1, 1), (2, 1), (2, 2), (3, 1), (3, 3), (4, 2), (5, 1), (5, 2), (6, 3),
                                       (8, 2), (9, 2), (22, 5), (32, 1), (32, 4), (86, 8)])
def test_gemm_stage_counts_and_splits(stages, ks):
    for nw in (2, 4):
        for B in (64, 16, 96):
            _run(B, 160, stages * 128, nw, ks, seed=stages)


@pytest.mark.parametrize("B", [16, 80, 128, 300])
def test_gemm_fp16_operands(B):
    """The same kernels on fp16 operands (exact products, fp32 accumulation: the same bound)."""
    _run(B, 288, 1024, 4, 2, dt=torch.float16)
    _run(B, 1000, 1000, 2, 1, dt=torch.float16)


@pytest.mark.parametrize("B", [1, 16, 33, 64, 80, 128, 200, 512])
@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
def test_gemm_two_term_operand(B, dt):
    """The activation operand as hi + lo (the layout the decoder layers use): the product must be that of
    the sum of both terms, i.e. of the fp32 activations to 2^-17."""
    _run(B, 288, 1024, 4, 2, dt=dt, terms=2)
    _run(B, 256, 512, 2, 1, dt=dt, terms=2)
    _run(B, 1000, 1000, 4, 3, dt=dt, terms=2)


def test_gemm_ragged_shapes():
    _run(50, 1000, 1000, 4, 2)   # N not a multiple of the 4-tile group, K padded to 1024
    _run(7, 40, 200, 2, 1)
    _run(64, 4096, 4096, 4, 8)


@pytest.mark.parametrize("B,F,K,nw", [(16, 96, 256, 2), (16, 2752, 1024, 2), (64, 2752, 1024, 4), (80, 352, 640, 2),
                                       (80, 17920, 256, 4),
                                       (128, 704, 256, 4), (33, 64, 4096, 2), (300, 704, 256, 4), (512, 352, 640, 2),
                                       (160, 2752, 1024, 4)])
@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("terms", [1, 2])
def test_gemm_swiglu_epilogue(B, F, K, nw, dt, terms):
    dev = "cuda:0"
    gen = torch.Generator(device="cpu").manual_seed(F)
    Kp, rows = (K + 127) // 128 * 128, (B + 31) // 32 * 32
    a, a_exact = _operand(torch.randn((B, K), generator=gen), _a_rows(B), Kp, dt, terms, dev)
    wg = (torch.randn((F, K), generator=gen) * 0.05).to(dt)
    wu = (torch.randn((F, K), generator=gen) * 0.05).to(dt)
    assert F % 16 == 0
    inter = torch.stack([wg.view(F // 16, 16, K), wu.view(F // 16, 16, K)], dim=1).reshape(2 * F, K).contiguous()
    gd, ud = torch.from_numpy(a_exact) @ wg.double().T, torch.from_numpy(a_exact) @ wu.double().T
    ref = (gd / (1 + torch.exp(-gd)) * ud).numpy()
    packed = torch.zeros(g.goose_packed_matrix_bytes(2 * F, K), dtype=torch.uint8, device=dev)
    g.goose_pack_matrix(inter.to(dev), 2 * F, K, packed)
    h = torch.full((rows, F * terms), float("nan"), dtype=dt, device=dev)
    if terms == 1:
        g.goose_gemm_swiglu_packed(a, Kp, packed, 2 * F, K, B, nw, h, F)
    else:
        g.goose_gemm_swiglu_packed_ex(a, Kp * terms, terms, packed, 2 * F, K, B, nw, h, F * terms)
    torch.cuda.synchronize()
    if terms == 1:
        out = h[:B].double().cpu().numpy()
        # one rounding of the result to the storage type (relative to the element, hence to the largest)
        tol = 6e-3 if dt == torch.bfloat16 else 8e-4
    else:   # the result keeps two terms as well: hi + lo carries it to 2^-17 (the silu itself is fp32)
        pair = h[:B].view(B, F // 8, 2, 8).double().cpu()
        out = (pair[:, :, 0] + pair[:, :, 1]).reshape(B, F).numpy()
        tol = 2e-5
    assert np.abs(out - ref).max() <= tol * np.abs(ref).max()


def test_gemm_more_tiles_than_one_round_of_four_tile_workgroups():
    """Beyond 1024 column tiles the launcher switches to five-wavefront workgroups (one round of 256)."""
    _run(80, 33024, 256, 4, 1)            # 1032 tiles
    _run(64, 20000, 512, 4, 2, seed=3)    # 625 tiles x 2 K ranges
    _run(33, 40960, 128, 4, 1, seed=4)    # 1280 tiles: the last five-wide grid that fits


def test_gemm_repeated_large_launches_are_stable():
    """The weight stream is hand scheduled (asynchronous loads awaited by count): hammer the
    big shapes of the 7B model, where memory latency is longest, and check every launch."""
    for rep in range(6):
        _run(64, 4096, 4096, 4, 8, seed=rep)
        _run(64, 4096, 11008, 4, 8, seed=rep)
        _run(64, 2048, 4096, 2, 1, seed=rep)
        _run(16, 4096, 4096, 2, 4, seed=rep)
        _run(128, 1024, 4096, 4, 2, seed=rep)
