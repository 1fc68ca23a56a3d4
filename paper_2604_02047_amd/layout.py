"""Index maps of the bf16 KV cache as the library stores it (MFMA operand order, see goose.h).

Only addresses are computed here: `k_offsets` / `v_offsets` give, for cache slots and head-dim
columns, the element offset inside one head's cache, so that the binding can copy logical rows
[slot][d] in and out with torch indexing.  No value of the method is computed.
"""
import torch


def _sigma_inv(kk):
    return (((kk >> 2) & 3) << 3) | ((kk >> 4) << 2) | (kk & 3)


def k_offsets(slots: torch.Tensor, head_dim: int) -> torch.Tensor:
    """int64 [n_slots][head_dim]: offset of K element (slot, c) in a head's operand-ordered K cache."""
    g = slots.to(torch.int64).view(-1, 1)
    c = torch.arange(head_dim, dtype=torch.int64, device=slots.device).view(1, -1)
    blk, kk = g >> 5, g & 31
    s, hh, e = c >> 4, (c >> 3) & 1, c & 7
    return ((blk * (head_dim // 16) + s) * 64 + _sigma_inv(kk) + 32 * hh) * 8 + e


def v_offsets(slots: torch.Tensor, head_dim: int) -> torch.Tensor:
    """int64 [n_slots][head_dim]: offset of V element (slot, c) in a head's operand-ordered V cache."""
    g = slots.to(torch.int64).view(-1, 1)
    c = torch.arange(head_dim, dtype=torch.int64, device=slots.device).view(1, -1)
    blk, kk = g >> 5, g & 31
    return (((blk * (head_dim // 32) + (c >> 5)) * 2 + ((kk >> 3) & 1)) * 64 + (c & 31) + 32 * (kk >> 4)) * 8 + (kk & 7)
