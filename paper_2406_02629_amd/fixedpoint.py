"""Plaintext side of the harness: fixed-point encode / decode between float64
tensors and field elements (Sec. II-B: F_p stands for the signed range
[-(p-1)/2, (p-1)/2]; values are scaled by 2^f and rounded to nearest-even).
These run on the data owner's side, outside the share arithmetic.
"""
import torch

P61 = (1 << 61) - 1


def encode(x: torch.Tensor, f: int, p: int = P61) -> torch.Tensor:
    """float64 -> field elements as int64: round-half-even(x * 2^f) mod p."""
    v = torch.round(x.to(torch.float64) * float(1 << f))
    if bool((v.abs() >= float(1 << 40)).any()):
        raise ValueError("value exceeds 2^40 after scaling")
    v = v.to(torch.int64)
    return torch.where(v < 0, v + p, v)


def lift(u: torch.Tensor, p: int = P61) -> torch.Tensor:
    """field element -> signed integer: u if u <= (p-1)/2 else u - p."""
    return torch.where(u > (p - 1) // 2, u - p, u)


def from_signed(v: torch.Tensor, p: int = P61) -> torch.Tensor:
    return torch.where(v < 0, v + p, v)


def decode(u: torch.Tensor, s: int, p: int = P61) -> torch.Tensor:
    """field element -> float64 lift(u) / 2^s."""
    return lift(u, p).to(torch.float64) / float(1 << s)
