"""64-bit position-weighted checksum of a tensor, the same function on the CPU and on the GPU (torch int64
arithmetic wraps modulo 2^64 on both).  Used to compare complete outputs at benchmark sizes with values the
oracle produced offline: digest = sum_i (w_i + 1) * (mix(i) | 1) mod 2^64 over the tensor's 32-bit words
(bytes for uint8 tensors), mix = the published splitmix64 finaliser.  A changed, missing or moved word
changes the sum (up to 2^-64 coincidences)."""
import torch

_M1 = 0xBF58476D1CE4E5B9 - (1 << 64)
_M2 = 0x94D049BB133111EB - (1 << 64)
_G = 0x9E3779B97F4A7C15 - (1 << 64)


def _lsr(x, s):
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(z):
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def digest(t, chunk=1 << 24):
    t = t.contiguous().view(-1)
    if t.dtype == torch.uint8:
        words = t
    else:
        assert t.element_size() == 4
        words = t.view(torch.int32)
    total = 0
    for lo in range(0, words.numel(), chunk):
        w = words[lo:lo + chunk].to(torch.int64)
        if words.dtype != torch.uint8:
            w = w & 0xFFFFFFFF
        i = torch.arange(lo, lo + w.numel(), dtype=torch.int64, device=w.device)
        h = _mix(i * _G + 0x1234567) | 1
        total = (total + int(((w + 1) * h).sum().item())) & ((1 << 64) - 1)
    return total
