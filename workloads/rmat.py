"""R-MAT graph generator -> CSR (int64 rowptr, int32 col), identical on host and device.

Recipe: edge e picks one quadrant per bit level with probabilities (a,b,c,d) =
(0.57, 0.19, 0.19, 0.05); the choice is a 16-bit field of an integer hash of
(graph seed, e, level group), compared with integer thresholds, so there is no floating
point and a CPU run and a GPU run give the same edges.  Edges with an endpoint >= V are
dropped (V need not be a power of two), node ids go through a fixed affine bijection of
[0, V) so that hubs are not all at low ids, duplicate (u, v) pairs are removed, and the
result is sorted by (u, v).
"""
import math
import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int -> the int64 with the same low 64 bits."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_C_GOLD = _s64(0x9E3779B97F4A7C15)
_C_M1 = _s64(0xBF58476D1CE4E5B9)
_C_M2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """SplitMix64 finaliser on int64 tensors with wrapping arithmetic (a bijection of 2^64)."""
    x = x + _C_GOLD
    x = (x ^ _lsr(x, 30)) * _C_M1
    x = (x ^ _lsr(x, 27)) * _C_M2
    return x ^ _lsr(x, 31)


# cumulative quadrant thresholds on a 16-bit uniform: a | a+b | a+b+c
_TA = round(0.57 * 65536)
_TB = round(0.76 * 65536)
_TC = round(0.95 * 65536)


def _affine_bijection(V: int):
    a = 0x5DEECE66D % V if V > 1 else 1
    a = max(a, 1)
    while math.gcd(a, V) != 1:
        a += 1
    b = 0x2545F491 % V
    return a, b


def rmat_edge_keys(V: int, E: int, seed: int, device="cpu", chunk: int = 1 << 25,
                   permute: bool = True) -> torch.Tensor:
    """Sorted unique keys u*V+v (int64) of the de-duplicated R-MAT edge set."""
    levels = max(1, math.ceil(math.log2(V)))
    a, b = _affine_bijection(V)
    seed_mix = _s64(seed * 0xD6E8FEB86659FD93)
    parts = []
    for lo in range(0, E, chunk):
        hi = min(E, lo + chunk)
        e = torch.arange(lo, hi, dtype=torch.int64, device=device)
        base = mix64(e ^ seed_mix)
        u = torch.zeros_like(e)
        v = torch.zeros_like(e)
        for g in range((levels + 3) // 4):
            h = mix64(base + g)
            for t in range(4):
                lvl = 4 * g + t
                if lvl >= levels:
                    break
                r = _lsr(h, 16 * t) & 0xFFFF
                sbit = (r >= _TB).to(torch.int64)
                dbit = (((r >= _TA) & (r < _TB)) | (r >= _TC)).to(torch.int64)
                u = (u << 1) | sbit
                v = (v << 1) | dbit
            del h
        keep = (u < V) & (v < V)
        u = u[keep]
        v = v[keep]
        if permute:
            u = (u * a + b) % V
            v = (v * a + b) % V
        parts.append(torch.unique(u * V + v))
        del e, base, u, v, keep
    keys = torch.cat(parts) if len(parts) > 1 else parts[0]
    del parts
    return torch.unique(keys)


def _csr_from_keys(keys: torch.Tensor, V: int):
    src = keys // V
    col = (keys - src * V).to(torch.int32)
    deg = torch.bincount(src, minlength=V)
    del src
    rowptr = torch.zeros(V + 1, dtype=torch.int64, device=keys.device)
    torch.cumsum(deg, 0, out=rowptr[1:])
    return rowptr, col


def rmat_csr(V: int, E: int, seed: int = 1, device="cpu", chunk: int = 1 << 25, permute: bool = True):
    """CSR by source of the R-MAT graph: (rowptr int64[V+1], col int32[E'])  with col ascending per row."""
    keys = rmat_edge_keys(V, E, seed, device=device, chunk=chunk, permute=permute)
    return _csr_from_keys(keys, V)


def transpose_csr(rowptr: torch.Tensor, col: torch.Tensor, chunk: int = 1 << 27):
    """CSR of the reversed edges (i.e. the CSC of the input), same conventions."""
    V = rowptr.numel() - 1
    deg = rowptr[1:] - rowptr[:-1]
    src = torch.repeat_interleave(torch.arange(V, dtype=torch.int64, device=col.device), deg)
    keys = col.to(torch.int64) * V + src
    del src, deg
    keys, _ = torch.sort(keys)
    return _csr_from_keys(keys, V)
