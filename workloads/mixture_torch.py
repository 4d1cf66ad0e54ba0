"""Device-side twin of workloads.mixture for databases too large to generate on the host.

Same distribution (same component means, same sigma, same clipping) drawn with
torch's generator on the GPU, so the values differ from the NumPy stream; rows
are produced in fixed blocks with per-block seeds, so a row range does not
depend on how the caller chunks it.  Input generation only: no quantizer, no
encoding, no distances.
"""

from __future__ import annotations

import torch

from .mixture import MixtureSpec, mixture_params

BLOCK = 1 << 18


def mixture_vectors_torch(spec: MixtureSpec, stream_seed: int, start: int, count: int,
                          device="cuda:0") -> torch.Tensor:
    """Rows [start, start+count), float32 [count][d] on `device`; start must be a multiple of BLOCK."""
    if start % BLOCK:
        raise ValueError("start must be a multiple of BLOCK")
    means = torch.from_numpy(mixture_params(spec)).to(device)
    out = torch.empty((count, spec.d), dtype=torch.float32, device=device)
    gen = torch.Generator(device=device)
    pos = 0
    b = start // BLOCK
    while pos < count:
        take = min(BLOCK, count - pos)
        gen.manual_seed((spec.seed * 1_000_003 + stream_seed) * 1_000_003 + b)
        labels = torch.randint(0, spec.ncomp, (BLOCK,), generator=gen, device=device)
        noise = torch.randn((BLOCK, spec.d), generator=gen, device=device, dtype=torch.float32)
        x = means[labels] + spec.sigma * noise
        out[pos:pos + take] = x[:take].clamp_(spec.lo, spec.hi)
        pos += take
        b += 1
    return out
