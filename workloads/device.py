"""Seeded synthetic inputs drawn directly on the GPU (for the large workloads, where drawing on
the host and uploading would dominate).  Only torch's generator and dtype conversion are used;
none of the method's arithmetic lives here."""
from __future__ import annotations


def make_device_inputs(wl, micro_steps, device):
    """Seeded synthetic inputs generated on the device: x ~ |N(0,1)|, dy ~ N(0, 1e-4) (variance),
    rounded to bf16 (nearest-even) by the dtype conversion."""
    import torch
    gen = torch.Generator(device=device)
    out = []
    for m in range(micro_steps):
        layers = []
        for li, l in enumerate(wl.layers):
            gen.manual_seed(wl.data_seed * 1_000_003 + m * 1009 + li)
            x = torch.randn((wl.n,) + tuple(l.x_shape), generator=gen, device=device, dtype=torch.float32)
            dist = wl.x_dist[li]
            if dist == "absnormal":
                x = x.abs_()
            elif dist == "relu":
                x = x.clamp_(min=0)
            dy = torch.randn((wl.n,) + tuple(l.dy_shape), generator=gen, device=device, dtype=torch.float32)
            dy.mul_(wl.dy_std)
            if wl.dtype == "bf16":
                x, dy = x.to(torch.bfloat16), dy.to(torch.bfloat16)
            layers.append((x.contiguous(), dy.contiguous()))
        out.append(layers)
    return out
