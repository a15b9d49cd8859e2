"""Profile-guided partition: time every unit of the UNet on the device (each unit run alone as its own
component through ad_component_forward) and split the units into N components of comparable measured time
with the library's own partition rule (ad_balance_cuts).  Section 3.2 of the paper asks for components of
comparable load; FLOPs are the default measure (ad_create), measured time is the better one on a device
whose small layers run far below its peak."""
import time

import torch

from .binding import AD_BF16, AsyncDiff, balance_cuts


def measure_unit_times(cfg_dict, dtype, weights, device="cuda:0", reps=5):
    """Microseconds per unit (list of ints), one stream, inputs of the right shape filled with noise."""
    probe = AsyncDiff(cfg_dict, 1, 0, 1, dtype)
    nu = len(probe.units())
    probe.close()
    m = AsyncDiff(cfg_dict, nu, 1, 1, dtype, cuts=list(range(1, nu)))
    m.allocate(device)
    m.load_weights(weights)
    m.reset(50)
    tdt = torch.bfloat16 if dtype == AD_BF16 else torch.float32
    frames = cfg_dict.get("frames", 0)           # video model: one latent per frame, one text embedding for all frames
    text = torch.randn(1 if frames else cfg_dict["batch"], cfg_dict["ctx_len"], cfg_dict["ctx_dim"], device=device).to(tdt)
    pooled = torch.randn(cfg_dict["batch"], cfg_dict["pooled_dim"], device=device) if cfg_dict.get("pooled_dim") else None
    latent = torch.randn(max(1, frames), cfg_dict["latent_channels"], cfg_dict["height"], cfg_dict["width"], device=device)

    def alloc(u):
        (b, h, w, c), _ = m.tensor_shape(u)
        if u == nu - 1:
            return torch.zeros(b, c, h, w, device=device)
        return (torch.randn(b, h, w, c, device=device) * 0.5).to(tdt)

    s = torch.cuda.Stream(device=device)
    m.precompute_text(text, s)
    torch.cuda.synchronize()
    out = []
    for comp in range(1, nu + 1):
        ins, outs = m.component_io(comp)
        tin = [latent if u < 0 else alloc(u) for u in ins]
        tout = [alloc(u) for u in outs]
        m.component_forward(comp, tin, 10, text, tout, s, pooled=pooled)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            m.component_forward(comp, tin, 10, text, tout, s, pooled=pooled)
        torch.cuda.synchronize()
        out.append(max(1, int(round((time.perf_counter() - t0) / reps * 1e6))))
    m.close()
    return out


def time_balanced_cuts(cfg_dict, n_components, dtype, weights, device="cuda:0"):
    """Cuts for AsyncDiff(..., cuts=...) that balance the measured unit times; also returns the times."""
    times = measure_unit_times(cfg_dict, dtype, weights, device)
    return balance_cuts(times, n_components), times
