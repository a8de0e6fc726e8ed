"""Shared test plumbing: upload a synthetic workload, call the C-ABI through the binding, and
compare against the float64 oracle."""
import numpy as np


def to_device(p, dtype, device="cuda:0", layout="bhnd"):
    """NumPy workload dict -> torch tensors on the GPU (storage dtype for the big tensors)."""
    import torch
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    t = {}
    for k in ("Q", "K", "V", "dO"):
        if k in p:
            x = torch.from_numpy(p[k]).to(device).to(tdt)
            if layout == "bnhd":   # physically (B, n, H, d), presented as (B, H, n, d)
                x = x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            t[k] = x
    t["Omega"] = torch.from_numpy(p["Omega"]).to(device).to(tdt)
    for k in ("Wg", "bg", "omega"):
        t[k] = torch.from_numpy(np.ascontiguousarray(p[k], dtype=np.float32)).to(device)
    t["sigma"] = torch.tensor([float(p["sigma"])], dtype=torch.float32, device=device)
    return t


def gpu_forward_backward(p, cfg, backward=True, eps=1e-6, bw_floor=1e-6, layout="bhnd"):
    import torch
    from paper_2507_08637_amd import binding
    t = to_device(p, cfg["dtype"], layout=layout)
    out, saved = binding.wersa_forward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"],
                                       t["omega"], cfg["L"], eps=eps, bw_floor=bw_floor)
    res = dict(O=out)
    desc = binding.make_desc(t["Q"], cfg["L"], cfg["m"], eps, bw_floor)
    res["saved"] = {k: v.clone() for k, v in binding.saved_views(desc, saved).items()}
    if backward:
        g = binding.wersa_backward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"],
                                   t["omega"], out, t["dO"], saved, cfg["L"], eps=eps, bw_floor=bw_floor)
        res.update(dQ=g["dq"], dK=g["dk"], dV=g["dv"], dWg=g["dgate_w"], dbg=g["dgate_b"],
                   domega=g["dscale_w"], dsigma=g["dsigma"])
    torch.cuda.synchronize()
    return res


def oracle_backward(p, cfg, eps=1e-6, bw_floor=1e-6, slices=None):
    from oracle import wersa_oracle as wo
    return wo.backward(p["Q"], p["K"], p["V"], p["Omega"], float(p["sigma"]), p["Wg"], p["bg"],
                       p["omega"], cfg["L"], p["dO"], eps=eps, bw_floor=bw_floor, slices=slices)


def oracle_forward(p, cfg, eps=1e-6, bw_floor=1e-6, slices=None,
                   keep=("O", "S", "z", "qbar", "s", "F", "D")):
    from oracle import wersa_oracle as wo
    return wo.forward(p["Q"], p["K"], p["V"], p["Omega"], float(p["sigma"]), p["Wg"], p["bg"],
                      p["omega"], cfg["L"], eps=eps, bw_floor=bw_floor, slices=slices, keep=keep)


def rel_err(gpu, ref):
    """||gpu - ref||_F / ||ref||_F with gpu a torch tensor and ref a float64 array."""
    a = gpu.detach().float().cpu().numpy().astype(np.float64).reshape(ref.shape)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(a - ref) / (den if den > 0 else 1.0))
