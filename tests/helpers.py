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
    om = p["Omega"] if "OmegaK" not in p else np.stack([p["Omega"], p["OmegaK"]])
    t["Omega"] = torch.from_numpy(np.ascontiguousarray(om)).to(device).to(tdt)
    for k in ("Wg", "bg", "omega"):
        t[k] = torch.from_numpy(np.ascontiguousarray(p[k], dtype=np.float32)).to(device)
    t["sigma"] = torch.tensor([float(p["sigma"])], dtype=torch.float32, device=device)
    return t


def gpu_forward_backward(p, cfg, backward=True, eps=1e-6, bw_floor=1e-6, layout="bhnd", flags=0):
    import torch
    from paper_2507_08637_amd import binding
    t = to_device(p, cfg["dtype"], layout=layout)
    out, saved = binding.wersa_forward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"],
                                       t["omega"], cfg["L"], eps=eps, bw_floor=bw_floor, flags=flags)
    res = dict(O=out)
    desc = binding.make_desc(t["Q"], cfg["L"], cfg["m"], eps, bw_floor, flags)
    res["saved"] = {k: v.clone() for k, v in binding.saved_views(desc, saved).items()}
    if backward:
        g = binding.wersa_backward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"],
                                   t["omega"], out, t["dO"], saved, cfg["L"], eps=eps, bw_floor=bw_floor,
                                   flags=flags)
        res.update(dQ=g["dq"], dK=g["dk"], dV=g["dv"], dWg=g["dgate_w"], dbg=g["dgate_b"],
                   domega=g["dscale_w"], dsigma=g["dsigma"])
    torch.cuda.synchronize()
    return res


def oracle_backward(p, cfg, eps=1e-6, bw_floor=1e-6, slices=None, proj_dtype=None, pooled=False,
                    layernorm=False):
    from oracle import wersa_oracle as wo
    return wo.backward(p["Q"], p["K"], p["V"], p["Omega"], float(p["sigma"]), p["Wg"], p["bg"],
                       p["omega"], cfg["L"], p["dO"], eps=eps, bw_floor=bw_floor, slices=slices,
                       proj_dtype=proj_dtype, Omega_K=p.get("OmegaK"), pooled=pooled, layernorm=layernorm)


def oracle_forward(p, cfg, eps=1e-6, bw_floor=1e-6, slices=None,
                   keep=("O", "S", "z", "qbar", "s", "F", "D"), layernorm=False):
    from oracle import wersa_oracle as wo
    return wo.forward(p["Q"], p["K"], p["V"], p["Omega"], float(p["sigma"]), p["Wg"], p["bg"],
                      p["omega"], cfg["L"], eps=eps, bw_floor=bw_floor, slices=slices, keep=keep,
                      Omega_K=p.get("OmegaK"), layernorm=layernorm)


def rel_err(gpu, ref):
    """||gpu - ref||_F / ||ref||_F with gpu a torch tensor and ref a float64 array."""
    a = gpu.detach().float().cpu().numpy().astype(np.float64).reshape(ref.shape)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(a - ref) / (den if den > 0 else 1.0))


def gate_grad_scales(p, cfg, eps=1e-6, bw_floor=1e-6, layernorm=False):
    """Un-cancelled magnitudes of the gate-parameter gradients, for conditioning-aware checks.

    dF_i of one slice is an inner product <band_i(W dX_F), band_i(W X)> summed over Q and K.  On
    seeded random inputs the two factors are uncorrelated, so the product nearly cancels:
    |dF_i| is about ||g_i|| ||c_i|| / sqrt(N_i) or less.  A kernel that delivers dX_F with a
    relative error tau therefore delivers dF_i with an absolute error of about
    tau * ||g_i|| ||c_i|| / sqrt(N_i), whatever |dF_i| happens to be.  This returns that scale
    (without tau), pushed through the gate chain to dWg, dbg and domega.
    """
    from oracle import wersa_oracle as wo
    B, H, L, d = cfg["B"], cfg["H"], cfg["L"], cfg["d"]
    floor = np.zeros((B, H, L + 1))
    s_all = np.zeros((B, H, L + 1))
    qbar = np.zeros((B, H, d))
    omega = np.asarray(p["omega"], np.float64)
    Om = np.asarray(p["Omega"], np.float64)
    for b in range(B):
        for h in range(H):
            args = (np.asarray(p["Q"][b, h], np.float64), np.asarray(p["K"][b, h], np.float64),
                    np.asarray(p["V"][b, h], np.float64), Om, float(p["sigma"]),
                    np.asarray(p["Wg"][h], np.float64), np.asarray(p["bg"][h], np.float64), omega, L,
                    eps, bw_floor)
            r = wo.backward_slice(*args, np.asarray(p["dO"][b, h], np.float64), Omega_K=p.get("OmegaK"),
                                  layernorm=layernorm)
            f = wo.forward_slice(*args, Omega_K=p.get("OmegaK"), layernorm=layernorm)
            s_all[b, h], qbar[b, h] = f["s"], f["qbar"]
            for X, G in ((args[0], r["dQF"]), (args[1], r["dKF"])):
                cx, _ = wo.haar_dwt(X, L)
                cg, _ = wo.haar_dwt(G, L)
                for i in range(L + 1):
                    floor[b, h, i] += np.linalg.norm(cx[i]) * np.linalg.norm(cg[i]) / np.sqrt(cx[i].size)
    dlogit = floor * omega[None, None, :] * s_all * (1.0 - s_all)
    return dict(domega=np.sqrt(np.sum((floor * s_all) ** 2, axis=(0, 1))),
                dbg=np.sqrt(np.sum(dlogit ** 2, axis=0)),
                dWg=np.sqrt(np.einsum("bhi,bhj->hij", dlogit ** 2, qbar ** 2)))


def scaled_err(gpu, ref, scale):
    """||gpu - ref||_F / ||scale||_F."""
    a = gpu.detach().float().cpu().numpy().astype(np.float64).reshape(ref.shape)
    return float(np.linalg.norm(a - ref) / np.linalg.norm(scale))


def err_stats(gpu, ref, rows=64):
    """Error figures of one (..., n, d) output against the oracle: relative Frobenius error, largest
    absolute error over the largest absolute value of the oracle, and the worst relative Frobenius
    error over the aligned blocks of `rows` rows (a partial last block counts as a block)."""
    a = gpu.detach().float().cpu().numpy().astype(np.float64).reshape(ref.shape)
    diff = a - ref
    n, d = ref.shape[-2], ref.shape[-1]
    lead = int(np.prod(ref.shape[:-2])) if ref.ndim > 2 else 1
    d2 = (diff.reshape(lead, n, d) ** 2).sum(-1)
    r2 = (ref.reshape(lead, n, d) ** 2).sum(-1)
    pad = (-n) % rows
    if pad:
        d2 = np.pad(d2, ((0, 0), (0, pad)))
        r2 = np.pad(r2, ((0, 0), (0, pad)))
    db = d2.reshape(lead, -1, rows).sum(-1)
    rb = r2.reshape(lead, -1, rows).sum(-1)
    return dict(fro=float(np.sqrt(d2.sum() / r2.sum())),
                maxabs=float(np.abs(diff).max() / np.abs(ref).max()),
                worst_block=float(np.sqrt((db / np.maximum(rb, 1e-300)).max())))
