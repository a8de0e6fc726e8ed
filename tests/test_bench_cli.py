"""Host-side checks of bench.py's command line (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    """This build runs on one GPU: any other --gpus value exits before anything touches a device."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_kernel_models_count_the_contractions():
    """Algorithmic work per launch at configuration 4: one contraction is 2 n d m flops per slice."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2507_08637_amd import workloads
    cfg = dict(workloads.CONFIGS[4])
    unit = 2.0 * cfg["n"] * cfg["d"] * cfg["m"] * cfg["B"] * cfg["H"]
    m = bench.kernel_models(cfg)
    assert m["wersa_phiT_contract"][2] == 2 * unit and m["wersa_rows_fwd"][2] == 2 * unit
    assert m["wersa_rows_bwd_q"][2] == 3 * unit and m["wersa_rows_bwd_k"][2] == 4 * unit   # with dV
    nd = cfg["n"] * cfg["d"] * cfg["B"] * cfg["H"]
    assert m["wersa_qbar"][2] == 2 * nd and m["wersa_add_pooled"][2] == 4 * nd            # bf16 bytes
    cfg3 = dict(cfg, n=cfg["n"] + 1)                                                       # partial last block:
    assert bench.kernel_models(cfg3)["wersa_rows_bwd_k"][2] == 3 * 2.0 * cfg3["n"] * cfg["d"] * cfg["m"] * 8   # dV is its own launch
