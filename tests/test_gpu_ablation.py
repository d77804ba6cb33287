"""The ablation module runs and reports what the definitions fix: with the cache emptied
before every step every selected row is fetched (miss rate 1); with the hit/miss cache fewer."""
import io
import re

import pytest

pytestmark = pytest.mark.gpu


def test_no_hit_miss_fetches_every_selected_row():
    from paper_2510_23649_amd import ablation
    buf = io.StringIO()
    ablation.no_hit_miss(steps=4, layers=1, out=buf)
    rows = [ln for ln in buf.getvalue().splitlines() if ln.startswith("| ") and "variant" not in ln]
    default, emptied = (re.split(r"\s*\|\s*", ln.strip("| ")) for ln in rows[-2:])
    assert int(emptied[2]) == 32 * 2048            # B * Hq * k rows of workload 3
    assert 0 < int(default[2]) < int(emptied[2]) // 2
    assert float(emptied[1]) > float(default[1])   # and it costs time


# ---- the two cache experiments against the oracle, step by step -----------------------------------

def _steps_vs_oracle(cfg, n_steps, empty_before_every_step):
    """Per-step n_miss of lrqk_decode_step and of the oracle's decode_step on the same seeds."""
    import numpy as np
    import torch
    import paper_2510_23649_amd as L
    from gen import make_layer, QueryStream, as_numpy
    from gpu_harness import DEV, DeviceLayer, StepBuffers
    from oracle import lrqk_oracle as orc
    data = make_layer(cfg)
    dl = DeviceLayer(cfg, data)
    plan = L.Plan(dl.shape)
    qs = QueryStream(data)
    sb = StepBuffers(cfg)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    per_step = []
    for step in range(1, n_steps + 1):
        q, q_hat = qs.next()
        if empty_before_every_step:          # App. C.2, "no hit/miss": nothing is kept on the GPU
            L.lrqk_cache_init(dl.shape, dl.slot_of, dl.token_of, dl.last_used)
            dl.ost = orc.CacheState(cfg.B, cfg.Hq, cfg.l, cfg.C)
        flags = L.LRQK_SELECT_FRESH if step == 1 else 0
        L.lrqk_decode_step(plan, dl.shape, step, dl.struct(), q_hat.to(DEV), q.to(DEV), out,
                           L.LRQK_FETCH_DIRECT | flags, sb.debug())
        got = sb.to_np()
        ref = orc.decode_step(dl.np["A_K"], as_numpy(q_hat), as_numpy(q), dl.np["K"], dl.np["V"],
                              dl.ost, dl.ocK, dl.ocV, step, cfg.k, cfg.w, cfg.scale)
        assert ref["ok"]
        assert np.array_equal(got["n_miss"], ref["n_miss"]), f"step {step}: n_miss differs"
        assert np.array_equal(got["sel_idx"], ref["sel_idx"]), f"step {step}: selection differs"
        assert np.array_equal(got["hit"], ref["hit"]), f"step {step}: hit map differs"
        assert np.abs(out.cpu().numpy() - ref["out"]).max() <= 2e-3
        # Sec. 5.3: miss rate = rows fetched / rows selected
        per_step.append(float(got["n_miss"].sum()) / (cfg.B * cfg.Hq * cfg.k))
        assert per_step[-1] == pytest.approx(ref["miss_rate"], abs=1e-12)
    plan.close()
    return per_step


@pytest.mark.parametrize("r", [8, 64])
def test_miss_rate_grid_cell_matches_oracle(r):
    """Two cells of the miss-rate grid (Sec. 5.3): cache of exactly k slots, l = 4096, 256 active
    and 8 lite tokens, rank 8 and 64; 10 steps, every step's n_miss per head equal to the oracle's."""
    from gen import get_config
    cfg = get_config("c2").with_(l=4096, r=r, k=256, w=8, C=256, n_heavy=64, pool_mult=4)
    rates = _steps_vs_oracle(cfg, 10, empty_before_every_step=False)
    print(f"miss-rate grid cell r={r}: " + " ".join(f"{x:.3f}" for x in rates), flush=True)
    assert rates[0] == 1.0 and 0.0 < rates[-1] < 1.0


def test_no_hit_miss_variant_matches_oracle():
    """App. C.2 "no hit/miss": the cache is emptied before every step, so every selected row is
    fetched again -- n_miss = k for every head and step, on the GPU and in the oracle alike."""
    from gen import get_config
    cfg = get_config("c2").with_(l=4096, r=32, k=256, w=8, C=256, n_heavy=64, pool_mult=4)
    rates = _steps_vs_oracle(cfg, 8, empty_before_every_step=True)
    assert rates == [1.0] * 8
