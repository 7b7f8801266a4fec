"""Seeded random small batches through lora_apply and lora_linear_plan, every token against the fp64
oracle: projection widths from 64 to 1024, ranks anywhere in 1..128, any mix of decode tokens, prompts
and requests without an adapter, per-entry factors, every tile threshold and both forms of the GEMV
launch.  The cases are drawn from the seed alone, so a failure names its case."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TOL = {"bf16": dict(rel_fro=1e-2, max_abs_over_rms=2e-2, delta_rel_fro=2e-2),
       "f32": dict(rel_fro=1e-5, max_abs_over_rms=1e-4, delta_rel_fro=1e-4)}


def _draw(case):
    from paper_2411_17741_amd import binding as B
    rng = np.random.default_rng(1000 + case)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    dims = [int(64 * rng.integers(1, 17)) for _ in range(3)]
    projs = [wl.Projection("a", dims[0], dims[1], 0), wl.Projection("b", dims[1], dims[2], 1)]
    ranks = set(int(r) for r in rng.integers(1, 129, size=int(rng.integers(1, 6))))
    if rng.random() < 0.5:
        ranks |= {8, 128}
    lens = [int(rng.integers(1, 300)) for _ in range(int(rng.integers(0, 6)))]
    kw = dict(dtype=dtype, seed=case, projs=projs, n_adapters=int(rng.integers(1, 20)), rank_choices=sorted(ranks),
              n_decode=int(rng.integers(0, 90)), prompt_lens=lens, zipf_alpha=float(rng.choice([0.8, 1.0, 1.5, 2.5])),
              n_base_only=int(rng.integers(0, 5)), scale=float(rng.choice([0.5, 1.0, 2.0])))
    if kw["n_decode"] + len(lens) + kw["n_base_only"] == 0:
        kw["n_decode"] = 1
    m0 = int(rng.choice([0, 1, 8, 16, 64, 1000]))
    flags = int(rng.choice([0, B.LORA_CACHE_FUSED_GEMV, B.LORA_CACHE_SPLIT_GEMV]))
    inst = wl.make_instance(f"random{case}", **kw)
    inst.alpha = (1.0 + 0.25 * (np.arange(inst.n_adapters) % 3)).astype(np.float32)
    return inst, m0, flags


@pytest.mark.parametrize("case", range(24))
def test_random_instance(case):
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd import harness as H
    inst, m0, flags = _draw(case)
    what = f"case {case}: {inst.dtype} {[(p.h_in, p.h_out) for p in inst.projs]} tile threshold {m0} flags {flags}"
    pi = H.PooledInstance(inst, mfma_min_tokens=m0, flags=flags)
    try:
        ta = inst.token_adapter()
        for p, pr in enumerate(inst.projs):
            x, base = inst.x(p), inst.base_out(p)
            xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
            pi.apply(0, p, xd, yd)
            pi.pool.check_fault()
            y = yd.float().cpu().numpy()
            ads = {int(a): (*inst.adapter_weights(int(a), p), float(inst.alpha[a])) for a in inst.used_adapters()}
            ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, ads, inst.scale)
            m = H.error_metrics(y, ref, base, inst.dtype)
            for k, lim in TOL[inst.dtype].items():
                assert m[k] <= lim, f"{what}, proj {p}: {k} = {m[k]:.3e} > {lim}"
            assert np.array_equal(y[ta < 0], base[ta < 0]), f"{what}: tokens without adapter must be untouched"
            if inst.dtype != "bf16":
                continue
            W = wl.bf16_round(np.random.default_rng(case).normal(0, 0.02, size=(pr.h_in, pr.h_out)).astype(np.float32))
            wtd = H.to_device(np.ascontiguousarray(W.T), pi.dtype)
            yl = torch.full((inst.T, pr.h_out), float("nan"), dtype=torch.bfloat16, device=xd.device)
            plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
            rc, ws_bytes = B.lora_linear_workspace_bytes(pi.pool.handle, plan, p)
            B.check(rc)
            ws = torch.full((max(1, ws_bytes // 4),), float("nan"), dtype=torch.float32, device=xd.device)
            B.check(B.lora_linear_plan(pi.pool.handle, plan, 0, p, xd.data_ptr(), wtd.data_ptr(), yl.data_ptr(), inst.scale,
                                       torch.cuda.current_stream().cuda_stream, workspace=ws.data_ptr(), workspace_bytes=ws_bytes))
            pi.pool.check_fault()
            ylin = yl.float().cpu().numpy()
            pi.pool.plan_destroy(plan)
            assert np.isfinite(ylin).all(), f"{what}, proj {p}: lora_linear_plan left rows unwritten"
            base64 = x.astype(np.float64) @ W.astype(np.float64)
            ref = oracle.lora_apply(x, base64, inst.seg_offsets, inst.seg_adapter, ads, inst.scale)
            m = H.error_metrics(ylin, ref, base64)
            for k, lim in TOL["bf16"].items():
                if k == "delta_rel_fro" and not (ta >= 0).any():
                    continue  # a batch without any adapter has no delta to measure against
                assert m[k] <= lim, f"{what}, proj {p}, fused linear: {k} = {m[k]:.3e} > {lim}"
    finally:
        pi.close()
