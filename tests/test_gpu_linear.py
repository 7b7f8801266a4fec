"""Base projection and adapter update in one pass (lora_linear_plan): y = x.W + s.(x.A).B for every token
of a mixed batch, against the fp64 oracle applied to the fp64 base product."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TOL = dict(rel_fro=1e-2, max_abs_over_rms=2e-2, delta_rel_fro=2e-2)


def _mods():
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd import harness as H
    return B, H


def _weight(inst, p, seed):
    pr = inst.projs[p]
    w = np.random.default_rng(seed).normal(0.0, 0.02, size=(pr.h_in, pr.h_out)).astype(np.float32)
    return wl.bf16_round(w)


def _run(inst, p, rows, seed=0, mfma_min_tokens=0, workspace=True):
    B, H = _mods()
    pi = H.PooledInstance(inst, n_layers=1, mfma_min_tokens=mfma_min_tokens)
    try:
        x, W = inst.x(p), _weight(inst, p, seed)
        xd = H.to_device(x, pi.dtype)
        wtd = H.to_device(np.ascontiguousarray(W.T), pi.dtype)                 # [h_out][h_in]
        yd = torch.full((inst.T, inst.projs[p].h_out), float("nan"), dtype=torch.bfloat16, device=xd.device)  # written only
        plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        st = torch.cuda.current_stream().cuda_stream
        rc, ws_bytes = B.lora_linear_workspace_bytes(pi.pool.handle, plan, p)
        B.check(rc)
        ws = torch.full((max(1, ws_bytes // 4),), float("nan"), dtype=torch.float32, device=xd.device) if workspace else None
        B.check(B.lora_linear_plan(pi.pool.handle, plan, 0, p, xd.data_ptr(), wtd.data_ptr(), yd.data_ptr(), inst.scale, st,
                                   workspace=ws.data_ptr() if workspace else 0, workspace_bytes=ws_bytes if workspace else 0))
        pi.pool.check_fault()
        y_rows = yd[torch.from_numpy(rows).to(yd.device)].float().cpu().numpy()
        assert np.isfinite(y_rows).all()
        base_rows = x[rows].astype(np.float64) @ W.astype(np.float64)
        ta = inst.token_adapter()[rows]
        ads = {int(a): (*inst.adapter_weights(int(a), p), float(inst.alpha[a])) for a in np.unique(ta[ta >= 0])}
        ref = oracle.lora_apply(x[rows], base_rows, np.arange(len(rows) + 1, dtype=np.int32), ta.astype(np.int32), ads, inst.scale)
        m = H.error_metrics(y_rows, ref, base_rows)
        for k, lim in TOL.items():
            assert m[k] <= lim, f"{inst.name} proj {p}: {k} = {m[k]:.3e} > {lim}"
        # tokens without an adapter get the base product alone (to the rounding of the stored bf16)
        none = ta < 0
        if none.any():
            assert np.abs(y_rows[none] - base_rows[none]).max() <= 2.0**-8 * np.abs(base_rows[none]).max()
        pi.pool.plan_destroy(plan)
        return m
    finally:
        pi.close()


@pytest.mark.parametrize("workspace", [True, False])
@pytest.mark.parametrize("mfma_min_tokens", [0, 16])
def test_linear_small_mixed_every_token(mfma_min_tokens, workspace):
    """Decode tokens, short and long prompts with ragged tails, a hot adapter, tokens without an adapter;
    512 -> 640: the last column block is partial.  With the fp32 workspace for the adapter term of the GEMV
    tokens and without (the term then passes through the bf16 output rows)."""
    base = wl.small_mixed(seed=5)
    projs = [wl.Projection("g", 512, 640, 0), wl.Projection("d", 640, 320, 1)]
    inst = wl.Instance(name="lin_small", dtype="bf16", seed=5, projs=projs, ranks=base.ranks, adapter_ids=base.adapter_ids,
                       alpha=base.alpha, scale=base.scale, seg_offsets=base.seg_offsets, seg_adapter=base.seg_adapter)
    for p in range(2):
        _run(inst, p, np.arange(inst.T, dtype=np.int64), seed=p, mfma_min_tokens=mfma_min_tokens, workspace=workspace)


def test_linear_prefill_config_sampled():
    inst = wl.prefill()
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([rng.integers(0, inst.T, size=160), inst.seg_offsets[:-1], inst.seg_offsets[1:] - 1,
                                     inst.seg_offsets[:-1] + 63, inst.seg_offsets[:-1] + 64])).astype(np.int64)
    rows = rows[rows < inst.T]
    _run(inst, 0, rows)


def test_linear_workspace_arguments():
    B, H = _mods()
    inst = wl.small_mixed(seed=2)
    pi = H.PooledInstance(inst, n_layers=1)
    try:
        plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        rc, need = B.lora_linear_workspace_bytes(pi.pool.handle, plan, 0)
        assert rc == B.LORA_OK and need == inst.T * inst.projs[0].h_out * 4   # the small batch is all on the GEMV path
        x = H.to_device(inst.x(0), pi.dtype)
        wt = torch.zeros((inst.projs[0].h_out, inst.projs[0].h_in), dtype=torch.bfloat16, device=x.device)
        y = torch.zeros((inst.T, inst.projs[0].h_out), dtype=torch.bfloat16, device=x.device)
        ws = torch.zeros((need // 4 + 4,), dtype=torch.float32, device=x.device)
        call = lambda ptr, n: B.lora_linear_plan(pi.pool.handle, plan, 0, 0, x.data_ptr(), wt.data_ptr(), y.data_ptr(), 1.0, 0,
                                                 workspace=ptr, workspace_bytes=n)
        assert call(ws.data_ptr(), need - 4) == B.LORA_E_INVAL       # too small
        assert call(ws.data_ptr() + 4, need) == B.LORA_E_INVAL       # not 16-byte aligned
        assert call(ws.data_ptr(), need) == B.LORA_OK
        assert B.lora_linear_workspace_bytes(pi.pool.handle, plan, 9)[0] == B.LORA_E_INVAL
        torch.cuda.synchronize()
        pi.pool.plan_destroy(plan)
    finally:
        pi.close()
