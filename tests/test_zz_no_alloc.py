"""lora_apply_plan_static (the entry point for callers that cannot allocate: its intermediate buffers
are a fixed array in the library's device image) against lora_apply_plan on the same plans, two calls
in a row, the second on a smaller batch; and its refusal of a batch beyond its fixed maximum."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = dict(rel_fro=1e-2, max_abs_over_rms=2e-2, delta_rel_fro=2e-2)


def _mods():
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd import harness as H
    return B, H


def _both_ways(B, H, pi, inst, T, seg_offsets, seg_slot, seg_rank, what):
    """The first T tokens of the instance as one batch through both entry points."""
    h = pi.pool.handle
    sh = torch.cuda.current_stream().cuda_stream
    x, base = inst.x(0)[:T], inst.base_out(0)[:T]
    xd = H.to_device(x, pi.dtype)
    y_pool, y_static = H.to_device(base, pi.dtype), H.to_device(base, pi.dtype)
    rc, plan = B.lora_plan_create(h, T, seg_offsets, seg_slot, seg_rank, sh)
    B.check(rc, "lora_plan_create")
    rc, info = B.lora_plan_info(plan)
    B.check(B.lora_apply_plan(h, plan, 0, 0, xd.data_ptr(), y_pool.data_ptr(), inst.scale, sh), "lora_apply_plan")
    B.check(B.lora_apply_plan_static(h, plan, 0, 0, xd.data_ptr(), y_static.data_ptr(), inst.scale, sh), "lora_apply_plan_static")
    pi.pool.check_fault()
    B.check(B.lora_plan_destroy(h, plan))
    got, want = y_static.float().cpu().numpy(), y_pool.float().cpu().numpy()
    assert not np.array_equal(want, base), f"{what}: the batch must change something"
    m = H.error_metrics(got, want, base)
    for k, lim in TOL.items():
        assert m[k] <= lim, f"{what}: {k} = {m[k]:.3e} > {lim}"
    ta = np.repeat(np.asarray(seg_slot), np.diff(seg_offsets))
    assert np.array_equal(got[ta < 0], base[ta < 0]), f"{what}: tokens without adapter must be untouched"
    return info, bool(np.array_equal(got, want))


def test_static_scratch_entry_point_matches_the_pool_scratch_one():
    B, H = _mods()
    # decode tokens, short and long prompts, requests without adapter; rows long enough for the tile shrink to
    # split them over several blocks (partial sums in the scratch), few enough tokens for the one-launch GEMV form
    inst = wl.make_instance("static", dtype="bf16", seed=4, projs=[wl.Projection("p", 4096, 1024, 0)], n_adapters=12,
                            rank_choices=[8, 16, 32, 64, 128], n_decode=40, prompt_lens=[3, 17, 64, 100, 7, 129], zipf_alpha=1.5,
                            n_base_only=3)
    pi = H.PooledInstance(inst, mfma_min_tokens=16)
    try:
        info, same = _both_ways(B, H, pi, inst, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, "whole batch")
        assert info.n_tiles > 0 and info.n_gemv_shrink_items > 0
        print("first call: outputs bit-identical:", same, flush=True)
        # second call right behind it, on a smaller batch: the leading segments only (the scratch still holds
        # the first call's intermediates)
        n_seg = max(3, inst.n_seg // 3)
        off = np.asarray(inst.seg_offsets[: n_seg + 1], np.int32)
        info2, same2 = _both_ways(B, H, pi, inst, int(off[-1]), off, pi.seg_slot[:n_seg], pi.seg_rank[:n_seg], "leading segments")
        assert info2.T < info.T
        print("second call: outputs bit-identical:", same2, flush=True)
    finally:
        pi.close()


def test_static_scratch_entry_point_refuses_a_batch_beyond_its_maximum():
    B, H = _mods()
    T = B.LORA_STATIC_MAX_TOKENS + 1
    inst = wl.make_instance("long", dtype="bf16", seed=1, projs=[wl.Projection("p", 64, 64, 0)], n_adapters=2,
                            rank_choices=[8], n_decode=0, prompt_lens=[T], zipf_alpha=None)
    pi = H.PooledInstance(inst)
    try:
        h = pi.pool.handle
        sh = torch.cuda.current_stream().cuda_stream
        xd = torch.zeros((T, 64), dtype=torch.bfloat16, device="cuda:0")
        yd = torch.ones((T, 64), dtype=torch.bfloat16, device="cuda:0")
        rc, plan = B.lora_plan_create(h, T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, sh)
        B.check(rc)
        assert B.lora_apply_plan_static(h, plan, 0, 0, xd.data_ptr(), yd.data_ptr(), 2.0, sh) == B.LORA_E_NOMEM
        torch.cuda.synchronize()
        assert bool((yd == 1).all())  # nothing was enqueued
        B.check(B.lora_apply_plan(h, plan, 0, 0, xd.data_ptr(), yd.data_ptr(), 2.0, sh))  # the pool's scratch takes it
        torch.cuda.synchronize()
        B.check(B.lora_plan_destroy(h, plan))
    finally:
        pi.close()
