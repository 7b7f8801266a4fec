"""GPU parity at the full sizes of the larger configurations, in the launch configuration the
benchmark times (same batch, shapes, pool and plan flow: one plan, the projections of a layer
handed to lora_apply_plan_multi in order, so that q,k,v and gate,up go out as groups).  Every
token of every projection is compared with the oracle (which takes the batch in slices of whole
segments to bound its memory).  Also here: fills on a side stream overlapped with applies (a miss
of the next iteration is loaded while the current one runs) and a refill of a slot that an
enqueued apply still reads."""
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


def _check_every_token(inst, p, y, x, base, seg_adapter, what, max_slice_tokens=3072):
    """y, x, base: full [T][..] arrays of projection p; seg_adapter: adapter per segment (-1: none)."""
    B, H = _mods()
    off = np.asarray(inst.seg_offsets, np.int64)
    n_seg = len(seg_adapter)
    weights = {}
    ref = np.empty_like(base, dtype=np.float64)
    g = 0
    while g < n_seg:
        e = g + 1
        while e < n_seg and off[e + 1] - off[g] <= max_slice_tokens:
            e += 1
        lo, hi = int(off[g]), int(off[e])
        sa = np.asarray(seg_adapter[g:e], np.int32)
        for a in np.unique(sa[sa >= 0]):
            if int(a) not in weights:
                weights[int(a)] = (*inst.adapter_weights(int(a), p), float(inst.alpha[a]))
        ads = {int(a): weights[int(a)] for a in np.unique(sa[sa >= 0])}
        ref[lo:hi] = oracle.lora_apply(x[lo:hi], base[lo:hi], (off[g : e + 1] - lo).astype(np.int32), sa, ads, inst.scale)
        g = e
    m = H.error_metrics(y, ref, base)
    for k, lim in TOL.items():
        assert m[k] <= lim, f"{what}: {k} = {m[k]:.3e} > {lim}"
    ta = np.repeat(np.asarray(seg_adapter), np.diff(off))
    assert np.array_equal(y[ta < 0], base[ta < 0]), f"{what}: tokens without adapter must be untouched"
    return m


def _run_full(inst, n_layers=1, layer=0, adapters=None):
    """Plan once, apply all projections of the layer in one lora_apply_plan_multi call (the
    benchmark's flow: consecutive projections that read the same activations form a group),
    compare every token of every projection."""
    B, H = _mods()
    pi = H.PooledInstance(inst, n_layers=n_layers, fill_layers=[layer], adapters=adapters)
    try:
        from plan_checks import check_plan_units

        plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        # the lists the kernels will read, fetched back from the device
        alpha_of_slot = {int(pi.slot_of[a]): float(inst.alpha[a]) for a in inst.used_adapters()}
        check_plan_units(pi.pool.handle, plan, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank,
                         [(pr.h_in, pr.h_out) for pr in inst.projs], alpha_of_slot)
        xs, xds, yds = {}, {}, []
        for p, pr in enumerate(inst.projs):
            if pr.x_key not in xs:
                xs[pr.x_key] = inst.x(p)
                xds[pr.x_key] = H.to_device(xs[pr.x_key], pi.dtype)
            yds.append(H.to_device(inst.base_out(p), pi.dtype))
        descs = B.make_descs([(layer, p, xds[pr.x_key].data_ptr(), yds[p].data_ptr()) for p, pr in enumerate(inst.projs)])
        sh = torch.cuda.current_stream().cuda_stream
        B.check(B.lora_apply_plan_multi(pi.pool.handle, plan, descs, inst.scale, sh), "lora_apply_plan_multi")
        pi.pool.check_fault()
        for p, pr in enumerate(inst.projs):
            print(f"checking {inst.name} projection {pr.name}", flush=True)
            y = yds[p].float().cpu().numpy()
            _check_every_token(inst, p, y, xs[pr.x_key], inst.base_out(p), inst.seg_adapter, f"{inst.name} proj {pr.name}")
            yds[p] = None
        pi.pool.plan_destroy(plan)
    finally:
        pi.close()


def test_mixed_config_full_size_every_token_of_all_projections():
    _run_full(wl.mixed())


def test_stress_config_full_size_every_token_of_all_projections():
    """All seven projections of the 13B-shaped layer (q,k,v,o 5120 -> 5120, gate, up 5120 -> 13824, down
    13824 -> 5120: the tile shrink splits its long rows over several blocks) with every adapter of the batch
    resident.  One layer copy: the 39 GB pool is the subject of the next test."""
    _run_full(wl.stress())


def test_prefill_config_full_size_other_seed():
    _run_full(wl.prefill(seed=1))


@pytest.mark.parametrize("n_adapters,n_decode", [(10, 64), (200, 64), (150, 512)])
def test_decode_with_the_papers_adapter_population(n_adapters, n_decode):
    """The adapter population of the paper's own workload (N_a / 5 adapters of every rank, rank
    uniform, power law within the rank) at both ends of its sweep over N_a: every token checked."""
    inst = wl.decode_paper(n_adapters=n_adapters, n_decode=n_decode)
    assert np.array_equal(np.bincount(inst.ranks)[[8, 16, 32, 64, 128]], [n_adapters // 5] * 5)
    _run_full(inst)


def test_stress_config_with_fills_overlapping_applies():
    """13B-shaped layer, pool of 1000 adapters in 4 layer copies (~39 GB).  Iteration k runs
    without the requests whose adapters are missing while those adapters are filled from pinned
    host memory on a side stream; iteration k+1 runs the whole batch and waits, on the device,
    for the fills it needs."""
    B, H = _mods()
    inst = wl.stress()
    assert len(inst.miss_adapters) > 0
    layer = 2
    resident = np.setdiff1d(inst.used_adapters(), inst.miss_adapters)
    pi = H.PooledInstance(inst, n_layers=inst.n_layers, fill_layers=[layer], adapters=resident)
    try:
        assert pi.pool.bytes > 35e9
        ta_full = inst.token_adapter()
        miss_mask_seg = np.isin(inst.seg_adapter, inst.miss_adapters)
        seg_slot_k = np.where(miss_mask_seg, -1, pi.seg_slot).astype(np.int32)   # iteration k: misses deferred
        seg_adapter_k = np.where(miss_mask_seg, -1, inst.seg_adapter).astype(np.int32)
        assert np.isin(ta_full, inst.miss_adapters).sum() > 0

        side = torch.cuda.Stream()
        main = torch.cuda.current_stream()
        p = 4  # gate projection: 5120 -> 13824
        x, base = inst.x(p), inst.base_out(p)
        xd = H.to_device(x, pi.dtype)
        y_k, y_k1 = H.to_device(base, pi.dtype), H.to_device(base, pi.dtype)
        torch.cuda.synchronize()

        # iteration k on the main stream, fills of the missing adapters on the side stream
        B.check(B.lora_apply(pi.pool.handle, layer, p, xd.data_ptr(), y_k.data_ptr(), inst.T, inst.seg_offsets, seg_slot_k,
                             pi.seg_rank * (seg_slot_k >= 0), inst.scale, main.cuda_stream))
        n_bytes = pi.fill(inst.miss_adapters, [layer], stream=side, sync=False)
        assert n_bytes > 0
        # iteration k+1 names the slots being filled: the apply must wait for them on the device
        B.check(B.lora_apply(pi.pool.handle, layer, p, xd.data_ptr(), y_k1.data_ptr(), inst.T, inst.seg_offsets, pi.seg_slot,
                             pi.seg_rank, inst.scale, main.cuda_stream))
        pi.pool.check_fault()
        side.synchronize()
        pi.pool.fills_done()

        _check_every_token(inst, p, y_k.float().cpu().numpy(), x, base, seg_adapter_k, "stress iteration k")
        _check_every_token(inst, p, y_k1.float().cpu().numpy(), x, base, inst.seg_adapter, "stress iteration k+1")
        rc, st = B.lora_cache_stats(pi.pool.handle)
        assert st.fills == (len(resident) + len(inst.miss_adapters)) * len(inst.projs)
        rc, info = B.lora_cache_slot_info(pi.pool.handle, int(pi.slot_of[inst.miss_adapters[0]]))
        assert info.state == B.LORA_SLOT_FILLING and info.parts_filled == len(inst.projs)  # 1 of 4 layer copies
    finally:
        pi.close()


@pytest.mark.parametrize("form", ["auto", "split"])
def test_large_decode_batch_in_both_gemv_forms(form):
    """2048 decode requests over 300 adapters, uniform popularity (so hardly any slot reaches the
    tile threshold): several thousand GEMV shrink items -- as one launch with the in-kernel hand-over
    (what the library picks up to 8192 items) and as two launches.  Sampled tokens against the oracle."""
    B, H = _mods()
    inst = wl.make_instance("big_decode", dtype="bf16", seed=3, projs=[wl.Projection("q", 4096, 4096, 0)], n_adapters=300,
                            rank_choices=[8, 16, 32, 64, 128], n_decode=2048, prompt_lens=[], zipf_alpha=None, n_base_only=16)
    pi = H.PooledInstance(inst, flags=B.LORA_CACHE_SPLIT_GEMV if form == "split" else 0)
    try:
        h = pi.pool.handle
        plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        rc, info = B.lora_plan_info(plan)
        assert rc == B.LORA_OK and 4096 < info.n_gemv_shrink_items <= 8192
        pi.pool.plan_destroy(plan)
        B.check(B.lora_cache_set_timing(h, 1))
        x, base = inst.x(0), inst.base_out(0)
        xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
        pi.apply(0, 0, xd, yd)
        pi.pool.check_fault()
        rc, tm = B.lora_cache_read_timing(h)
        if form == "split":
            assert tm["gemv_shrink"][1] == 1 and tm["gemv_expand"][1] == 1 and tm["gemv_fused"][1] == 0
        else:
            assert tm["gemv_shrink"][1] == 0 and tm["gemv_expand"][1] == 0 and tm["gemv_fused"][1] == 1
        _check_every_token(inst, 0, yd.float().cpu().numpy(), x, base, inst.seg_adapter, "large decode batch")
    finally:
        pi.close()


def test_plans_choose_the_tile_threshold_per_batch():
    """With the threshold left to the library: a pure decode batch has no tiles; a decode batch
    whose few hot adapters would make a handful of tiles stays all-GEMV (the tile launches would
    cost more than they save); a batch with prompts takes the lower threshold.  lora_index with the
    reported threshold reproduces the plan's list sizes."""
    B, H = _mods()
    for make, want in ((lambda: wl.decode(), B.LORA_MFMA_MIN_TOKENS), (lambda: wl.decode_heavy(), 0),
                       (lambda: wl.prefill(), B.LORA_MFMA_MIN_TOKENS_MIXED)):
        inst = make()
        pi = H.PooledInstance(inst, adapters=[])   # plans need bound slots only for the named adapters
        try:
            pi.fill(inst.used_adapters(), [0])
            plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
            rc, info = B.lora_plan_info(plan)
            assert rc == B.LORA_OK and info.T == inst.T and info.mfma_min_tokens == want, (inst.name, info.mfma_min_tokens)
            rc, w = B.lora_index(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, info.mfma_min_tokens, counts_only=True)
            assert w["n_tiles"] == info.n_tiles and (w["n_groups"] > 0) == (info.n_gemv_shrink_items > 0)
            if want == 0:
                rc, w16 = B.lora_index(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, 16, counts_only=True)
                assert w16["n_tiles"] > 0 and info.n_tiles == 0
            pi.pool.plan_destroy(plan)
        finally:
            pi.close()


def test_refill_waits_for_applies_that_still_read_the_slot():
    """Evict an adapter and load another one into its slot right behind an apply that reads it,
    without any host synchronisation: the first result must come from the old weights, the
    second from the new ones."""
    B, H = _mods()
    lens = [1] * 24 + [200, 300]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    mk = lambda seed, adapters: wl.Instance(
        name="refill", dtype="bf16", seed=seed, projs=[wl.Projection("p", 4096, 4096, 0)],
        ranks=np.asarray([64, 64], np.int32), adapter_ids=np.asarray([501, 502], np.int64), alpha=np.ones(2, np.float32),
        scale=2.0, seg_offsets=off, seg_adapter=np.asarray(adapters, np.int32))
    inst_a = mk(11, [0] * 26)   # everything on adapter 0 ...
    inst_b = mk(11, [1] * 26)   # ... then on adapter 1, which takes over the same slot
    pi = H.PooledInstance(inst_a, adapters=[0])
    try:
        h = pi.pool.handle
        slot = int(pi.slot_of[0])
        x, base = inst_a.x(0), inst_a.base_out(0)
        xd = H.to_device(x, pi.dtype)
        y1, y2 = H.to_device(base, pi.dtype), H.to_device(base, pi.dtype)
        A1, B1 = inst_b.adapter_weights(1, 0)
        ta = torch.from_numpy(A1).to(torch.bfloat16).pin_memory()
        tb = torch.from_numpy(B1).to(torch.bfloat16).pin_memory()
        side = torch.cuda.Stream()
        main = torch.cuda.current_stream()
        seg_slot = np.full(26, slot, np.int32)
        seg_rank = np.full(26, 64, np.int32)
        torch.cuda.synchronize()
        for _ in range(3):  # a few applies in flight
            B.check(B.lora_apply(h, 0, 0, xd.data_ptr(), y1.data_ptr(), inst_a.T, off, seg_slot, seg_rank, 0.0, main.cuda_stream))
        B.check(B.lora_apply(h, 0, 0, xd.data_ptr(), y1.data_ptr(), inst_a.T, off, seg_slot, seg_rank, 2.0, main.cuda_stream))
        B.check(B.lora_cache_release_slot(h, slot))
        B.check(B.lora_cache_fill_slot(h, slot, 502, 64, 1.0, 0, 0, ta.data_ptr(), tb.data_ptr(), side.cuda_stream))
        B.check(B.lora_apply(h, 0, 0, xd.data_ptr(), y2.data_ptr(), inst_a.T, off, seg_slot, seg_rank, 2.0, main.cuda_stream))
        pi.pool.check_fault()
        torch.cuda.synchronize()
        rows = np.arange(inst_a.T)
        for inst, yd, a_idx, what in ((inst_a, y1, 0, "before refill"), (inst_b, y2, 1, "after refill")):
            ads = {a_idx: (*inst.adapter_weights(a_idx, 0), 1.0)}
            ref = oracle.lora_apply(x, base, off, np.full(26, a_idx, np.int32), ads, 2.0)
            m = H.error_metrics(yd.float().cpu().numpy(), ref, base)
            for k, lim in TOL.items():
                assert m[k] <= lim, f"{what}: {k} = {m[k]:.3e} > {lim}"
        assert B.lora_cache_lookup(h, 501)[0] == B.LORA_E_NOTFOUND and B.lora_cache_lookup(h, 502)[1] == slot
    finally:
        pi.close()
