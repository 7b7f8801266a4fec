"""GPU parity at the full sizes of the larger configurations, in the launch configuration the
benchmark times (same batch, shapes, pool and plan flow).  The oracle computes sampled tokens
one by one (every sampled token as its own one-token segment): all tile boundaries of some
prompts, tokens of hot and cold adapters, and a random spread.  Also here: fills on a side
stream overlapped with applies (a miss of the next iteration is loaded while the current one
runs) and a refill of a slot that an enqueued apply still reads."""
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


def _sample_tokens(inst, n_random=96, seed=0):
    rng = np.random.default_rng(seed)
    off = inst.seg_offsets
    picks = set(int(t) for t in rng.integers(0, inst.T, size=n_random))
    lens = np.diff(off)
    for g in np.argsort(-lens)[:3]:  # three longest prompts: first/last token and tile edges
        for t in (off[g], off[g] + 63, off[g] + 64, off[g] + 65, off[g + 1] - 65, off[g + 1] - 64, off[g + 1] - 1):
            if off[g] <= t < off[g + 1]:
                picks.add(int(t))
    ta = inst.token_adapter()
    decode_tokens = np.flatnonzero(np.repeat(lens == 1, lens))
    for t in decode_tokens[:48]:
        picks.add(int(t))
    u, c = np.unique(ta[decode_tokens][ta[decode_tokens] >= 0], return_counts=True)
    if len(u):
        hot = u[np.argmax(c)]  # every decode token of the most popular adapter
        for t in decode_tokens[ta[decode_tokens] == hot]:
            picks.add(int(t))
    return np.array(sorted(picks), np.int64)


def _check_sampled(inst, p, rows, y_rows, x_rows, base_rows, seg_adapter_rows, what):
    B, H = _mods()
    ads = {int(a): (*inst.adapter_weights(int(a), p), float(inst.alpha[a])) for a in np.unique(seg_adapter_rows[seg_adapter_rows >= 0])}
    ref = oracle.lora_apply(x_rows, base_rows, np.arange(len(rows) + 1, dtype=np.int32), seg_adapter_rows, ads, inst.scale)
    m = H.error_metrics(y_rows, ref, base_rows)
    for k, lim in TOL.items():
        assert m[k] <= lim, f"{what}: {k} = {m[k]:.3e} > {lim}"
    none = seg_adapter_rows < 0
    assert np.array_equal(y_rows[none], base_rows[none])
    return m


def _run_full(inst, rows, n_layers=1, layer=0):
    """Plan once, apply every projection (the benchmark's flow), compare sampled rows."""
    B, H = _mods()
    pi = H.PooledInstance(inst, n_layers=n_layers, fill_layers=[layer])
    try:
        plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        ta = inst.token_adapter()[rows]
        xs = {}
        for p, pr in enumerate(inst.projs):
            if pr.x_key not in xs:
                xs[pr.x_key] = (inst.x(p), None)
                xs[pr.x_key] = (xs[pr.x_key][0], H.to_device(xs[pr.x_key][0], pi.dtype))
            x, xd = xs[pr.x_key]
            base = inst.base_out(p)
            yd = H.to_device(base, pi.dtype)
            pi.pool.apply_plan(plan, layer, p, xd, yd, inst.scale)
            pi.pool.check_fault()
            y_rows = yd[torch.from_numpy(rows).to(yd.device)].float().cpu().numpy()
            _check_sampled(inst, p, rows, y_rows, x[rows], base[rows], ta, f"{inst.name} proj {pr.name}")
            del yd, base
        pi.pool.plan_destroy(plan)
    finally:
        pi.close()


def test_mixed_config_full_size_sampled():
    inst = wl.mixed()
    _run_full(inst, _sample_tokens(inst))


def test_prefill_config_full_size_sampled_other_seed():
    inst = wl.prefill(seed=1)
    _run_full(inst, _sample_tokens(inst, seed=1))


@pytest.mark.parametrize("n_adapters,n_decode", [(10, 64), (200, 64), (150, 512)])
def test_decode_with_the_papers_adapter_population(n_adapters, n_decode):
    """The adapter population of the paper's own workload (N_a / 5 adapters of every rank, rank
    uniform, power law within the rank) at both ends of its sweep over N_a: every token checked."""
    inst = wl.decode_paper(n_adapters=n_adapters, n_decode=n_decode)
    assert np.array_equal(np.bincount(inst.ranks)[[8, 16, 32, 64, 128]], [n_adapters // 5] * 5)
    _run_full(inst, np.arange(inst.T, dtype=np.int64))


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
        rows = _sample_tokens(inst, n_random=64)
        ta_full = inst.token_adapter()
        miss_mask_seg = np.isin(inst.seg_adapter, inst.miss_adapters)
        seg_slot_k = np.where(miss_mask_seg, -1, pi.seg_slot).astype(np.int32)   # iteration k: misses deferred
        seg_adapter_k = np.where(miss_mask_seg, -1, inst.seg_adapter).astype(np.int32)
        ta_k = np.repeat(seg_adapter_k, np.diff(inst.seg_offsets))
        # make sure the sample sees requests that miss
        miss_tokens = np.flatnonzero(np.isin(ta_full, inst.miss_adapters))
        rows = np.unique(np.concatenate([rows, miss_tokens[:: max(1, len(miss_tokens) // 24)]]))

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

        idx = torch.from_numpy(rows).to(y_k.device)
        _check_sampled(inst, p, rows, y_k[idx].float().cpu().numpy(), x[rows], base[rows], ta_k[rows], "stress iteration k")
        _check_sampled(inst, p, rows, y_k1[idx].float().cpu().numpy(), x[rows], base[rows], ta_full[rows], "stress iteration k+1")
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
        rc, w = B.lora_index(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, B.LORA_MFMA_MIN_TOKENS, counts_only=True)
        assert 4096 < w["n_gs_items"] <= 8192
        h = pi.pool.handle
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
        rows = _sample_tokens(inst, n_random=160, seed=3)
        y_rows = yd[torch.from_numpy(rows).to(yd.device)].float().cpu().numpy()
        _check_sampled(inst, 0, rows, y_rows, x[rows], base[rows], inst.token_adapter()[rows], "large decode batch")
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
            assert (w["n_tiles"], w["n_gs_items"], w["n_ge_items"]) == (info.n_tiles, info.n_gemv_shrink_items, info.n_gemv_expand_items)
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
