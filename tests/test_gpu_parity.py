"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on the same seeded
inputs.  Tolerances for bf16 storage with fp32 accumulation: relative Frobenius error <= 1e-2
and every element within 2e-2 * RMS(y).  Because the adapter delta is several times smaller
than base_out, the error is also measured against the delta alone: what is left of the
Frobenius error after allowing for the single bf16 rounding of the stored output (at most 2^-9
of |y|) must stay within 2e-2 of |y - base_out|_F, so a kernel that does nothing, or drops a
segment, fails.  fp32 instances: 1e-5 / 1e-4 / 1e-4 with 2^-24.  Integer-valued inputs must match
bit for bit."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = {"bf16": dict(rel_fro=1e-2, max_abs_over_rms=2e-2, delta_rel_fro=2e-2),
       "f32": dict(rel_fro=1e-5, max_abs_over_rms=1e-4, delta_rel_fro=1e-4)}


def _mods():
    from paper_2411_17741_amd import binding as B
    from paper_2411_17741_amd import harness as H
    return B, H


def _oracle_adapters(inst, p, which):
    return {int(a): (*inst.adapter_weights(int(a), p), float(inst.alpha[a])) for a in which}




def _check(m, dtype, what):
    for k, lim in TOL[dtype].items():
        assert m[k] <= lim, f"{what}: {k} = {m[k]:.3e} > {lim}"


def _full_parity(inst, p=0, layer=0, pi=None, mfma_min_tokens=0, flags=0):
    B, H = _mods()
    own = pi is None
    if own:
        pi = H.PooledInstance(inst, mfma_min_tokens=mfma_min_tokens, flags=flags)
    try:
        x, base = inst.x(p), inst.base_out(p)
        xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
        pi.apply(layer, p, xd, yd)
        pi.pool.check_fault()
        y = yd.float().cpu().numpy()
        ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _oracle_adapters(inst, p, inst.used_adapters()), inst.scale)
        m = H.error_metrics(y, ref, base, inst.dtype)
        _check(m, inst.dtype, f"{inst.name} proj {p}")
        ta = inst.token_adapter()
        assert np.array_equal(y[ta < 0], base[ta < 0]), "tokens without adapter must be untouched"
        return m
    finally:
        if own:
            pi.close()


def test_tiny_fp32():
    B, H = _mods()
    inst = wl.tiny()
    pi = H.PooledInstance(inst)
    x = inst.x(0)
    base = (x.astype(np.float64) @ inst.base_weight(0).astype(np.float64)).astype(np.float32)
    xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
    pi.apply(0, 0, xd, yd)
    torch.cuda.synchronize()
    ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _oracle_adapters(inst, 0, inst.used_adapters()), inst.scale)
    _check(H.error_metrics(yd.cpu().numpy(), ref, base, "f32"), "f32", "tiny")
    pi.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("seed", [0, 1])
def test_small_mixed_all_paths(dtype, seed):
    """With the tile threshold fixed at 16 (tiles, gathered tiles and GEMV groups all occur) and
    left to the library (which keeps a batch this small all-GEMV)."""
    inst = wl.small_mixed(seed=seed, dtype=dtype)
    B, H = _mods()
    for m0 in (B.LORA_MFMA_MIN_TOKENS, 0):
        pi = H.PooledInstance(inst, mfma_min_tokens=m0)
        try:
            for p in range(len(inst.projs)):
                _full_parity(inst, p, pi=pi)
        finally:
            pi.close()


def test_decode_config():
    _full_parity(wl.decode())


def test_gemv_as_one_launch_or_two_gives_the_same_results():
    """The GEMV phases run as one launch with an in-kernel hand-over or as two launches; by
    default the library picks by size.  Force each form."""
    B, H = _mods()
    for flags in (B.LORA_CACHE_FUSED_GEMV, B.LORA_CACHE_SPLIT_GEMV):
        _full_parity(wl.decode(), flags=flags)
        _full_parity(wl.small_mixed(seed=4), p=1, flags=flags)
        _full_parity(wl.small_mixed(seed=4, dtype="f32"), p=0, flags=flags)


def test_fused_gemv_repeated_applies_of_one_plan():
    """The fused launch tells this apply's intermediate from older ones by its number: apply one
    plan many times (as the layers of an iteration do) with activations that change from apply to
    apply, and check the last result."""
    B, H = _mods()
    inst = wl.decode(seed=3)
    pi = H.PooledInstance(inst, flags=B.LORA_CACHE_FUSED_GEMV)
    try:
        x, base = inst.x(0), inst.base_out(0)
        xd = H.to_device(x, pi.dtype)
        others = [H.to_device(wl.bf16_round(x * f), pi.dtype) for f in (-1.0, 0.5, 3.0)]
        plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        for rep in range(40):
            yd = H.to_device(base, pi.dtype)
            pi.pool.apply_plan(plan, 0, 0, xd if rep == 39 else others[rep % 3], yd, inst.scale)
        pi.pool.check_fault()
        ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _oracle_adapters(inst, 0, inst.used_adapters()), inst.scale)
        _check(H.error_metrics(yd.float().cpu().numpy(), ref, base), "bf16", "40th apply of one plan")
    finally:
        pi.close()


def test_prefill_config():
    _full_parity(wl.prefill())


@pytest.mark.parametrize("m0", [1, 8, 64])
def test_threshold_between_paths_does_not_change_results(m0):
    _full_parity(wl.small_mixed(seed=2), p=0, mfma_min_tokens=m0)
    _full_parity(wl.small_mixed(seed=2), p=1, mfma_min_tokens=m0)


def test_integer_inputs_are_bit_exact():
    """Small integers: every product and partial sum is exact in fp32 and the result is a
    bf16 number, so any difference is an indexing error, not rounding."""
    B, H = _mods()
    rng = np.random.default_rng(0)
    ii = wl.small_mixed(seed=5)
    wcache = {}

    def adapter_weights(a, p):
        if (a, p) not in wcache:
            pr, r = ii.projs[p], int(ii.ranks[a])
            g = np.random.default_rng(1000 * a + p)
            A = g.integers(-1, 2, size=(pr.h_in, r)).astype(np.float32) * (g.random((pr.h_in, r)) < 0.02)
            Bm = g.integers(-1, 2, size=(r, pr.h_out)).astype(np.float32) * (g.random((r, pr.h_out)) < 0.1)
            wcache[(a, p)] = (A.astype(np.float32), Bm.astype(np.float32))
        return wcache[(a, p)]

    ii.adapter_weights = adapter_weights
    ii.scale = 1.0
    pi = H.PooledInstance(ii, mfma_min_tokens=16)  # tiles, gathered tiles and GEMV groups
    try:
        for p in range(len(ii.projs)):
            x = rng.integers(-2, 3, size=(ii.T, ii.projs[p].h_in)).astype(np.float32)
            base = rng.integers(-8, 9, size=(ii.T, ii.projs[p].h_out)).astype(np.float32)
            xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
            pi.apply(0, p, xd, yd)
            torch.cuda.synchronize()
            ref = oracle.lora_apply(x, base, ii.seg_offsets, ii.seg_adapter, _oracle_adapters(ii, p, ii.used_adapters()), ii.scale)
            y = yd.float().cpu().numpy().astype(np.float64)
            assert np.abs(ref).max() < 256 and np.array_equal(ref, np.round(ref))
            assert np.abs(ref - base).max() > 0
            assert np.array_equal(y, ref)
    finally:
        pi.close()


def test_zero_B_leaves_base_bit_identical():
    B, H = _mods()
    inst = wl.small_mixed(seed=3)
    orig = inst.adapter_weights
    inst.adapter_weights = lambda a, p: (orig(a, p)[0], np.zeros_like(orig(a, p)[1]))
    pi = H.PooledInstance(inst, mfma_min_tokens=16)
    try:
        x, base = inst.x(0), inst.base_out(0)
        xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
        pi.apply(0, 0, xd, yd)
        torch.cuda.synchronize()
        assert np.array_equal(yd.float().cpu().numpy(), base)
    finally:
        pi.close()


def _custom_instance(lens, adapters, ranks, h_in=256, h_out=320, dtype="bf16", seed=0):
    """Segments of the given lengths, segment g -> pool adapter adapters[g] (-1 = none)."""
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return wl.Instance(
        name="custom", dtype=dtype, seed=seed, projs=[wl.Projection("p", h_in, h_out, 0)],
        ranks=np.asarray(ranks, np.int32), adapter_ids=np.arange(len(ranks), dtype=np.int64) + 1,
        alpha=np.linspace(0.5, 1.5, len(ranks)).astype(np.float32), scale=2.0,
        seg_offsets=off, seg_adapter=np.asarray(adapters, np.int32),
    )


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_lengths_and_odd_ranks(dtype):
    """Tile boundaries (15/16/17, 63/64/65, 128/129), empty segments, base-only segments,
    ranks that are not multiples of 8 or 16, per-adapter alpha."""
    lens = [15, 16, 17, 0, 63, 64, 65, 1, 129, 128, 2, 0, 1]
    ranks = [1, 4, 8, 12, 16, 24, 40, 100, 128, 7]
    adapters = [0, 1, 2, 3, 4, 5, 6, -1, 7, 8, 9, 2, 9]
    for m0 in (16, 8, 0):  # fixed thresholds (the tile path at every boundary), and the library's choice
        _full_parity(_custom_instance(lens, adapters, ranks, dtype=dtype), mfma_min_tokens=m0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("form", ["fused", "split"])
def test_gemv_path_every_rank_shape_and_batch_size(dtype, form):
    """No tiles at all: every adapter has 1..7 tokens (token batches of 1, 2, 3, 4 and 4+k), ranks
    cover every body of the GEMV kernels (vector-ALU bodies below 32 stored ranks and for fp32,
    matrix-core bodies with 1, 2 (both unit widths), 3 and 4 k steps, ranks that are no multiple
    of 8), rows end in a ragged run of chunks, and the last column unit of a super-chunk is cut."""
    B, H = _mods()
    ranks = [1, 4, 8, 12, 16, 24, 32, 37, 40, 48, 56, 64, 72, 96, 100, 128]
    n_tok = [1, 2, 3, 4, 5, 6, 7, 1, 2, 3, 4, 5, 6, 7, 3, 5]
    lens, adapters = [], []
    for rnd in range(7):  # interleave the requests as a decode batch would
        for a, n in enumerate(n_tok):
            if rnd < n:
                lens.append(1)
                adapters.append(a)
    inst = _custom_instance(lens, adapters, ranks, h_in=4160, h_out=1216, dtype=dtype, seed=5)
    flags = {"fused": B.LORA_CACHE_FUSED_GEMV, "split": B.LORA_CACHE_SPLIT_GEMV}[form]
    _full_parity(inst, flags=flags)


@pytest.mark.parametrize("form", ["fused", "split"])
def test_gemv_path_long_rows(form):
    """Rows longer than one pass of a 16-wavefront block (h_in > 16384) and the 13B-shaped
    13824 (14 wavefronts per item in the stand-alone shrink, several passes of 4 in the fused)."""
    B, H = _mods()
    flags = {"fused": B.LORA_CACHE_FUSED_GEMV, "split": B.LORA_CACHE_SPLIT_GEMV}[form]
    for h_in in (13824, 16448):
        inst = _custom_instance([1, 1, 1, 2, 1], [0, 1, 0, 2, 1], [16, 64, 128], h_in=h_in, h_out=256, seed=h_in)
        _full_parity(inst, flags=flags)


def test_empty_and_adapterless_batches():
    B, H = _mods()
    inst = _custom_instance([3, 2], [-1, -1], [8])
    pi = H.PooledInstance(inst, adapters=[0])
    try:
        x, base = inst.x(0), inst.base_out(0)
        xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
        pi.apply(0, 0, xd, yd)
        torch.cuda.synchronize()
        assert np.array_equal(yd.float().cpu().numpy(), base)
        # T = 0
        assert B.lora_apply(pi.pool.handle, 0, 0, 0, 0, 0, [0], [], [], 1.0) == B.LORA_OK
        assert B.lora_apply(pi.pool.handle, 0, 0, xd.data_ptr(), yd.data_ptr(), 0, [0, 0], [0], [8], 1.0) == B.LORA_OK
        torch.cuda.synchronize()
        assert np.array_equal(yd.float().cpu().numpy(), base)
    finally:
        pi.close()


def test_single_token_max_rank_wide_projection():
    inst = _custom_instance([1], [0], [128], h_in=11008, h_out=4096)
    _full_parity(inst)
    inst = _custom_instance([1, 70], [0, 1], [128, 128], h_in=4096, h_out=11008, seed=1)
    _full_parity(inst, mfma_min_tokens=16)
    _full_parity(inst)


def test_apply_errors():
    B, H = _mods()
    inst = _custom_instance([4, 4], [0, 1], [8, 16])
    pi = H.PooledInstance(inst, adapters=[0])  # adapter 1 is not resident
    try:
        x, base = inst.x(0), inst.base_out(0)
        xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
        h = pi.pool.handle
        args = (inst.seg_offsets, pi.seg_slot, pi.seg_rank, 2.0)
        assert B.lora_apply(h, 0, 0, xd.data_ptr(), yd.data_ptr(), inst.T, *args) == B.LORA_E_STATE
        pi.fill([1], [0])
        assert B.lora_apply(h, 1, 0, xd.data_ptr(), yd.data_ptr(), inst.T, *args) == B.LORA_E_INVAL  # no such layer
        assert B.lora_apply(h, 0, 0, 0, yd.data_ptr(), inst.T, *args) == B.LORA_E_INVAL
        assert B.lora_apply(h, 0, 0, xd.data_ptr() + 2, yd.data_ptr(), inst.T, *args) == B.LORA_E_INVAL  # misaligned
        torch.cuda.synchronize()
        assert np.array_equal(yd.float().cpu().numpy(), base), "failed calls must not touch base_out"
        assert B.lora_apply(h, 0, 0, xd.data_ptr(), yd.data_ptr(), inst.T, *args) == B.LORA_OK
        torch.cuda.synchronize()
        # evicted slot: plan made before the eviction is refused
        rc, plan = B.lora_plan_create(h, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        assert rc == B.LORA_OK
        assert B.lora_cache_release_slot(h, int(pi.slot_of[1])) == B.LORA_OK
        assert B.lora_apply_plan(h, plan, 0, 0, xd.data_ptr(), yd.data_ptr(), 2.0) == B.LORA_E_STATE
    finally:
        pi.close()


def test_fill_paths_give_the_same_slabs():
    """A part reaches its slot through a staging copy (from pinned or from pageable host memory)
    or, with LORA_CACHE_DIRECT_FILL, straight from pinned host memory read by the repack kernel.
    Same bytes in the pool every way; more parts than staging buffers in flight."""
    B, H = _mods()
    inst = _custom_instance([3, 20, 1, 70, 2, 5], [0, 1, 2, 3, 4, 5], [7, 16, 64, 128, 1, 100], h_in=320, h_out=448, seed=21)
    outs = []
    for pinned, flags, whole in ((True, 0, False), (False, 0, False), (True, B.LORA_CACHE_DIRECT_FILL, False),
                                 (True, B.LORA_CACHE_DIRECT_FILL, True), (True, 0, True), (False, B.LORA_CACHE_DIRECT_FILL, True)):
        pi = H.PooledInstance(inst, adapters=[], mfma_min_tokens=16, flags=flags)
        try:
            keep = []
            for a in range(len(inst.ranks)):
                A, Bm = inst.adapter_weights(a, 0)
                ta, tb = torch.from_numpy(A).to(torch.bfloat16), torch.from_numpy(Bm).to(torch.bfloat16)
                if pinned:
                    ta, tb = ta.pin_memory(), tb.pin_memory()
                assert ta.is_pinned() == pinned
                keep += [ta, tb]
                if whole:  # the adapter's parts in one call (here it has one)
                    B.check(B.lora_cache_fill_slot_parts(pi.pool.handle, int(pi.slot_of[a]), int(inst.adapter_ids[a]), int(inst.ranks[a]),
                                                         float(inst.alpha[a]), B.make_fill_parts([(0, 0, ta.data_ptr(), tb.data_ptr())]),
                                                         torch.cuda.current_stream().cuda_stream))
                    continue
                pi.pool.fill(int(pi.slot_of[a]), int(inst.adapter_ids[a]), int(inst.ranks[a]), float(inst.alpha[a]), 0, 0, ta, tb, pin=False)
            torch.cuda.synchronize()
            pi.pool.fills_done()
            x, base = inst.x(0), inst.base_out(0)
            xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
            pi.apply(0, 0, xd, yd)
            pi.pool.check_fault()
            outs.append(yd.float().cpu().numpy())
        finally:
            pi.close()
    assert all(np.array_equal(outs[0], o) for o in outs[1:])
    ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _oracle_adapters(inst, 0, inst.used_adapters()), inst.scale)
    _check(H.error_metrics(outs[0], ref, base), "bf16", "fill paths")


def test_whole_adapter_fill_in_one_call():
    """All (layer, projection) parts of an adapter handed over in one lora_cache_fill_slot_parts call, read
    from pinned host memory by one kernel per 32 parts: 21 layers x 2 projections of different shapes (42
    parts, so two launches).  Every layer copy must then give the results of part-by-part fills."""
    B, H = _mods()
    inst = wl.small_mixed(seed=13)
    n_layers = 21
    ref_pi = H.PooledInstance(inst, n_layers=1)
    pi = H.PooledInstance(inst, n_layers=n_layers, adapters=[], flags=B.LORA_CACHE_DIRECT_FILL)
    try:
        keep = []
        for a in inst.used_adapters():
            a = int(a)
            host = []
            for p in range(len(inst.projs)):
                A, Bm = inst.adapter_weights(a, p)
                host.append((torch.from_numpy(A).to(torch.bfloat16).pin_memory(), torch.from_numpy(Bm).to(torch.bfloat16).pin_memory()))
            keep += host
            parts = B.make_fill_parts([(l, p, host[p][0].data_ptr(), host[p][1].data_ptr()) for l in range(n_layers) for p in range(len(inst.projs))])
            B.check(B.lora_cache_fill_slot_parts(pi.pool.handle, int(pi.slot_of[a]), int(inst.adapter_ids[a]), int(inst.ranks[a]),
                                                 float(inst.alpha[a]), parts, torch.cuda.current_stream().cuda_stream))
            rc, info = B.lora_cache_slot_info(pi.pool.handle, int(pi.slot_of[a]))
            assert info.parts_filled == n_layers * len(inst.projs)
        torch.cuda.synchronize()
        for p in range(len(inst.projs)):
            x, base = inst.x(p), inst.base_out(p)
            xd, want = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
            ref_pi.apply(0, p, xd, want)
            ref_pi.pool.check_fault()
            for layer in (0, 7, n_layers - 1):
                yd = H.to_device(base, pi.dtype)
                pi.apply(layer, p, xd, yd)
                pi.pool.check_fault()
                assert torch.equal(yd, want), f"projection {p}, layer copy {layer}"
    finally:
        pi.close()
        ref_pi.close()


def test_multi_apply_groups_projections_that_share_their_input():
    """q, k, v read one x: the list form runs one tile-shrink launch for all of them, then their
    expands.  Results must be those of one apply after the other -- also when one of the outputs
    is the shared input itself (then nothing may be reordered) -- for both GEMV launch forms, with the
    GEMV launch beside the tile kernels on the cache's side stream (the default) and behind them on the
    caller's."""
    B, H = _mods()
    base_inst = wl.small_mixed(seed=9)
    projs = [wl.Projection("q", 512, 512, 0), wl.Projection("k", 512, 256, 0), wl.Projection("v", 512, 384, 0),
             wl.Projection("o", 384, 512, 1), wl.Projection("g", 512, 640, 2), wl.Projection("u", 512, 640, 2),
             wl.Projection("w", 2048, 256, 3), wl.Projection("z", 2048, 320, 3)]
    inst = wl.Instance(name="qkv", dtype="bf16", seed=9, projs=projs, ranks=base_inst.ranks, adapter_ids=base_inst.adapter_ids,
                       alpha=base_inst.alpha, scale=base_inst.scale, seg_offsets=base_inst.seg_offsets,
                       seg_adapter=base_inst.seg_adapter)
    for flags in (B.LORA_CACHE_FUSED_GEMV, B.LORA_CACHE_SPLIT_GEMV, B.LORA_CACHE_FUSED_GEMV | B.LORA_CACHE_NO_OVERLAP):
        pi = H.PooledInstance(inst, mfma_min_tokens=16, flags=flags)
        try:
            plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
            sh = torch.cuda.current_stream().cuda_stream
            xs = {pr.x_key: H.to_device(inst.x(p), pi.dtype) for p, pr in enumerate(projs)}
            ys = [H.to_device(inst.base_out(p), pi.dtype) for p in range(len(projs))]
            descs = B.make_descs([(0, p, xs[pr.x_key].data_ptr(), ys[p].data_ptr()) for p, pr in enumerate(projs)])
            B.check(B.lora_apply_plan_multi(pi.pool.handle, plan, descs, inst.scale, sh))
            pi.pool.check_fault()
            ads = lambda p: _oracle_adapters(inst, p, inst.used_adapters())
            for p in range(len(projs)):
                ref = oracle.lora_apply(inst.x(p), inst.base_out(p), inst.seg_offsets, inst.seg_adapter, ads(p), inst.scale)
                _check(H.error_metrics(ys[p].float().cpu().numpy(), ref, inst.base_out(p)), "bf16", f"grouped proj {p}")

            # q writes into the shared input: k must then see the updated x, as in sequential order
            x0 = inst.x(0)
            xq = H.to_device(x0, pi.dtype)
            yk = H.to_device(inst.base_out(1), pi.dtype)
            descs = B.make_descs([(0, 0, xq.data_ptr(), xq.data_ptr()), (0, 1, xq.data_ptr(), yk.data_ptr())])
            B.check(B.lora_apply_plan_multi(pi.pool.handle, plan, descs, inst.scale, sh))
            pi.pool.check_fault()
            x1 = wl.bf16_round(oracle.lora_apply(x0, x0, inst.seg_offsets, inst.seg_adapter, ads(0), inst.scale).astype(np.float32))
            got_x1 = xq.float().cpu().numpy()
            _check(H.error_metrics(got_x1, x1, x0), "bf16", "in-place q")
            ref_k = oracle.lora_apply(got_x1, inst.base_out(1), inst.seg_offsets, inst.seg_adapter, ads(1), inst.scale)
            _check(H.error_metrics(yk.float().cpu().numpy(), ref_k, inst.base_out(1)), "bf16", "k after in-place q")
            pi.pool.plan_destroy(plan)
        finally:
            pi.close()


def test_applies_captured_in_a_graph_replay_correctly():
    """An apply of a plan captured into a HIP graph (fencing off, as the header asks) and replayed
    several times, with the activations changed by eager work between the replays: every replay
    must give what the eager call gives.  (Under capture the GEMV part always takes the two-launch
    form: the one-launch form numbers its launches, and a graph would freeze the number.)"""
    B, H = _mods()
    for inst, m0 in ((wl.decode(seed=2), 0), (wl.small_mixed(seed=3), 16)):
        pi = H.PooledInstance(inst, mfma_min_tokens=m0, flags=B.LORA_CACHE_FUSED_GEMV)
        try:
            h = pi.pool.handle
            x, base = inst.x(0), inst.base_out(0)
            xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
            base_d = yd.clone()
            plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
            pi.pool.apply_plan(plan, 0, 0, xd, yd, inst.scale)  # eager once: fills are seen as done, kernels loaded
            torch.cuda.synchronize()
            B.check(B.lora_cache_set_fencing(h, 0))
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, capture_error_mode="thread_local"):
                pi.pool.apply_plan(plan, 0, 0, xd, yd, inst.scale)
            B.check(B.lora_cache_set_fencing(h, 1))
            for rep, f in enumerate((1.0, -0.5, 2.0, 1.0)):
                xd.copy_(H.to_device(wl.bf16_round(x * f), pi.dtype))   # eager work between the replays
                yd.copy_(base_d)
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                got = yd.float().cpu().numpy()
                y_eager = base_d.clone()
                pi.pool.apply_plan(plan, 0, 0, xd, y_eager, inst.scale)
                pi.pool.check_fault()
                assert np.array_equal(got, y_eager.float().cpu().numpy()), f"{inst.name}: replay {rep} differs from the eager apply"
            ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _oracle_adapters(inst, 0, inst.used_adapters()), inst.scale)
            _check(H.error_metrics(got, ref, base), "bf16", "last replay")
            pi.pool.plan_destroy(plan)
        finally:
            pi.close()


def test_plan_reuse_over_projections_and_layers():
    """One plan per iteration, applied to every projection of every layer copy."""
    B, H = _mods()
    inst = wl.small_mixed(seed=7)
    pi = H.PooledInstance(inst, n_layers=2, mfma_min_tokens=16)
    try:
        plan = pi.pool.plan(inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank)
        for layer in range(2):
            for p in range(len(inst.projs)):
                x, base = inst.x(p), inst.base_out(p)
                xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
                pi.pool.apply_plan(plan, layer, p, xd, yd, inst.scale)
                torch.cuda.synchronize()
                ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _oracle_adapters(inst, p, inst.used_adapters()), inst.scale)
                _check(H.error_metrics(yd.float().cpu().numpy(), ref, base), "bf16", f"layer {layer} proj {p}")
        pi.pool.plan_destroy(plan)
        rc, info = B.lora_cache_slot_info(pi.pool.handle, int(pi.seg_slot[pi.seg_slot >= 0][0]))
        assert info.use_count == 4 and info.last_used > 0 and info.state == B.LORA_SLOT_READY
    finally:
        pi.close()


def test_plan_made_on_one_stream_and_applied_on_another():
    """The upload of a plan's work lists is enqueued on the stream given to lora_plan_create; an
    apply on a different stream must wait for it on the device.  The creating stream is kept busy
    (a long chain of copies enqueued before the plan) so that an apply that did not wait would read
    the lists of the plan that held the buffer before -- the same batch with adapters of equal rank
    swapped, i.e. lists of the same sizes that name other slots: wrong results, never a wild address."""
    B, H = _mods()
    inst = wl.small_mixed(seed=5)
    pi = H.PooledInstance(inst, mfma_min_tokens=16, n_plans=1)
    try:
        h = pi.pool.handle
        s_plan, s_apply = torch.cuda.Stream(), torch.cuda.Stream()
        x, base = inst.x(0), inst.base_out(0)
        xd, yd = H.to_device(x, pi.dtype), H.to_device(base, pi.dtype)
        # the buffer first holds the lists of the batch with pairs of equal-rank adapters swapped
        used = [int(a) for a in inst.used_adapters()]
        swap = {a: a for a in used}
        by_rank = {}
        for a in used:
            by_rank.setdefault(int(inst.ranks[a]), []).append(a)
        for group in by_rank.values():
            for a, b in zip(group[0::2], group[1::2]):
                swap[a], swap[b] = b, a
        assert any(k != v for k, v in swap.items())
        stale_slot = np.array([pi.slot_of[swap[int(a)]] if a >= 0 else -1 for a in inst.seg_adapter], np.int32)
        rc, stale = B.lora_plan_create(h, inst.T, inst.seg_offsets, stale_slot, pi.seg_rank, s_plan.cuda_stream)
        B.check(rc)
        rc, stale_info = B.lora_plan_info(stale)
        B.check(B.lora_plan_destroy(h, stale))
        torch.cuda.synchronize()
        big = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
        big2 = torch.empty_like(big)
        with torch.cuda.stream(s_plan):
            for _ in range(40):
                big2.copy_(big)
        rc, plan = B.lora_plan_create(h, inst.T, inst.seg_offsets, pi.seg_slot, pi.seg_rank, s_plan.cuda_stream)
        B.check(rc)
        rc, info = B.lora_plan_info(plan)
        assert [getattr(info, f) for f, _ in info._fields_] == [getattr(stale_info, f) for f, _ in stale_info._fields_]  # same list sizes
        B.check(B.lora_apply_plan(h, plan, 0, 0, xd.data_ptr(), yd.data_ptr(), inst.scale, s_apply.cuda_stream))
        s_apply.synchronize()
        pi.pool.check_fault(s_apply)
        ref = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _oracle_adapters(inst, 0, inst.used_adapters()), inst.scale)
        _check(H.error_metrics(yd.float().cpu().numpy(), ref, base), "bf16", "apply on another stream")
        torch.cuda.synchronize()
        B.check(B.lora_plan_destroy(h, plan))
    finally:
        pi.close()
