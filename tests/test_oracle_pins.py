"""Pins for the CPU oracle: things the mathematics fixes, computed without the oracle.

The paper (section 3.1) names the steps -- base product, two adapter products, one
addition -- but prints no worked example, so nothing here is a paper-printed value.
Each pin is chosen so that a dropped term, a wrong sign, a transposed operand, a
wrong segment/adapter index or a mis-applied scale fails at least one of them.
"""
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _adapters(inst, p=0):
    return {int(a): (*inst.adapter_weights(int(a), p), float(inst.alpha[a])) for a in inst.used_adapters()}


def _parse_golden(path):
    d, ads, cur = {}, {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        if k == "adapter":
            cur = int(v[0])
            ads[cur] = {"rank": int(v[2]), "alpha": float(v[4])}
        elif k in ("A", "B"):
            ads[cur][k] = np.array([float(s) for s in v])
        else:
            d[k] = [float(s) for s in v]
    return d, ads


def test_handworked_example():
    d, ads = _parse_golden(os.path.join(GOLDEN, "handworked_lora_apply.txt"))
    h_in, h_out = int(d["h_in"][0]), int(d["h_out"][0])
    adapters = {i: (a["A"].reshape(h_in, a["rank"]), a["B"].reshape(a["rank"], h_out), a["alpha"]) for i, a in ads.items()}
    x = np.array(d["x"]).reshape(-1, h_in)
    base = np.array(d["base"]).reshape(-1, h_out)
    y = oracle.lora_apply(x, base, np.array(d["seg_offsets"], np.int32), np.array(d["seg_adapter"], np.int32), adapters, d["scale"][0])
    assert np.array_equal(y, np.array(d["y"]).reshape(-1, h_out))


def test_tiny_config_vs_dense_bruteforce():
    """Per token, form W_eff = W + s.A_i.B_i densely and multiply: the textbook merged-weights
    form of LoRA (section 2: the straightforward way is to merge adapter and base model)."""
    inst = wl.tiny()
    x = inst.x(0).astype(np.float64)
    W = inst.base_weight(0).astype(np.float64)
    base = x @ W
    ads = _adapters(inst)
    y = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, ads, inst.scale)
    ta = inst.token_adapter()
    for t in range(inst.T):
        A, B, al = ads[int(ta[t])]
        W_eff = W + inst.scale * al * (A.astype(np.float64) @ B.astype(np.float64))
        ref = x[t] @ W_eff
        assert np.max(np.abs(y[t] - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # the delta is not negligible, so the check above does see it
    assert np.linalg.norm(y - base) > 1e-3 * np.linalg.norm(base)


def test_single_adapter_batch_is_one_gemm():
    rng = np.random.default_rng(1)
    T, h_in, h_out, r = 37, 48, 40, 5
    x, base = rng.standard_normal((T, h_in)), rng.standard_normal((T, h_out))
    A, B = rng.standard_normal((h_in, r)), rng.standard_normal((r, h_out))
    y = oracle.lora_apply(x, base, [0, 10, 10, 37], [3, 3, 3], {3: (A, B, 0.25)}, 3.0)
    ref = base + 0.75 * (x @ A) @ B
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_alpha_and_scale_multiply():
    rng = np.random.default_rng(2)
    x, base = rng.standard_normal((4, 8)), rng.standard_normal((4, 6))
    A, B = rng.standard_normal((8, 2)), rng.standard_normal((2, 6))
    y1 = oracle.lora_apply(x, base, [0, 4], [0], {0: (A, B, 0.5)}, 4.0)
    y2 = oracle.lora_apply(x, base, [0, 4], [0], {0: (A, B, 2.0)}, 1.0)
    assert np.allclose(y1, y2, rtol=1e-14)
    assert np.allclose(y1 - base, 2.0 * (x @ A @ B), rtol=1e-12)


def test_zero_B_and_zero_scale_leave_base_unchanged():
    inst = wl.small_mixed()
    p = 0
    x, base = inst.x(p), inst.base_out(p)
    ads = _adapters(inst, p)
    zeroB = {i: (A, np.zeros_like(B), al) for i, (A, B, al) in ads.items()}
    y = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, zeroB, inst.scale)
    assert np.array_equal(y, base.astype(np.float64))
    y = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, ads, 0.0)
    assert np.array_equal(y, base.astype(np.float64))


def test_tokens_without_adapter_keep_base():
    inst = wl.small_mixed()
    x, base = inst.x(0), inst.base_out(0)
    y = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, _adapters(inst), inst.scale)
    ta = inst.token_adapter()
    assert (ta < 0).any() and (ta >= 0).any()
    assert np.array_equal(y[ta < 0], base[ta < 0].astype(np.float64))
    assert not np.array_equal(y[ta >= 0], base[ta >= 0].astype(np.float64))


def test_linearity_in_x():
    inst = wl.small_mixed(seed=3)
    ads = _adapters(inst)
    rng = np.random.default_rng(5)
    x1, x2 = rng.standard_normal((2, inst.T, inst.projs[0].h_in))
    zero = np.zeros((inst.T, inst.projs[0].h_out))
    f = lambda x: oracle.lora_apply(x, zero, inst.seg_offsets, inst.seg_adapter, ads, inst.scale)
    lhs = f(1.5 * x1 - 0.25 * x2)
    rhs = 1.5 * f(x1) - 0.25 * f(x2)
    assert np.allclose(lhs, rhs, rtol=1e-10, atol=1e-12)


def test_permuting_segments_permutes_outputs():
    inst = wl.small_mixed(seed=4)
    x, base = inst.x(0), inst.base_out(0)
    ads = _adapters(inst)
    y = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, ads, inst.scale)
    perm = np.random.default_rng(0).permutation(inst.n_seg)
    lens = np.diff(inst.seg_offsets)
    rows = np.concatenate([np.arange(inst.seg_offsets[g], inst.seg_offsets[g + 1]) for g in perm]).astype(np.int64)
    off2 = np.concatenate([[0], np.cumsum(lens[perm])]).astype(np.int32)
    y2 = oracle.lora_apply(x[rows], base[rows], off2, inst.seg_adapter[perm], ads, inst.scale)
    assert np.array_equal(y2, y[rows])


def test_splitting_a_segment_changes_nothing():
    rng = np.random.default_rng(7)
    x, base = rng.standard_normal((20, 16)), rng.standard_normal((20, 12))
    ads = {0: (rng.standard_normal((16, 3)), rng.standard_normal((3, 12)), 1.0), 1: (rng.standard_normal((16, 2)), rng.standard_normal((2, 12)), 1.0)}
    y1 = oracle.lora_apply(x, base, [0, 13, 20], [0, 1], ads, 2.0)
    y2 = oracle.lora_apply(x, base, [0, 4, 4, 13, 20], [0, 1, 0, 1], ads, 2.0)
    assert np.array_equal(y1, y2)


def test_zero_padded_rank_growth_changes_nothing():
    rng = np.random.default_rng(8)
    x, base = rng.standard_normal((9, 16)), rng.standard_normal((9, 12))
    A, B = rng.standard_normal((16, 3)), rng.standard_normal((3, 12))
    Ag = np.concatenate([A, np.zeros((16, 5))], axis=1)
    Bg = np.concatenate([B, rng.standard_normal((5, 12))], axis=0)  # rows met only by zero columns of A
    y1 = oracle.lora_apply(x, base, [0, 9], [0], {0: (A, B, 1.0)}, 2.0)
    y2 = oracle.lora_apply(x, base, [0, 9], [0], {0: (Ag, Bg, 1.0)}, 2.0)
    assert np.allclose(y1, y2, rtol=1e-13, atol=1e-13)


def test_two_adapters_in_sequence_add_their_deltas():
    rng = np.random.default_rng(9)
    x, base = rng.standard_normal((6, 10)), rng.standard_normal((6, 7))
    a0 = (rng.standard_normal((10, 2)), rng.standard_normal((2, 7)), 1.0)
    a1 = (rng.standard_normal((10, 4)), rng.standard_normal((4, 7)), 0.5)
    y0 = oracle.lora_apply(x, base, [0, 6], [0], {0: a0}, 2.0)
    y01 = oracle.lora_apply(x, y0, [0, 6], [1], {1: a1}, 2.0)
    ref = base + 2.0 * (x @ a0[0]) @ a0[1] + 1.0 * (x @ a1[0]) @ a1[1]
    assert np.allclose(y01, ref, rtol=1e-12, atol=1e-12)


def test_identity_slices_closed_form():
    """A = first r columns of I, B = first r rows of I, s = 2^k  =>  y[:, :r] = base + s.x[:, :r]."""
    rng = np.random.default_rng(10)
    h, r, T = 32, 8, 5
    x, base = rng.standard_normal((T, h)), rng.standard_normal((T, h))
    A, B = np.eye(h)[:, :r], np.eye(h)[:r, :]
    y = oracle.lora_apply(x, base, [0, T], [0], {0: (A, B, 1.0)}, 4.0)
    assert np.array_equal(y[:, :r], base[:, :r] + 4.0 * x[:, :r])
    assert np.array_equal(y[:, r:], base[:, r:])


def test_one_hot_x_selects_a_row_of_A():
    rng = np.random.default_rng(11)
    h_in, h_out, r = 12, 9, 4
    A, B = rng.standard_normal((h_in, r)), rng.standard_normal((r, h_out))
    x = np.zeros((h_in, h_in))
    x[np.arange(h_in), np.arange(h_in)] = 1.0
    y = oracle.lora_apply(x, np.zeros((h_in, h_out)), [0, h_in], [0], {0: (A, B, 1.0)}, 1.0)
    assert np.allclose(y, A @ B, rtol=1e-13, atol=1e-15)


def test_heterogeneous_ranks_bruteforce_per_token():
    inst = wl.small_mixed(seed=6)
    for p in range(len(inst.projs)):
        x, base = inst.x(p).astype(np.float64), inst.base_out(p).astype(np.float64)
        ads = _adapters(inst, p)
        y = oracle.lora_apply(x, base, inst.seg_offsets, inst.seg_adapter, ads, inst.scale)
        ta = inst.token_adapter()
        for t in range(0, inst.T, 7):
            if ta[t] < 0:
                ref = base[t]
            else:
                A, B, al = ads[int(ta[t])]
                ref = base[t] + inst.scale * al * ((x[t] @ A.astype(np.float64)) @ B.astype(np.float64))
            assert np.allclose(y[t], ref, rtol=1e-12, atol=1e-12)


def test_rejects_bad_offsets():
    x, base = np.zeros((4, 2)), np.zeros((4, 2))
    ad = {0: (np.zeros((2, 1)), np.zeros((1, 2)), 1.0)}
    for off in ([1, 4], [0, 3], [0, 3, 2, 4]):
        with pytest.raises(ValueError):
            oracle.lora_apply(x, base, off, [0] * (len(off) - 1), ad, 1.0)


def test_adapter_footprint_closed_form():
    """Section 3.2: a rank-32 adapter of a 7B model (q, k, v, o of 32 layers, 16-bit) is 64 MB."""
    assert 4 * 32 * 2 * (4096 * 32 + 32 * 4096) == 64 * 1024 * 1024
