"""Pins for the CPU oracle: each part of oracle/ is checked against something other than itself - closed forms,
invariants, special cases that reduce to a textbook or library routine, brute force on tiny inputs, the one
figure the paper prints for this path (Table 4's theoretical activation size), finite differences and torch
autograd.  No GPU is used."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import xmoe_inputs as xi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------------------------ gate logits
def _fold64(partial):
    partial = list(partial)
    off = 32
    while off >= 1:
        for l in range(off):
            partial[l] = np.float32(partial[l] + partial[l + off])
        off //= 2
    return partial[0]


def _round_fraction_to_f32(s: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) float32 of an exact rational."""
    if s == 0:
        return np.float32(0.0)
    c = np.float32(float(s))
    cands = [c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))]
    best = None
    for v in cands:
        err = abs(Fraction(float(v)) - s)
        even = (int(np.float32(v).view(np.uint32)) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, v)
    return np.float32(best[1])


def test_gate_logits_contract_exact_rational_f32():
    """Tiny float32 case: every fmaf and every add of the fixed order redone in exact rational arithmetic."""
    rng = np.random.default_rng(5)
    T, d, E = 3, 150, 4                       # d not a multiple of 64: lanes 22..63 see one term less
    x = rng.standard_normal((T, d)).astype(np.float32)
    w = rng.standard_normal((d, E)).astype(np.float32)
    b = rng.standard_normal(E).astype(np.float32)
    got = oracle.gate_logits_contract(x, w, b)
    for t in range(T):
        for e in range(E):
            partial = [np.float32(0.0)] * 64
            for i in range(d):
                l = i % 64
                s = Fraction(float(x[t, i])) * Fraction(float(w[i, e])) + Fraction(float(partial[l]))
                partial[l] = _round_fraction_to_f32(s)
            v = np.float32(_fold64(partial) + b[e])
            assert got[t, e] == v, (t, e, got[t, e], v)


def test_gate_logits_contract_bf16_inputs_numpy_emulation():
    """bf16 x bf16 products are exact in float32, so fmaf == float32 add of the exact product: a vectorised
    numpy float32 emulation of the order must agree bit for bit."""
    cfg = xi.CONFIGS["mini_bf16_skew"]
    x, w, b = xi.make_x(cfg)[:40], xi.make_w_router(cfg), xi.make_gate_bias(cfg)
    got = oracle.gate_logits_contract(x, w, b)
    T, d = x.shape
    E = w.shape[1]
    partial = np.zeros((T, E, 64), dtype=np.float32)
    for i in range(d):
        prod = (x[:, i:i + 1] * w[i][None, :]).astype(np.float32)       # exact
        partial[:, :, i % 64] = partial[:, :, i % 64] + prod
    off = 32
    while off >= 1:
        partial[:, :, :off] = partial[:, :, :off] + partial[:, :, off:2 * off]
        off //= 2
    want = partial[:, :, 0] + b[None, :]
    assert np.array_equal(got, want)


@pytest.mark.parametrize("name", ["tiny_f32", "mini_bf16", "odd_f32"])
def test_gate_logits_contract_close_to_float64(name):
    cfg = xi.CONFIGS[name]
    x, w = xi.make_x(cfg), xi.make_w_router(cfg)
    got = oracle.gate_logits_contract(x, w, None).astype(np.float64)
    want = oracle.gate_logits_f64(x, w, None)
    # forward error bound of any float32 summation of d terms: d * 2^-24 * sum |x_i w_i|
    bound = cfg.d * 2.0 ** -24 * (np.abs(x).astype(np.float64) @ np.abs(w).astype(np.float64))
    assert np.all(np.abs(got - want) <= bound + 1e-30)


# ------------------------------------------------------------------------------------------------ softmax, top-k
def test_softmax_rows_sum_to_one_and_shift_invariant():
    l = xi.make_logits(64, 17, seed=3, std=4.0)
    p = oracle.softmax(l)
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
    p2 = oracle.softmax(l.astype(np.float64) + 123.5)
    assert np.allclose(p, p2, atol=1e-13)
    import scipy.special
    assert np.allclose(p, scipy.special.softmax(l.astype(np.float64), axis=1), atol=1e-15)


def test_route_all_equal_logits_closed_form():
    T, E, k = 5, 12, 4
    idx, w, p = oracle.route(np.full((T, E), 0.75, dtype=np.float32), k)
    assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (T, 1)))
    assert np.allclose(w, 1.0 / E, atol=1e-15)


def test_route_k_equals_E_is_argsort():
    l = xi.make_logits(50, 9, seed=1)
    idx, w, p = oracle.route(l, 9)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-14)
    assert np.array_equal(idx, np.argsort(-l.astype(np.float64), axis=1, kind="stable").astype(np.int32))


def test_route_explicit_ties_lower_index_wins():
    l = np.array([[1.0, 3.0, 3.0, 0.0, 3.0, 2.0],
                  [5.0, 5.0, 5.0, 5.0, 5.0, 5.0],
                  [0.0, -1.0, 2.0, 2.0, -1.0, 0.0]], dtype=np.float32)
    idx, w, _ = oracle.route(l, 4)
    assert idx.tolist() == [[1, 2, 4, 5], [0, 1, 2, 3], [2, 3, 0, 5]]


def test_route_brute_force_subsets():
    """For distinct logits the chosen set is the k-subset with the largest logit sum, slots in descending order,
    and the weights are the softmax probabilities of the chosen experts (not renormalised)."""
    rng = np.random.default_rng(11)
    for E, k in [(4, 1), (5, 2), (6, 3), (6, 5)]:
        l = rng.standard_normal((40, E)).astype(np.float32)
        idx, w, p = oracle.route(l, k)
        for t in range(l.shape[0]):
            best = max(itertools.combinations(range(E), k), key=lambda s: sum(float(l[t, e]) for e in s))
            assert set(idx[t].tolist()) == set(best)
            vals = [float(l[t, e]) for e in idx[t]]
            assert vals == sorted(vals, reverse=True)
            ez = [math.exp(float(v)) for v in l[t]]
            for j in range(k):
                assert abs(w[t, j] - ez[idx[t, j]] / sum(ez)) < 1e-12


# ------------------------------------------------------------------------------------------------ ERI arrays
def _eri_brute_force(topk_idx, topk_w, E):
    T, k = topk_idx.shape
    flat = topk_idx.reshape(-1)
    n_tot = T * k
    row = np.empty(n_tot, dtype=np.int64)
    for n in range(n_tot):
        # rows before n: smaller expert id anywhere, or the same expert at an earlier flat index
        row[n] = sum(1 for m in range(n_tot) if flat[m] < flat[n] or (flat[m] == flat[n] and m < n))
    return row


@pytest.mark.parametrize("T,E,k,seed", [(16, 4, 2, 0), (32, 6, 3, 1), (9, 3, 3, 2), (20, 8, 1, 3)])
def test_eri_brute_force(T, E, k, seed):
    idx, w, _ = oracle.route(xi.make_logits(T, E, seed=seed), k)
    eri = oracle.build_eri(idx, w, E)
    row = _eri_brute_force(idx, w, E)
    assert np.array_equal(eri["row_of_slot"], row.astype(np.int32))
    flat_w = w.reshape(-1)
    for n in range(T * k):
        i = row[n]
        assert eri["token_ids"][i] == n // k
        assert eri["expert_ids"][i] == idx.reshape(-1)[n]
        assert eri["combine_weights"][i] == flat_w[n]


def check_eri_invariants(eri, topk_idx, E):
    T, k = topk_idx.shape
    B = T * k
    tpe, off = eri["tokens_per_expert"], eri["expert_offsets"]
    assert tpe.sum() == B and off[0] == 0 and off[-1] == B
    assert np.array_equal(np.diff(off), tpe)
    assert np.all(np.diff(eri["expert_ids"]) >= 0)
    assert np.array_equal(np.sort(eri["row_of_slot"]), np.arange(B))           # a permutation
    n = np.arange(B)
    assert np.array_equal(eri["token_ids"][eri["row_of_slot"]], n // k)
    assert np.array_equal(eri["expert_ids"][eri["row_of_slot"]], topk_idx.reshape(-1))
    for e in range(E):
        seg = eri["token_ids"][off[e]:off[e + 1]]
        assert np.all(np.diff(seg) > 0)                                        # strictly ascending tokens
        assert np.all(eri["expert_ids"][off[e]:off[e + 1]] == e)
    # (token, slot) pairs form a permutation of all T*k pairs
    slot_of_row = np.empty(B, dtype=np.int64)
    slot_of_row[eri["row_of_slot"]] = n % k
    pairs = set(zip(eri["token_ids"].tolist(), slot_of_row.tolist()))
    assert len(pairs) == B


@pytest.mark.parametrize("name", ["tiny_f32", "mini_bf16_skew", "odd_bf16"])
def test_eri_invariants(name):
    cfg = xi.CONFIGS[name]
    logits = oracle.gate_logits_contract(xi.make_x(cfg), xi.make_w_router(cfg), xi.make_gate_bias(cfg))
    idx, w, _ = oracle.route(logits, cfg.k)
    eri = oracle.build_eri(idx, w, cfg.E)
    check_eri_invariants(eri, idx, cfg.E)
    # the same arrays from plain Python sorting of (expert, flat index) tuples
    keys = sorted((int(e), n) for n, e in enumerate(idx.reshape(-1)))
    assert eri["token_ids"].tolist() == [n // cfg.k for _, n in keys]
    assert eri["expert_ids"].tolist() == [e for e, _ in keys]


def test_eri_empty_experts():
    l = xi.make_logits(40, 6, seed=4)
    l[:, 2] = -1e30
    l[:, 5] = -1e30
    idx, w, _ = oracle.route(l, 2)
    eri = oracle.build_eri(idx, w, 6)
    assert eri["tokens_per_expert"][2] == 0 and eri["tokens_per_expert"][5] == 0
    check_eri_invariants(eri, idx, 6)


# ------------------------------------------------------------------------------------------------ dispatch / FFN / combine
def test_dispatch_is_bit_copy():
    cfg = xi.CONFIGS["odd_bf16"]
    x = xi.make_x(cfg)
    ids = np.array([5, 5, 0, 130, 7], dtype=np.int32)
    xd = oracle.dispatch(x, ids)
    for i, t in enumerate(ids):
        assert np.array_equal(xd[i], x[t])


def _torch_swiglu(x, wg, wu, wd):
    x, wg, wu, wd = (torch.from_numpy(np.asarray(a, np.float64)) for a in (x, wg, wu, wd))
    return (torch.nn.functional.silu(x @ wg) * (x @ wu)) @ wd


def test_single_expert_reduces_to_dense_swiglu():
    """E=1, k=1: p = 1, so the layer is one dense SwiGLU FFN (checked against torch's silu and matmul)."""
    cfg = xi.MoEConfig("e1", T=33, d=24, E=1, k=1, f=10, dtype="f32", router_std=0.3)
    inp = xi.make_layer_inputs(cfg)
    fwd = oracle.moe_layer_fwd(inp, 1)
    assert np.allclose(fwd["topk_w"], 1.0)
    want = _torch_swiglu(inp["x"], inp["wg"][0], inp["wu"][0], inp["wd"][0]).numpy()
    assert np.allclose(fwd["out"], want, rtol=1e-12, atol=1e-15)


def test_identical_experts_closed_form():
    cfg = xi.CONFIGS["odd_f32"]
    inp = xi.make_layer_inputs(cfg)
    for key in ("wg", "wu", "wd"):
        inp[key] = np.repeat(inp[key][:1], cfg.E, axis=0)
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    ffn = _torch_swiglu(inp["x"], inp["wg"][0], inp["wu"][0], inp["wd"][0]).numpy()
    want = fwd["topk_w"].sum(axis=1, keepdims=True) * ffn
    assert np.allclose(fwd["out"], want, rtol=1e-11, atol=1e-16)


@pytest.mark.parametrize("name", ["odd_f32", "mini_f32"])
def test_pipeline_equals_dense_definition(name):
    """gather -> ragged GEMMs -> scatter-add equals the definition that loops over every (token, expert)."""
    cfg = xi.CONFIGS[name]
    inp = xi.make_layer_inputs(cfg)
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    want = oracle.moe_dense_definition(inp, cfg.k, fwd["logits"])
    assert np.allclose(fwd["out"], want, rtol=1e-11, atol=1e-16)


def test_linearity_in_wd_and_segment_shuffle_invariance():
    cfg = xi.CONFIGS["odd_f32"]
    inp = xi.make_layer_inputs(cfg)
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    inp2 = dict(inp)
    inp2["wd"] = inp["wd"] * np.float32(2.0)
    assert np.allclose(oracle.moe_layer_fwd(inp2, cfg.k)["out"], 2.0 * fwd["out"], rtol=1e-12)
    # shuffle rows inside each expert segment: out must not change beyond rounding
    eri = fwd["eri"]
    rng = np.random.default_rng(0)
    perm = np.arange(cfg.B)
    for e in range(cfg.E):
        lo, hi = eri["expert_offsets"][e], eri["expert_offsets"][e + 1]
        perm[lo:hi] = rng.permutation(np.arange(lo, hi))
    tok, cw = eri["token_ids"][perm], eri["combine_weights"][perm]
    Y, _, _ = oracle.expert_ffn_fwd(oracle.dispatch(inp["x"], tok), eri["expert_offsets"],
                                    inp["wg"], inp["wu"], inp["wd"])
    assert np.allclose(oracle.combine(Y, tok, cw, cfg.T), fwd["out"], rtol=1e-11, atol=1e-17)


def test_shared_experts_only_limit():
    cfg = xi.CONFIGS["mini_f32"]
    inp = xi.make_layer_inputs(cfg)
    inp["wd"] = np.zeros_like(inp["wd"])
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    want = sum(_torch_swiglu(inp["x"], inp["shared_wg"][s], inp["shared_wu"][s], inp["shared_wd"][s]).numpy()
               for s in range(cfg.E_s))
    assert np.allclose(fwd["out"], want, rtol=1e-12, atol=1e-16)


# ------------------------------------------------------------------------------------------------ backward
def _loss(inp, k, topk_ref=None):
    fwd = oracle.moe_layer_fwd(inp, k, logits_mode="f64")
    if topk_ref is not None:
        assert np.array_equal(fwd["topk_idx"], topk_ref), "finite-difference step crossed a routing boundary"
    return float((np.asarray(inp["dout"], np.float64) * fwd["out"]).sum()), fwd


def _small_cfg():
    return xi.MoEConfig("fd", T=12, d=10, E=5, k=2, f=6, dtype="f32", E_s=1, router_std=0.5, w_std=0.4, seed=7)


def test_backward_matches_central_finite_differences():
    cfg = _small_cfg()
    inp = {k_: (None if v is None else np.asarray(v, np.float64)) for k_, v in xi.make_layer_inputs(cfg).items()}
    _, fwd = _loss(inp, cfg.k)
    # keep away from routing ties: margin between the k-th and (k+1)-th logit
    srt = np.sort(fwd["logits"], axis=1)[:, ::-1]
    assert (srt[:, cfg.k - 1] - srt[:, cfg.k]).min() > 1e-3
    bwd = oracle.moe_layer_bwd(inp, fwd, cfg.k)
    pairs = [("x", "dx"), ("w_router", "dw_router"), ("wg", "dwg"), ("wu", "dwu"), ("wd", "dwd"),
             ("shared_wg", "dshared_wg"), ("shared_wu", "dshared_wu"), ("shared_wd", "dshared_wd")]
    rng = np.random.default_rng(0)
    h = 1e-6
    for name, gname in pairs:
        g = bwd[gname]
        flat_idx = rng.choice(inp[name].size, size=min(25, inp[name].size), replace=False)
        for fi in flat_idx:
            ix = np.unravel_index(fi, inp[name].shape)
            old = inp[name][ix]
            inp[name][ix] = old + h
            lp, _ = _loss(inp, cfg.k, fwd["topk_idx"])
            inp[name][ix] = old - h
            lm, _ = _loss(inp, cfg.k, fwd["topk_idx"])
            inp[name][ix] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - g[ix]) <= 1e-6 * max(1.0, abs(fd)) + 1e-8, (name, ix, fd, g[ix])


def _torch_dense_layer(inp, k, topk_idx):
    """The layer's definition in torch float64 (fixed top-k indices), for autograd."""
    x = inp["x"]
    logits = x @ inp["w_router"]
    if inp.get("bias") is not None:
        logits = logits + inp["bias"]
    p = torch.softmax(logits, dim=1)
    out = torch.zeros_like(x)
    T = x.shape[0]
    for t in range(T):
        for j in range(k):
            e = int(topk_idx[t, j])
            y = (torch.nn.functional.silu(x[t] @ inp["wg"][e]) * (x[t] @ inp["wu"][e])) @ inp["wd"][e]
            out[t] = out[t] + p[t, e] * y
    for s in range(inp["shared_wg"].shape[0]):
        out = out + (torch.nn.functional.silu(x @ inp["shared_wg"][s]) * (x @ inp["shared_wu"][s])) @ inp["shared_wd"][s]
    return out


@pytest.mark.parametrize("skew", [0.0, 2.0])
def test_backward_matches_torch_autograd(skew):
    cfg = xi.MoEConfig("ag", T=40, d=16, E=6, k=3, f=8, dtype="f32", E_s=2, router_std=0.4, w_std=0.3,
                       skew_alpha=skew, seed=3)
    raw = xi.make_layer_inputs(cfg)
    inp = {k_: (None if v is None else np.asarray(v, np.float64)) for k_, v in raw.items()}
    fwd = oracle.moe_layer_fwd(inp, cfg.k, logits_mode="f64")
    bwd = oracle.moe_layer_bwd(inp, fwd, cfg.k)
    tin = {}
    for k_, v in inp.items():
        if v is None:
            tin[k_] = None
        else:
            tin[k_] = torch.from_numpy(v.copy()).requires_grad_(k_ not in ("dout", "bias"))
    out = _torch_dense_layer(tin, cfg.k, fwd["topk_idx"])
    assert np.allclose(out.detach().numpy(), fwd["out"], rtol=1e-11, atol=1e-15)
    (out * tin["dout"]).sum().backward()
    for name, gname in [("x", "dx"), ("w_router", "dw_router"), ("wg", "dwg"), ("wu", "dwu"), ("wd", "dwd"),
                        ("shared_wg", "dshared_wg"), ("shared_wu", "dshared_wu"), ("shared_wd", "dshared_wd")]:
        want = tin[name].grad.numpy()
        scale = np.abs(want).max() + 1e-30
        assert np.abs(bwd[gname] - want).max() <= 1e-11 * scale, name


# ------------------------------------------------------------------------------------------------ token dropping
def _capped_brute_force(topk_idx, topk_w, E, C):
    """Per expert: its (weight, flat index) pairs sorted by weight descending then index ascending, the first C kept,
    the kept ones listed again in ascending flat index.  Plain Python."""
    T, k = topk_idx.shape
    flat_e = [int(v) for v in topk_idx.reshape(-1)]
    flat_w = [float(v) for v in np.asarray(topk_w).reshape(-1)]
    rows = []
    for e in range(E):
        mine = [n for n in range(T * k) if flat_e[n] == e]
        best = sorted(mine, key=lambda n: (-flat_w[n], n))[:C]
        rows.append(sorted(best))
    return rows


@pytest.mark.parametrize("T,E,k,C,seed", [(40, 5, 2, 7, 0), (64, 8, 3, 1, 1), (33, 4, 4, 10, 2), (100, 16, 2, 5, 3),
                                          (17, 3, 1, 0, 4)])
def test_capped_eri_brute_force(T, E, k, C, seed):
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, w, _ = oracle.route(logits, k)
    got = oracle.build_eri_capped(idx, w, E, C)
    rows = _capped_brute_force(idx, w, E, C)
    flat = [n for r in rows for n in r]
    assert got["token_ids"].tolist() == [n // k for n in flat]
    assert got["expert_ids"].tolist() == [e for e, r in enumerate(rows) for _ in r]
    assert got["tokens_per_expert"].tolist() == [len(r) for r in rows]
    assert np.array_equal(got["combine_weights"], np.asarray(w).reshape(-1)[flat])
    ros = np.full(T * k, -1)
    ros[flat] = np.arange(len(flat))
    assert np.array_equal(got["row_of_slot"], ros)


def test_capped_eri_limits_and_invariants():
    rng = np.random.default_rng(7)
    T, E, k = 300, 12, 3
    logits = (rng.standard_normal((T, E)) + np.linspace(0, 2.5, E)).astype(np.float32)   # uneven load
    idx, w, _ = oracle.route(logits, k)
    full = oracle.build_eri(idx, w, E)
    # capacity at or above the largest segment: nothing is dropped, identical arrays
    big = oracle.build_eri_capped(idx, w, E, int(full["tokens_per_expert"].max()))
    for key in full:
        assert np.array_equal(big[key], full[key]), key
    C = int(np.median(full["tokens_per_expert"]))
    cap = oracle.build_eri_capped(idx, w, E, C)
    assert np.array_equal(cap["tokens_per_expert"], np.minimum(full["tokens_per_expert"], C))
    assert cap["expert_offsets"][-1] == cap["token_ids"].size == (cap["row_of_slot"] >= 0).sum()
    flat_w = np.asarray(w).reshape(-1)
    flat_e = idx.reshape(-1)
    kept = cap["row_of_slot"] >= 0
    for e in range(E):
        mine = flat_e == e
        if (mine & ~kept).any():     # every dropped entry is no heavier than every kept one of the same expert
            assert flat_w[mine & ~kept].max() <= flat_w[mine & kept].min()
    # retained rows keep the order of the dropless table
    rows_full = full["row_of_slot"][kept]
    assert np.array_equal(np.argsort(rows_full, kind="stable"), np.argsort(cap["row_of_slot"][kept], kind="stable"))
    assert np.all(np.diff(cap["expert_ids"]) >= 0)
    for e in range(E):
        seg = cap["token_ids"][cap["expert_offsets"][e]:cap["expert_offsets"][e + 1]]
        assert np.all(np.diff(seg) > 0)
    # capacity 0 drops everything
    none = oracle.build_eri_capped(idx, w, E, 0)
    assert none["token_ids"].size == 0 and not none["tokens_per_expert"].any() and (none["row_of_slot"] == -1).all()


def test_capped_eri_equal_weights_keep_the_lower_flat_index():
    T, E, k, C = 20, 3, 2, 4
    idx = np.stack([np.arange(T) % E, (np.arange(T) + 1) % E], axis=1).astype(np.int32)
    w = np.full((T, k), 0.25, dtype=np.float32)
    got = oracle.build_eri_capped(idx, w, E, C)
    flat_e = idx.reshape(-1)
    for e in range(E):
        first = np.flatnonzero(flat_e == e)[:C]
        seg = slice(got["expert_offsets"][e], got["expert_offsets"][e + 1])
        assert np.array_equal(got["token_ids"][seg], first // k)


def _torch_dense_layer_masked(inp, k, topk_idx, keep):
    """Dense definition with a constant keep mask on the (token, slot) pairs."""
    x = inp["x"]
    logits = x @ inp["w_router"]
    p = torch.softmax(logits, dim=1)
    out = torch.zeros_like(x)
    for t in range(x.shape[0]):
        for j in range(k):
            if keep[t, j]:
                e = int(topk_idx[t, j])
                y = (torch.nn.functional.silu(x[t] @ inp["wg"][e]) * (x[t] @ inp["wu"][e])) @ inp["wd"][e]
                out[t] = out[t] + p[t, e] * y
    for s in range(inp["shared_wg"].shape[0]):
        out = out + (torch.nn.functional.silu(x @ inp["shared_wg"][s]) * (x @ inp["shared_wu"][s])) @ inp["shared_wd"][s]
    return out


def test_layer_with_token_dropping_matches_masked_dense_definition_and_autograd():
    cfg = xi.MoEConfig("drop", T=48, d=16, E=6, k=3, f=8, dtype="f32", E_s=1, router_std=0.4, w_std=0.3,
                       skew_alpha=1.5, seed=5)
    raw = xi.make_layer_inputs(cfg)
    raw["bias"] = None
    inp = {k_: (None if v is None else np.asarray(v, np.float64)) for k_, v in raw.items()}
    C = 10
    fwd = oracle.moe_layer_fwd(inp, cfg.k, logits_mode="f64", max_token_count=C)
    bwd = oracle.moe_layer_bwd(inp, fwd, cfg.k)
    assert fwd["eri"]["tokens_per_expert"].max() == C and (fwd["eri"]["row_of_slot"] < 0).any()
    keep = (fwd["eri"]["row_of_slot"] >= 0).reshape(cfg.T, cfg.k)
    tin = {k_: (None if v is None else torch.from_numpy(v.copy()).requires_grad_(k_ != "dout"))
           for k_, v in inp.items()}
    out = _torch_dense_layer_masked(tin, cfg.k, fwd["topk_idx"], keep)
    assert np.allclose(out.detach().numpy(), fwd["out"], rtol=1e-11, atol=1e-15)
    (out * tin["dout"]).sum().backward()
    for name, gname in [("x", "dx"), ("w_router", "dw_router"), ("wg", "dwg"), ("wu", "dwu"), ("wd", "dwd"),
                        ("shared_wg", "dshared_wg")]:
        want = tin[name].grad.numpy()
        assert np.abs(bwd[gname] - want).max() <= 1e-11 * (np.abs(want).max() + 1e-30), name
    assert not bwd["dw"][~keep].any()


def test_backward_structure():
    cfg = xi.CONFIGS["mini_bf16_skew"]
    inp = xi.make_layer_inputs(cfg)
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    bwd = oracle.moe_layer_bwd(inp, fwd, cfg.k)
    assert np.abs(bwd["dlogits"].sum(axis=1)).max() < 1e-12        # softmax Jacobian annihilates constants
    tpe = fwd["eri"]["tokens_per_expert"]
    for e in range(cfg.E):
        if tpe[e] == 0:
            assert not bwd["dwg"][e].any() and not bwd["dwu"][e].any() and not bwd["dwd"][e].any()
    # adjoint identity <dOut, J v> = <J^T dOut, v> along a random direction in Wd (the layer is linear in Wd)
    rng = np.random.default_rng(1)
    v = rng.standard_normal(inp["wd"].shape)
    inp2 = dict(inp)
    inp2["wd"] = v
    inp2["shared_wd"] = np.zeros_like(inp["shared_wd"])
    jv = oracle.moe_layer_fwd(inp2, cfg.k)["out"]
    lhs = (np.asarray(inp["dout"], np.float64) * jv).sum()
    rhs = (bwd["dwd"] * v).sum()
    assert abs(lhs - rhs) <= 1e-10 * abs(lhs)


# ------------------------------------------------------------------------------------------------ footprint
def test_activation_bytes_matches_table4():
    with open(os.path.join(GOLDEN, "table4_theoretical_activation.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    S, H, F, k, s, printed = rows[0]
    got = oracle.activation_bytes(int(S), int(k), int(H), int(F), int(s)) / 2 ** 30
    assert abs(got - float(printed)) < 5e-4
