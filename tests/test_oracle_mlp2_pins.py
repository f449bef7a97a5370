"""Pins for the oracle's two-matrix expert (the paper's own expert: Listing 1 mlp(w1, w2); Tables 1 and 3): closed
forms, library routines that the special cases reduce to, the dense definition, torch autograd and finite
differences, and the parameter counts that Table 3 prints.  No GPU is used."""
import os

import numpy as np
import pytest
import torch

import oracle
import xmoe_inputs as xi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ACTS = ["identity", "gelu", "silu"]


def _torch_act(name):
    return {"identity": lambda h: h, "gelu": lambda h: torch.nn.functional.gelu(h),   # exact erf form
            "silu": torch.nn.functional.silu}[name]


def _inputs(T=40, d=24, E=5, f=12, seed=0, skew=False):
    rng = np.random.default_rng(seed)
    inp = {"x": rng.standard_normal((T, d)), "w_router": rng.standard_normal((d, E)) * 0.3,
           "bias": (rng.standard_normal(E) * 2.0) if skew else None,
           "w1": rng.standard_normal((E, d, f)) * 0.3, "w2": rng.standard_normal((E, f, d)) * 0.3,
           "dout": rng.standard_normal((T, d))}
    return inp


# ------------------------------------------------------------------------------------------------ activations
def test_gelu_closed_forms():
    h = np.linspace(-6, 6, 241)
    g = oracle.activation("gelu", h)
    assert oracle.activation("gelu", np.array([0.0]))[0] == 0.0
    # x Phi(x) - (-x) Phi(-x) = x (Phi(x) + Phi(-x)) = x
    np.testing.assert_allclose(g - oracle.activation("gelu", -h), h, rtol=0, atol=1e-14)
    # Phi(1) = 0.841344746068543 (standard normal table)
    assert abs(oracle.activation("gelu", np.array([1.0]))[0] - 0.841344746068543) < 1e-14
    # far tails: gelu(x) -> x and gelu(-x) -> 0
    assert abs(oracle.activation("gelu", np.array([10.0]))[0] - 10.0) < 1e-12
    assert abs(oracle.activation("gelu", np.array([-10.0]))[0]) < 1e-12


@pytest.mark.parametrize("act", ACTS)
def test_activation_matches_torch_and_its_derivative(act):
    h = np.linspace(-5, 5, 401)
    th = torch.tensor(h, dtype=torch.float64, requires_grad=True)
    ta = _torch_act(act)(th)
    np.testing.assert_allclose(oracle.activation(act, h), ta.detach().numpy(), rtol=1e-13, atol=1e-15)
    ta.sum().backward()
    np.testing.assert_allclose(oracle.activation_grad(act, h), th.grad.numpy(), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("act", ACTS)
def test_activation_grad_central_difference(act):
    h = np.linspace(-4, 4, 97)
    eps = 1e-6
    fd = (oracle.activation(act, h + eps) - oracle.activation(act, h - eps)) / (2 * eps)
    np.testing.assert_allclose(oracle.activation_grad(act, h), fd, rtol=0, atol=1e-8)


# ------------------------------------------------------------------------------------------------ forward
@pytest.mark.parametrize("act", ACTS)
def test_single_expert_reduces_to_dense_mlp(act):
    """E = 1, k = 1: p = 1 and the layer is a dense two-layer MLP (torch on the CPU, a library routine)."""
    inp = _inputs(T=33, d=20, E=1, f=14, seed=3)
    fwd = oracle.moe2_layer_fwd(inp, 1, act, logits_mode="f64")
    x = torch.tensor(inp["x"])
    ref = _torch_act(act)(x @ torch.tensor(inp["w1"][0])) @ torch.tensor(inp["w2"][0])
    np.testing.assert_allclose(fwd["out"], ref.numpy(), rtol=1e-12, atol=1e-13)
    assert np.array_equal(fwd["eri"]["token_ids"], np.arange(33))


def test_identity_activation_collapses_to_one_matrix():
    """With no activation (the listing as printed) an expert is the single matrix W1 W2."""
    inp = _inputs(seed=4)
    k = 2
    fwd = oracle.moe2_layer_fwd(inp, k, "identity", logits_mode="f64")
    eri = fwd["eri"]
    for e in range(inp["w1"].shape[0]):
        lo, hi = eri["expert_offsets"][e], eri["expert_offsets"][e + 1]
        W = inp["w1"][e] @ inp["w2"][e]
        np.testing.assert_allclose(fwd["Y"][lo:hi], fwd["Xd"][lo:hi] @ W, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("act", ACTS)
@pytest.mark.parametrize("skew", [False, True])
def test_pipeline_equals_dense_definition(act, skew):
    inp = _inputs(seed=5, skew=skew)
    k = 3
    fwd = oracle.moe2_layer_fwd(inp, k, act, logits_mode="f64")
    ref = oracle.moe2_dense_definition(inp, k, act, fwd["logits"])
    np.testing.assert_allclose(fwd["out"], ref, rtol=1e-11, atol=1e-12)


def test_identical_experts_closed_form():
    """All experts equal: out[t] = (sum_j topk_w[t,j]) * MLP(x[t])."""
    inp = _inputs(seed=6)
    inp["w1"][:] = inp["w1"][0]
    inp["w2"][:] = inp["w2"][0]
    fwd = oracle.moe2_layer_fwd(inp, 2, "gelu", logits_mode="f64")
    y, _ = oracle.mlp2_ffn(inp["x"], inp["w1"][0], inp["w2"][0], "gelu")
    np.testing.assert_allclose(fwd["out"], fwd["topk_w"].sum(axis=1, keepdims=True) * y, rtol=1e-11, atol=1e-12)


def test_empty_expert_gets_zero_gradients_and_no_rows():
    inp = _inputs(seed=7)
    E = inp["w1"].shape[0]
    inp["bias"] = np.zeros(E)
    inp["bias"][2] = -1e30
    fwd = oracle.moe2_layer_fwd(inp, 2, "gelu", logits_mode="f64")
    assert fwd["eri"]["tokens_per_expert"][2] == 0
    bwd = oracle.moe2_layer_bwd(inp, fwd, 2, "gelu")
    assert not bwd["dw1"][2].any() and not bwd["dw2"][2].any()


# ------------------------------------------------------------------------------------------------ backward
def _torch_dense(inp, k, act, topk_idx):
    """Dense definition in torch with the routing decision held constant; returns out and the leaf tensors."""
    leaves = {n: torch.tensor(np.asarray(inp[n], np.float64), requires_grad=True) for n in ("x", "w_router", "w1", "w2")}
    logits = leaves["x"] @ leaves["w_router"]
    if inp.get("bias") is not None:
        logits = logits + torch.tensor(inp["bias"])
    p = torch.softmax(logits, dim=1)
    T, E = p.shape
    mask = torch.zeros((T, E), dtype=torch.float64)
    mask[torch.arange(T)[:, None], torch.tensor(topk_idx.astype(np.int64))] = 1.0
    out = torch.zeros_like(leaves["x"])
    for e in range(E):
        y = _torch_act(act)(leaves["x"] @ leaves["w1"][e]) @ leaves["w2"][e]
        out = out + (mask[:, e] * p[:, e])[:, None] * y
    return out, leaves


@pytest.mark.parametrize("act", ACTS)
@pytest.mark.parametrize("skew", [False, True])
def test_backward_matches_autograd_of_dense_definition(act, skew):
    inp = _inputs(seed=8, skew=skew)
    k = 2
    fwd = oracle.moe2_layer_fwd(inp, k, act, logits_mode="f64")
    bwd = oracle.moe2_layer_bwd(inp, fwd, k, act)
    out, leaves = _torch_dense(inp, k, act, fwd["topk_idx"])
    np.testing.assert_allclose(out.detach().numpy(), fwd["out"], rtol=1e-11, atol=1e-12)
    (out * torch.tensor(inp["dout"])).sum().backward()
    for name, key in (("x", "dx"), ("w_router", "dw_router"), ("w1", "dw1"), ("w2", "dw2")):
        np.testing.assert_allclose(bwd[key], leaves[name].grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=name)


@pytest.mark.parametrize("act", ["gelu", "silu"])
def test_backward_matches_central_differences(act):
    inp = _inputs(T=12, d=8, E=4, f=6, seed=9)
    k = 2
    fwd = oracle.moe2_layer_fwd(inp, k, act, logits_mode="f64")
    bwd = oracle.moe2_layer_bwd(inp, fwd, k, act)
    # routing margin: the finite-difference step must not flip a top-k decision
    srt = np.sort(fwd["logits"], axis=1)[:, ::-1]
    assert (srt[:, k - 1] - srt[:, k]).min() > 1e-3
    rng = np.random.default_rng(10)
    eps = 1e-6

    def loss(i2):
        f2 = oracle.moe2_layer_fwd(i2, k, act, logits_mode="f64")
        assert np.array_equal(f2["topk_idx"], fwd["topk_idx"])
        return float((f2["out"] * inp["dout"]).sum())

    for name, key in (("x", "dx"), ("w_router", "dw_router"), ("w1", "dw1"), ("w2", "dw2")):
        v = rng.standard_normal(inp[name].shape)
        ip, im = dict(inp), dict(inp)
        ip[name] = inp[name] + eps * v
        im[name] = inp[name] - eps * v
        fd = (loss(ip) - loss(im)) / (2 * eps)
        an = float((bwd[key] * v).sum())
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)


def test_dlogits_rows_sum_to_zero():
    inp = _inputs(seed=11)
    fwd = oracle.moe2_layer_fwd(inp, 2, "gelu", logits_mode="f64")
    bwd = oracle.moe2_layer_bwd(inp, fwd, 2, "gelu")
    assert np.abs(bwd["dlogits"].sum(axis=1)).max() < 1e-12


# ------------------------------------------------------------------------------------------------ the paper's numbers
def test_table3_parameter_counts_need_two_matrices_per_expert():
    """Table 3's printed totals pin the expert as two d x f matrices."""
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "table3_model_params.txt")) if not ln.startswith("#")]
    assert len(rows) == 4
    for name, H, F, E, k, L, printed in rows:
        H, F, E, L, printed = int(H), int(F), int(E), int(L), float(printed)
        total = L * (oracle.expert_param_count(E, H, F) + 4 * H * H) / 2 ** 30
        assert abs(total - printed) < 0.06, (name, total, printed)          # printed to one decimal
        three = L * (oracle.expert_param_count(E, H, F, matrices=3) + 4 * H * H) / 2 ** 30
        assert abs(three - printed) > 1.0, name


def test_mlp2_configs_follow_table3():
    rows = {ln.split()[0]: ln.split()[1:] for ln in open(os.path.join(GOLDEN, "table3_model_params.txt"))
            if not ln.startswith("#")}
    for name, cfgname in (("Small", "small_mlp2"), ("Medium", "medium_mlp2"), ("Large", "large_mlp2"),
                          ("Super", "super_mlp2")):
        cfg = xi.CONFIGS[cfgname]
        H, F, E, k = (int(v) for v in rows[name][:4])
        assert (cfg.d, cfg.f, cfg.E, cfg.k) == (H, F, E, k) and cfg.expert == "mlp2" and cfg.E_s == 0
