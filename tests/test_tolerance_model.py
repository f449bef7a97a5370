"""Where the bf16 tolerance metric comes from (CPU only).

The benchmark definition asks for "max relative error 2e-2 for bf16 (fp32 accumulate)" and leaves the treatment of
elements near zero open.  This test redoes the backward of the expert MLP in float64 but rounds to bf16 exactly the
tensors that any bf16 implementation has to store (dG, dU and the result dXd) - i.e. it models an implementation
with perfect float32 accumulation.  Rounding a stored operand perturbs a dot product by about 2^-9 times the 2-norm
of its terms, which is the scale of the ROW of the result; token rows differ in scale by orders of magnitude (they
carry the token's combine weight).  So:
  * floored at the whole tensor's RMS, even this ideal implementation exceeds 2e-2 on rows with large combine
    weights: that metric cannot be met by any bf16-storing implementation;
  * floored at the RMS of the element's row, the ideal implementation sits near 1e-2, which leaves the stated
    2e-2 as a bound with a factor ~2 of slack for further stored intermediates (Y, dY).
The GPU tests therefore use the row floor for token-row tensors and the per-expert floor for weight gradients."""
import numpy as np
import pytest

import oracle
import xmoe_inputs as xi
from gpu_util import rel_err


def rt(a):
    return xi.round_to_storage(np.asarray(a, np.float32), "bf16").astype(np.float64)


@pytest.mark.parametrize("name", ["mini_bf16", "mid_bf16"])
def test_ideal_bf16_rounding_vs_metric(name):
    cfg = xi.CONFIGS[name]
    inp = xi.make_layer_inputs(cfg)
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    bwd = oracle.moe_layer_bwd(inp, fwd, cfg.k)
    G, U, dY = rt(fwd["G"]), rt(fwd["U"]), rt(bwd["dY"])
    off = fwd["eri"]["expert_offsets"]
    ref = oracle.expert_ffn_bwd(fwd["Xd"], G, U, dY, off, inp["wg"], inp["wu"], inp["wd"])[0]
    got = np.zeros_like(ref)
    for e in range(cfg.E):
        lo, hi = off[e], off[e + 1]
        if hi == lo:
            continue
        g, u = G[lo:hi], U[lo:hi]
        sig = 1.0 / (1.0 + np.exp(-g))
        dA = dY[lo:hi] @ inp["wd"][e].astype(np.float64).T
        dG = rt(dA * u * (sig * (1.0 + g * (1.0 - sig))))
        dU = rt(dA * g * sig)
        got[lo:hi] = rt(dG @ inp["wg"][e].astype(np.float64).T + dU @ inp["wu"][e].astype(np.float64).T)
    e_tensor = rel_err(got, ref, "tensor")
    e_row = rel_err(got, ref, "row")
    assert e_tensor > 2e-2, e_tensor          # the tensor-wide floor is unattainable in bf16
    assert e_row < 1.3e-2, e_row              # the row floor leaves a factor ~2 of slack under 2e-2


def test_ideal_bf16_chain_vs_metric():
    """The whole chain forward + backward with exact accumulation and bf16 storage of G, U, A, Y, dY, dG, dU and
    the results: row-wise relative error in the 2-norm stays near 5e-3 (well inside 2e-2), while the
    element-wise slice-floored figure of the weight gradients reaches 2e-2..4e-2.  Hence the two-part criterion
    of assert_close_chain."""
    from gpu_util import rel_err_norm
    cfg = xi.CONFIGS["mini_bf16_skew"]
    inp = xi.make_layer_inputs(cfg)
    fwd = oracle.moe_layer_fwd(inp, cfg.k)
    bwd = oracle.moe_layer_bwd(inp, fwd, cfg.k)
    eri = fwd["eri"]
    off = eri["expert_offsets"]
    Xd = fwd["Xd"]
    G, U, Y = np.zeros_like(fwd["G"]), np.zeros_like(fwd["U"]), np.zeros_like(fwd["Y"])
    w64 = {k_: inp[k_].astype(np.float64) for k_ in ("wg", "wu", "wd")}
    for e in range(cfg.E):
        lo, hi = off[e], off[e + 1]
        if hi == lo:
            continue
        g, u = Xd[lo:hi] @ w64["wg"][e], Xd[lo:hi] @ w64["wu"][e]
        G[lo:hi], U[lo:hi] = rt(g), rt(u)
        Y[lo:hi] = rt(rt(oracle.silu(g) * u) @ w64["wd"][e])
    cw = eri["combine_weights"].astype(np.float32).astype(np.float64)
    dY = rt(cw[:, None] * inp["dout"].astype(np.float64)[eri["token_ids"]])
    dXd = np.zeros_like(Xd)
    dW = {k_: np.zeros(inp[k_].shape) for k_ in ("wg", "wu", "wd")}
    for e in range(cfg.E):
        lo, hi = off[e], off[e + 1]
        if hi == lo:
            continue
        g, u = G[lo:hi], U[lo:hi]
        sig = 1.0 / (1.0 + np.exp(-g))
        dA = dY[lo:hi] @ w64["wd"][e].T
        dG, dU, A = rt(dA * u * (sig * (1.0 + g * (1.0 - sig)))), rt(dA * g * sig), rt(g * sig * u)
        dXd[lo:hi] = rt(dG @ w64["wg"][e].T + dU @ w64["wu"][e].T)
        dW["wg"][e], dW["wu"][e], dW["wd"][e] = rt(Xd[lo:hi].T @ dG), rt(Xd[lo:hi].T @ dU), rt(A.T @ dY[lo:hi])
    worst_elem = 0.0
    for got, ref, fl in ((Y, fwd["Y"], "row"), (dXd, bwd["dXd"], "row"), (dW["wg"], bwd["dwg"], "expert"),
                         (dW["wu"], bwd["dwu"], "expert"), (dW["wd"], bwd["dwd"], "expert")):
        assert rel_err_norm(got, ref) < 1e-2
        worst_elem = max(worst_elem, rel_err(got, ref, fl))
    assert 2e-2 < worst_elem < 8e-2, worst_elem
